"""ctypes binding of libhivis.so: the same entry points as include/hivis.h, argument
marshalling only.  Every step of the draft-verify path runs inside the library's HIP
kernels; there is no Python or CPU fallback -- if the library is missing, loading fails.
"""
import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libhivis.so")

HIVIS_OK, HIVIS_EINVAL, HIVIS_ESTATE, HIVIS_ECAP, HIVIS_EHIP = 0, -1, -2, -3, -4
HIVIS_F32, HIVIS_BF16 = 0, 1

LAYER_FIELDS = ("norm1", "wq", "wk", "wv", "wo", "norm2", "wg", "wu", "wd")
LAYER_OPTIONAL = ("bq", "bk", "bv")          # q/k/v projection biases: all three or none


class HivisError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"hivis error {code}: {msg}")
        self.code = code


class hivis_config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("ffn", C.c_int32), ("vocab", C.c_int32), ("dtype", C.c_int32),
                ("batch", C.c_int32), ("k_max", C.c_int32), ("max_vis", C.c_int32), ("max_text", C.c_int32),
                ("rope_theta", C.c_float), ("rms_eps", C.c_float), ("n_resid", C.c_int32)]


class hivis_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in LAYER_FIELDS + LAYER_OPTIONAL]


class hivis_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("layers", C.POINTER(hivis_layer_weights)), ("draft_layer", hivis_layer_weights),
                ("fuse_w", C.c_void_p), ("resid_rho", C.c_void_p)]


_lib = None


def load_library(path=LIB_PATH):
    """Loads libhivis.so (build it first with paper_2509_23928_amd.build.build())."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} not built: run `python -m paper_2509_23928_amd.build` (hipcc, gfx950)")
    lib = C.CDLL(path)
    P, I32 = C.c_void_p, C.c_int32
    sig = {
        "hivis_create": (C.c_int, [C.POINTER(hivis_config), C.POINTER(hivis_weights), P, C.POINTER(P)]),
        "hivis_destroy": (C.c_int, [P]),
        "hivis_prefill": (C.c_int, [P, P, I32, P, I32, P]),
        "hivis_draft": (C.c_int, [P, I32]),
        "hivis_draft_noalloc": (C.c_int, [P, I32]),
        "hivis_set_drafts": (C.c_int, [P, P, I32]),
        "hivis_verify": (C.c_int, [P]),
        "hivis_accept": (C.c_int, [P, P, P]),
        "hivis_prefill_sample": (C.c_int, [P, P, I32, P, I32, C.c_float, P, P]),
        "hivis_draft_sample": (C.c_int, [P, I32, C.c_float, P]),
        "hivis_accept_sample": (C.c_int, [P, C.c_float, P, P, P, P]),
        "hivis_rng_seed": (C.c_int, [P, C.c_uint64, P]),
        "hivis_tree_draft": (C.c_int, [P, I32, I32, I32]),
        "hivis_tree_set": (C.c_int, [P, I32, P, P]),
        "hivis_tree_verify": (C.c_int, [P]),
        "hivis_tree_accept": (C.c_int, [P, P, P]),
        "hivis_tree_accept_sample": (C.c_int, [P, C.c_float, P, P, P]),
        "hivis_tree_get": (C.c_int, [P, P, P, P, P, P, P, P, P, P]),
        "hivis_tree_get_logits": (C.c_int, [P, P]),
        "hivis_get_logits": (C.c_int, [P, I32, P]),
        "hivis_get_hidden": (C.c_int, [P, I32, P]),
        "hivis_kv_lengths": (C.c_int, [P, P, P]),
        "hivis_get_tokens": (C.c_int, [P, P, P]),
        "hivis_timing": (C.c_int, [P, I32]),
        "hivis_phase_ms": (C.c_int, [P, I32, C.POINTER(C.c_double), C.POINTER(C.c_int64)]),
        "hivis_kernel_timing": (C.c_int, [P, I32]),
        "hivis_kernel_ms": (C.c_int, [P, C.POINTER(C.c_double), C.POINTER(C.c_int64), C.POINTER(C.c_double)]),
        "hivis_algorithmic_bytes": (C.c_int, [P, C.POINTER(C.c_double), C.POINTER(C.c_double)]),
        "hivis_clamp_token": (I32, [I32, I32]),
        "hivis_calib_stream": (C.c_int, [P, C.c_int64, I32, I32, I32, C.POINTER(C.c_double), C.POINTER(C.c_double)]),
        "hivis_last_error": (C.c_char_p, [P]),
        "hivis_version": (C.c_char_p, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


EXPORTED_SYMBOLS = ("hivis_create", "hivis_destroy", "hivis_prefill", "hivis_draft", "hivis_draft_noalloc", "hivis_set_drafts",
                    "hivis_verify", "hivis_accept", "hivis_prefill_sample", "hivis_draft_sample", "hivis_accept_sample", "hivis_rng_seed", "hivis_tree_draft", "hivis_tree_set", "hivis_tree_verify", "hivis_tree_accept", "hivis_tree_accept_sample", "hivis_tree_get", "hivis_tree_get_logits", "hivis_get_logits", "hivis_get_hidden", "hivis_kv_lengths",
                    "hivis_get_tokens", "hivis_timing", "hivis_phase_ms", "hivis_kernel_timing", "hivis_kernel_ms", "hivis_algorithmic_bytes", "hivis_clamp_token", "hivis_calib_stream",
                    "hivis_last_error", "hivis_version")


def _ptr(a):
    """Address of a numpy array (host) or of anything with data_ptr() (a torch tensor, host or device)."""
    if a is None:
        return None
    if hasattr(a, "data_ptr"):
        return C.c_void_p(a.data_ptr())
    assert a.flags["C_CONTIGUOUS"]
    return C.c_void_p(a.ctypes.data)


def _host_weight(a, dtype):
    """Host array in the library's storage type: float32, or uint16 bf16 bit patterns."""
    a = np.asarray(a)
    if dtype == HIVIS_BF16:
        if a.dtype == np.uint16:
            return np.ascontiguousarray(a)
        assert a.dtype == np.float32
        bits = a.view(np.uint32)
        assert not np.any(bits & np.uint32(0xFFFF)), "float32 weights of a bf16 model must hold bf16-representable values"
        return np.ascontiguousarray((bits >> np.uint32(16)).astype(np.uint16))
    return np.ascontiguousarray(a, dtype=np.float32)


def calib_stream(buffer_bytes, n_buffers, passes, workgroups=1024, stream=None):
    """hivis_calib_stream: (GB/s, us per launch) of a plain read-only streaming kernel over rotating buffers."""
    lib = load_library()
    gbs, us = C.c_double(), C.c_double()
    rc = lib.hivis_calib_stream(C.c_void_p(stream or 0), int(buffer_bytes), int(n_buffers), int(passes), int(workgroups), C.byref(gbs), C.byref(us))
    if rc:
        raise HivisError(rc, "hivis_calib_stream failed")
    return gbs.value, us.value


class Hivis:
    """One library context.  Method names mirror the C entry points."""

    def __init__(self, cfg, weights, *, max_vis=None, max_text=None, k_max=None, batch=None, stream=None):
        self.lib = load_library()
        self.cfg = cfg
        dt = HIVIS_BF16 if cfg.dtype == "bf16" else HIVIS_F32
        self.dtype = dt
        self.B = cfg.batch if batch is None else batch
        self.k_max = cfg.K if k_max is None else k_max
        gen = cfg.gen_tokens if cfg.gen_tokens else cfg.gen_cycles * (self.k_max + 1)
        self.max_vis = cfg.n_vis if max_vis is None else max_vis
        self.max_text = (cfg.n_text + gen + 2 * (self.k_max + 2)) if max_text is None else max_text
        c = hivis_config(cfg.n_layers, cfg.d, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.ffn, cfg.vocab, dt,
                         self.B, self.k_max, self.max_vis, self.max_text, cfg.rope_theta, cfg.rms_eps, cfg.n_resid)
        keep = []

        def hw(a):
            h = _host_weight(a, dt)
            keep.append(h)
            return C.c_void_p(h.ctypes.data)

        def layer(lw):
            return hivis_layer_weights(*([hw(lw[n]) for n in LAYER_FIELDS] + [hw(lw[n]) if n in lw else None for n in LAYER_OPTIONAL]))

        layers = (hivis_layer_weights * cfg.n_layers)(*[layer(lw) for lw in weights["layers"]])
        w = hivis_weights(hw(weights["embed"]), hw(weights["lm_head"]), hw(weights["final_norm"]), layers,
                          layer(weights["draft_layer"]), hw(weights["fuse_w"]), hw(weights["resid_rho"]))
        self.ctx = C.c_void_p()
        rc = self.lib.hivis_create(C.byref(c), C.byref(w), C.c_void_p(stream or 0), C.byref(self.ctx))
        if rc:
            raise HivisError(rc, self.lib.hivis_last_error(None).decode())
        self.K = 0

    def _check(self, rc):
        if rc:
            raise HivisError(rc, self.lib.hivis_last_error(self.ctx).decode())

    def close(self):
        if getattr(self, "ctx", None):
            self.lib.hivis_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the four calls ------------------------------------------------------------
    def prefill(self, vis_embeds, text_ids):
        """vis_embeds [B][v][d] (numpy float32/uint16, or a torch tensor on host or device in the storage
        dtype), text_ids [B][l] int32.  Returns first tokens [B]."""
        if isinstance(vis_embeds, np.ndarray):
            vis_embeds = _host_weight(vis_embeds, self.dtype)
        if isinstance(text_ids, np.ndarray):
            text_ids = np.ascontiguousarray(text_ids, dtype=np.int32)
        v, l = int(vis_embeds.shape[-2]), int(text_ids.shape[-1])
        first = np.zeros(self.B, np.int32)
        self._check(self.lib.hivis_prefill(self.ctx, _ptr(vis_embeds), v, _ptr(text_ids), l, _ptr(first)))
        return first

    def rng_seed(self, seed):
        """Seeds the device-side generator; afterwards the sampling calls accept None for their uniforms.  Returns the
        number of drawing calls made since the previous seeding."""
        calls = C.c_uint64(0)
        self._check(self.lib.hivis_rng_seed(self.ctx, C.c_uint64(int(seed) & 0xFFFFFFFFFFFFFFFF), C.byref(calls)))
        return int(calls.value)

    def prefill_sample(self, vis_embeds, text_ids, temperature, u_first=None):
        """prefill() with the first token of every sequence drawn at `temperature` with u_first [B] (None: drawn on the device)."""
        if isinstance(vis_embeds, np.ndarray):
            vis_embeds = _host_weight(vis_embeds, self.dtype)
        if isinstance(text_ids, np.ndarray):
            text_ids = np.ascontiguousarray(text_ids, dtype=np.int32)
        v, l = int(vis_embeds.shape[-2]), int(text_ids.shape[-1])
        u = None if u_first is None else np.ascontiguousarray(u_first, dtype=np.float32).reshape(self.B)
        first = np.zeros(self.B, np.int32)
        self._check(self.lib.hivis_prefill_sample(self.ctx, _ptr(vis_embeds), v, _ptr(text_ids), l, float(temperature), _ptr(u), _ptr(first)))
        return first

    def draft(self, K):
        self._check(self.lib.hivis_draft(self.ctx, K))
        self.K = K

    def draft_noalloc(self, K):
        """draft() with every intermediate buffer in the library's static scratch array (no device allocation)."""
        self._check(self.lib.hivis_draft_noalloc(self.ctx, K))
        self.K = K

    def set_drafts(self, tokens):
        t = np.ascontiguousarray(tokens, dtype=np.int32).reshape(self.B, -1)
        self._check(self.lib.hivis_set_drafts(self.ctx, _ptr(t), t.shape[1]))
        self.K = t.shape[1]

    def verify(self):
        self._check(self.lib.hivis_verify(self.ctx))

    def accept(self):
        """Returns (n_accepted [B], tokens [B][k_max+1], -1 beyond n_b+1 entries)."""
        n = np.zeros(self.B, np.int32)
        t = np.zeros((self.B, self.k_max + 1), np.int32)
        self._check(self.lib.hivis_accept(self.ctx, _ptr(n), _ptr(t)))
        return n, t

    def draft_sample(self, K, temperature, u=None):
        """u: [B][K] uniform numbers in [0, 1) (None after rng_seed: drawn on the device)."""
        u = None if u is None else np.ascontiguousarray(u, dtype=np.float32).reshape(self.B, K)
        self._check(self.lib.hivis_draft_sample(self.ctx, K, float(temperature), _ptr(u)))
        self.K = K

    def accept_sample(self, temperature, u_accept=None, u_resample=None):
        """u_accept: [B][K], u_resample: [B] (both None after rng_seed: drawn on the device).  Returns (n_accepted [B], tokens [B][k_max+1])."""
        ua = None if u_accept is None else np.ascontiguousarray(u_accept, dtype=np.float32).reshape(self.B, self.K)
        ur = None if u_resample is None else np.ascontiguousarray(u_resample, dtype=np.float32).reshape(self.B)
        n = np.zeros(self.B, np.int32)
        t = np.zeros((self.B, self.k_max + 1), np.int32)
        self._check(self.lib.hivis_accept_sample(self.ctx, float(temperature), _ptr(ua), _ptr(ur), _ptr(n), _ptr(t)))
        return n, t

    # -- draft tree (batch 1) -----------------------------------------------------------
    def tree_draft(self, top_k, depth, n_nodes):
        self._check(self.lib.hivis_tree_draft(self.ctx, int(top_k), int(depth), int(n_nodes)))
        self.tree_shape = (int(top_k), int(depth), int(n_nodes))
        self.K = int(n_nodes)            # rows of the coming verify pass = n_nodes + 1 (get_logits / get_hidden shapes)

    def tree_set(self, tokens, parents):
        """Plants the candidates: tokens / parents [n_nodes], parents as verify-row indices (0 = root)."""
        tok = np.ascontiguousarray(tokens, dtype=np.int32)
        par = np.ascontiguousarray(parents, dtype=np.int32)
        self._check(self.lib.hivis_tree_set(self.ctx, len(tok), _ptr(tok), _ptr(par)))
        depth = {0: 0}
        for i, p in enumerate(par, start=1):
            depth[i] = depth[int(p)] + 1
        self.tree_shape = (0, max(depth.values()), len(tok))
        self.K = len(tok)

    def tree_verify(self):
        self._check(self.lib.hivis_tree_verify(self.ctx))

    def tree_accept(self):
        """Returns (n_accepted, tokens [depth+1], -1 beyond n+1 entries)."""
        n = np.zeros(1, np.int32)
        t = np.zeros(self.tree_shape[1] + 1, np.int32)
        self._check(self.lib.hivis_tree_accept(self.ctx, _ptr(n), _ptr(t)))
        return int(n[0]), t

    def tree_accept_sample(self, temperature, u=None):
        """tree_accept() with the target's tokens drawn at `temperature`; u: [depth+1] uniforms, one per depth (None after
        rng_seed: drawn on the device).  Returns (n_accepted, tokens [depth+1])."""
        n = np.zeros(1, np.int32)
        t = np.zeros(self.tree_shape[1] + 1, np.int32)
        uu = None if u is None else np.ascontiguousarray(u, dtype=np.float32).reshape(self.tree_shape[1] + 1)
        self._check(self.lib.hivis_tree_accept_sample(self.ctx, float(temperature), _ptr(uu), _ptr(n), _ptr(t)))
        return int(n[0]), t

    def tree_get(self, verified=False):
        """The last tree as a dict of host arrays (target_tokens only if verified)."""
        k, depth, N = self.tree_shape
        P = k + (depth - 1) * k * k
        if k == 0:        # planted tree: rows only
            out = {"row_tokens": np.zeros(N + 1, np.int32), "row_parents": np.zeros(N + 1, np.int32), "row_depths": np.zeros(N + 1, np.int32)}
            tt = np.zeros(N + 1, np.int32) if verified else None
            self._check(self.lib.hivis_tree_get(self.ctx, None, None, None, None, None, _ptr(out["row_tokens"]), _ptr(out["row_parents"]),
                                                _ptr(out["row_depths"]), _ptr(tt)))
            if verified:
                out["target_tokens"] = tt
            return out
        out = {"pool_tokens": np.zeros(P, np.int32), "pool_parents": np.zeros(P, np.int32), "pool_scores": np.zeros(P, np.float32),
               "expand": np.zeros((depth - 1, k), np.int32), "selected": np.zeros(N, np.int32), "row_tokens": np.zeros(N + 1, np.int32),
               "row_parents": np.zeros(N + 1, np.int32), "row_depths": np.zeros(N + 1, np.int32)}
        tt = np.zeros(N + 1, np.int32) if verified else None
        self._check(self.lib.hivis_tree_get(self.ctx, _ptr(out["pool_tokens"]), _ptr(out["pool_parents"]), _ptr(out["pool_scores"]),
                                            _ptr(out["expand"]) if depth > 1 else None, _ptr(out["selected"]), _ptr(out["row_tokens"]),
                                            _ptr(out["row_parents"]), _ptr(out["row_depths"]), _ptr(tt)))
        if verified:
            out["target_tokens"] = tt
        return out

    def tree_get_logits(self):
        k, depth, _ = self.tree_shape
        out = np.zeros((1 + (depth - 1) * k, self.cfg.vocab), np.float32)
        self._check(self.lib.hivis_tree_get_logits(self.ctx, _ptr(out)))
        return out

    # -- hooks -----------------------------------------------------------------------
    def get_logits(self, which):
        V = self.cfg.vocab
        shape = {0: (self.B, self.K + 1, V), 1: (self.K, self.B, V), 2: (self.B, V)}[which]
        out = np.zeros(shape, np.float32)
        self._check(self.lib.hivis_get_logits(self.ctx, which, _ptr(out)))
        return out

    def get_hidden(self, which):
        shape = {0: (self.B, self.K + 1, self.cfg.d), 1: (self.B, self.cfg.d)}[which]
        out = np.zeros(shape, np.float32)
        self._check(self.lib.hivis_get_hidden(self.ctx, which, _ptr(out)))
        return out

    def kv_lengths(self):
        t = np.zeros(self.B, np.int32)
        d = np.zeros(self.B, np.int32)
        self._check(self.lib.hivis_kv_lengths(self.ctx, _ptr(t), _ptr(d)))
        return t, d

    def get_tokens(self):
        dr = np.zeros((self.B, self.K), np.int32)
        tt = np.zeros((self.B, self.K + 1), np.int32)
        self._check(self.lib.hivis_get_tokens(self.ctx, _ptr(dr), _ptr(tt)))
        return dr, tt

    def timing(self, enable):
        self._check(self.lib.hivis_timing(self.ctx, int(enable)))

    def phase_ms(self, phase):
        ms, calls = C.c_double(), C.c_int64()
        self._check(self.lib.hivis_phase_ms(self.ctx, phase, C.byref(ms), C.byref(calls)))
        return ms.value, calls.value

    def kernel_timing(self, gemm_kind):
        self._check(self.lib.hivis_kernel_timing(self.ctx, int(gemm_kind)))

    def kernel_ms(self):
        ms, n, by = C.c_double(), C.c_int64(), C.c_double()
        self._check(self.lib.hivis_kernel_ms(self.ctx, C.byref(ms), C.byref(n), C.byref(by)))
        return ms.value, n.value, by.value

    def algorithmic_bytes(self):
        a, b = C.c_double(), C.c_double()
        self._check(self.lib.hivis_algorithmic_bytes(self.ctx, C.byref(a), C.byref(b)))
        return a.value, b.value

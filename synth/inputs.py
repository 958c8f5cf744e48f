"""Counter-based seeded generators for weights and prompts.

Every tensor has its own Philox stream keyed by (seed, tensor id), so any single
tensor of a large model can be regenerated without drawing the others.  Weights
are returned as float32 arrays; for "bf16" configs their values are already
rounded to bf16 (round-to-nearest-even), so that a consumer storing them in
bf16 and a consumer reading them as float32 see the same numbers.

Recipe: matrices N(0, 0.02); norm gains 1 + 0.1*N(0,1) (so that a forgotten
gain shows); residual vectors rho_i N(0, 0.02); visual embeddings N(0, 1);
text ids uniform in [0, vocab); for configs with qkv_bias, bias vectors bq, bk, bv
N(0, 0.5) per layer (large enough that a dropped or misplaced bias shows).

Matrix orientation is the paper's row-vector convention y = x W, i.e. W is
[in][out], except the embedding table and LM head, which are [vocab][d].
"""
import zlib
import numpy as np

# tensors of one decoder layer, in the order the C-ABI expects them
TENSOR_ORDER_LAYER = ("norm1", "wq", "wk", "wv", "wo", "norm2", "wg", "wu", "wd")


def tensor_rng(seed: int, name: str) -> np.random.Generator:
    key = zlib.crc32(name.encode()) & 0xFFFFFFFF
    return np.random.Generator(np.random.Philox(key=[int(seed) & 0xFFFFFFFFFFFFFFFF, key]))


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = u >> np.uint32(16)
    r &= np.uint32(1)
    r += np.uint32(0x7FFF)
    r += u
    r >>= np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(to_bf16_bits(x)).reshape(x.shape)


def _normal(seed, name, shape, std, dtype, mean=0.0, bits=False):
    """One tensor.  dtype "bf16": values rounded to bf16; returned as float32, or as
    the uint16 bit patterns when bits=True (half the host memory for 7B-13B shapes)."""
    w = tensor_rng(seed, name).standard_normal(shape, dtype=np.float32)
    w *= np.float32(std)
    if mean:
        w += np.float32(mean)
    if dtype == "bf16":
        b = to_bf16_bits(w).reshape(shape)
        return b if bits else bf16_bits_to_f32(b).reshape(shape)
    return w


def layer_shapes(cfg):
    d, F = cfg.d, cfg.ffn
    return {"norm1": (d,), "wq": (d, cfg.q_dim), "wk": (d, cfg.kv_dim), "wv": (d, cfg.kv_dim),
            "wo": (cfg.q_dim, d), "norm2": (d,), "wg": (d, F), "wu": (d, F), "wd": (F, d)}


def _tensor_specs(cfg):
    """(path, rng name, shape, std, mean) of every tensor of target + drafter."""
    specs = [(("embed",), "embed", (cfg.vocab, cfg.d), 0.02, 0.0),
             (("lm_head",), "lm_head", (cfg.vocab, cfg.d), 0.02, 0.0),
             (("final_norm",), "final_norm", (cfg.d,), 0.1, 1.0),
             (("fuse_w",), "fuse_w", (2 * cfg.d, cfg.d), 0.02, 0.0),
             (("resid_rho",), "resid_rho", (cfg.n_resid, cfg.d), 0.02, 0.0)]
    prefixes = [(("layers", i), f"layers.{i}") for i in range(cfg.n_layers)] + [(("draft_layer",), "drafter")]
    for path, prefix in prefixes:
        for name, shape in layer_shapes(cfg).items():
            is_norm = name.startswith("norm")
            specs.append((path + (name,), f"{prefix}.{name}", shape, 0.1 if is_norm else 0.02,
                          1.0 if is_norm else 0.0))
        if getattr(cfg, "qkv_bias", False):
            for name, n in (("bq", cfg.q_dim), ("bk", cfg.kv_dim), ("bv", cfg.kv_dim)):
                specs.append((path + (name,), f"{prefix}.{name}", (n,), 0.5, 0.0))
    return specs


def make_weights(cfg, seed=0, bits=False, threads=1):
    """dict: embed [V][d], lm_head [V][d], final_norm [d], layers [N]{...},
    draft_layer {...}, fuse_w [2d][d] (= [w1; w2]), resid_rho [n_resid][d].
    With cfg.qkv_bias every layer dict also holds bq [q_dim], bk [kv_dim], bv [kv_dim].
    bits=True (bf16 configs only): uint16 bf16 bit patterns instead of float32."""
    w = {"layers": [dict() for _ in range(cfg.n_layers)], "draft_layer": {}}

    def put(path, arr):
        node = w
        for p in path[:-1]:
            node = node[p]
        node[path[-1]] = arr

    specs = _tensor_specs(cfg)

    def gen(spec):
        path, name, shape, std, mean = spec
        return path, _normal(seed, name, shape, std, cfg.dtype, mean=mean, bits=bits)

    if threads > 1:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(threads) as ex:
            for path, arr in ex.map(gen, specs):
                put(path, arr)
    else:
        for spec in specs:
            put(*gen(spec))
    return w


def make_prompt(cfg, seed=0, batch=None):
    """vis_embeds [B][v][d] float32 (bf16-rounded for bf16 configs), text_ids [B][l] int32.
    Sequence b uses seed+b (independent prompts)."""
    B = cfg.batch if batch is None else batch
    vis = np.stack([_normal(seed + b, "vis_embeds", (cfg.n_vis, cfg.d), 1.0, cfg.dtype) for b in range(B)])
    ids = np.stack([tensor_rng(seed + b, "text_ids").integers(0, cfg.vocab, size=cfg.n_text, dtype=np.int32)
                    for b in range(B)])
    return vis, ids

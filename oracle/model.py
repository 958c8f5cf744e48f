"""CPU oracle, part 1: the decoder arithmetic (float64, numpy).

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain reference that the HIP
library is checked against.  Only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py may import it; the product path never does, and this
package never imports the HIP binding.

Everything is computed in float64 from the float32 (or bf16-rounded) weight values
it is given; nothing is blocked, fused or reordered.

What is modelled (paper section 3.2, "The overall framework"): the target VLM M_p
is a stack of N decoder layers, each doing causal self-attention over the one
sequence [visual embeddings ; text embeddings]; the final-layer outputs at the
text positions are the fused features f_fused.  The paper does not spell out the
decoder block; this oracle uses the block of the model families it evaluates
(section 4, "Models and Tasks": LLaVA-1.5 / LLaVA-NeXT / Qwen2.5-VL, i.e.
LLaMA-style pre-norm blocks): RMSNorm, rotary position embedding with rotate-half
pairing, grouped-query softmax attention, SwiGLU MLP; no biases, except the q/k/v
projection biases of the Qwen2.5 language model, which a layer's weight dict may carry
as bq, bk, bv (added to the projections before the rotation).

Orientation: y = x W with W stored [in][out] (the paper's row-vector notation,
e.g. "f_fused w_1"), except embed and lm_head, which are [vocab][d].
"""
import numpy as np

F64 = np.float64


def rmsnorm(x, gain, eps):
    """x * gain / sqrt(mean(x^2) + eps), over the last axis."""
    x = np.asarray(x, F64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x * np.asarray(gain, F64) / np.sqrt(ms + eps)


def rope(x, pos, theta):
    """Rotary embedding, rotate-half pairing: element i is paired with i + hd/2 and the
    pair is rotated by the angle pos * theta^(-2i/hd).
    x: [rows][heads][hd], pos: [rows] integer positions."""
    x = np.asarray(x, F64)
    hd = x.shape[-1]
    half = hd // 2
    inv_freq = F64(theta) ** (-2.0 * np.arange(half, dtype=F64) / hd)
    ang = np.asarray(pos, F64)[:, None] * inv_freq[None, :]          # [rows][half]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    x1 = x[..., :half]
    x2 = x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def softmax_rows(s):
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def attention(q, k, v, q_pos, k_pos, visible=None):
    """Causal grouped-query attention.
    q: [m][Hq][hd]; k, v: [n][Hkv][hd]; q_pos [m], k_pos [n] integer positions.
    Query at position p sees exactly the keys at positions <= p.
    Query head h reads kv head h // (Hq / Hkv).  Returns [m][Hq][hd].
    visible: optional boolean [m][n] that REPLACES the position rule (rows of a draft tree see their
    ancestors only, whatever the positions say)."""
    q = np.asarray(q, F64)
    k = np.asarray(k, F64)
    v = np.asarray(v, F64)
    m, Hq, hd = q.shape
    Hkv = k.shape[1]
    group = Hq // Hkv
    if visible is None:
        visible = np.asarray(k_pos)[None, :] <= np.asarray(q_pos)[:, None]  # [m][n]
    visible = np.asarray(visible, bool)
    assert visible.shape == (m, k.shape[0])
    out = np.empty((m, Hq, hd), F64)
    for h in range(Hq):
        g = h // group
        s = (q[:, h, :] @ k[:, g, :].T) / np.sqrt(F64(hd))
        s = np.where(visible, s, -np.inf)
        out[:, h, :] = softmax_rows(s) @ v[:, g, :]
    return out


def silu(x):
    return x / (1.0 + np.exp(-x))


class KVCache:
    """Keys (after RoPE) and values of one layer for one sequence, with their positions."""

    def __init__(self, n_kv_heads, head_dim):
        self.k = np.zeros((0, n_kv_heads, head_dim), F64)
        self.v = np.zeros((0, n_kv_heads, head_dim), F64)
        self.pos = np.zeros((0,), np.int64)

    def __len__(self):
        return self.k.shape[0]

    def append(self, k, v, pos):
        self.k = np.concatenate([self.k, k], axis=0)
        self.v = np.concatenate([self.v, v], axis=0)
        self.pos = np.concatenate([self.pos, np.asarray(pos, np.int64)])

    def truncate(self, n):
        self.k = self.k[:n]
        self.v = self.v[:n]
        self.pos = self.pos[:n]

    def keep(self, idx):
        """Keep exactly the entries idx (in that order)."""
        idx = np.asarray(idx, np.int64)
        self.k = self.k[idx]
        self.v = self.v[idx]
        self.pos = self.pos[idx]


def decoder_layer(h, w, cache, pos, cfg, visible=None):
    """One pre-norm decoder block on the rows h [m][d] at positions pos [m]; the rows'
    keys/values are appended to `cache`, and every row attends to all cached entries at
    positions <= its own (or, if `visible` [m][len(cache) + m] is given, to exactly the
    entries it marks).  w: dict with norm1, wq, wk, wv, wo, norm2, wg, wu, wd and optionally bq, bk, bv."""
    h = np.asarray(h, F64)
    m = h.shape[0]
    a = rmsnorm(h, w["norm1"], cfg.rms_eps)
    q = a @ np.asarray(w["wq"], F64)
    k = a @ np.asarray(w["wk"], F64)
    v = a @ np.asarray(w["wv"], F64)
    if "bq" in w:            # q/k/v projection biases (the Qwen2.5 language model has them), added before the rotation
        q = q + np.asarray(w["bq"], F64)
        k = k + np.asarray(w["bk"], F64)
        v = v + np.asarray(w["bv"], F64)
    q = q.reshape(m, cfg.n_q_heads, cfg.head_dim)
    k = k.reshape(m, cfg.n_kv_heads, cfg.head_dim)
    v = v.reshape(m, cfg.n_kv_heads, cfg.head_dim)
    q = rope(q, pos, cfg.rope_theta)
    k = rope(k, pos, cfg.rope_theta)
    cache.append(k, v, pos)
    o = attention(q, cache.k, cache.v, pos, cache.pos, visible).reshape(m, cfg.q_dim)
    h = h + o @ np.asarray(w["wo"], F64)
    b = rmsnorm(h, w["norm2"], cfg.rms_eps)
    gate = b @ np.asarray(w["wg"], F64)
    up = b @ np.asarray(w["wu"], F64)
    h = h + (silu(gate) * up) @ np.asarray(w["wd"], F64)
    return h


def lm_logits(f, lm_head):
    """logits[j] = f . lm_head[j]"""
    return np.asarray(f, F64) @ np.asarray(lm_head, F64).T


def argmax_lowest(logits):
    """Greedy token: index of the maximum, lowest index on exact ties (numpy's rule)."""
    return np.argmax(logits, axis=-1)


class Target:
    """The target VLM M_p for one sequence: embedding table, N decoder layers, final norm,
    LM head, and its KV cache over visual + text positions."""

    def __init__(self, cfg, weights):
        self.cfg = cfg
        self.w = weights
        self.caches = [KVCache(cfg.n_kv_heads, cfg.head_dim) for _ in range(cfg.n_layers)]

    @property
    def kv_len(self):
        return len(self.caches[0])

    def embed(self, ids):
        return np.asarray(self.w["embed"], F64)[np.asarray(ids, np.int64)]

    def forward(self, x, start_pos, pos=None, visible=None):
        """Run the rows x [m][d] (already embedded) at positions start_pos..start_pos+m-1
        through all layers; returns the final-layer features after the final norm [m][d]
        (the tensor the LM head reads; this is what is used as f_fused).
        pos / visible: explicit positions and visibility for the rows of a draft tree."""
        m = x.shape[0]
        if pos is None:
            pos = np.arange(start_pos, start_pos + m)
        h = np.asarray(x, F64)
        for i in range(self.cfg.n_layers):
            h = decoder_layer(h, self.w["layers"][i], self.caches[i], pos, self.cfg, visible)
        return rmsnorm(h, self.w["final_norm"], self.cfg.rms_eps)

    def logits(self, f):
        return lm_logits(f, self.w["lm_head"])

    def truncate(self, n):
        for c in self.caches:
            c.truncate(n)

    def keep(self, idx):
        for c in self.caches:
            c.keep(idx)


class Drafter:
    """The drafter M_q: ONE decoder layer with its own weights whose output goes straight
    to the target's LM head, over a KV cache that holds text positions only.  It has no
    access to the target's cache: the only thing it ever receives is its input rows."""

    def __init__(self, cfg, weights):
        self.cfg = cfg
        self.w = weights
        self.cache = KVCache(cfg.n_kv_heads, cfg.head_dim)

    @property
    def kv_len(self):
        return len(self.cache)

    def forward(self, u, start_pos, pos=None, visible=None):
        m = u.shape[0]
        if pos is None:
            pos = np.arange(start_pos, start_pos + m)
        return decoder_layer(u, self.w["draft_layer"], self.cache, pos, self.cfg, visible)

    def truncate(self, n):
        self.cache.truncate(n)

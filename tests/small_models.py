"""Small model shapes used by several tests (built on the shared seeded generators)."""
import synth


def tiny_cfg(**kw):
    base = dict(name="tiny", n_layers=2, d=48, n_q_heads=6, n_kv_heads=2, head_dim=8, ffn=80, vocab=97,
                dtype="f32", n_vis=7, n_text=5, K=3, batch=1, gen_tokens=0, gen_cycles=4)
    base.update(kw)
    return synth.HivisConfig(**base)

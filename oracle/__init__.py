"""Plain CPU oracle of the HiViS draft-verify path (float64 numpy).

TEST INFRASTRUCTURE ONLY: imported by tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py, never by the product path, and it imports nothing of
the HIP library.
"""
from .model import (rmsnorm, rope, softmax_rows, attention, silu, KVCache, decoder_layer, lm_logits,
                    argmax_lowest, Target, Drafter)
from .hivis import (fuse, accept_length, HivisOracle, greedy_reference, top2_gap, softmax_temperature, sample_inverse_cdf,
                    speculative_accept, HivisSamplingOracle, sampling_reference)
from .tree import (HivisTreeOracle, log_softmax, top_k_lowest, pool_size, ancestors_visible, accept_path, sample_tree_tokens)
from . import rng

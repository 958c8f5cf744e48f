/*
 * hivis.h -- C ABI of the HiViS draft-verify decode path on one MI355X (gfx950).
 *
 * The calls follow the paper's statement of the procedure (Algorithm 1, "Residual-Aided
 * Drafting and Verification Process", and section 3.2): the target VLM M_p is prefilled on
 * [visual embeddings ; text embeddings]; its final-layer features at the text positions
 * (f_fused) are fused with the causally shifted token embeddings by one FC (2d -> d),
 * get a step-dependent residual vector added, and feed a one-layer drafter M_q that keeps
 * a TEXT-ONLY KV cache; the drafter proposes K tokens autoregressively; the target scores
 * them in one pass against its visual+text cache; the longest matching prefix plus the
 * target's own next token is accepted (section 2.1).
 *
 * Conventions
 *   - Every function returns 0 (HIVIS_OK) or a negative HIVIS_E* code; none throws or aborts.
 *     hivis_last_error() returns a human-readable message for the last failure on a context.
 *   - "host" / "device" on a pointer says where the memory must live.  Pointers marked
 *     "host or device" may be either (they are read with a default-kind hipMemcpy).
 *   - The caller owns every buffer it passes; the library copies what it needs before the call
 *     returns (weights at create; prompts at prefill) and owns all device state of a context.
 *   - dtype: HIVIS_F32 = IEEE float32; HIVIS_BF16 = bfloat16 bit patterns (uint16_t).  It is the
 *     storage type of weights, embedding tables and vis_embeds.  The KV caches are float32 for
 *     HIVIS_F32; for HIVIS_BF16 every cached value is a pair of IEEE halves hi + lo (4 bytes, ~22
 *     mantissa bits; one half alone put the drafter's logits outside the parity tolerance at 32
 *     layers).  Activations between kernels and all accumulation are float32.
 *   - Matrix orientation is the paper's row-vector form y = x W: W is [in][out] row-major,
 *     except embed and lm_head, which are [vocab][d] row-major.
 *   - Work is enqueued on the hipStream_t given at create.  hivis_accept, hivis_prefill (for
 *     its first_token output) and the hivis_get_* / hivis_kv_lengths hooks synchronise that stream;
 *     hivis_draft and hivis_verify only enqueue.
 *   - A context is not thread-safe; use one per host thread.
 *   - Shape limits: d, n_q_heads*head_dim, n_kv_heads*head_dim, ffn and vocab must be multiples
 *     of 32 (16 for HIVIS_F32); head_dim is 64 or 128; batch*(k_max+1) <= 32.
 */
#ifndef HIVIS_H
#define HIVIS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HIVIS_OK       0
#define HIVIS_EINVAL  -1   /* null pointer, bad dimension, K out of range, token id >= vocab */
#define HIVIS_ESTATE  -2   /* call out of order (draft before prefill, accept before verify, ...) */
#define HIVIS_ECAP    -3   /* v, l or the generated length exceeds the capacity given at create */
#define HIVIS_EHIP    -4   /* HIP runtime error; see hivis_last_error */

#define HIVIS_F32  0
#define HIVIS_BF16 1

typedef struct hivis_ctx hivis_ctx;   /* opaque; created by hivis_create, freed by hivis_destroy */

typedef struct {
    int32_t n_layers;      /* N: decoder layers of the target (the drafter has exactly one) */
    int32_t d;             /* hidden size */
    int32_t n_q_heads, n_kv_heads, head_dim;
    int32_t ffn;           /* SwiGLU inner width */
    int32_t vocab;
    int32_t dtype;         /* HIVIS_F32 or HIVIS_BF16 */
    int32_t batch;         /* B independent sequences, same v and same prompt length */
    int32_t k_max;         /* largest chain draft length K that will be requested */
    int32_t max_vis;       /* capacity: visual embeddings per sequence */
    int32_t max_text;      /* capacity: text tokens per sequence (prompt + everything generated + k_max + 1) */
    float   rope_theta;
    float   rms_eps;
    int32_t n_resid;       /* number of residual vectors rho_0..rho_{n_resid-1}; the last is reused (section 4: r^3) */
} hivis_config;

/* Weights of one decoder layer, all host pointers of the context's dtype:
 * norm1 [d], wq [d][Hq*hd], wk [d][Hkv*hd], wv [d][Hkv*hd], wo [Hq*hd][d],
 * norm2 [d], wg [d][ffn], wu [d][ffn], wd [ffn][d].
 * bq [Hq*hd], bk [Hkv*hd], bv [Hkv*hd]: optional bias vectors of the q/k/v projections (the Qwen2.5 language model of
 * section 4's Qwen2.5-VL has them), added before the rotation; all three NULL (no biases) or all three given. */
typedef struct {
    const void *norm1, *wq, *wk, *wv, *wo, *norm2, *wg, *wu, *wd;
    const void *bq, *bk, *bv;
} hivis_layer_weights;

typedef struct {
    const void *embed;                  /* [vocab][d]; shared by target and drafter */
    const void *lm_head;                /* [vocab][d]; shared by target and drafter (Algorithm 1: "LM Head(f')") */
    const void *final_norm;             /* [d]; target's final RMSNorm gain */
    const hivis_layer_weights *layers;  /* [n_layers] */
    hivis_layer_weights draft_layer;    /* the drafter's single decoder layer */
    const void *fuse_w;                 /* [2d][d] = [w1 ; w2] of the fusion e^ = f w1 + e w2 (section 3.2) */
    const void *resid_rho;              /* [n_resid][d]: rho_i = r^i w, the folded bias-correction residuals */
} hivis_weights;

/* Create a context: validates the config, allocates device state (weights re-laid-out for
 * streaming, target KV for max_vis+max_text positions, drafter KV for max_text positions) and
 * copies the weights from host memory.  hip_stream: a hipStream_t (NULL = the default stream).
 * For bf16 models it also computes, once, the table Embed(x) w2 of the fusion's embedding half (section 3.2: e^ is linear
 * in its two inputs, and Embed(x) w2 depends on the token alone): vocab x d float32 values of device memory
 * (0.5 GB for a 32000 x 4096 model), so that a draft step streams w1 only.
 * Errors: HIVIS_EINVAL, HIVIS_EHIP (then *out is NULL). */
int hivis_create(const hivis_config *cfg, const hivis_weights *w, void *hip_stream, hivis_ctx **out);

/* Free everything the context owns.  NULL is accepted. */
int hivis_destroy(hivis_ctx *ctx);

/* Algorithm 1, inputs line and steps 1-2.  Target prefill over [vis_embeds ; Embed(text_ids)]
 * (positions 0..v+l-1, fully causal), which fills the target KV cache and yields f_fused^{1:l}
 * and the first generated token x_{l+1}; then the drafter is prefilled over the l text positions
 * only, with inputs f^j w1 + Embed(x_{j+1}) w2 + rho_0.
 *   vis_embeds : [B][v][d], context dtype, host or device.
 *   text_ids   : [B][l] int32, host or device; every id in [0, vocab).
 *   first_token: [B] int32, host; receives x_{l+1} (may be NULL).
 * May be called again at any time to start new sequences (all state is reset).
 * Errors: EINVAL (null, v<0, l<1, id out of range; also: the prompt's logits have no finite maximum, i.e. NaN or Inf
 * in vis_embeds or the weights -- the context then stays un-prefilled), ECAP (v>max_vis or l+k_max+2>max_text), EHIP. */
int hivis_prefill(hivis_ctx *ctx, const void *vis_embeds, int32_t v, const int32_t *text_ids, int32_t l,
                  int32_t *first_token);

/* Algorithm 1, the drafting loop: K serial drafter steps, each LM head -> greedy token ->
 * fusion FC on [f' ; Embed(token)] + rho_min(i, n_resid-1) -> drafter layer over the text-only
 * cache.  Tokens stay on the device.  1 <= K <= k_max.  State READY -> DRAFTED.
 * Errors: ESTATE, EINVAL, ECAP (a sequence would exceed max_text). */
int hivis_draft(hivis_ctx *ctx, int32_t K);

/* hivis_draft for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the same K drafter steps with the same kernels, one launch per step operation,
 * but every intermediate buffer of the round (rotary tables, fusion outputs, q/k/v rows, attention partials,
 * MLP activations, greedy candidates) lives in ONE static device array of HIVIS_NOALLOC_SCRATCH_BYTES that is part
 * of the library's code object; the call makes no hipMalloc / hipFree and creates no events (hivis_timing does not
 * cover it).  Inputs and outputs are those of hivis_draft: the context's pending hidden state and text-only cache
 * in, K drafted tokens (and their logits, hivis_get_logits(1)) out.
 *   - Limits: needs the phase programs (default; batch <= 8 for HIVIS_BF16, <= 16 for HIVIS_F32) and a round that
 *     fits the array: otherwise HIVIS_EINVAL / HIVIS_ECAP with a message, and nothing has run.
 *   - The array is one per GPU, shared by every context and every call on that GPU, and keeps the last call's
 *     contents; nothing in it has to start at zero (each word is written by the round before the round reads it).
 *     Calls that overlap on one GPU (two contexts on different streams, two host threads) race on it: serialise them.
 * State READY -> DRAFTED.  Errors: ESTATE, EINVAL, ECAP, EHIP. */
#define HIVIS_NOALLOC_SCRATCH_BYTES (16u << 20)
int hivis_draft_noalloc(hivis_ctx *ctx, int32_t K);

/* Test hook: plant drafts instead of running the drafter.  tokens: [B][K] int32, host.
 * State READY -> DRAFTED.  Errors: ESTATE, EINVAL, ECAP. */
int hivis_set_drafts(hivis_ctx *ctx, const int32_t *tokens, int32_t K);

/* Algorithm 1, "Parallel Verify": one target pass over the rows [x_{l+1}, x'_{l+2..l+1+K}] of
 * every sequence against its full visual+text cache (causal among the new rows), LM head and
 * greedy token per row.  State DRAFTED -> VERIFIED.  Errors: ESTATE, EHIP. */
int hivis_verify(hivis_ctx *ctx);

/* Greedy acceptance (section 2.1) and roll-forward.  Per sequence b: n_b = length of the longest
 * prefix of drafts equal to the target's greedy tokens; tokens[b][0..n_b-1] are those drafts and
 * tokens[b][n_b] is the target's own next token.  The target cache keeps n_b+1 new rows; the
 * drafter's speculative rows are dropped and n_b+1 rows rebuilt from the target's true features
 * (section 3.3, Eq. (1)).  Synchronises.  State VERIFIED -> READY.
 *   n_accepted: [B] int32 host.   tokens: [B][k_max+1] int32 host (entries beyond n_b are -1).
 * Errors: ESTATE, EINVAL, EHIP.  If a pass of the cycle met logits without a finite maximum (EINVAL), or the optional
 * one-launch pass aborted at its grid barrier (EHIP), the device state has already moved on: the context falls back
 * to the un-prefilled state and only hivis_prefill is accepted next (it also clears both conditions). */
int hivis_accept(hivis_ctx *ctx, int32_t *n_accepted, int32_t *tokens);

/* ---- the same cycle at a temperature T > 0 (section 2.1: the accepted prefix is kept, the token after it is
 * resampled, and if every candidate is accepted the target samples from its own distribution; the rule is the
 * speculative sampling rule of the works that section cites).  The uniform random numbers are INPUTS, each in [0, 1).
 * hivis_prefill's first token is the target's greedy token; hivis_prefill_sample draws it as well. ---- */

/* hivis_prefill with x_{l+1} of sequence b drawn from softmax(logits / T) by inversion with u_first[b] (host, [B]).
 * Errors as hivis_prefill, plus EINVAL for T <= 0 or a uniform outside [0, 1).  u_first may be NULL after hivis_rng_seed. */
int hivis_prefill_sample(hivis_ctx *ctx, const void *vis_embeds, int32_t v, const int32_t *text_ids, int32_t l,
                         float temperature, const float *u_first, int32_t *first_token);

/* K serial drafter steps as hivis_draft, but draft i of sequence b is DRAWN from q_i = softmax(logits_i / T) by
 * inversion with u[b][i-1]: the smallest token j whose running probability sum exceeds u.
 *   u: [B][K] float32, host (NULL after hivis_rng_seed: drawn on the device).   State READY -> DRAFTED.
 * Errors: ESTATE, EINVAL (K, T <= 0, null or out-of-range u), ECAP. */
int hivis_draft_sample(hivis_ctx *ctx, int32_t K, float temperature, const float *u);

/* Stochastic acceptance after hivis_verify of drafts made by hivis_draft_sample with the same T.  With p_i =
 * softmax(target logits of row i / T): draft i is accepted while u_accept[b][i] * q_i(x_i) < p_i(x_i); at the first
 * rejection the next token is drawn with u_resample[b] from the normalised positive part of p_i - q_i (from p_i if
 * it is empty); if all K are accepted it is drawn from p_K.  Then the same roll-forward as hivis_accept.
 *   u_accept: [B][K] float32 host; u_resample: [B] float32 host (both NULL after hivis_rng_seed: drawn on the
 *   device); outputs as hivis_accept.  Synchronises.
 * Errors: ESTATE (also: drafts were planted or drawn greedily, so q is unknown), EINVAL, EHIP. */
int hivis_accept_sample(hivis_ctx *ctx, float temperature, const float *u_accept, const float *u_resample,
                        int32_t *n_accepted, int32_t *tokens);

/* Random numbers drawn ON THE DEVICE for the three sampling calls above (section 2.1 leaves the source of randomness
 * open).  After hivis_rng_seed a sampling call whose uniform arrays are ALL NULL fills them itself, on the device, from the
 * published counter-based generator Philox4x32-10 (Salmon et al., SC'11): key = (seed low word, seed high word), counter =
 * (index of the number in its array, purpose, call count low word, call count high word), uniform = top 24 bits of output
 * word 0 times 2^-24.  Purposes and array shapes: 0 = u_first [B]; 1 = u [B][K] (index b*K + i); 2 = u_accept [B][K];
 * 3 = u_resample [B]; 4 = u of hivis_tree_accept_sample [depth + 1].  Every sampling call that draws this way uses the context's call count once (u_accept and
 * u_resample of one hivis_accept_sample share it) and then increments it; hivis_rng_seed resets it to 0.  Nothing crosses
 * the host-device link.  calls_so_far (may be NULL) receives the count before the reset.
 * Errors: EINVAL (null ctx).  A sampling call with NULL uniforms before any hivis_rng_seed: ESTATE; with only one of
 * u_accept / u_resample NULL: EINVAL. */
int hivis_rng_seed(hivis_ctx *ctx, uint64_t seed, uint64_t *calls_so_far);

/* ---- the same cycle with a draft TREE instead of a chain (section 4, inference setting: a top-k tree expanded to a
 * fixed depth, the candidates with the highest cumulative probability verified in one pass; section 2.1 names the tree
 * structure).  Greedy (T = 0), batch 1 only.  The three calls replace hivis_draft / hivis_verify / hivis_accept in a
 * cycle; chain and tree cycles may alternate on one context.  The first tree call on a context allocates the tree's
 * device arrays (a few MB plus [65][vocab] floats); they are freed by hivis_destroy. ---- */

/* Builds the pool and picks the candidates.  Level 1: the top_k most probable tokens after the drafter's pending
 * hidden state, scored by log-probability.  Level j+1 (j = 1..depth-1): the top_k best-scored nodes of level j go
 * through the drafter as one pass of top_k rows (fusion input with the residual of depth j; each row sees the
 * text-only cache, its ancestors and itself) and each contributes its top_k most probable continuations, scored
 * parent score + log-probability.  Pool = top_k + (depth-1) top_k^2 nodes, indexed level by level, expanded row by
 * expanded row, rank by rank.  Candidates = the n_nodes best-scored pool nodes (ties: lower pool index), kept in pool
 * order; verify row i (1..n_nodes) is candidate i-1, row 0 the last known token.
 * Limits: top_k <= 16, depth <= 16, pool <= 2048, (depth-1) top_k <= 64, n_nodes <= min(pool, 63).
 * State READY -> TREE_DRAFTED.  Errors: ESTATE, EINVAL (limits, batch != 1), ECAP, EHIP. */
int hivis_tree_draft(hivis_ctx *ctx, int32_t top_k, int32_t depth, int32_t n_nodes);

/* Test hook, the tree analogue of hivis_set_drafts: plants the candidates instead of drafting them.  tokens[i] /
 * parents[i] describe verify row i+1; parents are row indices (0 = the root) smaller than the row's own.
 *   tokens, parents: [n_nodes] int32 host.  State READY -> TREE_DRAFTED.  Errors: ESTATE, EINVAL, ECAP, EHIP. */
int hivis_tree_set(hivis_ctx *ctx, int32_t n_nodes, const int32_t *tokens, const int32_t *parents);

/* One target pass over the n_nodes + 1 rows: a row sits at position v + l + depth and attends to the whole
 * visual + text cache, its ancestors and itself.  State TREE_DRAFTED -> TREE_VERIFIED.  Errors: ESTATE, EHIP. */
int hivis_tree_verify(hivis_ctx *ctx);

/* Greedy acceptance on the tree: from the root, the child whose token equals the target's greedy token at the current
 * row is followed until there is none; tokens[0..n-1] are the followed tokens, tokens[n] the target's own token at the
 * last row.  The target cache keeps the followed rows (moved next to the root's), the drafter drops its tree rows and
 * is re-fed the true features of the path, as hivis_accept does.  Synchronises.  State TREE_VERIFIED -> READY.
 *   n_accepted: [1] int32 host.   tokens: [depth+1] int32 host (entries beyond n are -1).
 * Errors: ESTATE, EINVAL, EHIP. */
int hivis_tree_accept(hivis_ctx *ctx, int32_t *n_accepted, int32_t *tokens);

/* hivis_tree_accept at a temperature T > 0.  Table 2 reports T = 1 results with a tree, the paper does not spell the rule
 * out; the reading implemented: the tree holds deterministic candidates, so after every visited row the target DRAWS its
 * next token from softmax(logits of that row / T) by inversion, and a candidate child is followed exactly when it is the
 * drawn token; the walk ends with the first draw that is no child.  The emitted tokens are draws from the target's own
 * distribution whatever the tree holds: with the same uniforms they are the tokens that drawing one token at a time
 * emits.  A row of depth j (root: 0) draws with u[j].
 *   u: [depth + 1] float32 host, each in [0, 1) (depth as given to hivis_tree_draft, or the depth of the planted tree);
 *      NULL after hivis_rng_seed: drawn on the device (purpose 4, index j).  Outputs, state and errors as hivis_tree_accept,
 *      plus EINVAL for T <= 0 or a uniform outside [0, 1).  hivis_tree_get afterwards returns the DRAWN tokens as
 *      target_tokens. */
int hivis_tree_accept_sample(hivis_ctx *ctx, float temperature, const float *u, int32_t *n_accepted, int32_t *tokens);

/* ---- test / measurement hooks (all synchronise) ---- */

/* The last tree, any pointer may be null (host arrays): pool_tokens / pool_parents (pool index, -1 = root) /
 * pool_scores [pool]; expand [depth-1][top_k] pool indices of the expanded rows; selected [n_nodes] candidates;
 * row_tokens / row_parents (row index, -1 for the root) / row_depths [n_nodes+1]; target_tokens [n_nodes+1] (after
 * hivis_tree_verify only). */
int hivis_tree_get(hivis_ctx *ctx, int32_t *pool_tokens, int32_t *pool_parents, float *pool_scores, int32_t *expand,
                   int32_t *selected, int32_t *row_tokens, int32_t *row_parents, int32_t *row_depths, int32_t *target_tokens);

/* Drafter logits behind the last tree: row 0 = the pending hidden state, row 1 + (j-1) top_k + r = expanded row r of
 * level j.  out: [1 + (depth-1) top_k][vocab] float32, host. */
int hivis_tree_get_logits(hivis_ctx *ctx, float *out);

/* which = 0: logits of the last verify, [B][K+1][vocab] (tree: [n_nodes+1][vocab]); which = 1: logits of the last draft round,
 * [K][B][vocab]; which = 2: logits that chose x_{l+1} at prefill, [B][vocab].  out: float32, host. */
int hivis_get_logits(hivis_ctx *ctx, int32_t which, float *out);

/* which = 0: post-final-norm target features g of the last verify, [B][K+1][d] (tree: [n_nodes+1][d]);
 * which = 1: the drafter's pending hidden state f'_1 for the next round, [B][d].  out: float32, host. */
int hivis_get_hidden(hivis_ctx *ctx, int32_t which, float *out);

/* Current KV lengths per sequence: target (visual + text rows) and drafter (text rows only). */
int hivis_kv_lengths(hivis_ctx *ctx, int32_t *target_len, int32_t *drafter_len);

/* Drafts of the last round, [B][K] int32 host, and the target's greedy tokens of the last verify,
 * [B][K+1] int32 host.  Either pointer may be NULL. */
int hivis_get_tokens(hivis_ctx *ctx, int32_t *drafts, int32_t *target_tokens);

/* Timing hook: when enabled, hivis_draft / hivis_verify / hivis_accept / hivis_prefill record HIP
 * events on the context's stream around their work, without waiting for them (they are read at the next
 * hivis_accept, which synchronises anyway, or by hivis_phase_ms); hivis_phase_ms synchronises, returns and
 * clears the accumulated milliseconds and call counts.
 * phase: 0 prefill, 1 draft (one call = K steps), 2 verify, 3 accept+roll. */
int hivis_timing(hivis_ctx *ctx, int32_t enable);
int hivis_phase_ms(hivis_ctx *ctx, int32_t phase, double *total_ms, int64_t *calls);

/* Kernel-level timing of the verify pass's weight-streaming GEMM launches of one kind, with a pair of HIP events
 * attached to the dispatch itself (hipExtLaunchKernel's start/stop events: they read the kernel's own begin and end
 * timestamps, so no marker packets sit in the queue around it).  Every 8th such launch is timed (the launches of
 * one kind are alike across layers).  Resolved at the next hivis_accept.  gemm_kind: 1 = O / down
 * projection (+ residual), 3 = fused QKV (+ RMSNorm, RoPE, cache append), 4 = fused gate|up (+ RMSNorm, SiLU*up),
 * 5 = LM head (+ greedy candidates); -1 switches it off.  hivis_kernel_ms returns and clears the accumulated
 * milliseconds and launch count, and the algorithmic bytes of one such launch (its weight matrix, read once). */
int hivis_kernel_timing(hivis_ctx *ctx, int32_t gemm_kind);
int hivis_kernel_ms(hivis_ctx *ctx, double *total_ms, int64_t *launches, double *bytes_per_launch);

/* Algorithmic HBM bytes of the last verify pass and of one draft step at the current lengths
 * (every weight once, the KV rows read once; see the formulas in the implementation). */
int hivis_algorithmic_bytes(hivis_ctx *ctx, double *verify_bytes, double *draft_step_bytes);

/* Measurement hook, independent of any context: the rate at which a plain read-only kernel streams memory on this
 * GPU, with the access pattern of the library's weight-streaming GEMMs (1 KiB per wavefront and instruction, 8
 * independent 16-byte loads per lane, 64 KiB per workgroup and trip) and none of their work.  n_buffers device
 * buffers of buffer_bytes each are allocated, filled, read once untimed and then `passes` times in rotation, one launch
 * of `workgroups` x 512 threads per buffer, back to back on hip_stream (a hipStream_t, NULL = default).  Start / stop
 * events attached to the dispatches themselves (at most 256 of them, evenly spread) read each launch's own begin and end,
 * exactly as hivis_kernel_timing times the library's GEMM: launch gaps and the host's launch rate are not in the figure.
 * Choose n_buffers * buffer_bytes well above the 256 MB memory-side cache so that nothing is re-read from it.
 *   us_per_launch: average duration of one launch; gb_per_s: bytes one launch reads / that duration, in 1e9 bytes per
 *   second.  Either may be NULL.
 * Frees everything before it returns.  Errors: EINVAL (sizes), EHIP. */
int hivis_calib_stream(void *hip_stream, int64_t buffer_bytes, int32_t n_buffers, int32_t passes, int32_t workgroups,
                       double *gb_per_s, double *us_per_launch);

/* Host function, no GPU needed: the rule every greedy-token kernel applies before it stores a token id (the same
 * inline function, compiled for the host): ids below 0 become 0, ids >= vocab become vocab - 1.  Only a row of logits
 * with no finite maximum (NaN / Inf inputs) yields such an id; the calls that synchronise (hivis_prefill, hivis_accept,
 * hivis_tree_accept) then return HIVIS_EINVAL and the context must be prefilled again. */
int32_t hivis_clamp_token(int32_t id, int32_t vocab);

const char *hivis_last_error(hivis_ctx *ctx);   /* never NULL; "" if no error */
const char *hivis_version(void);

#ifdef __cplusplus
}
#endif
#endif /* HIVIS_H */

// Host side of the HiViS draft-verify library: context, state machine, launch sequences.
// The C ABI is declared and documented in include/hivis.h.
#include "hivis.h"
#include "hivis_kernels.h"
#include "hivis_fused.h"
#include "hivis_tree.h"

#include <hip/hip_ext.h>
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <cstdlib>
#include <map>
#include <mutex>
#include <string>
#include <vector>

using namespace hivis;

// Scratch memory of hivis_draft_noalloc: a file-scope device array instead of an allocation.  Every GPU the library runs on
// holds its own copy at its own address until the process ends.  In host code the name `scratch` is only a stand-in for
// the symbol: the device address is looked up once per device with hipGetSymbolAddress (scratch_for_device below) and that
// pointer, never the name, is what kernels receive.
#define HIVIS_SCRATCH_BYTES HIVIS_NOALLOC_SCRATCH_BYTES
static __device__ __align__(256) unsigned char scratch[HIVIS_SCRATCH_BYTES];

namespace {

enum State { ST_CREATED = 0, ST_READY, ST_DRAFTED, ST_VERIFIED, ST_TREE_DRAFTED, ST_TREE_VERIFIED };

constexpr int MAX_ROWS = 64;        // rows per pass that the activation buffers hold (tree verify: root + 63 candidates)
constexpr int CHAIN_MAX_ROWS = 32;  // chain verify rows B*(K+1); prefill chunk; rows per launch of the skinny GEMM

// Rows of a draft tree (null pointers: ordinary causal rows)
struct TreeRows { const int* pos_delta = nullptr; const unsigned long long* mask = nullptr; };

struct LayerDev {
    void* norm1 = nullptr; void* norm2 = nullptr;   // [d] storage dtype
    uint4* wqkv = nullptr;                          // packed [d] -> [q_dim + 2 kv_dim]
    uint4* wo = nullptr;                            // packed [q_dim] -> [d]
    uint4* wgu = nullptr;                           // packed [d] -> [2 ffn]  (gate | up)
    uint4* wd = nullptr;                            // packed [ffn] -> [d]
    float* bqkv = nullptr;                          // optional q/k/v projection biases [q_dim + 2 kv_dim], in wqkv's column order
};

struct KVDev { void* k = nullptr; void* v = nullptr; int maxL = 0; };   // [B][Hkv][maxL][hd]

}  // namespace

struct hivis_ctx {
    hivis_config cfg{};
    hipStream_t stream = nullptr;
    int state = ST_CREATED;
    std::string err;
    int esize = 4;
    int num_cu = 256;

    // weights
    void* embed = nullptr; void* final_norm = nullptr; void* rho = nullptr;
    uint4* lm_head = nullptr; uint4* fuse_w = nullptr;
    uint4* fuse_w1 = nullptr;            // rows [0, d) of the fusion FC, packed on their own (K = d), and
    bool lm_ext = false;                 // the packed LM head is followed by w1's tiles in one buffer (lm_head .. lm_head + (V + d) d)
    float* emb_w2 = nullptr;             // [V][d] fp32: Embed(token) . w2, the embedding half of the fusion FC per token (bf16 models)
    std::vector<LayerDev> layers; LayerDev draft;
    std::vector<KVDev> tkv; KVDev dkv;

    // per-sequence state (device) + host mirrors
    int* tlen = nullptr; int* dlen = nullptr; int* zeros = nullptr;
    int32_t* text = nullptr; int text_stride = 0;
    std::vector<int> h_tlen, h_dlen;
    int v = 0, K = 0;

    // activations (fp32)
    float *x = nullptr, *a = nullptr, *qkv = nullptr, *att = nullptr, *proj = nullptr, *gu = nullptr, *act = nullptr;
    float *catT = nullptr;      // [MAX_ROWS][2d]: verify features g | embeddings of the following tokens
    float *catD = nullptr;      // [B][2d]: drafter hidden f' | embedding of the drafted token
    float *u = nullptr, *dout = nullptr;
    float *feat = nullptr;      // [B][max_text][d] true features of prompt text rows (prefill only)
    float *attn_ws = nullptr; size_t attn_ws_floats = 0;
    float* zero_blk = nullptr;           // 1 KiB of zeros: the K blocks past the end in the large-tile prefill GEMM
    int* rows_cnt = nullptr; int rows_cnt_n = 0;      // arrival counters of the key-split attention launched outside a phase program (zero between launches)
    float *logits_v = nullptr, *logits_d = nullptr, *logits_p = nullptr;
    int32_t *row_tok = nullptr, *drafts = nullptr, *ttok = nullptr, *nacc = nullptr, *out_tok = nullptr, *next_tok = nullptr;
    int32_t* h_result = nullptr;         // pinned host mirror of [nacc | out_tok | abort flag | bad-logits flag]
    int* bad = nullptr;                  // device flag: a greedy-token kernel met a row without a finite maximum (cleared by hivis_prefill)
    bool rng_seeded = false; unsigned long long rng_seed = 0, rng_calls = 0;   // device-side uniforms (hivis_rng_seed): Philox key and draw-call count
    float* u_tree = nullptr;             // [TREE_MAX_DEPTH + 1] uniforms of hivis_tree_accept_sample, one per depth
    float *u_draft = nullptr, *u_acc = nullptr, *u_res = nullptr;   // uniform numbers of the sampling calls: [B][k_max], [B][k_max] (row stride K), [B]
    float inv_temp = 1.0f; bool drafts_sampled = false;             // set by hivis_draft_sample; hivis_accept_sample needs the drafter's distributions
    void* vis = nullptr;        // staging for vis_embeds [B][max_vis][d]
    // whole-prompt prefill buffers (bf16 models): all v+l rows of one sequence per layer
    int pf_rows = 0;
    float *pf_x = nullptr, *pf_a = nullptr, *pf_qkv = nullptr, *pf_att = nullptr, *pf_proj = nullptr, *pf_gu = nullptr, *pf_act = nullptr;
    uint4* pf_frag = nullptr;
    std::vector<int32_t> h_ids;

    // persistent-kernel path (passes of at most one MFMA tile of rows)
    bool fused = false;
    int fused_grid = 0; size_t fused_lds = 0;
    float* rope_tab = nullptr; float* pm = nullptr; int* pi = nullptr; unsigned* bar = nullptr;
    float* fattn_ws = nullptr; size_t fattn_ws_floats = 0;
    struct Program { hivis::Phase* dev = nullptr; int n = 0; std::vector<hivis::Phase>* host = nullptr; };
    bool tall_big = true; int tall_big_fill = 70;   // prefill GEMMs: the 128 x 256 tile when its workgroups fill at least this percentage of their rounds over the CUs
    int attn_shared_min = 128;           // rows per sequence from which a causal pass uses the shared-tile attention kernel (128 rows per workgroup)
    int keys_per_split = 192;            // attention: cached keys per workgroup (one or two 16-key tiles per wavefront) before the key range is split further
    bool attn_elect = true;              // key splits merged by the workgroup that arrives last (false: by a merge launch)
    int attn_flags = 3;                  // AttnShape::flags of the phase programs
    bool persistent = false;             // HIVIS_PERSISTENT=1: one cooperative launch per pass instead of one launch per phase
    std::map<int, Program> programs;     // key = kind * 64 + K
    unsigned long long* prof = nullptr; int prof_left = 0;   // developer aid: HIVIS_PROF=n dumps per-phase times of n verify passes

    // draft tree (batch 1): device arrays are allocated by the first hivis_tree_draft call, for the limits below
    hivis::TreeDev tree{}; bool tree_ready = false;
    int tk = 0, tdepth = 0, tn = 0;                       // top-k, depth, candidates of the current tree
    int vrows = 0;                                        // rows of the last verify pass (chain: B*(K+1); tree: N+1)
    float *tH = nullptr, *tlogits = nullptr, *tcat = nullptr, *troll = nullptr;
    float *tcand_v = nullptr, *tseg = nullptr; int32_t* tcand_i = nullptr; int tnseg = 0;   // per-segment top-k candidates and (max, sum) partials   // hidden rows, their logits, level inputs, re-feed inputs
    void** kv_ptrs = nullptr; void* kv_staging = nullptr;
    float* splitk_ws = nullptr; size_t splitk_floats = 0; bool no_wide_gemm = false; int wide_min = 11;   // measured: 10-row passes faster on the skinny kernels, 12-row passes on the split-K layer   // K-slice partials of the wide GEMM; HIVIS_WIDE_GEMM=0 disables it
    int32_t* h_tree_result = nullptr;                     // pinned [1 + TREE_MAX_DEPTH + 1]

    // timing
    int ktime_epi = -1;                                  // GEMM epilogue kind whose verify launches are event-timed (-1: none)
    int ktime_stride = 8; int64_t ktime_seen = 0;        // every ktime_stride-th such launch is timed (an event pair costs ~8 us of idle queue)
    std::vector<hipEvent_t> kev; size_t kev_used = 0;     // event pairs recorded since the last accept
    double kms = 0; int64_t klaunches = 0; double kbytes = 0;
    bool timing = false;
    // phase timing: event pairs recorded without waiting, resolved at the next point where the stream is synchronised anyway
    std::vector<hipEvent_t> pev; std::vector<int> pev_phase; size_t pev_used = 0;
    double phase_ms[4] = {0, 0, 0, 0}; int64_t phase_calls[4] = {0, 0, 0, 0};
    std::vector<void*> allocs;
    // hivis_draft_noalloc: this device's address of the static scratch array, and host storage for its phase list
    // (reserved at create, so the call itself allocates nothing on the host either)
    void* scratch_dev = nullptr;
    std::vector<hivis::Phase> na_phases;
};

namespace {

int fail(hivis_ctx* c, int code, const char* fmt, ...) {
    char buf[512];
    va_list ap; va_start(ap, fmt); vsnprintf(buf, sizeof buf, fmt, ap); va_end(ap);
    if (c) c->err = buf;
    return code;
}

#define HIP_TRY(c, expr)                                                                              \
    do {                                                                                              \
        hipError_t e_ = (expr);                                                                       \
        if (e_ != hipSuccess) return fail((c), HIVIS_EHIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

// Device address of the static scratch array on device `dev` (which must be the current device): looked up once per
// device, then kept for the life of the process.
constexpr int MAX_DEVICES = 64;
void* g_scratch_ptr[MAX_DEVICES] = {};
std::mutex g_scratch_mu;
int scratch_for_device(hivis_ctx* c, int dev) {
    if (dev < 0 || dev >= MAX_DEVICES) return fail(c, HIVIS_EINVAL, "device index %d outside [0,%d)", dev, MAX_DEVICES);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        HIP_TRY(c, hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return fail(c, HIVIS_EHIP, "hipGetSymbolAddress(scratch) returned a null address");
        g_scratch_ptr[dev] = ptr;
    }
    c->scratch_dev = g_scratch_ptr[dev];
    return HIVIS_OK;
}

template <typename T> int dev_alloc(hivis_ctx* c, T** p, size_t count) {
    void* q = nullptr;
    HIP_TRY(c, hipMalloc(&q, std::max<size_t>(count, 1) * sizeof(T)));
    c->allocs.push_back(q);
    *p = (T*)q;
    return HIVIS_OK;
}

// ---- weight upload + re-layout -------------------------------------------------------------
template <typename WT>
int pack_matrix(hivis_ctx* c, const void* const* srcs, const int* ncols, int nsrc, int K, int transposed, void* staging,
                uint4** out, int mode = PACK_PLAIN) {
    int N = 0;
    PackSrc ps{};
    char* st = (char*)staging;
    for (int i = 0; i < 3; ++i) { ps.p[i] = nullptr; ps.n[i] = 0; }
    for (int i = 0; i < nsrc; ++i) {
        const size_t bytes = (size_t)K * ncols[i] * sizeof(WT);
        HIP_TRY(c, hipMemcpy(st, srcs[i], bytes, hipMemcpyHostToDevice));
        ps.p[i] = st; ps.n[i] = ncols[i];
        st += (bytes + 255) & ~(size_t)255;
        N += ncols[i];
    }
    ps.transposed = transposed; ps.mode = mode; ps.hd = c->cfg.head_dim;
    const size_t n16 = (size_t)K * N * sizeof(WT) / 16;
    if (int rc = dev_alloc(c, out, n16)) return rc;
    const int blocks = (int)std::min<size_t>((n16 + 255) / 256, 65535);
    hipLaunchKernelGGL(pack_weights_kernel<WT>, dim3(blocks), dim3(256), 0, c->stream, ps, K, N, *out);
    HIP_TRY(c, hipGetLastError());
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return HIVIS_OK;
}

template <typename WT>
int upload_vec(hivis_ctx* c, const void* src, size_t count, void** out) {
    WT* p = nullptr;
    if (int rc = dev_alloc(c, &p, count)) return rc;
    HIP_TRY(c, hipMemcpy(p, src, count * sizeof(WT), hipMemcpyHostToDevice));
    *out = p;
    return HIVIS_OK;
}

template <typename WT>
int upload_layer(hivis_ctx* c, const hivis_layer_weights& w, void* staging, LayerDev& L) {
    const hivis_config& g = c->cfg;
    const int qd = g.n_q_heads * g.head_dim, kd = g.n_kv_heads * g.head_dim;
    if (!w.norm1 || !w.wq || !w.wk || !w.wv || !w.wo || !w.norm2 || !w.wg || !w.wu || !w.wd)
        return fail(c, HIVIS_EINVAL, "null layer weight pointer");
    if (int rc = upload_vec<WT>(c, w.norm1, g.d, &L.norm1)) return rc;
    if (int rc = upload_vec<WT>(c, w.norm2, g.d, &L.norm2)) return rc;
    { const void* s[3] = {w.wq, w.wk, w.wv}; int n[3] = {qd, kd, kd};
      if (int rc = pack_matrix<WT>(c, s, n, 3, g.d, 0, staging, &L.wqkv, PACK_QKV)) return rc; }
    { const void* s[1] = {w.wo}; int n[1] = {g.d};
      if (int rc = pack_matrix<WT>(c, s, n, 1, qd, 0, staging, &L.wo)) return rc; }
    { const void* s[2] = {w.wg, w.wu}; int n[2] = {g.ffn, g.ffn};
      if (int rc = pack_matrix<WT>(c, s, n, 2, g.d, 0, staging, &L.wgu, PACK_GATEUP)) return rc; }
    { const void* s[1] = {w.wd}; int n[1] = {g.d};
      if (int rc = pack_matrix<WT>(c, s, n, 1, g.ffn, 0, staging, &L.wd)) return rc; }
    if (w.bq || w.bk || w.bv) {
        if (!w.bq || !w.bk || !w.bv) return fail(c, HIVIS_EINVAL, "q/k/v biases: give all three or none");
        // the fused qkv columns: [q heads | k heads | v heads], inside every q and k head the rotary pair (i, i + hd/2)
        // in adjacent columns (2i, 2i+1): the biases follow their columns
        const int hd = g.head_dim, half = hd / 2;
        std::vector<float> b((size_t)qd + 2 * kd);
        auto val = [](const void* p, size_t i) -> float {
            if (sizeof(WT) == 2) { const uint32_t u = (uint32_t)((const uint16_t*)p)[i] << 16; float f; memcpy(&f, &u, 4); return f; }
            return ((const float*)p)[i];
        };
        for (int part = 0; part < 2; ++part) {
            const void* src = part == 0 ? w.bq : w.bk;
            const int n = part == 0 ? qd : kd, off = part == 0 ? 0 : qd;
            for (int col = 0; col < n; ++col) {
                const int h = col / hd, pc = col % hd;
                b[(size_t)off + col] = val(src, (size_t)h * hd + ((pc & 1) ? pc / 2 + half : pc / 2));
            }
        }
        for (int col = 0; col < kd; ++col) b[(size_t)qd + kd + col] = val(w.bv, col);
        if (int rc = dev_alloc(c, &L.bqkv, b.size())) return rc;
        HIP_TRY(c, hipMemcpy(L.bqkv, b.data(), b.size() * sizeof(float), hipMemcpyHostToDevice));
    }
    return HIVIS_OK;
}

// column chunks per row for the row-wise kernels: few rows -> split every row over several workgroups
static inline int row_chunks(int rows) { return rows >= 256 ? 1 : std::max(1, std::min(8, 256 / std::max(rows, 1))); }

int wide_gemm(hivis_ctx* c, const float* A, int lda, int M, int K, const uint4* Wp, int N, float* Y, int ldy, hivis::Parts* defer = nullptr);
template <typename WT>
int layer_forward_wide(hivis_ctx* c, const LayerDev& L, const KVDev& kv, float* h, hivis::Parts pending, const int* base,
                       int offset, int seq0, int nseq, int m, TreeRows tr, hivis::Parts* out_pending);

// ---- launches --------------------------------------------------------------------------------
template <typename WT>
int gemm(hivis_ctx* c, const float* A, int lda, int M, int K, const uint4* Wp, int N, float* Y, int ldy, int epi) {
    if (M < 1 || M > MAX_ROWS) return fail(c, HIVIS_EINVAL, "gemm rows %d out of range", M);
    if (sizeof(WT) == 2 && M >= c->wide_min && c->pf_frag && c->pf_rows >= MAX_ROWS && ldy == N && epi == EPI_STORE && !c->no_wide_gemm)
        return wide_gemm(c, A, lda, M, K, Wp, N, Y, ldy);
    if (M > CHAIN_MAX_ROWS) {            // wider passes (tree verify)
        // fp32 models: one launch per 32 rows
        for (int r0 = 0; r0 < M; r0 += CHAIN_MAX_ROWS)
            if (int rc = gemm<WT>(c, A + (size_t)r0 * lda, lda, std::min(CHAIN_MAX_ROWS, M - r0), K, Wp, N, Y + (size_t)r0 * ldy, ldy, epi)) return rc;
        return HIVIS_OK;
    }
    const int ntiles = N / 16;
    const int grid = std::min(ntiles, c->num_cu);
    constexpr int ROWS = WTraits<WT>::ROWS;
    const int T = (M + ROWS - 1) / ROWS;
    // dynamic LDS = cross-wavefront reduction buffer [NW][G][T][64][RPL] floats
#define HIVIS_SKINNY(T_, KBW_, G_, NW_) HIVIS_SKINNY_(T_, KBW_, G_, NW_, false)
#define HIVIS_SKINNY_(T_, KBW_, G_, NW_, UP_)                                                                      \
    do {                                                                                                           \
        constexpr size_t lds_ = (size_t)NW_ * G_ * T_ * 64 * WTraits<WT>::RPL * sizeof(float);                     \
        static bool attr_done_ = false;                                                                            \
        if (!attr_done_ && lds_ > 64 * 1024) {                                                                     \
            HIP_TRY(c, hipFuncSetAttribute((const void*)gemm_skinny_kernel<WT, T_, KBW_, G_, NW_, UP_>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_)); \
            attr_done_ = true;                                                                                     \
        }                                                                                                          \
        hipLaunchKernelGGL((gemm_skinny_kernel<WT, T_, KBW_, G_, NW_, UP_>), dim3(grid), dim3(NW_ * 64), lds_, c->stream, A, lda, M, K, Wp, N, Y, ldy, epi); \
    } while (0)
    if constexpr (sizeof(WT) == 2) {
        if (T == 1) HIVIS_SKINNY(1, 4, 8, 16);
        // 8 wavefronts for the wider row counts: every wavefront may use 256 registers (raw rows + fragments + accumulators
        // spill at 128)
        else if (T == 2) HIVIS_SKINNY(2, 4, 4, 8);
        else HIVIS_SKINNY_(4, 2, 4, 8, true);     // all 4 tiles' weights of a pass in flight together
    } else {
        if (T == 1) HIVIS_SKINNY(1, 4, 4, 16);
        else HIVIS_SKINNY(2, 4, 2, 16);
    }
#undef HIVIS_SKINNY
#undef HIVIS_SKINNY_
    HIP_TRY(c, hipGetLastError());
    return HIVIS_OK;
}

template <typename WT>
int attention(hivis_ctx* c, const float* q, int ldq, const KVDev& kv, const int* base, int offset, int seq0, int nseq,
              int m, int max_keys, float* out, int ldo, const unsigned long long* tmask = nullptr) {
    typedef typename KVType<WT>::type KT;
    const hivis_config& g = c->cfg;
    AttnShape sh{};
    sh.Hq = g.n_q_heads; sh.Hkv = g.n_kv_heads; sh.m = m;
    const int group = g.n_q_heads / g.n_kv_heads;
    if (m >= ATT_RMAX) { sh.mi = ATT_RMAX; sh.gh = 1; }
    else { sh.mi = m; sh.gh = std::max(1, std::min(group, ATT_RMAX / m)); }
    sh.n_hblk = (group + sh.gh - 1) / sh.gh; sh.n_rblk = (m + sh.mi - 1) / sh.mi;
    sh.seq0 = seq0; sh.offset = offset; sh.maxL = kv.maxL; sh.ldq = ldq; sh.nwaves = 4; sh.tmask = tmask;
    const int items = nseq * g.n_kv_heads * sh.n_hblk * sh.n_rblk;
    // enough workgroups to occupy the chip, at most one 64-key tile per wavefront slot
    const int tiles = (max_keys + 63) / 64;
    int nsplit = std::max(1, std::min((2 * c->num_cu + items - 1) / items, (tiles + 3) / 4));
    nsplit = std::min(nsplit, 16);
    sh.nsplit = nsplit;
    const size_t need = (size_t)items * nsplit * 4 * ATT_RMAX * (g.head_dim + 2);
    if (need > c->attn_ws_floats) return fail(c, HIVIS_EINVAL, "attention workspace too small (%zu > %zu)", need, c->attn_ws_floats);
    if (g.head_dim == 128) {
        hipLaunchKernelGGL((attn_partial_kernel<KT, 128>), dim3(items, nsplit), dim3(256), 0, c->stream, q, (const KT*)kv.k, (const KT*)kv.v, base, sh, c->attn_ws);
        hipLaunchKernelGGL((attn_merge_kernel<128>), dim3(items), dim3(256), 0, c->stream, c->attn_ws, base, sh, out, ldo);
    } else {
        hipLaunchKernelGGL((attn_partial_kernel<KT, 64>), dim3(items, nsplit), dim3(256), 0, c->stream, q, (const KT*)kv.k, (const KT*)kv.v, base, sh, c->attn_ws);
        hipLaunchKernelGGL((attn_merge_kernel<64>), dim3(items), dim3(256), 0, c->stream, c->attn_ws, base, sh, out, ldo);
    }
    HIP_TRY(c, hipGetLastError());
    return HIVIS_OK;
}

AttnShape fused_attn_shape(hivis_ctx* c, int nseq, int m, int offset, int maxL, int ldq, int* items_out);

// Attention of nseq x m rows on the matrix cores, outside a phase program (prefill; passes with more rows than one MFMA
// tile): the same workgroup routine as the verify pass (one item = one kv head x <= 8 (head,row) pairs, all visible
// keys, no key split), launched once over all items.  Rows of sequence seq0 + s sit at positions base[seq0 + s] + offset + i.
template <typename WT>
int attention_rows_mfma(hivis_ctx* c, const float* q, int ldq, const KVDev& kv, const int* base, int offset, int seq0, int nseq, int m,
                        float* out, int ldo, const unsigned long long* tmask = nullptr, uint4* frag_out = nullptr, bool* wrote_frag = nullptr) {
    // frag_out / wrote_frag (optional): where the kernel chosen can, the rows go out as A fragments of the next GEMM
    // (K = ldo) instead of fp32 rows, and *wrote_frag says so
    if (wrote_frag) *wrote_frag = false;
    const hivis_config& g = c->cfg;
    typedef typename KVType<WT>::type KT;
    if constexpr (std::is_same<KT, f16_t>::value) {
        if (m >= c->attn_shared_min && tmask == nullptr) {
            // long causal row ranges (prefill): 128 rows of one head per workgroup, key tiles shared through LDS
            AttnShape sh{};
            sh.Hq = g.n_q_heads; sh.Hkv = g.n_kv_heads; sh.m = m; sh.mi = ATTN_SHARED_ROWS; sh.gh = 1;
            sh.n_hblk = g.n_q_heads / g.n_kv_heads; sh.n_rblk = (m + ATTN_SHARED_ROWS - 1) / ATTN_SHARED_ROWS;
            sh.seq0 = seq0; sh.offset = offset; sh.maxL = kv.maxL; sh.ldq = ldq; sh.nwaves = FUSED_NW; sh.nsplit = 1; sh.tmask = nullptr;
            const int items = nseq * g.n_q_heads * sh.n_rblk;
            const size_t lds = attn_shared_lds_bytes(g.head_dim);
            if (g.head_dim == 128) hipLaunchKernelGGL((attn_rows_shared_kernel<128>), dim3(items), dim3(FUSED_NT), lds, c->stream, q, (const f16_t*)kv.k, (const f16_t*)kv.v, base, sh, out, ldo);
            else hipLaunchKernelGGL((attn_rows_shared_kernel<64>), dim3(items), dim3(FUSED_NT), lds, c->stream, q, (const f16_t*)kv.k, (const f16_t*)kv.v, base, sh, out, ldo);
            HIP_TRY(c, hipGetLastError());
            return HIVIS_OK;
        }
        if (m > FUSED_RMAX) {
            // many rows per sequence: 16 (head,row) pairs per work item
            AttnShape sh{};
            sh.Hq = g.n_q_heads; sh.Hkv = g.n_kv_heads; sh.m = m;
            const int group = g.n_q_heads / g.n_kv_heads;
            if (m >= ATTN_ROWS_RM) { sh.mi = ATTN_ROWS_RM; sh.gh = 1; }
            else { sh.mi = m; sh.gh = std::max(1, std::min(group, ATTN_ROWS_RM / m)); }
            sh.n_hblk = (group + sh.gh - 1) / sh.gh; sh.n_rblk = (m + sh.mi - 1) / sh.mi;
            sh.seq0 = seq0; sh.offset = offset; sh.maxL = kv.maxL; sh.ldq = ldq; sh.nwaves = FUSED_NW; sh.nsplit = 1; sh.tmask = tmask;
            const int items = nseq * g.n_kv_heads * sh.n_hblk * sh.n_rblk;
            const size_t lds = fused_attn_mfma_lds_floats(g.head_dim, FUSED_NW, ATTN_ROWS_RM) * sizeof(float);
            uint4* frag = (frag_out && wrote_frag && ldo % 32 == 0) ? frag_out : nullptr;
            if (frag) *wrote_frag = true;
            if (g.head_dim == 128) {
                static bool attr128 = false;
                if (!attr128) { HIP_TRY(c, hipFuncSetAttribute((const void*)attn_rows_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)); attr128 = true; }
                hipLaunchKernelGGL((attn_rows_kernel<128>), dim3(items), dim3(FUSED_NT), lds, c->stream, q, (const f16_t*)kv.k, (const f16_t*)kv.v, base, sh, out, ldo, frag);
            } else {
                static bool attr64 = false;
                if (!attr64) { HIP_TRY(c, hipFuncSetAttribute((const void*)attn_rows_kernel<64>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)); attr64 = true; }
                hipLaunchKernelGGL((attn_rows_kernel<64>), dim3(items), dim3(FUSED_NT), lds, c->stream, q, (const f16_t*)kv.k, (const f16_t*)kv.v, base, sh, out, ldo, frag);
            }
            HIP_TRY(c, hipGetLastError());
            return HIVIS_OK;
        }
    }
    int items = 0;
    Phase ph{};
    ph.type = PH_ATTN;
    ph.att = fused_attn_shape(c, nseq, m, offset, kv.maxL, ldq, &items);
    ph.att.seq0 = seq0; ph.att.nsplit = 1; ph.att.tmask = tmask; ph.att.flags = c->attn_flags;
    ph.att_items = items;
    ph.A = q; ph.kc = kv.k; ph.vc = kv.v; ph.maxL = kv.maxL; ph.base = base; ph.offset = offset;
    ph.Y = out; ph.ldy = ldo; ph.ws = nullptr; ph.cnt = nullptr;
    if (c->attn_elect && items <= c->rows_cnt_n) {
        // long caches: the key range of an item is split over workgroups and the last one to arrive merges (as in the
        // phase programs); the host mirrors the cache lengths that `base` holds
        const std::vector<int>* hl = base == c->tlen ? &c->h_tlen : base == c->dlen ? &c->h_dlen : nullptr;
        int max_keys = 0;
        for (int s = 0; s < nseq; ++s) max_keys = std::max(max_keys, (hl ? (*hl)[seq0 + s] : 0) + offset + m);
        int nsplit = std::min({ATTN_MAX_SPLITS, (max_keys + c->keys_per_split - 1) / c->keys_per_split, std::max(1, c->fused_grid / items)});    // no more workgroups than CUs: with more, C5's 160 items got slower (8.8 -> 9.6 ms per verify)
        while (nsplit > 1 && (size_t)items * nsplit * FUSED_RMAX * (g.head_dim + 2) > c->attn_ws_floats) --nsplit;
        if (nsplit > 1) { ph.att.nsplit = nsplit; ph.ws = c->attn_ws; ph.cnt = c->rows_cnt; }
    }
    if constexpr (std::is_same<typename KVType<WT>::type, f16_t>::value) {
        if (ph.att.nsplit == 1 && frag_out && wrote_frag && ldo % 32 == 0) { ph.frag = frag_out; *wrote_frag = true; }
    }
    const int grid = ((ph.att.flags & 2) ? 8 * ((items + 7) / 8) : items) * ph.att.nsplit;
    PassParams pp{};
    pp.M = nseq * m; pp.nseq = nseq; pp.m = m; pp.d = g.d; pp.Hq = g.n_q_heads; pp.Hkv = g.n_kv_heads; pp.hd = g.head_dim; pp.F = g.ffn; pp.V = g.vocab;
    hipLaunchKernelGGL((phase_kernel<WT, PH_ATTN, 0, false>), dim3(grid), dim3(FUSED_NT), c->fused_lds, c->stream, ph, pp);
    HIP_TRY(c, hipGetLastError());
    return HIVIS_OK;
}

// One decoder layer on M = nseq*m rows.  h: residual stream [M][d] (in place).  `pending` (may be null) is a delta
// from the previous layer that has not been added to h yet; on return *pending_out is this layer's MLP output, still
// to be added by the caller (the next layer's first norm, or a final norm/add, fuses that addition).
template <typename WT>
int layer_forward(hivis_ctx* c, const LayerDev& L, const KVDev& kv, float* h, const float* pending, const int* base,
                  int offset, int seq0, int nseq, int m, int max_keys, TreeRows tr = TreeRows()) {
    typedef typename KVType<WT>::type KT;
    const hivis_config& g = c->cfg;
    const int M = nseq * m, d = g.d, qd = g.n_q_heads * g.head_dim, kd = g.n_kv_heads * g.head_dim, F = g.ffn;
    const int nqkv = qd + 2 * kd;
    hipLaunchKernelGGL((add_rmsnorm_kernel<WT>), dim3(M), dim3(256), 0, c->stream, h, d, pending, d, (const WT*)L.norm1, c->a, d, d, g.rms_eps);
    if (int rc = gemm<WT>(c, c->a, d, M, d, L.wqkv, nqkv, c->qkv, nqkv, EPI_STORE)) return rc;
    hipLaunchKernelGGL((rope_append_kernel<KT>), dim3(M, row_chunks(M)), dim3(256), 0, c->stream, c->qkv, g.n_q_heads, g.n_kv_heads, g.head_dim, base, offset, seq0, m, (KT*)kv.k, (KT*)kv.v, kv.maxL, g.rope_theta, tr.pos_delta, (const float*)L.bqkv, (const float*)c->rope_tab, g.max_vis + g.max_text);
    if (c->fused && std::is_same<KT, f16_t>::value) { if (int rc = attention_rows_mfma<WT>(c, c->qkv, nqkv, kv, base, offset, seq0, nseq, m, c->att, qd, tr.mask)) return rc; }
    else if (int rc = attention<WT>(c, c->qkv, nqkv, kv, base, offset, seq0, nseq, m, max_keys, c->att, qd, tr.mask)) return rc;
    if (int rc = gemm<WT>(c, c->att, qd, M, qd, L.wo, d, c->proj, d, EPI_STORE)) return rc;
    hipLaunchKernelGGL((add_rmsnorm_kernel<WT>), dim3(M), dim3(256), 0, c->stream, h, d, (const float*)c->proj, d, (const WT*)L.norm2, c->a, d, d, g.rms_eps);
    if (int rc = gemm<WT>(c, c->a, d, M, d, L.wgu, 2 * F, c->gu, 2 * F, EPI_STORE)) return rc;
    hipLaunchKernelGGL(silu_mul_kernel, dim3(M, row_chunks(M)), dim3(256), 0, c->stream, (const float*)c->gu, c->act, F);
    if (int rc = gemm<WT>(c, c->act, F, M, F, L.wd, d, c->proj, d, EPI_STORE)) return rc;
    HIP_TRY(c, hipGetLastError());
    return HIVIS_OK;   // c->proj holds the MLP delta, not yet added to h
}

// Target pass over M = nseq*m rows already in c->x; leaves post-final-norm features in out (row stride ldo)
// for rows >= first_out_row (pointer arithmetic done by the caller through first_out_row).
template <typename WT>
int target_forward(hivis_ctx* c, int seq0, int nseq, int m, const int* base, int offset, int max_keys, float* out, int ldo,
                   int first_out_row, TreeRows tr = TreeRows()) {
    const hivis_config& g = c->cfg;
    const int M = nseq * m;
    const float* pending = nullptr;
    if constexpr (sizeof(WT) == 2) {
        if (M >= c->wide_min && M <= MAX_ROWS && c->fused && c->pf_frag && c->pf_rows >= MAX_ROWS && g.d <= 8192 && !c->no_wide_gemm) {
            Parts pend{nullptr, 0, 0};
            for (int l = 0; l < g.n_layers; ++l)
                if (int rc = layer_forward_wide<WT>(c, c->layers[l], c->tkv[l], c->x, pend, base, offset, seq0, nseq, m, tr, &pend)) return rc;
            if (pend.n > 1) hipLaunchKernelGGL(splitk_reduce_kernel, dim3(M, row_chunks(M)), dim3(256), 0, c->stream, pend.p, pend.n, M, g.d, g.d, c->proj, g.d);
            const int nout_w = M - first_out_row;
            if (nout_w > 0)
                hipLaunchKernelGGL((add_rmsnorm_kernel<WT>), dim3(nout_w), dim3(256), 0, c->stream, c->x + (size_t)first_out_row * g.d, g.d,
                                   (const float*)c->proj + (size_t)first_out_row * g.d, g.d, (const WT*)c->final_norm, out, ldo, g.d, g.rms_eps);
            HIP_TRY(c, hipGetLastError());
            return HIVIS_OK;
        }
    }
    for (int l = 0; l < g.n_layers; ++l) {
        // KV of layer l for all sequences
        if (int rc = layer_forward<WT>(c, c->layers[l], c->tkv[l], c->x, pending, base, offset, seq0, nseq, m, max_keys, tr)) return rc;
        pending = c->proj;
    }
    const int nout = M - first_out_row;
    if (nout > 0)
        hipLaunchKernelGGL((add_rmsnorm_kernel<WT>), dim3(nout), dim3(256), 0, c->stream, c->x + (size_t)first_out_row * g.d, g.d,
                           pending + (size_t)first_out_row * g.d, g.d, (const WT*)c->final_norm, out, ldo, g.d, g.rms_eps);
    HIP_TRY(c, hipGetLastError());
    return HIVIS_OK;
}

// Drafter: fusion FC on cat rows [M][2d] + rho_idx, then its single layer; output rows (h + mlp delta) to out.
template <typename WT>
int drafter_forward(hivis_ctx* c, const float* cat, int seq0, int nseq, int m, int rho_idx, int offset, int max_keys,
                    float* out, int ldo, TreeRows tr = TreeRows()) {
    const hivis_config& g = c->cfg;
    const int M = nseq * m, d = g.d;
    if (int rc = gemm<WT>(c, cat, 2 * d, M, 2 * d, c->fuse_w, d, c->u, d, EPI_STORE)) return rc;
    hipLaunchKernelGGL((add_rho_kernel<WT>), dim3(M), dim3(256), 0, c->stream, c->u, d, (const WT*)c->rho, rho_idx, d);
    bool wide = false;
    if constexpr (sizeof(WT) == 2) wide = M >= c->wide_min && M <= MAX_ROWS && c->fused && c->pf_frag && c->pf_rows >= MAX_ROWS && d <= 8192 && !c->no_wide_gemm;
    if (wide) {
        if constexpr (sizeof(WT) == 2) {
            Parts pend{nullptr, 0, 0};
            if (int rc = layer_forward_wide<WT>(c, c->draft, c->dkv, c->u, pend, c->dlen, offset, seq0, nseq, m, tr, &pend)) return rc;
            if (pend.n > 1) hipLaunchKernelGGL(splitk_reduce_kernel, dim3(M, row_chunks(M)), dim3(256), 0, c->stream, pend.p, pend.n, M, d, d, c->proj, d);
        }
    } else if (int rc = layer_forward<WT>(c, c->draft, c->dkv, c->u, nullptr, c->dlen, offset, seq0, nseq, m, max_keys, tr)) return rc;
    hipLaunchKernelGGL(add_rows_kernel, dim3(M), dim3(256), 0, c->stream, (const float*)c->u, d, (const float*)c->proj, d, out, ldo, d);
    HIP_TRY(c, hipGetLastError());
    return HIVIS_OK;
}


// ---- persistent-kernel path --------------------------------------------------------------------
enum { PROG_VERIFY = 0, PROG_DRAFT = 1, PROG_ROLL = 2, PROG_DRAFT_SAMPLE = 3 };

template <typename WT>
bool fused_rows_ok(int M) { return M <= WTraits<WT>::ROWS; }

AttnShape fused_attn_shape(hivis_ctx* c, int nseq, int m, int offset, int maxL, int ldq, int* items_out) {
    const hivis_config& g = c->cfg;
    AttnShape sh{};
    sh.Hq = g.n_q_heads; sh.Hkv = g.n_kv_heads; sh.m = m;
    const int group = g.n_q_heads / g.n_kv_heads;
    if (m >= FUSED_RMAX) { sh.mi = FUSED_RMAX; sh.gh = 1; }
    else { sh.mi = m; sh.gh = std::max(1, std::min(group, FUSED_RMAX / m)); }
    sh.n_hblk = (group + sh.gh - 1) / sh.gh; sh.n_rblk = (m + sh.mi - 1) / sh.mi;
    sh.seq0 = 0; sh.offset = offset; sh.maxL = maxL; sh.ldq = ldq; sh.nwaves = FUSED_NW;
    const int items = nseq * g.n_kv_heads * sh.n_hblk * sh.n_rblk;
    sh.nsplit = std::min(ATTN_MAX_SPLITS, std::max(1, c->fused_grid / items));
    *items_out = items;
    return sh;
}

// Bump allocator for the per-phase output buffers of one program (first pass counts, second pass hands out).
struct Pool {
    float* base = nullptr; size_t used = 0;
    float* take(size_t floats) {
        floats = (floats + 63) & ~(size_t)63;            // 256-byte granules: buffers never share a cache line
        float* p = base ? base + used : nullptr;
        used += floats;
        return p;
    }
};

// phases of one decoder layer on rows h [M][d]; returns the buffer holding h + attention + MLP.  Every phase
// writes into a buffer of its own (see the memory discipline in hivis_fused.h).  dst: optional fixed destination
// of the layer output (row stride ldd).
template <typename WT>
float* layer_phases(hivis_ctx* c, std::vector<Phase>& P, Pool& pool, const LayerDev& L, const KVDev& kv, float* h, const int* base,
                    int offset, int nseq, int m, float* dst, int ldd, int* ld_out, bool persistent, bool elect) {
    const hivis_config& g = c->cfg;
    const int M = nseq * m;
    const int d = g.d, qd = g.n_q_heads * g.head_dim, kd = g.n_kv_heads * g.head_dim, F = g.ffn, nqkv = qd + 2 * kd;
    float* qkv = pool.take((size_t)M * nqkv);
    float* att = pool.take((size_t)M * qd);
    float* h1 = pool.take((size_t)M * d);
    float* act = pool.take((size_t)M * F);
    float* h2 = dst ? dst : pool.take((size_t)M * d);
    const int ld2 = dst ? ldd : d;
    Phase q{}; q.type = PH_GEMM; q.pro = PRO_RMS; q.epi = FEPI_QKV; q.K = d; q.N = nqkv; q.W = L.wqkv; q.A = h; q.lda = d;
    q.gain = L.norm1; q.Y = qkv; q.ldy = nqkv; q.kc = kv.k; q.vc = kv.v; q.maxL = kv.maxL; q.base = base; q.offset = offset; q.rope = c->rope_tab; q.bias = L.bqkv;
    P.push_back(q);
    Phase a{}; a.type = PH_ATTN; a.A = qkv; a.lda = nqkv; a.kc = kv.k; a.vc = kv.v; a.maxL = kv.maxL; a.base = base; a.offset = offset;
    a.att = fused_attn_shape(c, nseq, m, offset, kv.maxL, nqkv, &a.att_items);
    a.ws = pool.take((size_t)a.att_items * a.att.nsplit * FUSED_RMAX * (g.head_dim + 2));
    if (persistent || elect) {
        a.cnt = (int*)pool.take((size_t)a.att_items);  // zero from the pool's memset; the merging workgroup re-zeroes it
        a.Y = att; a.ldy = qd;
        P.push_back(a);
    } else {
        // key splits merged by a launch of their own
        a.cnt = nullptr; a.Y = att; a.ldy = qd;
        P.push_back(a);
        Phase mg = a; mg.type = PH_ATTN_MERGE; mg.Y = att; mg.ldy = qd;
        P.push_back(mg);
    }
    Phase o{}; o.type = PH_GEMM; o.pro = PRO_PLAIN; o.epi = FEPI_ADD_TO; o.K = qd; o.N = d; o.W = L.wo; o.A = att; o.lda = qd;
    o.Y = h1; o.ldy = d; o.R = h; o.ldr = d;
    P.push_back(o);
    Phase gu{}; gu.type = PH_GEMM; gu.pro = PRO_RMS; gu.epi = FEPI_SILU; gu.K = d; gu.N = 2 * F; gu.W = L.wgu; gu.A = h1; gu.lda = d;
    gu.gain = L.norm2; gu.Y = act; gu.ldy = F;
    P.push_back(gu);
    Phase dn{}; dn.type = PH_GEMM; dn.pro = PRO_PLAIN; dn.epi = FEPI_ADD_TO; dn.K = F; dn.N = d; dn.W = L.wd; dn.A = act; dn.lda = F;
    dn.Y = h2; dn.ldy = ld2; dn.R = h1; dn.ldr = d;
    P.push_back(dn);
    *ld_out = ld2;
    return h2;
}

template <typename WT>
void build_phases(hivis_ctx* c, int kind, int K, Pool& pool, std::vector<Phase>& P, bool persistent, bool elect) {
    const hivis_config& g = c->cfg;
    const int B = g.batch, d = g.d, V = g.vocab, G = c->fused_grid;
    int ld = d;
    // Launch-per-phase programs fold two small phases away: the gather of Embed(x) into the fusion FC (its activation
    // columns [d, 2d) come straight from the embedding table), and, with `elect`, the greedy-token reduction into the
    // LM-head phase (the workgroup that arrives last reduces the candidates).  The single-launch program keeps both phases.
    const bool fold = !persistent;
    const bool lm_elect = elect && !persistent;
    if (kind == PROG_VERIFY) {
        const int m = K + 1, M = B * m;
        float* x = pool.take((size_t)M * d);
        Phase pr{}; pr.type = PH_PREP; pr.ids = c->row_tok; pr.id_sseq = m; pr.id_srow = 1; pr.gain = c->embed; pr.Y = x; pr.ldy = d;
        pr.base = c->tlen; pr.offset = 0;
        P.push_back(pr);
        for (int l = 0; l < g.n_layers; ++l) x = layer_phases<WT>(c, P, pool, c->layers[l], c->tkv[l], x, c->tlen, 0, B, m, nullptr, 0, &ld, persistent, elect);
        Phase nr{}; nr.type = PH_NORM_ROWS; nr.A = x; nr.lda = d; nr.gain = c->final_norm; nr.Y = c->catT; nr.ldy = 2 * d;
        P.push_back(nr);
        Phase lm{}; lm.type = PH_GEMM; lm.pro = PRO_PLAIN; lm.epi = FEPI_LOGITS; lm.K = d; lm.N = V; lm.W = c->lm_head; lm.A = c->catT; lm.lda = 2 * d;
        lm.Y = c->logits_v; lm.ldy = V; lm.pm = pool.take((size_t)M * G); lm.pi = (int*)pool.take((size_t)M * G);
        lm.tok_out = c->ttok; lm.o_sseq = g.k_max + 1; lm.o_srow = 1;
        if (lm_elect) lm.cnt = (int*)pool.take(1);         // zero from the pool's memset; the reducing workgroup re-zeroes it
        P.push_back(lm);
        if (!lm_elect) {
            Phase am{}; am.type = PH_ARGMAX; am.tok_out = c->ttok; am.o_sseq = g.k_max + 1; am.o_srow = 1; am.pm = lm.pm; am.pi = lm.pi; am.N = G;
            P.push_back(am);
        }
    } else if (kind == PROG_DRAFT || kind == PROG_DRAFT_SAMPLE) {
        // cat: [B][2d] = drafter hidden f' | embedding of the token drafted from it; a fresh buffer per step
        float* cat = c->catD;
        for (int i = 1; i <= K; ++i) {
            Phase lm{}; lm.type = PH_GEMM; lm.pro = PRO_PLAIN; lm.epi = FEPI_LOGITS; lm.K = d; lm.N = V; lm.W = c->lm_head; lm.A = cat; lm.lda = 2 * d;
            lm.Y = c->logits_d + (size_t)(i - 1) * B * V; lm.ldy = V; lm.pm = pool.take((size_t)B * G); lm.pi = (int*)pool.take((size_t)B * G);
            lm.tok_out = c->drafts + (i - 1); lm.o_sseq = g.k_max; lm.o_srow = 0;
            // greedy token of step i: reduced by the fusion FC that follows (steps before the last), by the LM head's last
            // workgroup (last step, with `elect`), or by a phase of its own
            const bool in_fc = fold && kind == PROG_DRAFT && i < K;
            // ... and with the extended LM head there is no FC phase: this LM-head launch also computes f' w1 + rho for the
            // next step (d extra columns), and the next step's QKV phase reduces the token and adds the table row of it
            const bool ext = in_fc && c->lm_ext && B <= 4;       // (the QKV variants that add the table rows stage two or four rows)
            float* u_part = ext ? pool.take((size_t)B * d) : nullptr;
            if (ext) { lm.N = V + d; lm.Y2 = u_part; lm.ldy2 = d; lm.vec = c->rho; lm.vec_idx = std::min(i, g.n_resid - 1); }
            const bool in_lm = !in_fc && lm_elect && kind == PROG_DRAFT;
            if (in_lm) lm.cnt = (int*)pool.take(1);
            P.push_back(lm);
            if (!in_lm && !in_fc) {
                Phase am{}; am.type = PH_ARGMAX; am.tok_out = c->drafts + (i - 1); am.o_sseq = g.k_max; am.o_srow = 0; am.pm = lm.pm; am.pi = lm.pi; am.N = G;
                if (kind == PROG_DRAFT_SAMPLE) {     // the token is drawn from softmax(logits / T) instead (uniforms [B][k_max], column i-1)
                    am.type = PH_SAMPLE; am.A = lm.Y; am.lda = V; am.u = c->u_draft; am.u_sseq = g.k_max; am.u_idx = i - 1;
                }
                P.push_back(am);
            }
            if (i < K) {
                float* u = pool.take((size_t)B * d);
                float* cat_next = pool.take((size_t)B * 2 * d);
                Phase fu{}; fu.type = PH_GEMM; fu.pro = PRO_PLAIN; fu.epi = FEPI_ADDVEC; fu.K = 2 * d; fu.N = d; fu.W = c->fuse_w; fu.A = cat; fu.lda = 2 * d;
                fu.Y = u; fu.ldy = d; fu.vec = c->rho; fu.vec_idx = std::min(i, g.n_resid - 1);
                if (fold) {
                    fu.emb = c->embed; fu.tok = c->drafts + (i - 1); fu.tok_sseq = g.k_max; fu.tok_srow = 0;
                    if (c->emb_w2) { fu.emb = nullptr; fu.add_rows = c->emb_w2; fu.K = d; fu.W = c->fuse_w1; }     // embedding half from the table
                    if (in_fc) { fu.tok = nullptr; fu.pm = lm.pm; fu.pi = lm.pi; fu.ncand = G; fu.tok_out = c->drafts + (i - 1); fu.o_sseq = g.k_max; fu.o_srow = 0; }
                }
                else {
                    Phase pr{}; pr.type = PH_PREP; pr.ids = c->drafts + (i - 1); pr.id_sseq = g.k_max; pr.id_srow = 0; pr.gain = c->embed;
                    pr.Y = cat + d; pr.ldy = 2 * d; pr.base = c->dlen; pr.offset = i - 1;
                    P.push_back(pr);
                }
                if (!ext) P.push_back(fu);
                const size_t qi = P.size();
                layer_phases<WT>(c, P, pool, c->draft, c->dkv, u, c->dlen, i - 1, B, 1, cat_next, 2 * d, &ld, persistent, elect);
                if (ext) {      // the layer's first phase (QKV): rows = u_part + table[token], tokens from this step's candidates, u written back
                    Phase& q = P[qi];
                    q.A = u_part; q.lda = d; q.add_rows = c->emb_w2; q.wb = u; q.tok = nullptr; q.pm = lm.pm; q.pi = lm.pi; q.ncand = G;
                    q.tok_out = c->drafts + (i - 1); q.o_sseq = g.k_max; q.o_srow = 0;
                }
                cat = cat_next;
            }
        }
    } else {
        const int m = K + 1, M = B * m;
        float* u = pool.take((size_t)M * d);
        Phase fu{}; fu.type = PH_GEMM; fu.pro = PRO_PLAIN; fu.epi = FEPI_ADDVEC; fu.K = 2 * d; fu.N = d; fu.W = c->fuse_w; fu.A = c->catT; fu.lda = 2 * d;
        fu.Y = u; fu.ldy = d; fu.vec = c->rho; fu.vec_idx = 0;
        if (fold) {
            fu.emb = c->embed; fu.tok = c->next_tok; fu.tok_sseq = g.k_max + 1; fu.tok_srow = 1;
            if (c->emb_w2) { fu.emb = nullptr; fu.add_rows = c->emb_w2; fu.K = d; fu.W = c->fuse_w1; }
        }
        else {
            Phase pr{}; pr.type = PH_PREP; pr.ids = c->next_tok; pr.id_sseq = g.k_max + 1; pr.id_srow = 1; pr.gain = c->embed;
            pr.Y = c->catT + d; pr.ldy = 2 * d; pr.base = c->dlen; pr.offset = 0;
            P.push_back(pr);
        }
        P.push_back(fu);
        layer_phases<WT>(c, P, pool, c->draft, c->dkv, u, c->dlen, 0, B, m, c->dout, d, &ld, persistent, elect);
    }
    // chain the GEMM phases for the cross-barrier weight prefetch
    for (size_t i = 0; i < P.size(); ++i) {
        if (P[i].type != PH_GEMM) continue;
        for (size_t j = i + 1; j < P.size(); ++j)
            if (P[j].type == PH_GEMM) { P[i].next_W = P[j].W; P[i].next_K = P[j].K; P[i].next_N = P[j].N; break; }
    }
}

template <typename WT>
int get_program(hivis_ctx* c, int kind, int K, hivis_ctx::Program* out) {
    const int key = kind * 64 + K;
    auto it = c->programs.find(key);
    if (it != c->programs.end()) { *out = it->second; return HIVIS_OK; }
    std::vector<Phase> P;
    Pool count;
    build_phases<WT>(c, kind, K, count, P, c->persistent, c->attn_elect);           // sizes only
    Pool pool;
    if (int rc = dev_alloc(c, &pool.base, count.used)) return rc;
    HIP_TRY(c, hipMemset(pool.base, 0, count.used * sizeof(float)));
    P.clear();
    build_phases<WT>(c, kind, K, pool, P, c->persistent, c->attn_elect);
    hivis_ctx::Program pg;
    pg.n = (int)P.size();
    if (int rc = dev_alloc(c, &pg.dev, P.size())) return rc;
    HIP_TRY(c, hipMemcpy(pg.dev, P.data(), P.size() * sizeof(Phase), hipMemcpyHostToDevice));
    pg.host = new std::vector<Phase>(P);
    c->programs[key] = pg;
    *out = pg;
    return HIVIS_OK;
}

// One launch per phase (the default way a pass runs): grids sized to the phase's work.  phases: host array of n phases.
template <typename WT>
int launch_phases(hivis_ctx* c, const Phase* phases, int n, int kind, int K, const PassParams& pp, bool do_prof) {
    const hivis_config& g = c->cfg;
    // one launch per phase; grids sized to the phase's work
    // key splits per attention item: enough workgroups to fill the chip for long caches, a single workgroup (and no
    // merge launch) for short ones; the program was sized for the largest split count
    int max_keys = 0;
    for (int b = 0; b < g.batch; ++b) max_keys = std::max(max_keys, (kind == PROG_VERIFY ? c->h_tlen[b] : c->h_dlen[b]) + K + 1);
    for (int p = 0; p < n; ++p) {
        Phase ph = phases[p];
        ph.next_W = nullptr;                       // nothing is prefetched across a kernel boundary (pulling the next launch's
                                                   // first units into L2 during the epilogue was measured: 3% slower)
        if (ph.type == PH_ATTN || ph.type == PH_ATTN_MERGE) {
            ph.att.nsplit = std::max(1, std::min(ph.att.nsplit, (max_keys + c->keys_per_split - 1) / c->keys_per_split));
            ph.att.flags = c->attn_flags;
        }
        if (ph.type == PH_ATTN || ph.type == PH_ATTN_MERGE || (ph.type == PH_GEMM && ph.epi == FEPI_QKV)) {
            if (g.batch <= 8 && ph.att.seq0 == 0) {          // the lengths the device arrays hold right now, by value
                ph.att.nbase = g.batch;
                for (int b = 0; b < g.batch; ++b) ph.att.base_val[b] = kind == PROG_VERIFY ? c->h_tlen[b] : c->h_dlen[b];
            }
            if (ph.type == PH_ATTN_MERGE && ph.att.nsplit == 1) continue;
        }
        int grid = c->fused_grid;
        if (ph.type == PH_ATTN) grid = std::min(grid, ((ph.att.flags & 2) ? 8 * ((ph.att_items + 7) / 8) : ph.att_items) * ph.att.nsplit);
        else if (ph.type == PH_ATTN_MERGE) grid = std::min(grid, ph.att_items);
        else if (ph.type == PH_PREP) grid = std::min(grid, pp.M);
        else if (ph.type == PH_NORM_ROWS) grid = std::min(grid, pp.M);
        else if (ph.type == PH_ARGMAX) grid = std::min(grid, (pp.M + FUSED_NW - 1) / FUSED_NW);
        else if (ph.type == PH_SAMPLE) grid = std::min(grid, pp.M);
        else if (ph.type == PH_GEMM && ph.epi != FEPI_LOGITS) grid = std::min(grid, ph.N / 16);
        PassParams ppl = pp;
        if (do_prof) { ppl.prof2 = pp.prof2 + (size_t)p * 8; if (p >= n / 2 && p < n / 2 + 8) ppl.prof3 = c->prof + 4096 * 11 + (size_t)(p - n / 2) * 4096; }
        // kev0/kev1 (null unless this launch is timed) are attached to the dispatch itself: they read the kernel's own
        // start and end timestamps, with no marker packets before or after it in the queue
#define HIVIS_LAUNCH(TY, EP) do { if (single) hipExtLaunchKernelGGL((phase_kernel<WT, TY, EP, true>), dim3(grid), dim3(FUSED_NT), c->fused_lds, c->stream, kev0, kev1, 0, ph, ppl); \
                              else hipExtLaunchKernelGGL((phase_kernel<WT, TY, EP, false>), dim3(grid), dim3(FUSED_NT), c->fused_lds, c->stream, kev0, kev1, 0, ph, ppl); } while (0)
        const bool single = ph.type == PH_GEMM && ph.epi != FEPI_LOGITS && ph.epi != FEPI_SILU && ph.epi != FEPI_QKV && ph.N / 16 <= grid;   // one tile per workgroup at most
        const bool kmatch = kind == PROG_VERIFY && ph.type == PH_GEMM && ph.epi == c->ktime_epi;
        const int64_t kseq = kmatch ? c->ktime_seen++ : 0;
        const bool ktimed = kmatch && (kseq % c->ktime_stride) == 0;
        hipEvent_t kev0 = nullptr, kev1 = nullptr;
        if (ktimed) {
            if (c->kev_used + 2 > c->kev.size()) { hipEvent_t e0, e1; HIP_TRY(c, hipEventCreate(&e0)); HIP_TRY(c, hipEventCreate(&e1)); c->kev.push_back(e0); c->kev.push_back(e1); }
            kev0 = c->kev[c->kev_used]; kev1 = c->kev[c->kev_used + 1];
            c->kev_used += 2;
            c->kbytes = (double)ph.K * ph.N * c->esize;
        }
        switch (ph.type) {
        case PH_GEMM:
            switch (ph.epi) {
            case FEPI_STORE: HIVIS_LAUNCH(PH_GEMM, FEPI_STORE); break;
            case FEPI_ADD_TO: HIVIS_LAUNCH(PH_GEMM, FEPI_ADD_TO); break;
            case FEPI_ADDVEC: HIVIS_LAUNCH(PH_GEMM, FEPI_ADDVEC); break;
            case FEPI_QKV:
                if (ph.add_rows && pp.M <= 2) HIVIS_LAUNCH(PH_GEMM, FEPI_QKV_TAB);
                else if (ph.add_rows) HIVIS_LAUNCH(PH_GEMM, FEPI_QKV_TAB4);
                else HIVIS_LAUNCH(PH_GEMM, FEPI_QKV);
                break;
            case FEPI_SILU: HIVIS_LAUNCH(PH_GEMM, FEPI_SILU); break;
            default: HIVIS_LAUNCH(PH_GEMM, FEPI_LOGITS); break;
            }
            break;
        case PH_ATTN: HIVIS_LAUNCH(PH_ATTN, 0); break;
        case PH_ATTN_MERGE: HIVIS_LAUNCH(PH_ATTN_MERGE, 0); break;
        case PH_PREP: HIVIS_LAUNCH(PH_PREP, 0); break;
        case PH_NORM_ROWS: HIVIS_LAUNCH(PH_NORM_ROWS, 0); break;
        case PH_SAMPLE: HIVIS_LAUNCH(PH_SAMPLE, 0); break;
        default: HIVIS_LAUNCH(PH_ARGMAX, 0); break;
        }
#undef HIVIS_LAUNCH
    }
    HIP_TRY(c, hipGetLastError());
    return HIVIS_OK;
}

template <typename WT>
int run_program(hivis_ctx* c, int kind, int K, int nseq, int m) {
    hivis_ctx::Program pg;
    if (int rc = get_program<WT>(c, kind, K, &pg)) return rc;
    const hivis_config& g = c->cfg;
    PassParams pp{};
    pp.phases = pg.dev; pp.nphases = pg.n;
    pp.M = nseq * m; pp.nseq = nseq; pp.m = m;
    pp.d = g.d; pp.Hq = g.n_q_heads; pp.Hkv = g.n_kv_heads; pp.hd = g.head_dim; pp.F = g.ffn; pp.V = g.vocab;
    pp.eps = g.rms_eps; pp.theta = g.rope_theta; pp.inv_temp = c->inv_temp;
    pp.bar = c->bar; pp.bad = c->bad;
    pp.spin_limit = 1u << 22;
    const bool do_prof = c->prof && kind == PROG_VERIFY && c->prof_left > 0;
    pp.prof = do_prof ? c->prof : nullptr;
    pp.prof2 = do_prof ? c->prof + 4096 * 3 : nullptr;
    if (!c->persistent) {
        if (int rc = launch_phases<WT>(c, pg.host->data(), pg.n, kind, K, pp, do_prof)) return rc;
        if (do_prof) {
            // developer aid: timestamps (100 MHz) that workgroup 0 of each launch wrote, for one layer in the middle
            std::vector<unsigned long long> t2((size_t)pg.n * 8);
            HIP_TRY(c, hipStreamSynchronize(c->stream));
            HIP_TRY(c, hipMemcpy(t2.data(), pp.prof2, t2.size() * 8, hipMemcpyDeviceToHost));
            const int p0 = std::min(pg.n / 2, pg.n - 1);
            for (int p = p0; p < std::min(pg.n, p0 + 14); ++p) {
                const Phase& P = (*pg.host)[p];
                fprintf(stderr, "[hivis prof] phase %d type %d epi %d: entry %+.2f us after previous entry;", p, P.type, P.epi, ((double)t2[p * 8] - (double)t2[(p - 1) * 8]) * 0.01);
                for (int k = 1; k < 7; ++k) fprintf(stderr, " m%d %+.2f", k, ((double)t2[p * 8 + k] - (double)t2[p * 8]) * 0.01);
                fprintf(stderr, "\n");
            }
            // per-workgroup entry/exit of the same launches: spread of the exits, the latest workgroups and where they ran
            std::vector<unsigned long long> t3((size_t)8 * 4096);
            HIP_TRY(c, hipMemcpy(t3.data(), c->prof + 4096 * 11, t3.size() * 8, hipMemcpyDeviceToHost));
            for (int p = p0; p < std::min(pg.n, p0 + 8); ++p) {
                const Phase& P = (*pg.host)[p];
                const unsigned long long* w = t3.data() + (size_t)(p - p0) * 4096;
                std::vector<std::pair<double, int>> ends; double s0 = 1e300, s1 = 0;
                for (int b = 0; b < c->fused_grid && b < 1024; ++b) if (w[b * 4]) { s0 = std::min(s0, (double)w[b * 4]); s1 = std::max(s1, (double)w[b * 4]); }
                for (int b = 0; b < c->fused_grid && b < 1024; ++b) if (w[b * 4]) ends.push_back({((double)w[b * 4 + 1] - s0) * 0.01, b});
                if (ends.empty()) continue;
                std::sort(ends.begin(), ends.end());
                const size_t n = ends.size();
                fprintf(stderr, "[hivis wg] phase %d type %d epi %d: %zu workgroups, entries within %.2f us; exits min %.2f p10 %.2f p50 %.2f p90 %.2f max %.2f us; latest:", p, P.type, P.epi, n,
                        (s1 - s0) * 0.01, ends[0].first, ends[n / 10].first, ends[n / 2].first, ends[n * 9 / 10].first, ends[n - 1].first);
                for (size_t k = n > 6 ? n - 6 : 0; k < n; ++k) {
                    const unsigned long long id = w[ends[k].second * 4 + 2];
                    fprintf(stderr, " wg%d(xcc%llu se%llu cu%llu)", ends[k].second, id >> 32, (id >> 13) & 7, (id >> 8) & 15);
                }
                double xs[8] = {}; int xn[8] = {};
                for (auto& e : ends) { const int x = (int)(w[e.second * 4 + 2] >> 32) & 7; xs[x] += e.first; xn[x]++; }
                fprintf(stderr, "; wg0: entry->mark0 %.2f, mark0->exit %.2f us", ((double)t2[p * 8] - (double)w[0]) * 0.01, ((double)w[1] - (double)t2[p * 8]) * 0.01);
                fprintf(stderr, "; mean exit per xcc:");
                for (int x = 0; x < 8; ++x) fprintf(stderr, " %.1f(%d)", xn[x] ? xs[x] / xn[x] : 0.0, xn[x]);
                fprintf(stderr, "\n");
            }
            HIP_TRY(c, hipMemset(c->prof + 4096 * 11, 0, (size_t)8 * 4096 * 8));
            c->prof_left--;
        }
        return HIVIS_OK;
    }
    hipLaunchKernelGGL(set_ints_kernel, dim3(1), dim3(64), 0, c->stream, (int*)c->bar, 1, 0);
    void* args[] = {&pp};
    HIP_TRY(c, hipLaunchCooperativeKernel((const void*)fused_pass_kernel<WT>, dim3(c->fused_grid), dim3(FUSED_NT), args, c->fused_lds, c->stream));
    if (do_prof) {
        std::vector<unsigned long long> t((size_t)pg.n * 3), t2((size_t)pg.n * 8);
        std::vector<Phase> P(pg.n);
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        HIP_TRY(c, hipMemcpy(t.data(), c->prof, t.size() * 8, hipMemcpyDeviceToHost));
        HIP_TRY(c, hipMemcpy(P.data(), pg.dev, P.size() * sizeof(Phase), hipMemcpyDeviceToHost));
        HIP_TRY(c, hipMemcpy(t2.data(), c->prof + 4096 * 3, t2.size() * 8, hipMemcpyDeviceToHost));
        for (int p = 7; p < 13 && p < pg.n; ++p) if (P[p].type == PH_GEMM)
            fprintf(stderr, "[hivis prof2] phase %d epi %d: entry+%.2f  staged+%.2f  pass0+%.2f  allpass+%.2f  reduced+%.2f  end+%.2f | work %.2f wait %.2f us\n", p, P[p].epi,
                    (t2[p*8]-t[p*3])*0.01, (t2[p*8+1]-t2[p*8])*0.01, (t2[p*8+2]-t2[p*8+1])*0.01, (t2[p*8+3]-t2[p*8+2])*0.01, (t2[p*8+4]-t2[p*8+3])*0.01, (t2[p*8+5]-t2[p*8+4])*0.01, (t[p*3+1]-t[p*3])*0.01, (t[p*3+2]-t[p*3+1])*0.01);
        double tot[8][8] = {}, bar[8][8] = {}; int cnt[8][8] = {};
        for (int p = 0; p < pg.n; ++p) {
            const int ty = P[p].type, ep = P[p].type == PH_GEMM ? P[p].epi : 0;
            tot[ty][ep] += (t[p * 3 + 1] - t[p * 3]) * 0.01; bar[ty][ep] += (t[p * 3 + 2] - t[p * 3 + 1]) * 0.01; cnt[ty][ep]++;
        }
        fprintf(stderr, "[hivis prof] verify pass %.1f us (workgroup 0 view)\n", (t[pg.n * 3 - 1] - t[0]) * 0.01);
        for (int ty = 0; ty < 8; ++ty) for (int ep = 0; ep < 8; ++ep) if (cnt[ty][ep])
            fprintf(stderr, "[hivis prof]   type %d epi %d: n=%3d  work %7.2f us avg, barrier wait %7.2f us avg\n", ty, ep, cnt[ty][ep], tot[ty][ep] / cnt[ty][ep], bar[ty][ep] / cnt[ty][ep]);
        c->prof_left--;
    }
    return HIVIS_OK;
}

// Phases a draft program of K steps needs at most (LM head, token, prep, fusion FC, QKV, attention, merge, O, gate|up, down)
static inline size_t draft_phase_capacity(int k_max) { return (size_t)k_max * 10 + 4; }

// The draft round of do_draft with every intermediate buffer inside the static scratch array: the same phase list and
// the same kernels (always one launch per phase), built into host storage reserved at create; no allocation of any kind.
template <typename WT>
int draft_noalloc(hivis_ctx* c, int K) {
    const hivis_config& g = c->cfg;
    std::vector<Phase>& P = c->na_phases;
    if (draft_phase_capacity(K) > P.capacity()) return fail(c, HIVIS_ECAP, "phase list of K=%d exceeds the storage reserved at create", K);
    P.clear();
    Pool count;
    build_phases<WT>(c, PROG_DRAFT, K, count, P, false, false);            // sizes only
    const size_t need = count.used * sizeof(float);
    if (need > (size_t)HIVIS_SCRATCH_BYTES)
        return fail(c, HIVIS_ECAP, "draft round of K=%d needs %zu bytes of scratch, the static array holds %u", K, need, (unsigned)HIVIS_SCRATCH_BYTES);
    P.clear();
    Pool pool; pool.base = (float*)c->scratch_dev;                  // the looked-up device address, not the array's name
    build_phases<WT>(c, PROG_DRAFT, K, pool, P, false, false);
    PassParams pp{};
    pp.phases = nullptr; pp.nphases = (int)P.size();
    pp.M = g.batch; pp.nseq = g.batch; pp.m = 1;
    pp.d = g.d; pp.Hq = g.n_q_heads; pp.Hkv = g.n_kv_heads; pp.hd = g.head_dim; pp.F = g.ffn; pp.V = g.vocab;
    pp.eps = g.rms_eps; pp.theta = g.rope_theta; pp.inv_temp = c->inv_temp;
    pp.bar = c->bar; pp.bad = c->bad; pp.spin_limit = 1u << 22;
    return launch_phases<WT>(c, P.data(), (int)P.size(), PROG_DRAFT, K, pp, false);
}

template <typename WT>
int fused_setup(hivis_ctx* c) {
    typedef WTraits<WT> TR;
    const hivis_config& g = c->cfg;
    const char* env = getenv("HIVIS_FUSED");
    if (env && env[0] == '0') { c->fused = false; return HIVIS_OK; }
    const size_t gemm_f = fused_gemm_lds_floats(FusedCfg<WT>::NW, FusedCfg<WT>::G, TR::RPL, FusedCfg<WT>::KBW);
    const size_t attn_f = std::max(fused_attn_lds_floats(g.head_dim, FUSED_NW, FUSED_RMAX), fused_attn_mfma_lds_floats(g.head_dim, FUSED_NW, FUSED_RMAX));
    c->fused_lds = std::max(gemm_f, attn_f) * sizeof(float);
    // the attribute is per kernel, not per context: contexts with different head sizes may be alive together, so it only grows
    static size_t lds_limit = 0;
    lds_limit = std::max(lds_limit, c->fused_lds);
    HIP_TRY(c, hipFuncSetAttribute((const void*)fused_pass_kernel<WT>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_limit));
    {
        const void* ks[] = {(const void*)phase_kernel<WT, PH_GEMM, FEPI_STORE, false>, (const void*)phase_kernel<WT, PH_GEMM, FEPI_ADD_TO, false>,
                            (const void*)phase_kernel<WT, PH_GEMM, FEPI_ADDVEC, false>, (const void*)phase_kernel<WT, PH_GEMM, FEPI_QKV, false>,
                            (const void*)phase_kernel<WT, PH_GEMM, FEPI_QKV_TAB, false>, (const void*)phase_kernel<WT, PH_GEMM, FEPI_QKV_TAB4, false>,
                            (const void*)phase_kernel<WT, PH_GEMM, FEPI_SILU, false>, (const void*)phase_kernel<WT, PH_GEMM, FEPI_LOGITS, false>,
                            (const void*)phase_kernel<WT, PH_GEMM, FEPI_STORE, true>, (const void*)phase_kernel<WT, PH_GEMM, FEPI_ADD_TO, true>,
                            (const void*)phase_kernel<WT, PH_GEMM, FEPI_ADDVEC, true>,
                            (const void*)phase_kernel<WT, PH_ATTN, 0, false>, (const void*)phase_kernel<WT, PH_ATTN_MERGE, 0, false>,
                            (const void*)phase_kernel<WT, PH_PREP, 0, false>, (const void*)phase_kernel<WT, PH_NORM_ROWS, 0, false>,
                            (const void*)phase_kernel<WT, PH_ARGMAX, 0, false>, (const void*)phase_kernel<WT, PH_SAMPLE, 0, false>};
        for (const void* k : ks) HIP_TRY(c, hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_limit));
    }
    { const char* pe = getenv("HIVIS_PERSISTENT"); c->persistent = pe && pe[0] == '1'; }
    { const char* we = getenv("HIVIS_WIDE_GEMM"); c->no_wide_gemm = we && we[0] == '0'; }
    { const char* we = getenv("HIVIS_WIDE_MIN"); if (we && atoi(we) >= 1) c->wide_min = atoi(we); }
    { const char* be = getenv("HIVIS_TALL_BIG"); if (be) c->tall_big = be[0] != '0'; }
    { const char* be = getenv("HIVIS_TALL_BIG_FILL"); if (be && atoi(be) >= 0 && atoi(be) <= 100) c->tall_big_fill = atoi(be); }
    { const char* ke = getenv("HIVIS_ATTN_SHARED_MIN"); if (ke && atoi(ke) >= 1) c->attn_shared_min = atoi(ke); }
    { const char* ke = getenv("HIVIS_KEYS_PER_SPLIT"); if (ke && atoi(ke) >= 16) c->keys_per_split = atoi(ke); }
    { const char* ee = getenv("HIVIS_ATTN_ELECT"); if (ee) c->attn_elect = ee[0] == '1'; }
    { const char* fe = getenv("HIVIS_ATTN_FLAGS"); if (fe) c->attn_flags = atoi(fe); }
    int nb = 0;
    HIP_TRY(c, hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, (const void*)fused_pass_kernel<WT>, FUSED_NT, c->fused_lds));
    if (nb < 1) return fail(c, HIVIS_EHIP, "persistent kernel does not fit on a compute unit");
    c->fused_grid = c->num_cu;
    int rc;
    if ((rc = dev_alloc(c, &c->bar, 2))) return rc;
    HIP_TRY(c, hipMemset(c->bar, 0, 2 * sizeof(unsigned)));
    if (const char* pe = getenv("HIVIS_PROF")) { c->prof_left = atoi(pe); if (c->prof_left > 0) { if ((rc = dev_alloc(c, &c->prof, (size_t)4096 * 19))) return rc; HIP_TRY(c, hipMemset(c->prof, 0, (size_t)4096 * 19 * 8)); } }
    c->fused = true;
    return HIVIS_OK;
}


// ---- whole-prompt prefill (bf16 models): tall MFMA GEMMs over all rows of a sequence --------------------------
int tall_gemm(hivis_ctx* c, const float* A, int lda, int M, int K, const uint4* Wp, int N, float* Y, int ldy) {
    const int kblks = K / 32, row_tiles = (M + 7) / 8, ntiles = N / 16;
    const size_t nfrag = (size_t)row_tiles * kblks * 64;
    // A == nullptr: the producing row kernel has already written the fragments to c->pf_frag
    if (A) hipLaunchKernelGGL(pack_afrag_kernel, dim3((unsigned)std::min<size_t>((nfrag + 255) / 256, 65535)), dim3(256), 0, c->stream, A, lda, M, kblks, c->pf_frag);
    // LDS-tiled kernel: 64 real rows x 256 columns per workgroup when that still gives >= 2 workgroups per CU, else x 128
    const int macro_rows = (row_tiles + 7) / 8;
    // grid: (column blocks rounded up to a multiple of the 8 XCDs) x row blocks, 1-D (see the kernel's mapping)
    // large tile (128 real rows x 256 columns, one workgroup per CU) where it fills the CUs in whole rounds well enough
    {
        const int big_rows = (row_tiles + 15) / 16, big_cols = (ntiles + 15) / 16;
        const long wgs = (long)big_rows * big_cols;
        const long rounds = (wgs + c->num_cu - 1) / c->num_cu;
        // rows padded to 128 must not waste more than rows padded to 64 would (832 rows: 7.7% against 0)
        const bool rows_ok = c->tall_big_fill == 0 || big_rows * 128 - M <= macro_rows * 64 - M + M / 32;
        if (c->tall_big && M >= 128 && rows_ok && wgs * 100 >= rounds * c->num_cu * c->tall_big_fill) {
            static bool attr = false;
            if (!attr) { HIP_TRY(c, hipFuncSetAttribute((const void*)gemm_tall_big_kernel<8>, hipFuncAttributeMaxDynamicSharedMemorySize, 3 * 32 * 1024)); attr = true; }
            // patches of RB x CB blocks, dealt to the 8 XCDs (the kernel's mapping)
            const int npr = (big_rows + 7) / 8, RB = (big_rows + npr - 1) / npr, CB = std::max(1, 32 / RB);
            const int npatch = ((big_rows + RB - 1) / RB) * ((big_cols + CB - 1) / CB);
            const int grid = ((npatch + 7) / 8) * 8 * RB * CB;
            hipLaunchKernelGGL((gemm_tall_big_kernel<8>), dim3(grid), dim3(256), 3 * 32 * 1024, c->stream,
                               (const v4u_t*)c->pf_frag, row_tiles, kblks, (const v4u_t*)Wp, ntiles, Y, ldy, M, (const v4u_t*)c->zero_blk);
            HIP_TRY(c, hipGetLastError());
            return HIVIS_OK;
        }
    }
    if ((size_t)macro_rows * ((ntiles + 15) / 16) >= (size_t)2 * c->num_cu) {
        const int ncol8 = (((ntiles + 15) / 16) + 7) & ~7;
        hipLaunchKernelGGL((gemm_tall_lds_kernel<8>), dim3(ncol8 * macro_rows), dim3(256), 2 * 24 * 1024, c->stream,
                           (const v4u_t*)c->pf_frag, row_tiles, kblks, (const v4u_t*)Wp, ntiles, Y, ldy, M, 1, (float*)nullptr);
    } else {
        const int ncol8 = (((ntiles + 7) / 8) + 7) & ~7;
        hipLaunchKernelGGL((gemm_tall_lds_kernel<4>), dim3(ncol8 * macro_rows), dim3(256), 2 * 16 * 1024, c->stream,
                           (const v4u_t*)c->pf_frag, row_tiles, kblks, (const v4u_t*)Wp, ntiles, Y, ldy, M, 1, (float*)nullptr);
    }
    HIP_TRY(c, hipGetLastError());
    return HIVIS_OK;
}

// 33..64 rows (tree verify) in ONE pass over the weights: the LDS-tiled MFMA kernel of the prefill with the K range cut
// into slices, so that a few hundred workgroups stream the weights (a workgroup owns 64 rows x 128 columns x one slice;
// the activation fragments it needs are re-read by the column blocks only, not by every workgroup as in the skinny kernel).
// A == nullptr: the fragments are already in c->pf_frag (written by the producing row kernel).  defer != nullptr: the
// slice partials are not reduced here; *defer describes them for the consuming row kernel.
int wide_gemm(hivis_ctx* c, const float* A, int lda, int M, int K, const uint4* Wp, int N, float* Y, int ldy, Parts* defer) {
    const int kblks = K / 32, row_tiles = (M + 7) / 8, ntiles = N / 16;
    const size_t nfrag = (size_t)row_tiles * kblks * 64;
    if (A) hipLaunchKernelGGL(pack_afrag_kernel, dim3((unsigned)std::min<size_t>((nfrag + 255) / 256, 65535)), dim3(256), 0, c->stream, A, lda, M, kblks, c->pf_frag);
    const int ncol = (ntiles + 7) / 8, ncol8 = (ncol + 7) & ~7;         // 8 column tiles per workgroup
    // about 3 workgroups per CU and at most 16 slices (swept at 61 rows: 256/384/512/768/1024 workgroups, 8/16 slices;
    // 256-column tiles with half the slices were no faster, at 61 rows and at 32)
    int S = std::max(1, std::min(16, 3 * c->num_cu / ncol));
    while (S > 1 && ((S - 1) * ((kblks + S - 1) / S) >= kblks || (kblks + S - 1) / S < 4)) --S;     // no empty slice, >= 4 K blocks each
    float* part = nullptr;
    if (S > 1) {
        const size_t need = (size_t)S * M * ldy;
        if (need > c->splitk_floats) {
            if (int rc = dev_alloc(c, &c->splitk_ws, need)) return rc;
            c->splitk_floats = need;
        }
        part = c->splitk_ws;
    }
    if (row_tiles <= 4)      // at most 32 rows: 4 row tiles per workgroup, half the fragment traffic and MFMA work
        hipLaunchKernelGGL((gemm_tall_lds_kernel<4, 4, 2>), dim3(ncol8 * S), dim3(256), 2 * 12 * 1024, c->stream,
                           (const v4u_t*)c->pf_frag, row_tiles, kblks, (const v4u_t*)Wp, ntiles, Y, ldy, M, S, part);
    else
        hipLaunchKernelGGL((gemm_tall_lds_kernel<4, 4>), dim3(ncol8 * S), dim3(256), 2 * 16 * 1024, c->stream,
                           (const v4u_t*)c->pf_frag, row_tiles, kblks, (const v4u_t*)Wp, ntiles, Y, ldy, M, S, part);
    if (defer) { defer->p = S > 1 ? part : Y; defer->n = S; defer->stride = (size_t)M * ldy; }
    else if (S > 1) hipLaunchKernelGGL(splitk_reduce_kernel, dim3(M, row_chunks(M)), dim3(256), 0, c->stream, (const float*)part, S, M, N, ldy, Y, ldy);
    HIP_TRY(c, hipGetLastError());
    return HIVIS_OK;
}

// One decoder layer on up to 64 rows (nseq sequences x m rows; bf16 models): the split-K GEMMs chained through row kernels
// that read the slice partials and write the next GEMM's fragments.  `pending` / `out_pending` as in layer_forward, as partials.
template <typename WT>
int layer_forward_wide(hivis_ctx* c, const LayerDev& L, const KVDev& kv, float* h, Parts pending, const int* base,
                       int offset, int seq0, int nseq, int m, TreeRows tr, Parts* out_pending) {
    typedef typename KVType<WT>::type KT;
    const hivis_config& g = c->cfg;
    const int M = nseq * m, d = g.d, qd = g.n_q_heads * g.head_dim, kd = g.n_kv_heads * g.head_dim, F = g.ffn;
    const int nqkv = qd + 2 * kd, Mp = ((M + 7) / 8) * 8;
    Parts pq{}, po{}, pg{};
    hipLaunchKernelGGL((wide_add_norm_frag_kernel<WT>), dim3(Mp), dim3(WNORM_NT), 0, c->stream, h, d, pending, d, M, (const WT*)L.norm1, c->pf_frag, d, g.rms_eps);
    if (int rc = wide_gemm(c, nullptr, 0, M, d, L.wqkv, nqkv, c->qkv, nqkv, &pq)) return rc;
    hipLaunchKernelGGL((wide_rope_append_kernel<KT>), dim3(M, 8), dim3(256), 0, c->stream, pq, c->qkv, nqkv, g.n_q_heads, g.n_kv_heads, g.head_dim, base, offset, seq0, m,
                       (KT*)kv.k, (KT*)kv.v, kv.maxL, g.rope_theta, tr.pos_delta, (const float*)L.bqkv, (const float*)c->rope_tab, g.max_vis + g.max_text);
    // (the attention writes the O projection's fragments itself where its kernel can; rows beyond M of the last row tile
    // then keep whatever the buffer held: an MFMA output row depends on its own A row only, and those rows are never stored)
    bool att_frag = false;
    if (int rc = attention_rows_mfma<WT>(c, c->qkv, nqkv, kv, base, offset, seq0, nseq, m, c->att, qd, tr.mask, c->pf_frag, &att_frag)) return rc;
    if (int rc = wide_gemm(c, att_frag ? nullptr : c->att, qd, M, qd, L.wo, d, c->proj, d, &po)) return rc;
    hipLaunchKernelGGL((wide_add_norm_frag_kernel<WT>), dim3(Mp), dim3(WNORM_NT), 0, c->stream, h, d, po, d, M, (const WT*)L.norm2, c->pf_frag, d, g.rms_eps);
    if (int rc = wide_gemm(c, nullptr, 0, M, d, L.wgu, 2 * F, c->gu, 2 * F, &pg)) return rc;
    hipLaunchKernelGGL(wide_silu_frag_kernel, dim3(Mp / 8, std::min(64, (F / 8 + 31) / 32)), dim3(256), 0, c->stream, pg, M, F, c->pf_frag);
    if (int rc = wide_gemm(c, nullptr, 0, M, F, L.wd, d, c->proj, d, out_pending)) return rc;
    HIP_TRY(c, hipGetLastError());
    return HIVIS_OK;
}

template <typename WT>
int prefill_target_tall(hivis_ctx* c, int b, int v, int l) {
    typedef typename KVType<WT>::type KT;
    const hivis_config& g = c->cfg;
    const int M = v + l, d = g.d, qd = g.n_q_heads * g.head_dim, kd = g.n_kv_heads * g.head_dim, F = g.ffn, nqkv = qd + 2 * kd;
    const int Mp = ((M + 7) / 8) * 8;
    hipLaunchKernelGGL((prefill_rows_kernel<WT>), dim3(M), dim3(256), 0, c->stream, (const WT*)c->vis + (size_t)b * g.max_vis * d, v,
                       (const WT*)c->embed, (const int32_t*)(c->text + (size_t)b * c->text_stride), 0, c->pf_x, d);
    const float* pending = nullptr;
    for (int l_ = 0; l_ < g.n_layers; ++l_) {
        const LayerDev& L = c->layers[l_];
        const KVDev& kv = c->tkv[l_];
        // residual add + RMSNorm write the GEMM's A fragments directly (rows padded to whole tiles), SiLU * up likewise
        const bool direct = d <= 8192 && d % 8 == 0 && F % 32 == 0;
        const Parts pend{pending, 1, 0};
        if (direct) hipLaunchKernelGGL((wide_add_norm_frag_kernel<WT>), dim3(Mp), dim3(WNORM_NT), 0, c->stream, c->pf_x, d, pend, d, M, (const WT*)L.norm1, c->pf_frag, d, g.rms_eps);
        else hipLaunchKernelGGL((add_rmsnorm_kernel<WT>), dim3(M), dim3(256), 0, c->stream, c->pf_x, d, pending, d, (const WT*)L.norm1, c->pf_a, d, d, g.rms_eps);
        if (int rc = tall_gemm(c, direct ? nullptr : c->pf_a, d, M, d, L.wqkv, nqkv, c->pf_qkv, nqkv)) return rc;
        hipLaunchKernelGGL((rope_append_kernel<KT>), dim3(M, row_chunks(M)), dim3(256), 0, c->stream, c->pf_qkv, g.n_q_heads, g.n_kv_heads, g.head_dim, (const int*)c->zeros, 0, b, M, (KT*)kv.k, (KT*)kv.v, kv.maxL, g.rope_theta, (const int*)nullptr, (const float*)L.bqkv, (const float*)c->rope_tab, g.max_vis + g.max_text);
        if (c->fused) { if (int rc = attention_rows_mfma<WT>(c, c->pf_qkv, nqkv, kv, c->zeros, 0, b, 1, M, c->pf_att, qd)) return rc; }
        else if (int rc = attention<WT>(c, c->pf_qkv, nqkv, kv, c->zeros, 0, b, 1, M, M, c->pf_att, qd)) return rc;
        if (int rc = tall_gemm(c, c->pf_att, qd, M, qd, L.wo, d, c->pf_proj, d)) return rc;
        const Parts proj{c->pf_proj, 1, 0};
        if (direct) hipLaunchKernelGGL((wide_add_norm_frag_kernel<WT>), dim3(Mp), dim3(WNORM_NT), 0, c->stream, c->pf_x, d, proj, d, M, (const WT*)L.norm2, c->pf_frag, d, g.rms_eps);
        else hipLaunchKernelGGL((add_rmsnorm_kernel<WT>), dim3(M), dim3(256), 0, c->stream, c->pf_x, d, (const float*)c->pf_proj, d, (const WT*)L.norm2, c->pf_a, d, d, g.rms_eps);
        if (int rc = tall_gemm(c, direct ? nullptr : c->pf_a, d, M, d, L.wgu, 2 * F, c->pf_gu, 2 * F)) return rc;
        if (direct) {
            const Parts gu{c->pf_gu, 1, 0};
            hipLaunchKernelGGL(wide_silu_frag_kernel, dim3(Mp / 8, std::min(64, (F / 8 + 31) / 32)), dim3(256), 0, c->stream, gu, M, F, c->pf_frag);
        } else hipLaunchKernelGGL(silu_mul_kernel, dim3(M, row_chunks(M)), dim3(256), 0, c->stream, (const float*)c->pf_gu, c->pf_act, F);
        if (int rc = tall_gemm(c, direct ? nullptr : c->pf_act, F, M, F, L.wd, d, c->pf_proj, d)) return rc;
        pending = c->pf_proj;
    }
    // features of the text rows: final norm of (x + last MLP delta)
    hipLaunchKernelGGL((add_rmsnorm_kernel<WT>), dim3(l), dim3(256), 0, c->stream, c->pf_x + (size_t)v * d, d, pending + (size_t)v * d, d,
                       (const WT*)c->final_norm, c->feat + (size_t)b * g.max_text * d, d, d, g.rms_eps);
    HIP_TRY(c, hipGetLastError());
    return HIVIS_OK;
}

struct PhaseTimer {
    hivis_ctx* c; int phase; bool on;
    PhaseTimer(hivis_ctx* c_, int p) : c(c_), phase(p), on(false) {
        if (!c->timing) return;
        while (c->pev_used + 2 > c->pev.size()) {
            hipEvent_t e = nullptr;
            if (hipEventCreate(&e) != hipSuccess) return;
            c->pev.push_back(e);
        }
        on = hipEventRecord(c->pev[c->pev_used], c->stream) == hipSuccess;
    }
    void stop() {
        if (!on) return;
        on = false;
        if (hipEventRecord(c->pev[c->pev_used + 1], c->stream) != hipSuccess) return;
        c->pev_phase.resize(c->pev.size() / 2);
        c->pev_phase[c->pev_used / 2] = phase;
        c->pev_used += 2;
    }
};
// after a stream synchronisation: fold the recorded pairs into the per-phase totals
static void resolve_phase_events(hivis_ctx* c) {
    for (size_t i = 0; i + 1 < c->pev_used; i += 2) {
        float ms = 0.f;
        const int ph = c->pev_phase[i / 2];
        if (hipEventElapsedTime(&ms, c->pev[i], c->pev[i + 1]) == hipSuccess) { c->phase_ms[ph] += ms; c->phase_calls[ph]++; }
    }
    c->pev_used = 0;
}

// ---- the four calls, typed -------------------------------------------------------------------
template <typename WT>
int do_prefill(hivis_ctx* c, const void* vis_embeds, int v, const int32_t* text_ids, int l, int32_t* first_token, bool sample) {
    const hivis_config& g = c->cfg;
    const int B = g.batch, d = g.d;
    PhaseTimer pt(c, 0);
    // stage inputs
    if (v > 0) {
        for (int b = 0; b < B; ++b)
            HIP_TRY(c, hipMemcpyAsync((char*)c->vis + (size_t)b * g.max_vis * d * sizeof(WT), (const char*)vis_embeds + (size_t)b * v * d * sizeof(WT),
                                      (size_t)v * d * sizeof(WT), hipMemcpyDefault, c->stream));
    }
    for (int b = 0; b < B; ++b)
        HIP_TRY(c, hipMemcpyAsync(c->text + (size_t)b * c->text_stride, c->h_ids.data() + (size_t)b * l, (size_t)l * sizeof(int32_t), hipMemcpyHostToDevice, c->stream));
    hipLaunchKernelGGL(set_ints_kernel, dim3(1), dim3(64), 0, c->stream, c->tlen, B, 0);
    hipLaunchKernelGGL(set_ints_kernel, dim3(1), dim3(64), 0, c->stream, c->dlen, B, 0);
    // a fresh start also clears the sticky error words: the bad-logits flag and, for the one-launch-per-pass path, the
    // barrier's arrival counter and abort flag (an aborted pass leaves the abort flag set)
    hipLaunchKernelGGL(set_ints_kernel, dim3(1), dim3(64), 0, c->stream, c->bad, 1, 0);
    if (c->bar) hipLaunchKernelGGL(set_ints_kernel, dim3(1), dim3(64), 0, c->stream, (int*)c->bar, 2, 0);

    const int total = v + l;
    for (int b = 0; b < B; ++b) {
        if (c->pf_rows >= total) {
            if (int rc = prefill_target_tall<WT>(c, b, v, l)) return rc;
            continue;
        }
        for (int p0 = 0; p0 < total; p0 += CHAIN_MAX_ROWS) {
            const int m = std::min(CHAIN_MAX_ROWS, total - p0);
            hipLaunchKernelGGL((prefill_rows_kernel<WT>), dim3(m), dim3(256), 0, c->stream, (const WT*)c->vis + (size_t)b * g.max_vis * d, v,
                               (const WT*)c->embed, (const int32_t*)(c->text + (size_t)b * c->text_stride), p0, c->x, d);
            const int first_out = std::max(0, v - p0);       // rows of this chunk before the first text row produce no feature
            float* out = c->feat + ((size_t)b * g.max_text + std::max(0, p0 - v)) * d;
            if (int rc = target_forward<WT>(c, b, 1, m, c->zeros, p0, p0 + m, out, d, std::min(first_out, m))) return rc;
        }
    }
    hipLaunchKernelGGL(set_ints_kernel, dim3(1), dim3(64), 0, c->stream, c->tlen, B, total);
    // first token x_{l+1}: LM head on the last text row of every sequence
    if (int rc = gemm<WT>(c, c->feat + (size_t)(l - 1) * d, g.max_text * d, B, d, c->lm_head, g.vocab, c->logits_p, g.vocab, EPI_STORE)) return rc;
    if (sample) hipLaunchKernelGGL(sample_rows_kernel, dim3(B), dim3(SAMPLE_NT), 0, c->stream, (const float*)c->logits_p, g.vocab, c->inv_temp, (const float*)c->u_res, 1, c->text + l, c->text_stride);
    else hipLaunchKernelGGL(argmax_kernel, dim3(B), dim3(256), 0, c->stream, (const float*)c->logits_p, g.vocab, c->text + l, c->text_stride, c->bad);
    // drafter prefill over the l text positions: rows [f^j ; Embed(x_{j+1})] + rho_0
    for (int b = 0; b < B; ++b) {
        for (int j0 = 0; j0 < l; j0 += CHAIN_MAX_ROWS) {
            const int m = std::min(CHAIN_MAX_ROWS, l - j0);
            hipLaunchKernelGGL((fuse_rows_kernel<WT>), dim3(m), dim3(256), 0, c->stream, (const float*)(c->feat + (size_t)b * g.max_text * d),
                               (const WT*)c->embed, (const int32_t*)(c->text + (size_t)b * c->text_stride), j0, c->catT, d);
            if (int rc = drafter_forward<WT>(c, c->catT, b, 1, m, 0, j0, j0 + m, c->dout, d)) return rc;
            if (j0 + m == l)   // f'_1: drafter output at the last true-feature row
                hipLaunchKernelGGL(copy_rows_kernel, dim3(1), dim3(256), 0, c->stream, (const float*)(c->dout + (size_t)(m - 1) * d), d, c->catD + (size_t)b * 2 * d, 2 * d, d);
        }
    }
    hipLaunchKernelGGL(set_ints_kernel, dim3(1), dim3(64), 0, c->stream, c->dlen, B, l);
    HIP_TRY(c, hipGetLastError());
    pt.stop();
    std::vector<int32_t> ft(B);
    for (int b = 0; b < B; ++b)
        HIP_TRY(c, hipMemcpyAsync(&ft[b], c->text + (size_t)b * c->text_stride + l, sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
    int bad = 0;
    HIP_TRY(c, hipMemcpyAsync(&bad, c->bad, sizeof(int), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    if (bad) return fail(c, HIVIS_EINVAL, "prefill produced logits without a finite maximum (NaN or Inf in vis_embeds or in the weights); prefill again with valid inputs");
    if (first_token) for (int b = 0; b < B; ++b) first_token[b] = ft[b];
    for (int b = 0; b < B; ++b) { c->h_tlen[b] = total; c->h_dlen[b] = l; }
    c->v = v;
    c->state = ST_READY;
    return HIVIS_OK;
}

template <typename WT>
int do_draft(hivis_ctx* c, int K, bool sample) {
    const hivis_config& g = c->cfg;
    const int B = g.batch, d = g.d, V = g.vocab;
    PhaseTimer pt(c, 1);
    if (c->fused && fused_rows_ok<WT>(B)) {
        if (int rc = run_program<WT>(c, sample ? PROG_DRAFT_SAMPLE : PROG_DRAFT, K, B, 1)) return rc;
        pt.stop();
        return HIVIS_OK;
    }
    int max_keys = 0;
    for (int b = 0; b < B; ++b) max_keys = std::max(max_keys, c->h_dlen[b]);
    for (int i = 1; i <= K; ++i) {
        float* lg = c->logits_d + (size_t)(i - 1) * B * V;
        if (int rc = gemm<WT>(c, c->catD, 2 * d, B, d, c->lm_head, V, lg, V, EPI_STORE)) return rc;
        if (sample) hipLaunchKernelGGL(sample_rows_kernel, dim3(B), dim3(SAMPLE_NT), 0, c->stream, (const float*)lg, V, c->inv_temp, (const float*)(c->u_draft + (i - 1)), g.k_max, c->drafts + (i - 1), g.k_max);
        else hipLaunchKernelGGL(argmax_kernel, dim3(B), dim3(256), 0, c->stream, (const float*)lg, V, c->drafts + (i - 1), g.k_max, c->bad);
        if (i < K) {
            hipLaunchKernelGGL((gather_rows_kernel<WT>), dim3(B), dim3(256), 0, c->stream, (const WT*)c->embed, (const int32_t*)(c->drafts + (i - 1)), g.k_max, c->catD + d, 2 * d, d);
            if (int rc = drafter_forward<WT>(c, c->catD, 0, B, 1, std::min(i, g.n_resid - 1), i - 1, max_keys + i, c->catD, 2 * d)) return rc;
        }
    }
    HIP_TRY(c, hipGetLastError());
    pt.stop();
    return HIVIS_OK;
}

template <typename WT>
int do_verify(hivis_ctx* c) {
    const hivis_config& g = c->cfg;
    const int B = g.batch, d = g.d, V = g.vocab, K = c->K, M = B * (K + 1);
    PhaseTimer pt(c, 2);
    int max_keys = 0;
    for (int b = 0; b < B; ++b) max_keys = std::max(max_keys, c->h_tlen[b]);
    hipLaunchKernelGGL(verify_tokens_kernel, dim3(1), dim3(64), 0, c->stream, (const int32_t*)c->text, c->text_stride, (const int*)c->dlen, (const int32_t*)c->drafts, g.k_max, K, c->row_tok, B);
    if (c->fused && fused_rows_ok<WT>(M)) {
        if (int rc = run_program<WT>(c, PROG_VERIFY, K, B, K + 1)) return rc;
        pt.stop();
        return HIVIS_OK;
    }
    hipLaunchKernelGGL((gather_rows_kernel<WT>), dim3(M), dim3(256), 0, c->stream, (const WT*)c->embed, (const int32_t*)c->row_tok, 1, c->x, d, d);
    if (int rc = target_forward<WT>(c, 0, B, K + 1, c->tlen, 0, max_keys + K + 1, c->catT, 2 * d, 0)) return rc;
    if (int rc = gemm<WT>(c, c->catT, 2 * d, M, d, c->lm_head, V, c->logits_v, V, EPI_STORE)) return rc;
    // target's greedy token after each row: ttok[b][i], row stride k_max+1
    for (int b = 0; b < B; ++b)
        hipLaunchKernelGGL(argmax_kernel, dim3(K + 1), dim3(256), 0, c->stream, (const float*)(c->logits_v + (size_t)b * (K + 1) * V), V, c->ttok + (size_t)b * (g.k_max + 1), 1, c->bad);
    HIP_TRY(c, hipGetLastError());
    pt.stop();
    return HIVIS_OK;
}

template <typename WT>
int do_accept(hivis_ctx* c, int32_t* n_accepted, int32_t* tokens, bool sample) {
    const hivis_config& g = c->cfg;
    const int B = g.batch, d = g.d, K = c->K, M = B * (K + 1);
    PhaseTimer pt(c, 3);
    if (sample)
        hipLaunchKernelGGL(accept_sample_kernel, dim3(B), dim3(ACCEPT_NT), 0, c->stream, (const int32_t*)c->drafts, (const float*)c->logits_v, (const float*)c->logits_d,
                           B, g.vocab, g.k_max, K, c->inv_temp, (const float*)c->u_acc, (const float*)c->u_res, c->text, c->text_stride,
                           (const int*)c->dlen, c->tlen, c->nacc, c->out_tok, c->next_tok);
    else
        hipLaunchKernelGGL(accept_kernel, dim3(B), dim3(64), 0, c->stream, (const int32_t*)c->drafts, (const int32_t*)c->ttok, g.k_max, K, c->text, c->text_stride,
                           (const int*)c->dlen, c->tlen, c->nacc, c->out_tok, c->next_tok);
    // roll-forward: K+1 rows per sequence [g_i ; Embed(token after row i)] + rho_0 through the drafter at positions
    // dlen..dlen+K; rows beyond n_b are computed but become dead (the drafter length advances by n_b+1 only).
    if (c->fused && fused_rows_ok<WT>(M)) {
        if (int rc = run_program<WT>(c, PROG_ROLL, K, B, K + 1)) return rc;
    } else {
        for (int b = 0; b < B; ++b)
            hipLaunchKernelGGL((gather_rows_kernel<WT>), dim3(K + 1), dim3(256), 0, c->stream, (const WT*)c->embed, (const int32_t*)(c->next_tok + (size_t)b * (g.k_max + 1)), 1,
                               c->catT + (size_t)b * (K + 1) * 2 * d + d, 2 * d, d);
        int max_keys = 0;
        for (int b = 0; b < B; ++b) max_keys = std::max(max_keys, c->h_dlen[b]);
        if (int rc = drafter_forward<WT>(c, c->catT, 0, B, K + 1, 0, 0, max_keys + K + 1, c->dout, d)) return rc;
    }
    hipLaunchKernelGGL(select_row_kernel, dim3(B), dim3(256), 0, c->stream, (const float*)c->dout, K + 1, (const int32_t*)c->nacc, c->catD, 2 * d, c->dlen, d);
    HIP_TRY(c, hipGetLastError());
    pt.stop();
    const size_t nres = (size_t)B + (size_t)B * (g.k_max + 1);
    HIP_TRY(c, hipMemcpyAsync(c->h_result, c->nacc, nres * sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
    c->h_result[nres] = 0;
    if (c->fused && c->persistent) HIP_TRY(c, hipMemcpyAsync(c->h_result + nres, c->bar + 1, sizeof(unsigned), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipMemcpyAsync(c->h_result + nres + 1, c->bad, sizeof(int), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    // Either flag means the device state (lengths, text) has already moved on from something invalid while the host
    // mirrors have not: the context is put back to "created", which only a new hivis_prefill leaves.
    if (c->h_result[nres]) { c->state = ST_CREATED; return fail(c, HIVIS_EHIP, "one-launch pass: grid barrier timed out (pass aborted); prefill again"); }
    if (c->h_result[nres + 1]) { c->state = ST_CREATED; return fail(c, HIVIS_EINVAL, "a pass produced logits without a finite maximum (NaN or Inf in the inputs or weights); prefill again"); }
    const int32_t* hn = c->h_result; const int32_t* ht = c->h_result + B;
    for (size_t i = 0; i + 1 < c->kev_used; i += 2) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, c->kev[i], c->kev[i + 1]) == hipSuccess) { c->kms += ms; c->klaunches++; }
    }
    c->kev_used = 0;
    resolve_phase_events(c);
    for (int b = 0; b < B; ++b) {
        c->h_tlen[b] += hn[b] + 1; c->h_dlen[b] += hn[b] + 1;
        if (n_accepted) n_accepted[b] = hn[b];
    }
    if (tokens) memcpy(tokens, ht, (size_t)B * (g.k_max + 1) * sizeof(int32_t));
    c->state = ST_READY;
    (void)M;
    return HIVIS_OK;
}


// ---- draft tree (batch 1) ---------------------------------------------------------------------------
// Device arrays of the tree, sized for the library's limits, allocated on the first tree call.
template <typename WT>
int tree_setup(hivis_ctx* c) {
    typedef typename KVType<WT>::type KT;
    if (c->tree_ready) return HIVIS_OK;
    const hivis_config& g = c->cfg;
    const int d = g.d, V = g.vocab, kd = g.n_kv_heads * g.head_dim;
    TreeDev& t = c->tree;
    int rc;
    const int P = TREE_MAX_POOL, R = TREE_MAX_ROWS, D = TREE_MAX_DEPTH;
    if ((rc = dev_alloc(c, &t.pool_tok, P)) || (rc = dev_alloc(c, &t.pool_par, P)) || (rc = dev_alloc(c, &t.pool_score, P)) ||
        (rc = dev_alloc(c, &t.pool_depth, P)) || (rc = dev_alloc(c, &t.pool_hid, P)) || (rc = dev_alloc(c, &t.pool_slot, P)) ||
        (rc = dev_alloc(c, &t.expand, R)) || (rc = dev_alloc(c, &t.dmask, R)) || (rc = dev_alloc(c, &t.dpos, R)) ||
        (rc = dev_alloc(c, &t.sel, R)) || (rc = dev_alloc(c, &t.row_par, R)) || (rc = dev_alloc(c, &t.row_depth, R)) ||
        (rc = dev_alloc(c, &t.vmask, R)) || (rc = dev_alloc(c, &t.ttok, R)) || (rc = dev_alloc(c, &t.path, D + 1)) ||
        (rc = dev_alloc(c, &t.next_tok, D + 1)) || (rc = dev_alloc(c, &t.result, D + 2)))
        return rc;
    t.row_tok = c->row_tok;
    if ((rc = dev_alloc(c, &c->tH, (size_t)(R + 1) * d))) return rc;
    if ((rc = dev_alloc(c, &c->tlogits, (size_t)(R + 1) * V))) return rc;
    if ((rc = dev_alloc(c, &c->tcat, (size_t)TREE_MAX_TOPK * 2 * d))) return rc;
    if ((rc = dev_alloc(c, &c->troll, (size_t)(D + 1) * 2 * d))) return rc;
    c->tnseg = (V + TOPK_SEG - 1) / TOPK_SEG;
    if ((rc = dev_alloc(c, &c->tcand_v, (size_t)TREE_MAX_TOPK * c->tnseg * TREE_MAX_TOPK))) return rc;
    if ((rc = dev_alloc(c, &c->tcand_i, (size_t)TREE_MAX_TOPK * c->tnseg * TREE_MAX_TOPK))) return rc;
    if ((rc = dev_alloc(c, &c->tseg, (size_t)TREE_MAX_TOPK * c->tnseg * 2))) return rc;
    // cache pointers of all target layers (keys, values) for the compaction kernels, and their staging rows
    std::vector<void*> ptrs;
    for (int l = 0; l < g.n_layers; ++l) { ptrs.push_back(c->tkv[l].k); ptrs.push_back(c->tkv[l].v); }
    if ((rc = dev_alloc(c, &c->kv_ptrs, ptrs.size()))) return rc;
    HIP_TRY(c, hipMemcpy(c->kv_ptrs, ptrs.data(), ptrs.size() * sizeof(void*), hipMemcpyHostToDevice));
    { KT* st; if ((rc = dev_alloc(c, &st, (size_t)g.n_layers * 2 * D * kd * KVWidth<KT>::W))) return rc; c->kv_staging = st; }
    HIP_TRY(c, hipHostMalloc((void**)&c->h_tree_result, (D + 3) * sizeof(int32_t), hipHostMallocDefault));     // result [D + 2] | bad-logits flag
    // pool and row arrays start at zero: a level whose logits have no finite maximum writes no entries, and what a later
    // kernel then reads as a token id must still be a valid one
    HIP_TRY(c, hipMemsetAsync(t.pool_tok, 0, P * sizeof(*t.pool_tok), c->stream)); HIP_TRY(c, hipMemsetAsync(t.pool_par, 0, P * sizeof(*t.pool_par), c->stream));
    HIP_TRY(c, hipMemsetAsync(t.pool_score, 0, P * sizeof(*t.pool_score), c->stream)); HIP_TRY(c, hipMemsetAsync(t.pool_depth, 0, P * sizeof(*t.pool_depth), c->stream));
    HIP_TRY(c, hipMemsetAsync(t.pool_hid, 0, P * sizeof(*t.pool_hid), c->stream)); HIP_TRY(c, hipMemsetAsync(t.pool_slot, 0, P * sizeof(*t.pool_slot), c->stream));
    HIP_TRY(c, hipMemsetAsync(t.expand, 0, R * sizeof(*t.expand), c->stream)); HIP_TRY(c, hipMemsetAsync(t.sel, 0, R * sizeof(*t.sel), c->stream));
    HIP_TRY(c, hipMemsetAsync(t.row_par, 0, R * sizeof(*t.row_par), c->stream)); HIP_TRY(c, hipMemsetAsync(t.row_depth, 0, R * sizeof(*t.row_depth), c->stream));
    HIP_TRY(c, hipMemsetAsync(t.ttok, 0, R * sizeof(*t.ttok), c->stream)); HIP_TRY(c, hipMemsetAsync(t.path, 0, (D + 1) * sizeof(*t.path), c->stream));
    HIP_TRY(c, hipMemsetAsync(t.next_tok, 0, (D + 1) * sizeof(*t.next_tok), c->stream)); HIP_TRY(c, hipMemsetAsync(t.result, 0, (D + 2) * sizeof(*t.result), c->stream));
    HIP_TRY(c, hipMemsetAsync(t.dmask, 0, R * sizeof(*t.dmask), c->stream)); HIP_TRY(c, hipMemsetAsync(t.dpos, 0, R * sizeof(*t.dpos), c->stream));
    HIP_TRY(c, hipMemsetAsync(t.vmask, 0, R * sizeof(*t.vmask), c->stream));
    c->tree_ready = true;
    return HIVIS_OK;
}

// Pool of k + (depth-1) k^2 nodes, level by level; then the N best-scored candidates and their verify rows.
template <typename WT>
int do_tree_draft(hivis_ctx* c, int k, int depth, int N) {
    const hivis_config& g = c->cfg;
    const int d = g.d, V = g.vocab;
    if (int rc = tree_setup<WT>(c)) return rc;
    PhaseTimer pt(c, 1);
    const TreeDev& t = c->tree;
    // hidden row 0 = the drafter's pending state f'_1; its distribution gives level 1
    hipLaunchKernelGGL(copy_rows_kernel, dim3(1), dim3(256), 0, c->stream, (const float*)c->catD, 2 * d, c->tH, d, d);
    if (int rc = gemm<WT>(c, c->tH, d, 1, d, c->lm_head, V, c->tlogits, V, EPI_STORE)) return rc;
    const int nseg = c->tnseg;
    const size_t child_lds = (size_t)nseg * k * 2 * sizeof(float);
    if (child_lds > 48 * 1024) return fail(c, HIVIS_EINVAL, "vocabulary too large for the top-k merge (%d segments x %d)", nseg, k);
    hipLaunchKernelGGL(tree_topk_part_kernel, dim3(1, nseg), dim3(TOPK_NT), 0, c->stream, (const float*)c->tlogits, V, k, c->tcand_v, c->tcand_i, c->tseg);
    hipLaunchKernelGGL(tree_children_kernel, dim3(1), dim3(CHILD_NT), child_lds, c->stream, (const float*)c->tcand_v, (const int32_t*)c->tcand_i, (const float*)c->tseg, nseg, k, 0,
                       (const int32_t*)nullptr, 1, 0, t);
    int lo = 0, n = k;
    for (int j = 1; j < depth; ++j) {
        const int n_prev = (j - 1) * k, row0 = 1 + n_prev;
        const int32_t* E = t.expand + n_prev;
        hipLaunchKernelGGL(tree_expand_kernel, dim3(1), dim3(256), 0, c->stream, lo, n, k, n_prev, j, t);
        hipLaunchKernelGGL((tree_cat_kernel<WT>), dim3(k), dim3(256), 0, c->stream, E, t, (const float*)c->tH, (const WT*)c->embed, c->tcat, d);
        TreeRows tr; tr.pos_delta = t.dpos + n_prev; tr.mask = t.dmask + n_prev;
        if (int rc = drafter_forward<WT>(c, c->tcat, 0, 1, k, std::min(j, g.n_resid - 1), n_prev, c->h_dlen[0] + n_prev + k,
                                         c->tH + (size_t)row0 * d, d, tr)) return rc;
        if (int rc = gemm<WT>(c, c->tH + (size_t)row0 * d, d, k, d, c->lm_head, V, c->tlogits + (size_t)row0 * V, V, EPI_STORE)) return rc;
        const int first = lo + n;
        hipLaunchKernelGGL(tree_topk_part_kernel, dim3(k, nseg), dim3(TOPK_NT), 0, c->stream, (const float*)(c->tlogits + (size_t)row0 * V), V, k, c->tcand_v, c->tcand_i, c->tseg);
        hipLaunchKernelGGL(tree_children_kernel, dim3(k), dim3(CHILD_NT), child_lds, c->stream, (const float*)c->tcand_v, (const int32_t*)c->tcand_i, (const float*)c->tseg, nseg, k, first,
                           E, j + 1, row0, t);
        lo = first; n = k * k;
    }
    hipLaunchKernelGGL(tree_select_kernel, dim3(1), dim3(1024), 0, c->stream, lo + n, N, (const int32_t*)c->text, (const int*)c->dlen, t);
    HIP_TRY(c, hipGetLastError());
    pt.stop();
    return HIVIS_OK;
}

template <typename WT>
int do_tree_verify(hivis_ctx* c) {
    const hivis_config& g = c->cfg;
    const int d = g.d, V = g.vocab, M = c->tn + 1;
    PhaseTimer pt(c, 2);
    const TreeDev& t = c->tree;
    hipLaunchKernelGGL((gather_rows_kernel<WT>), dim3(M), dim3(256), 0, c->stream, (const WT*)c->embed, (const int32_t*)t.row_tok, 1, c->x, d, d);
    TreeRows tr; tr.pos_delta = t.row_depth; tr.mask = t.vmask;
    if (int rc = target_forward<WT>(c, 0, 1, M, c->tlen, 0, c->h_tlen[0] + M, c->catT, 2 * d, 0, tr)) return rc;
    if (int rc = gemm<WT>(c, c->catT, 2 * d, M, d, c->lm_head, V, c->logits_v, V, EPI_STORE)) return rc;
    hipLaunchKernelGGL(argmax_kernel, dim3(M), dim3(256), 0, c->stream, (const float*)c->logits_v, V, t.ttok, 1, c->bad);
    HIP_TRY(c, hipGetLastError());
    pt.stop();
    c->vrows = M;
    return HIVIS_OK;
}

template <typename WT>
int do_tree_accept(hivis_ctx* c, int32_t* n_accepted, int32_t* tokens, bool sample) {
    typedef typename KVType<WT>::type KT;
    const hivis_config& g = c->cfg;
    const int d = g.d, N = c->tn, depth = c->tdepth;
    PhaseTimer pt(c, 3);
    const TreeDev& t = c->tree;
    // T > 0: the token the target DRAWS after every row replaces its greedy token (row of depth j: uniform u_tree[j]);
    // the walk below is the same: a candidate is followed when it is the token after its parent row
    if (sample) hipLaunchKernelGGL(sample_rows_kernel, dim3(N + 1), dim3(SAMPLE_NT), 0, c->stream, (const float*)c->logits_v, g.vocab, c->inv_temp,
                                   (const float*)c->u_tree, 1, t.ttok, 1, (const int32_t*)t.row_depth);
    hipLaunchKernelGGL(tree_accept_kernel, dim3(1), dim3(64), 0, c->stream, N, depth, c->text, (const int*)c->dlen, t);
    // target cache: the followed rows move to the slots right after the root's
    for (int scatter = 0; scatter < 2; ++scatter)
        hipLaunchKernelGGL((tree_kv_gather_kernel<KT>), dim3(depth, 2 * g.n_layers), dim3(256), 0, c->stream, (KT* const*)c->kv_ptrs, c->tkv[0].maxL,
                           g.n_kv_heads, g.head_dim * KVWidth<KT>::W, (const int*)c->tlen, (const int32_t*)t.result, (const int32_t*)t.path, depth, (KT*)c->kv_staging, scatter);
    // drafter: every tree row is dropped (its length never advanced); depth+1 rows rebuilt from the true features
    hipLaunchKernelGGL((tree_roll_cat_kernel<WT>), dim3(depth + 1), dim3(256), 0, c->stream, (const float*)c->catT, 2 * d, (const int32_t*)t.path,
                       (const int32_t*)t.next_tok, (const WT*)c->embed, c->troll, d);
    if (int rc = drafter_forward<WT>(c, c->troll, 0, 1, depth + 1, 0, 0, c->h_dlen[0] + depth + 1, c->dout, d)) return rc;
    hipLaunchKernelGGL(tree_finish_kernel, dim3(1), dim3(256), 0, c->stream, (const float*)c->dout, (const int32_t*)t.result, c->catD, c->dlen, c->tlen, d);
    HIP_TRY(c, hipGetLastError());
    pt.stop();
    HIP_TRY(c, hipMemcpyAsync(c->h_tree_result, t.result, (depth + 2) * sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipMemcpyAsync(c->h_tree_result + TREE_MAX_DEPTH + 2, c->bad, sizeof(int), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    resolve_phase_events(c);
    if (c->h_tree_result[TREE_MAX_DEPTH + 2]) { c->state = ST_CREATED; return fail(c, HIVIS_EINVAL, "a pass produced logits without a finite maximum (NaN or Inf in the inputs or weights); prefill again"); }
    const int n = c->h_tree_result[0];
    c->h_tlen[0] += n + 1; c->h_dlen[0] += n + 1;
    *n_accepted = n;
    memcpy(tokens, c->h_tree_result + 1, (size_t)(depth + 1) * sizeof(int32_t));
    c->state = ST_READY;
    return HIVIS_OK;
}

// The fusion FC is linear in its two halves: [f ; Embed(x)] [w1 ; w2] = f w1 + Embed(x) w2 (section 3.2), and the second
// term depends on the token alone.  For bf16 models the table T[x] = Embed(x) w2 ([V][d], fp32: bf16 x bf16 products summed
// in fp32) is computed here once, with the prefill's GEMM over ranges of embedding rows, and the phase programs' FC then
// streams w1 only (d x d instead of 2d x d per step) and adds T[x] in its epilogue.  HIVIS_EMB_TABLE=0 keeps the full FC.
template <typename WT>
int build_embed_fc_table(hivis_ctx* c, const hivis_weights* w) {
    if constexpr (sizeof(WT) != 2) return HIVIS_OK;
    const hivis_config& g = c->cfg;
    const int d = g.d, V = g.vocab;
    { const char* e = getenv("HIVIS_EMB_TABLE"); if (e && e[0] == '0') return HIVIS_OK; }
    if (!c->fused || c->persistent || !c->pf_frag || c->pf_rows < 8) return HIVIS_OK;
    void* staging = nullptr;
    HIP_TRY(c, hipMalloc(&staging, (size_t)d * d * sizeof(WT) + 4096));
    uint4* w2p = nullptr;
    int rc = HIVIS_OK;
    do {
        { const void* s[1] = {w->fuse_w}; int n[1] = {d};
          if ((rc = pack_matrix<WT>(c, s, n, 1, d, 0, staging, &c->fuse_w1))) break; }
        { const void* s[1] = {(const WT*)w->fuse_w + (size_t)d * d}; int n[1] = {d};
          if ((rc = pack_matrix<WT>(c, s, n, 1, d, 0, staging, &w2p))) break; }
        float* table = nullptr;
        {   // no room for the table is not an error: the FC then keeps multiplying the embedding half
            void* q = nullptr;
            if (hipMalloc(&q, (size_t)V * d * sizeof(float)) != hipSuccess) { (void)hipGetLastError(); break; }
            c->allocs.push_back(q);
            table = (float*)q;
        }
        const int R = c->pf_rows;                                  // rows per GEMM: what the prefill buffers hold
        for (int r0 = 0; r0 < V && !rc; r0 += R) {
            const int n = std::min(R, V - r0);
            hipLaunchKernelGGL((rows_to_f32_kernel<WT>), dim3(1024), dim3(256), 0, c->stream, (const WT*)c->embed + (size_t)r0 * d, (size_t)n * d, c->pf_x);
            rc = tall_gemm(c, c->pf_x, d, n, d, w2p, d, table + (size_t)r0 * d, d);
        }
        if (rc) break;
        if (hipStreamSynchronize(c->stream) != hipSuccess) { rc = fail(c, HIVIS_EHIP, "building the embedding table of the fusion FC failed"); break; }
        c->emb_w2 = table;
        // w1's tiles behind the LM head's, in one buffer: both have K = d, so a draft step's LM-head launch can compute
        // f' w1 as d more output columns and the fusion FC needs no launch of its own (HIVIS_LM_EXT=0: keep the FC phase)
        const char* le = getenv("HIVIS_LM_EXT");
        if (!(le && le[0] == '0')) {
            const size_t lm_bytes = (size_t)V * d * sizeof(WT), w1_bytes = (size_t)d * d * sizeof(WT);
            void* q = nullptr;
            if (hipMalloc(&q, lm_bytes + w1_bytes) != hipSuccess) { (void)hipGetLastError(); break; }
            if (hipMemcpyAsync(q, c->lm_head, lm_bytes, hipMemcpyDeviceToDevice, c->stream) != hipSuccess ||
                hipMemcpyAsync((char*)q + lm_bytes, c->fuse_w1, w1_bytes, hipMemcpyDeviceToDevice, c->stream) != hipSuccess ||
                hipStreamSynchronize(c->stream) != hipSuccess) { (void)hipFree(q); rc = fail(c, HIVIS_EHIP, "copying the LM head failed"); break; }
            // the separate LM-head buffer is no longer needed
            for (auto it = c->allocs.begin(); it != c->allocs.end(); ++it) if (*it == (void*)c->lm_head) { c->allocs.erase(it); break; }
            (void)hipFree(c->lm_head);
            c->allocs.push_back(q);
            c->lm_head = (uint4*)q;
            c->lm_ext = true;
        }
    } while (0);
    (void)hipFree(staging);
    return rc;
}

template <typename WT>
int do_create(hivis_ctx* c, const hivis_weights* w) {
    const hivis_config& g = c->cfg;
    const int d = g.d, qd = g.n_q_heads * g.head_dim, kd = g.n_kv_heads * g.head_dim, F = g.ffn, V = g.vocab, B = g.batch;
    // staging big enough for the largest source set of one packed matrix
    size_t stg = std::max({(size_t)d * (qd + 2 * kd), (size_t)qd * d, (size_t)2 * d * F, (size_t)F * d, (size_t)V * d, (size_t)2 * d * d}) * sizeof(WT) + 4096;
    void* staging = nullptr;
    HIP_TRY(c, hipMalloc(&staging, stg));
    int rc = HIVIS_OK;
    do {
        if ((rc = upload_vec<WT>(c, w->embed, (size_t)V * d, &c->embed))) break;
        if ((rc = upload_vec<WT>(c, w->final_norm, d, &c->final_norm))) break;
        if ((rc = upload_vec<WT>(c, w->resid_rho, (size_t)g.n_resid * d, &c->rho))) break;
        { const void* s[1] = {w->lm_head}; int n[1] = {V};
          if ((rc = pack_matrix<WT>(c, s, n, 1, d, 1, staging, &c->lm_head))) break; }
        { const void* s[1] = {w->fuse_w}; int n[1] = {d};
          if ((rc = pack_matrix<WT>(c, s, n, 1, 2 * d, 0, staging, &c->fuse_w))) break; }
        c->layers.resize(g.n_layers);
        for (int l = 0; l < g.n_layers && !rc; ++l) rc = upload_layer<WT>(c, w->layers[l], staging, c->layers[l]);
        if (rc) break;
        if ((rc = upload_layer<WT>(c, w->draft_layer, staging, c->draft))) break;
    } while (0);
    (void)hipFree(staging);
    if (rc) return rc;

    // KV caches (KW storage elements per cached value: hi and lo halves for bf16 models)
    constexpr int KW = KVWidth<typename KVType<WT>::type>::W;
    const int maxLt = g.max_vis + g.max_text, maxLd = g.max_text;
    c->tkv.resize(g.n_layers);
    for (int l = 0; l < g.n_layers; ++l) {
        typename KVType<WT>::type *k, *v;
        if ((rc = dev_alloc(c, &k, (size_t)B * kd * maxLt * KW))) return rc;
        if ((rc = dev_alloc(c, &v, (size_t)B * kd * maxLt * KW))) return rc;
        c->tkv[l].k = k; c->tkv[l].v = v; c->tkv[l].maxL = maxLt;
    }
    { typename KVType<WT>::type *k, *v;
      if ((rc = dev_alloc(c, &k, (size_t)B * kd * maxLd * KW))) return rc;
      if ((rc = dev_alloc(c, &v, (size_t)B * kd * maxLd * KW))) return rc;
      c->dkv.k = k; c->dkv.v = v; c->dkv.maxL = maxLd; }
    { WT* vis; if ((rc = dev_alloc(c, &vis, (size_t)B * std::max(1, g.max_vis) * d))) return rc; c->vis = vis; }

    // state + activations
    c->text_stride = g.max_text + g.k_max + 2;
    if ((rc = dev_alloc(c, &c->tlen, B))) return rc;
    if ((rc = dev_alloc(c, &c->dlen, B))) return rc;
    if ((rc = dev_alloc(c, &c->zeros, B))) return rc;
    if ((rc = dev_alloc(c, &c->zero_blk, 256))) return rc;
    HIP_TRY(c, hipMemset(c->zero_blk, 0, 256 * sizeof(float)));
    HIP_TRY(c, hipMemset(c->zeros, 0, B * sizeof(int)));
    if ((rc = dev_alloc(c, &c->text, (size_t)B * c->text_stride))) return rc;
    HIP_TRY(c, hipMemset(c->text, 0, (size_t)B * c->text_stride * sizeof(int32_t)));
    const int R = MAX_ROWS;
    if ((rc = dev_alloc(c, &c->x, (size_t)R * d))) return rc;
    if ((rc = dev_alloc(c, &c->a, (size_t)R * d))) return rc;
    if ((rc = dev_alloc(c, &c->qkv, (size_t)R * (qd + 2 * kd)))) return rc;
    if ((rc = dev_alloc(c, &c->att, (size_t)R * qd))) return rc;
    if ((rc = dev_alloc(c, &c->proj, (size_t)R * d))) return rc;
    if ((rc = dev_alloc(c, &c->gu, (size_t)R * 2 * F))) return rc;
    if ((rc = dev_alloc(c, &c->act, (size_t)R * F))) return rc;
    if ((rc = dev_alloc(c, &c->catT, (size_t)R * 2 * d))) return rc;
    if ((rc = dev_alloc(c, &c->catD, (size_t)B * 2 * d))) return rc;
    if ((rc = dev_alloc(c, &c->u, (size_t)R * d))) return rc;
    if ((rc = dev_alloc(c, &c->dout, (size_t)R * d))) return rc;
    if ((rc = dev_alloc(c, &c->feat, (size_t)B * g.max_text * d))) return rc;
    if (sizeof(WT) == 2) {
        const int PR = (g.max_vis + g.max_text + 7) & ~7;
        c->pf_rows = PR;
        const size_t kmax = std::max({(size_t)d, (size_t)qd, (size_t)F});
        if ((rc = dev_alloc(c, &c->pf_x, (size_t)PR * d))) return rc;
        if ((rc = dev_alloc(c, &c->pf_a, (size_t)PR * d))) return rc;
        if ((rc = dev_alloc(c, &c->pf_qkv, (size_t)PR * (qd + 2 * kd)))) return rc;
        if ((rc = dev_alloc(c, &c->pf_att, (size_t)PR * qd))) return rc;
        if ((rc = dev_alloc(c, &c->pf_proj, (size_t)PR * d))) return rc;
        if ((rc = dev_alloc(c, &c->pf_gu, (size_t)PR * 2 * F))) return rc;
        if ((rc = dev_alloc(c, &c->pf_act, (size_t)PR * F))) return rc;
        if ((rc = dev_alloc(c, &c->pf_frag, (size_t)PR * kmax / 4))) return rc;      // PR*kmax*4 bytes in 16-byte units
    }
    // attention workspace: (items * nsplit) work groups x 4 wave slots x RMAX rows x (hd + 2) floats, where
    // items * nsplit <= 2 * num_cu + items and items <= max(2, B) * n_q_heads
    {
        size_t max_items = (size_t)std::max({2, B, MAX_ROWS / ATT_RMAX}) * g.n_q_heads;
        if (c->pf_rows) max_items = std::max(max_items, (size_t)g.n_q_heads * ((c->pf_rows + ATT_RMAX - 1) / ATT_RMAX));
        c->attn_ws_floats = (2 * (size_t)c->num_cu + max_items) * 4 * ATT_RMAX * (g.head_dim + 2);
        if ((rc = dev_alloc(c, &c->attn_ws, c->attn_ws_floats))) return rc;
        c->rows_cnt_n = std::max(2, B) * g.n_q_heads;
        if ((rc = dev_alloc(c, &c->rows_cnt, (size_t)c->rows_cnt_n))) return rc;
        HIP_TRY(c, hipMemset(c->rows_cnt, 0, (size_t)c->rows_cnt_n * sizeof(int)));
    }
    if ((rc = dev_alloc(c, &c->logits_v, (size_t)R * V))) return rc;
    if ((rc = dev_alloc(c, &c->logits_d, (size_t)g.k_max * B * V))) return rc;
    if ((rc = dev_alloc(c, &c->logits_p, (size_t)B * V))) return rc;
    if ((rc = dev_alloc(c, &c->row_tok, R))) return rc;
    if ((rc = dev_alloc(c, &c->drafts, (size_t)B * g.k_max))) return rc;
    if ((rc = dev_alloc(c, &c->ttok, (size_t)B * (g.k_max + 1)))) return rc;
    if ((rc = dev_alloc(c, &c->u_draft, (size_t)B * g.k_max))) return rc;
    if ((rc = dev_alloc(c, &c->u_acc, (size_t)B * g.k_max))) return rc;
    if ((rc = dev_alloc(c, &c->u_res, (size_t)B))) return rc;
    if ((rc = dev_alloc(c, &c->u_tree, (size_t)TREE_MAX_DEPTH + 1))) return rc;
    // accepted counts and emitted tokens share one block, so one device-to-host copy into pinned memory returns both
    if ((rc = dev_alloc(c, &c->nacc, (size_t)B + (size_t)B * (g.k_max + 1)))) return rc;
    c->out_tok = c->nacc + B;
    HIP_TRY(c, hipHostMalloc((void**)&c->h_result, ((size_t)B + (size_t)B * (g.k_max + 1) + 2) * sizeof(int32_t), hipHostMallocDefault));
    if ((rc = dev_alloc(c, &c->bad, 1))) return rc;
    HIP_TRY(c, hipMemset(c->bad, 0, sizeof(int)));
    if ((rc = dev_alloc(c, &c->next_tok, (size_t)B * (g.k_max + 1)))) return rc;
    c->h_tlen.assign(B, 0); c->h_dlen.assign(B, 0);
    // rotary table over every position either cache can hold (read by the QKV epilogue of the phase programs)
    {
        const int npos = g.max_vis + g.max_text;
        if ((rc = dev_alloc(c, &c->rope_tab, (size_t)npos * g.head_dim))) return rc;
        const size_t n = (size_t)npos * (g.head_dim / 2);
        hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)std::min<size_t>((n + 255) / 256, 4096)), dim3(256), 0, c->stream, c->rope_tab, npos, g.head_dim, g.rope_theta);
        HIP_TRY(c, hipGetLastError());
    }
    if ((rc = fused_setup<WT>(c))) return rc;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    if ((rc = build_embed_fc_table<WT>(c, w))) return rc;
    return HIVIS_OK;
}

int check_config(const hivis_config* g, std::string& why) {
    char buf[256];
#define BAD(...) do { snprintf(buf, sizeof buf, __VA_ARGS__); why = buf; return HIVIS_EINVAL; } while (0)
    if (g->dtype != HIVIS_F32 && g->dtype != HIVIS_BF16) BAD("dtype %d unknown", g->dtype);
    const int al = g->dtype == HIVIS_BF16 ? 32 : 16;
    if (g->n_layers < 1 || g->d < al || g->n_q_heads < 1 || g->n_kv_heads < 1 || g->ffn < al || g->vocab < 16) BAD("non-positive dimension");
    if (g->head_dim != 64 && g->head_dim != 128) BAD("head_dim %d not in {64,128}", g->head_dim);
    if (g->n_q_heads % g->n_kv_heads) BAD("n_q_heads %% n_kv_heads != 0");
    if (g->d % al || (g->n_q_heads * g->head_dim) % al || (g->n_kv_heads * g->head_dim) % al || g->ffn % al) BAD("d, q_dim, kv_dim, ffn must be multiples of %d", al);
    if (g->vocab % 16) BAD("vocab must be a multiple of 16");
    if (g->batch < 1 || g->k_max < 1 || g->batch * (g->k_max + 1) > CHAIN_MAX_ROWS) BAD("batch*(k_max+1) must be in 2..%d", CHAIN_MAX_ROWS);
    if (g->max_vis < 0 || g->max_text < 2 + g->k_max) BAD("capacity too small");
    if (g->n_resid < 1) BAD("n_resid must be >= 1");
    if (!(g->rope_theta > 1.f) || !(g->rms_eps >= 0.f)) BAD("rope_theta / rms_eps out of range");
#undef BAD
    return HIVIS_OK;
}

thread_local std::string g_create_err;

}  // namespace

#define DISPATCH(c, fn, ...) ((c)->cfg.dtype == HIVIS_BF16 ? fn<bf16_t>(__VA_ARGS__) : fn<float>(__VA_ARGS__))

extern "C" {

int hivis_create(const hivis_config* cfg, const hivis_weights* w, void* hip_stream, hivis_ctx** out) {
    if (out) *out = nullptr;
    if (!cfg || !w || !out) { g_create_err = "null argument"; return HIVIS_EINVAL; }
    if (int rc = check_config(cfg, g_create_err)) return rc;
    if (!w->embed || !w->lm_head || !w->final_norm || !w->layers || !w->fuse_w || !w->resid_rho) { g_create_err = "null weight pointer"; return HIVIS_EINVAL; }
    hivis_ctx* c = new hivis_ctx();
    c->cfg = *cfg;
    c->stream = (hipStream_t)hip_stream;
    c->esize = cfg->dtype == HIVIS_BF16 ? 2 : 4;
    int dev = 0; hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
        g_create_err = "no HIP device"; delete c; return HIVIS_EHIP;
    }
    c->num_cu = prop.multiProcessorCount;
    c->na_phases.reserve(draft_phase_capacity(cfg->k_max));
    int rc = scratch_for_device(c, dev);
    if (!rc) rc = DISPATCH(c, do_create, c, w);
    if (rc) { g_create_err = c->err; hivis_destroy(c); return rc; }
    *out = c;
    return HIVIS_OK;
}

int hivis_destroy(hivis_ctx* c) {
    if (!c) return HIVIS_OK;
    (void)hipStreamSynchronize(c->stream);
    for (void* p : c->allocs) (void)hipFree(p);
    for (auto& kv : c->programs) delete kv.second.host;
    for (hipEvent_t e : c->pev) (void)hipEventDestroy(e);
    if (c->h_result) (void)hipHostFree(c->h_result);
    if (c->h_tree_result) (void)hipHostFree(c->h_tree_result);
    for (hipEvent_t e : c->kev) (void)hipEventDestroy(e);
    delete c;
    return HIVIS_OK;
}

int hivis_prefill(hivis_ctx* c, const void* vis_embeds, int32_t v, const int32_t* text_ids, int32_t l, int32_t* first_token) {
    if (!c) return HIVIS_EINVAL;
    const hivis_config& g = c->cfg;
    if (!text_ids || v < 0 || l < 1 || (v > 0 && !vis_embeds)) return fail(c, HIVIS_EINVAL, "bad prefill arguments (v=%d, l=%d)", v, l);
    if (v > g.max_vis || l + g.k_max + 2 > g.max_text) return fail(c, HIVIS_ECAP, "prompt exceeds capacity (v=%d/%d, l=%d/%d)", v, g.max_vis, l, g.max_text);
    c->h_ids.resize((size_t)g.batch * l);
    HIP_TRY(c, hipMemcpy(c->h_ids.data(), text_ids, c->h_ids.size() * sizeof(int32_t), hipMemcpyDefault));
    for (int32_t id : c->h_ids)
        if (id < 0 || id >= g.vocab) return fail(c, HIVIS_EINVAL, "token id %d outside [0,%d)", id, g.vocab);
    c->state = ST_CREATED;
    return DISPATCH(c, do_prefill, c, vis_embeds, v, text_ids, l, first_token, false);
}

static int check_uniforms(hivis_ctx* c, const float* u, size_t n, const char* what);

// Fills the uniform arrays of one sampling call on the device (up to two arrays share the call's number).
static int rng_fill(hivis_ctx* c, float* uA, int nA, int rowA, int strideA, unsigned purposeA, float* uB, int nB, unsigned purposeB) {
    if (!c->rng_seeded) return fail(c, HIVIS_ESTATE, "null uniform arrays need hivis_rng_seed first");
    const unsigned long long n = c->rng_calls++;
    const int total = nA + nB;
    hipLaunchKernelGGL(rng_fill_kernel, dim3((total + 255) / 256), dim3(256), 0, c->stream, uA, nA, std::max(rowA, 1), strideA, purposeA, uB, nB, purposeB,
                       (unsigned)(c->rng_seed & 0xFFFFFFFFull), (unsigned)(c->rng_seed >> 32), (unsigned)(n & 0xFFFFFFFFull), (unsigned)(n >> 32));
    HIP_TRY(c, hipGetLastError());
    return HIVIS_OK;
}

int hivis_rng_seed(hivis_ctx* c, uint64_t seed, uint64_t* calls_so_far) {
    if (!c) return HIVIS_EINVAL;
    if (calls_so_far) *calls_so_far = c->rng_calls;
    c->rng_seeded = true; c->rng_seed = seed; c->rng_calls = 0;
    return HIVIS_OK;
}

int hivis_prefill_sample(hivis_ctx* c, const void* vis_embeds, int32_t v, const int32_t* text_ids, int32_t l, float temperature,
                         const float* u_first, int32_t* first_token) {
    if (!c) return HIVIS_EINVAL;
    const hivis_config& g = c->cfg;
    if (!text_ids || v < 0 || l < 1 || (v > 0 && !vis_embeds)) return fail(c, HIVIS_EINVAL, "bad prefill arguments (v=%d, l=%d)", v, l);
    if (!(temperature > 0.0f)) return fail(c, HIVIS_EINVAL, "temperature must be positive");
    if (!u_first && !c->rng_seeded) return fail(c, HIVIS_ESTATE, "null u_first needs hivis_rng_seed first");
    if (u_first) { if (int rc = check_uniforms(c, u_first, (size_t)g.batch, "u_first")) return rc; }
    if (v > g.max_vis || l + g.k_max + 2 > g.max_text) return fail(c, HIVIS_ECAP, "prompt exceeds capacity (v=%d/%d, l=%d/%d)", v, g.max_vis, l, g.max_text);
    c->h_ids.resize((size_t)g.batch * l);
    HIP_TRY(c, hipMemcpy(c->h_ids.data(), text_ids, c->h_ids.size() * sizeof(int32_t), hipMemcpyDefault));
    for (int32_t id : c->h_ids)
        if (id < 0 || id >= g.vocab) return fail(c, HIVIS_EINVAL, "token id %d outside [0,%d)", id, g.vocab);
    if (u_first) { HIP_TRY(c, hipMemcpyAsync(c->u_res, u_first, (size_t)g.batch * sizeof(float), hipMemcpyHostToDevice, c->stream)); }
    else if (int rc = rng_fill(c, c->u_res, g.batch, 1, 1, 0u, nullptr, 0, 0u)) return rc;
    c->inv_temp = 1.0f / temperature;
    c->state = ST_CREATED;
    return DISPATCH(c, do_prefill, c, vis_embeds, v, text_ids, l, first_token, true);
}

static int check_room(hivis_ctx* c, int K) {
    const hivis_config& g = c->cfg;
    for (int b = 0; b < g.batch; ++b) {
        if (c->h_dlen[b] + K + 2 > g.max_text) return fail(c, HIVIS_ECAP, "sequence %d: text length %d + K + 2 exceeds max_text %d", b, c->h_dlen[b], g.max_text);
        if (c->h_tlen[b] + K + 1 > g.max_vis + g.max_text) return fail(c, HIVIS_ECAP, "sequence %d: target cache full", b);
    }
    return HIVIS_OK;
}

int hivis_draft(hivis_ctx* c, int32_t K) {
    if (!c) return HIVIS_EINVAL;
    if (c->state != ST_READY) return fail(c, HIVIS_ESTATE, "hivis_draft needs a prefilled/accepted context");
    if (K < 1 || K > c->cfg.k_max) return fail(c, HIVIS_EINVAL, "K=%d outside [1,%d]", K, c->cfg.k_max);
    if (int rc = check_room(c, K)) return rc;
    int rc = DISPATCH(c, do_draft, c, K, false);
    if (rc) return rc;
    c->K = K; c->state = ST_DRAFTED; c->drafts_sampled = false;
    return HIVIS_OK;
}

int hivis_draft_noalloc(hivis_ctx* c, int32_t K) {
    if (!c) return HIVIS_EINVAL;
    const hivis_config& g = c->cfg;
    if (c->state != ST_READY) return fail(c, HIVIS_ESTATE, "hivis_draft_noalloc needs a prefilled/accepted context");
    if (K < 1 || K > g.k_max) return fail(c, HIVIS_EINVAL, "K=%d outside [1,%d]", K, g.k_max);
    const int max_rows = g.dtype == HIVIS_BF16 ? WTraits<bf16_t>::ROWS : WTraits<float>::ROWS;
    if (!c->fused || g.batch > max_rows)
        return fail(c, HIVIS_EINVAL, "hivis_draft_noalloc needs the phase programs (HIVIS_FUSED not 0) and batch <= %d", max_rows);
    if (!c->scratch_dev) return fail(c, HIVIS_EHIP, "the static scratch array was not resolved at create");
    if (int rc = check_room(c, K)) return rc;
    int rc = DISPATCH(c, draft_noalloc, c, K);
    if (rc) return rc;
    c->K = K; c->state = ST_DRAFTED; c->drafts_sampled = false;
    return HIVIS_OK;
}

static int check_uniforms(hivis_ctx* c, const float* u, size_t n, const char* what) {
    if (!u) return fail(c, HIVIS_EINVAL, "null %s", what);
    for (size_t i = 0; i < n; ++i)
        if (!(u[i] >= 0.0f && u[i] < 1.0f)) return fail(c, HIVIS_EINVAL, "%s[%zu] = %g outside [0, 1)", what, i, (double)u[i]);
    return HIVIS_OK;
}

int hivis_draft_sample(hivis_ctx* c, int32_t K, float temperature, const float* u) {
    if (!c) return HIVIS_EINVAL;
    if (c->state != ST_READY) return fail(c, HIVIS_ESTATE, "hivis_draft_sample needs a prefilled/accepted context");
    if (K < 1 || K > c->cfg.k_max) return fail(c, HIVIS_EINVAL, "K=%d outside [1,%d]", K, c->cfg.k_max);
    if (!(temperature > 0.0f)) return fail(c, HIVIS_EINVAL, "temperature must be positive");
    const int B = c->cfg.batch;
    if (!u && !c->rng_seeded) return fail(c, HIVIS_ESTATE, "null u needs hivis_rng_seed first");
    if (u) { if (int rc = check_uniforms(c, u, (size_t)B * K, "u")) return rc; }
    if (int rc = check_room(c, K)) return rc;
    if (u) {
        for (int b = 0; b < B; ++b)
            HIP_TRY(c, hipMemcpyAsync(c->u_draft + (size_t)b * c->cfg.k_max, u + (size_t)b * K, K * sizeof(float), hipMemcpyHostToDevice, c->stream));
    } else if (int rc = rng_fill(c, c->u_draft, B * K, K, c->cfg.k_max, 1u, nullptr, 0, 0u)) return rc;
    c->inv_temp = 1.0f / temperature;
    int rc = DISPATCH(c, do_draft, c, K, true);
    if (rc) return rc;
    c->K = K; c->state = ST_DRAFTED; c->drafts_sampled = true;
    return HIVIS_OK;
}

int hivis_set_drafts(hivis_ctx* c, const int32_t* tokens, int32_t K) {
    if (!c) return HIVIS_EINVAL;
    if (c->state != ST_READY) return fail(c, HIVIS_ESTATE, "hivis_set_drafts needs a prefilled/accepted context");
    if (!tokens || K < 1 || K > c->cfg.k_max) return fail(c, HIVIS_EINVAL, "bad planted drafts (K=%d)", K);
    if (int rc = check_room(c, K)) return rc;
    for (int i = 0; i < c->cfg.batch * K; ++i)
        if (tokens[i] < 0 || tokens[i] >= c->cfg.vocab) return fail(c, HIVIS_EINVAL, "planted token %d outside vocab", tokens[i]);
    for (int b = 0; b < c->cfg.batch; ++b)
        HIP_TRY(c, hipMemcpyAsync(c->drafts + (size_t)b * c->cfg.k_max, tokens + (size_t)b * K, K * sizeof(int32_t), hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    c->K = K; c->state = ST_DRAFTED; c->drafts_sampled = false;
    return HIVIS_OK;
}

int hivis_verify(hivis_ctx* c) {
    if (!c) return HIVIS_EINVAL;
    if (c->state != ST_DRAFTED) return fail(c, HIVIS_ESTATE, "hivis_verify needs drafts");
    int rc = DISPATCH(c, do_verify, c);
    if (rc) return rc;
    c->state = ST_VERIFIED; c->vrows = c->cfg.batch * (c->K + 1);
    return HIVIS_OK;
}

int hivis_accept(hivis_ctx* c, int32_t* n_accepted, int32_t* tokens) {
    if (!c) return HIVIS_EINVAL;
    if (c->state != ST_VERIFIED) return fail(c, HIVIS_ESTATE, "hivis_accept needs a verified context");
    if (!n_accepted || !tokens) return fail(c, HIVIS_EINVAL, "null output pointer");
    return DISPATCH(c, do_accept, c, n_accepted, tokens, false);
}

int hivis_accept_sample(hivis_ctx* c, float temperature, const float* u_accept, const float* u_resample, int32_t* n_accepted, int32_t* tokens) {
    if (!c) return HIVIS_EINVAL;
    if (c->state != ST_VERIFIED) return fail(c, HIVIS_ESTATE, "hivis_accept_sample needs a verified context");
    if (!c->drafts_sampled) return fail(c, HIVIS_ESTATE, "hivis_accept_sample needs drafts drawn by hivis_draft_sample (their distributions)");
    if (!n_accepted || !tokens) return fail(c, HIVIS_EINVAL, "null output pointer");
    if (!(temperature > 0.0f)) return fail(c, HIVIS_EINVAL, "temperature must be positive");
    const int B = c->cfg.batch, K = c->K;
    if ((u_accept == nullptr) != (u_resample == nullptr)) return fail(c, HIVIS_EINVAL, "u_accept and u_resample must both be given or both be null");
    if (u_accept) {
        if (int rc = check_uniforms(c, u_accept, (size_t)B * K, "u_accept")) return rc;
        if (int rc = check_uniforms(c, u_resample, (size_t)B, "u_resample")) return rc;
        HIP_TRY(c, hipMemcpyAsync(c->u_acc, u_accept, (size_t)B * K * sizeof(float), hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, hipMemcpyAsync(c->u_res, u_resample, (size_t)B * sizeof(float), hipMemcpyHostToDevice, c->stream));
    } else if (int rc = rng_fill(c, c->u_acc, B * K, K, K, 2u, c->u_res, B, 3u)) return rc;
    c->inv_temp = 1.0f / temperature;
    return DISPATCH(c, do_accept, c, n_accepted, tokens, true);
}

int hivis_tree_draft(hivis_ctx* c, int32_t top_k, int32_t depth, int32_t n_nodes) {
    if (!c) return HIVIS_EINVAL;
    const hivis_config& g = c->cfg;
    if (g.batch != 1) return fail(c, HIVIS_EINVAL, "tree drafting needs batch 1 (got %d)", g.batch);
    if (c->state != ST_READY) return fail(c, HIVIS_ESTATE, "hivis_tree_draft needs a prefilled/accepted context");
    if (top_k < 1 || top_k > TREE_MAX_TOPK || depth < 1 || depth > TREE_MAX_DEPTH) return fail(c, HIVIS_EINVAL, "top_k=%d outside [1,%d] or depth=%d outside [1,%d]", top_k, TREE_MAX_TOPK, depth, TREE_MAX_DEPTH);
    const int P = top_k + (depth - 1) * top_k * top_k;
    if (P > TREE_MAX_POOL || (depth - 1) * top_k > TREE_MAX_ROWS) return fail(c, HIVIS_EINVAL, "tree too large: pool %d > %d or expanded rows %d > %d", P, TREE_MAX_POOL, (depth - 1) * top_k, TREE_MAX_ROWS);
    if (n_nodes < 1 || n_nodes > P || n_nodes + 1 > TREE_MAX_ROWS) return fail(c, HIVIS_EINVAL, "n_nodes=%d outside [1, min(pool %d, %d)]", n_nodes, P, TREE_MAX_ROWS - 1);
    if (c->h_dlen[0] + std::max((depth - 1) * top_k, depth + 1) + 2 > g.max_text) return fail(c, HIVIS_ECAP, "text length %d + tree rows exceeds max_text %d", c->h_dlen[0], g.max_text);
    if (c->h_tlen[0] + n_nodes + 1 > g.max_vis + g.max_text) return fail(c, HIVIS_ECAP, "target cache full");
    int rc = DISPATCH(c, do_tree_draft, c, top_k, depth, n_nodes);
    if (rc) return rc;
    c->tk = top_k; c->tdepth = depth; c->tn = n_nodes; c->state = ST_TREE_DRAFTED;
    return HIVIS_OK;
}

int hivis_tree_set(hivis_ctx* c, int32_t n_nodes, const int32_t* tokens, const int32_t* parents) {
    if (!c) return HIVIS_EINVAL;
    const hivis_config& g = c->cfg;
    if (g.batch != 1) return fail(c, HIVIS_EINVAL, "tree drafting needs batch 1 (got %d)", g.batch);
    if (c->state != ST_READY) return fail(c, HIVIS_ESTATE, "hivis_tree_set needs a prefilled/accepted context");
    if (!tokens || !parents || n_nodes < 1 || n_nodes + 1 > TREE_MAX_ROWS) return fail(c, HIVIS_EINVAL, "bad planted tree (n_nodes=%d)", n_nodes);
    // verify rows 1..n_nodes: parents are row indices (0 = root) and precede their children
    std::vector<int32_t> tok(n_nodes + 1, 0), par(n_nodes + 1, -1), dep(n_nodes + 1, 0);
    std::vector<unsigned long long> mask(n_nodes + 1, 1ull);
    int depth = 1;
    for (int i = 1; i <= n_nodes; ++i) {
        const int p = parents[i - 1], t = tokens[i - 1];
        if (p < 0 || p >= i) return fail(c, HIVIS_EINVAL, "planted row %d: parent %d outside [0,%d)", i, p, i);
        if (t < 0 || t >= g.vocab) return fail(c, HIVIS_EINVAL, "planted token %d outside vocab", t);
        tok[i] = t; par[i] = p; dep[i] = dep[p] + 1; mask[i] = mask[p] | (1ull << i);
        depth = std::max(depth, dep[i]);
    }
    if (depth > TREE_MAX_DEPTH) return fail(c, HIVIS_EINVAL, "planted tree depth %d > %d", depth, TREE_MAX_DEPTH);
    if (c->h_dlen[0] + depth + 3 > g.max_text) return fail(c, HIVIS_ECAP, "text length %d + tree rows exceeds max_text %d", c->h_dlen[0], g.max_text);
    if (c->h_tlen[0] + n_nodes + 1 > g.max_vis + g.max_text) return fail(c, HIVIS_ECAP, "target cache full");
    if (int rc = DISPATCH(c, tree_setup, c)) return rc;
    const TreeDev& t = c->tree;
    // row 0's token: the last known text token (device to device)
    HIP_TRY(c, hipMemcpyAsync(t.row_tok + 1, tok.data() + 1, n_nodes * sizeof(int32_t), hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipMemcpyAsync(t.row_tok, c->text + c->h_dlen[0], sizeof(int32_t), hipMemcpyDeviceToDevice, c->stream));
    HIP_TRY(c, hipMemcpyAsync(t.row_par, par.data(), (n_nodes + 1) * sizeof(int32_t), hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipMemcpyAsync(t.row_depth, dep.data(), (n_nodes + 1) * sizeof(int32_t), hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipMemcpyAsync(t.vmask, mask.data(), (n_nodes + 1) * sizeof(unsigned long long), hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    c->tk = 0; c->tdepth = depth; c->tn = n_nodes; c->state = ST_TREE_DRAFTED;
    return HIVIS_OK;
}

int hivis_tree_verify(hivis_ctx* c) {
    if (!c) return HIVIS_EINVAL;
    if (c->state != ST_TREE_DRAFTED) return fail(c, HIVIS_ESTATE, "hivis_tree_verify needs a drafted tree");
    int rc = DISPATCH(c, do_tree_verify, c);
    if (rc) return rc;
    c->state = ST_TREE_VERIFIED;
    return HIVIS_OK;
}

int hivis_tree_accept(hivis_ctx* c, int32_t* n_accepted, int32_t* tokens) {
    if (!c) return HIVIS_EINVAL;
    if (c->state != ST_TREE_VERIFIED) return fail(c, HIVIS_ESTATE, "hivis_tree_accept needs a verified tree");
    if (!n_accepted || !tokens) return fail(c, HIVIS_EINVAL, "null output pointer");
    return DISPATCH(c, do_tree_accept, c, n_accepted, tokens, false);
}

int hivis_tree_accept_sample(hivis_ctx* c, float temperature, const float* u, int32_t* n_accepted, int32_t* tokens) {
    if (!c) return HIVIS_EINVAL;
    if (c->state != ST_TREE_VERIFIED) return fail(c, HIVIS_ESTATE, "hivis_tree_accept_sample needs a verified tree");
    if (!n_accepted || !tokens) return fail(c, HIVIS_EINVAL, "null output pointer");
    if (!(temperature > 0.0f)) return fail(c, HIVIS_EINVAL, "temperature must be positive");
    const int n = c->tdepth + 1;
    if (u) {
        if (int rc = check_uniforms(c, u, (size_t)n, "u")) return rc;
        HIP_TRY(c, hipMemcpyAsync(c->u_tree, u, (size_t)n * sizeof(float), hipMemcpyHostToDevice, c->stream));
    } else if (int rc = rng_fill(c, c->u_tree, n, 1, 1, 4u, nullptr, 0, 0u)) return rc;
    c->inv_temp = 1.0f / temperature;
    return DISPATCH(c, do_tree_accept, c, n_accepted, tokens, true);
}

int hivis_tree_get(hivis_ctx* c, int32_t* pool_tokens, int32_t* pool_parents, float* pool_scores, int32_t* expand, int32_t* selected,
                   int32_t* row_tokens, int32_t* row_parents, int32_t* row_depths, int32_t* target_tokens) {
    if (!c) return HIVIS_EINVAL;
    if (!c->tree_ready || c->tn < 1) return fail(c, HIVIS_ESTATE, "no tree drafted yet");
    const TreeDev& t = c->tree;
    const int k = c->tk, P = k + (c->tdepth - 1) * k * k, N = c->tn;
    if (k == 0 && (pool_tokens || pool_parents || pool_scores || expand || selected)) return fail(c, HIVIS_ESTATE, "the last tree was planted: it has no pool");
#define GET(dst, src, n) do { if (dst) HIP_TRY(c, hipMemcpyAsync(dst, src, (size_t)(n) * 4, hipMemcpyDeviceToHost, c->stream)); } while (0)
    GET(pool_tokens, t.pool_tok, P); GET(pool_parents, t.pool_par, P); GET(pool_scores, t.pool_score, P);
    GET(expand, t.expand, (c->tdepth - 1) * k); GET(selected, t.sel, N);
    GET(row_tokens, t.row_tok, N + 1); GET(row_parents, t.row_par, N + 1); GET(row_depths, t.row_depth, N + 1);
    if (target_tokens) {
        if (c->state != ST_TREE_VERIFIED && c->state != ST_READY) return fail(c, HIVIS_ESTATE, "tree not verified yet");
        GET(target_tokens, t.ttok, N + 1);
    }
#undef GET
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return HIVIS_OK;
}

int hivis_tree_get_logits(hivis_ctx* c, float* out) {
    if (!c || !out) return HIVIS_EINVAL;
    if (!c->tree_ready || c->tn < 1 || c->tk < 1) return fail(c, HIVIS_ESTATE, "no tree drafted yet");
    const size_t rows = 1 + (size_t)(c->tdepth - 1) * c->tk;
    HIP_TRY(c, hipMemcpyAsync(out, c->tlogits, rows * c->cfg.vocab * sizeof(float), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return HIVIS_OK;
}

int hivis_get_logits(hivis_ctx* c, int32_t which, float* out) {
    if (!c || !out) return HIVIS_EINVAL;
    const hivis_config& g = c->cfg;
    const float* src; size_t n;
    if (which == 0) { if ((c->state != ST_VERIFIED && c->state != ST_TREE_VERIFIED && c->state != ST_READY) || c->vrows < 1) return fail(c, HIVIS_ESTATE, "no verify logits"); src = c->logits_v; n = (size_t)c->vrows * g.vocab; }
    else if (which == 1) { src = c->logits_d; n = (size_t)c->K * g.batch * g.vocab; }
    else if (which == 2) { src = c->logits_p; n = (size_t)g.batch * g.vocab; }
    else return fail(c, HIVIS_EINVAL, "which=%d", which);
    if (c->state == ST_CREATED) return fail(c, HIVIS_ESTATE, "nothing computed yet");
    HIP_TRY(c, hipMemcpyAsync(out, src, n * sizeof(float), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return HIVIS_OK;
}

int hivis_get_hidden(hivis_ctx* c, int32_t which, float* out) {
    if (!c || !out) return HIVIS_EINVAL;
    const hivis_config& g = c->cfg;
    if (c->state == ST_CREATED) return fail(c, HIVIS_ESTATE, "nothing computed yet");
    const int d = g.d;
    if (which == 0) {
        if (c->vrows < 1) return fail(c, HIVIS_ESTATE, "no verify pass yet");
        HIP_TRY(c, hipMemcpy2DAsync(out, d * sizeof(float), c->catT, 2 * d * sizeof(float), d * sizeof(float), (size_t)c->vrows, hipMemcpyDeviceToHost, c->stream));
    } else if (which == 1) {
        HIP_TRY(c, hipMemcpy2DAsync(out, d * sizeof(float), c->catD, 2 * d * sizeof(float), d * sizeof(float), (size_t)g.batch, hipMemcpyDeviceToHost, c->stream));
    } else return fail(c, HIVIS_EINVAL, "which=%d", which);
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return HIVIS_OK;
}

int hivis_kv_lengths(hivis_ctx* c, int32_t* target_len, int32_t* drafter_len) {
    if (!c) return HIVIS_EINVAL;
    const int B = c->cfg.batch;
    if (target_len) HIP_TRY(c, hipMemcpyAsync(target_len, c->tlen, B * sizeof(int), hipMemcpyDeviceToHost, c->stream));
    if (drafter_len) HIP_TRY(c, hipMemcpyAsync(drafter_len, c->dlen, B * sizeof(int), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return HIVIS_OK;
}

int hivis_get_tokens(hivis_ctx* c, int32_t* drafts, int32_t* target_tokens) {
    if (!c) return HIVIS_EINVAL;
    const hivis_config& g = c->cfg;
    if (c->state == ST_CREATED || c->K < 1) return fail(c, HIVIS_ESTATE, "no draft round yet");
    if (c->state == ST_TREE_DRAFTED || c->state == ST_TREE_VERIFIED) return fail(c, HIVIS_ESTATE, "a tree round is in progress: use hivis_tree_get");
    std::vector<int32_t> hd((size_t)g.batch * g.k_max), ht((size_t)g.batch * (g.k_max + 1));
    HIP_TRY(c, hipMemcpyAsync(hd.data(), c->drafts, hd.size() * sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipMemcpyAsync(ht.data(), c->ttok, ht.size() * sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    for (int b = 0; b < g.batch; ++b) {
        if (drafts) for (int i = 0; i < c->K; ++i) drafts[b * c->K + i] = hd[(size_t)b * g.k_max + i];
        if (target_tokens) for (int i = 0; i <= c->K; ++i) target_tokens[b * (c->K + 1) + i] = ht[(size_t)b * (g.k_max + 1) + i];
    }
    return HIVIS_OK;
}

int hivis_timing(hivis_ctx* c, int32_t enable) {
    if (!c) return HIVIS_EINVAL;
    c->timing = enable != 0;
    return HIVIS_OK;
}

int hivis_kernel_timing(hivis_ctx* c, int32_t gemm_kind) {
    if (!c || gemm_kind < -1 || gemm_kind > 5) return HIVIS_EINVAL;
    c->ktime_epi = gemm_kind; c->kms = 0; c->klaunches = 0; c->kev_used = 0; c->ktime_seen = 0;
    return HIVIS_OK;
}

int hivis_kernel_ms(hivis_ctx* c, double* total_ms, int64_t* launches, double* bytes_per_launch) {
    if (!c) return HIVIS_EINVAL;
    if (total_ms) *total_ms = c->kms;
    if (launches) *launches = c->klaunches;
    if (bytes_per_launch) *bytes_per_launch = c->kbytes;
    c->kms = 0; c->klaunches = 0;
    return HIVIS_OK;
}

int hivis_phase_ms(hivis_ctx* c, int32_t phase, double* total_ms, int64_t* calls) {
    if (!c || phase < 0 || phase > 3) return HIVIS_EINVAL;
    if (c->pev_used) { HIP_TRY(c, hipStreamSynchronize(c->stream)); resolve_phase_events(c); }
    if (total_ms) *total_ms = c->phase_ms[phase];
    if (calls) *calls = c->phase_calls[phase];
    c->phase_ms[phase] = 0; c->phase_calls[phase] = 0;
    return HIVIS_OK;
}

int hivis_algorithmic_bytes(hivis_ctx* c, double* verify_bytes, double* draft_step_bytes) {
    if (!c) return HIVIS_EINVAL;
    const hivis_config& g = c->cfg;
    const double b = c->esize, d = g.d, qd = (double)g.n_q_heads * g.head_dim, kd = (double)g.n_kv_heads * g.head_dim, F = g.ffn, V = g.vocab;
    const double w_layer = (2 * d * qd + 2 * d * kd + 3 * d * F) * b;
    double kv_t = 0, kv_d = 0;
    for (int s = 0; s < g.batch; ++s) { kv_t += 2.0 * c->h_tlen[s] * kd * b * g.n_layers; kv_d += 2.0 * c->h_dlen[s] * kd * b; }
    if (verify_bytes) *verify_bytes = g.n_layers * w_layer + V * d * b + kv_t;
    // (the method's bytes: the fusion FC as [2d x d] weights, also where the library reads only w1 and a table row per sequence)
    if (draft_step_bytes) *draft_step_bytes = w_layer + 2 * d * d * b + V * d * b + kv_d;
    return HIVIS_OK;
}

int32_t hivis_clamp_token(int32_t id, int32_t vocab) { return clamp_token(id, vocab); }

int hivis_calib_stream(void* hip_stream, int64_t buffer_bytes, int32_t n_buffers, int32_t passes, int32_t workgroups, double* gb_per_s,
                       double* us_per_launch) {
    if (buffer_bytes < (1 << 20) || n_buffers < 1 || n_buffers > 64 || passes < 1 || workgroups < 1 || workgroups > 65535) return HIVIS_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    const size_t n16 = (size_t)buffer_bytes / 16;
    const size_t trips = n16 / 4096;
    if (trips == 0) return HIVIS_EINVAL;
    std::vector<void*> bufs;
    unsigned* sink = nullptr;
    std::vector<hipEvent_t> ev;
    int rc = HIVIS_OK;
    auto cleanup = [&]() {
        for (void* b : bufs) (void)hipFree(b);
        if (sink) (void)hipFree(sink);
        for (hipEvent_t e : ev) (void)hipEventDestroy(e);
    };
#define CAL_TRY(expr) do { if ((expr) != hipSuccess) { cleanup(); return HIVIS_EHIP; } } while (0)
    CAL_TRY(hipMalloc((void**)&sink, sizeof(unsigned)));
    for (int i = 0; i < n_buffers; ++i) {
        void* b = nullptr;
        CAL_TRY(hipMalloc(&b, n16 * 16));
        bufs.push_back(b);
        CAL_TRY(hipMemsetAsync(b, 0x5A, n16 * 16, st));
    }
    // Timed like the dominant GEMM in hivis_kernel_timing: start / stop events attached to the dispatch itself read the
    // kernel's own begin and end (events recorded around a batch of short launches measure the host's launch rate
    // instead: 12 us per launch for a 6.8 us kernel).  At most 256 launches carry events (every k-th beyond that).
    const int total = passes * n_buffers;
    const int stride = (total + 255) / 256;
    const int timed = (total + stride - 1) / stride;
    ev.resize((size_t)2 * timed, nullptr);
    for (hipEvent_t& e : ev) CAL_TRY(hipEventCreate(&e));
    // one untimed round over all buffers, then `passes` timed rounds; the buffers rotate so that nothing read comes from a cache
    for (int i = 0; i < n_buffers; ++i) hipLaunchKernelGGL(calib_stream_kernel, dim3(workgroups), dim3(512), 0, st, (const uint4*)bufs[i], n16, sink);
    for (int l = 0, t = 0; l < total; ++l) {
        hipEvent_t a = nullptr, b = nullptr;
        if (l % stride == 0) { a = ev[2 * t]; b = ev[2 * t + 1]; ++t; }
        hipExtLaunchKernelGGL(calib_stream_kernel, dim3(workgroups), dim3(512), 0, st, a, b, 0, (const uint4*)bufs[l % n_buffers], n16, sink);
    }
    CAL_TRY(hipStreamSynchronize(st));
    CAL_TRY(hipGetLastError());
    double ms_sum = 0.0;
    for (int t = 0; t < timed; ++t) {
        float ms = 0.f;
        CAL_TRY(hipEventElapsedTime(&ms, ev[2 * t], ev[2 * t + 1]));
        ms_sum += ms;
    }
#undef CAL_TRY
    const double bytes = (double)trips * 4096 * 16.0;                 // what one launch reads
    const double us = ms_sum * 1e3 / timed;                           // average duration of one launch
    if (gb_per_s) *gb_per_s = bytes / (us * 1e-6) / 1e9;
    if (us_per_launch) *us_per_launch = us;
    cleanup();
    return rc;
}

const char* hivis_last_error(hivis_ctx* c) { return c ? c->err.c_str() : g_create_err.c_str(); }
const char* hivis_version(void) { return "hivis-gfx950 0.1"; }

}  // extern "C"

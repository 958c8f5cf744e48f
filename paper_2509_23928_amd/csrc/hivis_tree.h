// Draft-tree kernels (section 4 inference setting: top-k tree expanded to a fixed depth, the best-scored candidates
// verified in one pass; section 2.1 names the tree structure).  Batch 1.
//
// Pool layout (P = k + (depth-1) k^2 nodes): level 1 = the k most probable tokens after the drafter's pending hidden
// state; level j+1 = k children of each of the k rows expanded at level j, row by row, rank by rank.  A node's score
// is the sum of the log-probabilities along its path.  Everything that decides an index (top-k, expansion set,
// candidate set, acceptance walk) orders by (score descending, index ascending), so results are unique.
#pragma once
#include "hivis_kernels.h"

namespace hivis {

constexpr int TREE_MAX_TOPK = 16;       // k
constexpr int TREE_MAX_ROWS = 64;       // verify rows (root + candidates); drafter tree rows (depth-1)*k: one 64-bit mask each
constexpr int TREE_MAX_DEPTH = 16;
constexpr int TREE_MAX_POOL = 2048;

struct TreeDev {
    int32_t* pool_tok; int32_t* pool_par; float* pool_score; int32_t* pool_depth;   // [P]
    int32_t* pool_hid;                  // [P] hidden row whose distribution the node was taken from
    int32_t* pool_slot;                 // [P] drafter tree row of an expanded node
    int32_t* expand;                    // [depth-1][k] pool indices of the expanded rows
    unsigned long long* dmask;          // [(depth-1) k] ancestor masks of the drafter's tree rows (bit = tree row)
    int32_t* dpos;                      // [(depth-1) k] rotary position of a drafter tree row, relative to the cache length
    int32_t* sel;                       // [N] candidates, ascending pool index
    int32_t* row_tok; int32_t* row_par; int32_t* row_depth;   // [N+1] verify rows (row 0 = root)
    unsigned long long* vmask;          // [N+1] ancestor masks of the verify rows
    int32_t* ttok;                      // [N+1] the target's greedy token after each row
    int32_t* path;                      // [depth+1] rows re-fed after acceptance: root, followed rows, then the last one repeated
    int32_t* next_tok;                  // [depth+1] token that follows each re-fed row
    int32_t* result;                    // [1 + depth+1] accepted length | emitted tokens (-1 padded)
};

// (value, index) maximum over the workgroup under the order (value descending, index ascending); every thread gets it.
template <int NT>
__device__ __forceinline__ void block_best(float& v, int& i, float* smf, int* smi) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(v, o, 64); const int oi = __shfl_xor(i, o, 64);
        if (ov > v || (ov == v && oi < i)) { v = ov; i = oi; }
    }
    __syncthreads();
    if ((threadIdx.x & 63) == 0) { smf[threadIdx.x >> 6] = v; smi[threadIdx.x >> 6] = i; }
    __syncthreads();
    v = smf[0]; i = smi[0];
#pragma unroll
    for (int w = 1; w < NT / 64; ++w) {
        const float ov = smf[w]; const int oi = smi[w];
        if (ov > v || (ov == v && oi < i)) { v = ov; i = oi; }
    }
}

// Children of the rows of one level, in two kernels.  Row r of `logits` is the drafter's distribution behind node
// expand_row[r] (or behind the root if expand_row is null); its k most probable tokens (best first) become pool nodes
// first + r k + q with score = parent score + log softmax.
//  1. tree_topk_part_kernel, grid (rows, segments): a workgroup holds one segment of <= 4096 logits in registers
//     (8 per thread, loaded once), writes the segment's (max, sum of exp) and its k best (value, index) pairs; round q
//     picks the best element not yet taken under the order (value descending, index ascending).
//  2. tree_children_kernel, one workgroup per row: log-normaliser from the segment partials (fixed order), the k best
//     of the segments' candidates by rank counting, pool entries written.
constexpr int TOPK_NT = 512, TOPK_PER = 8, TOPK_SEG = TOPK_NT * TOPK_PER;
__global__ __launch_bounds__(TOPK_NT) void tree_topk_part_kernel(const float* __restrict__ logits, int V, int k,
                                                                 float* __restrict__ cand_v, int32_t* __restrict__ cand_i,
                                                                 float* __restrict__ seg_ms) {
    __shared__ float smf[TOPK_NT / 64];
    __shared__ int smi[TOPK_NT / 64];
    const int r = blockIdx.x, seg = blockIdx.y, nseg = gridDim.y;
    const float* x = logits + (size_t)r * V;
    const int j0 = seg * TOPK_SEG;
    float v[TOPK_PER];
#pragma unroll
    for (int e = 0; e < TOPK_PER; ++e) {
        const int j = j0 + e * TOPK_NT + threadIdx.x;
        v[e] = j < V ? x[j] : -INFINITY;
    }
    float m = v[0];
#pragma unroll
    for (int e = 1; e < TOPK_PER; ++e) m = fmaxf(m, v[e]);
    m = block_reduce_max<TOPK_NT>(m, smf);                  // the segment is never empty (the host sizes the grid)
    float sum = 0.f;
#pragma unroll
    for (int e = 0; e < TOPK_PER; ++e) sum += expf(v[e] - m);       // exp(-inf) = 0 for the padding
    sum = wave_sum(sum);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) smf[threadIdx.x >> 6] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        float total = 0.f;
        for (int w = 0; w < TOPK_NT / 64; ++w) total += smf[w];
        seg_ms[((size_t)r * nseg + seg) * 2] = m; seg_ms[((size_t)r * nseg + seg) * 2 + 1] = total;
    }
    for (int q = 0; q < k; ++q) {
        float bv = -INFINITY; int bi = 0x7FFFFFFF;
#pragma unroll
        for (int e = 0; e < TOPK_PER; ++e) {
            const int j = j0 + e * TOPK_NT + threadIdx.x;
            if (j < V && (v[e] > bv || (v[e] == bv && j < bi))) { bv = v[e]; bi = j; }
        }
        block_best<TOPK_NT>(bv, bi, smf, smi);
#pragma unroll
        for (int e = 0; e < TOPK_PER; ++e) if (j0 + e * TOPK_NT + (int)threadIdx.x == bi) v[e] = -INFINITY;   // taken (logits are finite)
        if (threadIdx.x == 0) {
            const size_t o = ((size_t)r * nseg + seg) * k + q;
            cand_v[o] = bv; cand_i[o] = bi;                    // a segment shorter than k pads with (-inf, INT_MAX)
        }
    }
}

constexpr int CHILD_NT = 256;
__global__ __launch_bounds__(CHILD_NT) void tree_children_kernel(const float* __restrict__ cand_v, const int32_t* __restrict__ cand_i,
                                                                 const float* __restrict__ seg_ms, int nseg, int k, int first,
                                                                 const int32_t* __restrict__ expand_row, int depth, int hid_row0,
                                                                 TreeDev t) {
    extern __shared__ float child_lds[];                     // [nseg * k] values, [nseg * k] indices
    const int r = blockIdx.x, n = nseg * k;
    float* cv = child_lds; int* ci = reinterpret_cast<int*>(child_lds + n);
    for (int i = threadIdx.x; i < n; i += CHILD_NT) { cv[i] = cand_v[(size_t)r * n + i]; ci[i] = cand_i[(size_t)r * n + i]; }
    __syncthreads();
    // log-normaliser: every thread adds the segments in the same order
    float mx = -INFINITY;
    for (int s = 0; s < nseg; ++s) mx = fmaxf(mx, seg_ms[((size_t)r * nseg + s) * 2]);
    float sum = 0.f;
    for (int s = 0; s < nseg; ++s) sum += seg_ms[((size_t)r * nseg + s) * 2 + 1] * expf(seg_ms[((size_t)r * nseg + s) * 2] - mx);
    const float logz = mx + logf(sum);
    const int parent = expand_row ? expand_row[r] : -1;
    const float pscore = parent >= 0 ? t.pool_score[parent] : 0.f;
    for (int i = threadIdx.x; i < n; i += CHILD_NT) {
        const float vi = cv[i]; const int ii = ci[i];
        int rank = 0;
        for (int j = 0; j < n; ++j) rank += (cv[j] > vi || (cv[j] == vi && ci[j] < ii)) ? 1 : 0;
        if (rank < k && ii != 0x7FFFFFFF) {
            const int node = first + r * k + rank;
            t.pool_tok[node] = ii; t.pool_par[node] = parent; t.pool_depth[node] = depth; t.pool_hid[node] = hid_row0 + r;
            t.pool_score[node] = pscore + (vi - logz);
            t.pool_slot[node] = -1;
        }
    }
}

// The k best-scored of the n nodes [lo, lo + n) of one level become the drafter's tree rows n_prev .. n_prev + k - 1
// (rank order).  One workgroup, n <= 256.
__global__ __launch_bounds__(256) void tree_expand_kernel(int lo, int n, int k, int n_prev, int level, TreeDev t) {
    __shared__ float s[256];
    const int i = threadIdx.x;
    s[i] = i < n ? t.pool_score[lo + i] : -INFINITY;
    __syncthreads();
    if (i >= n) return;
    const float si = s[i];
    int rank = 0;
    for (int j = 0; j < n; ++j) rank += (s[j] > si || (s[j] == si && j < i)) ? 1 : 0;
    if (rank >= k) return;
    const int slot = n_prev + rank, node = lo + i;
    t.expand[(level - 1) * k + rank] = node;
    t.pool_slot[node] = slot;
    const int parent = t.pool_par[node];      // expanded at the level before (or the root): its row and mask already exist
    t.dmask[slot] = (parent >= 0 ? t.dmask[t.pool_slot[parent]] : 0ull) | (1ull << slot);
    t.dpos[slot] = level - 1;
}

// Fusion input rows of one level: [hidden row the node was drawn from ; Embed(node token)].
template <typename WT>
__global__ void tree_cat_kernel(const int32_t* __restrict__ expand_row, TreeDev t, const float* __restrict__ H,
                                const WT* __restrict__ table, float* __restrict__ cat, int d) {
    const int r = blockIdx.x, node = expand_row[r];
    const float* h = H + (size_t)t.pool_hid[node] * d;
    const WT* e = table + (size_t)t.pool_tok[node] * d;
    float* o = cat + (size_t)r * 2 * d;
    for (int c = threadIdx.x; c < d; c += blockDim.x) { o[c] = h[c]; o[d + c] = to_f32(e[c]); }
}

// Candidates: the N best-scored pool nodes, in pool order; verify rows 1..N (row 0 = root = the last known token).
// One workgroup of 1024 threads, P <= 2048.
__global__ __launch_bounds__(1024) void tree_select_kernel(int P, int N, const int32_t* __restrict__ text,
                                                           const int* __restrict__ dlen, TreeDev t) {
    __shared__ float s[TREE_MAX_POOL];
    __shared__ short rowof[TREE_MAX_POOL];      // verify row of a pool node, 0 if not a candidate
    for (int i = threadIdx.x; i < P; i += 1024) s[i] = t.pool_score[i];
    __syncthreads();
    bool chosen[2] = {false, false};
    for (int e = 0; e < 2; ++e) {
        const int i = threadIdx.x + e * 1024;
        if (i >= P) continue;
        const float si = s[i];
        int rank = 0;
        for (int j = 0; j < P; ++j) rank += (s[j] > si || (s[j] == si && j < i)) ? 1 : 0;
        chosen[e] = rank < N;
    }
    for (int e = 0; e < 2; ++e) { const int i = threadIdx.x + e * 1024; if (i < P) rowof[i] = chosen[e] ? 1 : 0; }
    __syncthreads();
    int myrow[2] = {0, 0};
    for (int e = 0; e < 2; ++e) {
        const int i = threadIdx.x + e * 1024;
        if (i >= P || !chosen[e]) continue;
        int below = 0;
        for (int j = 0; j < i; ++j) below += rowof[j] ? 1 : 0;
        myrow[e] = below + 1;
    }
    __syncthreads();
    for (int e = 0; e < 2; ++e) { const int i = threadIdx.x + e * 1024; if (i < P) rowof[i] = (short)myrow[e]; }
    __syncthreads();
    for (int e = 0; e < 2; ++e) {
        const int i = threadIdx.x + e * 1024;
        if (i >= P || !chosen[e]) continue;
        const int row = myrow[e];
        if (row > N) continue;                                    // only with NaN scores (ranks are then not a permutation)
        t.sel[row - 1] = i;
        t.row_tok[row] = t.pool_tok[i];
        t.row_depth[row] = t.pool_depth[i];
        const int parent = t.pool_par[i];
        t.row_par[row] = parent >= 0 ? rowof[parent] : 0;        // the candidate set is closed under ancestors
        unsigned long long m = 1ull;                              // the root
        for (int a = i; a >= 0; a = t.pool_par[a]) m |= 1ull << rowof[a];
        t.vmask[row] = m;
    }
    if (threadIdx.x == 0) { t.row_tok[0] = text[dlen[0]]; t.row_par[0] = -1; t.row_depth[0] = 0; t.vmask[0] = 1ull; }
}

// Greedy acceptance on the tree: from the root, follow the child whose token is the target's greedy token at the
// current row until there is none.  Emits the followed tokens plus the target's token at the last row, appends them
// to the text, and lists the rows whose true features re-condition the drafter.  One wavefront.
__global__ __launch_bounds__(64) void tree_accept_kernel(int N, int depth, int32_t* __restrict__ text, const int* __restrict__ dlen, TreeDev t) {
    const int lane = threadIdx.x;
    int cur = 0, n = 0;
    int mine = 0;                                   // lane e ends up holding re-fed row e (lane 0: the root)
    while (n < depth) {
        const int want = t.ttok[cur];
        int found = 0x7FFFFFFF;
        for (int c = 1 + lane; c <= N; c += 64)
            if (t.row_par[c] == cur && t.row_tok[c] == want) found = min(found, c);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) found = min(found, __shfl_xor(found, o, 64));
        if (found == 0x7FFFFFFF) break;
        cur = found; ++n;
        if (lane == n) mine = cur;
    }
    if (lane > n) mine = cur;                       // dead rows repeat the last followed row
    const int bonus = t.ttok[cur];
    const int next_row = __shfl(mine, min(lane + 1, 63), 64);
    if (lane <= depth) {
        const int tok = (lane < n) ? t.row_tok[next_row] : bonus;          // token that follows re-fed row `lane`
        t.path[lane] = mine;
        t.next_tok[lane] = tok;
        t.result[1 + lane] = (lane <= n) ? tok : -1;
        if (lane <= n) text[dlen[0] + 1 + lane] = tok;
    }
    if (lane == 0) t.result[0] = n;
}

// Cache compaction after acceptance, for all layers at once: the rows of the followed path move from their tree
// slots base + path[j] to base + j (j = 1..n).  Two kernels (gather into a staging buffer, scatter back) because a
// destination slot of one row can be the source slot of another.
// kv: [n_layers][2] cache pointers; cache layout [Hkv][maxL][HD]; staging [n_layers][2][depth][Hkv*HD], where HD here is
// the STORAGE width of a cached row (head_dim * KVWidth: hi and lo halves of a half-precision cache move together).
template <typename KT>
__global__ void tree_kv_gather_kernel(KT* const* __restrict__ kv, int maxL, int Hkv, int HD, const int* __restrict__ tlen,
                                      const int32_t* __restrict__ result, const int32_t* __restrict__ path, int depth,
                                      KT* __restrict__ staging, int scatter) {
    const int j = blockIdx.x + 1, lk = blockIdx.y;                  // lk = layer * 2 + (0: keys, 1: values)
    const int n = result[0];
    if (j > n) return;
    const int src = path[j];
    if (src == j) return;                                           // already in place
    KT* cache = kv[lk];
    KT* st = staging + ((size_t)lk * depth + (j - 1)) * Hkv * HD;
    const int base = tlen[0];
    for (int idx = threadIdx.x; idx < Hkv * HD; idx += blockDim.x) {
        const int h = idx / HD, c = idx % HD;
        if (scatter) cache[((size_t)h * maxL + base + j) * HD + c] = st[idx];
        else st[idx] = cache[((size_t)h * maxL + base + src) * HD + c];
    }
}

// Re-feed rows after acceptance: [true feature of path row e ; Embed(token after it)], e = 0..depth (rows beyond the
// accepted length repeat the last one and are dead).  g: verify features, row stride ldg.
template <typename WT>
__global__ void tree_roll_cat_kernel(const float* __restrict__ g, int ldg, const int32_t* __restrict__ path,
                                     const int32_t* __restrict__ next_tok, const WT* __restrict__ table,
                                     float* __restrict__ cat, int d) {
    const int e = blockIdx.x;
    const float* f = g + (size_t)path[e] * ldg;
    const WT* em = table + (size_t)next_tok[e] * d;
    float* o = cat + (size_t)e * 2 * d;
    for (int c = threadIdx.x; c < d; c += blockDim.x) { o[c] = f[c]; o[d + c] = to_f32(em[c]); }
}

// After the re-feed: pending hidden state = drafter output at row n; both caches keep n + 1 more rows.
__global__ void tree_finish_kernel(const float* __restrict__ dout, const int32_t* __restrict__ result, float* __restrict__ fnext,
                                   int* __restrict__ dlen, int* __restrict__ tlen, int d) {
    const int n = result[0];
    for (int c = threadIdx.x; c < d; c += blockDim.x) fnext[c] = dout[(size_t)n * d + c];
    if (threadIdx.x == 0) { dlen[0] += n + 1; tlen[0] += n + 1; }
}

// ------------------------------------------------------------------------------------------
// Row-wise kernels of the 33..64-row passes (bf16 models).  They read a GEMM result as the sum of its K-slice partials
// (value = sum over s < nparts of p[s * pstride + index], fixed order) and, where the consumer is the next split-K GEMM,
// write its A operand directly as MFMA fragments (bf16 hi/lo split, layout of pack_afrag_kernel:
// frag[(row tile * kblks + kb) * 64 + lane], lane = 16 g + i holds k = 32 kb + 8 g .. +8 of row 8 tt + 2 (i >> 2) + (i & 1),
// i & 2 selecting the low part), so neither the reduction nor the fragment packing is a launch of its own.
// ------------------------------------------------------------------------------------------
struct Parts { const float* p; int n; size_t stride; };

// B slices per trip, their loads issued together (a one-load-per-trip loop costs a memory round trip per slice)
template <int B>
__device__ __forceinline__ void parts_add(float4& a, const Parts& ps, size_t idx, int s0) {
    for (int s = s0; s < ps.n; s += B) {
        float4 v[B];
#pragma unroll
        for (int j = 0; j < B; ++j) v[j] = *reinterpret_cast<const float4*>(ps.p + (size_t)min(s + j, ps.n - 1) * ps.stride + idx);
#pragma unroll
        for (int j = 0; j < B; ++j)
            if (s + j < ps.n) { a.x += v[j].x; a.y += v[j].y; a.z += v[j].z; a.w += v[j].w; }
    }
}
__device__ __forceinline__ float4 parts_load4(const Parts& ps, size_t idx) {
    float4 a = *reinterpret_cast<const float4*>(ps.p + idx);
    if (ps.n <= 4) parts_add<3>(a, ps, idx, 1);       // slices 1..3 in one trip
    else parts_add<8>(a, ps, idx, 1);
    return a;
}

// h[row] += delta (sum of partials, optional); fragments of h[row] * gain / sqrt(mean(h^2) + eps).  One workgroup of 1024
// threads per row of the padded row range (rows >= M write zero fragments); d <= 8192, d % 8 == 0.  A thread owns 4
// consecutive columns and requests all slices of them at once (up to 16 loads in flight: with 8 columns per thread and
// 8 slices per trip the kernel paid four memory round trips per row); two neighbouring lanes then hold the 8 values of
// one fragment chunk, exchange them, and the even lane writes the chunk's high parts, the odd lane its low parts.
constexpr int WNORM_NT = 1024;
template <typename WT>
__global__ __launch_bounds__(WNORM_NT) void wide_add_norm_frag_kernel(float* __restrict__ h, int ldh, Parts delta, int ldd, int M,
                                                                  const WT* __restrict__ gain, uint4* __restrict__ frag, int d, float eps) {
    __shared__ float part[WNORM_NT / 64];
    constexpr int MAXG = 2;                         // groups of 4 values per thread
    const int row = blockIdx.x, ng = d / 4, kblks = d / 32;
    const bool live = row < M;
    const int rr = min(row, M - 1);
    float4 x[MAXG];
    float ss = 0.f;
#pragma unroll
    for (int k = 0; k < MAXG; ++k) {
        const int gi = (int)threadIdx.x + WNORM_NT * k;
        x[k] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (gi < ng) {
            float4 a = *reinterpret_cast<const float4*>(h + (size_t)rr * ldh + 4 * gi);
            if (delta.p) {
                const size_t idx = (size_t)rr * ldd + 4 * gi;
                float4 da = *reinterpret_cast<const float4*>(delta.p + idx);
                if (delta.n <= 4) parts_add<3>(da, delta, idx, 1);
                else if (delta.n <= 8) parts_add<7>(da, delta, idx, 1);
                else parts_add<15>(da, delta, idx, 1);        // slices 1..15 in one trip (at most 16 slices)
                a.x += da.x; a.y += da.y; a.z += da.z; a.w += da.w;
                if (live) *reinterpret_cast<float4*>(h + (size_t)rr * ldh + 4 * gi) = a;
            }
            x[k] = a;
            ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
        }
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < WNORM_NT / 64; ++w) tot += part[w];
    const float inv = 1.0f / sqrtf(tot / (float)d + eps);
    const int odd = threadIdx.x & 1;
#pragma unroll
    for (int k = 0; k < MAXG; ++k) {
        const int gi = (int)threadIdx.x + WNORM_NT * k;
        // (ng is even, so a lane and its neighbour are in range together; out-of-range lanes still take part in the exchange)
        float4 y = make_float4(0.f, 0.f, 0.f, 0.f);
        if (gi < ng) {
            const WT* gp = gain + 4 * gi;
            y = make_float4(x[k].x * to_f32(gp[0]) * inv, x[k].y * to_f32(gp[1]) * inv, x[k].z * to_f32(gp[2]) * inv, x[k].w * to_f32(gp[3]) * inv);
        }
        const float4 o = make_float4(__shfl_xor(y.x, 1, 64), __shfl_xor(y.y, 1, 64), __shfl_xor(y.z, 1, 64), __shfl_xor(y.w, 1, 64));
        if (gi < ng) {
            const float4 lo4 = odd ? o : y, hi4 = odd ? y : o;        // values 0..3 and 4..7 of the chunk
            uint32_t wh[4], wl[4];
            f32_to_bf16x2_hilo(lo4.x, lo4.y, wh[0], wl[0]);
            f32_to_bf16x2_hilo(lo4.z, lo4.w, wh[1], wl[1]);
            f32_to_bf16x2_hilo(hi4.x, hi4.y, wh[2], wl[2]);
            f32_to_bf16x2_hilo(hi4.z, hi4.w, wh[3], wl[3]);
            const int k0 = 8 * (gi >> 1);
            const int tt = row >> 3, r8 = row & 7, i_hi = 4 * (r8 >> 1) + (r8 & 1);
            const size_t base = ((size_t)tt * kblks + (k0 >> 5)) * 64 + ((k0 >> 3) & 3) * 16;
            uint4 w4 = odd ? make_uint4(wl[0], wl[1], wl[2], wl[3]) : make_uint4(wh[0], wh[1], wh[2], wh[3]);
            if (!live) w4 = make_uint4(0u, 0u, 0u, 0u);
            frag[base + i_hi + (odd ? 2 : 0)] = w4;
        }
    }
}

// act = silu(gate) * up from the interleaved gate|up result (sum of partials), written as fragments of the down projection.
// grid (row tiles of 8 rows, column chunks), 256 threads; F % 8 == 0.  Eight consecutive threads serve the eight rows of
// the tile for one group of 8 activations: together they write one whole 256-byte piece of a fragment block (a thread
// per (row, group) in row-major order scattered 16-byte stores over the buffer: 137 us for a 3008-row prefill layer).
__global__ void wide_silu_frag_kernel(Parts gu, int M, int F, uint4* __restrict__ frag) {
    const int row = blockIdx.x * 8 + (threadIdx.x & 7), kblks = F / 32;
    const bool live = row < M;
    const int rr = min(row, M - 1);
    const int per = blockDim.x >> 3;
    for (int gi = blockIdx.y * per + (threadIdx.x >> 3); gi < F / 8; gi += gridDim.y * per) {
        const size_t o = (size_t)rr * 2 * F + (size_t)gi * 16;
        const float4 g0 = parts_load4(gu, o), g1 = parts_load4(gu, o + 4), u0 = parts_load4(gu, o + 8), u1 = parts_load4(gu, o + 12);
        const float g[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w}, u[8] = {u0.x, u0.y, u0.z, u0.w, u1.x, u1.y, u1.z, u1.w};
        float y[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) y[e] = g[e] / (1.0f + expf(-g[e])) * u[e];
        store_afrag8(frag, kblks, row, 8 * gi, y, !live);
    }
}

// rope_append_kernel for rows whose fused QKV result arrives as partials: sums them, rotates q and k, writes q to `q_out`
// (row stride ldq, the buffer the attention reads) and k, v to the cache.  Same position / slot rule and optional bias as
// rope_append_kernel.
template <typename ST>
__global__ void wide_rope_append_kernel(Parts qkv, float* __restrict__ q_out, int ldq, int Hq, int Hkv, int HD, const int* __restrict__ base,
                                        int offset, int seq0, int m, ST* __restrict__ kc, ST* __restrict__ vc, int maxL,
                                        float theta, const int* __restrict__ pos_delta, const float* __restrict__ bias,
                                        const float* __restrict__ rope_tab = nullptr, int npos = 0) {
    const int row = blockIdx.x;
    const int seq = seq0 + row / m;
    const int slot = base[seq] + offset + row % m;
    const int pos = pos_delta ? base[seq] + pos_delta[row] : slot;
    const int half = HD / 2;
    const size_t rbase = (size_t)row * (Hq + 2 * Hkv) * HD;
    const int npair2 = (Hq + Hkv) * half / 2;                 // two pairs (4 adjacent columns) per trip
    for (int idx = blockIdx.y * blockDim.x + threadIdx.x; idx < npair2; idx += gridDim.y * blockDim.x) {
        const int head = (2 * idx) / half, i = (2 * idx) % half;
        float4 x = parts_load4(qkv, rbase + (size_t)head * HD + 2 * i);            // pairs (i, i + hd/2) sit in columns 2i, 2i+1
        if (bias) { const float4 b = *reinterpret_cast<const float4*>(bias + (size_t)head * HD + 2 * i); x.x += b.x; x.y += b.y; x.z += b.z; x.w += b.w; }
        float y[4];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            double s, c;
            if (rope_tab) {
                const float2 t = *reinterpret_cast<const float2*>(rope_tab + ((size_t)min(pos, npos - 1) * half + i + e) * 2);
                c = (double)t.x; s = (double)t.y;
            } else {
                const double inv_freq = exp2(-2.0 * (double)(i + e) / (double)HD * log2((double)theta));
                sincos((double)pos * inv_freq, &s, &c);
            }
            const float x1 = e ? x.z : x.x, x2 = e ? x.w : x.y;
            y[2 * e] = (float)((double)x1 * c - (double)x2 * s);
            y[2 * e + 1] = (float)((double)x2 * c + (double)x1 * s);
        }
        if (head < Hq) {
            *reinterpret_cast<float4*>(q_out + (size_t)row * ldq + (size_t)head * HD + 2 * i) = make_float4(y[0], y[1], y[2], y[3]);
        } else {
            ST* dst = kc + (((size_t)seq * Hkv + (head - Hq)) * maxL + slot) * HD * KVWidth<ST>::W;
#pragma unroll
            for (int e = 0; e < 4; ++e) kv_put(dst, HD, 2 * i + e, y[e]);
        }
    }
    for (int idx = blockIdx.y * blockDim.x + threadIdx.x; idx < Hkv * HD / 4; idx += gridDim.y * blockDim.x) {
        const int head = (4 * idx) / HD, c = (4 * idx) % HD;
        float4 v = parts_load4(qkv, rbase + (size_t)(Hq + Hkv) * HD + 4 * idx);
        if (bias) { const float4 b = *reinterpret_cast<const float4*>(bias + (size_t)(Hq + Hkv) * HD + 4 * idx); v.x += b.x; v.y += b.y; v.z += b.z; v.w += b.w; }
        ST* dst = vc + (((size_t)seq * Hkv + head) * maxL + slot) * HD * KVWidth<ST>::W;
        kv_put(dst, HD, c, v.x); kv_put(dst, HD, c + 1, v.y); kv_put(dst, HD, c + 2, v.z); kv_put(dst, HD, c + 3, v.w);
    }
}

}  // namespace hivis

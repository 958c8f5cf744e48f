// Phase programs: a verify pass (N layers + LM head + greedy tokens), a K-step draft round and the
// roll-forward of the drafter are lists of phases executed by one 512-thread workgroup per compute
// unit.  By default every phase is one kernel launch (phase_kernel; the kernel boundary orders the
// phases); optionally the whole list runs as ONE cooperative launch with a grid-wide barrier between
// phases and weight prefetch across the barriers (fused_pass_kernel; measured slower, kept as an option).  The small row-wise operations are folded into the GEMM phases:
//   RMSNorm     -> prologue (gain applied while building the MFMA A fragments, 1/rms in the epilogue)
//   RoPE+append -> epilogue of the fused QKV GEMM (rotary pairs are adjacent columns of a tile)
//   SiLU*up     -> epilogue of the fused gate|up GEMM (gate and up columns share a tile)
//   residual    -> epilogue of the O and down GEMMs (each output element has exactly one writer)
//   argmax      -> epilogue of the LM-head GEMM (per-workgroup candidates) + a tiny reduction phase
// Used for passes of at most one MFMA tile of rows (8 rows for bf16 weights, 16 for fp32).
//
// Memory discipline between phases (the L2 is per XCD and not coherent across XCDs): every buffer that one
// phase writes and a later phase reads is written AT MOST ONCE per launch, with write-through stores, and is
// not read before that write in the same launch (the host gives every phase its own output buffer).  A
// reader's first touch therefore misses its caches and fetches the fresh value from memory, and the grid
// barrier needs no cache write-back or invalidation.  The few words that are rewritten inside one launch
// (drafted token ids) are read with agent-scope loads.
#pragma once
#include <type_traits>
#include "hivis_kernels.h"

namespace hivis {

enum { PH_GEMM = 0, PH_ATTN = 1, PH_ATTN_MERGE = 2, PH_PREP = 3, PH_NORM_ROWS = 4, PH_ARGMAX = 5, PH_SAMPLE = 6 };
enum { PRO_PLAIN = 0, PRO_RMS = 1 };
constexpr int FUSED_RMAX = 8;      // (head,row) pairs per attention work item in the persistent kernel
enum { FEPI_STORE = 0, FEPI_ADD_TO = 1, FEPI_ADDVEC = 2, FEPI_QKV = 3, FEPI_SILU = 4, FEPI_LOGITS = 5,
       FEPI_QKV_TAB = 6,     // kernel variants only (never a Phase.epi): QKV whose rows are A + add_rows[token], see Phase.wb;
       FEPI_QKV_TAB4 = 7 };  // two staged rows (at most two sequences) / four staged rows (three or four sequences)

struct Phase {
    int type, pro, epi;
    int K, N;
    const uint4* W;            // GEMM: packed weights
    const float* A; int lda;   // GEMM: activation rows; ATTN: q rows (fused qkv buffer)
    const void* gain;          // PRO_RMS: gain vector (weight dtype); GATHER: embedding table
    float* Y; int ldy;         // output rows (STORE / ADD_TO / ADDVEC / LOGITS / QKV q part / SILU act / ATTN_MERGE / PREP gather / NORM_ROWS)
    const float* R; int ldr;   // ADD_TO: Y = R + result (R == Y: accumulate into the residual stream)
    const void* vec; int vec_idx;          // ADDVEC: table [*][N] of the weight dtype and the row to add
    // ADDVEC (fusion FC), optional: columns [K/2, K) of activation row (seq, i) are row tok[seq*tok_sseq + i*tok_srow] of
    // the embedding table emb ([vocab][K/2], weight dtype) instead of A's: the gather of Embed(x) needs no launch
    const void* emb; const int32_t* tok; int tok_sseq, tok_srow;
    // ADDVEC, alternative to emb: the embedding half of the fusion FC as a table.  [f ; e] [w1 ; w2] = f w1 + e w2, and
    // e w2 depends on the token alone, so add_rows[token][N] (fp32, computed once at create) is ADDED in the epilogue and
    // the GEMM runs over f's K = d only: half the weight bytes per step.  The token of a row as for emb (tok, or reduced).
    const float* add_rows;
    // QKV with add_rows (the drafter's first phase of a step, when the fusion FC's w1 half rode on the LM-head launch
    // before it): activation row r is A[r] + add_rows[token of r], the token as above (tok, or reduced from pm / pi), and
    // workgroup 0 writes the sum back to wb [M][K] (the layer's residual stream, read later by the O projection)
    float* wb;
    // LOGITS with N > vocab: columns [vocab, N) are not logits but extra output columns (the packed weights carry another
    // matrix of the same K behind the LM head: w1 of the fusion FC); they go to Y2 [M][ldy2] plus vec[vec_idx], and
    // take no part in the greedy candidates
    float* Y2; int ldy2;
    // ... and if tok is null the token of row r is the greedy token of the LM-head phase before it, reduced here from
    // that phase's per-workgroup candidates pm / pi ([row][ncand]); workgroup 0 also stores it to tok_out
    int ncand;
    void* kc; void* vc; int maxL;          // QKV epilogue / ATTN: cache of this layer
    const int* base; int offset;           // row positions: base[seq] + offset + i
    const int32_t* ids; int id_sseq, id_srow;      // PREP: token of row (seq, i) = ids[seq*id_sseq + i*id_srow] (ids may be null: no gather)
    int32_t* tok_out; int o_sseq, o_srow;          // ARGMAX: destination of the greedy token of row (seq, i)
    AttnShape att; int att_items;                  // ATTN / ATTN_MERGE
    const float* rope;                             // QKV epilogue: rotary table of the context, [position][hd/2][2] cos, sin
    const float* bias;                             // QKV epilogue: optional q/k/v projection biases [N] in packed column order
    float* ws;                                     // ATTN: per-workgroup partials of the key splits
    int* cnt;                                      // ATTN: arrival counter per item; LM head: one arrival counter (zero between launches)
    float* pm; int* pi;                            // LOGITS writes, ARGMAX reads: greedy candidates [row][workgroup]
    const float* u; int u_sseq, u_idx;             // SAMPLE: uniform number of row (seq, i) = u[seq*u_sseq + u_idx]; logits rows in A (stride lda)
    const uint4* next_W; int next_K, next_N;       // GEMM: weights of the next GEMM phase of the program (prefetch), or null
    uint4* frag;                                   // ATTN with one key split, optional: the rows go out as A fragments of the next GEMM (K = ldy) instead of to Y
};

struct PassParams {
    const Phase* phases; int nphases;
    int M, nseq, m;                 // rows of the pass = nseq * m
    int d, Hq, Hkv, hd, F, V;
    float eps, theta;
    float inv_temp;                 // SAMPLE: 1 / temperature
    unsigned* bar;                  // [0] arrival counter (zeroed before launch), [1] abort flag
    int* bad;                       // set to 1 when a row has no greedy token (no logit above -inf: NaN input); may be null
    unsigned spin_limit;
    unsigned long long* prof3;      // optional [grid][4] per-workgroup entry time, exit time, hardware id of one launch (one launch per phase only)
    unsigned long long* prof2;      // optional [nphases][8] finer timestamps inside GEMM phases (workgroup 0)
    unsigned long long* prof;       // optional [nphases][3] timestamps of workgroup 0 (phase start, phase end, barrier end), 100 MHz
};

// Grid-wide barrier.  Every thread first waits until its own write-through stores have been acknowledged (a GEMM
// phase has done so itself before requesting the next phase's weights: stores_drained), then one thread arrives and spins; bounded: on timeout the abort flag is raised and every workgroup leaves.  No
// cache write-back or invalidation is needed (see the memory discipline above).  Returns false
// if the pass was aborted.
__device__ __forceinline__ bool grid_barrier(unsigned* bar, unsigned target, unsigned spin_limit, bool stores_drained) {
    if (!stores_drained) wait_vmem();
    lds_barrier();
    if (threadIdx.x == 0) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");     // publishes the workgroup's write-through stores to the other XCDs
        __hip_atomic_fetch_add(&bar[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        unsigned spins = 0;
        while (__hip_atomic_load(&bar[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            __builtin_amdgcn_s_sleep(1);
            ++spins;
            if ((spins & 255u) == 0u && __hip_atomic_load(&bar[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) break;
            if (spins > spin_limit) { __hip_atomic_store(&bar[1], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); break; }
        }
    }
    lds_barrier();
    return __hip_atomic_load(&bar[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u;
}

// ---- GEMM phase -----------------------------------------------------------------------------------
template <typename WT> struct FusedCfg;
// KBW weight blocks per wavefront per K pass (= one unit of the software pipeline); G tiles per tile group
// 512 threads (8 wavefronts, two per SIMD) so that every wavefront may use up to 256 registers: the pipeline
// state (two 8 KiB weight units, 8 activation fragments, accumulators, staged rows) must never spill, because a
// spill reload after the barrier's cache invalidation is a full memory round trip.
constexpr int FUSED_NW = 8, FUSED_NT = FUSED_NW * 64;
template <> struct FusedCfg<bf16_t> { static constexpr int KBW = 8, G = 8, NW = FUSED_NW; };
template <> struct FusedCfg<float> { static constexpr int KBW = 8, G = 4, NW = FUSED_NW; };
constexpr int FUSED_U = 8;
constexpr int FUSED_QM = 8;       // activation rows staged per lane per pass (bf16: rows q; fp32: rows 2 q + lane / 32)

// LDS of a GEMM phase (floats): cross-wave reduction [NW][TILE] | reduced tiles [TILE] | ssq partials [NW][16]
// | inv_rms [16] | A chunk of one K pass in MFMA fragment order [NW*KBW blocks][4][RU] x 16 bytes
__host__ __device__ constexpr size_t fused_gemm_lds_floats(int NW, int G, int RPL, int KBW) {
    return (size_t)NW * G * 64 * RPL + (size_t)G * 64 * RPL + (size_t)NW * 16 + 16 + (size_t)NW * KBW * 4 * 16 * 4;
}

// Four consecutive RMSNorm gains as loaded (raw bits of the weight type); converted to float where they are used
template <typename WT> struct Gain4;
template <> struct Gain4<bf16_t> {
    typedef uint2 type;
    static __device__ __forceinline__ float get(const uint2& g, int e) {
        const uint32_t w = (e < 2) ? g.x : g.y;
        return __uint_as_float((e & 1) ? (w & 0xFFFF0000u) : (w << 16));
    }
};
template <> struct Gain4<float> {
    typedef float4 type;
    static __device__ __forceinline__ float get(const float4& g, int e) { return e == 0 ? g.x : e == 1 ? g.y : e == 2 ? g.z : g.w; }
};

// four consecutive values of the weight dtype as floats
__device__ __forceinline__ float4 load4_f32(const bf16_t* p) {
    const uint2 u = *reinterpret_cast<const uint2*>(p);
    return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xFFFF0000u), __uint_as_float(u.y << 16), __uint_as_float(u.y & 0xFFFF0000u));
}
__device__ __forceinline__ float4 load4_f32(const float* p) { return *reinterpret_cast<const float4*>(p); }

// K blocks of pass p that wavefront `wave` owns.  A full pass gives every wavefront KBW consecutive blocks; a ragged
// last pass is dealt out evenly (ceil(rest / NW) blocks each), so that no wavefront streams a whole unit more than the
// others (with K = 11008 the last pass has 24 blocks: 3 per wavefront instead of 8 for three of them).
template <int NW, int KBW> __device__ __forceinline__ int unit_bw(int kblks, int p) {
    const int rest = kblks - p * NW * KBW;
    return rest >= NW * KBW ? KBW : max(0, (rest + NW - 1) / NW);
}
template <int NW, int KBW> __device__ __forceinline__ int unit_kb0(int kblks, int p, int wave) { return p * NW * KBW + wave * unit_bw<NW, KBW>(kblks, p); }
template <int NW, int KBW> __device__ __forceinline__ int unit_nkb(int kblks, int p, int wave) {
    const int bw = unit_bw<NW, KBW>(kblks, p);
    return max(0, min(bw, kblks - p * NW * KBW - wave * bw));
}

// Loads of one unit: the wavefront's K blocks [kb0, kb0+nkb) of tile `tile`.
__device__ __forceinline__ void issue_unit(uint4 (&wb)[FUSED_U], const uint4* __restrict__ W, int kblks, int tile, int kb0,
                                           int nkb, int lane) {
    const uint4* p = W + ((size_t)tile * kblks + kb0) * 64 + lane;
#pragma unroll
    for (int j = 0; j < FUSED_U; ++j)
        if (j < nkb) wb[j] = p[(size_t)j * 64]; else wb[j] = make_uint4(0, 0, 0, 0);
}

// tile row (MFMA A row) that holds activation row `row`: bf16 keeps hi at 4*(row/2) + row%2 and lo two rows below
template <typename WT> __device__ __forceinline__ int tile_row_of(int row);
template <> __device__ __forceinline__ int tile_row_of<bf16_t>(int row) { return 4 * (row >> 1) + (row & 1); }
template <> __device__ __forceinline__ int tile_row_of<float>(int row) { return row; }

// Writes 4 consecutive k of one activation row (already multiplied by the gain) into the LDS chunk.
__device__ __forceinline__ void stage_store(bf16_t, uint4* chunk, int RU, int row, int kl /*k within the chunk, multiple of 4*/,
                                            const float (&x)[4]) {
    const int kb = kl >> 5, g = (kl & 31) >> 3, e0 = kl & 7;
    const int slot = (kb * 4 + g) * RU + tile_row_of<bf16_t>(row);
    uint32_t h01, l01, h23, l23;
    f32_to_bf16x2_hilo(x[0], x[1], h01, l01);
    f32_to_bf16x2_hilo(x[2], x[3], h23, l23);
    uint2* ph = reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(chunk + slot) + e0);
    uint2* pl = reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(chunk + slot + 2) + e0);
    *ph = make_uint2(h01, h23);
    *pl = make_uint2(l01, l23);
}
__device__ __forceinline__ void stage_store(float, uint4* chunk, int RU, int row, int kl, const float (&x)[4]) {
    const int kb = kl >> 4, g = (kl & 15) >> 2;
    chunk[(kb * 4 + g) * RU + row] = make_uint4(__float_as_uint(x[0]), __float_as_uint(x[1]), __float_as_uint(x[2]), __float_as_uint(x[3]));
}
__device__ __forceinline__ void frag_from(bf16x8_t& f, const uint4& u) { f = __builtin_bit_cast(bf16x8_t, u); }
__device__ __forceinline__ void frag_from(float4& f, const uint4& u) {
    f = make_float4(__uint_as_float(u.x), __uint_as_float(u.y), __uint_as_float(u.z), __uint_as_float(u.w));
}

// Greedy tokens without a launch of their own: after a workgroup of the LM-head phase has stored its per-row
// candidates (write-through) and those stores have completed, it arrives on the phase's counter; the workgroup that
// arrives last reduces the gridDim.x candidates of every row (lowest index wins ties, as everywhere) and stores the
// tokens.  Agent-scope atomics only (stores, counter, loads), as in the attention's key-split merge.  flag: one LDS word.
__device__ __forceinline__ void lm_head_elect(const Phase& ph, const PassParams& pp, int* __restrict__ flag) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    wait_vmem();
    lds_barrier();
    if (threadIdx.x == 0) flag[0] = __hip_atomic_fetch_add(ph.cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    lds_barrier();
    if (flag[0] != (int)gridDim.x - 1) return;
    const int ncand = gridDim.x;
    for (int row = wave; row < pp.M; row += FUSED_NW) {
        float bv = -INFINITY; int bi = 0x7FFFFFFF;
        for (int w = lane; w < ncand; w += 64) {
            const float v = ld_agent(&ph.pm[(size_t)row * ncand + w]);
            const int i = __hip_atomic_load(&ph.pi[(size_t)row * ncand + w], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const float ov = __shfl_xor(bv, o, 64); const int oi = __shfl_xor(bi, o, 64);
            if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
        }
        if (lane == 0) {
            if (pp.bad && (unsigned)bi >= (unsigned)pp.V) st_wt(pp.bad, 1);
            st_wt(&ph.tok_out[(row / pp.m) * ph.o_sseq + (row % pp.m) * ph.o_srow], clamp_token(bi, pp.V));
        }
    }
    if (threadIdx.x == 0) st_wt(ph.cnt, 0);
}

// GEMM phase of the persistent kernel (rows <= one MFMA tile).  Work split as in gemm_skinny_kernel: the
// workgroup owns a contiguous range of 16-column tiles and covers all of K; in K pass p wavefront w owns
// blocks [(p*NW + w)*KBW, +KBW) of every tile.
//  * Activations: per pass the workgroup's threads load the pass's K range of all rows once (coalesced float4), apply
//    the RMSNorm gain, accumulate the rows' sums of squares, convert to MFMA fragments and park them in LDS;
//    the wavefronts then fetch their fragments with ds_read (LDS traffic is counted separately from global
//    loads, so waiting for fragments never waits for weight loads).  The next pass's rows are already being
//    loaded into registers while the current pass streams.
//  * Weights: one unit (KBW KiB per wavefront) ahead, and the chain of prefetches does not stop at the end of
//    a tile group, a pass or the phase: the last unit of a phase loads the first unit of the NEXT GEMM phase
//    (`head`), so those loads are in flight while the workgroup waits at the grid barrier.
template <typename WT, int EPI, bool SINGLE>
__device__ __forceinline__ void gemm_phase(const Phase& ph, const PassParams& pp, float* __restrict__ lds, uint4 (&head)[FUSED_U],
                           bool& head_valid, uint4 (&wb1)[FUSED_U], bool& wb1_valid, int pidx) {
#define HIVIS_MARK(k) if (pp.prof2 && blockIdx.x == 0 && threadIdx.x == 0) pp.prof2[pidx * 8 + (k)] = wall_clock64();
    typedef WTraits<WT> TR;
    typedef typename AFrag<WT>::type afrag_t;
    typedef typename KVType<WT>::type KT;
    constexpr int RPL = TR::RPL, ROWS = TR::ROWS, KB = TR::KB, KBW = FusedCfg<WT>::KBW, NW = FusedCfg<WT>::NW;
    // tiles per group: the full group size where a workgroup owns many tiles (LM head, gate|up; also the generic
    // interpreter), half of it for the kernels whose workgroups own at most a few tiles (fewer accumulators)
    constexpr int G = (!SINGLE && (EPI < 0 || EPI == FEPI_LOGITS || EPI == FEPI_SILU)) ? FusedCfg<WT>::G : FusedCfg<WT>::G / 2;
    // rows staged per lane and pass; the table-add QKV variants serve draft steps of at most two / four sequences and stage
    // that many rows only (with eight, their second set of row registers spills)
    constexpr int U = FUSED_U, QM = (EPI == FEPI_QKV_TAB) ? 2 : (EPI == FEPI_QKV_TAB4) ? 4 : FUSED_QM, NT = FUSED_NT;
    static_assert(KBW == U && (G % 2) == 0, "one unit per tile slice; tiles are processed in pairs");
    constexpr int TILE = G * 64 * RPL;
    constexpr int SLOTS = TILE / NT;         // epilogue slots per thread (all of the same row and column-in-tile)
    static_assert(TILE % NT == 0, "whole epilogue slots per thread");
    constexpr int CW = NW * KBW * KB;        // k per pass (64 blocks)
    constexpr int SL4 = KBW * KB / 4;        // float4 columns of one wavefront's K slice of a pass (64 bf16 / 32 fp32)
    constexpr int RS = 64 / SL4;             // rows a wavefront covers per load step (1 / 2)
    static_assert(RS == 1 || RS == 2, "a wavefront's lanes cover one or two rows of its slice at a time");
    float* red = lds;                        // [NW][G][64][RPL]
    float* tile = red + (size_t)NW * TILE;   // [G][64][RPL]
    float* ssq_w = tile + TILE;              // [NW][16]
    float* inv_rms = ssq_w + NW * 16;        // [16]
    uint4* chunk = reinterpret_cast<uint4*>(inv_rms + 16);

    constexpr bool TAB = EPI == FEPI_QKV_TAB || EPI == FEPI_QKV_TAB4;        // the drafter's QKV with table rows added in the prologue: a kernel of its own, so
                                                     // that the QKV kernel of the verify pass carries none of its registers
    const int epi = (EPI >= 0) ? (TAB ? (int)FEPI_QKV : EPI) : ph.epi;       // compile-time epilogue when the phase has its own kernel
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wavefront index as a scalar: branches on it are uniform
    const int M = pp.M, K = ph.K, N = ph.N;
    const int kblks = K / KB, ntiles = N / 16;
    // (the divisions run on the vector ALU; read back as scalars so that every branch on the tile range is uniform)
    // Workgroups are dealt to the 8 XCDs round-robin, so workgroup b runs on XCD b % 8.  When the tiles do not divide
    // evenly, the workgroups with one tile more must be spread over all XCDs (each has its own L2 and memory path):
    // XCD x takes the contiguous share [x * grid/8, (x+1) * grid/8) of the virtual workgroup order.
    const int vb = (gridDim.x % 8 == 0) ? (int)((blockIdx.x % 8) * (gridDim.x / 8) + blockIdx.x / 8) : (int)blockIdx.x;
    const int t_begin = __builtin_amdgcn_readfirstlane((int)(((long long)vb * ntiles) / gridDim.x));
    const int t_end = __builtin_amdgcn_readfirstlane((int)(((long long)(vb + 1) * ntiles) / gridDim.x));
    const int ntl = t_end - t_begin;
    const int npass = (kblks + NW * KBW - 1) / (NW * KBW);
    const WT* gain = (ph.pro == PRO_RMS) ? (const WT*)ph.gain : nullptr;
    const float* A = ph.A;
    const int lda = ph.lda;
    const uint4* W = ph.W;
    const int RU = (RPL == 2) ? 4 * ((M + 1) >> 1) : ((M + 3) & ~3);      // tile rows in use
    // Activation staging is PRIVATE to a wavefront: it loads, converts and parks exactly the K slice its own weight
    // blocks multiply (lane: float4 column col4 of the slice, rows row0 + q*RS), into its own part of the LDS chunk, and
    // reads its fragments back; no workgroup barrier is involved, so the eight wavefronts stream independently until the
    // cross-wavefront reduction at the end (with workgroup-wide staging every pass waited twice for the slowest one).
    const int col4 = lane % SL4, row0 = lane / SL4;
    uint4* slice = chunk + (size_t)wave * (KBW * 4 * 16);               // [KBW blocks][4][RU] x 16 bytes of this wavefront
    float ssq_acc[QM];
#pragma unroll
    for (int q = 0; q < QM; ++q) ssq_acc[q] = 0.f;
    float best_v = -INFINITY; int best_i = 0x7FFFFFFF;   // greedy-token candidate (LOGITS): a thread always serves one row

    // first units of the next GEMM phase for this wavefront (persistent mode only: requested at the end of this phase)
    const int n_kblks = ph.next_K / KB, n_ntiles = ph.next_N / 16;
    const int n_tile = __builtin_amdgcn_readfirstlane(ph.next_W ? (int)(((long long)vb * n_ntiles) / gridDim.x) : 0);
    const int n_tend = __builtin_amdgcn_readfirstlane(ph.next_W ? (int)(((long long)(vb + 1) * n_ntiles) / gridDim.x) : 0);
    const bool n_has = ph.next_W && n_tile < n_tend;
    const int n_npass = (n_kblks + NW * KBW - 1) / (NW * KBW);
    // The unit order of a phase is tile-inner, pass-outer within a tile group.  `head` holds the first unit and
    // `wb1` the second one: the next tile of the same pass, or, for a workgroup with a single tile, the same tile
    // of the next pass.
#define HIVIS_FIRST_UNITS(W_, kblks_, tile_, ntl_, npass_)                                                         \
    {                                                                                                              \
        issue_unit(head, W_, kblks_, tile_, unit_kb0<NW, KBW>(kblks_, 0, wave), unit_nkb<NW, KBW>(kblks_, 0, wave), lane); \
        head_valid = true;                                                                                         \
        /* one call site for the second unit (two alternative ones make the compiler drain the first unit's loads) */ \
        const bool next_tile_ = (ntl_) >= 2;                                                                       \
        wb1_valid = next_tile_ || (SINGLE && (npass_) >= 2);                                                       \
        const int p1_ = next_tile_ ? 0 : 1;                                                                        \
        if (wb1_valid) issue_unit(wb1, W_, kblks_, (tile_) + (next_tile_ ? 1 : 0), unit_kb0<NW, KBW>(kblks_, p1_, wave), unit_nkb<NW, KBW>(kblks_, p1_, wave), lane); \
    }

    if (ntl <= 0) {
        if (epi == FEPI_LOGITS && threadIdx.x < ROWS && (int)threadIdx.x < M) {
            st_wt(&ph.pm[(size_t)threadIdx.x * gridDim.x + blockIdx.x], -INFINITY); st_wt(&ph.pi[(size_t)threadIdx.x * gridDim.x + blockIdx.x], 0x7FFFFFFF);
        }
        if (epi == FEPI_LOGITS && ph.cnt) lm_head_elect(ph, pp, reinterpret_cast<int*>(inv_rms));
        wait_vmem();
        if (!head_valid && n_has) HIVIS_FIRST_UNITS(ph.next_W, n_kblks, n_tile, n_tend - n_tile, n_npass)
        return;
    }

    // raw activation loads of pass `ps`: float4 (row0 + q*RS, first k of the wavefront's slice + 4*col4) and the gain of
    // those 4 columns (unconditional loads from clamped addresses: a load under a divergent branch is followed by a
    // full wait, which would serialise the rows into one memory round trip each)
    static_assert(EPI == FEPI_QKV_TAB || EPI == FEPI_QKV_TAB4 || QM * RS >= ROWS, "every row is staged by some lane");
    typedef typename Gain4<WT>::type gain4_t;
    // fusion FC with the embedding half taken from the table: the tokens of this lane's rows
    int tokr[QM];        // as loaded; forced into [0, V) where it is used, so that nothing waits for the load here
#pragma unroll
    for (int q = 0; q < QM; ++q) {
        tokr[q] = 0;
        if ((EPI == FEPI_ADDVEC && ph.emb != nullptr && ph.tok != nullptr) || (TAB && ph.tok != nullptr)) {
            const int r_ = min(row0 + q * RS, M - 1);
            tokr[q] = __hip_atomic_load(&ph.tok[(r_ / pp.m) * ph.tok_sseq + (r_ % pp.m) * ph.tok_srow], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    float4 araw[QM]; gain4_t graw = gain4_t();
    float4 araw2[SINGLE ? QM : 1]; gain4_t graw2 = gain4_t();      // rows of the second pass of a pair (one tile per workgroup)
    float4 braw[TAB ? QM : 1];                                     // QKV with add_rows: the table rows added to the activation rows
#define HIVIS_LOAD_RAW_TO(ps, ARAW, GRAW)                                                                          \
    {                                                                                                              \
        const int k_ = min(unit_kb0<NW, KBW>(kblks, ps, wave) * KB + 4 * col4, K - 4);                             \
        if (gain) GRAW = *reinterpret_cast<const gain4_t*>(gain + k_);   /* converted where it is used: no wait here */ \
        const bool from_emb_ = EPI == FEPI_ADDVEC && ph.emb != nullptr && k_ >= K / 2;                             \
        _Pragma("unroll") for (int q = 0; q < QM; ++q) {                                                           \
            const int row_ = min(row0 + q * RS, M - 1);                                                            \
            if (from_emb_) ARAW[q] = load4_f32(reinterpret_cast<const WT*>(ph.emb) + (size_t)clamp_token(tokr[q], pp.V) * (K / 2) + (k_ - K / 2)); \
            else ARAW[q] = *reinterpret_cast<const float4*>(A + (size_t)row_ * lda + k_);                          \
            if (TAB) braw[q] = *reinterpret_cast<const float4*>(ph.add_rows + (size_t)clamp_token(tokr[q], pp.V) * K + k_); \
        }                                                                                                          \
    }
#define HIVIS_LOAD_RAW(ps) HIVIS_LOAD_RAW_TO(ps, araw, graw)
    // Stage this wavefront's slice of pass `ps` (whose rows are in ARAW) into its LDS slice as MFMA fragments, run
    // NEXT (the request for the rows staged next, or nothing), and fetch the fragments af[0..KBW).
#define HIVIS_STAGE_FROM(ps, ARAW, GRAW, do_ssq, NEXT)                                                             \
    {                                                                                                              \
        const int nkb_ = unit_nkb<NW, KBW>(kblks, ps, wave);                                                       \
        _Pragma("unroll") for (int q = 0; q < QM; ++q) {                                                           \
            const int row_ = row0 + q * RS;                                                                        \
            if (row_ < M && 4 * col4 < nkb_ * KB) {                                                                \
                float x_[4] = {ARAW[q].x, ARAW[q].y, ARAW[q].z, ARAW[q].w};                                        \
                if (TAB) {                                                                                         \
                    x_[0] += braw[q].x; x_[1] += braw[q].y; x_[2] += braw[q].z; x_[3] += braw[q].w;                \
                    if (blockIdx.x == 0 && tg == t_begin) {                                                        \
                        float* wb_ = ph.wb + (size_t)row_ * K + unit_kb0<NW, KBW>(kblks, ps, wave) * KB + 4 * col4; \
                        st_wt(wb_, x_[0]); st_wt(wb_ + 1, x_[1]); st_wt(wb_ + 2, x_[2]); st_wt(wb_ + 3, x_[3]);    \
                    }                                                                                              \
                }                                                                                                  \
                if (do_ssq) ssq_acc[q] += x_[0] * x_[0] + x_[1] * x_[1] + x_[2] * x_[2] + x_[3] * x_[3];           \
                if (gain) { _Pragma("unroll") for (int e = 0; e < 4; ++e) x_[e] *= Gain4<WT>::get(GRAW, e); }      \
                stage_store(WT(), slice, RU, row_, 4 * col4, x_);                                                  \
            }                                                                                                      \
        }                                                                                                          \
        NEXT                                                                                                       \
        /* the slice is written and read by this wavefront only */                                                 \
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");                                                     \
        __builtin_amdgcn_wave_barrier();                                                                           \
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");                                                     \
        const int i_ = min(lane & 15, RU - 1), g4_ = lane >> 4;                                                    \
        _Pragma("unroll") for (int j = 0; j < KBW; ++j) {                                                          \
            const uint4 u_ = slice[(j * 4 + g4_) * RU + i_];                                                       \
            frag_from(af[j], (j < nkb_) ? u_ : make_uint4(0, 0, 0, 0));                                            \
        }                                                                                                          \
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");                                                     \
        __builtin_amdgcn_wave_barrier();                                                                           \
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");                                                     \
    }
#define HIVIS_STAGE(ps, nx, do_ssq) HIVIS_STAGE_FROM(ps, araw, graw, do_ssq, if ((nx) >= 0) HIVIS_LOAD_RAW(nx))
    // Tokens = greedy tokens of the LM-head phase before this one (fusion FC with ph.tok == null): every wavefront
    // reduces that phase's candidates itself (lowest index wins ties); workgroup 0 also stores them.
    const bool cand_tokens = ((EPI == FEPI_ADDVEC && (ph.emb != nullptr || ph.add_rows != nullptr)) || TAB) && ph.tok == nullptr;
    // the token of THIS thread's epilogue row (all of a thread's epilogue slots serve one row), for the table form
    const int row_e = min(RPL * (((int)threadIdx.x / RPL & 63) >> 4) + (int)threadIdx.x % RPL, M - 1);
    int tok_e = 0;
    if (EPI == FEPI_ADDVEC && ph.add_rows != nullptr && ph.tok != nullptr)
        tok_e = __hip_atomic_load(&ph.tok[(row_e / pp.m) * ph.tok_sseq + (row_e % pp.m) * ph.tok_srow], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    auto reduce_tokens = [&]() {
        for (int r = 0; r < M; ++r) {
            float bv = -INFINITY; int bi = 0x7FFFFFFF;
            for (int w = lane; w < ph.ncand; w += 64) {
                const float v = ph.pm[(size_t)r * ph.ncand + w]; const int i = ph.pi[(size_t)r * ph.ncand + w];
                if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                const float ov = __shfl_xor(bv, o, 64); const int oi = __shfl_xor(bi, o, 64);
                if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
            }
            if (blockIdx.x == 0 && threadIdx.x == 0) {
                if (pp.bad && (unsigned)bi >= (unsigned)pp.V) st_wt(pp.bad, 1);
                st_wt(&ph.tok_out[(r / pp.m) * ph.o_sseq + (r % pp.m) * ph.o_srow], clamp_token(bi, pp.V));
            }
#pragma unroll
            for (int q = 0; q < QM; ++q) if (row0 + q * RS == r) tokr[q] = bi;
            if (r == row_e) tok_e = bi;
        }
    };
    // The tokens come first: a tiny model's first K pass already reads embedding rows, and for the others requesting the
    // candidates behind the first weight units (they return in order) was measured 0.8 us per draft step slower.
    if (cand_tokens) reduce_tokens();
    HIVIS_MARK(0)
    // The activation rows are requested BEFORE the first weight units: loads return in order, so rows requested
    // after 16 KiB of weights per wavefront could not be staged until those weights had arrived from HBM.
    HIVIS_LOAD_RAW(0)
    // nothing prefetched for this phase (always the case with one launch per phase): request its first two units now
    if (!head_valid) HIVIS_FIRST_UNITS(W, kblks, t_begin, ntl, npass)
    head_valid = false;
    const bool wb1_first = wb1_valid;       // wb1 already holds the second unit of the phase
    wb1_valid = false;

    for (int tg = t_begin; tg < t_end; tg += G) {
        const int ng = min(G, t_end - tg);
        const bool first = (tg == t_begin);
        f32x4_t acc[G];
#pragma unroll
        for (int g = 0; g < G; ++g) acc[g] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        afrag_t af[KBW];
        if constexpr (SINGLE) {
            // ---- every workgroup owns at most one tile.  The K passes go in pairs, and everything the NEXT pair needs
            //      (two weight units, the rows of both passes) is requested in one go after the pair's arithmetic: the
            //      compiler waits for "all loads" wherever one is used (conditional loads defeat its counting), so what
            //      matters is how much is in flight per wait: two units here.  With one unit requested per pass every
            //      pass paid a memory round trip for 8 KiB per wavefront and the kernel was latency-bound.
            if (npass > 1) HIVIS_LOAD_RAW_TO(1, araw2, graw2)
            if (!wb1_first && npass > 1) issue_unit(wb1, W, kblks, tg, unit_kb0<NW, KBW>(kblks, 1, wave), unit_nkb<NW, KBW>(kblks, 1, wave), lane);
            for (int pass = 0; pass < npass; pass += 2) {
                HIVIS_STAGE_FROM(pass, araw, graw, true, )
                if (pass == 0) { HIVIS_MARK(1) }
#pragma unroll
                for (int j = 0; j < U; ++j) mfma_block(acc[0], af[j], head[j]);
                if (pass + 1 < npass) {
                    HIVIS_STAGE_FROM(pass + 1, araw2, graw2, true, )
#pragma unroll
                    for (int j = 0; j < U; ++j) mfma_block(acc[0], af[j], wb1[j]);
                }
                if (pass + 2 < npass) {
                    HIVIS_LOAD_RAW_TO(pass + 2, araw, graw)
                    issue_unit(head, W, kblks, tg, unit_kb0<NW, KBW>(kblks, pass + 2, wave), unit_nkb<NW, KBW>(kblks, pass + 2, wave), lane);
                }
                if (pass + 3 < npass) {
                    HIVIS_LOAD_RAW_TO(pass + 3, araw2, graw2)
                    issue_unit(wb1, W, kblks, tg, unit_kb0<NW, KBW>(kblks, pass + 3, wave), unit_nkb<NW, KBW>(kblks, pass + 3, wave), lane);
                }
            }
        } else {
            for (int pass = 0; pass < npass; ++pass) {
                const int kb0 = unit_kb0<NW, KBW>(kblks, pass, wave);
                const int nkb = unit_nkb<NW, KBW>(kblks, pass, wave);
                // where the prefetch chain goes after the last unit of this (tile group, pass)
                int ntile = tg, npass_i = pass + 1, ntiles2 = ng; bool nvalid = true;
                if (pass + 1 < npass) { }
                else if (tg + G < t_end) { ntile = tg + G; npass_i = 0; ntiles2 = t_end - ntile; }
                else nvalid = false;     // the next phase's first units are requested after this phase's stores (see the end)
                const int nkb0 = unit_kb0<NW, KBW>(kblks, npass_i, wave);
                const int nnkb = unit_nkb<NW, KBW>(kblks, npass_i, wave);
                const bool have_wb1 = (first && pass == 0) ? wb1_first : wb1_valid;
                wb1_valid = false;
                HIVIS_STAGE(pass, (pass + 1 < npass) ? pass + 1 : ((tg + G < t_end) ? 0 : -1), first)
                if (first && pass == 0) { HIVIS_MARK(1) }
                // ---- stream the tiles of the group, two at a time
#pragma unroll
                for (int g0 = 0; g0 < G; g0 += 2) {
                    if (g0 < ng) {
                        if (g0 + 1 < ng && !(g0 == 0 && have_wb1)) issue_unit(wb1, W, kblks, tg + g0 + 1, kb0, nkb, lane);
#pragma unroll
                        for (int j = 0; j < U; ++j) mfma_block(acc[g0], af[j], head[j]);
                        if (g0 + 2 < ng) issue_unit(head, W, kblks, tg + g0 + 2, kb0, nkb, lane);
                        else if (nvalid) issue_unit(head, W, kblks, ntile, nkb0, nnkb, lane);
                        if (g0 + 1 < ng) {
#pragma unroll
                            for (int j = 0; j < U; ++j) mfma_block(acc[g0 + 1], af[j], wb1[j]);
                        }
                    }
                }
                // second unit of the next (tile group, pass): its registers are free now
                if (nvalid && ntiles2 >= 2) { issue_unit(wb1, W, kblks, ntile + 1, nkb0, nnkb, lane); wb1_valid = true; }
                if (first && pass == 0) { HIVIS_MARK(2) }
            }
        }
        if (first) { HIVIS_MARK(3) }
        // operands of this thread's epilogue slots, requested now so that they arrive during the reduction
        float epi_a[SLOTS], epi_b[SLOTS];
#pragma unroll
        for (int sl = 0; sl < SLOTS; ++sl) {
            epi_a[sl] = 0.f; epi_b[sl] = 0.f;
            const int idx = threadIdx.x + sl * NT, r = idx % RPL, ln = (idx / RPL) & 63, g = idx / (RPL * 64);
            const int row = min(RPL * (ln >> 4) + r, M - 1), col = min((tg + g) * 16 + (ln & 15), N - 1);
            if (epi == FEPI_ADD_TO) epi_a[sl] = ph.R[(size_t)row * ph.ldr + col];
            else if (epi == FEPI_ADDVEC && ph.add_rows != nullptr) epi_a[sl] = ph.add_rows[(size_t)clamp_token(tok_e, pp.V) * N + col];
            else if (epi == FEPI_QKV) {
                const int p2 = (col % pp.hd) >> 1;
                const int seq_ = row / pp.m;
                const int pos_ = min((ph.att.nbase > 0 ? ph.att.base_val[seq_] : ph.base[seq_]) + ph.offset + row % pp.m, ph.maxL - 1);
                const float2 cs_ = *reinterpret_cast<const float2*>(ph.rope + ((size_t)pos_ * (pp.hd / 2) + p2) * 2);
                epi_a[sl] = cs_.x; epi_b[sl] = cs_.y;
            }
        }
        // ---- cross-wave reduction
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float* dst = red + ((size_t)(wave * G + g) * 64 + lane) * RPL;
            if constexpr (RPL == 2) {
                dst[0] = acc[g][0] + acc[g][2];
                dst[1] = acc[g][1] + acc[g][3];
            } else {
                dst[0] = acc[g][0]; dst[1] = acc[g][1]; dst[2] = acc[g][2]; dst[3] = acc[g][3];
            }
        }
        if (first && gain) {
            // this wavefront's share of every row's sum of squares (its lanes with row0 == h hold rows h + q*RS)
#pragma unroll
            for (int q = 0; q < QM; ++q) {
#pragma unroll
                for (int h = 0; h < RS; ++h) {
                    const float s = wave_sum(row0 == h ? ssq_acc[q] : 0.f);
                    if (lane == 0) ssq_w[wave * 16 + q * RS + h] = s;
                }
            }
        }
        lds_barrier();
        for (int idx = threadIdx.x; idx < TILE; idx += NT) {
            float s = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) s += red[(size_t)w * TILE + idx];
            tile[idx] = s;
        }
        if (first && gain && (int)threadIdx.x < M) {
            const int r = threadIdx.x;
            float s = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) s += ssq_w[w * 16 + r];
            inv_rms[r] = 1.0f / sqrtf(s / (float)K + pp.eps);
        }
        lds_barrier();
        if (first) { HIVIS_MARK(4) }
        // ---- epilogue on the reduced tiles
#pragma unroll
        for (int sl = 0; sl < SLOTS; ++sl) {
            const int idx = threadIdx.x + sl * NT;
            const int r = idx % RPL;
            const int ln = (idx / RPL) & 63;
            const int g = idx / (RPL * 64);
            const int row = RPL * (ln >> 4) + r;
            const int cl = ln & 15;
            const int col = (tg + g) * 16 + cl;
            if (g >= ng || row >= M) continue;
            const float sc = gain ? inv_rms[row] : 1.0f;
            const float v = tile[idx] * sc;
            switch (epi) {
            case FEPI_STORE: st_wt(&ph.Y[(size_t)row * ph.ldy + col], v); break;
            case FEPI_ADD_TO: st_wt(&ph.Y[(size_t)row * ph.ldy + col], epi_a[sl] + v); break;
            case FEPI_ADDVEC: st_wt(&ph.Y[(size_t)row * ph.ldy + col], v + to_f32(((const WT*)ph.vec)[(size_t)ph.vec_idx * N + col]) + epi_a[sl]); break;
            case FEPI_LOGITS:
                if (col < pp.V) {
                    st_wt(&ph.Y[(size_t)row * ph.ldy + col], v);
                    if (v > best_v || (v == best_v && col < best_i)) { best_v = v; best_i = col; }
                } else {
                    st_wt(&ph.Y2[(size_t)row * ph.ldy2 + (col - pp.V)], v + to_f32(((const WT*)ph.vec)[(size_t)ph.vec_idx * (N - pp.V) + (col - pp.V)]));
                }
                break;
            case FEPI_SILU:
                if (cl < 8) {
                    const float up = tile[idx + 8 * RPL] * sc;
                    st_wt(&ph.Y[(size_t)row * ph.ldy + (tg + g) * 8 + cl], v / (1.0f + expf(-v)) * up);
                }
                break;
            case FEPI_QKV: {
                // every even column handles the pair (col, col+1): a rotary pair of q or k, or two v elements
                const int qd = pp.Hq * pp.hd, kd = pp.Hkv * pp.hd, hd = pp.hd;
                const int seq = row / pp.m;
                const int pos = min((ph.att.nbase > 0 ? ph.att.base_val[seq] : ph.base[seq]) + ph.offset + row % pp.m, ph.maxL - 1);
                if ((cl & 1) == 0) {
                    float x1 = v, x2 = tile[idx + RPL] * sc;
                    if (ph.bias) { x1 += ph.bias[col]; x2 += ph.bias[col + 1]; }
                    if (col < qd + kd) {
                        const float c = epi_a[sl], s = epi_b[sl];
                        const float y1 = x1 * c - x2 * s, y2 = x2 * c + x1 * s;
                        if (col < qd) {
                            st_wt_pair(&ph.Y[(size_t)row * ph.ldy + col], y1, y2);
                        } else {
                            const int c2 = col - qd;
                            st_wt_kv_pair((KT*)ph.kc + (((size_t)seq * pp.Hkv + c2 / hd) * ph.maxL + pos) * hd * KVWidth<KT>::W, hd, c2 % hd, y1, y2);
                        }
                    } else {
                        const int c2 = col - qd - kd;
                        st_wt_kv_pair((KT*)ph.vc + (((size_t)seq * pp.Hkv + c2 / hd) * ph.maxL + pos) * hd * KVWidth<KT>::W, hd, c2 % hd, x1, x2);
                    }
                }
            } break;
            }
        }
    }
#undef HIVIS_LOAD_RAW
#undef HIVIS_LOAD_RAW_TO
#undef HIVIS_STAGE
#undef HIVIS_STAGE_FROM
    HIVIS_MARK(5)
    if (epi == FEPI_LOGITS) {
        // per-row candidate of this workgroup: the threads of one row meet through LDS
        lds_barrier();
        float* cv = red; int* ci = (int*)(red + NT);
        cv[threadIdx.x] = best_v; ci[threadIdx.x] = best_i;
        lds_barrier();
        // one wavefront per row: lanes scan the threads that serve that row, then a shuffle reduction (lowest index wins ties)
        for (int row = wave; row < ROWS; row += NW) {
            float bv = -INFINITY; int bi = 0x7FFFFFFF;
            for (int t = lane; t < NT; t += 64) {
                const int r = t % RPL, ln = (t / RPL) & 63;
                if (RPL * (ln >> 4) + r != row) continue;
                const float v = cv[t]; const int i = ci[t];
                if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                const float ov = __shfl_xor(bv, o, 64); const int oi = __shfl_xor(bi, o, 64);
                if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
            }
            if (lane == 0 && row < M) { st_wt(&ph.pm[(size_t)row * gridDim.x + blockIdx.x], bv); st_wt(&ph.pi[(size_t)row * gridDim.x + blockIdx.x], bi); }
        }
        if (ph.cnt) lm_head_elect(ph, pp, reinterpret_cast<int*>(inv_rms));
    }
    // The stores of this phase must be acknowledged before the workgroup arrives at the grid barrier, and the
    // only wait available (vmcnt) also covers loads: so first drain, THEN request the first two units of the next
    // GEMM phase, which stay in flight across the barrier (persistent mode).
    wait_vmem();
    HIVIS_MARK(6)
#undef HIVIS_MARK
    if (n_has) HIVIS_FIRST_UNITS(ph.next_W, n_kblks, n_tile, n_tend - n_tile, n_npass)
#undef HIVIS_FIRST_UNITS
}

// ---- attention phase ---------------------------------------------------------------------------------
// One (item, split) per workgroup: item = (sequence, kv head, block of query heads, block of rows) with at most
// FUSED_RMAX (head,row) pairs; split = a contiguous range of keys.  Wavefront w takes keys 16w..16w+15 of every
// block of 16*NW keys.  K rows are read as [16 keys][4 quarters] (each lane 1/4 of a key row, a wavefront reads
// 16 whole rows = one contiguous span), V rows as [keys][16-byte chunks]; all loads of a block are issued before
// any arithmetic.  Each wavefront keeps its own running (max, sum, accumulator); the NW partials are merged
// through LDS and ONE partial per workgroup goes to memory: ws[(item*nsplit + split)][RM][HD + 2].
__host__ __device__ constexpr size_t fused_attn_lds_floats(int hd, int nw, int rm) {
    return (size_t)rm * hd + (size_t)nw * rm * 16 + (size_t)nw * rm * (hd + 2);
}

#define HIVIS_AMARK(k) if (marks && blockIdx.x == 0 && threadIdx.x == 0) marks[k] = wall_clock64();

// Merge of the key-split partials of one item (pbase: [nsplit][RM][HD + 2], each row = weighted value sums, running
// maximum, sum of weights) in split order, by the whole workgroup; writes the attention rows.  Every load is
// requested before anything waits (the partials come from memory, a round trip of more than a microsecond: a loop
// that loads split after split spent 8-10 us here), which is why the split count is bounded at compile time.
// wl: LDS scratch of 3 * ATTN_MAX_SPLITS * RM floats that nothing else uses until the routine returns.
constexpr int ATTN_MAX_SPLITS = 16;
template <int HD, int RM, int MAXS>
__device__ __forceinline__ void attn_merge_splits_n(const float* __restrict__ pbase, int nsplit, int R, int ni, int head0, int i0, int sl,
                                                    const AttnShape& sh, float* __restrict__ wl, float* __restrict__ att_out, int ldo) {
    constexpr int PER = (RM * HD + FUSED_NT - 1) / FUSED_NT;       // output elements per thread
    static_assert(MAXS * RM <= FUSED_NT, "one thread per (split, row) pair of statistics");
    float* wm = wl; float* wsum = wl + MAXS * RM; float* ww = wl + 2 * MAXS * RM;
    float v[PER][MAXS];
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        const int idx = threadIdx.x + e * FUSED_NT;
        const int r = min(idx / HD, R - 1), c = idx % HD;
#pragma unroll
        for (int sp = 0; sp < MAXS; ++sp) v[e][sp] = ld_agent(&pbase[((size_t)min(sp, nsplit - 1) * RM + r) * (HD + 2) + c]);
    }
    if ((int)threadIdx.x < MAXS * RM) {
        const int sp = threadIdx.x / RM, r = threadIdx.x % RM;
        const float* p = pbase + ((size_t)min(sp, nsplit - 1) * RM + min(r, R - 1)) * (HD + 2);
        const float ms = ld_agent(&p[HD]), ls = ld_agent(&p[HD + 1]);
        const bool live = sp < nsplit && r < R;
        wm[threadIdx.x] = live ? ms : -INFINITY; wsum[threadIdx.x] = live ? ls : 0.f;
    }
    lds_barrier();
    if ((int)threadIdx.x < MAXS * RM) {
        const int sp = threadIdx.x / RM, r = threadIdx.x % RM;
        float mx = -INFINITY;
#pragma unroll
        for (int s2 = 0; s2 < MAXS; ++s2) mx = fmaxf(mx, wm[s2 * RM + r]);
        float den = 0.f;
#pragma unroll
        for (int s2 = 0; s2 < MAXS; ++s2) {
            const float m2 = wm[s2 * RM + r];
            if (m2 != -INFINITY) den += wsum[s2 * RM + r] * __expf(m2 - mx);
        }
        const float ms = wm[threadIdx.x];
        ww[threadIdx.x] = (ms == -INFINITY) ? 0.f : __expf(ms - mx) / den;
    }
    lds_barrier();
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        const int idx = threadIdx.x + e * FUSED_NT;
        const int r = idx / HD, c = idx % HD;
        if (r < R) {
            float o = 0.f;
#pragma unroll
            for (int sp = 0; sp < MAXS; ++sp) o += ww[sp * RM + r] * v[e][sp];
            const int hh = head0 + r / ni, i = i0 + r % ni;
            st_wt(&att_out[(size_t)(sl * sh.m + i) * ldo + (size_t)hh * HD + c], o);
        }
    }
    lds_barrier();
}
// (the loads are unrolled to a compile-time bound: the smallest of 4 / 8 / 16 that holds the split count)
template <int HD, int RM>
__device__ __forceinline__ void attn_merge_splits(const float* __restrict__ pbase, int nsplit, int R, int ni, int head0, int i0, int sl,
                                                  const AttnShape& sh, float* __restrict__ wl, float* __restrict__ att_out, int ldo) {
    if (nsplit <= 4) attn_merge_splits_n<HD, RM, 4>(pbase, nsplit, R, ni, head0, i0, sl, sh, wl, att_out, ldo);
    else if (nsplit <= 8) attn_merge_splits_n<HD, RM, 8>(pbase, nsplit, R, ni, head0, i0, sl, sh, wl, att_out, ldo);
    else attn_merge_splits_n<HD, RM, ATTN_MAX_SPLITS>(pbase, nsplit, R, ni, head0, i0, sl, sh, wl, att_out, ldo);
}
// Tail shared by the attention variants: the NW per-wavefront partials in mrg ([NW][RM][HD + 2]: weighted value
// sums, running maximum, sum of weights) are merged in wavefront order; with one key split the attention rows are
// written directly, otherwise ONE partial of the workgroup goes to ws for the merge phase (or, when cnt is given,
// the workgroup that completes the item merges all of its partials).
template <int HD, int RM>
__device__ __forceinline__ void attn_wg_finish(const float* __restrict__ mrg, int* __restrict__ flag, const AttnShape& sh, int item_id, int split,
                                               int R, int ni, int head0, int i0, int sl, float* __restrict__ ws, int* __restrict__ cnt,
                                               float* __restrict__ att_out, int ldo, unsigned long long* marks, uint4* __restrict__ frag_out = nullptr) {
    constexpr int NW = FUSED_NW;
    lds_barrier();
    HIVIS_AMARK(4)
    if (sh.nsplit == 1 && frag_out != nullptr) {
        // the attention rows go straight out as A fragments of the O projection (K = ldo, bf16 hi/lo split, layout of
        // pack_afrag_kernel): 8 consecutive dims of one row per thread and trip
        for (int idx = threadIdx.x; idx < R * (HD / 8); idx += FUSED_NT) {
            const int r = idx / (HD / 8), c0 = (idx % (HD / 8)) * 8;
            float mx = -INFINITY;
#pragma unroll
            for (int w = 0; w < NW; ++w) mx = fmaxf(mx, mrg[(w * RM + r) * (HD + 2) + HD]);
            float num[8], den = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) num[e] = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                const float mw = mrg[(w * RM + r) * (HD + 2) + HD];
                if (mw != -INFINITY) {
                    const float ew = __expf(mw - mx);
#pragma unroll
                    for (int e = 0; e < 8; ++e) num[e] += mrg[(w * RM + r) * (HD + 2) + c0 + e] * ew;
                    den += mrg[(w * RM + r) * (HD + 2) + HD + 1] * ew;
                }
            }
            float y[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) y[e] = num[e] / den;
            const int hh = head0 + r / ni, i = i0 + r % ni;
            store_afrag8(frag_out, ldo / 32, sl * sh.m + i, hh * HD + c0, y, false);
        }
        lds_barrier();
        return;
    }
    if (sh.nsplit == 1) {
        // the whole key range was handled here: merge the NW partials and write the attention rows directly
        for (int idx = threadIdx.x; idx < R * HD; idx += FUSED_NT) {
            const int r = idx / HD, c = idx % HD;
            float mx = -INFINITY;
#pragma unroll
            for (int w = 0; w < NW; ++w) mx = fmaxf(mx, mrg[(w * RM + r) * (HD + 2) + HD]);
            float num = 0.f, den = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                const float mw = mrg[(w * RM + r) * (HD + 2) + HD];
                if (mw != -INFINITY) {
                    const float e = __expf(mw - mx);
                    num += mrg[(w * RM + r) * (HD + 2) + c] * e; den += mrg[(w * RM + r) * (HD + 2) + HD + 1] * e;
                }
            }
            const int hh = head0 + r / ni, i = i0 + r % ni;
            st_wt(&att_out[(size_t)(sl * sh.m + i) * ldo + (size_t)hh * HD + c], num / den);
        }
        lds_barrier();
        return;
    }
    // ---- merge the NW partials (fixed order) and write ONE partial of this workgroup
    float* out = ws + ((size_t)item_id * sh.nsplit + split) * RM * (HD + 2);
    for (int idx = threadIdx.x; idx < R * (HD + 2); idx += FUSED_NT) {
        const int r = idx / (HD + 2), c = idx % (HD + 2);
        float mx = -INFINITY;
#pragma unroll
        for (int w = 0; w < NW; ++w) mx = fmaxf(mx, mrg[(w * RM + r) * (HD + 2) + HD]);
        float v;
        if (c == HD) v = mx;
        else {
            v = 0.f;
            const int cc = (c == HD + 1) ? HD + 1 : c;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                const float mw = mrg[(w * RM + r) * (HD + 2) + HD];
                if (mw != -INFINITY) v += mrg[(w * RM + r) * (HD + 2) + cc] * __expf(mw - mx);
            }
        }
        st_wt(&out[r * (HD + 2) + c], v);
    }
    HIVIS_AMARK(5)
    if (cnt == nullptr) { lds_barrier(); return; }        // the partials are merged by a separate phase
    // ---- the workgroup whose partial completes the item merges all of them (no merge launch, no grid barrier):
    // partial stored -> stores complete -> arrive on the item's counter -> the last arriver reads the nsplit partials.
    // Every access involved is an agent-scope atomic (write-through stores, the counter, the loads of the merge), and
    // the stores have completed (vmcnt) before the arrival is issued: that orders them for every XCD without writing
    // back or invalidating an L2.  (Measured with the fence pair as well: 1.8 us more per layer; parity was identical
    // with the splits of an item on one XCD and spread over all of them.)
    wait_vmem();
    lds_barrier();
    if (threadIdx.x == 0) {
        if (!(sh.flags & 1)) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        flag[0] = __hip_atomic_fetch_add(&cnt[item_id], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    lds_barrier();
    const bool last = flag[0] == sh.nsplit - 1;
    if (last) {
        if (!(sh.flags & 1)) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        const float* pbase = ws + (size_t)item_id * sh.nsplit * RM * (HD + 2);
        // (the wavefront partials in mrg are dead since the barrier before the arrival: their space is the scratch)
        attn_merge_splits<HD, RM>(pbase, sh.nsplit, R, ni, head0, i0, sl, sh, const_cast<float*>(mrg), att_out, ldo);
        if (threadIdx.x == 0) st_wt(&cnt[item_id], 0);
    }
    lds_barrier();
}

// ---- attention on the matrix cores (half-precision caches) ---------------------------------------------
// Same work split as attn_wg_partial, but both contractions run as MFMA with the (head,row) pairs as the 16-wide
// N dimension, so the queries live in registers instead of LDS and a 16-key tile costs a few dozen MFMA instead of
// ~500 scalar FMAs:
//   S^T[key][row]  = K[key][:] . Q^T          mfma 16x16x32 f16; A = 16 cached key rows (lane: key lane%16, 8 dims at
//                                             32 ks + 8 (lane/16)), B = q*scale
//   O^T[dim][row] += V^T[dim][key] . P^T      mfma 16x16x16 f16; B = the probabilities exactly where the first product
//                                             left them (lane: row lane%16, keys 4 (lane/16) + r); A = V^T, which needs
//                                             4 keys of one dim per lane: the V tile goes through LDS row-major and
//                                             comes back through the transposing LDS read
// Every operand is a pair of halves, hi + lo (the cache stores K and V that way, see KVType; q*scale and the
// probabilities are split in registers), and each product is three MFMA: hi.hi + lo.hi + hi.lo (lo.lo is below
// fp32 resolution).  That keeps ~22 bits in all four operands at 3x the (small) MFMA work.
// The running maximum / sum / rescale are per lane (row = lane%16 everywhere), only the maximum crosses lanes.
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));

// LDS (floats): per-wavefront K and V tiles of 16 keys (a row = hi | lo halves = 4 hd bytes, plus padding); the
// per-wavefront partials [nw][rm][hd + 2] reuse the tile space after the key loop; 16 words for the election flag.
__host__ __device__ constexpr size_t fused_attn_mfma_lds_floats(int hd, int nw, int rm) {
    const size_t tiles = ((size_t)nw * 16 * (hd * 4 + 32) + (size_t)nw * 16 * (hd * 4 + 16)) / 4;
    const size_t mrg = (size_t)nw * rm * (hd + 2);
    return (tiles > mrg ? tiles : mrg) + 16;
}

template <int HD, int RM>
__device__ __forceinline__ void attn_wg_mfma(const float* __restrict__ q, const f16_t* __restrict__ kc, const f16_t* __restrict__ vc,
                                             const int* __restrict__ base, const AttnShape& sh, int item_id, int split,
                                             float* __restrict__ lds, float* __restrict__ ws, int* __restrict__ cnt,
                                             float* __restrict__ att_out, int ldo, unsigned long long* marks = nullptr,
                                             uint4* __restrict__ frag_out = nullptr) {
    HIVIS_AMARK(0)
    static_assert(RM <= 16 && HD % 32 == 0, "rows are the 16-wide MFMA dimension");
    constexpr int NW = FUSED_NW;
    constexpr int HALFB = HD * 2;                  // bytes of the hi (or lo) halves of one cached row
    constexpr int ROWB = HD * 4;                   // bytes of one cached row: hi halves, then lo halves
    constexpr int KS = HD / 32;                    // k-steps of the score product
    constexpr int NB = HD / 16;                    // 16-dim blocks of the value product
    constexpr int NCH = ROWB / 16;                 // 16-byte chunks per cached row
    constexpr int KPI = 64 / NCH;                  // cached rows per load instruction
    constexpr int VT = 16 / KPI;                   // load instructions per 16 keys
    static_assert(NCH <= 64 && KPI >= 1, "row too long for this mapping");
    // row stride of the V tile in LDS: 32 bytes more than the row, so the 4 rows a 16-lane group transposes
    // start 8 banks apart and the 64-bit transposing reads of a half wavefront touch every bank twice (the minimum)
    constexpr int VSTRIDE = ROWB + 32;
    // K tile in LDS: 16 bytes more than the row, so the 8 lanes a 128-bit read serves per clock hit 32 different banks
    constexpr int KSTRIDE = ROWB + 16;
    char* vt_all = reinterpret_cast<char*>(lds);                    // [NW][16 keys][VSTRIDE]
    char* kt_all = vt_all + NW * 16 * VSTRIDE;                      // [NW][16 keys][KSTRIDE]
    float* mrg = lds;                                               // [NW][RM][HD + 2] per-wavefront partials: same space, after the loop
    int* flag = reinterpret_cast<int*>(lds + fused_attn_mfma_lds_floats(HD, NW, RM) - 16);

    int item = item_id;
    const int rblk = item % sh.n_rblk; item /= sh.n_rblk;
    const int hblk = item % sh.n_hblk; item /= sh.n_hblk;
    const int kvh = item % sh.Hkv;
    const int sl = item / sh.Hkv;
    const int seq = sh.seq0 + sl;
    const int group = sh.Hq / sh.Hkv;
    const int h0 = hblk * sh.gh, nh = min(sh.gh, group - h0);
    const int i0 = rblk * sh.mi, ni = min(sh.mi, sh.m - i0);
    const int R = nh * ni;
    const int pos0 = (sh.nbase > 0 ? sh.base_val[sl] : base[seq]) + sh.offset;
    const int nkeys = min(pos0 + i0 + ni, sh.maxL);
    const int cs = ((nkeys + sh.nsplit - 1) / sh.nsplit + 15) & ~15;        // keys per split, multiple of 16
    const int k0 = split * cs, k1 = min(nkeys, k0 + cs);
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wavefront index as a scalar: branches on it are uniform
    const int n16 = lane & 15, g = lane >> 4;
    const int vks = lane / NCH, vdc = lane % NCH;

    const char* kbase = reinterpret_cast<const char*>(kc) + ((size_t)seq * sh.Hkv + kvh) * sh.maxL * ROWB;
    const char* vbase = reinterpret_cast<const char*>(vc) + ((size_t)seq * sh.Hkv + kvh) * sh.maxL * ROWB;
    char* vt = vt_all + wave * 16 * VSTRIDE;
    char* kt = kt_all + wave * 16 * KSTRIDE;

    // all loads of this wavefront's 16 keys starting at kb_ (rows clamped into the range; masked later).  K and V rows
    // are both read as whole rows (1 KiB contiguous per instruction): reading K directly in fragment order (16 rows x
    // 64 bytes per instruction) costs the address coalescer 4x the cycles and bounded the loop.
    // One tile ahead is enough (two in flight measured slower).
    u32x4_t knext[VT], vnext[VT];
#define HIVIS_ATTN_LOADS(kb_)                                                                                      \
    {                                                                                                              \
        _Pragma("unroll") for (int t = 0; t < VT; ++t) {                                                           \
            const size_t off_ = (size_t)min((kb_) + t * KPI + vks, nkeys - 1) * ROWB + vdc * 16;                   \
            knext[t] = *reinterpret_cast<const u32x4_t*>(kbase + off_);                                            \
            vnext[t] = *reinterpret_cast<const u32x4_t*>(vbase + off_);                                            \
        }                                                                                                          \
    }
    if (k0 + 16 * wave < k1) HIVIS_ATTN_LOADS(k0 + 16 * wave)
    HIVIS_AMARK(1)

    // B operand of the score product: q[row lane%16][32 ks + 8 (lane/16) .. +8] * scale as hi + lo halves; rows >= R are zero
    f16x8_t qh[KS], ql[KS];
    {
        const int rq = min(n16, R - 1);
        const int hh = kvh * group + h0 + rq / ni, i = i0 + rq % ni;
        const float* qrow = q + (size_t)(sl * sh.m + i) * sh.ldq + (size_t)hh * HD + g * 8;
        const float scale = (n16 < R) ? rsqrtf((float)HD) : 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const float4 a = *reinterpret_cast<const float4*>(qrow + ks * 32);
            const float4 b = *reinterpret_cast<const float4*>(qrow + ks * 32 + 4);
            const float x[8] = {a.x * scale, a.y * scale, a.z * scale, a.w * scale, b.x * scale, b.y * scale, b.z * scale, b.w * scale};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const _Float16 hi = (_Float16)fminf(fmaxf(x[e], -65504.f), 65504.f);
                qh[ks][e] = hi; ql[ks][e] = (_Float16)(x[e] - (float)hi);
            }
        }
    }
    const int qpos = (n16 < R) ? pos0 + i0 + n16 % ni : 0x7FFFFFFF;     // causal limit of this lane's row
    const bool tree = sh.tmask != nullptr;                              // rows of a draft tree: ancestor mask instead
    const unsigned long long tmk = (tree && n16 < R) ? sh.tmask[sl * sh.m + i0 + n16 % ni] : ~0ull;
    const int tb = pos0 - sh.offset;
    HIVIS_AMARK(2)

    float mrun = -INFINITY, lrun = 0.f;
    f32x4_t acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    for (int kb = k0 + 16 * wave; kb < k1; kb += 16 * NW) {
        u32x4_t vraw[VT];
        // ---- both tiles -> LDS (row-major); the K fragments come back as plain 128-bit reads (key lane%16,
        //      dims 32 ks + 8 (lane/16) .. +8, hi halves and HALFB further the lo halves), the V^T fragments through
        //      the transposing read further down
#pragma unroll
        for (int t = 0; t < VT; ++t) {
            *reinterpret_cast<u32x4_t*>(kt + (t * KPI + vks) * KSTRIDE + vdc * 16) = knext[t];
            vraw[t] = vnext[t];
        }
        if (kb + 16 * NW < k1) HIVIS_ATTN_LOADS(kb + 16 * NW)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        // ---- scores, transposed: this lane gets keys kb + 4 (lane/16) + r of row lane%16
        f32x4_t st = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const f16x8_t kh = *reinterpret_cast<const f16x8_t*>(kt + n16 * KSTRIDE + ks * 64 + g * 16);
            const f16x8_t kl = *reinterpret_cast<const f16x8_t*>(kt + n16 * KSTRIDE + HALFB + ks * 64 + g * 16);
            st = __builtin_amdgcn_mfma_f32_16x16x32_f16(kl, qh[ks], st, 0, 0, 0);
            st = __builtin_amdgcn_mfma_f32_16x16x32_f16(kh, ql[ks], st, 0, 0, 0);
            st = __builtin_amdgcn_mfma_f32_16x16x32_f16(kh, qh[ks], st, 0, 0, 0);
        }
        float sv[4], tmax = -INFINITY;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int key = kb + 4 * g + r;
            sv[r] = (key < k1 && attn_visible(tree, key, qpos, tmk, tb)) ? st[r] : -INFINITY;
            tmax = fmaxf(tmax, sv[r]);
        }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
        const float mnew = fmaxf(mrun, tmax);
        const float mref = (mnew == -INFINITY) ? 0.f : mnew;       // nothing visible yet: every exponential below is 0
        const float alpha = __expf(mrun - mref);
        float p[4], psum = 0.f;
#pragma unroll
        for (int r = 0; r < 4; ++r) { p[r] = __expf(sv[r] - mref); psum += p[r]; }
        mrun = mnew;
        lrun = lrun * alpha + psum;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[nb][r] *= alpha;
        }
        f16x4_t pbh, pbl;
#pragma unroll
        for (int r = 0; r < 4; ++r) { pbh[r] = (_Float16)p[r]; pbl[r] = (_Float16)(p[r] - (float)pbh[r]); }
        // ---- V tile -> LDS (row-major), back as V^T fragments, O^T += V^T . P^T
#pragma unroll
        for (int t = 0; t < VT; ++t) *reinterpret_cast<u32x4_t*>(vt + (t * KPI + vks) * VSTRIDE + vdc * 16) = vraw[t];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            // transposing read: within a 16-lane group, lane i element e comes from the address of lane 4e + i/4,
            // its element i%4; so lane s points at key 4 (lane/16) + s/4, dims 16 nb + 4 (s%4) .. +3
            const char* src = vt + (4 * g + (n16 >> 2)) * VSTRIDE + (nb * 16 + 4 * (n16 & 3)) * 2;
            const s16x4_t rh = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(src));
            const s16x4_t rl = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(src + HALFB));
            acc[nb] = __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4_t, rl), pbh, acc[nb], 0, 0, 0);
            acc[nb] = __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4_t, rh), pbl, acc[nb], 0, 0, 0);
            acc[nb] = __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4_t, rh), pbh, acc[nb], 0, 0, 0);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
#undef HIVIS_ATTN_LOADS
    HIVIS_AMARK(3)
    // ---- per-wavefront partial -> LDS: this lane holds dims 16 nb + 4 (lane/16) + r of row lane%16.  The partials
    //      reuse the tile space, so every wavefront must have left its key loop first.
    lds_barrier();
    float lsum = lrun;
    lsum += __shfl_xor(lsum, 16, 64);
    lsum += __shfl_xor(lsum, 32, 64);
    if (n16 < R) {
        float* mr = mrg + (wave * RM + n16) * (HD + 2);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
            for (int r = 0; r < 4; ++r) mr[nb * 16 + 4 * g + r] = acc[nb][r];
        }
        if (g == 0) { mr[HD] = mrun; mr[HD + 1] = lsum; }
    }
    attn_wg_finish<HD, RM>(mrg, flag, sh, item_id, split, R, ni, kvh * group + h0, i0, sl, ws, cnt, att_out, ldo, marks, frag_out);
}

// The MFMA attention as a kernel of its own, with all 16 MFMA columns holding real (head,row) pairs: passes with many
// rows per sequence (prefill, tree verify) read every cached key half as often as with 8 pairs per work item.
constexpr int ATTN_ROWS_RM = 16;
template <int HD>
__global__ __launch_bounds__(FUSED_NT) void attn_rows_kernel(const float* __restrict__ q, const f16_t* __restrict__ kc, const f16_t* __restrict__ vc,
                                                             const int* __restrict__ base, AttnShape sh, float* __restrict__ out, int ldo,
                                                             uint4* __restrict__ frag_out) {
    // frag_out (optional): the rows are written as A fragments of the next GEMM (K = ldo) instead of fp32 rows to `out`
    extern __shared__ __align__(16) float attn_rows_lds[];
    // Work items are numbered row block fastest, and workgroup b runs on XCD b % 8: the row blocks of one head would land
    // on different XCDs and each fetch the head's cached K and V rows from memory (61-row pass: 86 MB per layer for 23 MB
    // of cache rows).  Where the heads divide by 8, XCD x takes the heads x, x + 8, ... with all their row blocks.
    int item = blockIdx.x;
    const int nr = sh.n_rblk, ngrp = (int)gridDim.x / nr;
    if (nr > 1 && (ngrp & 7) == 0 && ngrp * nr == (int)gridDim.x) { const int x = item & 7, slot = item >> 3; item = (x + 8 * (slot / nr)) * nr + slot % nr; }
    attn_wg_mfma<HD, ATTN_ROWS_RM>(q, kc, vc, base, sh, item, 0, attn_rows_lds, nullptr, nullptr, out, ldo, nullptr, frag_out);
}

// Attention of long row ranges (prefill): the published flash-attention work split.  A workgroup owns 128 consecutive
// rows of ONE query head, 16 per wavefront, and walks the keys in tiles of 16 that the whole workgroup loads once and
// shares through LDS (two buffers, one workgroup barrier per tile), so a cached row is fetched once per 128 query rows
// instead of once per 16; every wavefront keeps its own running maximum / sum / accumulator, and nothing is merged
// across wavefronts.  Arithmetic per tile is exactly attn_wg_mfma's (hi/lo operands, three MFMA per product).
// Items: heads vary fastest, row blocks run from the last (most keys) to the first.
constexpr int ATTN_SHARED_ROWS = 16 * FUSED_NW;
__host__ __device__ constexpr size_t attn_shared_lds_bytes(int hd) { return 2 * 16 * ((size_t)hd * 4 + 16 + (size_t)hd * 4 + 32); }

template <int HD>
__global__ __launch_bounds__(FUSED_NT) void attn_rows_shared_kernel(const float* __restrict__ q, const f16_t* __restrict__ kc, const f16_t* __restrict__ vc,
                                                                    const int* __restrict__ base, AttnShape sh, float* __restrict__ out, int ldo) {
    extern __shared__ __align__(16) float attn_shared_lds[];
    constexpr int HALFB = HD * 2, ROWB = HD * 4, KS = HD / 32, NB = HD / 16, NCH = ROWB / 16;
    constexpr int VSTRIDE = ROWB + 32, KSTRIDE = ROWB + 16;
    constexpr int KTB = 16 * KSTRIDE, BUFB = KTB + 16 * VSTRIDE;
    static_assert(16 * NCH <= FUSED_NT, "one 16-key tile is loaded by one instruction of the workgroup");
    char* bufs = reinterpret_cast<char*>(attn_shared_lds);          // [2][K tile | V tile]

    const int group = sh.Hq / sh.Hkv;
    const int nh_total = sh.Hq;                                      // heads per sequence
    int item = blockIdx.x;
    const int per_rblk = nh_total * (int)(gridDim.x / (unsigned)(nh_total * sh.n_rblk));   // sequences x heads
    const int rblk = sh.n_rblk - 1 - item / per_rblk; item %= per_rblk;
    const int hh = item % nh_total;
    const int sl = item / nh_total;
    const int kvh = hh / group;
    const int seq = sh.seq0 + sl;
    const int i0 = rblk * ATTN_SHARED_ROWS, ni = min(ATTN_SHARED_ROWS, sh.m - i0);
    const int pos0 = (sh.nbase > 0 ? sh.base_val[sl] : base[seq]) + sh.offset;
    const int nkeys = min(pos0 + i0 + ni, sh.maxL);
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n16 = lane & 15, g = lane >> 4;
    const int r = 16 * wave + n16;
    const bool valid = r < ni;
    const bool active = 16 * wave < ni;                              // uniform per wavefront
    const int wq_max = pos0 + i0 + min(16 * wave + 15, ni - 1);      // last position any row of this wavefront may see

    const char* kbase = reinterpret_cast<const char*>(kc) + ((size_t)seq * sh.Hkv + kvh) * sh.maxL * ROWB;
    const char* vbase = reinterpret_cast<const char*>(vc) + ((size_t)seq * sh.Hkv + kvh) * sh.maxL * ROWB;
    const int tid = threadIdx.x;
    const bool loader = tid < 16 * NCH;
    const int lkey = min(tid / NCH, 15), lch = tid % NCH;
    u32x4_t knext, vnext;
#define HIVIS_SHARED_LOADS(kb_)                                                                 \
    {                                                                                           \
        const size_t off_ = (size_t)min((kb_) + lkey, nkeys - 1) * ROWB + lch * 16;             \
        knext = *reinterpret_cast<const u32x4_t*>(kbase + off_);                                \
        vnext = *reinterpret_cast<const u32x4_t*>(vbase + off_);                                \
    }
    HIVIS_SHARED_LOADS(0)

    f16x8_t qh[KS], ql[KS];
    {
        const float* qrow = q + (size_t)(sl * sh.m + i0 + min(r, ni - 1)) * sh.ldq + (size_t)hh * HD + g * 8;
        const float scale = valid ? rsqrtf((float)HD) : 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const float4 a = *reinterpret_cast<const float4*>(qrow + ks * 32);
            const float4 b = *reinterpret_cast<const float4*>(qrow + ks * 32 + 4);
            const float x[8] = {a.x * scale, a.y * scale, a.z * scale, a.w * scale, b.x * scale, b.y * scale, b.z * scale, b.w * scale};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const _Float16 hi = (_Float16)fminf(fmaxf(x[e], -65504.f), 65504.f);
                qh[ks][e] = hi; ql[ks][e] = (_Float16)(x[e] - (float)hi);
            }
        }
    }
    const int qpos = valid ? pos0 + i0 + r : 0x7FFFFFFF;

    float mrun = -INFINITY, lrun = 0.f;
    f32x4_t acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    for (int kb = 0, t = 0; kb < nkeys; kb += 16, ++t) {
        char* kt = bufs + (t & 1) * BUFB;
        char* vt = kt + KTB;
        // tile t -> LDS buffer t % 2 (its last readers, of tile t - 2, are behind the barrier of tile t - 1); request tile t + 1
        if (loader) {
            *reinterpret_cast<u32x4_t*>(kt + lkey * KSTRIDE + lch * 16) = knext;
            *reinterpret_cast<u32x4_t*>(vt + lkey * VSTRIDE + lch * 16) = vnext;
        }
        HIVIS_SHARED_LOADS(min(kb + 16, nkeys - 1))
        lds_barrier();
        if (!active || kb > wq_max) continue;                    // uniform: no row of this wavefront sees the tile
        f32x4_t st = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const f16x8_t kh = *reinterpret_cast<const f16x8_t*>(kt + n16 * KSTRIDE + ks * 64 + g * 16);
            const f16x8_t kl = *reinterpret_cast<const f16x8_t*>(kt + n16 * KSTRIDE + HALFB + ks * 64 + g * 16);
            st = __builtin_amdgcn_mfma_f32_16x16x32_f16(kl, qh[ks], st, 0, 0, 0);
            st = __builtin_amdgcn_mfma_f32_16x16x32_f16(kh, ql[ks], st, 0, 0, 0);
            st = __builtin_amdgcn_mfma_f32_16x16x32_f16(kh, qh[ks], st, 0, 0, 0);
        }
        float sv[4], tmax = -INFINITY;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const int key = kb + 4 * g + rr;
            sv[rr] = (key < nkeys && key <= qpos) ? st[rr] : -INFINITY;
            tmax = fmaxf(tmax, sv[rr]);
        }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
        const float mnew = fmaxf(mrun, tmax);
        const float mref = (mnew == -INFINITY) ? 0.f : mnew;
        const float alpha = __expf(mrun - mref);
        float p[4], psum = 0.f;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) { p[rr] = __expf(sv[rr] - mref); psum += p[rr]; }
        mrun = mnew;
        lrun = lrun * alpha + psum;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) acc[nb][rr] *= alpha;
        }
        f16x4_t pbh, pbl;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) { pbh[rr] = (_Float16)p[rr]; pbl[rr] = (_Float16)(p[rr] - (float)pbh[rr]); }
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const char* src = vt + (4 * g + (n16 >> 2)) * VSTRIDE + (nb * 16 + 4 * (n16 & 3)) * 2;
            const s16x4_t rh = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(src));
            const s16x4_t rl = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(src + HALFB));
            acc[nb] = __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4_t, rl), pbh, acc[nb], 0, 0, 0);
            acc[nb] = __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4_t, rh), pbl, acc[nb], 0, 0, 0);
            acc[nb] = __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4_t, rh), pbh, acc[nb], 0, 0, 0);
        }
    }
#undef HIVIS_SHARED_LOADS
    // this lane holds dims 16 nb + 4 (lane/16) + 0..3 of row r; the row's sum of weights is spread over the four lane groups
    float lsum = lrun;
    lsum += __shfl_xor(lsum, 16, 64);
    lsum += __shfl_xor(lsum, 32, 64);
    if (valid) {
        const float inv = 1.f / lsum;
        float* orow = out + (size_t)(sl * sh.m + i0 + r) * ldo + (size_t)hh * HD + 4 * g;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
            *reinterpret_cast<float4*>(orow + nb * 16) = make_float4(acc[nb][0] * inv, acc[nb][1] * inv, acc[nb][2] * inv, acc[nb][3] * inv);
    }
}

template <typename KT, int HD, int RM>
__device__ __forceinline__ void attn_wg_partial(const float* __restrict__ q, const KT* __restrict__ kc, const KT* __restrict__ vc,
                                                const int* __restrict__ base, const AttnShape& sh, int item_id, int split,
                                                float* __restrict__ lds, float* __restrict__ ws, int* __restrict__ cnt,
                                                float* __restrict__ att_out, int ldo, unsigned long long* marks = nullptr) {
    HIVIS_AMARK(0)
    constexpr int NW = FUSED_NW;
    constexpr int ROWB = HD * (int)sizeof(KT);     // bytes of one cached row
    constexpr int CH = 16 / (int)sizeof(KT);       // elements per 16-byte chunk
    constexpr int KL = ROWB / 64;                  // 16-byte loads per lane for its quarter of a K row
    constexpr int QD = HD / 4;                     // dims per quarter
    constexpr int NCH = ROWB / 16;                 // chunks per V row
    constexpr int KPI = 64 / NCH;                  // V rows per load instruction
    constexpr int VT = 16 / KPI;                   // V load instructions per 16 keys
    static_assert(NCH <= 64 && KPI >= 1 && VT >= 1, "row too long for this mapping");
    float* qs = lds;                               // [RM][HD] scaled queries
    float* pw_all = qs + RM * HD;                  // [NW][RM][16] probabilities of the wavefront's 16 keys
    float* mrg = pw_all + NW * RM * 16;            // [NW][RM][HD + 2] per-wavefront partials

    int item = item_id;
    const int rblk = item % sh.n_rblk; item /= sh.n_rblk;
    const int hblk = item % sh.n_hblk; item /= sh.n_hblk;
    const int kvh = item % sh.Hkv;
    const int sl = item / sh.Hkv;
    const int seq = sh.seq0 + sl;
    const int group = sh.Hq / sh.Hkv;
    const int h0 = hblk * sh.gh, nh = min(sh.gh, group - h0);
    const int i0 = rblk * sh.mi, ni = min(sh.mi, sh.m - i0);
    const int R = nh * ni;
    const int pos0 = (sh.nbase > 0 ? sh.base_val[sl] : base[seq]) + sh.offset;
    const int nkeys = min(pos0 + i0 + ni, sh.maxL);
    const int cs = ((nkeys + sh.nsplit - 1) / sh.nsplit + 15) & ~15;        // keys per split, multiple of 16
    const int k0 = split * cs, k1 = min(nkeys, k0 + cs);
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wavefront index as a scalar: branches on it are uniform
    const float scale = rsqrtf((float)HD);

    const KT* kbase = kc + ((size_t)seq * sh.Hkv + kvh) * sh.maxL * HD;
    const KT* vbase = vc + ((size_t)seq * sh.Hkv + kvh) * sh.maxL * HD;
    float* pw = pw_all + wave * RM * 16;
    const int kk = lane >> 2, quarter = lane & 3;      // K mapping: key within the 16, quarter of the row
    const int vks = lane / NCH, vdc = lane % NCH;      // V mapping: row within the instruction, chunk of the row

    // all loads of this wavefront's 16 keys starting at kb_ (addresses clamped into the range; masked later)
    uint4 knext[KL], vnext[VT];
#define HIVIS_ATTN_LOADS(kb_)                                                                                      \
    {                                                                                                              \
        const int key_ = min((kb_) + kk, nkeys - 1);                                                               \
        const uint4* kp_ = reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(kbase) + (size_t)key_ * ROWB + quarter * (ROWB / 4)); \
        _Pragma("unroll") for (int j = 0; j < KL; ++j) knext[j] = kp_[j];                                          \
        _Pragma("unroll") for (int t = 0; t < VT; ++t) {                                                           \
            const int vkey_ = min((kb_) + t * KPI + vks, nkeys - 1);                                               \
            vnext[t] = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(vbase) + (size_t)vkey_ * ROWB + vdc * 16); \
        }                                                                                                          \
    }
    // the cached keys do not depend on the queries: request the first block before staging q
    if (k0 + 16 * wave < k1) HIVIS_ATTN_LOADS(k0 + 16 * wave)
    HIVIS_AMARK(1)

    for (int idx = threadIdx.x; idx < R * HD; idx += FUSED_NT) {
        const int r = idx / HD, c = idx % HD;
        const int hh = kvh * group + h0 + r / ni, i = i0 + r % ni;
        qs[idx] = q[(size_t)(sl * sh.m + i) * sh.ldq + (size_t)hh * HD + c] * scale;
    }
    lds_barrier();
    HIVIS_AMARK(2)

    float mrun[RM], lrun[RM], acc[RM][CH];
#pragma unroll
    for (int r = 0; r < RM; ++r) {
        mrun[r] = -INFINITY; lrun[r] = 0.f;
#pragma unroll
        for (int e = 0; e < CH; ++e) acc[r][e] = 0.f;
    }

    for (int kb = k0 + 16 * wave; kb < k1; kb += 16 * NW) {
        uint4 kraw[KL], vraw[VT];
#pragma unroll
        for (int j = 0; j < KL; ++j) kraw[j] = knext[j];
#pragma unroll
        for (int t = 0; t < VT; ++t) vraw[t] = vnext[t];
        if (kb + 16 * NW < k1) HIVIS_ATTN_LOADS(kb + 16 * NW)
        // ---- scores of (key kk, all rows): this lane's quarter, then summed over the 4 quarter lanes
        float s[RM];
#pragma unroll
        for (int r = 0; r < RM; ++r) s[r] = 0.f;
#pragma unroll
        for (int j = 0; j < KL; ++j) {
            float kf[CH];
            decode_chunk(kraw[j], kf, KT());
#pragma unroll
            for (int r = 0; r < RM; ++r) {
                if (r < R) {
                    const float* qr = qs + r * HD + quarter * QD + j * CH;
#pragma unroll
                    for (int e = 0; e < CH; ++e) s[r] += qr[e] * kf[e];
                }
            }
        }
        const int key = kb + kk;
#pragma unroll
        for (int r = 0; r < RM; ++r) {
            if (r < R) {
                float sv = quad_sum(s[r]);                // the 4 lanes of a key hold its 4 quarter dot products
                const int qpos = pos0 + i0 + r % ni;
                if (key >= k1 || key > qpos) sv = -INFINITY;
                const float tmax = wave_max(sv);
                const float mnew = fmaxf(mrun[r], tmax);
                float alpha = 1.f, p = 0.f;
                if (mnew != -INFINITY) {
                    alpha = (mrun[r] == -INFINITY) ? 0.f : __expf(mrun[r] - mnew);
                    p = (sv == -INFINITY) ? 0.f : __expf(sv - mnew);
                }
                mrun[r] = mnew;
                lrun[r] = lrun[r] * alpha + ((quarter == 0) ? p : 0.f);
#pragma unroll
                for (int e = 0; e < CH; ++e) acc[r][e] *= alpha;
                if (quarter == 0) pw[r * 16 + kk] = p;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        // ---- acc += p * V for this lane's chunk of the rows it loaded
#pragma unroll
        for (int t = 0; t < VT; ++t) {
            float vf[CH];
            decode_chunk(vraw[t], vf, KT());
            const int kl = t * KPI + vks;                // key within the 16 (its p is 0 if masked)
#pragma unroll
            for (int r = 0; r < RM; ++r) {
                if (r < R) {
                    const float p = pw[r * 16 + kl];
#pragma unroll
                    for (int e = 0; e < CH; ++e) acc[r][e] += p * vf[e];
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    HIVIS_AMARK(3)
    // ---- per-wavefront partial -> LDS (sum over the lanes that share a chunk / over all lanes for l)
#pragma unroll
    for (int r = 0; r < RM; ++r) {
        if (r < R) {
            const float lsum = wave_sum(lrun[r]);
#pragma unroll
            for (int e = 0; e < CH; ++e) {
                float a = acc[r][e];
#pragma unroll
                for (int o = NCH; o < 64; o <<= 1) a += __shfl_xor(a, o, 64);
                if (lane < NCH) mrg[(wave * RM + r) * (HD + 2) + lane * CH + e] = a;
            }
            if (lane == 0) { mrg[(wave * RM + r) * (HD + 2) + HD] = mrun[r]; mrg[(wave * RM + r) * (HD + 2) + HD + 1] = lsum; }
        }
    }
    attn_wg_finish<HD, RM>(mrg, reinterpret_cast<int*>(pw_all), sh, item_id, split, R, ni, kvh * group + h0, i0, sl, ws, cnt, att_out, ldo, marks);
#undef HIVIS_ATTN_LOADS
}

// Merge of the nsplit workgroup partials of one item, in split order; writes the attention output rows.
template <int HD, int RM>
__device__ __forceinline__ void attn_wg_merge(const float* __restrict__ ws, const AttnShape& sh, int item_id,
                                              float* __restrict__ lds, float* __restrict__ out, int ldo) {
    int item = item_id;
    const int rblk = item % sh.n_rblk; item /= sh.n_rblk;
    const int hblk = item % sh.n_hblk; item /= sh.n_hblk;
    const int kvh = item % sh.Hkv;
    const int sl = item / sh.Hkv;
    const int group = sh.Hq / sh.Hkv;
    const int h0 = hblk * sh.gh, nh = min(sh.gh, group - h0);
    const int i0 = rblk * sh.mi, ni = min(sh.mi, sh.m - i0);
    const int R = nh * ni;
    const float* base = ws + (size_t)item_id * sh.nsplit * RM * (HD + 2);
    attn_merge_splits<HD, RM>(base, sh.nsplit, R, ni, kvh * group + h0, i0, sl, sh, lds, out, ldo);
}

// One phase, executed by the calling grid (every workgroup calls this with the same arguments).
template <typename WT, int TYPE, int EPI, bool SINGLE>
__device__ __forceinline__ void run_phase(const Phase& ph, const PassParams& pp, float* __restrict__ lds, uint4 (&head)[FUSED_U],
                                          bool& head_valid, uint4 (&wb1)[FUSED_U], bool& wb1_valid, int p) {
    typedef typename KVType<WT>::type KT;
    const int type = (TYPE >= 0) ? TYPE : ph.type;
    switch (type) {
    case PH_GEMM: gemm_phase<WT, EPI, SINGLE>(ph, pp, lds, head, head_valid, wb1, wb1_valid, p); break;
    case PH_ATTN: {
        // (item, split) of a workgroup.  Default: split-minor.  flags & 2: every split of an item on ONE XCD (workgroup w
        // runs on XCD w % 8): XCD x works on the items x, x + 8, ..., so an item's partials meet in one L2.
        const int nsp = ph.att.nsplit;
        const bool xcd_map = (ph.att.flags & 2) != 0;
        const int total = xcd_map ? 8 * ((ph.att_items + 7) / 8) * nsp : ph.att_items * nsp;
        for (int w = blockIdx.x; w < total; w += gridDim.x) {
            int item, split;
            if (xcd_map) { const int j = w >> 3; item = (w & 7) + 8 * (j / nsp); split = j % nsp; if (item >= ph.att_items) continue; }
            else { item = w / nsp; split = w % nsp; }
            if constexpr (std::is_same<KT, f16_t>::value) {
                if (pp.hd == 128) attn_wg_mfma<128, FUSED_RMAX>(ph.A, (const KT*)ph.kc, (const KT*)ph.vc, ph.base, ph.att, item, split, lds, ph.ws, ph.cnt, ph.Y, ph.ldy, pp.prof2, ph.frag);
                else attn_wg_mfma<64, FUSED_RMAX>(ph.A, (const KT*)ph.kc, (const KT*)ph.vc, ph.base, ph.att, item, split, lds, ph.ws, ph.cnt, ph.Y, ph.ldy, pp.prof2, ph.frag);
            } else {
                if (pp.hd == 128) attn_wg_partial<KT, 128, FUSED_RMAX>(ph.A, (const KT*)ph.kc, (const KT*)ph.vc, ph.base, ph.att, item, split, lds, ph.ws, ph.cnt, ph.Y, ph.ldy, pp.prof2);
                else attn_wg_partial<KT, 64, FUSED_RMAX>(ph.A, (const KT*)ph.kc, (const KT*)ph.vc, ph.base, ph.att, item, split, lds, ph.ws, ph.cnt, ph.Y, ph.ldy, pp.prof2);
            }
        }
    } break;
    case PH_ATTN_MERGE:
        if (pp.prof2 && blockIdx.x == 0 && threadIdx.x == 0) pp.prof2[0] = wall_clock64();
        for (int item = blockIdx.x; item < ph.att_items; item += gridDim.x) {
            if (pp.hd == 128) attn_wg_merge<128, FUSED_RMAX>(ph.ws, ph.att, item, lds, ph.Y, ph.ldy);
            else attn_wg_merge<64, FUSED_RMAX>(ph.ws, ph.att, item, lds, ph.Y, ph.ldy);
        }
        break;
    case PH_PREP: {
        // embedding gather of the rows' tokens
        if (ph.ids) {
            for (int row = blockIdx.x; row < pp.M; row += gridDim.x) {
                // token ids may have been written earlier in this launch: agent-scope load; clamped for safety
                int32_t tok = __hip_atomic_load(&ph.ids[(row / pp.m) * ph.id_sseq + (row % pp.m) * ph.id_srow], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                tok = min(max(tok, 0), pp.V - 1);
                const WT* src = (const WT*)ph.gain + (size_t)tok * pp.d;
                for (int c = threadIdx.x; c < pp.d; c += FUSED_NT) st_wt(&ph.Y[(size_t)row * ph.ldy + c], to_f32(src[c]));
            }
        }
    } break;
    case PH_NORM_ROWS:
        // Y[row] = A[row] * gain / sqrt(mean(A[row]^2) + eps): one workgroup per row
        for (int row = blockIdx.x; row < pp.M; row += gridDim.x) {
            const float* x = ph.A + (size_t)row * ph.lda;
            float ss = 0.f;
            for (int c = threadIdx.x; c < pp.d; c += FUSED_NT) ss += x[c] * x[c];
            ss = wave_sum(ss);
            lds_barrier();
            if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = ss;
            lds_barrier();
            float tot = 0.f;
#pragma unroll
            for (int w = 0; w < FUSED_NW; ++w) tot += lds[w];
            const float inv = 1.0f / sqrtf(tot / (float)pp.d + pp.eps);
            for (int c = threadIdx.x; c < pp.d; c += FUSED_NT)
                st_wt(&ph.Y[(size_t)row * ph.ldy + c], x[c] * to_f32(((const WT*)ph.gain)[c]) * inv);
        }
        break;
    case PH_ARGMAX:
        // one wavefront per row reduces the per-workgroup candidates (lowest index wins ties)
        for (int row = blockIdx.x * FUSED_NW + (threadIdx.x >> 6); row < pp.M; row += gridDim.x * FUSED_NW) {
            float bv = -INFINITY; int bi = 0x7FFFFFFF;
            // ph.N = number of candidate slots per row (the grid size of the LM-head phase that wrote them)
            for (int w = threadIdx.x & 63; w < ph.N; w += 64) {
                const float v = ph.pm[(size_t)row * ph.N + w]; const int i = ph.pi[(size_t)row * ph.N + w];
                if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                const float ov = __shfl_xor(bv, o, 64); const int oi = __shfl_xor(bi, o, 64);
                if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
            }
            if ((threadIdx.x & 63) == 0) {
                if (pp.bad && (unsigned)bi >= (unsigned)pp.V) st_wt(pp.bad, 1);
                st_wt(&ph.tok_out[(row / pp.m) * ph.o_sseq + (row % pp.m) * ph.o_srow], clamp_token(bi, pp.V));
            }
        }
        break;
    case PH_SAMPLE:
        // one workgroup per row: token drawn from softmax(logits / T) by inversion with the row's uniform number
        for (int row = blockIdx.x; row < pp.M; row += gridDim.x) {
            float* smf = lds; int* smi = reinterpret_cast<int*>(lds + 16);
            const float u = ph.u[(row / pp.m) * ph.u_sseq + ph.u_idx];
            const int tok = block_sample_softmax<FUSED_NT>(ph.A + (size_t)row * ph.lda, pp.V, pp.inv_temp, u, smf, smi);
            if (threadIdx.x == 0) st_wt(&ph.tok_out[(row / pp.m) * ph.o_sseq + (row % pp.m) * ph.o_srow], tok);
        }
        break;
    }
}

// Whole pass in one cooperative launch: phases separated by grid barriers (see the notes at the top).
template <typename WT>
__global__ __launch_bounds__(FUSED_NT) void fused_pass_kernel(PassParams pp) {
    extern __shared__ __align__(16) float lds[];
    uint4 head[FUSED_U], wb1[FUSED_U];   // weight blocks prefetched for the next GEMM phase (in flight across barriers)
    bool head_valid = false, wb1_valid = false;
    for (int p = 0; p < pp.nphases; ++p) {
        const Phase& ph = pp.phases[p];
        if (pp.prof && blockIdx.x == 0 && threadIdx.x == 0) pp.prof[p * 3] = wall_clock64();
        run_phase<WT, -1, -1, false>(ph, pp, lds, head, head_valid, wb1, wb1_valid, p);
        if (pp.prof && blockIdx.x == 0 && threadIdx.x == 0) pp.prof[p * 3 + 1] = wall_clock64();
        const bool ok = grid_barrier(pp.bar, (unsigned)(p + 1) * gridDim.x, pp.spin_limit, ph.type == PH_GEMM);
        if (pp.prof && blockIdx.x == 0 && threadIdx.x == 0) pp.prof[p * 3 + 2] = wall_clock64();
        if (!ok) return;
    }
}

// One phase per launch: the kernel boundary orders the phases (and makes every store visible), so nothing is
// prefetched across it and no barrier is needed.  This is the default way the passes are run.
// Touches every 64-byte line of the kernel-argument segment with one batch of scalar loads.  The arguments of a phase
// (two structs, ~0.6 KB) live in memory that no cache holds when the launch starts, and the compiler loads each field
// just before its first use: a chain of dependent scalar round trips (four to six in the attention phase, ~0.4 us each)
// before the first vector load is requested.  After this batch those loads hit the scalar cache.
template <int BYTES>
__device__ __forceinline__ void kernarg_warm() {
    typedef const int __attribute__((address_space(4))) cint_t;
    cint_t* kp = (cint_t*)__builtin_amdgcn_kernarg_segment_ptr();
    int acc = 0;
#pragma unroll
    for (int i = 0; i < (BYTES + 63) / 64; ++i) acc |= kp[16 * i];
    asm volatile("" ::"s"(acc));
}

template <typename WT, int TYPE, int EPI, bool SINGLE>
__global__ __launch_bounds__(FUSED_NT) void phase_kernel(Phase ph, PassParams pp) {
    extern __shared__ __align__(16) float lds[];
    kernarg_warm<sizeof(Phase) + sizeof(PassParams)>();
    uint4 head[FUSED_U], wb1[FUSED_U];
    bool head_valid = false, wb1_valid = false;
    if (pp.prof3 && threadIdx.x == 0) {
        pp.prof3[blockIdx.x * 4] = wall_clock64();
        // HW_ID (wave, SIMD, CU, shader array, shader engine) and XCC_ID of the wavefront
        pp.prof3[blockIdx.x * 4 + 2] = (unsigned long long)__builtin_amdgcn_s_getreg((31 << 11) | 4) | ((unsigned long long)__builtin_amdgcn_s_getreg((3 << 11) | 20) << 32);
    }
    run_phase<WT, TYPE, EPI, SINGLE>(ph, pp, lds, head, head_valid, wb1, wb1_valid, 0);
    if (pp.prof3) {
        lds_barrier();
        if (threadIdx.x == 0) pp.prof3[blockIdx.x * 4 + 1] = wall_clock64();
    }
}

}  // namespace hivis

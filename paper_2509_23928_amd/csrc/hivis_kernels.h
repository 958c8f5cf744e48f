// HIP kernels of the HiViS draft-verify path for gfx950 (CDNA4, 64-wide wavefronts).
//
// Decode, draft and verify are weight-streaming problems: every weight is read once per pass
// and multiplies a handful of activation rows.  The weights are therefore re-laid-out once,
// at load time, into 1 KiB blocks that one wavefront reads with a single 16-byte-per-lane load
// in exactly the register layout the MFMA B operand wants; the kernel is a linear stream of
// such blocks.  The activation rows are the MFMA A operand: for bf16 weights each fp32
// activation is split into a bf16 "hi" and a bf16 "lo" part which occupy two of the 16 tile
// rows (8 real rows per tile), so activations keep ~16 mantissa bits at no extra HBM traffic;
// fp32 weights use the fp32 MFMA with 16 real rows per tile.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hivis {

typedef uint16_t bf16_t;                                  // bfloat16 bit pattern
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
// round to nearest even: the conversion instruction of gfx950 (v_cvt_pk_bf16_f32), bit for bit what the integer
// recipe u += 0x7FFF + ((u >> 16) & 1) gives for finite inputs, at a fifth of the instructions
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }
// two values -> two bf16 in one 32-bit word (a in the low half)
__device__ __forceinline__ uint32_t f32_to_bf16x2(float a, float b) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
// hi and lo parts of two values: hi = bf16(x), lo = bf16(x - hi)
__device__ __forceinline__ void f32_to_bf16x2_hilo(float a, float b, uint32_t& hi, uint32_t& lo) {
    hi = f32_to_bf16x2(a, b);
    lo = f32_to_bf16x2(a - __uint_as_float(hi << 16), b - __uint_as_float(hi & 0xFFFF0000u));
}
typedef _Float16 f16_t;                                   // IEEE half: KV-cache storage of bf16 models
__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return bf16_to_f32(x); }
__device__ __forceinline__ float to_f32(f16_t x) { return (float)x; }
__device__ __forceinline__ void from_f32(float& dst, float x) { dst = x; }
__device__ __forceinline__ void from_f32(bf16_t& dst, float x) { dst = f32_to_bf16(x); }
__device__ __forceinline__ void from_f32(f16_t& dst, float x) {   // round to nearest even, saturating
    dst = (f16_t)fminf(fmaxf(x, -65504.f), 65504.f);
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every outstanding global
// load of the wavefront, which would drain the weight prefetch pipeline at each use.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Wait until every vector memory operation of this wavefront, in particular its write-through stores, has been
// acknowledged (s_waitcnt vmcnt(0); the other counters are left alone).  A workgroup-scope release fence does
// NOT do this on this target: it only orders LDS traffic, because wavefronts of one workgroup share their L1.
__device__ __forceinline__ void wait_vmem() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// Write-through stores (agent scope): the value is sent to memory, not left dirty in this XCD's L2, so a
// workgroup on another XCD that reads the address for the first time sees it without cache maintenance.
__device__ __forceinline__ void st_wt(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_wt(int* p, int v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_wt(uint32_t* p, uint32_t v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
// Agent-scope load: reads what an agent-scope (write-through) store of another workgroup, on any XCD, has completed.
__device__ __forceinline__ float ld_agent(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
// two adjacent cache elements (dst 4-byte aligned)
__device__ __forceinline__ void st_wt_pair(float* dst, float a, float b) { st_wt(dst, a); st_wt(dst + 1, b); }
__device__ __forceinline__ void st_wt_pair(_Float16* dst, float a, float b) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    h2 v;
    v[0] = (_Float16)fminf(fmaxf(a, -65504.f), 65504.f);
    v[1] = (_Float16)fminf(fmaxf(b, -65504.f), 65504.f);
    st_wt(reinterpret_cast<uint32_t*>(dst), __builtin_bit_cast(uint32_t, v));
}

// two adjacent values (c, c+1; c even) of a cache row of HD values, hi and lo halves for half-precision caches
__device__ __forceinline__ void st_wt_kv_pair(float* row, int HD, int c, float a, float b) { st_wt_pair(row + c, a, b); }
__device__ __forceinline__ void st_wt_kv_pair(_Float16* row, int HD, int c, float a, float b) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    h2 hi, lo;
    hi[0] = (_Float16)fminf(fmaxf(a, -65504.f), 65504.f);
    hi[1] = (_Float16)fminf(fmaxf(b, -65504.f), 65504.f);
    lo[0] = (_Float16)(a - (float)hi[0]);
    lo[1] = (_Float16)(b - (float)hi[1]);
    st_wt(reinterpret_cast<uint32_t*>(row + c), __builtin_bit_cast(uint32_t, hi));
    st_wt(reinterpret_cast<uint32_t*>(row + HD + c), __builtin_bit_cast(uint32_t, lo));
}

// KV-cache storage that goes with a weight type.  fp32 models keep K and V in fp32.  bf16 models keep every cached
// value as TWO IEEE halves, hi = half(x) and lo = half(x - hi) (about 22 mantissa bits), in one row of 2*HD halves:
// [hi 0..HD) | lo 0..HD)].  Both halves are MFMA operands as they are.  One half alone is not enough at depth: the
// rounding of K and V (2^-11 relative) is amplified layer after layer (text rows carry a tiny residual stream next
// to what attention adds to it) and again by the drafter; at 32 layers it put the drafter's logits at 1.7x the
// parity tolerance, with q and the probabilities rounded to half contributing as much again.
template <typename WT> struct KVType;
template <> struct KVType<bf16_t> { typedef f16_t type; };
template <> struct KVType<float> { typedef float type; };
// elements of storage per cached value (row width = HD * KVW)
template <typename KT> struct KVWidth { static constexpr int W = 1; };
template <> struct KVWidth<f16_t> { static constexpr int W = 2; };

// value c of the cache row starting at `row` (HD values per row)
__device__ __forceinline__ void kv_put(float* row, int HD, int c, float x) { row[c] = x; }
__device__ __forceinline__ void kv_put(f16_t* row, int HD, int c, float x) {
    const f16_t hi = (f16_t)fminf(fmaxf(x, -65504.f), 65504.f);
    row[c] = hi;
    row[HD + c] = (f16_t)(x - (float)hi);
}
// two adjacent values c, c + 1 (c even): the hi halves and the lo halves each go out as one 32-bit store
__device__ __forceinline__ void kv_put_pair(float* row, int HD, int c, float a, float b) { row[c] = a; row[c + 1] = b; }
__device__ __forceinline__ void kv_put_pair(f16_t* row, int HD, int c, float a, float b) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    h2 hi, lo;
    hi[0] = (f16_t)fminf(fmaxf(a, -65504.f), 65504.f);
    hi[1] = (f16_t)fminf(fmaxf(b, -65504.f), 65504.f);
    lo[0] = (f16_t)(a - (float)hi[0]);
    lo[1] = (f16_t)(b - (float)hi[1]);
    *reinterpret_cast<h2*>(row + c) = hi;
    *reinterpret_cast<h2*>(row + HD + c) = lo;
}
__device__ __forceinline__ float kv_get(const float* row, int HD, int c) { return row[c]; }
__device__ __forceinline__ float kv_get(const f16_t* row, int HD, int c) { return (float)row[c] + (float)row[HD + c]; }

// 16 raw bytes of cache -> floats
__device__ __forceinline__ void decode_chunk(const uint4& raw, float (&kf)[8], f16_t) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const h2 v = __builtin_bit_cast(h2, w[e]);
        kf[2 * e] = (float)v[0]; kf[2 * e + 1] = (float)v[1];
    }
}
__device__ __forceinline__ void decode_chunk(const uint4& raw, float (&kf)[4], float) {
    kf[0] = __uint_as_float(raw.x); kf[1] = __uint_as_float(raw.y);
    kf[2] = __uint_as_float(raw.z); kf[3] = __uint_as_float(raw.w);
}

// ------------------------------------------------------------------------------------------
// Streaming layout of a weight matrix W (logical [K][N], y = x W).
//   tile  t = n / 16      (16 output columns)
//   block kb = k / KB     (KB = 32 k-values for bf16, 16 for fp32)  -> 1 KiB = 64 lanes x 16 B
//   lane  = (n % 16) + 16 * g
//     bf16: the lane's 8 values are k = 32 kb + 8 g + e, e = 0..7
//     fp32: the lane's 4 values are k = 16 kb + 4 g + e, e = 0..3
//   address (in 16-byte units) = (t * (K / KB) + kb) * 64 + lane
// ------------------------------------------------------------------------------------------
template <typename WT> struct WTraits;
template <> struct WTraits<bf16_t> {
    static constexpr int KB = 32;      // k per block
    static constexpr int EPL = 8;      // elements per lane per block
    static constexpr int ROWS = 8;     // real activation rows per MFMA tile (hi/lo split)
    static constexpr int RPL = 2;      // real output rows per lane
};
template <> struct WTraits<float> {
    static constexpr int KB = 16;
    static constexpr int EPL = 4;
    static constexpr int ROWS = 16;
    static constexpr int RPL = 4;
};

// Sources of a packed matrix: up to three matrices concatenated along the output dimension
// (fused QKV, fused gate|up).  transposed = 1 means the source is [N][K] (LM head).
struct PackSrc {
    const void* p[3];
    int n[3];          // output columns of each source
    int transposed;
    int mode;          // PACK_PLAIN, PACK_QKV, PACK_GATEUP
    int hd;            // head_dim (PACK_QKV)
};
// Column orders of the packed matrices (chosen so that the GEMM epilogues are local to a 16-column tile):
//   PACK_QKV    [q heads | k heads | v heads]; inside every q and k head the rotary pair (i, i + hd/2) is
//               stored in adjacent columns (2i, 2i+1).  q and k are only ever used in dot products with
//               each other, so the K cache simply keeps this order; v keeps the natural order.
//   PACK_GATEUP tile t holds gate columns 8t..8t+7 in its first 8 columns and up columns 8t..8t+7 in its
//               last 8, so silu(gate)*up needs one tile only.
enum { PACK_PLAIN = 0, PACK_QKV = 1, PACK_GATEUP = 2 };

template <typename WT>
__global__ void pack_weights_kernel(PackSrc src, int K, int N, uint4* __restrict__ dst) {
    constexpr int KB = WTraits<WT>::KB, EPL = WTraits<WT>::EPL;
    const size_t total = (size_t)(N / 16) * (K / KB) * 64;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
        const int lane = (int)(idx & 63);
        const size_t blk = idx >> 6;
        const int kb = (int)(blk % (size_t)(K / KB));
        const int t = (int)(blk / (size_t)(K / KB));
        int n = t * 16 + (lane & 15);
        const int g = lane >> 4;
        const int k0 = kb * KB + g * EPL;
        int s = 0;
        if (src.mode == PACK_GATEUP) {
            s = (lane & 15) >> 3;                 // 0 = gate, 1 = up
            n = t * 8 + (lane & 7);
        } else {
            while (s < 2 && n >= src.n[s]) { n -= src.n[s]; ++s; }
            if (src.mode == PACK_QKV && s < 2) {  // q or k: un-interleave the rotary pair
                const int within = n % src.hd;
                n = n - within + (within >> 1) + (within & 1) * (src.hd / 2);
            }
        }
        const WT* base = (const WT*)src.p[s];
        const int ns = src.n[s];
        WT vals[EPL];
#pragma unroll
        for (int e = 0; e < EPL; ++e)
            vals[e] = src.transposed ? base[(size_t)n * K + (k0 + e)] : base[(size_t)(k0 + e) * ns + n];
        dst[idx] = *reinterpret_cast<const uint4*>(vals);
    }
}

// ------------------------------------------------------------------------------------------
// Skinny GEMM  Y[M][N] (+)= A[M][K] . W      (M <= T * ROWS rows; W in streaming layout)
//
// One workgroup of NW wavefronts owns a contiguous range of 16-column tiles and always covers
// the whole K range, so every output element is produced by exactly one workgroup in a fixed
// summation order (bit-reproducible; no atomics).  Inside the workgroup the K range is cut
// into passes of NW*KBW blocks; in a pass wave w holds the A fragments of its KBW blocks in
// registers and streams the matching weight blocks of up to G tiles through the MFMA unit,
// with the loads of the next tile issued before the MFMAs of the current one.  The NW partial
// tiles are then summed through LDS.
// ------------------------------------------------------------------------------------------
template <typename WT> struct AFrag;
template <> struct AFrag<bf16_t> { typedef bf16x8_t type; };
template <> struct AFrag<float> { typedef float4 type; };

// A fragment of tile tt, block kb for this lane.  a_scale (optional, per k) multiplies the
// activation before the hi/lo split (used to apply an RMSNorm gain on the fly).
// Raw activation values of one A fragment (loaded unconditionally from a clamped row; converted later)
template <typename WT> struct ARaw;
template <> struct ARaw<bf16_t> { float4 x0, x1; };
template <> struct ARaw<float> { float4 x0; };
__device__ __forceinline__ void load_afrag_raw(ARaw<bf16_t>& r, const float* __restrict__ A, int lda, int M, int tt, int kb, int lane) {
    const int i = lane & 15, g = lane >> 4;
    const int row = min(tt * 8 + 2 * (i >> 2) + (i & 1), M - 1);
    const float4* p = reinterpret_cast<const float4*>(A + (size_t)row * lda + kb * 32 + g * 8);
    r.x0 = p[0]; r.x1 = p[1];
}
__device__ __forceinline__ void load_afrag_raw(ARaw<float>& r, const float* __restrict__ A, int lda, int M, int tt, int kb, int lane) {
    const int i = lane & 15, g = lane >> 4;
    const int row = min(tt * 16 + i, M - 1);
    r.x0 = *reinterpret_cast<const float4*>(A + (size_t)row * lda + kb * 16 + g * 4);
}
__device__ __forceinline__ void make_afrag(bf16x8_t& out, const ARaw<bf16_t>& r, int M, int tt, bool valid, int lane) {
    const int i = lane & 15;
    const int row = tt * 8 + 2 * (i >> 2) + (i & 1);
    const bool lo = (i & 2) != 0;
    const bool on = valid && row < M;
    const float x[8] = {r.x0.x, r.x0.y, r.x0.z, r.x0.w, r.x1.x, r.x1.y, r.x1.z, r.x1.w};
    uint32_t pk[4];
    bf16_t h[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const bf16_t hi = f32_to_bf16(x[e]);
        h[e] = lo ? f32_to_bf16(x[e] - bf16_to_f32(hi)) : hi;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) pk[e] = on ? ((uint32_t)h[2 * e] | ((uint32_t)h[2 * e + 1] << 16)) : 0u;
    out = __builtin_bit_cast(bf16x8_t, make_uint4(pk[0], pk[1], pk[2], pk[3]));
}
__device__ __forceinline__ void make_afrag(float4& out, const ARaw<float>& r, int M, int tt, bool valid, int lane) {
    const bool on = valid && (tt * 16 + (lane & 15)) < M;
    out = on ? r.x0 : make_float4(0.f, 0.f, 0.f, 0.f);
}
__device__ __forceinline__ void load_afrag(bf16x8_t& out, const float* __restrict__ A, int lda, int M, int tt, int kb,
                                           int lane) {
    const int i = lane & 15, g = lane >> 4;
    const int row = tt * 8 + 2 * (i >> 2) + (i & 1);
    const bool lo = (i & 2) != 0;
    uint32_t pk[4] = {0u, 0u, 0u, 0u};
    if (row < M) {
        const float4* p = reinterpret_cast<const float4*>(A + (size_t)row * lda + kb * 32 + g * 8);
        float4 x0 = p[0], x1 = p[1];
        float x[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
        bf16_t h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            bf16_t hi = f32_to_bf16(x[e]);
            h[e] = lo ? f32_to_bf16(x[e] - bf16_to_f32(hi)) : hi;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) pk[e] = (uint32_t)h[2 * e] | ((uint32_t)h[2 * e + 1] << 16);
    }
    uint4 u = make_uint4(pk[0], pk[1], pk[2], pk[3]);
    out = __builtin_bit_cast(bf16x8_t, u);
}
__device__ __forceinline__ void load_afrag(float4& out, const float* __restrict__ A, int lda, int M, int tt, int kb,
                                           int lane) {
    const int i = lane & 15, g = lane >> 4;
    const int row = tt * 16 + i;
    out = make_float4(0.f, 0.f, 0.f, 0.f);
    if (row < M) out = *reinterpret_cast<const float4*>(A + (size_t)row * lda + kb * 16 + g * 4);
}

__device__ __forceinline__ void mfma_block(f32x4_t& d, const bf16x8_t& a, const uint4& w) {
    d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8_t, w), d, 0, 0, 0);
}
__device__ __forceinline__ void mfma_block(f32x4_t& d, const float4& a, const uint4& w) {
    d = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x, __uint_as_float(w.x), d, 0, 0, 0);
    d = __builtin_amdgcn_mfma_f32_16x16x4f32(a.y, __uint_as_float(w.y), d, 0, 0, 0);
    d = __builtin_amdgcn_mfma_f32_16x16x4f32(a.z, __uint_as_float(w.z), d, 0, 0, 0);
    d = __builtin_amdgcn_mfma_f32_16x16x4f32(a.w, __uint_as_float(w.w), d, 0, 0, 0);
}

// Epilogue modes of the skinny GEMM
enum { EPI_STORE = 0, EPI_ACCUM = 1 };

template <typename WT, int T, int KBW, int G, int NW, bool UPFRONT = false>
__global__ __launch_bounds__(NW * 64) void gemm_skinny_kernel(const float* __restrict__ A, int lda, int M, int K,
                                                               const uint4* __restrict__ Wp, int N,
                                                               float* __restrict__ Y, int ldy, int epi) {
    typedef WTraits<WT> TR;
    typedef typename AFrag<WT>::type afrag_t;
    constexpr int RPL = TR::RPL;
    static_assert(NW * G * T * RPL * 64 * 4 <= 160 * 1024, "LDS reduction buffer must fit the 160 KiB of a compute unit");
    extern __shared__ __align__(16) float red[];       // [NW][G][T][64][RPL] (dynamic: up to 128 KiB for the 32-row variant)

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: uniform branches
    const int kblks = K / TR::KB;
    const int ntiles = N / 16;
    const int t_begin = (int)(((long long)blockIdx.x * ntiles) / gridDim.x);
    const int t_end = (int)(((long long)(blockIdx.x + 1) * ntiles) / gridDim.x);
    const int npass = (kblks + NW * KBW - 1) / (NW * KBW);

    for (int tg = t_begin; tg < t_end; tg += G) {
        const int ng = min(G, t_end - tg);
        f32x4_t acc[G][T];
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int tt = 0; tt < T; ++tt) acc[g][tt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

        for (int pass = 0; pass < npass; ++pass) {
            const int kb0 = (pass * NW + wave) * KBW;
            const int nkb = max(0, min(KBW, kblks - kb0));       // wave-uniform
            if (nkb == 0) continue;
            // first tile's weights (UPFRONT: the weights of ALL tiles of the group, so that one memory round trip serves the
            // whole pass instead of one per tile) and ALL activation rows of the pass are requested before anything is
            // converted: a conversion right behind each (conditional) row load costs one memory round trip per fragment
            uint4 wb[UPFRONT ? G : 2][KBW];
            const uint4* wp = Wp + ((size_t)tg * kblks + kb0) * 64 + lane;
#pragma unroll
            for (int j = 0; j < KBW; ++j)
                if (j < nkb) wb[0][j] = wp[(size_t)j * 64]; else wb[0][j] = make_uint4(0, 0, 0, 0);
            if constexpr (UPFRONT) {
#pragma unroll
                for (int g = 1; g < G; ++g) {
                    const uint4* wn = wp + (size_t)min(g, ng - 1) * kblks * 64;      // tiles beyond the group: a clamped (unused) one
#pragma unroll
                    for (int j = 0; j < KBW; ++j)
                        if (j < nkb) wb[g][j] = wn[(size_t)j * 64]; else wb[g][j] = make_uint4(0, 0, 0, 0);
                }
            }
            ARaw<WT> raw[T][KBW];
#pragma unroll
            for (int tt = 0; tt < T; ++tt)
#pragma unroll
                for (int j = 0; j < KBW; ++j) load_afrag_raw(raw[tt][j], A, lda, M, tt, min(kb0 + j, kblks - 1), lane);
            afrag_t af[T][KBW];
#pragma unroll
            for (int tt = 0; tt < T; ++tt)
#pragma unroll
                for (int j = 0; j < KBW; ++j) make_afrag(af[tt][j], raw[tt][j], M, tt, j < nkb, lane);
#pragma unroll
            for (int g = 0; g < G; ++g) {
                if (g < ng) {
                    if constexpr (!UPFRONT) {
                        if (g + 1 < ng) {
                            const uint4* wn = wp + (size_t)(g + 1) * kblks * 64;
#pragma unroll
                            for (int j = 0; j < KBW; ++j)
                                if (j < nkb) wb[(g + 1) & 1][j] = wn[(size_t)j * 64]; else wb[(g + 1) & 1][j] = make_uint4(0, 0, 0, 0);
                        }
                    }
#pragma unroll
                    for (int j = 0; j < KBW; ++j)
#pragma unroll
                        for (int tt = 0; tt < T; ++tt) mfma_block(acc[g][tt], af[tt][j], wb[UPFRONT ? g : (g & 1)][j]);
                }
            }
        }
        // cross-wave reduction through LDS: red[wave][g][tt][lane][r]
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int tt = 0; tt < T; ++tt) {
                float* dst = red + ((((size_t)wave * G + g) * T + tt) * 64 + lane) * RPL;
                if constexpr (RPL == 2) {
                    dst[0] = acc[g][tt][0] + acc[g][tt][2];          // hi + lo of real row 2a
                    dst[1] = acc[g][tt][1] + acc[g][tt][3];          // hi + lo of real row 2a+1
                } else {
                    dst[0] = acc[g][tt][0]; dst[1] = acc[g][tt][1]; dst[2] = acc[g][tt][2]; dst[3] = acc[g][tt][3];
                }
            }
        __syncthreads();
        constexpr int PER_WAVE = G * T * 64 * RPL;
        for (int idx = threadIdx.x; idx < PER_WAVE; idx += NW * 64) {
            float s = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) s += red[(size_t)w * PER_WAVE + idx];
            const int r = idx % RPL;
            const int ln = (idx / RPL) & 63;
            const int tt = (idx / (RPL * 64)) % T;
            const int g = idx / (RPL * 64 * T);
            const int row = tt * TR::ROWS + RPL * (ln >> 4) + r;
            const int col = (tg + g) * 16 + (ln & 15);
            if (g < ng && row < M) {
                float* y = Y + (size_t)row * ldy + col;
                *y = (epi == EPI_ACCUM) ? (*y + s) : s;
            }
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------------------------------
// Tall GEMM for prefill (hundreds to thousands of rows; a true dense contraction -> MFMA bound).
// The activation rows are first converted once into MFMA A fragments (bf16 hi/lo split, 8 real rows
// per 16-row tile, same layout as load_afrag) and stored as [row tile][K block][64 lanes] x 16 bytes,
// the mirror image of the weights' streaming layout.  Each wavefront then owns RT row tiles x CT column
// tiles and walks K, loading RT + CT fragments (16 bytes per lane each, fully coalesced) per RT*CT MFMAs;
// the 4 wavefronts of a workgroup form a 2 x 2 arrangement so that neighbours share fragments through L1.
// ------------------------------------------------------------------------------------------
__global__ void pack_afrag_kernel(const float* __restrict__ A, int lda, int M, int kblks, uint4* __restrict__ out) {
    const int row_tiles = (M + 7) / 8;
    const size_t total = (size_t)row_tiles * kblks * 64;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
        const int lane = (int)(idx & 63);
        const size_t blk = idx >> 6;
        const int kb = (int)(blk % (size_t)kblks), tt = (int)(blk / (size_t)kblks);
        bf16x8_t f;
        load_afrag(f, A, lda, M, tt, kb, lane);
        out[idx] = __builtin_bit_cast(uint4, f);
    }
}

// 8 consecutive values x[0..8) of row `row` at k0 (a multiple of 8) -> the two fragment chunks (high and low parts)
__device__ __forceinline__ void store_afrag8(uint4* __restrict__ frag, int kblks, int row, int k0, const float (&x)[8], bool zero) {
    const int tt = row >> 3, rr = row & 7, i_hi = 4 * (rr >> 1) + (rr & 1);
    const size_t base = ((size_t)tt * kblks + (k0 >> 5)) * 64 + ((k0 >> 3) & 3) * 16;
    uint32_t hi[4], lo[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        f32_to_bf16x2_hilo(x[2 * e], x[2 * e + 1], hi[e], lo[e]);
        if (zero) { hi[e] = 0u; lo[e] = 0u; }
    }
    frag[base + i_hi] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
    frag[base + i_hi + 2] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
}

// Tall GEMM of the prefill: a workgroup of 2 x 2 wavefronts computes 8 row tiles x 2*CTW column tiles (64 real rows x
// 32*CTW columns); each wavefront owns 4 x CTW MFMA tiles.  Per K block the workgroup copies the 8 A blocks and 2*CTW B blocks
// (1 KiB each, already in fragment order) from global memory to LDS once, and the wavefronts read their fragments with
// 128-bit LDS reads (lane-contiguous: conflict-free), so the L1 sees each block once per workgroup instead of once per
// wavefront (a register-only version, 8 fragment loads per 16 MFMAs per wavefront, was bound by L1 fill bandwidth).
// Two LDS stages; the global loads of K block k+1 are in flight while block k is multiplied; one LDS-only barrier per block.
typedef unsigned v4u_t __attribute__((ext_vector_type(4)));
template <int CTW, int NSET = 2, int RTW = 4>
__global__ __launch_bounds__(256, 2) void gemm_tall_lds_kernel(const v4u_t* __restrict__ Af, int row_tiles, int kblks,
                                                             const v4u_t* __restrict__ Wp, int ntiles, float* __restrict__ Y,
                                                             int ldy, int M, int ksplit, float* __restrict__ part) {
    // RTW = row tiles per wavefront: 4 (64 real rows per workgroup), or 2 for passes of at most 32 rows
    constexpr int NA = 2 * RTW, NB = 2 * CTW;    // A / B blocks per K block and workgroup
    constexpr int NBLK = NA + NB;
    constexpr int PER_WAVE = NBLK / 4;           // blocks each wavefront copies per K block
    static_assert(NBLK % 4 == 0, "blocks are dealt evenly to the 4 wavefronts");
    extern __shared__ __align__(16) v4u_t tall_lds[];      // [2 stages][NBLK][64]
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wr = wave >> 1, wc = wave & 1;
    // 1-D grid, XCD-aware: workgroup L runs on XCD L % 8 (round-robin dispatch) and each XCD has its own L2.  The nrow
    // workgroups that share one block of weight columns are given consecutive slots of ONE XCD, so the weights come
    // from HBM once and from that L2 nrow-1 times (with a plain 2-D grid every XCD fetched its own copy: 10x the bytes).
    // ksplit > 1 (few rows, weight-streaming regime): the K range is cut into ksplit slices, one workgroup each, so that
    // enough workgroups stream the weights; slice s writes its partial sums to part[s][M][ldy] and a second kernel adds them.
    const int ncol = (ntiles + NB - 1) / NB, nrow = (row_tiles + NA - 1) / NA;
    const int split = blockIdx.x % ksplit, bid = blockIdx.x / ksplit;
    const int xcd = bid % 8, slot = bid / 8;
    const int cblk = 8 * (slot / nrow) + xcd, rblk = slot % nrow;
    if (cblk >= ncol) return;
    const int kper = (kblks + ksplit - 1) / ksplit, kb0 = split * kper;
    const int nkb = min(kblks, kb0 + kper) - kb0;            // >= 1: the host picks ksplit so that no slice is empty
    if (nkb <= 0) return;
    if (ksplit > 1) Y = part + (size_t)split * M * ldy;
    const int rt_wg = rblk * NA, ct_wg = cblk * NB;
    // the blocks this wavefront copies: block id b = wave + 4 i; b < NA is an A block (row tile rt_wg + b), else a B block
    const v4u_t* src[PER_WAVE];
#pragma unroll
    for (int i = 0; i < PER_WAVE; ++i) {
        const int b = wave + 4 * i;
        // out-of-range tiles are replaced by in-range ones (clamped index); their results are never stored
        src[i] = (b < NA) ? Af + ((size_t)min(rt_wg + b, row_tiles - 1) * kblks + kb0) * 64 + lane
                          : Wp + ((size_t)min(ct_wg + (b - NA), ntiles - 1) * kblks + kb0) * 64 + lane;
    }
    f32x4_t acc[RTW][CTW];
#pragma unroll
    for (int r = 0; r < RTW; ++r)
#pragma unroll
        for (int c = 0; c < CTW; ++c) acc[r][c] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    // Global loads run NSET K blocks ahead of the multiplication: block kb+1 waits in register set (kb+1) % NSET while
    // blocks kb+2 .. kb+NSET are in flight in the other sets.  NSET = 2 for the prefill (one block is ~0.4 us of MFMA
    // work, a little less than an L2 round trip); NSET = 4 in the few-row weight-streaming regime, where the MFMA work
    // per block is small and the bytes in flight per workgroup set the bandwidth.
    v4u_t st[NSET][PER_WAVE];
#pragma unroll
    for (int i = 0; i < PER_WAVE; ++i) st[0][i] = src[i][0];
#pragma unroll
    for (int i = 0; i < PER_WAVE; ++i) tall_lds[(size_t)(wave + 4 * i) * 64 + lane] = st[0][i];
#pragma unroll
    for (int b = 1; b <= NSET; ++b) {
        if (b < nkb) {
#pragma unroll
            for (int i = 0; i < PER_WAVE; ++i) st[b % NSET][i] = src[i][(size_t)b * 64];
        }
    }
    lds_barrier();
    for (int kb0_ = 0; kb0_ < nkb; kb0_ += NSET) {
#pragma unroll
        for (int u = 0; u < NSET; ++u) {
            // one K block: multiply block kb from its LDS stage, park block kb+1 (register set (u+1) % NSET) in the other
            // stage, request block kb+1+NSET into that set
            const int kb = kb0_ + u;
            if (kb < nkb) {
                const v4u_t* cur = tall_lds + (size_t)(kb & 1) * NBLK * 64;
                v4u_t* nxt = tall_lds + (size_t)((kb + 1) & 1) * NBLK * 64;
                v4u_t a[RTW], b[CTW];
#pragma unroll
                for (int r = 0; r < RTW; ++r) a[r] = cur[(size_t)(wr * RTW + r) * 64 + lane];
#pragma unroll
                for (int c = 0; c < CTW; ++c) b[c] = cur[(size_t)(NA + wc * CTW + c) * 64 + lane];
#pragma unroll
                for (int r = 0; r < RTW; ++r)
#pragma unroll
                    for (int c = 0; c < CTW; ++c)
                        acc[r][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a[r]), __builtin_bit_cast(bf16x8_t, b[c]), acc[r][c], 0, 0, 0);
                if (kb + 1 < nkb) {
#pragma unroll
                    for (int i = 0; i < PER_WAVE; ++i) nxt[(size_t)(wave + 4 * i) * 64 + lane] = st[(u + 1) % NSET][i];
                    if (kb + 1 + NSET < nkb) {
#pragma unroll
                        for (int i = 0; i < PER_WAVE; ++i) st[(u + 1) % NSET][i] = src[i][(size_t)(kb + 1 + NSET) * 64];
                    }
                }
                lds_barrier();
            }
        }
    }
    const int j = lane & 15, a4 = lane >> 4;
#pragma unroll
    for (int r = 0; r < RTW; ++r) {
        const int rt = rt_wg + wr * RTW + r;
        if (rt >= row_tiles) continue;
        const int row = rt * 8 + 2 * a4;
#pragma unroll
        for (int c = 0; c < CTW; ++c) {
            const int ct = ct_wg + wc * CTW + c;
            if (ct >= ntiles) continue;
            const int col = ct * 16 + j;
            if (row < M) Y[(size_t)row * ldy + col] = acc[r][c][0] + acc[r][c][2];
            if (row + 1 < M) Y[(size_t)(row + 1) * ldy + col] = acc[r][c][1] + acc[r][c][3];
        }
    }
}

// Tall GEMM, large tile: a workgroup of 2 x 2 wavefronts computes 16 row tiles x 16 column tiles (128 real rows x 256
// columns), each wavefront 8 x 8 MFMA tiles whose 256 accumulator registers leave room for ONE wavefront per SIMD, so
// the wavefront has to overlap its own latencies.  Step kb (one K block): park block kb+2 in LDS (three stages), request
// block kb+5 from memory into the register set that just became free (three sets: a block has three steps to arrive),
// read the A fragments of block kb+1 into the second fragment set, all spread over the 64 MFMAs of block kb, whose
// operands were read earlier; one LDS-only barrier per step.  The steps are branch-free (so that the
// loads in flight can be counted) and unrolled by six (register sets are static); past the last K block they multiply a
// block of zeros (`zero`, 1 KiB) instead.
template <int CTW>
__global__ __launch_bounds__(256, 1) void gemm_tall_big_kernel(const v4u_t* __restrict__ Af, int row_tiles, int kblks,
                                                             const v4u_t* __restrict__ Wp, int ntiles, float* __restrict__ Y,
                                                             int ldy, int M, const v4u_t* __restrict__ zero) {
    constexpr int RTW = 8, NA = 2 * RTW, NB = 2 * CTW, NBLK = NA + NB, PER_WAVE = NBLK / 4;
    static_assert(NBLK % 4 == 0, "blocks are dealt evenly to the 4 wavefronts");
    extern __shared__ __align__(16) v4u_t big_lds[];       // [3 stages][NBLK][64]
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wr = wave >> 1, wc = wave & 1;
    // XCD-aware 1-D grid (workgroup L runs on XCD L % 8, one workgroup per CU, 32 CUs per XCD): the workgroups an XCD runs
    // at one time form a compact patch of RB row blocks x CB column blocks, so that per K block the XCD's L2 is asked for
    // RB + CB different 16 KiB operand blocks instead of ~RB * CB (with one column block per XCD, every activation block
    // came from beyond the L2 for a single use).  The weights of a column block are then fetched by nrow / RB XCDs, which
    // HBM has room for in this compute-bound regime.  Patch p of the (row, column) block space goes to XCD p % 8.
    const int ncol = (ntiles + NB - 1) / NB, nrow = (row_tiles + NA - 1) / NA;
    const int npr_ = (nrow + 7) / 8, RB = (nrow + npr_ - 1) / npr_, CB = max(1, 32 / RB), S = RB * CB;    // row blocks dealt evenly to the patches
    const int prow = (nrow + RB - 1) / RB;
    const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
    const int patch = (slot / S) * 8 + xcd, within = slot % S;
    const int rblk = (patch % prow) * RB + within % RB, cblk = (patch / prow) * CB + within / RB;
    if (cblk >= ncol || rblk >= nrow) return;
    const int rt_wg = rblk * NA, ct_wg = cblk * NB;
    const v4u_t* src[PER_WAVE];
#pragma unroll
    for (int i = 0; i < PER_WAVE; ++i) {
        const int b = wave + 4 * i;
        // (wavefront-uniform: the lane is added at the access, so the bases stay in scalar registers)
        src[i] = (b < NA) ? Af + ((size_t)min(rt_wg + b, row_tiles - 1) * kblks) * 64
                          : Wp + ((size_t)min(ct_wg + (b - NA), ntiles - 1) * kblks) * 64;
    }
    f32x4_t acc[RTW][CTW];
#pragma unroll
    for (int r = 0; r < RTW; ++r)
#pragma unroll
        for (int c = 0; c < CTW; ++c) acc[r][c] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    v4u_t st[3][PER_WAVE];                  // blocks on their way from memory to LDS: block j waits in set j % 3
    // A fragments of the block being multiplied (set kb % 2) and of the next one; the B fragments are single-buffered (a
    // second set does not fit beside three staging sets): each is read two columns before the column that uses it, and
    // the MFMAs run column-major
    v4u_t fa[2][RTW], fb[CTW];
#define HIVIS_BIG_LOAD(set_, blk_)                                                                         \
    {                                                                                                      \
        const int j_ = (blk_);                                                                             \
        _Pragma("unroll") for (int i = 0; i < PER_WAVE; ++i) { const v4u_t* p_ = (j_ < kblks) ? src[i] + (size_t)j_ * 64 : zero; st[set_][i] = p_[lane]; } \
    }
#define HIVIS_BIG_PARK(set_, stage_)                                                                       \
    {                                                                                                      \
        v4u_t* dst_ = big_lds + (size_t)(stage_) * NBLK * 64;                                               \
        _Pragma("unroll") for (int i = 0; i < PER_WAVE; ++i) dst_[(size_t)(wave + 4 * i) * 64 + lane] = st[set_][i]; \
    }
#define HIVIS_BIG_AFRAGS(fs_, stage_)                                                                      \
    {                                                                                                      \
        const v4u_t* s_ = big_lds + (size_t)(stage_) * NBLK * 64;                                           \
        _Pragma("unroll") for (int r = 0; r < RTW; ++r) fa[fs_][r] = s_[(size_t)(wr * RTW + r) * 64 + lane]; \
    }
    // prologue: blocks 0 and 1 into stages 0 and 1, blocks 2, 3, 4 requested, fragments of block 0 read
    HIVIS_BIG_LOAD(0, 0)
    HIVIS_BIG_LOAD(1, 1)
    HIVIS_BIG_PARK(0, 0)
    HIVIS_BIG_PARK(1, 1)
    HIVIS_BIG_LOAD(2, 2)
    HIVIS_BIG_LOAD(0, 3)
    HIVIS_BIG_LOAD(1, 4)
    lds_barrier();
    HIVIS_BIG_AFRAGS(0, 0)
    fb[0] = big_lds[(size_t)(NA + wc * CTW + 0) * 64 + lane];
    fb[1] = big_lds[(size_t)(NA + wc * CTW + 1) * 64 + lane];
    // nothing may be pending on the LDS counter when the loop is entered: inside it the fragments read during one step
    // are only awaited at that step's barrier, after its MFMAs have been issued
    lds_barrier();
    int stage2 = 2, stage1 = 1, stage0 = 0; // (kb + 2) % 3, (kb + 1) % 3, kb % 3
    for (int kb0 = 0; kb0 < kblks; kb0 += 6) {
#pragma unroll
        for (int u = 0; u < 6; ++u) {
            const int kb = kb0 + u;
            // The step's memory instructions are spread over its MFMAs, one of each kind per column of 8 MFMAs (issued in
            // one lump at the start they kept the matrix pipeline idle: a lone wavefront issues nothing else meanwhile):
            //   park piece c of block kb+2 in its stage (last read, as block kb-1, two barriers ago), request the same
            //   piece of block kb+5 into the freed registers, read A fragment c of block kb+1 (in LDS since the previous
            //   barrier) and the B fragment needed two columns later (of block kb+1 for the last two columns).
            const v4u_t* s0_ = big_lds + (size_t)stage0 * NBLK * 64;
            const v4u_t* s1_ = big_lds + (size_t)stage1 * NBLK * 64;
            v4u_t* s2_ = big_lds + (size_t)stage2 * NBLK * 64;
            const v4u_t* nsrc_[PER_WAVE];
#pragma unroll
            for (int i = 0; i < PER_WAVE; ++i) nsrc_[i] = (kb + 5 < kblks) ? src[i] + (size_t)(kb + 5) * 64 : zero;
#pragma unroll
            for (int c = 0; c < CTW; ++c) {
                static_assert(CTW == PER_WAVE && RTW == CTW, "one piece of every kind per column");
                s2_[(size_t)(wave + 4 * c) * 64 + lane] = st[(u + 2) % 3][c];
                st[(u + 2) % 3][c] = nsrc_[c][lane];
                fa[(u + 1) % 2][c] = s1_[(size_t)(wr * RTW + c) * 64 + lane];
                fb[(c + 2) % CTW] = (c + 2 < CTW ? s0_ : s1_)[(size_t)(NA + wc * CTW + (c + 2) % CTW) * 64 + lane];
#pragma unroll
                for (int r = 0; r < RTW; ++r)
                    // accumulators pinned to the accumulation registers (the register allocator otherwise keeps them in
                    // ordinary registers and copies each tile in and out around every MFMA)
                    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[r][c]) : "v"(fa[u % 2][r]), "v"(fb[c]));
                __builtin_amdgcn_sched_barrier(0);
            }
            lds_barrier();
            stage0 = stage1; stage1 = stage2; stage2 = (stage2 == 2) ? 0 : stage2 + 1;
        }
    }
#undef HIVIS_BIG_LOAD
#undef HIVIS_BIG_PARK
#undef HIVIS_BIG_AFRAGS
    // the last MFMA results are read below by ordinary moves: let the matrix pipeline drain first (the compiler does not
    // see an MFMA inside the asm statements, so it inserts no wait states of its own)
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
    const int j = lane & 15, a4 = lane >> 4;
#pragma unroll
    for (int r = 0; r < RTW; ++r) {
        const int rt = rt_wg + wr * RTW + r;
        if (rt >= row_tiles) continue;
        const int row = rt * 8 + 2 * a4;
#pragma unroll
        for (int c = 0; c < CTW; ++c) {
            const int ct = ct_wg + wc * CTW + c;
            if (ct >= ntiles) continue;
            const int col = ct * 16 + j;
            if (row < M) Y[(size_t)row * ldy + col] = acc[r][c][0] + acc[r][c][2];
            if (row + 1 < M) Y[(size_t)(row + 1) * ldy + col] = acc[r][c][1] + acc[r][c][3];
        }
    }
}

// Y[r][c] = sum over the K slices of part[s][r][c] (fixed order), r < M, c < N (N a multiple of 4).
__global__ void splitk_reduce_kernel(const float* __restrict__ part, int ksplit, int M, int N, int ldp, float* __restrict__ Y, int ldy) {
    const int row = blockIdx.x;
    for (int c4 = blockIdx.y * blockDim.x + threadIdx.x; c4 < N / 4; c4 += gridDim.y * blockDim.x) {
        float4 acc = *reinterpret_cast<const float4*>(part + (size_t)row * ldp + 4 * c4);
        for (int s = 1; s < ksplit; ++s) {
            const float4 v = *reinterpret_cast<const float4*>(part + ((size_t)s * M + row) * ldp + 4 * c4);
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
        *reinterpret_cast<float4*>(Y + (size_t)row * ldy + 4 * c4) = acc;
    }
}

// ------------------------------------------------------------------------------------------
// Row-wise small kernels (activations are a few rows of fp32; these are launch-bound, not
// bandwidth-bound)
// ------------------------------------------------------------------------------------------
// Cross-lane reductions with DPP (data-parallel primitives: the operand of a VALU instruction is taken from
// another lane of the same row of 16 lanes, or broadcast from the previous row) instead of ds_bpermute, which
// goes through the LDS crossbar and costs an LDS round trip per step.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_move(float keep, float src) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(keep), __float_as_int(src), CTRL, ROW_MASK, 0xF, false));
}
constexpr int DPP_QUAD_XOR1 = 0xB1;      // quad_perm [1,0,3,2]
constexpr int DPP_QUAD_XOR2 = 0x4E;      // quad_perm [2,3,0,1]
constexpr int DPP_ROW_ROR4 = 0x124, DPP_ROW_ROR8 = 0x128;
constexpr int DPP_ROW_BCAST15 = 0x142, DPP_ROW_BCAST31 = 0x143;

// all 4 lanes of a quad get the quad's sum
__device__ __forceinline__ float quad_sum(float v) {
    v += dpp_move<DPP_QUAD_XOR1, 0xF>(v, v);
    v += dpp_move<DPP_QUAD_XOR2, 0xF>(v, v);
    return v;
}
// Every lane gets the reduction over all 64 lanes: quad, row of 16 (two rotations), then row 0 -> 1 and 2 -> 3
// (row_bcast:15 into rows 1,3), then rows 0-1 -> 2,3 (row_bcast:31), and lane 63 is read back.
__device__ __forceinline__ float wave_sum(float v) {
    v = quad_sum(v);
    v += dpp_move<DPP_ROW_ROR4, 0xF>(v, v);
    v += dpp_move<DPP_ROW_ROR8, 0xF>(v, v);
    v += dpp_move<DPP_ROW_BCAST15, 0xA>(0.f, v);
    v += dpp_move<DPP_ROW_BCAST31, 0xC>(0.f, v);
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp_move<DPP_QUAD_XOR1, 0xF>(v, v));
    v = fmaxf(v, dpp_move<DPP_QUAD_XOR2, 0xF>(v, v));
    v = fmaxf(v, dpp_move<DPP_ROW_ROR4, 0xF>(v, v));
    v = fmaxf(v, dpp_move<DPP_ROW_ROR8, 0xF>(v, v));
    v = fmaxf(v, dpp_move<DPP_ROW_BCAST15, 0xA>(v, v));
    v = fmaxf(v, dpp_move<DPP_ROW_BCAST31, 0xC>(v, v));
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// h[row] += delta[row] (if delta), then out[row] = h[row] * gain / sqrt(mean(h^2) + eps).
// One workgroup (256 threads) per row.  A row of up to 8192 values is held in registers (8 float4 per thread), with all
// loads of a pass issued together: a one-load-per-trip loop costs a memory round trip per trip when only a few
// workgroups run (the 32-row passes).
template <typename WT>
__global__ __launch_bounds__(256) void add_rmsnorm_kernel(float* __restrict__ h, int ldh, const float* __restrict__ delta,
                                                           int ldd, const WT* __restrict__ gain, float* __restrict__ out,
                                                           int ldo, int d, float eps) {
    __shared__ float part[4];
    constexpr int MAXV = 8;
    const int row = blockIdx.x;
    float* hr = h + (size_t)row * ldh;
    const float* dr = delta ? delta + (size_t)row * ldd : nullptr;
    float* o = out + (size_t)row * ldo;
    const int n4 = d / 4;
    if (n4 <= 256 * MAXV) {
        float4 xs[MAXV], ds[MAXV];
#pragma unroll
        for (int k = 0; k < MAXV; ++k) {
            const int c4 = min((int)threadIdx.x + 256 * k, n4 - 1);
            xs[k] = reinterpret_cast<const float4*>(hr)[c4];
            ds[k] = dr ? reinterpret_cast<const float4*>(dr)[c4] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        float ss = 0.f;
#pragma unroll
        for (int k = 0; k < MAXV; ++k) {
            const int c4 = (int)threadIdx.x + 256 * k;
            if (c4 < n4) {
                xs[k].x += ds[k].x; xs[k].y += ds[k].y; xs[k].z += ds[k].z; xs[k].w += ds[k].w;
                if (dr) reinterpret_cast<float4*>(hr)[c4] = xs[k];
                ss += xs[k].x * xs[k].x + xs[k].y * xs[k].y + xs[k].z * xs[k].z + xs[k].w * xs[k].w;
            }
        }
        ss = wave_sum(ss);
        if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
        __syncthreads();
        const float inv = 1.0f / sqrtf((part[0] + part[1] + part[2] + part[3]) / (float)d + eps);
#pragma unroll
        for (int k = 0; k < MAXV; ++k) {
            const int c4 = (int)threadIdx.x + 256 * k;
            if (c4 < n4) {
                const WT* gp = gain + 4 * c4;
                reinterpret_cast<float4*>(o)[c4] = make_float4(xs[k].x * to_f32(gp[0]) * inv, xs[k].y * to_f32(gp[1]) * inv,
                                                               xs[k].z * to_f32(gp[2]) * inv, xs[k].w * to_f32(gp[3]) * inv);
            }
        }
        return;
    }
    float ss = 0.f;
    for (int c = threadIdx.x; c < d; c += 256) {
        float x = hr[c];
        if (dr) { x += dr[c]; hr[c] = x; }
        ss += x * x;
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float tot = part[0] + part[1] + part[2] + part[3];
    const float inv = 1.0f / sqrtf(tot / (float)d + eps);
    for (int c = threadIdx.x; c < d; c += 256) o[c] = hr[c] * to_f32(gain[c]) * inv;
}

// out[row] = h[row] + delta[row]
__global__ void add_rows_kernel(const float* __restrict__ h, int ldh, const float* __restrict__ delta, int ldd,
                                float* __restrict__ out, int ldo, int d) {
    const int row = blockIdx.x;
    for (int c = threadIdx.x; c < d; c += blockDim.x)
        out[(size_t)row * ldo + c] = h[(size_t)row * ldh + c] + delta[(size_t)row * ldd + c];
}

// u[row] += rho[idx]   (residual vector of the row: step-dependent bias correction)
template <typename WT>
__global__ void add_rho_kernel(float* __restrict__ u, int ldu, const WT* __restrict__ rho, int idx, int d) {
    const int row = blockIdx.x;
    for (int c = threadIdx.x; c < d; c += blockDim.x) u[(size_t)row * ldu + c] += to_f32(rho[(size_t)idx * d + c]);
}

// act[row][c] = silu(gate c) * up c, with gate|up interleaved per 16-column tile (PACK_GATEUP order)
__global__ void silu_mul_kernel(const float* __restrict__ gu, float* __restrict__ act, int F) {
    // grid (rows, column chunks); 4 consecutive activations per thread (they share one 8-column gate group)
    const int row = blockIdx.x;
    for (int c4 = blockIdx.y * blockDim.x + threadIdx.x; c4 < F / 4; c4 += gridDim.y * blockDim.x) {
        const int c = 4 * c4;
        const size_t o = (size_t)row * 2 * F + (size_t)(c >> 3) * 16 + (c & 7);
        const float4 g = *reinterpret_cast<const float4*>(gu + o), u = *reinterpret_cast<const float4*>(gu + o + 8);
        *reinterpret_cast<float4*>(act + (size_t)row * F + c) =
            make_float4(g.x / (1.0f + expf(-g.x)) * u.x, g.y / (1.0f + expf(-g.y)) * u.y, g.z / (1.0f + expf(-g.z)) * u.z, g.w / (1.0f + expf(-g.w)) * u.w);
    }
}

// RoPE (rotate-half pairing, pairs stored in adjacent columns) on q and k of the fused qkv rows, then append k, v.
// Row r belongs to sequence seq0 + r / m and sits at position base[seq] + offset + r % m, which is
// both its rotary position and its slot in the cache.  Cache layout: [seq][Hkv][maxL][HD * KVWidth] (see KVType).
// The angle is evaluated in double so that large positions keep full fp32 accuracy.
// pos_delta (optional, rows of a draft tree): the rotary position of row r is base[seq] + pos_delta[r] instead, its
// cache slot stays base[seq] + offset + r % m.
// bias (optional): q/k/v projection biases in the column order of the fused qkv rows, added before the rotation.
template <typename ST>
__global__ void rope_append_kernel(float* __restrict__ qkv, int Hq, int Hkv, int HD, const int* __restrict__ base,
                                   int offset, int seq0, int m, ST* __restrict__ kc, ST* __restrict__ vc, int maxL,
                                   float theta, const int* __restrict__ pos_delta = nullptr, const float* __restrict__ bias = nullptr,
                                   const float* __restrict__ rope_tab = nullptr, int npos = 0) {
    // rope_tab (optional): the context's table [npos][HD/2] of (cos, sin), see rope_table_kernel; without it the angle's
    // sine and cosine are evaluated here (in double: ~100 us per layer for a 3008-row prefill)
    const int row = blockIdx.x;
    const int seq = seq0 + row / m;
    const int slot = base[seq] + offset + row % m;
    const int pos = pos_delta ? base[seq] + pos_delta[row] : slot;
    const int half = HD / 2;
    float* r = qkv + (size_t)row * (Hq + 2 * Hkv) * HD;
    const int npair = (Hq + Hkv) * half;
    for (int idx = blockIdx.y * blockDim.x + threadIdx.x; idx < npair; idx += gridDim.y * blockDim.x) {
        const int head = idx / half, i = idx % half;
        double s, c;
        if (rope_tab) {
            const float2 t = *reinterpret_cast<const float2*>(rope_tab + ((size_t)min(pos, npos - 1) * half + i) * 2);
            c = (double)t.x; s = (double)t.y;
        } else {
            const double inv_freq = exp2(-2.0 * (double)i / (double)HD * log2((double)theta));
            sincos((double)pos * inv_freq, &s, &c);
        }
        float* x = r + (size_t)head * HD;          // the pair (i, i + hd/2) sits in columns 2i, 2i+1 (PACK_QKV order)
        const float b1 = bias ? bias[(size_t)head * HD + 2 * i] : 0.f, b2 = bias ? bias[(size_t)head * HD + 2 * i + 1] : 0.f;
        const float x1 = x[2 * i] + b1, x2 = x[2 * i + 1] + b2;
        const float y1 = (float)((double)x1 * c - (double)x2 * s);
        const float y2 = (float)((double)x2 * c + (double)x1 * s);
        if (head < Hq) {
            x[2 * i] = y1; x[2 * i + 1] = y2;
        } else {
            ST* dst = kc + (((size_t)seq * Hkv + (head - Hq)) * maxL + slot) * HD * KVWidth<ST>::W;
            kv_put_pair(dst, HD, 2 * i, y1, y2);
        }
    }
    const float* v = r + (size_t)(Hq + Hkv) * HD;
    for (int idx = blockIdx.y * blockDim.x + threadIdx.x; idx < Hkv * HD / 2; idx += gridDim.y * blockDim.x) {
        const int head = (2 * idx) / HD, c = (2 * idx) % HD;
        const float b0 = bias ? bias[(size_t)(Hq + Hkv) * HD + 2 * idx] : 0.f, b1 = bias ? bias[(size_t)(Hq + Hkv) * HD + 2 * idx + 1] : 0.f;
        kv_put_pair(vc + (((size_t)seq * Hkv + head) * maxL + slot) * HD * KVWidth<ST>::W, HD, c, v[2 * idx] + b0, v[2 * idx + 1] + b1);
    }
}

// ------------------------------------------------------------------------------------------
// Uniform numbers for the sampling kernels, drawn on the device: Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11).
// One round maps the counter (c0..c3) under the round key (k0, k1) to
//   (hi(M1 c2) ^ c1 ^ k0,  lo(M1 c2),  hi(M0 c0) ^ c3 ^ k1,  lo(M0 c0));
// ten rounds, the key advancing by the two Weyl constants between rounds.  A uniform is the top 24 bits of output
// word 0 times 2^-24.  Counter = (index in the array, purpose of the array, draw-call count low, high); key = seed.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ unsigned philox4x32_10_word0(unsigned c0, unsigned c1, unsigned c2, unsigned c3, unsigned k0, unsigned k1) {
#pragma unroll
    for (int rnd = 0; rnd < 10; ++rnd) {
        if (rnd > 0) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
        const unsigned hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const unsigned hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const unsigned n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    }
    return c0;
}

// Fills up to two arrays of one sampling call: array A holds nA numbers laid out [nA / rowA][rowA] with row stride
// strideA (number i sits at (i / rowA) * strideA + i % rowA), array B holds nB numbers contiguously.
__global__ void rng_fill_kernel(float* __restrict__ uA, int nA, int rowA, int strideA, unsigned purposeA,
                                float* __restrict__ uB, int nB, unsigned purposeB,
                                unsigned key0, unsigned key1, unsigned call_lo, unsigned call_hi) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < nA) {
        const unsigned w = philox4x32_10_word0((unsigned)t, purposeA, call_lo, call_hi, key0, key1);
        uA[(size_t)(t / rowA) * strideA + t % rowA] = (float)(w >> 8) * 0x1p-24f;
    } else if (t < nA + nB) {
        const unsigned w = philox4x32_10_word0((unsigned)(t - nA), purposeB, call_lo, call_hi, key0, key1);
        uB[t - nA] = (float)(w >> 8) * 0x1p-24f;
    }
}

// ------------------------------------------------------------------------------------------
// Attention of a few query rows against a long cached K/V (verify: K+1 rows; draft: 1 row;
// prefill chunks: up to 16 rows of one head).  A work item is (sequence, kv head, a range of
// query heads of that kv head, a range of rows) with at most RMAX (head,row) pairs; it is
// processed by `nsplit` workgroups x 4 wavefronts, each wavefront taking every (4*nsplit)-th
// tile of 64 keys and writing an (unnormalised accumulator, max, sum) partial; a second kernel
// merges the partials in a fixed order.
// Query row i of a sequence sits at position base[seq] + offset + i and sees keys 0..position.
// ------------------------------------------------------------------------------------------
constexpr int ATT_RMAX = 16;

struct AttnShape {
    int Hq, Hkv, m;          // m rows per sequence in this pass
    int gh, mi;              // query heads / rows per work item (gh*mi <= ATT_RMAX)
    int n_hblk, n_rblk;      // ceil(group/gh), ceil(m/mi)
    int seq0, offset, maxL, nsplit;
    int ldq;                 // row stride of the q buffer
    int nwaves;              // wavefronts per workgroup working on one (item, split)
    int flags;               // bit 0: the election of the merging workgroup relies on agent-scope stores, loads and the
                             //        arrival counter alone (clear: an agent-scope release / acquire fence pair around it as well);
                             // bit 1: every key split of an item on one XCD (the partials meet in one L2)
    // cache lengths by value (nbase > 0): the host knows them at launch, and reading base[seq] from memory first costs the
    // attention a dependent round trip before its first key can be requested.  base_val[s] replaces base[seq0 + s].
    int nbase; int base_val[8];
    // rows of a draft tree (optional): row i sees every key before base[seq] plus the keys base[seq] + b whose bit b is
    // set in tmask[i] (its ancestors among the tree rows and itself), instead of the causal rule
    const unsigned long long* tmask;
};
// visibility of key `key` for a row with causal limit qpos (tm, tb: the row's tree mask and the tree's first slot)
__device__ __forceinline__ bool attn_visible(bool tree, int key, int qpos, unsigned long long tm, int tb) {
    if (!tree) return key <= qpos;
    return key < tb || ((unsigned)(key - tb) < 64u && ((tm >> ((key - tb) & 63)) & 1ull));
}

// LDS needed by attn_item_partial: q rows + one probability tile per wavefront
__host__ __device__ constexpr size_t attn_lds_floats(int hd, int nwaves, int rmax = ATT_RMAX) {
    return (size_t)rmax * hd + (size_t)nwaves * rmax * 64;
}

// One (item, split) by the calling workgroup of sh.nwaves wavefronts.  Partial results go to
// ws[(item * nslots + slot)][ATT_RMAX][HD + 2] with slot = wave * nsplit + split; slots beyond the
// number of key tiles have no work and write nothing.
template <typename ST, int HD, int RM>
__device__ __forceinline__ void attn_item_partial(const float* __restrict__ q, const ST* __restrict__ kc,
                                                  const ST* __restrict__ vc, const int* __restrict__ base,
                                                  const AttnShape& sh, int item_id, int split, float* __restrict__ lds,
                                                  float* __restrict__ ws) {
    constexpr int CH = 16 / sizeof(ST);          // elements per 16-byte chunk
    constexpr int DPL = HD / 64;                 // value dims per lane
    constexpr int KW = KVWidth<ST>::W;           // storage elements per value (half-precision caches: hi row | lo row)
    const int nthreads = sh.nwaves * 64;
    float* qs = lds;                                         // [RM][HD]
    float* pw_all = lds + RM * HD;                     // [nwaves][RM][64]

    int item = item_id;
    const int rblk = item % sh.n_rblk; item /= sh.n_rblk;
    const int hblk = item % sh.n_hblk; item /= sh.n_hblk;
    const int kvh = item % sh.Hkv;
    const int sl = item / sh.Hkv;                 // local sequence index
    const int seq = sh.seq0 + sl;
    const int group = sh.Hq / sh.Hkv;
    const int h0 = hblk * sh.gh, nh = min(sh.gh, group - h0);
    const int i0 = rblk * sh.mi, ni = min(sh.mi, sh.m - i0);
    const int R = nh * ni;
    const int pos0 = base[seq] + sh.offset;       // position of row 0 of this sequence
    const int nkeys = pos0 + i0 + ni;             // keys visible to the last row of the item
    const int ntiles = (nkeys + 63) / 64;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int slot = wave * sh.nsplit + split, nslots = sh.nsplit * sh.nwaves;   // consecutive tiles go to different workgroups
    const float scale = rsqrtf((float)HD);
    float* pw = pw_all + (size_t)wave * RM * 64;

    for (int idx = threadIdx.x; idx < R * HD; idx += nthreads) {
        const int r = idx / HD, c = idx % HD;
        const int hh = kvh * group + h0 + r / ni, i = i0 + r % ni;
        qs[idx] = q[(size_t)(sl * sh.m + i) * sh.ldq + (size_t)hh * HD + c] * scale;
    }
    lds_barrier();

    const ST* kbase = kc + ((size_t)seq * sh.Hkv + kvh) * sh.maxL * HD * KW;
    const ST* vbase = vc + ((size_t)seq * sh.Hkv + kvh) * sh.maxL * HD * KW;

    float mrun[RM], lrun[RM], acc[RM][DPL];
#pragma unroll
    for (int r = 0; r < RM; ++r) {
        mrun[r] = -INFINITY; lrun[r] = 0.f;
#pragma unroll
        for (int e = 0; e < DPL; ++e) acc[r][e] = 0.f;
    }

    for (int ti = slot; ti < ntiles; ti += nslots) {
        const int j = ti * 64 + lane;
        const bool valid = j < nkeys;
        float s[RM];
#pragma unroll
        for (int r = 0; r < RM; ++r) s[r] = 0.f;
        if (valid) {
            const uint4* kp = reinterpret_cast<const uint4*>(kbase + (size_t)j * HD * KW);
#pragma unroll 4
            for (int c = 0; c < HD / CH; ++c) {
                const uint4 raw = kp[c];
                float kf[CH];
                decode_chunk(raw, kf, ST());
                if constexpr (KW == 2) {             // the lo halves of the same values follow the hi row
                    float kl[CH];
                    decode_chunk(kp[HD / CH + c], kl, ST());
#pragma unroll
                    for (int e = 0; e < CH; ++e) kf[e] += kl[e];
                }
#pragma unroll
                for (int r = 0; r < RM; ++r) {
                    if (r < R) {
                        const float* qr = qs + r * HD + c * CH;
#pragma unroll
                        for (int e = 0; e < CH; ++e) s[r] += qr[e] * kf[e];
                    }
                }
            }
        }
#pragma unroll
        for (int r = 0; r < RM; ++r) {
            if (r < R) {
                const int qpos = pos0 + i0 + r % ni;
                const bool tree = sh.tmask != nullptr;
                const unsigned long long tm = tree ? sh.tmask[sl * sh.m + i0 + r % ni] : 0ull;
                const float sv = (valid && attn_visible(tree, j, qpos, tm, pos0 - sh.offset)) ? s[r] : -INFINITY;
                const float tmax = wave_max(sv);
                const float mnew = fmaxf(mrun[r], tmax);
                float alpha = 1.f, p = 0.f;
                if (mnew != -INFINITY) {
                    alpha = (mrun[r] == -INFINITY) ? 0.f : __expf(mrun[r] - mnew);
                    p = (sv == -INFINITY) ? 0.f : __expf(sv - mnew);
                }
                mrun[r] = mnew;
                lrun[r] = lrun[r] * alpha + p;
#pragma unroll
                for (int e = 0; e < DPL; ++e) acc[r][e] *= alpha;
                pw[r * 64 + lane] = p;
            }
        }
        // the probabilities of this wavefront's tile are read back by the same wavefront only
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int nk = min(64, nkeys - ti * 64);
        for (int jj = 0; jj < nk; ++jj) {
            float vf[DPL];
            const ST* vrow = vbase + (size_t)(ti * 64 + jj) * HD * KW;
#pragma unroll
            for (int e = 0; e < DPL; ++e) vf[e] = kv_get(vrow, HD, lane * DPL + e);
#pragma unroll
            for (int r = 0; r < RM; ++r) {
                if (r < R) {
                    const float p = pw[r * 64 + jj];
#pragma unroll
                    for (int e = 0; e < DPL; ++e) acc[r][e] += p * vf[e];
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    if (slot >= ntiles) return;
    float* out = ws + ((size_t)item_id * nslots + slot) * RM * (HD + 2);
#pragma unroll
    for (int r = 0; r < RM; ++r) {
        if (r < R) {
            const float lsum = wave_sum(lrun[r]);
#pragma unroll
            for (int e = 0; e < DPL; ++e) st_wt(&out[r * (HD + 2) + lane * DPL + e], acc[r][e]);
            if (lane == 0) { st_wt(&out[r * (HD + 2) + HD], mrun[r]); st_wt(&out[r * (HD + 2) + HD + 1], lsum); }
        }
    }
}

// Merge of the partials of one item by `nthreads` threads, in slot order (fixed summation order).
template <int HD, int RM>
__device__ __forceinline__ void attn_item_merge(const float* __restrict__ ws, const int* __restrict__ kvbase,
                                                const AttnShape& sh, int item_id, int nthreads, float* __restrict__ out,
                                                int ldo) {
    int item = item_id;
    const int rblk = item % sh.n_rblk; item /= sh.n_rblk;
    const int hblk = item % sh.n_hblk; item /= sh.n_hblk;
    const int kvh = item % sh.Hkv;
    const int sl = item / sh.Hkv;
    const int group = sh.Hq / sh.Hkv;
    const int h0 = hblk * sh.gh, nh = min(sh.gh, group - h0);
    const int i0 = rblk * sh.mi, ni = min(sh.mi, sh.m - i0);
    const int R = nh * ni;
    const int nkeys = kvbase[sh.seq0 + sl] + sh.offset + i0 + ni;
    const int nslots = min(sh.nsplit * sh.nwaves, (nkeys + 63) / 64);   // slots that had a key tile
    const float* base = ws + (size_t)item_id * (sh.nsplit * sh.nwaves) * RM * (HD + 2);
    for (int idx = threadIdx.x; idx < R * HD; idx += nthreads) {
        const int r = idx / HD, c = idx % HD;
        float mx = -INFINITY;
        for (int s = 0; s < nslots; ++s) mx = fmaxf(mx, base[((size_t)s * RM + r) * (HD + 2) + HD]);
        float num = 0.f, den = 0.f;
        for (int s = 0; s < nslots; ++s) {
            const float* p = base + ((size_t)s * RM + r) * (HD + 2);
            const float ms = p[HD];
            if (ms == -INFINITY) continue;
            const float w = __expf(ms - mx);
            num += p[c] * w; den += p[HD + 1] * w;
        }
        const int hh = kvh * group + h0 + r / ni, i = i0 + r % ni;
        st_wt(&out[(size_t)(sl * sh.m + i) * ldo + (size_t)hh * HD + c], num / den);
    }
}

template <typename ST, int HD>
__global__ __launch_bounds__(256) void attn_partial_kernel(const float* __restrict__ q, const ST* __restrict__ kc,
                                                            const ST* __restrict__ vc, const int* __restrict__ base,
                                                            AttnShape sh, float* __restrict__ ws) {
    __shared__ float lds[attn_lds_floats(HD, 4)];
    attn_item_partial<ST, HD, ATT_RMAX>(q, kc, vc, base, sh, blockIdx.x, blockIdx.y, lds, ws);
}

template <int HD>
__global__ __launch_bounds__(256) void attn_merge_kernel(const float* __restrict__ ws, const int* __restrict__ base,
                                                          AttnShape sh, float* __restrict__ out, int ldo) {
    attn_item_merge<HD, ATT_RMAX>(ws, base, sh, blockIdx.x, 256, out, ldo);
}

// Rotary table of a context: tab[pos][i] = (cos, sin)(pos * theta^(-2i/hd)), i < hd/2, angle evaluated in double (so that
// large positions keep full fp32 accuracy).  Written once at create; the QKV epilogue of the phase programs reads it.
__global__ void rope_table_kernel(float* __restrict__ tab, int npos, int hd, float theta) {
    const int half = hd / 2;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < (size_t)npos * half; idx += (size_t)gridDim.x * blockDim.x) {
        const int pos = (int)(idx / half), i = (int)(idx % half);
        const double inv_freq = exp2(-2.0 * (double)i / (double)hd * log2((double)theta));
        double s, c;
        sincos((double)pos * inv_freq, &s, &c);
        tab[idx * 2] = (float)c; tab[idx * 2 + 1] = (float)s;
    }
}

// ------------------------------------------------------------------------------------------
// Calibration: a plain read-only stream over a buffer, the access pattern of the weight-streaming GEMMs without any
// of their work (one wavefront reads 1 KiB per instruction, 8 independent 16-byte loads per lane and trip, a workgroup
// 64 KiB per trip).  What it reaches is the ceiling any weight-streaming kernel on this machine works under.
// n16: buffer size in 16-byte units.  The xor of everything read goes to `sink` only if it equals a value it
// cannot practically take, which keeps the loads alive.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(512) void calib_stream_kernel(const uint4* __restrict__ buf, size_t n16, unsigned* __restrict__ sink) {
    const size_t trips = n16 / 4096;                                         // 64 KiB per workgroup and trip: 8 wavefronts x 8 loads x 64 lanes
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    uint4 acc = make_uint4(0, 0, 0, 0);
    for (size_t t = blockIdx.x; t < trips; t += gridDim.x) {
        const uint4* p = buf + t * 4096 + (size_t)wave * 512 + lane;
        uint4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = p[(size_t)j * 64];
#pragma unroll
        for (int j = 0; j < 8; ++j) { acc.x ^= v[j].x; acc.y ^= v[j].y; acc.z ^= v[j].z; acc.w ^= v[j].w; }
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9E3779B9u && acc.x == 0x7F4A7C15u) *sink = acc.x;
}

// ------------------------------------------------------------------------------------------
// Token-level kernels
// ------------------------------------------------------------------------------------------
// Token id forced into [0, V-1] (an id outside it can only come from a row without a greedy token, see argmax_kernel)
__host__ __device__ __forceinline__ int clamp_token(int id, int V) { return id < 0 ? 0 : (id >= V ? V - 1 : id); }
// Greedy token per row: index of the largest logit, lowest index on ties.  One workgroup per row.
// A row in which no logit compares greater than -inf (all NaN, or all -inf) has no greedy token: the stored id is
// clamped into [0, V-1] so that nothing downstream indexes a table out of bounds, and *bad (if given) is set to 1.
__global__ __launch_bounds__(256) void argmax_kernel(const float* __restrict__ logits, int V, int32_t* __restrict__ out,
                                                      int out_stride, int* __restrict__ bad) {
    __shared__ float bv[4];
    __shared__ int bi[4];
    const int row = blockIdx.x;
    const float* l = logits + (size_t)row * V;
    float best = -INFINITY; int besti = 0x7FFFFFFF;
    // eight independent loads per trip (a one-load-per-trip loop pays a memory round trip per trip: 39 us for the 61
    // rows of a tree verify pass); a thread still sees its columns in ascending order, so ties keep the lowest index
    constexpr int U = 8;
    for (int c0 = threadIdx.x; c0 < V; c0 += 256 * U) {
        float x[U];
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = l[min(c0 + 256 * u, V - 1)];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = c0 + 256 * u;
            if (c < V && (x[u] > best || (x[u] == best && c < besti))) { best = x[u]; besti = c; }
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(best, o, 64); const int oi = __shfl_xor(besti, o, 64);
        if (ov > best || (ov == best && oi < besti)) { best = ov; besti = oi; }
    }
    if ((threadIdx.x & 63) == 0) { bv[threadIdx.x >> 6] = best; bi[threadIdx.x >> 6] = besti; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 4; ++w)
            if (bv[w] > best || (bv[w] == best && bi[w] < besti)) { best = bv[w]; besti = bi[w]; }
        if (bad && (unsigned)besti >= (unsigned)V) *bad = 1;
        out[(size_t)row * out_stride] = clamp_token(besti, V);
    }
}

// dst[i] = src[i] widened to fp32 (a range of embedding rows, as the A operand of the GEMM that folds the embedding half
// of the fusion FC into a table)
template <typename WT>
__global__ void rows_to_f32_kernel(const WT* __restrict__ src, size_t n, float* __restrict__ dst) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) dst[i] = to_f32(src[i]);
}

// rows[r][0..d) = table[ids[r]]  (embedding gather, converted to fp32)
template <typename WT>
__global__ void gather_rows_kernel(const WT* __restrict__ table, const int32_t* __restrict__ ids, int id_stride,
                                   float* __restrict__ out, int ldo, int d) {
    const int row = blockIdx.x;
    const WT* src = table + (size_t)ids[(size_t)row * id_stride] * d;
    for (int c = threadIdx.x; c < d; c += blockDim.x) out[(size_t)row * ldo + c] = to_f32(src[c]);
}

// Prefill input rows of one sequence: position p < v -> visual embedding p, else Embed(text[p - v]).
template <typename WT>
__global__ void prefill_rows_kernel(const WT* __restrict__ vis, int v, const WT* __restrict__ table,
                                    const int32_t* __restrict__ text, int p0, float* __restrict__ out, int d) {
    const int p = p0 + blockIdx.x;
    const WT* src = (p < v) ? vis + (size_t)p * d : table + (size_t)text[p - v] * d;
    for (int c = threadIdx.x; c < d; c += blockDim.x) out[(size_t)blockIdx.x * d + c] = to_f32(src[c]);
}

// Fusion input rows [f_j ; Embed(x_{j+1})] for drafter prefill rows j0.. of one sequence.
template <typename WT>
__global__ void fuse_rows_kernel(const float* __restrict__ feat, const WT* __restrict__ table,
                                 const int32_t* __restrict__ text, int j0, float* __restrict__ cat, int d) {
    const int j = j0 + blockIdx.x;
    const float* f = feat + (size_t)j * d;
    const WT* e = table + (size_t)text[j + 1] * d;
    float* o = cat + (size_t)blockIdx.x * 2 * d;
    for (int c = threadIdx.x; c < d; c += blockDim.x) { o[c] = f[c]; o[d + c] = to_f32(e[c]); }
}

// Verify input tokens: row 0 of sequence b = last known text token, rows 1..K = its drafts.
__global__ void verify_tokens_kernel(const int32_t* __restrict__ text, int text_stride, const int* __restrict__ dlen,
                                     const int32_t* __restrict__ drafts, int kmax, int K, int32_t* __restrict__ rows,
                                     int B) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= B * (K + 1)) return;
    const int b = idx / (K + 1), i = idx % (K + 1);
    rows[idx] = (i == 0) ? text[(size_t)b * text_stride + dlen[b]] : drafts[b * kmax + i - 1];
}

// Greedy acceptance: one wavefront per sequence.  Lane i < K compares draft i with the target's
// token for the same position; the accepted length is the number of leading matches, read off
// the ballot mask.  Also emits tokens, appends them to the text, advances the target length and
// prepares the tokens that follow each re-fed row.
__global__ __launch_bounds__(64) void accept_kernel(const int32_t* __restrict__ drafts, const int32_t* __restrict__ tt,
                                                     int kmax, int K, int32_t* __restrict__ text, int text_stride,
                                                     const int* __restrict__ dlen, int* __restrict__ tlen,
                                                     int32_t* __restrict__ nacc, int32_t* __restrict__ out_tokens,
                                                     int32_t* __restrict__ next_tok) {
    const int b = blockIdx.x, lane = threadIdx.x;
    const bool match = (lane < K) ? (drafts[b * kmax + lane] == tt[b * (kmax + 1) + lane]) : false;
    const unsigned long long mism = ~__ballot(match);
    const int n = min(K, (int)__builtin_ctzll(mism | (1ull << 63)));
    if (lane <= kmax) {
        int tok = -1;
        if (lane < n) tok = drafts[b * kmax + lane];
        else if (lane == n) tok = tt[b * (kmax + 1) + n];
        out_tokens[b * (kmax + 1) + lane] = tok;
        if (lane <= n) text[(size_t)b * text_stride + dlen[b] + 1 + lane] = tok;
        if (lane <= K) {
            const int e = min(lane, n);
            next_tok[b * (kmax + 1) + lane] = (e < n) ? drafts[b * kmax + e] : tt[b * (kmax + 1) + n];
        }
    }
    if (lane == 0) { nacc[b] = n; tlen[b] += n + 1; }
}

// ------------------------------------------------------------------------------------------
// Temperature sampling (section 2.1 at T > 0; the speculative sampling rule of the works it cites).
// The uniform random numbers are inputs.  One workgroup of NT threads works on one row of V logits; every sum has
// one fixed order (bit-reproducible).
// ------------------------------------------------------------------------------------------
template <int NT>
__device__ __forceinline__ float block_reduce_max(float v, float* sm) {
    v = wave_max(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = sm[0];
#pragma unroll
    for (int w = 1; w < NT / 64; ++w) r = fmaxf(r, sm[w]);
    return r;
}
// maximum of x[j] * it over one row, 8 independent loads per trip
template <int NT>
__device__ __forceinline__ float block_row_max(const float* __restrict__ x, int V, float it, float* sm) {
    float m = -INFINITY;
    for (int j = threadIdx.x; j < V; j += NT * 8) {
        float x8[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) x8[k] = x[min(j + NT * k, V - 1)];
#pragma unroll
        for (int k = 0; k < 8; ++k) m = fmaxf(m, x8[k] * it);       // clamped duplicates of the last element do not change a maximum
    }
    return block_reduce_max<NT>(m, sm);
}
template <int NT>
__device__ __forceinline__ int block_reduce_min_int(int v, int* sm) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = min(v, __shfl_xor(v, o, 64));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
    __syncthreads();
    int r = sm[0];
#pragma unroll
    for (int w = 1; w < NT / 64; ++w) r = min(r, sm[w]);
    return r;
}
// Index drawn by inversion from the non-negative weights wf(j), j in [0, V): the smallest j whose running sum
// exceeds u * total; if rounding leaves none, the last index with a positive weight.  All threads return the index.
// Wavefront w owns the contiguous segment [w*L, (w+1)*L) (L a multiple of 64) and reads it 64 consecutive elements
// at a time (coalesced).  Pass A: segment totals.  Pass B: the wavefront whose segment contains the target walks it
// again, 64 elements per step, with an in-order wavefront scan, and takes the first lane whose prefix exceeds it.
template <int NT, typename WF>
__device__ __forceinline__ int block_sample_inverse_cdf(WF wf, int V, float u, float* smf, int* smi) {
    constexpr int NWV = NT / 64;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int L = ((V + NWV * 64 - 1) / (NWV * 64)) * 64;
    const int s0 = min(wave * L, V), s1 = min(s0 + L, V);
    float part = 0.f;
    int last_pos = -1;
    // (8 independent loads per trip: a one-load-per-trip loop pays a memory round trip per element)
    for (int j = s0 + lane; j < s1; j += 64 * 8) {
        float w8[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) w8[k] = wf(min(j + 64 * k, V - 1));
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            if (j + 64 * k < s1) { part += w8[k]; if (w8[k] > 0.f) last_pos = j + 64 * k; }
        }
    }
    const float tw = wave_sum(part);
    __syncthreads();
    if (lane == 0) smf[wave] = tw;
    __syncthreads();
    float base = 0.f, total = 0.f;
#pragma unroll
    for (int w = 0; w < NWV; ++w) { if (w < wave) base += smf[w]; total += smf[w]; }
    const float target = u * total;
    int wsel = -1;
    {
        float run = 0.f;
#pragma unroll
        for (int w = 0; w < NWV; ++w) { run += smf[w]; if (wsel < 0 && run > target) wsel = w; }
    }
    int found = 0x7FFFFFFF;
    if (wave == wsel) {
        float run = base;
        for (int r = s0; r < s1; r += 64) {
            const int j = r + lane;
            const float w = (j < s1) ? wf(j) : 0.f;
            float incl = w;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const float up = __shfl_up(incl, o, 64);
                if (lane >= o) incl += up;
            }
            const unsigned long long hit = __ballot(run + incl > target && j < s1);
            if (hit) { found = r + (int)__builtin_ctzll(hit); break; }
            run += __shfl(incl, 63, 64);
        }
        if (found == 0x7FFFFFFF) {            // rounding: the segment total said "here", the in-order walk did not get there
            int lp = last_pos;
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) lp = max(lp, __shfl_xor(lp, o, 64));
            if (lp >= 0) found = lp;
        }
    }
    found = block_reduce_min_int<NT>(found, smi);
    if (found == 0x7FFFFFFF) found = -block_reduce_min_int<NT>(-last_pos, smi);     // maximum of last_pos over the row
    return min(max(found, 0), V - 1);
}

// softmax statistics of one row at inverse temperature it: maximum of x*it and the sum of exp(x*it - max)
template <int NT>
__device__ __forceinline__ void block_softmax_stats(const float* __restrict__ x, int V, float it, float* smf, float* mx, float* sum) {
    float m = block_row_max<NT>(x, V, it, smf);
    float s = 0.f;
    for (int j = threadIdx.x; j < V; j += NT * 8) {
        float x8[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) x8[k] = x[min(j + NT * k, V - 1)];
#pragma unroll
        for (int k = 0; k < 8; ++k) if (j + NT * k < V) s += expf(x8[k] * it - m);
    }
    s = wave_sum(s);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) smf[threadIdx.x >> 6] = s;
    __syncthreads();
    float total = 0.f;
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) total += smf[w];
    *mx = m; *sum = total;
}

// One token per row drawn from softmax(logits / T) with the row's uniform number.  One workgroup per row.
template <int NT>
__device__ __forceinline__ int block_sample_softmax(const float* __restrict__ x, int V, float it, float u, float* smf, int* smi) {
    const float m = block_row_max<NT>(x, V, it, smf);
    return block_sample_inverse_cdf<NT>([&](int j) { return expf(x[j] * it - m); }, V, u, smf, smi);
}
constexpr int SAMPLE_NT = 512;
// (u_index, optional: row r draws with u[u_index[r] * u_stride] instead of u[r * u_stride]; the rows of a draft tree draw
//  with the uniform of their depth)
__global__ __launch_bounds__(SAMPLE_NT) void sample_rows_kernel(const float* __restrict__ logits, int V, float inv_temp,
                                                                const float* __restrict__ u, int u_stride,
                                                                int32_t* __restrict__ out, int out_stride,
                                                                const int32_t* __restrict__ u_index = nullptr) {
    __shared__ float smf[SAMPLE_NT / 64];
    __shared__ int smi[SAMPLE_NT / 64];
    const int row = blockIdx.x;
    const int ui = u_index ? u_index[row] : row;
    const int tok = block_sample_softmax<SAMPLE_NT>(logits + (size_t)row * V, V, inv_temp, u[(size_t)ui * u_stride], smf, smi);
    if (threadIdx.x == 0) out[(size_t)row * out_stride] = tok;
}

// Stochastic acceptance, one workgroup per sequence.  p_i = softmax(target logits of row i / T), q_i =
// softmax(drafter logits of step i / T).  Draft i is accepted while u_acc[i] * q_i(x_i) < p_i(x_i); at the first
// rejection the replacement is drawn (u_res) from the positive part of p_i - q_i (from p_i if that is empty); if all
// K are accepted the extra token is drawn from p_K.  Outputs as accept_kernel.
constexpr int ACCEPT_NT = 1024;
__global__ __launch_bounds__(ACCEPT_NT) void accept_sample_kernel(const int32_t* __restrict__ drafts, const float* __restrict__ vlogits,
                                                                  const float* __restrict__ dlogits, int B, int V, int kmax, int K,
                                                                  float inv_temp, const float* __restrict__ u_acc,
                                                                  const float* __restrict__ u_res, int32_t* __restrict__ text,
                                                                  int text_stride, const int* __restrict__ dlen, int* __restrict__ tlen,
                                                                  int32_t* __restrict__ nacc, int32_t* __restrict__ out_tokens,
                                                                  int32_t* __restrict__ next_tok) {
    __shared__ float smf[ACCEPT_NT / 64];
    __shared__ int smi[ACCEPT_NT / 64];
    const int b = blockIdx.x;
    int n = K, tok = 0;
    for (int i = 0; i < K; ++i) {
        const float* lp = vlogits + ((size_t)b * (K + 1) + i) * V;
        const float* lq = dlogits + ((size_t)i * B + b) * V;
        const int x = min(max(drafts[b * kmax + i], 0), V - 1);
        float mp, sp, mq, sq;
        block_softmax_stats<ACCEPT_NT>(lp, V, inv_temp, smf, &mp, &sp);
        block_softmax_stats<ACCEPT_NT>(lq, V, inv_temp, smf, &mq, &sq);
        const float px = expf(lp[x] * inv_temp - mp) / sp, qx = expf(lq[x] * inv_temp - mq) / sq;
        if (u_acc[b * K + i] * qx < px) continue;
        // rejected: does p - q have a positive part at all?
        const float isp = 1.0f / sp, isq = 1.0f / sq;
        auto resid = [&](int j) { return fmaxf(expf(lp[j] * inv_temp - mp) * isp - expf(lq[j] * inv_temp - mq) * isq, 0.f); };
        float any = 0.f;
        for (int j = threadIdx.x; j < V; j += ACCEPT_NT * 4) {
            float r4[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) r4[k] = resid(min(j + ACCEPT_NT * k, V - 1));
#pragma unroll
            for (int k = 0; k < 4; ++k) any = fmaxf(any, r4[k]);
        }
        any = block_reduce_max<ACCEPT_NT>(any, smf);
        if (any > 0.f) tok = block_sample_inverse_cdf<ACCEPT_NT>(resid, V, u_res[b], smf, smi);
        else tok = block_sample_inverse_cdf<ACCEPT_NT>([&](int j) { return expf(lp[j] * inv_temp - mp); }, V, u_res[b], smf, smi);
        n = i;
        break;
    }
    if (n == K) tok = block_sample_softmax<ACCEPT_NT>(vlogits + ((size_t)b * (K + 1) + K) * V, V, inv_temp, u_res[b], smf, smi);
    const int lane = threadIdx.x;
    if (lane <= kmax) {
        int t = -1;
        if (lane < n) t = drafts[b * kmax + lane];
        else if (lane == n) t = tok;
        out_tokens[b * (kmax + 1) + lane] = t;
        if (lane <= n) text[(size_t)b * text_stride + dlen[b] + 1 + lane] = t;
        if (lane <= K) {
            const int e = min(lane, n);
            next_tok[b * (kmax + 1) + lane] = (e < n) ? drafts[b * kmax + e] : tok;
        }
    }
    if (lane == 0) { nacc[b] = n; tlen[b] += n + 1; }
}

// After the re-feed: the drafter's pending hidden state is its output at row n_b; its cache keeps n_b+1 rows.
__global__ void select_row_kernel(const float* __restrict__ dout, int m, const int32_t* __restrict__ nacc,
                                  float* __restrict__ fnext, int ldf, int* __restrict__ dlen, int d) {
    const int b = blockIdx.x;
    const int n = nacc[b];
    for (int c = threadIdx.x; c < d; c += blockDim.x) fnext[(size_t)b * ldf + c] = dout[((size_t)b * m + n) * d + c];
    if (threadIdx.x == 0) dlen[b] += n + 1;
}

__global__ void set_ints_kernel(int* __restrict__ p, int n, int val) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = val;
}

__global__ void copy_rows_kernel(const float* __restrict__ src, int lds, float* __restrict__ dst, int ldd, int d) {
    const int row = blockIdx.x;
    for (int c = threadIdx.x; c < d; c += blockDim.x) dst[(size_t)row * ldd + c] = src[(size_t)row * lds + c];
}

}  // namespace hivis

// Persistent "pass" kernel: a whole verify pass (N layers + LM head + greedy tokens), a whole
// K-step draft round, or the roll-forward of the drafter runs as ONE cooperative launch of one
// 1024-thread workgroup per compute unit that interprets a list of phases, with a grid-wide
// barrier between phases.  The small row-wise operations are folded into the GEMM phases:
//   RMSNorm     -> prologue (gain applied while building the MFMA A fragments, 1/rms in the epilogue)
//   RoPE+append -> epilogue of the fused QKV GEMM (rotary pairs are adjacent columns of a tile)
//   SiLU*up     -> epilogue of the fused gate|up GEMM (gate and up columns share a tile)
//   residual    -> epilogue of the O and down GEMMs (each output element has exactly one writer)
//   argmax      -> epilogue of the LM-head GEMM (per-workgroup candidates) + a tiny reduction phase
// Used for passes of at most one MFMA tile of rows (8 rows for bf16 weights, 16 for fp32).
#pragma once
#include "hivis_kernels.h"

namespace hivis {

enum { PH_GEMM = 0, PH_ATTN = 1, PH_ATTN_MERGE = 2, PH_PREP = 3, PH_NORM_ROWS = 4, PH_ARGMAX = 5 };
enum { PRO_PLAIN = 0, PRO_RMS = 1 };
constexpr int FUSED_RMAX = 8;      // (head,row) pairs per attention work item in the persistent kernel
enum { FEPI_STORE = 0, FEPI_ADD_TO = 1, FEPI_ADDVEC = 2, FEPI_QKV = 3, FEPI_SILU = 4, FEPI_LOGITS = 5 };

struct Phase {
    int type, pro, epi;
    int K, N;
    const uint4* W;            // GEMM: packed weights
    const float* A; int lda;   // GEMM: activation rows; ATTN: q rows (fused qkv buffer)
    const void* gain;          // PRO_RMS: gain vector (weight dtype); GATHER: embedding table
    float* Y; int ldy;         // output rows (STORE / ADD_TO / ADDVEC / LOGITS / QKV q part / SILU act / ATTN_MERGE / PREP gather / NORM_ROWS)
    const float* R; int ldr;   // ADD_TO: Y = R + result (R == Y: accumulate into the residual stream)
    const void* vec; int vec_idx;          // ADDVEC: table [*][N] of the weight dtype and the row to add
    void* kc; void* vc; int maxL;          // QKV epilogue / ATTN: cache of this layer
    const int* base; int offset;           // row positions: base[seq] + offset + i
    const int32_t* ids; int id_sseq, id_srow;      // PREP: token of row (seq, i) = ids[seq*id_sseq + i*id_srow] (ids may be null: no gather)
    int32_t* tok_out; int o_sseq, o_srow;          // ARGMAX: destination of the greedy token of row (seq, i)
    AttnShape att; int att_items;                  // ATTN / ATTN_MERGE
};

struct PassParams {
    const Phase* phases; int nphases;
    int M, nseq, m;                 // rows of the pass = nseq * m
    int d, Hq, Hkv, hd, F, V;
    float eps, theta;
    float* rope_tab;                // [rows][hd/2][2] cos, sin
    float* attn_ws;
    float* pm; int* pi;             // greedy-token candidates [row][workgroup]
    unsigned* bar;                  // [0] arrival counter (zeroed before launch), [1] abort flag
    unsigned spin_limit;
};

// Grid-wide barrier.  Every thread releases its writes at agent scope, one thread arrives and
// spins (bounded: on timeout the abort flag is raised and every workgroup leaves), every
// thread acquires.  Returns false if the pass was aborted.
__device__ __forceinline__ bool grid_barrier(unsigned* bar, unsigned target, unsigned spin_limit) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    __syncthreads();
    if (threadIdx.x == 0) {
        __hip_atomic_fetch_add(&bar[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        unsigned spins = 0;
        while (__hip_atomic_load(&bar[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            __builtin_amdgcn_s_sleep(1);
            ++spins;
            if ((spins & 255u) == 0u && __hip_atomic_load(&bar[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) break;
            if (spins > spin_limit) { __hip_atomic_store(&bar[1], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); break; }
        }
    }
    __syncthreads();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    return __hip_atomic_load(&bar[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u;
}

// ---- A fragments with optional gain and sum of squares ------------------------------------------
template <typename WT>
__device__ __forceinline__ void fused_afrag(bf16x8_t& out, const float* __restrict__ A, int lda, int M, int kb, int lane,
                                            const WT* __restrict__ gain, float& ssq) {
    const int i = lane & 15, g = lane >> 4;
    const int row = 2 * (i >> 2) + (i & 1);
    const bool lo = (i & 2) != 0;
    uint32_t pk[4] = {0u, 0u, 0u, 0u};
    if (row < M) {
        const int k0 = kb * 32 + g * 8;
        const float4* p = reinterpret_cast<const float4*>(A + (size_t)row * lda + k0);
        float4 x0 = p[0], x1 = p[1];
        float x[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
        if (gain) {
            float s = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) { s += x[e] * x[e]; x[e] *= to_f32(gain[k0 + e]); }
            if (!lo) ssq += s;
        }
        bf16_t h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            bf16_t hi = f32_to_bf16(x[e]);
            h[e] = lo ? f32_to_bf16(x[e] - bf16_to_f32(hi)) : hi;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) pk[e] = (uint32_t)h[2 * e] | ((uint32_t)h[2 * e + 1] << 16);
    }
    out = __builtin_bit_cast(bf16x8_t, make_uint4(pk[0], pk[1], pk[2], pk[3]));
}
template <typename WT>
__device__ __forceinline__ void fused_afrag(float4& out, const float* __restrict__ A, int lda, int M, int kb, int lane,
                                            const WT* __restrict__ gain, float& ssq) {
    const int i = lane & 15, g = lane >> 4;
    out = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < M) {
        const int k0 = kb * 16 + g * 4;
        float4 x = *reinterpret_cast<const float4*>(A + (size_t)i * lda + k0);
        if (gain) {
            ssq += x.x * x.x + x.y * x.y + x.z * x.z + x.w * x.w;
            x.x *= to_f32(gain[k0]); x.y *= to_f32(gain[k0 + 1]); x.z *= to_f32(gain[k0 + 2]); x.w *= to_f32(gain[k0 + 3]);
        }
        out = x;
    }
}

// lane (i = lane & 15) -> activation row whose sum of squares this lane accumulated, or -1
template <typename WT> __device__ __forceinline__ int ssq_row_of_lane(int i);
template <> __device__ __forceinline__ int ssq_row_of_lane<bf16_t>(int i) { return (i & 2) ? -1 : 2 * (i >> 2) + (i & 1); }
template <> __device__ __forceinline__ int ssq_row_of_lane<float>(int i) { return i; }

template <typename WT> struct FusedCfg;
template <> struct FusedCfg<bf16_t> { static constexpr int KBW = 2, G = 4, NW = 16; };
template <> struct FusedCfg<float> { static constexpr int KBW = 2, G = 2, NW = 16; };

__host__ __device__ constexpr size_t fused_gemm_lds_floats(int NW, int G, int RPL, int ROWS) {
    return (size_t)NW * G * 64 * RPL + (size_t)G * 64 * RPL + (size_t)NW * 16 + 16 + 4 * 16;
}

template <typename WT>
__device__ void gemm_phase(const Phase& ph, const PassParams& pp, float* __restrict__ lds) {
    typedef WTraits<WT> TR;
    typedef typename AFrag<WT>::type afrag_t;
    typedef typename KVType<WT>::type KT;
    constexpr int RPL = TR::RPL, ROWS = TR::ROWS, KBW = FusedCfg<WT>::KBW, G = FusedCfg<WT>::G, NW = FusedCfg<WT>::NW;
    constexpr int TILE = G * 64 * RPL;
    float* red = lds;                       // [NW][G][64][RPL]
    float* tile = red + (size_t)NW * TILE;  // [G][64][RPL]
    float* ssq_w = tile + TILE;             // [NW][16]
    float* inv_rms = ssq_w + NW * 16;       // [16]
    float* cand_v = inv_rms + 16;           // [16] per-row best value (LOGITS)
    int* cand_i = (int*)(cand_v + 16);      // [16]

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int M = pp.M, K = ph.K, N = ph.N;
    const int kblks = K / TR::KB, ntiles = N / 16;
    const int t_begin = (int)(((long long)blockIdx.x * ntiles) / gridDim.x);
    const int t_end = (int)(((long long)(blockIdx.x + 1) * ntiles) / gridDim.x);
    const int npass = (kblks + NW * KBW - 1) / (NW * KBW);
    const WT* gain = (ph.pro == PRO_RMS) ? (const WT*)ph.gain : nullptr;
    const float* A = ph.A;
    const int lda = ph.lda;
    float ssq = 0.f;
    // greedy-token candidate of this thread's output slots (LOGITS): a thread always serves the same row
    float best_v = -INFINITY; int best_i = 0x7FFFFFFF;

    for (int tg = t_begin; tg < t_end; tg += G) {
        const int ng = min(G, t_end - tg);
        const bool first = (tg == t_begin);
        f32x4_t acc[G];
#pragma unroll
        for (int g = 0; g < G; ++g) acc[g] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        for (int pass = 0; pass < npass; ++pass) {
            const int kb0 = (pass * NW + wave) * KBW;
            const int nkb = max(0, min(KBW, kblks - kb0));
            if (nkb == 0) continue;
            afrag_t af[KBW];
            float ssq_dummy = 0.f;
#pragma unroll
            for (int j = 0; j < KBW; ++j) {
                if (j < nkb) fused_afrag<WT>(af[j], A, lda, M, kb0 + j, lane, gain, first ? ssq : ssq_dummy);
                else fused_afrag<WT>(af[j], A, lda, 0, 0, lane, (const WT*)nullptr, ssq_dummy);
            }
            uint4 wb[2][KBW];
            const uint4* wp = ph.W + ((size_t)tg * kblks + kb0) * 64 + lane;
#pragma unroll
            for (int j = 0; j < KBW; ++j)
                if (j < nkb) wb[0][j] = wp[(size_t)j * 64]; else wb[0][j] = make_uint4(0, 0, 0, 0);
#pragma unroll
            for (int g = 0; g < G; ++g) {
                if (g < ng) {
                    if (g + 1 < ng) {
                        const uint4* wn = wp + (size_t)(g + 1) * kblks * 64;
#pragma unroll
                        for (int j = 0; j < KBW; ++j)
                            if (j < nkb) wb[(g + 1) & 1][j] = wn[(size_t)j * 64]; else wb[(g + 1) & 1][j] = make_uint4(0, 0, 0, 0);
                    }
#pragma unroll
                    for (int j = 0; j < KBW; ++j) mfma_block(acc[g], af[j], wb[g & 1][j]);
                }
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
            float s = ssq;
            s += __shfl_xor(s, 16, 64);
            s += __shfl_xor(s, 32, 64);
            if (lane < 16) ssq_w[wave * 16 + lane] = s;
        }
        __syncthreads();
        for (int idx = threadIdx.x; idx < TILE; idx += NW * 64) {
            float s = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) s += red[(size_t)w * TILE + idx];
            tile[idx] = s;
        }
        if (first && gain && threadIdx.x < 16) {
            const int row = ssq_row_of_lane<WT>(threadIdx.x);
            if (row >= 0) {
                float s = 0.f;
#pragma unroll
                for (int w = 0; w < NW; ++w) s += ssq_w[w * 16 + threadIdx.x];
                inv_rms[row] = 1.0f / sqrtf(s / (float)K + pp.eps);
            }
        }
        __syncthreads();
        // ---- epilogue on the reduced tiles
        for (int idx = threadIdx.x; idx < TILE; idx += NW * 64) {
            const int r = idx % RPL;
            const int ln = (idx / RPL) & 63;
            const int g = idx / (RPL * 64);
            const int row = RPL * (ln >> 4) + r;
            const int cl = ln & 15;
            const int col = (tg + g) * 16 + cl;
            if (g >= ng || row >= M) continue;
            const float sc = gain ? inv_rms[row] : 1.0f;
            const float v = tile[idx] * sc;
            switch (ph.epi) {
            case FEPI_STORE: ph.Y[(size_t)row * ph.ldy + col] = v; break;
            case FEPI_ADD_TO: ph.Y[(size_t)row * ph.ldy + col] = ph.R[(size_t)row * ph.ldr + col] + v; break;
            case FEPI_ADDVEC: ph.Y[(size_t)row * ph.ldy + col] = v + to_f32(((const WT*)ph.vec)[(size_t)ph.vec_idx * N + col]); break;
            case FEPI_LOGITS:
                ph.Y[(size_t)row * ph.ldy + col] = v;
                if (v > best_v || (v == best_v && col < best_i)) { best_v = v; best_i = col; }
                break;
            case FEPI_SILU:
                if (cl < 8) {
                    const float up = tile[idx + 8 * RPL] * sc;
                    ph.Y[(size_t)row * ph.ldy + (tg + g) * 8 + cl] = v / (1.0f + expf(-v)) * up;
                }
                break;
            case FEPI_QKV: {
                const int qd = pp.Hq * pp.hd, kd = pp.Hkv * pp.hd, hd = pp.hd;
                const int seq = row / pp.m;
                const int pos = ph.base[seq] + ph.offset + row % pp.m;
                if (col < qd + kd) {
                    if ((cl & 1) == 0) {
                        const float x1 = v, x2 = tile[idx + RPL] * sc;
                        const int p = (col % hd) >> 1;
                        const float c = pp.rope_tab[((size_t)row * (hd / 2) + p) * 2], s = pp.rope_tab[((size_t)row * (hd / 2) + p) * 2 + 1];
                        const float y1 = x1 * c - x2 * s, y2 = x2 * c + x1 * s;
                        if (col < qd) {
                            ph.Y[(size_t)row * ph.ldy + col] = y1; ph.Y[(size_t)row * ph.ldy + col + 1] = y2;
                        } else {
                            const int c2 = col - qd;
                            KT* dst = (KT*)ph.kc + (((size_t)seq * pp.Hkv + c2 / hd) * ph.maxL + pos) * hd + c2 % hd;
                            from_f32(dst[0], y1); from_f32(dst[1], y2);
                        }
                    }
                } else {
                    const int c2 = col - qd - kd;
                    from_f32(((KT*)ph.vc)[(((size_t)seq * pp.Hkv + c2 / hd) * ph.maxL + pos) * hd + c2 % hd], v);
                }
            } break;
            }
        }
        __syncthreads();
    }
    if (ph.epi == FEPI_LOGITS) {
        // per-row candidate of this workgroup: threads of one row meet through LDS (tile buffer reused)
        float* cv = red; int* ci = (int*)(red + NW * 64);
        cv[threadIdx.x] = best_v; ci[threadIdx.x] = best_i;
        __syncthreads();
        if (threadIdx.x < ROWS) {
            const int row = threadIdx.x;
            float bv = -INFINITY; int bi = 0x7FFFFFFF;
            for (int t = 0; t < NW * 64; ++t) {
                if (t >= TILE) break;
                const int r = t % RPL, ln = (t / RPL) & 63;
                if (RPL * (ln >> 4) + r != row) continue;
                // thread t served slots t, t + NW*64, ... : all have the same row because NW*64 is a multiple of 64*RPL
                const float v = cv[t]; const int i = ci[t];
                if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
            }
            if (row < M) { pp.pm[(size_t)row * gridDim.x + blockIdx.x] = bv; pp.pi[(size_t)row * gridDim.x + blockIdx.x] = bi; }
        }
        __syncthreads();
    }
}

template <typename WT>
__global__ __launch_bounds__(1024) void fused_pass_kernel(PassParams pp) {
    typedef typename KVType<WT>::type KT;
    extern __shared__ __align__(16) float lds[];
    for (int p = 0; p < pp.nphases; ++p) {
        const Phase& ph = pp.phases[p];
        switch (ph.type) {
        case PH_GEMM: gemm_phase<WT>(ph, pp, lds); break;
        case PH_ATTN: {
            const int total = ph.att_items * ph.att.nsplit;
            for (int w = blockIdx.x; w < total; w += gridDim.x) {
                const int item = w / ph.att.nsplit, split = w % ph.att.nsplit;
                if (pp.hd == 128) attn_item_partial<KT, 128, FUSED_RMAX>(ph.A, (const KT*)ph.kc, (const KT*)ph.vc, ph.base, ph.att, item, split, lds, pp.attn_ws);
                else attn_item_partial<KT, 64, FUSED_RMAX>(ph.A, (const KT*)ph.kc, (const KT*)ph.vc, ph.base, ph.att, item, split, lds, pp.attn_ws);
                __syncthreads();
            }
        } break;
        case PH_ATTN_MERGE:
            for (int item = blockIdx.x; item < ph.att_items; item += gridDim.x) {
                if (pp.hd == 128) attn_item_merge<128, FUSED_RMAX>(pp.attn_ws, ph.base, ph.att, item, 1024, ph.Y, ph.ldy);
                else attn_item_merge<64, FUSED_RMAX>(pp.attn_ws, ph.base, ph.att, item, 1024, ph.Y, ph.ldy);
            }
            break;
        case PH_PREP: {
            // embedding gather of the rows' tokens (optional) and the rotary cos/sin table of the rows' positions
            if (ph.ids) {
                for (int row = blockIdx.x; row < pp.M; row += gridDim.x) {
                    const int32_t tok = ph.ids[(row / pp.m) * ph.id_sseq + (row % pp.m) * ph.id_srow];
                    const WT* src = (const WT*)ph.gain + (size_t)tok * pp.d;
                    for (int c = threadIdx.x; c < pp.d; c += 1024) ph.Y[(size_t)row * ph.ldy + c] = to_f32(src[c]);
                }
            }
            const int half = pp.hd / 2;
            for (int idx = blockIdx.x * 1024 + threadIdx.x; idx < pp.M * half; idx += gridDim.x * 1024) {
                const int row = idx / half, i = idx % half;
                const int pos = ph.base[row / pp.m] + ph.offset + row % pp.m;
                const double inv_freq = exp2(-2.0 * (double)i / (double)pp.hd * log2((double)pp.theta));
                double s, c;
                sincos((double)pos * inv_freq, &s, &c);
                pp.rope_tab[(size_t)idx * 2] = (float)c; pp.rope_tab[(size_t)idx * 2 + 1] = (float)s;
            }
        } break;
        case PH_NORM_ROWS:
            // Y[row] = A[row] * gain / sqrt(mean(A[row]^2) + eps): one workgroup per row
            for (int row = blockIdx.x; row < pp.M; row += gridDim.x) {
                const float* x = ph.A + (size_t)row * ph.lda;
                float ss = 0.f;
                for (int c = threadIdx.x; c < pp.d; c += 1024) ss += x[c] * x[c];
                ss = wave_sum(ss);
                __syncthreads();
                if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = ss;
                __syncthreads();
                float tot = 0.f;
#pragma unroll
                for (int w = 0; w < 16; ++w) tot += lds[w];
                const float inv = 1.0f / sqrtf(tot / (float)pp.d + pp.eps);
                for (int c = threadIdx.x; c < pp.d; c += 1024)
                    ph.Y[(size_t)row * ph.ldy + c] = x[c] * to_f32(((const WT*)ph.gain)[c]) * inv;
            }
            break;
        case PH_ARGMAX:
            // one wavefront per row reduces the per-workgroup candidates (lowest index wins ties)
            for (int row = blockIdx.x * 16 + (threadIdx.x >> 6); row < pp.M; row += gridDim.x * 16) {
                float bv = -INFINITY; int bi = 0x7FFFFFFF;
                for (int w = threadIdx.x & 63; w < (int)gridDim.x; w += 64) {
                    const float v = pp.pm[(size_t)row * gridDim.x + w]; const int i = pp.pi[(size_t)row * gridDim.x + w];
                    if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
                }
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) {
                    const float ov = __shfl_xor(bv, o, 64); const int oi = __shfl_xor(bi, o, 64);
                    if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
                }
                if ((threadIdx.x & 63) == 0) ph.tok_out[(row / pp.m) * ph.o_sseq + (row % pp.m) * ph.o_srow] = bi;
            }
            break;
        }
        if (!grid_barrier(pp.bar, (unsigned)(p + 1) * gridDim.x, pp.spin_limit)) return;
    }
}

}  // namespace hivis

// Gate: fp64-accumulated logits, wavefront top-k, softmax over the chosen k
// (paper section 2.1 step 1), plus the per-block / per-destination histograms
// that feed the dispatch plan.
#pragma once
#include "common.hpp"

namespace moe {

typedef __attribute__((ext_vector_type(4))) double f64x4_t;
typedef __attribute__((ext_vector_type(4))) u32 u32x4_t;  // 16 bytes in registers

// How a gate task lays out its work.  The gate weights and the task's 16 rows
// of x pass through LDS in chunks of KC reduction indices (weights: row stride
// RS bytes, x: row stride XRS bytes), two buffers, the next chunk in flight
// while this one multiplies.  A chunk is made as large as LDS allows (72 KB in
// all, so that two workgroups still share a CU): its multiplications then
// outlast the trip to memory of the next one.  The E/16 expert blocks are dealt
// to `groups` groups of wavefronts, and the `parts` wavefronts of a group take
// alternate 16-index pieces of every chunk.
constexpr int kRouteLds = 72 * 1024;
constexpr int kRouteMaxKC = 512;
struct RouteShape {
    int RS, XRS, KC, nb, groups, parts, nbw;
};
__host__ __device__ inline RouteShape route_shape(int E, int elem_size) {
    RouteShape r;
    r.RS = (E * elem_size + 15) / 16 * 16;
    const int budget = (kRouteLds - kRouteTokens * E * 8) / 2;  // bytes per buffer
    r.KC = budget / (r.RS + kRouteTokens * elem_size) / 16 * 16;
    if (r.KC > kRouteMaxKC) r.KC = kRouteMaxKC;
    if (r.KC < 16) r.KC = 16;
    r.XRS = r.KC * elem_size;
    r.nb = (E + 15) / 16;
    r.groups = r.nb >= 4 ? 4 : r.nb >= 2 ? 2 : 1;
    r.parts = 4 / r.groups;
    r.nbw = (r.nb + r.groups - 1) / r.groups;
    return r;
}
__host__ __device__ inline size_t route_stage_bytes(const RouteShape &r) {
    return (size_t)r.KC * r.RS + (size_t)kRouteTokens * r.XRS;
}
__host__ __device__ inline size_t route_smem_bytes(int E, int elem_size) {
    const RouteShape r = route_shape(E, elem_size);
    return (size_t)kRouteTokens * E * 8 + 2 * route_stage_bytes(r);  // logits [16][E] f64 + two chunks
}

// (value, index) argmax step: larger value wins, equal values -> lower index
__device__ __forceinline__ void argmax_merge(double &v, int &i, double ov, int oi) {
    if (ov > v || (ov == v && oi < i)) {
        v = ov;
        i = oi;
    }
}

template <typename ET>
struct RouteLoad;
template <>
struct RouteLoad<bf16_t> {
    typedef uint2 x4_t;  // four consecutive bf16
    static __device__ __forceinline__ double get(const x4_t &v, int s) {
        const u32 w = (s < 2) ? v.x : v.y;
        return (double)__uint_as_float((s & 1) ? (w & 0xffff0000u) : (w << 16));
    }
    // value of the raw element, or 0.0 when keep == 0 (keep is 0 or ~0: no branch around the load)
    static __device__ __forceinline__ double to_double(bf16_t r, u32 keep) {
        return (double)__uint_as_float(((u32)r << 16) & keep);
    }
};
template <>
struct RouteLoad<float> {
    typedef float4 x4_t;
    static __device__ __forceinline__ double get(const x4_t &v, int s) {
        return (double)(s == 0 ? v.x : s == 1 ? v.y : s == 2 ? v.z : v.w);
    }
    static __device__ __forceinline__ double to_double(float r, u32 keep) {
        return (double)__uint_as_float(__float_as_uint(r) & keep);
    }
};

// Logits of tokens [t0, t0+16) into lg[16][E] (LDS, fp64) with the fp64 matrix
// cores: D[token][expert] += x[token][k] * Wg[k][expert], 16 x 16 x 4 per
// instruction.  bf16/fp32 inputs convert exactly and their products are exact
// in fp64, so the only rounding is the fp64 accumulation.  Lane l feeds token
// (or expert) l % 16 and reduction index 4*(l / 16) + s within a piece of 16.
// Both operands come through LDS: wide coalesced loads one chunk ahead, double
// buffered, one barrier per chunk.  Wavefronts of different groups own
// different experts; the PARTS wavefronts of a group add their partial sums
// into LDS one after the other (fixed order: deterministic).
template <typename ET, int NBW, int PARTS>
__device__ __forceinline__ void route_logits(const KArgs &a, int t0, char *smem) {
    typedef RouteLoad<ET> L;
    typedef typename L::x4_t x4_t;
    constexpr int ES = (int)sizeof(ET);
    constexpr int GROUPS = 4 / PARTS;
    constexpr int MAXPW = 7, MAXPX = 8;  // 16-byte pieces of a chunk per thread (the most route_shape() can ask for)
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int E = a.E, d = a.d;
    const RouteShape rs = route_shape(E, ES);
    const int li = lane & 15, kq = lane >> 4;
    const int g = wave % GROUPS, part = wave / GROUPS;
    double *lg = (double *)smem;  // [16][E]
    char *stage = smem + (size_t)kRouteTokens * E * 8;
    const int stage_bytes = (int)route_stage_bytes(rs);
    const int x_off = rs.KC * rs.RS;  // x rows follow the weight rows of a buffer
    const char *x = (const char *)a.x;
    const char *Wg = (const char *)a.Wg;
    const int row_bytes = E * ES;
    const bool wide = (row_bytes % 16) == 0;
    const int ppr = row_bytes / 16;
    const int nchunk = (d + rs.KC - 1) / rs.KC;

    // this wavefront's expert columns; lanes past E read a valid column and are masked
    u32 keep[NBW];
    int col_off[NBW];
#pragma unroll
    for (int b = 0; b < NBW; ++b) {
        const int e = (g + b * GROUPS) * 16 + li;
        keep[b] = e < E ? ~0u : 0u;
        col_off[b] = (e < E ? e : 0) * ES;
    }
    f64x4_t acc[NBW];
#pragma unroll
    for (int b = 0; b < NBW; ++b) acc[b] = f64x4_t{0.0, 0.0, 0.0, 0.0};

    u32x4_t prew[MAXPW], prex[MAXPX];
    auto fetch = [&](int c) __attribute__((always_inline)) {  // chunk c -> registers
        const int k0 = c * rs.KC, rows = min(rs.KC, d - k0);
        if (wide) {
#pragma unroll
            for (int i = 0; i < MAXPW; ++i) {
                const int q = tid + i * kThreads;
                if (q < rows * ppr) prew[i] = *(const u32x4_t *)(Wg + (size_t)(k0 + q / ppr) * row_bytes + (q % ppr) * 16);
            }
        }
        const int ppx = rows * ES / 16;
#pragma unroll
        for (int i = 0; i < MAXPX; ++i) {
            const int q = tid + i * kThreads;
            if (q < kRouteTokens * ppx) {
                const int tok = min(t0 + q / ppx, a.T - 1);
                prex[i] = *(const u32x4_t *)(x + ((size_t)tok * d + k0) * ES + (q % ppx) * 16);
            }
        }
    };
    auto store = [&](int c, int buf) __attribute__((always_inline)) {  // registers -> LDS buffer
        const int k0 = c * rs.KC, rows = min(rs.KC, d - k0);
        char *dst = stage + buf * stage_bytes;
        if (wide) {
#pragma unroll
            for (int i = 0; i < MAXPW; ++i) {
                const int q = tid + i * kThreads;
                if (q < rows * ppr) *(u32x4_t *)(dst + (q / ppr) * rs.RS + (q % ppr) * 16) = prew[i];
            }
        } else {  // odd row sizes (tiny expert counts): element by element, straight from global memory
            for (int q = tid; q < rows * E; q += kThreads)
                *(ET *)(dst + (q / E) * rs.RS + (q % E) * ES) = *(const ET *)(Wg + ((size_t)(k0 + q / E) * E + q % E) * ES);
        }
        const int ppx = rows * ES / 16;
#pragma unroll
        for (int i = 0; i < MAXPX; ++i) {
            const int q = tid + i * kThreads;
            if (q < kRouteTokens * ppx) *(u32x4_t *)(dst + x_off + (q / ppx) * rs.XRS + (q % ppx) * 16) = prex[i];
        }
    };
    auto mul = [&](int c, int buf) __attribute__((always_inline)) {
        const int pieces = min(rs.KC, d - c * rs.KC) / 16;
        const char *src = stage + buf * stage_bytes;
        const char *xs = src + x_off + li * rs.XRS + 4 * kq * ES;
        for (int u = part; u < pieces; u += PARTS) {
            const x4_t xv = *(const x4_t *)(xs + 16 * u * ES);
#pragma unroll
            for (int s2 = 0; s2 < 4; ++s2) {
                const double av = L::get(xv, s2);
                const char *wrow = src + (16 * u + 4 * kq + s2) * rs.RS;
#pragma unroll
                for (int b = 0; b < NBW; ++b) {
                    const double bv = L::to_double(*(const ET *)(wrow + col_off[b]), keep[b]);
                    acc[b] = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc[b], 0, 0, 0);
                }
            }
        }
    };

    fetch(0);
    store(0, 0);
    __syncthreads();
    for (int c = 0; c < nchunk; ++c) {
        const int buf = c & 1;
        if (c + 1 < nchunk) fetch(c + 1);
        mul(c, buf);
        if (c + 1 < nchunk) store(c + 1, buf ^ 1);
        __syncthreads();
    }
    // D layout: lane l, register v -> token 4*v + l/16, expert (block) l % 16
    for (int p2 = 0; p2 < PARTS; ++p2) {
        if (part == p2) {
#pragma unroll
            for (int b = 0; b < NBW; ++b) {
                const int e = (g + b * GROUPS) * 16 + li;
                if (e < E) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int t = 4 * v + kq;
                        const double prev = (p2 == 0) ? (a.bias ? (double)a.bias[e] : 0.0) : lg[t * E + e];
                        lg[t * E + e] = prev + acc[b][v];
                    }
                }
            }
        }
        __syncthreads();
    }
}

template <typename ET>
__device__ __forceinline__ void route_logits_dispatch(const KArgs &a, int t0, char *smem) {
    const RouteShape rs = route_shape(a.E, (int)sizeof(ET));
    if (rs.parts == 4)
        route_logits<ET, 1, 4>(a, t0, smem);
    else if (rs.parts == 2) {
        if (rs.nbw == 1)
            route_logits<ET, 1, 2>(a, t0, smem);
        else
            route_logits<ET, 2, 2>(a, t0, smem);
    } else if (rs.nbw == 1)
        route_logits<ET, 1, 1>(a, t0, smem);
    else if (rs.nbw == 2)
        route_logits<ET, 2, 1>(a, t0, smem);
    else if (rs.nbw == 3)
        route_logits<ET, 3, 1>(a, t0, smem);
    else
        route_logits<ET, 4, 1>(a, t0, smem);
}

// One gate task: tokens [task*16, task*16+16).  With a.Wg == NULL the routing
// is an input and only the histograms are produced.
template <typename ET>
__device__ __forceinline__ void route_task(const KArgs &a, int task, char *smem, bool do_hist) {
    const int t0 = task * kRouteTokens;
    const int E = a.E, k = a.k;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool compute = (a.Wg != nullptr);
    MOE_TT_BEGIN();
    if (compute) route_logits_dispatch<ET>(a, t0, smem);
    MOE_TT(a.ctrl, 32);
    const double *lg = (const double *)smem;
    const double NEG = -__builtin_huge_val();

    // Each wavefront selects for its four tokens (wave, wave + 4, ...) at once: the four
    // shuffle chains are independent, so their latencies overlap.
    constexpr int TPW = kRouteTokens / 4;
    int my_e[TPW];
#pragma unroll
    for (int i = 0; i < TPW; ++i) my_e[i] = -1;
    if (compute) {
        double v[TPW][4], my_v[TPW];
#pragma unroll
        for (int i = 0; i < TPW; ++i) {
            const int tl = wave + 4 * i;
            my_v[i] = 0.0;
#pragma unroll
            for (int q = 0; q < 4; ++q) v[i][q] = (lane + 64 * q < E) ? lg[tl * E + lane + 64 * q] : NEG;
        }
        for (int j = 0; j < k; ++j) {
            double bv[TPW];
            int bi[TPW];
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                bv[i] = v[i][0];
                bi[i] = lane;
#pragma unroll
                for (int q = 1; q < 4; ++q) argmax_merge(bv[i], bi[i], v[i][q], lane + 64 * q);
            }
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
#pragma unroll
                for (int i = 0; i < TPW; ++i) {
                    const double ov = __shfl_xor(bv[i], off, 64);
                    const int oi = __shfl_xor(bi[i], off, 64);
                    argmax_merge(bv[i], bi[i], ov, oi);
                }
            }
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (bi[i] == lane + 64 * q) v[i][q] = NEG;
                if (lane == j) {
                    my_v[i] = bv[i];
                    my_e[i] = bi[i];
                }
            }
        }
        // softmax over the k chosen logits
        double ex[TPW], sum[TPW];
#pragma unroll
        for (int i = 0; i < TPW; ++i) {
            const double m = __shfl(my_v[i], 0, 64);
            ex[i] = (lane < k) ? exp(my_v[i] - m) : 0.0;
            sum[i] = ex[i];
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1)
#pragma unroll
            for (int i = 0; i < TPW; ++i) sum[i] += __shfl_xor(sum[i], off, 64);
#pragma unroll
        for (int i = 0; i < TPW; ++i) {
            const int t = t0 + wave + 4 * i;
            if (t < a.T && lane < k) {
                a.idx[(size_t)t * k + lane] = my_e[i];
                a.w[(size_t)t * k + lane] = (float)(ex[i] / sum[i]);
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < TPW; ++i) {
            const int t = t0 + wave + 4 * i;
            if (t < a.T && lane < k) my_e[i] = a.idx[(size_t)t * k + lane];
        }
    }
    if (do_hist) {
        // The task's 16 tokens lie in one permutation block: count them per expert in LDS
        // (behind the logits; the staging buffers are free by now), then add the non-zero
        // counts to the block's histogram: few, uncontended global atomics.  The
        // per-destination counts come from the block histograms in the plan whenever
        // destinations are whole blocks; else they are counted here, slot by slot.
        int *cnt = (int *)(smem + (compute ? (size_t)kRouteTokens * E * 8 : 0));  // (no logits in LDS: E ints suffice)
        for (int e = threadIdx.x; e < E; e += kThreads) cnt[e] = 0;
        __syncthreads();
        if (lane < k) {
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                const int t = t0 + wave + 4 * i;
                if (t >= a.T) continue;
                if (my_e[i] < 0 || my_e[i] >= E) {
                    set_error(a.ctrl, MOE_ERR_BAD_ROUTING);
                } else {
                    atomicAdd(&cnt[my_e[i]], 1);
                    if (!a.seg_from_blocks) atomicAdd(&a.seg_cnt[(size_t)my_e[i] * a.R + t / a.per_dest], 1);
                }
            }
        }
        __syncthreads();
        int32_t *bh = a.blk_hist + (size_t)(t0 / kPermBlock) * E;
        for (int e = threadIdx.x; e < E; e += kThreads)
            if (cnt[e] != 0) atomicAdd(&bh[e], cnt[e]);
    }
    MOE_TT(a.ctrl, 33);
}

}  // namespace moe

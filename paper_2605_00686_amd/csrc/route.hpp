// Gate: fp64-accumulated logits, wavefront top-k, softmax over the chosen k
// (paper section 2.1 step 1), plus the per-block / per-destination histograms
// that feed the dispatch plan.
#pragma once
#include "common.hpp"

namespace moe {

typedef __attribute__((ext_vector_type(4))) double f64x4_t;

__host__ __device__ inline size_t route_smem_bytes(int E) {
    return (size_t)kRouteTokens * E * 8;  // logits [16][E] f64
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
    typedef u32 raw_t;   // one bf16 in the low half
    static __device__ __forceinline__ double get(const x4_t &v, int s) {
        const u32 w = (s < 2) ? v.x : v.y;
        return (double)__uint_as_float((s & 1) ? (w & 0xffff0000u) : (w << 16));
    }
    static __device__ __forceinline__ raw_t load_raw(const bf16_t *p) { return (u32)*p; }
    static __device__ __forceinline__ double to_double(raw_t r) { return (double)__uint_as_float(r << 16); }
};
template <>
struct RouteLoad<float> {
    typedef float4 x4_t;
    typedef float raw_t;
    static __device__ __forceinline__ double get(const x4_t &v, int s) {
        return (double)(s == 0 ? v.x : s == 1 ? v.y : s == 2 ? v.z : v.w);
    }
    static __device__ __forceinline__ raw_t load_raw(const float *p) { return *p; }
    static __device__ __forceinline__ double to_double(raw_t r) { return (double)r; }
};

// Logits of tokens [t0, t0+16) into lg[16][E] (LDS, fp64) with the fp64 matrix
// cores: D[token][expert] += x[token][k] * Wg[k][expert], 16 x 16 x 4 per
// instruction.  bf16/fp32 inputs convert exactly and their products are exact
// in fp64, so the only rounding is the fp64 accumulation.  Lane l feeds token
// (or expert) l % 16 and reduction index 4*(l / 16) + s within a chunk of 16;
// the four wavefronts take contiguous quarters of the reduction and add their
// partial sums into LDS one after the other (fixed order: deterministic).
// NB expert blocks of 16 starting at block eb0; U chunks of 16 per iteration,
// the operands of the next iteration are in flight while this one multiplies
// (U * NB is kept near 8 so that an iteration hides a trip to L2).
template <typename ET, int NB, int U>
__device__ void route_logits(const KArgs &a, int t0, int eb0, char *smem) {
    typedef RouteLoad<ET> L;
    typedef typename L::x4_t x4_t;
    typedef typename L::raw_t raw_t;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int E = a.E, d = a.d;
    const int li = lane & 15, kq = lane >> 4;
    double *lg = (double *)smem;  // [16][E]
    const ET *x = (const ET *)a.x;
    const ET *Wg = (const ET *)a.Wg;
    const int nchunk = d / 16;
    const int c_begin = (nchunk * wave) / 4, c_end = (nchunk * (wave + 1)) / 4;
    const int tok = min(t0 + li, a.T - 1);
    const ET *xrow = x + (size_t)tok * d + 4 * kq;
    // expert column of this lane in block eb0 + eb; lanes past E re-read a valid column and are masked
    bool live[NB];
    const ET *wcol[NB];
#pragma unroll
    for (int eb = 0; eb < NB; ++eb) {
        const int e = (eb0 + eb) * 16 + li;
        live[eb] = e < E;
        wcol[eb] = Wg + (size_t)(4 * kq) * E + (live[eb] ? e : 0);
    }

    f64x4_t acc[NB];
#pragma unroll
    for (int eb = 0; eb < NB; ++eb) acc[eb] = f64x4_t{0.0, 0.0, 0.0, 0.0};

    struct Raw {
        x4_t xv[U];
        raw_t w[U][4][NB];
    };
    auto load = [&](int c0, Raw &r) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = min(c0 + u, c_end - 1);  // past the end: re-read the last chunk, masked in mul()
            r.xv[u] = *(const x4_t *)(xrow + c * 16);
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int eb = 0; eb < NB; ++eb) r.w[u][s][eb] = L::load_raw(wcol[eb] + (size_t)(c * 16 + s) * E);
        }
    };
    auto mul = [&](int c0, const Raw &r) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool in = c0 + u < c_end;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const double av = in ? L::get(r.xv[u], s) : 0.0;
#pragma unroll
                for (int eb = 0; eb < NB; ++eb) {
                    const double bv = live[eb] ? L::to_double(r.w[u][s][eb]) : 0.0;
                    acc[eb] = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc[eb], 0, 0, 0);
                }
            }
        }
    };
    Raw r0, r1;
    if (c_begin < c_end) {
        load(c_begin, r0);
        for (int c = c_begin; c < c_end; c += 2 * U) {
            load(c + U, r1);
            mul(c, r0);
            load(c + 2 * U, r0);
            mul(c + U, r1);
        }
    }
    // D layout: lane l, register v -> token 4*v + l/16, expert (block) l % 16
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int eb = 0; eb < NB; ++eb) {
                const int e = (eb0 + eb) * 16 + li;
                if (e < E) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int t = 4 * v + kq;
                        const double prev = (w == 0) ? (a.bias ? (double)a.bias[e] : 0.0) : lg[t * E + e];
                        lg[t * E + e] = prev + acc[eb][v];
                    }
                }
            }
        }
        __syncthreads();
    }
}

template <typename ET>
__device__ void route_logits_dispatch(const KArgs &a, int t0, char *smem) {
    const int nb = (a.E + 15) / 16;
    if (nb <= 1)
        route_logits<ET, 1, 8>(a, t0, 0, smem);
    else if (nb <= 2)
        route_logits<ET, 2, 4>(a, t0, 0, smem);
    else if (nb <= 4)
        route_logits<ET, 4, 2>(a, t0, 0, smem);
    else
        for (int eb0 = 0; eb0 < nb; eb0 += 8) route_logits<ET, 8, 1>(a, t0, eb0, smem);  // 128 experts per pass
}

// One gate task: tokens [task*16, task*16+16).  With a.Wg == NULL the routing
// is an input and only the histograms are produced.
template <typename ET>
__device__ void route_task(const KArgs &a, int task, char *smem, bool do_hist) {
    const int t0 = task * kRouteTokens;
    const int E = a.E, k = a.k;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool compute = (a.Wg != nullptr);
    if (compute) route_logits_dispatch<ET>(a, t0, smem);
    const double *lg = (const double *)smem;
    const double NEG = -__builtin_huge_val();

    for (int tl = wave; tl < kRouteTokens; tl += 4) {
        const int t = t0 + tl;
        if (t >= a.T) break;
        int my_e = -1;
        if (compute) {
            double v0 = (lane < E) ? lg[tl * E + lane] : NEG;
            double v1 = (lane + 64 < E) ? lg[tl * E + lane + 64] : NEG;
            double v2 = (lane + 128 < E) ? lg[tl * E + lane + 128] : NEG;
            double v3 = (lane + 192 < E) ? lg[tl * E + lane + 192] : NEG;
            double my_v = 0.0;
            for (int j = 0; j < k; ++j) {
                double bv = v0;
                int bi = lane;
                argmax_merge(bv, bi, v1, lane + 64);
                argmax_merge(bv, bi, v2, lane + 128);
                argmax_merge(bv, bi, v3, lane + 192);
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1) {
                    double ov = __shfl_xor(bv, off, 64);
                    int oi = __shfl_xor(bi, off, 64);
                    argmax_merge(bv, bi, ov, oi);
                }
                if (bi == lane) v0 = NEG;
                if (bi == lane + 64) v1 = NEG;
                if (bi == lane + 128) v2 = NEG;
                if (bi == lane + 192) v3 = NEG;
                if (lane == j) {
                    my_v = bv;
                    my_e = bi;
                }
            }
            // softmax over the k chosen logits
            const double m = __shfl(my_v, 0, 64);
            double ex = (lane < k) ? exp(my_v - m) : 0.0;
            double s = ex;
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
            if (lane < k) {
                a.idx[(size_t)t * k + lane] = my_e;
                a.w[(size_t)t * k + lane] = (float)(ex / s);
            }
        } else if (lane < k) {
            my_e = a.idx[(size_t)t * k + lane];
        }
        if (do_hist && lane < k) {
            if (my_e < 0 || my_e >= E) {
                set_error(a.ctrl, MOE_ERR_BAD_ROUTING);
            } else {
                atomicAdd(&a.blk_hist[(size_t)(t / kPermBlock) * E + my_e], 1);
                atomicAdd(&a.seg_cnt[(size_t)my_e * a.R + t / a.per_dest], 1);
            }
        }
    }
}

}  // namespace moe

// Gate: fp64-accumulated logits, wavefront top-k, softmax over the chosen k
// (paper section 2.1 step 1), plus the per-block / per-destination histograms
// that feed the dispatch plan.
#pragma once
#include "common.hpp"

namespace moe {

constexpr int kRouteKC = 64;  // reduction chunk staged in LDS

__host__ __device__ inline int route_lanes_e(int E) {
    int l = 1;
    while (l < E && l < 32) l <<= 1;
    return l;
}
__host__ __device__ inline size_t route_smem_bytes(int E) {
    // x chunk [16][KC+4] f32, Wg chunk transposed [E][KC+4] f32, logits [16][E] f64
    size_t a = (size_t)kRouteTokens * (kRouteKC + 4) * 4 + (size_t)E * (kRouteKC + 4) * 4;
    size_t b = (size_t)kRouteTokens * E * 8;
    return a + b;
}

// (value, index) argmax step: larger value wins, equal values -> lower index
__device__ __forceinline__ void argmax_merge(double &v, int &i, double ov, int oi) {
    if (ov > v || (ov == v && oi < i)) {
        v = ov;
        i = oi;
    }
}

// Logits of tokens [t0, t0+16) into lg[16][E] (LDS, fp64).  Thread (e_lane,
// t_lane) owns experts e_lane + lanes_e*j (j < NE) and tokens t_lane + t_lanes*n
// (n < NT); bf16/fp32 products are exact in fp64, so the only rounding is the
// fp64 accumulation itself.
template <typename ET, int NE, int NT>
__device__ void route_logits(const KArgs &a, int t0, char *smem) {
    const int tid = threadIdx.x;
    const int E = a.E, d = a.d;
    const int lanes_e = route_lanes_e(E);
    const int t_lanes = kThreads / lanes_e;
    const int e_lane = tid % lanes_e, t_lane = tid / lanes_e;
    constexpr int LD = kRouteKC + 4;
    float *xs = (float *)smem;             // [16][LD]
    float *ws = xs + kRouteTokens * LD;    // [E][LD]
    double *lg = (double *)(ws + E * LD);  // [16][E]
    const ET *x = (const ET *)a.x;
    const ET *Wg = (const ET *)a.Wg;

    double acc[NE][NT];
#pragma unroll
    for (int j = 0; j < NE; ++j)
#pragma unroll
        for (int n = 0; n < NT; ++n) acc[j][n] = 0.0;

    for (int i0 = 0; i0 < d; i0 += kRouteKC) {
        const int kc = min(kRouteKC, d - i0);
        for (int q = tid; q < kRouteTokens * kRouteKC; q += kThreads) {
            int t = q / kRouteKC, i = q % kRouteKC;
            float v = 0.f;
            if (t0 + t < a.T && i < kc) v = Elem<ET>::load(x, (size_t)(t0 + t) * d + i0 + i);
            xs[t * LD + i] = v;
        }
        for (int q = tid; q < kRouteKC * E; q += kThreads) {
            int i = q / E, e = q % E;  // consecutive threads -> consecutive e: coalesced
            float v = 0.f;
            if (i < kc) v = Elem<ET>::load(Wg, (size_t)(i0 + i) * E + e);
            ws[e * LD + i] = v;
        }
        __syncthreads();
#pragma unroll 2
        for (int i = 0; i < kRouteKC; i += 4) {
            float4 xv[NT], wv[NE];
#pragma unroll
            for (int n = 0; n < NT; ++n) {
                int t = t_lane + t_lanes * n;
                xv[n] = (t < kRouteTokens) ? *(const float4 *)&xs[t * LD + i] : make_float4(0, 0, 0, 0);
            }
#pragma unroll
            for (int j = 0; j < NE; ++j) {
                int e = e_lane + lanes_e * j;
                wv[j] = (e < E) ? *(const float4 *)&ws[e * LD + i] : make_float4(0, 0, 0, 0);
            }
#pragma unroll
            for (int j = 0; j < NE; ++j)
#pragma unroll
                for (int n = 0; n < NT; ++n) {
                    acc[j][n] = fma((double)xv[n].x, (double)wv[j].x, acc[j][n]);
                    acc[j][n] = fma((double)xv[n].y, (double)wv[j].y, acc[j][n]);
                    acc[j][n] = fma((double)xv[n].z, (double)wv[j].z, acc[j][n]);
                    acc[j][n] = fma((double)xv[n].w, (double)wv[j].w, acc[j][n]);
                }
        }
        __syncthreads();
    }
#pragma unroll
    for (int j = 0; j < NE; ++j)
#pragma unroll
        for (int n = 0; n < NT; ++n) {
            int e = e_lane + lanes_e * j, t = t_lane + t_lanes * n;
            if (e < E && t < kRouteTokens) lg[t * E + e] = acc[j][n] + (a.bias ? (double)a.bias[e] : 0.0);
        }
    __syncthreads();
}

template <typename ET>
__device__ void route_logits_dispatch(const KArgs &a, int t0, char *smem) {
    const int lanes_e = route_lanes_e(a.E);
    const int ne = (a.E + lanes_e - 1) / lanes_e;
    if (lanes_e < 32)
        route_logits<ET, 1, 1>(a, t0, smem);
    else if (ne <= 1)
        route_logits<ET, 1, 2>(a, t0, smem);
    else if (ne <= 2)
        route_logits<ET, 2, 2>(a, t0, smem);
    else if (ne <= 4)
        route_logits<ET, 4, 2>(a, t0, smem);
    else
        route_logits<ET, 8, 2>(a, t0, smem);
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
    const double *lg = (const double *)((float *)smem + (kRouteTokens + E) * (kRouteKC + 4));
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

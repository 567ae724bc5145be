// Gate: fp64-accumulated logits, wavefront top-k, softmax over the chosen k
// (paper section 2.1 step 1), plus the per-block / per-destination histograms
// that feed the dispatch plan.
#pragma once
#include "common.hpp"

namespace moe {

typedef __attribute__((ext_vector_type(4))) double f64x4_t;

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
// Only the reduction indices [k_begin, k_end) are summed (both multiples of 16), in chunks of up to
// RouteShape::KC; the bias is added if add_bias.
template <typename ET, int NBW, int PARTS>
__device__ __forceinline__ void route_logits(const KArgs &a, int t0, char *smem, int k_begin, int k_end, bool add_bias) {
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
        const int k0 = k_begin + c * rs.KC, rows = min(rs.KC, k_end - k0);
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
        const int k0 = k_begin + c * rs.KC, rows = min(rs.KC, k_end - k0);
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
        const int pieces = min(rs.KC, k_end - k_begin - c * rs.KC) / 16;
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

    const int c_end = (k_end - k_begin + rs.KC - 1) / rs.KC;
    fetch(0);
    store(0, 0);
    __syncthreads();
    for (int c = 0; c < c_end; ++c) {
        const int buf = c & 1;
        if (c + 1 < c_end) fetch(c + 1);
        mul(c, buf);
        if (c + 1 < c_end) store(c + 1, buf ^ 1);
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
                        const double prev = (p2 == 0) ? (add_bias && a.bias ? (double)a.bias[e] : 0.0) : lg[t * E + e];
                        lg[t * E + e] = prev + acc[b][v];
                    }
                }
            }
        }
        __syncthreads();
    }
}

// A gate split over its reduction gives every task a slice of whole 16-index pieces, at least
// kRouteMinSlice indices long: the most slices a reduction of length d can have.
constexpr int kRouteMinSlice = 128;
__host__ __device__ inline int route_max_slices(int d) { return d / kRouteMinSlice > 1 ? d / kRouteMinSlice : 1; }

template <typename ET>
__device__ __forceinline__ void route_logits_dispatch(const KArgs &a, int t0, char *smem, int k0, int k1, bool bias) {
    const RouteShape rs = route_shape(a.E, (int)sizeof(ET));
    if (rs.parts == 4)
        route_logits<ET, 1, 4>(a, t0, smem, k0, k1, bias);
    else if (rs.parts == 2) {
        if (rs.nbw == 1)
            route_logits<ET, 1, 2>(a, t0, smem, k0, k1, bias);
        else
            route_logits<ET, 2, 2>(a, t0, smem, k0, k1, bias);
    } else if (rs.nbw == 1)
        route_logits<ET, 1, 1>(a, t0, smem, k0, k1, bias);
    else if (rs.nbw == 2)
        route_logits<ET, 2, 1>(a, t0, smem, k0, k1, bias);
    else if (rs.nbw == 3)
        route_logits<ET, 3, 1>(a, t0, smem, k0, k1, bias);
    else
        route_logits<ET, 4, 1>(a, t0, smem, k0, k1, bias);
}

// ---- bf16 problems inside the megakernel: screen in bf16, decide in fp64 -----
//
// The fp64 matrix cores deliver 30-45 TFLOP/s, which makes the exact logits of
// all E experts the longest part of a gate task by far.  Only the k largest
// matter, so the task first computes every logit approximately on the bf16
// matrix cores together with a rigorous bound on its error, keeps the experts
// that could be among the k largest, and computes exact fp64 logits for those
// few only.  The result is identical to selecting on exact logits of all
// experts:
//   approximate  L~[t,e] = sum_i x*w (fp32 accumulation of exact products) + bias
//   bound        eps[t,e] >= |L~ - L|, from A[t,e] = sum_i |x|*|w| (second MFMA on the
//                magnitudes): every one of the d additions rounds (or truncates) by at
//                most 2^-23 of a partial sum that is at most A, so |L~ - L| <= d * 2^-23 * A
//                and twice that is taken, plus the rounding of the bias addition
//   threshold    tau[t] = the k-th largest of (L~ - eps): at least k experts have an exact
//                logit >= tau
//   candidates   {e : L~ + eps >= tau}: every expert whose exact logit reaches the k-th
//                largest exact logit is among them, ties included
// Both MFMA operands must be contiguous along the reduction: x is, the gate
// weights are not, so the front of the kernel first writes their transpose
// WgT[E][d] into the workspace (wgt_task).  If a token ever has more than 64
// candidates (logits closer together than their error bound, e.g. all equal)
// the task falls back to exact logits for all experts.

constexpr int kWgtTile = 64;  // transposition tile: 64 reduction indices x 64 experts
__host__ __device__ inline int wgt_tasks(int d, int E) { return (d / kWgtTile) * ((E + kWgtTile - 1) / kWgtTile); }

// WgT[e][k0 .. k0+64) = Wg[k0 .. k0+64)[e] for 64 experts, through LDS.
__device__ __forceinline__ void wgt_task(const KArgs &a, int task, char *smem) {
    const int tid = threadIdx.x;
    const int E = a.E, d = a.d;
    const int ebn = (E + kWgtTile - 1) / kWgtTile;
    const int k0 = (task / ebn) * kWgtTile, e0 = (task % ebn) * kWgtTile;
    constexpr int LD = kWgtTile + 2;  // LDS row length in elements (odd number of dwords: column reads spread over banks)
    bf16_t *tile = (bf16_t *)smem;    // [64 k][LD]
    const bf16_t *Wg = (const bf16_t *)a.Wg;
    bf16_t *WgT = (bf16_t *)a.WgT;
    if ((E & 7) == 0) {
        // 16-byte pieces both ways, all loads of a thread in flight together: this task sits in front of
        // every gate task, so its latency is the kernel's
        constexpr int PPT = kWgtTile * kWgtTile / 8 / kThreads;  // pieces per thread
        u32x4_t v[PPT];
#pragma unroll
        for (int u = 0; u < PPT; ++u) {
            const int q = tid + kThreads * u, kk = q >> 3, e = e0 + (q & 7) * 8;
            v[u] = u32x4_t{0u, 0u, 0u, 0u};
            if (e < E) v[u] = *(const u32x4_t *)(Wg + (size_t)(k0 + kk) * E + e);
        }
#pragma unroll
        for (int u = 0; u < PPT; ++u) {
            const int q = tid + kThreads * u, kk = q >> 3, pc = q & 7;
            u32 *dst = (u32 *)(tile + kk * LD + pc * 8);
#pragma unroll
            for (int i = 0; i < 4; ++i) dst[i] = v[u][i];
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < PPT; ++u) {
            const int q = tid + kThreads * u, ee = q >> 3, kp = (q & 7) * 8;
            u32x4_t o;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                o[i] = (u32)tile[(kp + 2 * i) * LD + ee] | ((u32)tile[(kp + 2 * i + 1) * LD + ee] << 16);
            if (e0 + ee < E) *(u32x4_t *)(WgT + (size_t)(e0 + ee) * d + k0 + kp) = o;
        }
        __syncthreads();
        return;
    }
    for (int q = tid; q < kWgtTile * kWgtTile; q += kThreads) {
        const int kk = q / kWgtTile, ee = q % kWgtTile;
        tile[kk * LD + ee] = (e0 + ee < E) ? Wg[(size_t)(k0 + kk) * E + e0 + ee] : (bf16_t)0;
    }
    __syncthreads();
    for (int q = tid; q < kWgtTile * kWgtTile / 2; q += kThreads) {  // two reduction indices per store
        const int ee = q / (kWgtTile / 2), kk = (q % (kWgtTile / 2)) * 2;
        if (e0 + ee < E)
            *(u32 *)(WgT + (size_t)(e0 + ee) * d + k0 + kk) = (u32)tile[kk * LD + ee] | ((u32)tile[(kk + 1) * LD + ee] << 16);
    }
    __syncthreads();
}

__device__ __forceinline__ u32 float_key(float f) {  // order-preserving map of floats to unsigned integers
    const u32 u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

constexpr int kMaxCand = 64;
// LDS of the screened gate: approximate logits and bounds, candidate lists, exact logits, the selection
__host__ __device__ inline size_t screen_smem_bytes(int E) {
    return (size_t)kRouteTokens * E * 8 + (size_t)kRouteTokens * kMaxCand * 12 + (size_t)kRouteTokens * 32 * 12 + 64;
}

// Returns true if the selection was made (my_e[i] = expert of output position `lane` of the
// wavefront's token i, for lanes < k; idx and w written), false if the task must fall back to
// exact logits of all experts (nothing written).
template <int NBW>
__device__ __forceinline__ bool route_screened(const KArgs &a, int t0, char *smem, int (&my_e)[kRouteTokens / 4]) {
    constexpr int TPW = kRouteTokens / 4;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int E = a.E, d = a.d, k = a.k;
    const int li = lane & 15, kq = lane >> 4;
    float *Ls = (float *)smem;                                  // [16][E] approximate logits
    float *As = Ls + kRouteTokens * E;                          // [16][E] error bounds
    int *cand = (int *)(As + kRouteTokens * E);                 // [16][64] candidate experts
    double *exact = (double *)(cand + kRouteTokens * kMaxCand); // [16][64] their exact logits
    double *sel_v = exact + kRouteTokens * kMaxCand;            // [16][32] selected logits by output position
    int *sel_e = (int *)(sel_v + kRouteTokens * 32);            // [16][32]
    int *s_ncand = sel_e + kRouteTokens * 32;                   // [16] (0 = fall back)
    const bf16_t *x = (const bf16_t *)a.x;
    const bf16_t *WgT = (const bf16_t *)a.WgT;
    MOE_TT_BEGIN();

    // ---- screen: D[token][expert] on the bf16 matrix cores (16 x 16 x 32), values and magnitudes.
    // Lane l feeds token (or expert) l % 16 and reduction indices 8 * (l / 16) .. + 7 of a chunk of 32.
    {
        const int tok = min(t0 + li, a.T - 1);
        const bf16_t *xrow = x + (size_t)tok * d + 8 * kq;
        const bf16_t *wrow[NBW];
#pragma unroll
        for (int b = 0; b < NBW; ++b) {
            const int e = min((wave + 4 * b) * 16 + li, E - 1);
            wrow[b] = WgT + (size_t)e * d + 8 * kq;
        }
        f32x4_t acc[NBW], mag[NBW];
#pragma unroll
        for (int b = 0; b < NBW; ++b) {
            acc[b] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            mag[b] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        }
        const u32x4_t absmask = u32x4_t{0x7fff7fffu, 0x7fff7fffu, 0x7fff7fffu, 0x7fff7fffu};
        // U chunks of 32 per step; the loads of the next step are issued before this step's
        // multiplications: the loop does almost no arithmetic per byte, so what counts is how many
        // loads are in flight all the time
        constexpr int U = NBW <= 2 ? 8 : 4;
        const int nchunk = d / 32;
        struct Batch {
            u32x4_t xv[U], wv[U][NBW];
        };
        auto fetch = [&](int c0, Batch &r) __attribute__((always_inline)) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = min(c0 + u, nchunk - 1);  // past the end: repeat the last chunk, masked in mul()
                r.xv[u] = *(const u32x4_t *)(xrow + c * 32);
#pragma unroll
                for (int b = 0; b < NBW; ++b) r.wv[u][b] = *(const u32x4_t *)(wrow[b] + c * 32);
            }
        };
        auto mul = [&](int c0, const Batch &r) __attribute__((always_inline)) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const u32 live = (c0 + u < nchunk) ? ~0u : 0u;
                const u32x4_t xl = r.xv[u] & u32x4_t{live, live, live, live};
                const u32x4_t xa = xl & absmask;
#pragma unroll
                for (int b = 0; b < NBW; ++b) {
                    const u32x4_t wa = r.wv[u][b] & absmask;
                    acc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, xl),
                                                                     __builtin_bit_cast(bf16x8_t, r.wv[u][b]), acc[b], 0, 0, 0);
                    mag[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, xa),
                                                                     __builtin_bit_cast(bf16x8_t, wa), mag[b], 0, 0, 0);
                }
            }
        };
        Batch r0, r1;
        fetch(0, r0);
        for (int c0 = 0; c0 < nchunk; c0 += 2 * U) {
            fetch(c0 + U, r1);
            mul(c0, r0);
            fetch(c0 + 2 * U, r0);
            mul(c0 + U, r1);
        }
        // D layout: lane l, register v -> token 4 * (l / 16) + v, expert (block) l % 16
        const float scale = (float)(d + 64) * (1.0f / 4194304.0f);  // (d + 64) * 2^-22
#pragma unroll
        for (int b = 0; b < NBW; ++b) {
            const int e = (wave + 4 * b) * 16 + li;
            if (e < E) {
                const float bias = a.bias ? a.bias[e] : 0.f;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int t = 4 * kq + v;
                    const float l = acc[b][v] + bias;
                    Ls[t * E + e] = l;
                    As[t * E + e] = 1.01f * (mag[b][v] * scale + (fabsf(l) + fabsf(bias)) * (1.0f / 4194304.0f)) + 1e-30f;
                }
            }
        }
    }
    __syncthreads();
    MOE_TT(a.ctrl, 40);

    // ---- threshold and candidates: the wavefront's four tokens side by side (independent chains)
    {
        u32 klo[TPW][4], khi[TPW][4], K[TPW];
#pragma unroll
        for (int i = 0; i < TPW; ++i) {
            const int tl = wave + 4 * i;
            K[i] = 0u;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int e = lane + 64 * q;
                klo[i][q] = 0u;
                khi[i][q] = 0u;
                if (e < E) {
                    const float l = Ls[tl * E + e], eps = As[tl * E + e];
                    klo[i][q] = float_key(l - eps);
                    khi[i][q] = float_key(l + eps);
                }
            }
        }
        // the k-th largest lower bound: largest key K with at least k lower bounds >= K, found bit by
        // bit; the lowest 8 bits are left zero (a slightly smaller threshold is still a valid one)
        for (int bit = 31; bit >= 8; --bit) {
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                const u32 trial = K[i] | (1u << bit);
                int cnt = 0;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (64 * q < E) cnt += __popcll(__ballot(klo[i][q] >= trial));
                if (cnt >= k) K[i] = trial;
            }
        }
#pragma unroll
        for (int i = 0; i < TPW; ++i) {
            const int tl = wave + 4 * i;
            int before = 0, mine[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const bool in = (lane + 64 * q < E) && khi[i][q] >= K[i];
                const u64 m = __ballot(in);
                mine[q] = in ? before + __popcll(m & ((1ull << lane) - 1ull)) : -1;
                before += __popcll(m);
            }
            const int n = before;
            if (n <= kMaxCand) {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (mine[q] >= 0) cand[tl * kMaxCand + mine[q]] = lane + 64 * q;
            }
            if (lane == 0) s_ncand[tl] = (n <= kMaxCand) ? n : 0;
        }
    }
    __syncthreads();
    bool ok = true;  // (tokens past T repeat token T-1: they fail only if it does)
    for (int t = 0; t < kRouteTokens; ++t) ok = ok && s_ncand[t] > 0;
    if (!ok) {
#ifdef MOE_TILE_TIMING
        if (tid == 0) atomicAdd(&a.ctrl->dbg[44], 1ull);
#endif
        __syncthreads();
        return false;
    }

    MOE_TT(a.ctrl, 41);
    // ---- exact fp64 logits of the candidates: 16 lanes per candidate, four candidates at a time
    {
        const int g = lane >> 4, j = lane & 15;
#pragma unroll
        for (int i = 0; i < TPW; ++i) {
            const int tl = wave + 4 * i;
            const int tok = min(t0 + tl, a.T - 1);
            const int n = s_ncand[tl];
            const bf16_t *xr = x + (size_t)tok * d;
            for (int base = 0; base < n; base += 4) {
                const int ci = min(base + g, n - 1);
                const int e = cand[tl * kMaxCand + ci];
                const bf16_t *wr = WgT + (size_t)e * d;
                // 16-byte pieces j, j + 16, ... of the two rows, eight pieces' loads in flight at a time;
                // a bf16 x bf16 product is exact in fp32, the accumulation is in fp64, in four
                // independent chains (a single one is bound by the latency of the fp64 adder)
                double s4[4] = {0.0, 0.0, 0.0, 0.0};
                constexpr int PB = 8;
                for (int m0 = 8 * j; m0 < d; m0 += 128 * PB) {
                    u32x4_t xv[PB], wv[PB];
#pragma unroll
                    for (int u = 0; u < PB; ++u) {
                        const int m = m0 + 128 * u;
                        if (m < d) {
                            xv[u] = *(const u32x4_t *)(xr + m);
                            wv[u] = *(const u32x4_t *)(wr + m);
                        }
                    }
#pragma unroll
                    for (int u = 0; u < PB; ++u) {
                        if (m0 + 128 * u < d) {
#pragma unroll
                            for (int c = 0; c < 4; ++c) {
                                const float p0 = __uint_as_float(xv[u][c] << 16) * __uint_as_float(wv[u][c] << 16);
                                const float p1 = __uint_as_float(xv[u][c] & 0xffff0000u) * __uint_as_float(wv[u][c] & 0xffff0000u);
                                s4[c] += (double)p0;
                                s4[c] += (double)p1;
                            }
                        }
                    }
                }
                double sum = (s4[0] + s4[1]) + (s4[2] + s4[3]);
#pragma unroll
                for (int off = 8; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, 64);
                if (j == 0 && base + g < n) exact[tl * kMaxCand + base + g] = sum + (a.bias ? (double)a.bias[e] : 0.0);
            }
        }
    }
    __syncthreads();
    MOE_TT(a.ctrl, 42);

    // ---- select: the output position of a candidate is the number of candidates that beat it
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
        const int tl = wave + 4 * i;
        const int n = s_ncand[tl];
        if (lane < n) {
            const double v = exact[tl * kMaxCand + lane];
            const int e = cand[tl * kMaxCand + lane];
            int rank = 0;
            for (int c = 0; c < n; ++c) {
                const double ov = exact[tl * kMaxCand + c];
                const int oe = cand[tl * kMaxCand + c];
                rank += (ov > v || (ov == v && oe < e)) ? 1 : 0;
            }
            if (rank < k) {
                sel_v[tl * 32 + rank] = v;
                sel_e[tl * 32 + rank] = e;
            }
        }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
        const int tl = wave + 4 * i;
        const int t = t0 + tl;
        my_e[i] = -1;
        const double m = sel_v[tl * 32];
        const double ex = (lane < k) ? exp(sel_v[tl * 32 + min(lane, k - 1)] - m) : 0.0;
        double sum = ex;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, 64);
        if (lane < k) {
            my_e[i] = sel_e[tl * 32 + lane];
            if (t < a.T) {
                a.idx[(size_t)t * k + lane] = my_e[i];
                a.w[(size_t)t * k + lane] = (float)(ex / sum);
            }
        }
    }
    __syncthreads();
    MOE_TT(a.ctrl, 43);
    return true;
}

// Exact logits of all experts in lg[16][E] (LDS) -> top-k by k rounds of a 64-lane butterfly
// argmax on (value, index), softmax over the chosen k; each wavefront selects for its four
// tokens (wave, wave + 4, ...) at once, so that the four shuffle chains overlap.
__device__ __forceinline__ void select_full(const KArgs &a, int t0, const double *lg, int (&my_e)[kRouteTokens / 4]) {
    constexpr int TPW = kRouteTokens / 4;
    const int E = a.E, k = a.k;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const double NEG = -__builtin_huge_val();
    double v[TPW][4], my_v[TPW];
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
        const int tl = wave + 4 * i;
        my_v[i] = 0.0;
#pragma unroll
        for (int q = 0; q < 4; ++q) v[i][q] = (lane + 64 * q < E) ? lg[tl * E + lane + 64 * q] : NEG;
    }
    if (E <= 64) {
        // one logit per lane: its output position is the number of logits that beat it (larger value, or
        // equal value and lower expert id: the order of the argmax rounds below), counted against
        // broadcast reads of the row; position j then goes to lane j.  E steps instead of k shuffle trees.
        int rank[TPW];
#pragma unroll
        for (int i = 0; i < TPW; ++i) rank[i] = lane < E ? 0 : (1 << 20);
        for (int c = 0; c < E; ++c) {
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                const double ov = lg[(wave + 4 * i) * E + c];
                rank[i] += (ov > v[i][0] || (ov == v[i][0] && c < lane)) ? 1 : 0;
            }
        }
        for (int j = 0; j < k; ++j) {
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                const int src = __ffsll((long long)__ballot(rank[i] == j)) - 1;
                const double bv = __shfl(v[i][0], src, 64);
                if (lane == j) {
                    my_v[i] = bv;
                    my_e[i] = src;
                }
            }
        }
    } else {
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
}

template <typename ET>
__device__ __forceinline__ bool route_screened_dispatch(const KArgs &a, int t0, char *smem, int (&my_e)[kRouteTokens / 4]) {
    if (sizeof(ET) != 2 || a.WgT == nullptr) return false;
    const int nbw = ((a.E + 15) / 16 + 3) / 4;
    if (nbw <= 1) return route_screened<1>(a, t0, smem, my_e);
    if (nbw == 2) return route_screened<2>(a, t0, smem, my_e);
    if (nbw == 3) return route_screened<3>(a, t0, smem, my_e);
    return route_screened<4>(a, t0, smem, my_e);
}

// One gate task: tokens [b*16, b*16+16) of block b = task.  With a.Wg == NULL the routing
// is an input and only the histograms are produced.
// Few tokens (a decode-sized batch) mean few blocks and an idle GPU while they run, so the
// megakernel may split the gate: a.gate_split = S > 1 tasks per block, task = b*S + s sums slice s
// of the reduction and leaves its partial logits in the workspace; whichever task of a block
// finishes last adds the S partial sums in slice order (so the result does not depend on who that
// is) and goes on to the selection; the others are done.
template <typename ET>
__device__ __forceinline__ void route_task(const KArgs &a, int task, char *smem, bool do_hist) {
    constexpr int TPW = kRouteTokens / 4;
    const int E = a.E, k = a.k;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool compute = (a.Wg != nullptr);
    const int S = (compute && a.gate_split > 1) ? a.gate_split : 1;
    const int block = task / S, slice = task % S;
    const int t0 = block * kRouteTokens;
    int my_e[TPW];
#pragma unroll
    for (int i = 0; i < TPW; ++i) my_e[i] = -1;
    MOE_TT_BEGIN();
    if (compute) {
        if (S > 1 || !route_screened_dispatch<ET>(a, t0, smem, my_e)) {
            __shared__ int s_gate_last;
            const int pieces = a.d / 16;  // slice s of S: pieces [pieces * s / S, pieces * (s + 1) / S)
            route_logits_dispatch<ET>(a, t0, smem, 16 * (int)((long long)pieces * slice / S),
                                      16 * (int)((long long)pieces * (slice + 1) / S), S == 1);
            MOE_TT(a.ctrl, 40);
            if (S > 1) {
                double *lg = (double *)smem;
                const size_t per = (size_t)kRouteTokens * E;
                double *mine = a.gate_partial + ((size_t)block * S + slice) * per;
                for (int i = threadIdx.x; i < (int)per; i += kThreads) mine[i] = lg[i];
                sync_stores();
                if (threadIdx.x == 0) {
                    fence_release(0);
                    const u32 before = atomicAdd(&a.gate_parts[block], 1u);
                    s_gate_last = (before == (u32)(S - 1)) ? 1 : 0;
                    if (s_gate_last) fence_acquire(0);
                }
                __syncthreads();
                MOE_TT(a.ctrl, 41);
                if (!s_gate_last) return;
                // (the partial sums come from memory: all S loads of two logits are issued before the first
                // addition; one load at a time, the S round trips of a logit would come one after the other)
                const double *all = a.gate_partial + (size_t)block * S * per;
                constexpr int MAXS = 16, EU = 2;  // S <= MAXS (the host's limit)
                for (int i0 = threadIdx.x; i0 < (int)per; i0 += kThreads * EU) {
                    double part[EU][MAXS];
#pragma unroll
                    for (int u = 0; u < EU; ++u) {
                        const int i = min(i0 + u * kThreads, (int)per - 1);
#pragma unroll
                        for (int s2 = 0; s2 < MAXS; ++s2)
                            if (s2 < S) part[u][s2] = all[(size_t)s2 * per + i];
                    }
#pragma unroll
                    for (int u = 0; u < EU; ++u) {
                        const int i = i0 + u * kThreads;
                        if (i < (int)per) {
                            double v = a.bias ? (double)a.bias[i % E] : 0.0;
#pragma unroll
                            for (int s2 = 0; s2 < MAXS; ++s2)
                                if (s2 < S) v += part[u][s2];
                            lg[i] = v;
                        }
                    }
                }
                __syncthreads();
            }
            MOE_TT(a.ctrl, 32);
            select_full(a, t0, (const double *)smem, my_e);
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

// fp32 tile GEMM for fp32 problems (the small validation layer): plain FMA,
// LDS-tiled, 128 x 64 outputs per workgroup, 8 x 4 per thread.  Same contract as
// the bf16 kernel: the result is left in an LDS C tile (fp32 here).
#pragma once
#include "common.hpp"

namespace moe {

struct TileF32 {
    static constexpr int BM = 128, BN = 64, BK = 16;
    static constexpr int A_LD = BM + 4;                // floats per k-row of the transposed A tile
    static constexpr int C_STRIDE = BN * 4 + 16;       // bytes per C-tile row
    static constexpr int C_BYTES = BM * C_STRIDE;
    static constexpr int STAGE = BK * A_LD * 4 + 2 * BK * BN * 4;
    static constexpr int SMEM_MAIN = (STAGE > C_BYTES) ? STAGE : C_BYTES;
};

template <bool GATED, class RowPtr, class Hook>
__device__ void gemm_tile_f32(RowPtr rowptr, const float *B0, const float *B1, int ldb, int ncols, int K,
                              char *smem, Hook while_loading) {
    using C = TileF32;
    while_loading();  // (see gemm_tile_bf16; this loop has no loads in flight to hide it behind)
    const int tid = threadIdx.x;
    const int ty = tid >> 4, tx = tid & 15;
    float *As = (float *)smem;              // [BK][A_LD]
    float *Bs0 = As + C::BK * C::A_LD;      // [BK][BN]
    float *Bs1 = Bs0 + C::BK * C::BN;       // [BK][BN] (gated)

    const int a_row = tid >> 1, a_kq = (tid & 1) * 8;
    const float *a_src = rowptr(a_row) + a_kq;
    const int b_kr = tid >> 4;
    int b_c4 = (tid & 15) * 4;
    const int b_col = (b_c4 < ncols) ? b_c4 : 0;

    float g[8][4], u[8][4];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) g[i][j] = u[i][j] = 0.f;

    for (int k0 = 0; k0 < K; k0 += C::BK) {
        const float4 av = *(const float4 *)(a_src + k0);
        const float4 aw = *(const float4 *)(a_src + k0 + 4);
        As[(a_kq + 0) * C::A_LD + a_row] = av.x;
        As[(a_kq + 1) * C::A_LD + a_row] = av.y;
        As[(a_kq + 2) * C::A_LD + a_row] = av.z;
        As[(a_kq + 3) * C::A_LD + a_row] = av.w;
        As[(a_kq + 4) * C::A_LD + a_row] = aw.x;
        As[(a_kq + 5) * C::A_LD + a_row] = aw.y;
        As[(a_kq + 6) * C::A_LD + a_row] = aw.z;
        As[(a_kq + 7) * C::A_LD + a_row] = aw.w;
        *(float4 *)&Bs0[b_kr * C::BN + b_c4] = *(const float4 *)(B0 + (size_t)(k0 + b_kr) * ldb + b_col);
        if (GATED)
            *(float4 *)&Bs1[b_kr * C::BN + b_c4] = *(const float4 *)(B1 + (size_t)(k0 + b_kr) * ldb + b_col);
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < C::BK; ++kk) {
            const float4 a4 = *(const float4 *)&As[kk * C::A_LD + ty * 8];
            const float4 a5 = *(const float4 *)&As[kk * C::A_LD + ty * 8 + 4];
            const float4 b4 = *(const float4 *)&Bs0[kk * C::BN + tx * 4];
            const float a[8] = {a4.x, a4.y, a4.z, a4.w, a5.x, a5.y, a5.z, a5.w};
            const float b[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) g[i][j] = fmaf(a[i], b[j], g[i][j]);
            if (GATED) {
                const float4 c4 = *(const float4 *)&Bs1[kk * C::BN + tx * 4];
                const float c[4] = {c4.x, c4.y, c4.z, c4.w};
#pragma unroll
                for (int i = 0; i < 8; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) u[i][j] = fmaf(a[i], c[j], u[i][j]);
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float4 o;
        if (GATED) {
            o.x = g[i][0] / (1.0f + expf(-g[i][0])) * u[i][0];
            o.y = g[i][1] / (1.0f + expf(-g[i][1])) * u[i][1];
            o.z = g[i][2] / (1.0f + expf(-g[i][2])) * u[i][2];
            o.w = g[i][3] / (1.0f + expf(-g[i][3])) * u[i][3];
        } else {
            o = make_float4(g[i][0], g[i][1], g[i][2], g[i][3]);
        }
        *(float4 *)(smem + (ty * 8 + i) * C::C_STRIDE + tx * 16) = o;
    }
    __syncthreads();
}

}  // namespace moe

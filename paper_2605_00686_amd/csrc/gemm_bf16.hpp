// bf16 MFMA tile GEMM for the expert FFN (paper section 2.1 step 3): one
// workgroup computes a BM x BN block of  A[rows, K] * B[K, cols]  with fp32
// accumulation and leaves the result, rounded to bf16, in an LDS "C tile" that
// the caller stores or publishes.
//
// Layout notes (gfx950):
//  * A rows are K-contiguous in memory; weights are [K, N] row-major, i.e.
//    N-contiguous.  v_mfma_f32_32x32x16_bf16 wants, per lane, 8 consecutive K
//    values of one row / column.  A fragments are therefore plain 16-byte LDS
//    reads; weight fragments use ds_read_b64_tr_b16, which transposes a
//    4(K) x 16(N) block across 16 lanes on the way out of LDS.
//  * The product is formed transposed (weights as the first MFMA operand), so
//    a lane ends up with 4 consecutive output columns of one output row and
//    can write them as one 8-byte piece.
//  * LDS tiles are XOR-swizzled so that both the 16-byte writes and the
//    fragment reads are bank-conflict free.
#pragma once
#include "common.hpp"

namespace moe {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) short s16x8_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

// MB x NB MFMA blocks (32 x 32) per wavefront, WM x WN wavefronts (WM*WN = 4).
template <int MB_, int NB_, int WM_, int WN_>
struct TileCfg {
    static constexpr int MB = MB_, NB = NB_, WM = WM_, WN = WN_;
    static constexpr int BM = 32 * MB * WM;   // rows per tile
    static constexpr int BNW = 32 * NB;       // weight columns per wavefront
    static constexpr int BN = BNW * WN;       // weight columns per tile (gated: half from W1, half from W3)
    static constexpr int BK = 64;             // K per pipeline stage
    static constexpr int A_BYTES = BM * BK * 2;
    static constexpr int B_BYTES = BK * BN * 2;
    static constexpr int STAGE = A_BYTES + B_BYTES;
    static constexpr int C_STRIDE = BN * 2 + 16;  // bytes per row of the LDS C tile (bf16, padded)
    static constexpr int C_BYTES = BM * C_STRIDE;
    static constexpr int SMEM_MAIN = (2 * STAGE > C_BYTES) ? 2 * STAGE : C_BYTES;
    static constexpr int NA = BM / 32;   // 16-byte A pieces per thread per stage
    static constexpr int CPR = BN / 8;   // 16-byte pieces per weight row
    static constexpr int RPP = kThreads / CPR;  // weight rows covered per pass
    static constexpr int NBL = BK / RPP;        // weight pieces per thread per stage
    static_assert(WM * WN == 4, "four wavefronts per workgroup");
    static_assert(kThreads % CPR == 0 && BK % RPP == 0, "weight tile must divide evenly");
};

__device__ __forceinline__ float silu_mul(float g, float u) { return g / (1.0f + __expf(-g)) * u; }

// Main loop + epilogue into LDS.
//   rowptr(r): pointer to local row r of A (K contiguous bf16), valid for every r < BM
//   B0 / B1:   weight matrices already offset to the tile's first column; row stride ldb.
//              GATED: LDS columns [0, BN/2) come from B0 and [BN/2, BN) from B1, and the
//              C tile holds silu(A*B0) * (A*B1) with BN/2 columns; else C = A*B0, BN columns.
//   ncols:     valid columns of each weight matrix from its first column (others: don't care)
//   K:         multiple of 64
// On return (after a barrier) the C tile is complete in smem; row stride C_STRIDE bytes.
template <class C, bool GATED, class RowPtr>
__device__ void gemm_tile_bf16(RowPtr rowptr, const bf16_t *B0, const bf16_t *B1, int ldb, int ncols,
                               int K, char *smem) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / C::WN, wn = wave % C::WN;
    constexpr int HALF = C::BN / 2;

    // ---- global -> register -> LDS staging assignments
    const int a_chunk = tid & 7;  // 16-byte piece within the 128-byte K slice of a row
    const bf16_t *a_ptr[C::NA];
    int a_lds[C::NA];
#pragma unroll
    for (int i = 0; i < C::NA; ++i) {
        const int row = (tid >> 3) + 32 * i;
        a_ptr[i] = rowptr(row) + a_chunk * 8;
        a_lds[i] = row * 128 + ((a_chunk ^ ((row >> 1) & 7)) << 4);
    }
    const int b_chunk = tid % C::CPR;
    const int b_row0 = tid / C::CPR;
    const bf16_t *b_ptr;
    {
        int col = b_chunk * 8;
        const bf16_t *base = B0;
        if (GATED && col >= HALF) {
            base = B1;
            col -= HALF;
        }
        if (col >= ncols) col = 0;  // out-of-range columns: read something valid, never stored
        b_ptr = base + col;
    }
    int b_lds[C::NBL];
#pragma unroll
    for (int i = 0; i < C::NBL; ++i) {
        const int kr = b_row0 + C::RPP * i;
        const int phys = ((((b_chunk >> 2) ^ (kr & 3)) << 2) | (b_chunk & 3));
        b_lds[i] = kr * (C::BN * 2) + (phys << 4);
    }

    // ---- fragment read addresses
    const int a_rd_row = wm * 32 * C::MB + (lane & 31);
    const int a_rd_swz = ((lane & 31) >> 1) & 7;
    const int a_rd_half = lane >> 5;
    int b_rd_col[C::NB];
#pragma unroll
    for (int nb = 0; nb < C::NB; ++nb) {
        int cb;
        if (GATED)
            cb = (nb < C::NB / 2) ? wn * (C::BNW / 2) + nb * 32 : HALF + wn * (C::BNW / 2) + (nb - C::NB / 2) * 32;
        else
            cb = wn * C::BNW + nb * 32;
        const int col = cb + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
        const int chunk = col >> 3;
        const int phys = ((((chunk >> 2) ^ ((lane & 15) >> 2)) << 2) | (chunk & 3));
        b_rd_col[nb] = (phys << 4) + ((col & 7) << 1);
    }
    const int b_rd_row = 8 * (lane >> 5) + ((lane & 15) >> 2);

    f32x16_t acc[C::MB][C::NB];
#pragma unroll
    for (int mb = 0; mb < C::MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < C::NB; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][nb][v] = 0.f;

    uint4 ra[C::NA], rb[C::NBL];
    auto gload = [&](int kt) {
#pragma unroll
        for (int i = 0; i < C::NA; ++i) ra[i] = *(const uint4 *)(a_ptr[i] + kt * C::BK);
#pragma unroll
        for (int i = 0; i < C::NBL; ++i)
            rb[i] = *(const uint4 *)(b_ptr + (size_t)(kt * C::BK + b_row0 + C::RPP * i) * ldb);
    };
    auto lstore = [&](int buf) {
        char *sa = smem + buf * C::STAGE;
        char *sb = sa + C::A_BYTES;
#pragma unroll
        for (int i = 0; i < C::NA; ++i) *(uint4 *)(sa + a_lds[i]) = ra[i];
#pragma unroll
        for (int i = 0; i < C::NBL; ++i) *(uint4 *)(sb + b_lds[i]) = rb[i];
    };
    auto compute = [&](int buf) {
        const char *sa = smem + buf * C::STAGE;
        const char *sb = sa + C::A_BYTES;
#pragma unroll
        for (int kk = 0; kk < C::BK / 16; ++kk) {
            bf16x8_t af[C::MB], bfr[C::NB];
#pragma unroll
            for (int mb = 0; mb < C::MB; ++mb) {
                const int off = (a_rd_row + mb * 32) * 128 + ((((kk << 1) | a_rd_half) ^ a_rd_swz) << 4);
                af[mb] = __builtin_bit_cast(bf16x8_t, *(const uint4 *)(sa + off));
            }
#pragma unroll
            for (int nb = 0; nb < C::NB; ++nb) {
                const int off = (kk * 16 + b_rd_row) * (C::BN * 2) + b_rd_col[nb];
                s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (s16x4_t __attribute__((address_space(3))) *)(sb + off));
                s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (s16x4_t __attribute__((address_space(3))) *)(sb + off + 4 * C::BN * 2));
                s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                bfr[nb] = __builtin_bit_cast(bf16x8_t, v);
            }
#pragma unroll
            for (int mb = 0; mb < C::MB; ++mb)
#pragma unroll
                for (int nb = 0; nb < C::NB; ++nb)
                    acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[nb], af[mb], acc[mb][nb], 0, 0, 0);
        }
    };

    const int nk = K / C::BK;
    gload(0);
    lstore(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) gload(kt + 1);
        compute(kt & 1);
        if (kt + 1 < nk) lstore((kt + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue: fp32 accumulators -> bf16 C tile in LDS.  Lane l holds, for
    // MFMA block (mb, nb) and register group vq, output row (l & 31) and the 4
    // consecutive columns 8*vq + 4*(l >> 5) .. +3 of that block.
    const int c_row = wm * 32 * C::MB + (lane & 31);
#pragma unroll
    for (int mb = 0; mb < C::MB; ++mb) {
        char *crow = smem + (c_row + mb * 32) * C::C_STRIDE;
        if (GATED) {
#pragma unroll
            for (int nb = 0; nb < C::NB / 2; ++nb)
#pragma unroll
                for (int vq = 0; vq < 4; ++vq) {
                    const int col = wn * (C::BNW / 2) + nb * 32 + 8 * vq + 4 * (lane >> 5);
                    const f32x16_t &g = acc[mb][nb];
                    const f32x16_t &u = acc[mb][nb + C::NB / 2];
                    uint2 o;
                    o.x = pack_bf16x2(silu_mul(g[4 * vq], u[4 * vq]), silu_mul(g[4 * vq + 1], u[4 * vq + 1]));
                    o.y = pack_bf16x2(silu_mul(g[4 * vq + 2], u[4 * vq + 2]), silu_mul(g[4 * vq + 3], u[4 * vq + 3]));
                    *(uint2 *)(crow + col * 2) = o;
                }
        } else {
#pragma unroll
            for (int nb = 0; nb < C::NB; ++nb)
#pragma unroll
                for (int vq = 0; vq < 4; ++vq) {
                    const int col = wn * C::BNW + nb * 32 + 8 * vq + 4 * (lane >> 5);
                    const f32x16_t &y = acc[mb][nb];
                    uint2 o;
                    o.x = pack_bf16x2(y[4 * vq], y[4 * vq + 1]);
                    o.y = pack_bf16x2(y[4 * vq + 2], y[4 * vq + 3]);
                    *(uint2 *)(crow + col * 2) = o;
                }
        }
    }
    __syncthreads();
}

}  // namespace moe

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
    static_assert(WM * WN == 4, "four wavefronts per workgroup");
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

    // ---- global -> LDS staging.  Loads go straight into LDS (no staging
    // registers): one instruction moves 64 lanes x 16 bytes into 1 KB of
    // consecutive LDS, lane l landing at byte 16*l, so the XOR swizzle is
    // applied by choosing WHICH global piece each lane fetches.
    // A: 1 KB = 8 rows x 128 bytes; wavefront w issues rows [w*8*NA8 ...), NA8 = BM/32 per stage.
    // B: 1 KB = 2 weight rows x 512 bytes (BN = 256).
    static_assert(C::BN == 256, "weight tile rows are 512 bytes");
    constexpr int NAI = C::BM / 32;  // A instructions per wavefront per stage
    constexpr int NBI = C::BK / 8;   // B instructions per wavefront per stage (64 rows / 2 rows / 4 waves)
    const int uw = __builtin_amdgcn_readfirstlane(wave);
    const bf16_t *a_ptr[NAI];
#pragma unroll
    for (int i = 0; i < NAI; ++i) {
        const int row = (uw * NAI + i) * 8 + (lane >> 3);
        const int chunk = (lane & 7) ^ ((row >> 1) & 7);
        a_ptr[i] = rowptr(row) + chunk * 8;
    }
    // weight rows of instruction i: kr = (uw*NBI + i)*2 + (lane >> 5); kr & 3 depends on i's parity only
    const bf16_t *b_ptr[2];
#pragma unroll
    for (int par = 0; par < 2; ++par) {
        const int kr = par * 2 + (lane >> 5);
        const int pc = lane & 31;
        const int chunk = ((((pc >> 2) ^ (kr & 3)) << 2) | (pc & 3));
        int col = chunk * 8;
        const bf16_t *base = B0;
        if (GATED && col >= HALF) {
            base = B1;
            col -= HALF;
        }
        if (col >= ncols) col = 0;  // out-of-range columns: read something valid, never stored
        b_ptr[par] = base + col + (size_t)(lane >> 5) * ldb;
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

    typedef __attribute__((address_space(3))) void lds_void_t;
    auto issue_loads = [&](int kt, int buf) {
        char *sa = smem + buf * C::STAGE;
        char *sb = sa + C::A_BYTES;
#pragma unroll
        for (int i = 0; i < NAI; ++i)
            __builtin_amdgcn_global_load_lds(a_ptr[i] + kt * C::BK, (lds_void_t *)(sa + (uw * NAI + i) * 1024), 16, 0, 0);
#pragma unroll
        for (int i = 0; i < NBI; ++i) {
            const int r2 = (uw * NBI + i) * 2;  // first of the two weight rows of this instruction
            __builtin_amdgcn_global_load_lds(b_ptr[i & 1] + (size_t)(kt * C::BK + r2) * ldb,
                                             (lds_void_t *)(sb + r2 * (C::BN * 2)), 16, 0, 0);
        }
    };
    auto wait_loads = [&]() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };
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
    issue_loads(0, 0);
    wait_loads();
    __syncthreads();
    for (int kt = 0; kt < nk - 1; ++kt) {
        issue_loads(kt + 1, (kt + 1) & 1);  // in flight while this stage is consumed
        compute(kt & 1);
        wait_loads();
        __syncthreads();
    }
    compute((nk - 1) & 1);
    __syncthreads();

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

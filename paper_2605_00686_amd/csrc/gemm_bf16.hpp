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
//  * Global loads go straight into LDS (no staging registers): one instruction
//    moves 64 lanes x 16 bytes into 1 KB of consecutive LDS, lane l landing at
//    byte 16*l.  LDS tiles are XOR-swizzled so that fragment reads are free of
//    bank conflicts; since the destination of a direct load is fixed, the
//    swizzle is applied by choosing WHICH global piece each lane fetches.
//  * NS pipeline stages of BK reduction steps each: loads run NS-1 stages ahead
//    of the MFMAs, one workgroup barrier per stage.
#pragma once
#include "common.hpp"

namespace moe {

typedef __attribute__((ext_vector_type(8))) short s16x8_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

// MB x NB MFMA blocks (32 x 32) per wavefront, WM x WN wavefronts (WM*WN = 4),
// BK reduction steps per stage (32 or 64), NS stages.
template <int MB_, int NB_, int WM_, int WN_, int BK_, int NS_>
struct TileCfg {
    static constexpr int MB = MB_, NB = NB_, WM = WM_, WN = WN_, BK = BK_, NS = NS_;
    static constexpr int BM = 32 * MB * WM;   // rows per tile
    static constexpr int BNW = 32 * NB;       // weight columns per wavefront
    static constexpr int BN = BNW * WN;       // weight columns per tile (gated: half from W1, half from W3)
    static constexpr int A_ROW = BK * 2;      // bytes of one A row in a stage
    static constexpr int A_BYTES = BM * A_ROW;
    static constexpr int B_BYTES = BK * BN * 2;
    static constexpr int STAGE = A_BYTES + B_BYTES;
    static constexpr int C_STRIDE = BN * 2 + 16;  // bytes per row of the LDS C tile (bf16, padded)
    static constexpr int C_BYTES = BM * C_STRIDE;
    static constexpr int SMEM_MAIN = (NS * STAGE > C_BYTES) ? NS * STAGE : C_BYTES;
    // direct loads: 1 KB each; every wavefront issues the same number per stage
    static constexpr int A_INSTR = A_BYTES / 1024;
    static constexpr int NAI = (A_INSTR + 3) / 4;   // A loads per wavefront per stage
    static constexpr int NBI = B_BYTES / 1024 / 4;  // B loads per wavefront per stage
    static constexpr int LPS = NAI + NBI;           // loads per wavefront per stage
    static_assert(WM * WN == 4, "four wavefronts per workgroup");
    static_assert(BN == 256, "weight tile rows are 512 bytes");
    static_assert(BK == 32 || BK == 64, "stage depth");
    static_assert((NS - 1) * LPS <= 63, "vmcnt range");
};

// silu(g) * u; the hardware reciprocal (1 ulp) is far inside the bf16 rounding of the result
__device__ __forceinline__ float silu_mul(float g, float u) { return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u; }

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Main loop + epilogue into LDS.
//   rowptr(r): pointer to local row r of A (K contiguous bf16), valid for every r < BM
//   B0 / B1:   weight matrices already offset to the tile's first column; row stride ldb.
//              GATED: LDS columns [0, BN/2) come from B0 and [BN/2, BN) from B1, and the
//              C tile holds silu(A*B0) * (A*B1) with BN/2 columns; else C = A*B0, BN columns.
//   ncols:     valid columns of each weight matrix from its first column (others: don't care)
//   K:         multiple of 64
// On return (after a barrier) the C tile is complete in smem; row stride C_STRIDE bytes.
//   while_loading(): called by every thread once the first stages' loads are in flight, for
//              work of the caller that fits into that trip to memory (it may use barriers and
//              LDS beyond SMEM_MAIN)
// Two variations for a workgroup that takes a row block through both GEMMs of the FFN with the intermediate h
// kept in LDS (paper section 2.3: a tile traverses GEMM -> activation -> GEMM):
//   HRES: (GATED only) the result is not left in a C tile but written into `res`, an LDS buffer that holds the
//         row block's h in the layout of A stages: stage s (columns [s*BK, (s+1)*BK) of h) at res + s*A_BYTES,
//         rows of A_ROW bytes, swizzled like a staged A tile; n0 = first h column of this tile, ntot = f.
//   ARES: A is not loaded: stage s of A is read from res + s*A_BYTES (written by HRES tiles before); only the
//         weights stream through the stage buffers (their A parts stay unused); rowptr is not called.
template <class C, bool GATED, bool HRES = false, bool ARES = false, class RowPtr, class Hook>
__device__ void gemm_tile_bf16(RowPtr rowptr, const bf16_t *B0, const bf16_t *B1, int ldb, int ncols,
                               int K, char *smem, Hook while_loading, char *res = nullptr, int n0 = 0, int ntot = 0) {
    static_assert(!(HRES && !GATED) && !(HRES && ARES), "h is produced by the gated GEMM and consumed by the other one");
    constexpr int LPSX = ARES ? C::NBI : C::LPS;  // loads per wavefront per stage
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / C::WN, wn = wave % C::WN;
    constexpr int HALF = C::BN / 2;
    constexpr int CPRA = C::BK / 8;            // 16-byte pieces per A row
    constexpr int RPI = 1024 / C::A_ROW;       // A rows per load instruction
    // swizzle of the A tile: piece c of row r sits at piece c ^ swz(r)
    auto a_swz = [](int row) { return C::BK == 64 ? ((row >> 1) & 7) : ((row >> 2) & 3); };

    const int uw = __builtin_amdgcn_readfirstlane(wave);
    // ---- A loads.  Instruction (uw*NAI + i) covers rows [.. * RPI, +RPI); when the
    // tile has fewer than 4 instructions the upper wavefronts repeat the lower ones'
    // loads (same bytes to the same place) so that all wavefronts count alike.
    const bf16_t *a_ptr[C::NAI];
    int a_dst[C::NAI];
#pragma unroll
    for (int i = 0; i < C::NAI; ++i) {
        const int instr = (uw * C::NAI + i) % C::A_INSTR;
        const int row = instr * RPI + lane / CPRA;
        const int chunk = (lane % CPRA) ^ a_swz(row);
        a_ptr[i] = ARES ? nullptr : rowptr(row) + chunk * 8;
        a_dst[i] = instr * 1024;
    }
    // ---- B loads.  Instruction covers 2 weight rows (2 x 512 bytes); weight row
    // kr = (uw*NBI + i)*2 + (lane >> 5), and kr & 3 depends on i's parity only.
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
    const int a_rd_swz = a_swz(lane & 31);  // tile rows are multiples of 32 apart: same swizzle
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

    // load number i (0 .. LPS-1) of stage kt into stage buffer buf.  Written as
    // inline assembly on purpose: the compiler tracks its own LDS-DMA loads and,
    // unable to prove that a later ds_read touches another buffer, puts
    // s_waitcnt vmcnt(0) in front of the next LDS read, which serialises the
    // whole pipeline.  Here the waits are placed by hand (wait_vmcnt below).
    // M0 carries the LDS byte address of the 1 KB destination.
    const u32 lds_base = (u32)(uintptr_t)(__attribute__((address_space(3))) char *)smem;
    auto dma16 = [&](const bf16_t *src, u32 lds_addr) {
        // the address is uniform by construction; make the compiler see it as scalar
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                     :
                     : "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(src)
                     : "m0");
    };
    auto issue_one = [&](int kt, int buf, int i) {
        const u32 sa = lds_base + buf * C::STAGE;
        const u32 sb = sa + C::A_BYTES;
        if (!ARES && i < C::NAI) {
            dma16(a_ptr[i] + kt * C::BK, sa + a_dst[i]);
        } else {
            const int j = ARES ? i : i - C::NAI;
            const int r2 = (uw * C::NBI + j) * 2;  // first of the two weight rows of this instruction
            dma16(b_ptr[j & 1] + (size_t)(kt * C::BK + r2) * ldb, sb + r2 * (C::BN * 2));
        }
    };
    auto issue_loads = [&](int kt, int buf) {
#pragma unroll
        for (int i = 0; i < LPSX; ++i) issue_one(kt, buf, i);
    };
    constexpr int KK = C::BK / 16;  // MFMA reduction steps per stage
    struct Frag {
        bf16x8_t a[C::MB], b[C::NB];
    };
    auto load_frag = [&](int buf, int kt, int kk, Frag &f) {  // fragments of step kk of stage kt, which sits in buffer buf
        const char *sa = ARES ? res + kt * C::A_BYTES : smem + buf * C::STAGE;
        const char *sb = smem + buf * C::STAGE + C::A_BYTES;
#pragma unroll
        for (int mb = 0; mb < C::MB; ++mb) {
            const int off = (a_rd_row + mb * 32) * C::A_ROW + ((((kk << 1) | a_rd_half) ^ a_rd_swz) << 4);
            f.a[mb] = __builtin_bit_cast(bf16x8_t, *(const uint4 *)(sa + off));
        }
#pragma unroll
        for (int nb = 0; nb < C::NB; ++nb) {
            const int off = (kk * 16 + b_rd_row) * (C::BN * 2) + b_rd_col[nb];
            s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (s16x4_t __attribute__((address_space(3))) *)(sb + off));
            s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (s16x4_t __attribute__((address_space(3))) *)(sb + off + 4 * C::BN * 2));
            s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            f.b[nb] = __builtin_bit_cast(bf16x8_t, v);
        }
    };
    auto mfma_all = [&](const Frag &f) {
#pragma unroll
        for (int mb = 0; mb < C::MB; ++mb)
#pragma unroll
            for (int nb = 0; nb < C::NB; ++nb)
                acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[nb], f.a[mb], acc[mb][nb], 0, 0, 0);
    };
    // One MFMA step of the software pipeline: fetch the fragments `nxt` of the
    // step after, issue a share of the refill loads, multiply with `cur`.  A burst
    // of global->LDS loads blocks the wavefront for as long as the texture path
    // takes to accept it (about 2000 cycles for a whole 256 x 256 stage), so the
    // loads are dealt out over the steps and the scheduler is asked to interleave:
    // one LDS read behind each MFMA, one global load every few MFMAs.
    constexpr int LPK = (LPSX + KK - 1) / KK;  // refill loads per step
    constexpr int NREAD = C::MB + 2 * C::NB, NMFMA = C::MB * C::NB;
    auto step = [&](int frag_buf, int frag_kt, int frag_kk, Frag &nxt, const Frag &cur, int fill_kt, int fill_buf, int part) {
        load_frag(frag_buf, frag_kt, frag_kk, nxt);
#pragma unroll
        for (int mb = 0; mb < C::MB; ++mb)
#pragma unroll
            for (int nb = 0; nb < C::NB; ++nb) {
                const int i = mb * C::NB + nb;
                // share j of this step's loads goes in front of MFMA number j*NMFMA/LPK
#pragma unroll
                for (int j = 0; j < LPK; ++j)
                    if ((j * NMFMA) / LPK == i && part * LPK + j < LPSX) issue_one(fill_kt, fill_buf, part * LPK + j);
                acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur.b[nb], cur.a[mb], acc[mb][nb], 0, 0, 0);
            }
#pragma unroll
        for (int i = 0; i < NMFMA; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                 // one MFMA
            if (i < NREAD) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // one LDS read
        }
        if (NREAD > NMFMA) __builtin_amdgcn_sched_group_barrier(0x100, NREAD - NMFMA, 0);
    };

    // ---- pipeline.  NS stage buffers; loads run NS-1 stages ahead of the
    // MFMAs.  A stage's buffer is free as soon as every wavefront has READ its
    // last fragments (not when the MFMAs retire), so the barrier sits before the
    // last MFMA step of the stage; the refill of that buffer (stage kt+NS) is dealt
    // out over the KK steps that follow the barrier.  Past the end of K the refill
    // re-loads the last stage into a buffer nobody reads any more: every wavefront
    // then always has the same number of loads in flight and one vmcnt value fits
    // every iteration.  Fragments are double-buffered in registers throughout.
    const int nk = K / C::BK;
    // prologue: stages 0 .. NS-2 whole, plus the first share of stage NS-1 (its other
    // shares ride on the first stage's MFMA steps like every later refill)
#pragma unroll
    for (int s = 0; s + 1 < C::NS; ++s) issue_loads(min(s, nk - 1), s);
    int fill_kt = min(C::NS - 1, nk - 1), fill_buf = C::NS - 1;
    constexpr int PART0 = LPK < LPSX ? LPK : LPSX;
#pragma unroll
    for (int i = 0; i < PART0; ++i) issue_one(fill_kt, fill_buf, i);
    // (loads the caller issues here are younger than the stage loads: if they are still in
    // flight at a vmcnt wait below, that wait only becomes stricter)
    while_loading();
    wait_vmcnt<(C::NS - 2) * LPSX + PART0>();
    __syncthreads();
    Frag f0, f1;
    load_frag(0, 0, 0, f0);
    int buf = 0;
    static_assert(KK % 2 == 0, "fragment double buffer assumes an even number of steps per stage");
    // steps 0 .. KK-2 of a stage; they also carry shares 1 .. KK-1 of the refill in progress
    auto main_steps = [&](int b, int kt) {
#pragma unroll
        for (int kk = 0; kk + 1 < KK; ++kk) {
            if (kk & 1)
                step(b, kt, kk + 1, f0, f1, fill_kt, fill_buf, kk + 1);
            else
                step(b, kt, kk + 1, f1, f0, fill_kt, fill_buf, kk + 1);
        }
    };
    // KK is even: a stage starts in f0 and its last step multiplies f1
    for (int kt = 0; kt + 1 < nk; ++kt) {
        main_steps(buf, kt);
        // last step of the stage: cross into the next stage first.  Stage kt+1 must
        // have landed; the NS-2 stages issued after it may stay in flight.
        wait_vmcnt<(C::NS - 2) * LPSX>();
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // this stage's fragments are in registers
        __syncthreads();
        const int nbuf = (buf + 1 == C::NS) ? 0 : buf + 1;
        fill_kt = min(kt + C::NS, nk - 1);
        fill_buf = buf;
        step(nbuf, kt + 1, 0, f0, f1, fill_kt, fill_buf, 0);
        buf = nbuf;
    }
    main_steps(buf, nk - 1);
    mfma_all(f1);
    wait_vmcnt<0>();  // nothing may still be landing in LDS when the C tile is written over the stage buffers
    __syncthreads();

    // ---- epilogue: fp32 accumulators -> bf16 C tile in LDS.  Lane l holds, for
    // MFMA block (mb, nb) and register group vq, output row (l & 31) and the 4
    // consecutive columns 8*vq + 4*(l >> 5) .. +3 of that block.
    const int c_row = wm * 32 * C::MB + (lane & 31);
    if (HRES) {
        // h of the row block, as the A operand of the GEMM that follows: column c of h belongs to stage c / BK
#pragma unroll
        for (int mb = 0; mb < C::MB; ++mb) {
            const int row = c_row + mb * 32;
#pragma unroll
            for (int nb = 0; nb < C::NB / 2; ++nb)
#pragma unroll
                for (int vq = 0; vq < 4; ++vq) {
                    const int col = n0 + wn * (C::BNW / 2) + nb * 32 + 8 * vq + 4 * (lane >> 5);
                    if (col < ntot) {
                        const f32x16_t &g = acc[mb][nb];
                        const f32x16_t &u = acc[mb][nb + C::NB / 2];
                        uint2 o;
                        o.x = pack_bf16x2(silu_mul(g[4 * vq], u[4 * vq]), silu_mul(g[4 * vq + 1], u[4 * vq + 1]));
                        o.y = pack_bf16x2(silu_mul(g[4 * vq + 2], u[4 * vq + 2]), silu_mul(g[4 * vq + 3], u[4 * vq + 3]));
                        const int cin = col % C::BK;
                        *(uint2 *)(res + (col / C::BK) * C::A_BYTES + row * C::A_ROW + (((cin >> 3) ^ a_swz(row)) << 4) +
                                   (cin & 7) * 2) = o;
                    }
                }
        }
        __syncthreads();
        return;
    }
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

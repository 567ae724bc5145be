// Grouped SwiGLU FFN tiles, publication of finished output tiles with ready
// flags (paper sections 2.3 and 4.1), and the weighted combine (section 2.1
// step 4).
#pragma once
#include "common.hpp"
#include "gemm_bf16.hpp"
#include "gemm_f32.hpp"

namespace moe {

// ---- GEMM policies: element type + tile shape + main loop
template <class C>
struct Bf16Policy {
    using ET = bf16_t;
    using Cfg = C;
    static constexpr bool FUSED = false;
    static constexpr int BM = C::BM, BN1 = C::BN / 2, BN2 = C::BN;
    static constexpr int C_STRIDE = C::C_STRIDE;
    static constexpr int SMEM_MAIN = C::SMEM_MAIN;
    // wavefronts per SIMD the kernel is built for: two workgroups per CU where their LDS fits
    static constexpr int MIN_WAVES = (2 * (C::SMEM_MAIN + 8 * 1024) <= 160 * 1024) ? 2 : 1;
    template <bool GATED, class RowPtr, class Hook>
    static __device__ __forceinline__ void gemm(RowPtr rp, const ET *B0, const ET *B1, int ldb, int ncols, int K,
                                                char *smem, Hook while_loading) {
        gemm_tile_bf16<C, GATED>(rp, B0, B1, ldb, ncols, K, smem, while_loading);
    }
};
struct F32Policy {
    using ET = float;
    static constexpr bool FUSED = false;
    static constexpr int BM = TileF32::BM, BN1 = TileF32::BN, BN2 = TileF32::BN;
    static constexpr int C_STRIDE = TileF32::C_STRIDE;
    static constexpr int SMEM_MAIN = TileF32::SMEM_MAIN;
    static constexpr int MIN_WAVES = 1;
    template <bool GATED, class RowPtr, class Hook>
    static __device__ __forceinline__ void gemm(RowPtr rp, const ET *B0, const ET *B1, int ldb, int ncols, int K,
                                                char *smem, Hook while_loading) {
        gemm_tile_f32<GATED>(rp, B0, B1, ldb, ncols, K, smem, while_loading);
    }
};
// The fused FFN (moe_problem_t::fuse_ffn): same main loops, other tile loop (see fused_stage)
template <class C>
struct FusedPolicy : Bf16Policy<C> {
    static constexpr bool FUSED = true;
    static constexpr int MIN_WAVES = 1;  // the row block's h takes the LDS a second workgroup would need
};
// LDS after the GEMM region: per-row slot / destination, publish row-tile list
template <class P>
constexpr int tile_smem_bytes() {
    return P::SMEM_MAIN + (3 * P::BM + 8) * 4;
}

// stage depth / count per shape: the best of the variants measured on MI355X
using CfgL = TileCfg<4, 4, 2, 2, 32, 4>;  // 256 x 256, wavefront 128 x 128
using CfgM = TileCfg<2, 4, 2, 2, 64, 3>;  // 128 x 256, wavefront  64 x 128
using CfgS = TileCfg<1, 2, 1, 4, 64, 4>;  //  32 x 256, wavefront  32 x  64, deep pipeline: weight streaming

// row blocks of the fused FFN: short enough for a block's h to stay in LDS beside three stages
using CfgFS = TileCfg<1, 2, 1, 4, 64, 3>;  // 32 x 256, wavefront 32 x 64 (decode-sized experts)
using CfgFM = TileCfg<2, 2, 1, 4, 32, 3>;  // 64 x 256, wavefront 64 x 64

constexpr int kTileGroupRows = 4, kTileGroupCols = 8;  // see decode_tile

struct TileInfo {
    int e, rb, row0, nrows, lrow0, n0, ncols;
    bool valid;
};

// The small tables a tile decode reads; they point into LDS once a workgroup has
// copied them there (after the plan), else into the workspace.
//
// Row blocks come in one height, or in two (mixed heights): big blocks of
// Tiling::BM rows, and for an expert whose last rows fit into Tiling::BMS rows
// one small block for them.  Square-ish tiles move the fewest operand bytes per
// flop, so an expert gets as many 256-row tiles as it can fill and the 128-row
// tile only for a short tail, instead of padding the tail to 256 rows or cutting
// everything to 128.
// The two kinds have separate block numbers, tables and tile code (SMALL).
struct Tables {
    const int32_t *offsets, *counts, *rb_base, *rb_expert, *rbs_base, *rbs_expert;
    int n_rb, n_rbs;
};

// The row blocks [0, n) of one kind of all experts, in expert order, are cut
// into kTileQueues contiguous shares, one per XCD, and each share has four tile
// lists: GEMM1 and GEMM2, for its big and for its small blocks.  Workgroups go
// through the four kinds in the order GEMM1 big, GEMM1 small, GEMM2 big, GEMM2
// small, and within a kind draw from the list of the XCD they run on first, then
// from the others.  Tiles that read the same weights or the same rows therefore
// meet in one L2 instead of fetching the operand once per XCD, and by the time
// anybody draws a GEMM2 tile every GEMM1 tile has been drawn.
struct TileQueue {
    int r0, r1;   // big row blocks of this share
    int s0, s1;   // small row blocks of this share
    int n1b, n1s; // GEMM1 tiles, big / small
    int n2b, n2s; // GEMM2 tiles, big / small
    __device__ __forceinline__ int n1() const { return n1b + n1s; }
    __device__ __forceinline__ int total() const { return n1b + n1s + n2b + n2s; }
};
__device__ __forceinline__ TileQueue tile_queue(const KArgs &a, int n_rb, int n_rbs, int q) {
    TileQueue tq;
    tq.r0 = (int)(((long long)n_rb * q) / kTileQueues);
    tq.r1 = (int)(((long long)n_rb * (q + 1)) / kTileQueues);
    tq.s0 = (int)(((long long)n_rbs * q) / kTileQueues);
    tq.s1 = (int)(((long long)n_rbs * (q + 1)) / kTileQueues);
    tq.n1b = (tq.r1 - tq.r0) * a.tl.NT1;
    tq.n1s = (tq.s1 - tq.s0) * a.tl.NT1;
    tq.n2b = (tq.r1 - tq.r0) * a.tl.NT2;
    tq.n2s = (tq.s1 - tq.s0) * a.tl.NT2;
    return tq;
}

// Entry i of one phase and kind of a queue -> tile.  Inside the share, the tiles
// of one expert are consecutive, in an order that lets tiles running at the same
// time share weight column blocks and rows in the XCD's L2 (see below).
// ti.rb numbers big blocks from 0 and small blocks from n_rb (index into h_ready).
template <bool SMALL>
__device__ __forceinline__ TileInfo decode_tile(const KArgs &a, const Tables &tb, const TileQueue &tq, int i, int NT,
                                                int BN, int total_cols) {
    TileInfo ti;
    const int32_t *base = SMALL ? tb.rbs_base : tb.rb_base;
    const int q0 = SMALL ? tq.s0 : tq.r0, q1 = SMALL ? tq.s1 : tq.r1;
    const int BMK = SMALL ? a.tl.BMS : a.tl.BM;
    const int e = (SMALL ? tb.rbs_expert : tb.rb_expert)[q0 + i / NT];
    const int e_rb0 = base[e];
    const int s0 = max(e_rb0, q0), s1 = min(base[e + 1], q1);  // the expert's row blocks of this kind in this share
    const int nrb = s1 - s0;
    const int loc = i - (s0 - q0) * NT;
    // The expert's tiles (nrb row blocks x NT column tiles) are listed in blocks of GR row blocks x
    // GC column tiles, column tile slowest inside a block: the 32 workgroups of an XCD then work on
    // 4 + 8 different operand panels at a time.  (All row blocks of one column tile side by side, 16 + 2
    // panels when an expert has 16 row blocks, made the L2 fetch 28 GB per cfg4 launch.)
    constexpr int GR = kTileGroupRows, GC = kTileGroupCols;
    const int rg = min(loc / (GR * NT), (nrb - 1) / GR);
    const int l2 = loc - rg * GR * NT;
    const int rows_g = min(GR, nrb - rg * GR);
    const int cg = l2 / (rows_g * GC);
    const int l3 = l2 - cg * rows_g * GC;
    const int ct = cg * GC + l3 / rows_g, rbl = rg * GR + l3 % rows_g;
    const int rb = s0 + rbl;
    ti.e = e;
    ti.rb = SMALL ? tb.n_rb + rb : rb;
    // the small block follows the expert's big blocks
    ti.lrow0 = SMALL ? (tb.rb_base[e + 1] - tb.rb_base[e]) * a.tl.BM : (rb - e_rb0) * BMK;
    ti.row0 = tb.offsets[e] + ti.lrow0;
    ti.nrows = min(BMK, tb.counts[e] - ti.lrow0);  // (an expert's rows end at counts[e], not at the next expert's first row)
    ti.n0 = ct * BN;
    ti.ncols = min(BN, total_cols - ti.n0);
    ti.valid = true;
    return ti;
}

// The tile (row block rb of its kind, column tile ct): how the ready-queue scheduler names a
// GEMM2 tile.
template <bool SMALL>
__device__ __forceinline__ TileInfo decode_block_tile(const KArgs &a, const Tables &tb, int rb, int ct, int BN,
                                                      int total_cols) {
    TileInfo ti;
    const int BMK = SMALL ? a.tl.BMS : a.tl.BM;
    const int e = (SMALL ? tb.rbs_expert : tb.rb_expert)[rb];
    ti.e = e;
    ti.rb = SMALL ? tb.n_rb + rb : rb;
    ti.lrow0 = SMALL ? (tb.rb_base[e + 1] - tb.rb_base[e]) * a.tl.BM : (rb - tb.rb_base[e]) * BMK;
    ti.row0 = tb.offsets[e] + ti.lrow0;
    ti.nrows = min(BMK, tb.counts[e] - ti.lrow0);  // (an expert's rows end at counts[e], not at the next expert's first row)
    ti.n0 = ct * BN;
    ti.ncols = min(BN, total_cols - ti.n0);
    ti.valid = true;
    return ti;
}

// ---- ready queues (MOE_SCHED_READY_QUEUE).  One queue per XCD.  Every task that goes through
// a queue has a fixed one: the GEMM2 tiles of a row block go to the queue of the XCD whose share
// (see TileQueue) the block is in, the combine tasks of destination r to queue r mod 8; so the
// number of entries each queue will receive is known once the plan is.  A queue is an array of
// entries that starts all zero, a tail counter with which producers reserve entries, and a head
// counter from which consumers draw tickets: ticket t is the right, and the duty, to run entry t
// of that queue, whenever it gets written.  A consumer empties the entry it ran, so the array is
// all zero again after the call.  An entry is 1 + (row block * NT2 + column tile) for a GEMM2 tile
// (row blocks numbered as in h_ready) or kReadyCombine | task for a combine task.
constexpr u32 kReadyCombine = 0x80000000u;
// entries queue q receives in this call
__device__ __forceinline__ int ready_queue_size(const KArgs &a, int n_rb, int n_rbs, int q) {
    const TileQueue tq = tile_queue(a, n_rb, n_rbs, q);
    const int dests = a.R > q ? (a.R - q + kTileQueues - 1) / kTileQueues : 0;
    return tq.n2b + tq.n2s + dests * (a.per_dest / a.comb_tokens);
}
// the share that row block rb of n (of one kind) lies in
__device__ __forceinline__ int ready_queue_of_block(int n, int rb) {
    int q = 0;
    while (q + 1 < kTileQueues && rb >= (int)(((long long)n * (q + 1)) / kTileQueues)) ++q;
    return q;
}
// `n` consecutive entries first, first + 1, ... to queue q, by all lanes of one wavefront
__device__ __forceinline__ void ready_push(const KArgs &a, int q, u32 first, int n, int lane) {
    u32 base = 0;
    if (lane == 0) base = atomicAdd(&a.ctrl->rq_tail[q], (u32)n);
    base = (u32)__builtin_amdgcn_readfirstlane((int)base);
    u32 *slots = a.rq_slots + (size_t)q * a.rq_cap;
    for (int i = lane; i < n; i += 64)
        if (base + i < (u32)a.rq_cap) st_relaxed(&slots[base + i], first + (u32)i, 0);
}
// Wavefront-wide: `n` more flags of destination dst carry the epoch.  Whoever reports the
// last ones enqueues the combine tasks of the destination's tokens (the host makes combine
// tasks lie inside one destination for this scheduler).  The consumer still checks the
// flags itself before it reads a row, so no ordering beyond the counter is needed here.
__device__ __forceinline__ void ready_flags_stored(const KArgs &a, int dst, int n, int lane) {
    u32 old = 0;
    if (lane == 0) old = atomicAdd(&a.dest_done[dst], (u32)n);
    old = (u32)__builtin_amdgcn_readfirstlane((int)old);
    const u32 all = (u32)(a.dest_flag_begin[dst + 1] - a.dest_flag_begin[dst]);
    if (old + (u32)n == all) {
        const int per = a.per_dest / a.comb_tokens;
        ready_push(a, dst % kTileQueues, kReadyCombine | (u32)(dst * per), per, lane);
    }
}

// Every pointer of the argument block, marked as pointing to global memory
// (see as_global).
__device__ __forceinline__ void mark_global(KArgs &a) {
    a.x = as_global((const char *)a.x);
    a.Wg = as_global((const char *)a.Wg);
    a.bias = as_global(a.bias);
    a.W1 = as_global((const char *)a.W1);
    a.W3 = as_global((const char *)a.W3);
    a.W2 = as_global((const char *)a.W2);
    a.idx = as_global(a.idx);
    a.w = as_global(a.w);
    a.counts = as_global(a.counts);
    a.offsets = as_global(a.offsets);
    a.perm = as_global(a.perm);
    a.inv_perm = as_global(a.inv_perm);
    a.slot_flag = as_global(a.slot_flag);
    a.staging = as_global((char *)a.staging);
    a.flags = as_global(a.flags);
    a.out = as_global((char *)a.out);
    a.ctrl = as_global(a.ctrl);
    a.blk_hist = as_global(a.blk_hist);
    a.blk_base = as_global(a.blk_base);
    a.seg_cnt = as_global(a.seg_cnt);
    a.seg_begin = as_global(a.seg_begin);
    a.flag_base = as_global(a.flag_base);
    a.dest_flag_begin = as_global(a.dest_flag_begin);
    a.dest_group_begin = as_global(a.dest_group_begin);
    a.group_counter = as_global(a.group_counter);
    a.rb_base = as_global(a.rb_base);
    a.rb_expert = as_global(a.rb_expert);
    a.rbs_base = as_global(a.rbs_base);
    a.rbs_expert = as_global(a.rbs_expert);
    a.h_ready = as_global(a.h_ready);
    a.h = as_global((char *)a.h);
    a.dest_done = as_global(a.dest_done);
    a.rq_slots = as_global(a.rq_slots);
}

// The decode tables: the copies a workgroup made in LDS after the plan (see the
// megakernel), else the workspace arrays.
__device__ __forceinline__ Tables decode_tables(const KArgs &a, char *smem, int n_rb, int n_rbs) {
    Tables tb;
    tb.n_rb = n_rb;
    tb.n_rbs = n_rbs;
    if (a.tab_lds_off > 0) {  // layout: see the copy in the megakernel
        tb.offsets = (const int32_t *)(smem + a.tab_lds_off);
        tb.rb_base = tb.offsets + a.E + 1;
        tb.rbs_base = tb.rb_base + a.E + 1;
        tb.counts = tb.rbs_base + a.E + 1;
        tb.rb_expert = tb.counts + a.E + 1;
        tb.rbs_expert = tb.rb_expert + n_rb;
    } else {
        tb.offsets = a.offsets;
        tb.counts = a.counts;
        tb.rb_base = a.rb_base;
        tb.rb_expert = a.rb_expert;
        tb.rbs_base = a.rbs_base;
        tb.rbs_expert = a.rbs_expert;
    }
    return tb;
}

// GEMM1 + SwiGLU: h[rows of the block, n0 .. n0+ncols) = silu(x W1[e]) * (x W3[e]).
// Rows are gathered straight from x through perm: the permuted activations are
// never materialised.
// `after_gemm()` runs between the main loop and the write-out (the megakernel draws
// its next tile there, so that the counter's latency hides behind the write-out).
// Returns, in thread 0, how many GEMM1 tiles of the row block had finished before this one.
template <class P, class Hook>
__device__ __forceinline__ u32 g1_tile(const KArgs &a, const TileInfo &ti, char *smem, Hook after_gemm) {
    using ET = typename P::ET;
    const ET *x = (const ET *)a.x;
    const int N = a.N;
    auto rowptr = [&](int r) {
        int s = a.perm[ti.row0 + min(r, ti.nrows - 1)];
        s = min(max(s, 0), N - 1);
        return x + (size_t)(s / a.k) * a.d;
    };
    const size_t wofs = (size_t)ti.e * a.d * a.f + ti.n0;
    MOE_TT_BEGIN();
    P::template gemm<true>(rowptr, (const ET *)a.W1 + wofs, (const ET *)a.W3 + wofs, a.f, ti.ncols, a.d, smem, [] {});
    after_gemm();
    MOE_TT(a.ctrl, 1);
    const int ppr = ti.ncols * (int)sizeof(ET) / 16;
    char *h = (char *)a.h;
    for (int q = threadIdx.x; q < ti.nrows * ppr; q += kThreads) {
        const int r = q / ppr, c = q % ppr;
        store_tile16(h + ((size_t)(ti.row0 + r) * a.f + ti.n0) * sizeof(ET) + c * 16,
                     *(const uint4 *)(smem + r * P::C_STRIDE + c * 16));
    }
    sync_stores();
    MOE_TT(a.ctrl, 2);
    u32 before = 0;
    if (threadIdx.x == 0) {
        fence_release(0);
        before = atomicAdd(&a.h_ready[ti.rb], 1u);
        atomicAdd(&a.ctrl->stats[4], 1ull);
    }
    MOE_TT(a.ctrl, 3);
    return before;
}

// Publish the y tile sitting in the LDS C tile.  A publish tile is the part of
// the compute tile that lies in one (row block of tile_m rows, destination,
// column block of tile_n columns); each has its own ready flag.
//   PER_TILE: for every publish tile in turn: write it, barrier, release fence, flag
//             (the coupled PUT -> FENCE -> SIGNAL of section 2.3).
//   PER_DEST: write the whole compute tile, one release so the rows may be counted,
//             add the publish tiles to the counter of their fence group (Algorithm 1,
//             phase 1; a group is all flags of a destination, or group_size consecutive
//             ones: the granularity knob of section 4.1).  Whoever completes a group's
//             count is its leader: one fence at the requested scope, then all flags of
//             the group, stored by a whole wavefront (phase 2; lane-parallel signals as
//             in appendix B).
// Row bookkeeping of a publish: slot and destination of every row of the compute
// tile and the list of publish row-tiles, into LDS behind the GEMM's region (so it
// can run while the GEMM's first loads are in flight).
template <class P>
__device__ __forceinline__ void publish_prepare(const KArgs &a, const TileInfo &ti, char *smem) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int *s_slot = (int *)(smem + P::SMEM_MAIN);  // [BM] slot (= staging row) of local row r
    int *s_dest = s_slot + P::BM;                // [BM] destination of local row r
    int *s_seg = s_dest + P::BM;                 // [BM+1] first local row of publish row-tile i
    int *s_nseg = s_seg + P::BM + 1;
    const int N = a.N;
    MOE_TT_BEGIN();
    for (int r = tid; r < ti.nrows; r += kThreads) {
        int s = a.perm[ti.row0 + r];
        s = min(max(s, 0), N - 1);
        s_slot[r] = s;
        s_dest[r] = (s / a.k) / a.per_dest;
    }
    __syncthreads();
    if (wave == 0) {
        int cnt = 0;
        for (int base = 0; base < ti.nrows; base += 64) {
            const int r = base + lane;
            const bool st = r < ti.nrows && (r == 0 || ((ti.lrow0 + r) % a.tile_m) == 0 || s_dest[r] != s_dest[r - 1]);
            const u64 m = __ballot(st);
            if (st) s_seg[cnt + __popcll(m & ((1ull << lane) - 1ull))] = r;
            cnt += __popcll(m);
        }
        if (lane == 0) {
            s_seg[cnt] = ti.nrows;
            *s_nseg = cnt;
        }
    }
    __syncthreads();
    MOE_TT(a.ctrl, 11);
}

template <class P>
__device__ void publish_tile(const KArgs &a, const TileInfo &ti, char *smem) {
    using ET = typename P::ET;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int *s_slot = (const int *)(smem + P::SMEM_MAIN);  // filled by publish_prepare
    const int *s_dest = s_slot + P::BM;
    const int *s_seg = s_dest + P::BM;
    const int *s_nseg = s_seg + P::BM + 1;
    MOE_TT_BEGIN();
    const int nseg = *s_nseg;
    const int cbn = (ti.ncols + a.tile_n - 1) / a.tile_n;  // column blocks in this compute tile
    const int cb0 = ti.n0 / a.tile_n;
    const int ES = (int)sizeof(ET);
    char *staging = (char *)a.staging;
    const int sys = a.fence_scope;

    auto copy_rows = [&](int r0, int r1, int p0, int p1) {  // 16-byte pieces [p0, p1) of rows [r0, r1)
        const int w = p1 - p0;
        for (int q = tid; q < (r1 - r0) * w; q += kThreads) {
            const int r = r0 + q / w, c = p0 + q % w;
            store_tile16(staging + ((size_t)s_slot[r] * a.d + ti.n0) * ES + c * 16,
                         *(const uint4 *)(smem + r * P::C_STRIDE + c * 16));
        }
    };

    if (a.signal_mode == MOE_SIGNAL_PER_TILE) {
        for (int i = 0; i < nseg; ++i) {
            const int r0 = s_seg[i], r1 = s_seg[i + 1];
            for (int j = 0; j < cbn; ++j) {
                const int p0 = j * a.tile_n * ES / 16;
                const int p1 = min((j + 1) * a.tile_n, ti.ncols) * ES / 16;
                copy_rows(r0, r1, p0, p1);
                sync_stores();
                if (tid == 0) {
                    fence_release(sys);
                    st_relaxed(&a.flags[a.slot_flag[s_slot[r0]] + cb0 + j], a.epoch, sys);
                }
            }
        }
        if (tid == 0) {
            const u64 n = (u64)nseg * cbn;
            atomicAdd(&a.ctrl->stats[0], n);
            atomicAdd(&a.ctrl->stats[1], n);
            atomicAdd(&a.ctrl->stats[2], n);
        }
        // (the flags were stored by lane 0 of this wavefront)
        if (a.dest_done && wave == 0)
            for (int i = 0; i < nseg; ++i) ready_flags_stored(a, s_dest[s_seg[i]], cbn, lane);
    } else {
        copy_rows(0, ti.nrows, 0, ti.ncols * ES / 16);
        sync_stores();
        MOE_TT(a.ctrl, 12);
        if (wave == 0) {
            fence_release(0);  // the rows of this tile may now be counted
            u64 n_fence = 0, n_flag = 0;
            for (int base = 0; base < nseg; base += 64) {
                // lane i: the cbn flags [f0, f0 + cbn) of publish row-tile i; they lie in one
                // destination and in one or more of its fence groups
                const int i = base + lane;
                const bool active = i < nseg;
                int f0 = 0, fb = 0, fe = 0, gs = 1, g_first = 0, g_last = -1, gid0 = 0, dst = 0;
                if (active) {
                    const int r0 = s_seg[i];
                    dst = s_dest[r0];
                    fb = a.dest_flag_begin[dst];
                    fe = a.dest_flag_begin[dst + 1];
                    f0 = a.slot_flag[s_slot[r0]] + cb0;
                    gs = a.group_size > 0 ? a.group_size : fe - fb;
                    g_first = (f0 - fb) / gs;
                    g_last = (f0 + cbn - 1 - fb) / gs;
                    gid0 = a.dest_group_begin[dst];
                }
                for (int j = 0;; ++j) {
                    const bool has = active && g_first + j <= g_last;
                    if (__ballot(has) == 0ull) break;
                    bool lead = false;
                    const int gl = g_first + j;
                    const int gbeg = fb + gl * gs, gend = min(gbeg + gs, fe);
                    const int gid = gid0 + gl;
                    if (has) {
                        const u32 cnt = (u32)(min(f0 + cbn, gend) - max(f0, gbeg));
                        const u32 old = atomicAdd(&a.group_counter[gid], cnt);
                        lead = (old + cnt == (u32)(gend - gbeg));
                    }
                    u64 m = __ballot(lead);
                    while (m) {
                        const int src = __ffsll((long long)m) - 1;
                        m &= m - 1;
                        const int gb = __shfl(gbeg, src, 64), ge = __shfl(gend, src, 64), gi = __shfl(gid, src, 64);
                        // every tile counted for this group was released (device scope) by its
                        // writer before it was counted
                        fence_acquire(0);
                        fence_release(sys);  // the one fence of this group
                        for (int fi = gb + lane; fi < ge; fi += 64) st_relaxed(&a.flags[fi], a.epoch, sys);
                        if (lane == 0)
                            __hip_atomic_store(&a.group_counter[gi], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        n_fence += 1;
                        n_flag += (u64)(ge - gb);
                        if (a.dest_done) ready_flags_stored(a, __shfl(dst, src, 64), ge - gb, lane);
                    }
                }
            }
            if (lane == 0) {
                if (n_fence) {
                    atomicAdd(&a.ctrl->stats[0], n_fence);
                    atomicAdd(&a.ctrl->stats[1], n_flag);
                }
                atomicAdd(&a.ctrl->stats[2], (u64)nseg * cbn);
                atomicAdd(&a.ctrl->stats[3], 1ull);
            }
        }
    }
    __syncthreads();
    MOE_TT(a.ctrl, 13);
}

// GEMM2 + publish: y[rows of the block, n0 .. n0+ncols) = h W2[e], written to
// staging row perm[p] (the slot that asked for it).  The caller has already
// waited for the block's h rows.
template <class P, class Hook>
__device__ __forceinline__ void g2_tile(const KArgs &a, const TileInfo &ti, char *smem, Hook after_gemm) {
    using ET = typename P::ET;
    const ET *h = (const ET *)a.h;
    auto rowptr = [&](int r) { return h + (size_t)(ti.row0 + min(r, ti.nrows - 1)) * a.f; };
    const ET *B0 = (const ET *)a.W2 + (size_t)ti.e * a.f * a.d + ti.n0;
    MOE_TT_BEGIN();
    P::template gemm<false>(rowptr, B0, B0, a.d, ti.ncols, a.f, smem, [&] { publish_prepare<P>(a, ti, smem); });
    after_gemm();
    MOE_TT(a.ctrl, 7);
    publish_tile<P>(a, ti, smem);
    MOE_TT(a.ctrl, 8);
    if (threadIdx.x == 0) atomicAdd(&a.ctrl->stats[5], 1ull);
}

// ---- the stages of the megakernel
// The megakernel is a sequence of stages, each of which draws work from a
// counter of the control block until there is none left for it.  The two GEMM
// stages are real calls (not inlined), so that each GEMM main loop gets a
// register allocation of its own whatever else the kernel contains; a stage
// loops over its tiles inside the call, which keeps the cost of a call (saving
// and restoring registers through scratch memory) out of the tile loop.  They
// take the argument block by address and read it with scalar loads (a
// reference to the kernel's own copy would force that copy into per-lane
// scratch memory, for every stage), and LDS as an offset.  Everything else is
// inlined into the kernel, so that the kernel's launch bounds govern it.
struct StageLds {  // broadcast slots of a stage's task loop, in dynamic LDS at KArgs::sched_lds_off
    int next, ok;
    int pick;  // tile stage: the list to draw from next, -1 = all lists are empty
    int q, hops, ticket, g1_left;  // ready-queue scheduler: the workgroup's state (see ready_queue_stage)
};

// One kind of tile (GEMM1 if GATED, else GEMM2; big or SMALL row blocks) from the eight tile
// queues, the one of XCD `home` first, until none is left; or, when one_a >= 0, exactly one
// tile that the caller has taken already: entry one_b of list one_a (GEMM1), or row block
// one_a of this kind, column tile one_b (GEMM2, whose rows of h are known to be complete).
// In that case, if ticket_q >= 0, a ticket of ready queue ticket_q is drawn where the list
// mode draws its next tile, and left in StageLds::next (0x7fffffff: none drawn).
template <class P, bool GATED, bool SMALL>
static __device__ __attribute__((noinline)) void tile_stage(KArgsAddr args, u32 smem_off, int home, int n_rb, int n_rbs,
                                                           int one_a, int one_b, int ticket_q,
                                                           volatile int *caller_local) {
    KArgs a = load_kernel_args(args);
    mark_global(a);
    char *smem = lds_at((u32)uniform((int)smem_off));
    home = uniform(home), n_rb = uniform(n_rb), n_rbs = uniform(n_rbs);
    one_a = uniform(one_a), one_b = uniform(one_b), ticket_q = uniform(ticket_q);
    const bool single = one_a >= 0;
    const int tid = threadIdx.x;
    Ctrl *c = a.ctrl;
    StageLds *sl = (StageLds *)(smem + a.sched_lds_off);
    const Tables tb = decode_tables(a, smem, n_rb, n_rbs);
    const u64 t0 = kernel_start_ticks(c);
    constexpr int LIST = (GATED ? 0 : 2) + (SMALL ? 1 : 0);
    *caller_local = LIST;  // (see the call sites)
    bool more = true;
    while (more) {
        int q, n, i;
        u32 *counter;
        if (single) {
            more = false;
            q = GATED ? one_a : 0;
            i = GATED ? one_b : 0;
            n = i + 1;
            counter = &c->rq_head[ticket_q >= 0 ? ticket_q : 0];
        } else {
            // one look at the eight counters of this kind picks the first list, from this XCD's on, that
            // still has entries (a draw from an empty list costs a trip to memory and two barriers)
            __syncthreads();
            if (tid < 64) {
                bool has = false;
                if (tid < kTileQueues) {
                    const int qq = (home + tid) % kTileQueues;
                    const TileQueue t2 = tile_queue(a, n_rb, n_rbs, qq);
                    const int n2 = GATED ? (SMALL ? t2.n1s : t2.n1b) : (SMALL ? t2.n2s : t2.n2b);
                    has = ld_relaxed_agent(&c->tile_next[LIST][qq]) < (u32)n2;
                }
                const u64 m = __ballot(has);
                if (tid == 0) sl->pick = m ? (home + __ffsll((long long)m) - 1) % kTileQueues : -1;
            }
            __syncthreads();
            q = uniform(sl->pick);
            if (q < 0) break;
            const TileQueue tq0 = tile_queue(a, n_rb, n_rbs, q);
            n = GATED ? (SMALL ? tq0.n1s : tq0.n1b) : (SMALL ? tq0.n2s : tq0.n2b);
            counter = &c->tile_next[LIST][q];
            __syncthreads();
            if (tid == 0) sl->next = (int)atomicAdd(counter, 1u);
            __syncthreads();
            i = uniform(sl->next);
        }
        const TileQueue tq = tile_queue(a, n_rb, n_rbs, q);
        while (i < n) {
            // the next entry is drawn after this tile's main loop and consumed at the end of the tile
            u32 next = 0x7fffffffu;
            auto draw = [&]() {
                if ((!single || ticket_q >= 0) && tid == 0) next = atomicAdd(counter, 1u);
            };
            MOE_TT_BEGIN();
            if (GATED) {
                const TileInfo ti = decode_tile<SMALL>(a, tb, tq, i, a.tl.NT1, P::BN1, a.f);
                MOE_TT(c, 0);
                const u32 before = g1_tile<P>(a, ti, smem, draw);
                // ready-queue scheduler: the last GEMM1 tile of a row block enqueues the block's GEMM2
                // tiles (every writer of the block released its rows before it was counted)
                if (a.rq_slots && tid == 0 && before + 1 == (u32)a.tl.NT1) {
                    const int rq = SMALL ? ready_queue_of_block(n_rbs, ti.rb - n_rb) : ready_queue_of_block(n_rb, ti.rb);
                    const u32 base = atomicAdd(&c->rq_tail[rq], (u32)a.tl.NT2);
                    u32 *slots = a.rq_slots + (size_t)rq * a.rq_cap;
                    for (int j = 0; j < a.tl.NT2; ++j)
                        if (base + j < (u32)a.rq_cap) st_relaxed(&slots[base + j], 1u + (u32)ti.rb * a.tl.NT2 + j, 0);
                }
                MOE_TT(c, 4);
            } else {
                const TileInfo ti = single ? decode_block_tile<SMALL>(a, tb, one_a, one_b, P::BN2, a.d)
                                           : decode_tile<SMALL>(a, tb, tq, i, a.tl.NT2, P::BN2, a.d);
                // h rows were released (agent scope) by their GEMM1 tiles before those counted themselves
                if (tid == 0) sl->ok = (single || wait_ge(c, &a.h_ready[ti.rb], (u32)a.tl.NT1, a.wait_ticks)) ? 1 : 0;
                if (single) fence_acquire(0);
                __syncthreads();
                MOE_TT(c, 5);
                if (sl->ok)
                    g2_tile<P>(a, ti, smem, draw);
                else
                    draw();
                MOE_TT(c, 9);
            }
            __syncthreads();
            if (tid == 0) {
                mark_phase_end(c, GATED ? 3 : 4, t0);
                sl->next = (int)next;
            }
            __syncthreads();
            i = uniform(sl->next);
            MOE_TT(c, 10);
#ifdef MOE_TILE_TIMING
            if (tid == 0) atomicMax(&c->dbg[24 + q], now_ticks() - c->t0);
#endif
        }
    }
}

// ---- the fused FFN (moe_problem_t::fuse_ffn; paper section 2.3: a tile traverses dispatch -> GEMM -> activation ->
// GEMM).  A workgroup takes one row block of an expert (32 or 64 rows) through the whole FFN: every column tile of
// GEMM1 + SwiGLU writes its piece of h into an LDS buffer laid out like staged A tiles, a barrier, then every column
// tile of GEMM2 reads A from that buffer and streams only W2; each y tile is published as usual.  h never leaves
// the CU and no workgroup waits for another between the two GEMMs; the price is that every row block streams its
// expert's W1, W3 and W2 by itself (row blocks of one expert are neighbours in an XCD's list, so the L2 serves the
// repeats), on matrix-core tiles of 32 or 64 rows.  Row blocks come from the same per-XCD lists as the tiles of the
// unfused path (list 0, one entry per row block).
template <class P>
__device__ __forceinline__ void fused_block(const KArgs &a, const TileInfo &rb, char *smem) {
    using C = typename P::Cfg;
    using ET = typename P::ET;
    char *hres = smem + a.fused_h_off;
    const ET *x = (const ET *)a.x;
    const int N = a.N;
    auto xrow = [&](int r) {
        int s = a.perm[rb.row0 + min(r, rb.nrows - 1)];
        s = min(max(s, 0), N - 1);
        return x + (size_t)(s / a.k) * a.d;
    };
    for (int ct = 0; ct < a.tl.NT1; ++ct) {
        const int n0 = ct * P::BN1, ncols = min(P::BN1, a.f - n0);
        const size_t wofs = (size_t)rb.e * a.d * a.f + n0;
        gemm_tile_bf16<C, true, true, false>(xrow, (const ET *)a.W1 + wofs, (const ET *)a.W3 + wofs, a.f, ncols, a.d, smem,
                                             [] {}, hres, n0, a.f);
        if (threadIdx.x == 0) atomicAdd(&a.ctrl->stats[4], 1ull);
    }
    // (the last tile's epilogue ended with a barrier: h is complete for every wavefront)
    TileInfo ti = rb;
    publish_prepare<P>(a, ti, smem);
    for (int ct = 0; ct < a.tl.NT2; ++ct) {
        ti.n0 = ct * P::BN2;
        ti.ncols = min(P::BN2, a.d - ti.n0);
        const ET *B0 = (const ET *)a.W2 + (size_t)rb.e * a.f * a.d + ti.n0;
        gemm_tile_bf16<C, false, false, true>([](int) { return (const ET *)nullptr; }, B0, B0, a.d, ti.ncols, a.f, smem, [] {},
                                              hres, 0, 0);
        publish_tile<P>(a, ti, smem);
        if (threadIdx.x == 0) atomicAdd(&a.ctrl->stats[5], 1ull);
    }
}

template <class P>
static __device__ __attribute__((noinline)) void fused_stage(KArgsAddr args, u32 smem_off, int home, int n_rb,
                                                            volatile int *caller_local) {
    KArgs a = load_kernel_args(args);
    mark_global(a);
    char *smem = lds_at((u32)uniform((int)smem_off));
    home = uniform(home), n_rb = uniform(n_rb);
    const int tid = threadIdx.x;
    Ctrl *c = a.ctrl;
    StageLds *sl = (StageLds *)(smem + a.sched_lds_off);
    const Tables tb = decode_tables(a, smem, n_rb, 0);
    const u64 t0 = kernel_start_ticks(c);
    *caller_local = 4;  // (see the call sites of tile_stage)
    while (true) {
        // the first list, from this XCD's on, that still has row blocks
        __syncthreads();
        if (tid < 64) {
            bool has = false;
            if (tid < kTileQueues) {
                const int qq = (home + tid) % kTileQueues;
                const TileQueue t2 = tile_queue(a, n_rb, 0, qq);
                has = ld_relaxed_agent(&c->tile_next[0][qq]) < (u32)(t2.r1 - t2.r0);
            }
            const u64 m = __ballot(has);
            if (tid == 0) sl->pick = m ? (home + __ffsll((long long)m) - 1) % kTileQueues : -1;
        }
        __syncthreads();
        const int q = uniform(sl->pick);
        if (q < 0) break;
        const TileQueue tq = tile_queue(a, n_rb, 0, q);
        const int n = tq.r1 - tq.r0;
        if (tid == 0) sl->next = (int)atomicAdd(&c->tile_next[0][q], 1u);
        __syncthreads();
        int i = uniform(sl->next);
        while (i < n) {
            u32 next = 0;
            if (tid == 0) next = atomicAdd(&c->tile_next[0][q], 1u);  // consumed at the end of the block
            TileInfo rb;
            rb.rb = tq.r0 + i;
            rb.e = tb.rb_expert[rb.rb];
            rb.lrow0 = (rb.rb - tb.rb_base[rb.e]) * a.tl.BM;
            rb.row0 = tb.offsets[rb.e] + rb.lrow0;
            rb.nrows = min(a.tl.BM, tb.counts[rb.e] - rb.lrow0);
            rb.n0 = 0, rb.ncols = 0, rb.valid = true;
            fused_block<P>(a, rb, smem);
            __syncthreads();
            if (tid == 0) {
                mark_phase_end(c, 3, t0);
                mark_phase_end(c, 4, t0);
                sl->next = (int)next;
            }
            __syncthreads();
            i = uniform(sl->next);
        }
    }
}

// ---- combine
template <typename ET>
struct Vec16;
template <>
struct Vec16<bf16_t> {
    static constexpr int N = 8;
    static __device__ __forceinline__ void unpack(const uint4 &v, float *f) {
        f[0] = __uint_as_float(v.x << 16);
        f[1] = __uint_as_float(v.x & 0xffff0000u);
        f[2] = __uint_as_float(v.y << 16);
        f[3] = __uint_as_float(v.y & 0xffff0000u);
        f[4] = __uint_as_float(v.z << 16);
        f[5] = __uint_as_float(v.z & 0xffff0000u);
        f[6] = __uint_as_float(v.w << 16);
        f[7] = __uint_as_float(v.w & 0xffff0000u);
    }
    static __device__ __forceinline__ void store(char *p, const float *f) {
        uint4 o;
        o.x = pack_bf16x2(f[0], f[1]);
        o.y = pack_bf16x2(f[2], f[3]);
        o.z = pack_bf16x2(f[4], f[5]);
        o.w = pack_bf16x2(f[6], f[7]);
        *(uint4 *)p = o;
    }
};
template <>
struct Vec16<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void unpack(const uint4 &v, float *f) {
        f[0] = __uint_as_float(v.x);
        f[1] = __uint_as_float(v.y);
        f[2] = __uint_as_float(v.z);
        f[3] = __uint_as_float(v.w);
    }
    static __device__ __forceinline__ void store(char *p, const float *f) {
        *(float4 *)p = make_float4(f[0], f[1], f[2], f[3]);
    }
};

// One token by one wavefront: out_row = sum_j wt[j] * rows[j], fp32 accumulation in
// slot order, one rounding.  Each lane handles U 16-byte pieces of the row at a
// time and loads 8/U slots of each before it accumulates them.  STREAM: the rows are read with
// non-temporal loads (for inputs larger than the last-level cache, which would only churn it).
template <typename ET, int U, bool STREAM>
__device__ __forceinline__ void combine_token(const char *rows, const float *wt, char *out_row, int k, int pieces,
                                              size_t rstride, int lane) {
    using V = Vec16<ET>;
    constexpr int KB = 8 / U;
    for (int c0 = lane; c0 < pieces; c0 += 64 * U) {
        float acc[U][V::N];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int i = 0; i < V::N; ++i) acc[u][i] = 0.f;
        for (int j0 = 0; j0 < k; j0 += KB) {
            uint4 v[U][KB];
#pragma unroll
            for (int jj = 0; jj < KB; ++jj)
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int c = c0 + 64 * u;
                    if (j0 + jj < k && c < pieces) {
                        const char *src = rows + (size_t)(j0 + jj) * rstride + (size_t)c * 16;
                        if (STREAM) {
                            const u32x4_t t4 = __builtin_nontemporal_load((const u32x4_t *)src);
                            v[u][jj] = make_uint4(t4[0], t4[1], t4[2], t4[3]);
                        } else {
                            v[u][jj] = *(const uint4 *)src;
                        }
                    }
                }
#pragma unroll
            for (int jj = 0; jj < KB; ++jj) {
                if (j0 + jj < k) {
                    const float wj = wt[j0 + jj];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        if (c0 + 64 * u < pieces) {
                            float f[V::N];
                            V::unpack(v[u][jj], f);
#pragma unroll
                            for (int i = 0; i < V::N; ++i) acc[u][i] = fmaf(wj, f[i], acc[u][i]);
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = c0 + 64 * u;
            if (c < pieces) V::store(out_row + (size_t)c * 16, acc[u]);
        }
    }
}

// out[t] = sum_j w[t,j] * staging[t*k+j] for the tokens of one task.  WAIT:
// spin (bounded) until the flags covering the task's rows carry this call's
// epoch; otherwise check once and report.  Flags are read with relaxed atomic
// loads (a first pass that keeps many loads in flight, then a spin on whatever
// was not ready) followed by one acquire fence at the requested scope.  Then
// one wavefront per token, 16-byte pieces, up to eight rows in flight per lane.
template <typename ET, bool WAIT, bool STREAM = false>
__device__ __forceinline__ void combine_task(const KArgs &a, int task) {
    using V = Vec16<ET>;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int k = a.k, sys = a.fence_scope;
    const char *staging = (const char *)a.staging;
    const int pieces = a.d * (int)sizeof(ET) / 16;
    const int t_first = task * a.comb_tokens;
    const int nt = min(a.comb_tokens, a.T - t_first);
    if (a.slot_flag && a.flags) {
        const int per_tok = k * a.ncb;
        const int nflag = nt * per_tok;
        bool ok = true;
        const u64 tw0 = WAIT ? now_ticks() : 0ull;
#pragma unroll 4
        for (int q = tid; q < nflag; q += kThreads) {
            const int slot = t_first * k + q / a.ncb;
            ok = ok && (ld_relaxed(&a.flags[a.slot_flag[slot] + q % a.ncb], sys) == a.epoch);
        }
        if (WAIT && !ok) {
            for (int q = tid; q < nflag; q += kThreads) {
                const int slot = t_first * k + q / a.ncb;
                const u32 *fp = &a.flags[a.slot_flag[slot] + q % a.ncb];
                const u64 t0 = now_ticks();
                int spins = 0;
                while (ld_relaxed(fp, sys) != a.epoch) {
                    __builtin_amdgcn_s_sleep(2);
                    if ((++spins & 63) == 0) {
                        if (ld_relaxed_agent(&a.ctrl->error) != 0) break;
                        if (now_ticks() - t0 > a.wait_ticks) {
                            set_error(a.ctrl, MOE_ERR_TIMEOUT);
                            atomicAdd(&a.ctrl->stats[6], 1ull);
                            break;
                        }
                    }
                }
            }
        }
        fence_acquire(sys);
        if (!WAIT && !ok && a.status_dev) atomicExch(a.status_dev, (int)MOE_ERR_NOT_READY);
        // rows guarded by flags another lane polled; the time the workgroup waited is added once
        const int waited = __syncthreads_or(WAIT && !ok);
        if (WAIT && waited && tid == 0) atomicAdd(&a.ctrl->stats[14], now_ticks() - tw0);
    }
    const size_t rstride = (size_t)a.d * sizeof(ET);
    for (int tt = wave; tt < nt; tt += 4) {
        const int t = t_first + tt;
        const char *rows = staging + (size_t)t * k * rstride;
        char *orow = (char *)a.out + (size_t)t * rstride;
        const float *wt = a.w + (size_t)t * k;
        // eight 16-byte loads in flight per lane whatever k is
        if (k == 1)
            combine_token<ET, 8, STREAM>(rows, wt, orow, k, pieces, rstride, lane);
        else if (k <= 2)
            combine_token<ET, 4, STREAM>(rows, wt, orow, k, pieces, rstride, lane);
        else if (k <= 4)
            combine_token<ET, 2, STREAM>(rows, wt, orow, k, pieces, rstride, lane);
        else
            combine_token<ET, 1, STREAM>(rows, wt, orow, k, pieces, rstride, lane);
    }
}

// Combine tasks from their counter until none is left.  (Inlined into the
// kernel: only the GEMM stages need a register allocation of their own.)
template <typename ET>
__device__ __forceinline__ void combine_stage(const KArgs &a, char *smem) {
    const int tid = threadIdx.x;
    Ctrl *c = a.ctrl;
    StageLds *sl = (StageLds *)(smem + a.sched_lds_off);
    const u64 t0 = kernel_start_ticks(c);
    __syncthreads();
    if (tid == 0) sl->next = (int)atomicAdd(&c->comb_next, 1u);
    __syncthreads();
    int t = uniform(sl->next);
    while (t < a.nCT) {
        u32 next = 0;
        if (tid == 0) next = atomicAdd(&c->comb_next, 1u);
        combine_task<ET, true>(a, t);
        __syncthreads();
        if (tid == 0) {
            mark_phase_end(c, 5, t0);
            sl->next = (int)next;
        }
        __syncthreads();
        t = uniform(sl->next);
    }
}

// ---- the ready-queue scheduler (MOE_SCHED_READY_QUEUE; paper section 2.3: tasks are
// enqueued when the data they need has arrived and processors take them from the queue).
// After the front stage a workgroup holds at most one ticket of a ready queue (its own XCD's
// until that queue's tickets are used up, then the next one's) and loops: if the entry of its
// ticket has been written, run it (a GEMM2 tile or a combine task) and draw the next ticket
// while it runs; else run a GEMM1 tile (big before small, own XCD's list first); else sleep.
// So ready tasks go before new GEMM1 tiles, GEMM2 tiles and combine tasks start in the order
// in which their inputs became complete, and nothing that runs ever waits.  No deadlock,
// whatever the grid size: a workgroup sleeps only when every GEMM1 tile has been handed out,
// and then every entry still to be written will be written by a workgroup that is running a
// tile; every ticket below the queue's size is held by a workgroup that runs its entry as
// soon as it can.  A workgroup leaves when all queues are out of tickets and no GEMM1 tile
// is left (or the error flag is up; the sleep is bounded like every wait here).
template <class P, class PS, bool MIXED>
__device__ __forceinline__ void ready_queue_stage(const KArgs &a, KArgsAddr kargs, char *smem, int home, int n_rb,
                                                  int n_rbs, volatile int *caller_local) {
    using ET = typename P::ET;
    const int tid = threadIdx.x;
    Ctrl *c = a.ctrl;
    StageLds *sl = (StageLds *)(smem + a.sched_lds_off);
    const u32 lds = lds_offset_opaque(smem);
    const u64 t0 = kernel_start_ticks(c);
    int q = home, hops = 0;  // the queue tickets come from; hops == kTileQueues: all queues are used up
    int ticket = -1;         // entry of queue q this workgroup is to run (may lie beyond the queue's size), -1 = none
    int g1_left = 1;
    u64 idle_since = 0;      // thread 0: start of the current sleep, 0 = not sleeping
    while (true) {
        __syncthreads();
        if (tid < 64) {
            // lanes 0-7: big GEMM1 list of XCD home + lane; 8-15: its small one; 24: error flag
            const int kind = tid >> 3, qq = (home + (tid & 7)) % kTileQueues;
            bool has = false;
            if (g1_left && (kind == 0 || (kind == 1 && MIXED))) {
                const TileQueue tq = tile_queue(a, n_rb, n_rbs, qq);
                has = ld_relaxed_agent(&c->tile_next[kind][qq]) < (u32)(kind == 0 ? tq.n1b : tq.n1s);
            } else if (tid == 24) {
                has = ld_relaxed_agent(&c->error) != 0u;
            }
            const u64 m = __ballot(has);
            if (tid == 0) {
                // a ticket beyond its queue's size says the queue is used up: on to the next one
                if (ticket >= 0 && ticket >= ready_queue_size(a, n_rb, n_rbs, q)) ticket = -1, q = (q + 1) % kTileQueues, ++hops;
                while (ticket < 0 && hops < kTileQueues) {
                    ticket = (int)atomicAdd(&c->rq_head[q], 1u);
                    if (ticket >= ready_queue_size(a, n_rb, n_rbs, q)) ticket = -1, q = (q + 1) % kTileQueues, ++hops;
                }
                u32 *slot = &a.rq_slots[(size_t)q * a.rq_cap + (ticket >= 0 ? ticket : 0)];
                const u32 v = ticket >= 0 ? ld_relaxed_agent(slot) : 0u;
                int pick = 0, val = 0, lq = 0;  // pick: -2 leave, 0 sleep, 1 ready task, 2 / 3 big / small GEMM1 tile, 4 look again
                if ((m >> 24) & 1ull) {
                    pick = -2;
                } else if (v != 0u) {
                    st_relaxed(slot, 0u, 0);  // empty again for the next call
                    ticket = -1;
                    atomicAdd(&c->stats[16], 1ull);
                    // out of order: a GEMM2 tile goes first although GEMM1 tiles are still in the lists
                    if (!(v & kReadyCombine) && (m & 0xffffull)) atomicAdd(&c->stats[17], 1ull);
                    pick = 1, val = (int)v;
                } else if (m & 0xffffull) {
                    const u32 lists = (u32)(m & 0xffffull);
                    const int kd = (lists & 0xffu) ? 0 : 1;
                    lq = (home + __ffs((int)((lists >> (8 * kd)) & 0xffu)) - 1) % kTileQueues;
                    const TileQueue tq = tile_queue(a, n_rb, n_rbs, lq);
                    const u32 i = atomicAdd(&c->tile_next[kd][lq], 1u);
                    pick = (i < (u32)(kd == 0 ? tq.n1b : tq.n1s)) ? 2 + kd : 4;
                    val = (int)i;
                } else {
                    g1_left = 0;
                    if (ticket < 0) pick = -2;  // hops == kTileQueues: nothing more can come
                }
                if (pick == 0) {
                    const u64 now = now_ticks();
                    if (idle_since == 0) idle_since = now;
                    if (now - idle_since > a.wait_ticks) {
                        set_error(c, MOE_ERR_TIMEOUT);
                        atomicAdd(&c->stats[6], 1ull);
                        pick = -2;
                    }
                } else if (idle_since != 0) {
                    atomicAdd(&c->stats[14], now_ticks() - idle_since);
                    idle_since = 0;
                }
                sl->pick = pick, sl->next = val, sl->ok = lq;
                sl->q = q, sl->hops = hops, sl->ticket = ticket, sl->g1_left = g1_left;
            }
        }
        __syncthreads();
        const int pick = uniform(sl->pick), val = uniform(sl->next), lq = uniform(sl->ok);
        q = uniform(sl->q), hops = uniform(sl->hops), ticket = uniform(sl->ticket), g1_left = uniform(sl->g1_left);
        if (pick == -2) break;
        if (pick == 0) __builtin_amdgcn_s_sleep(8);
        if (pick == 0 || pick == 4) continue;
        // the next ticket is drawn while the task runs, if the workgroup holds none
        int tq_next = (ticket < 0 && hops < kTileQueues) ? q : -1;
        if ((pick == 3 && !MIXED) || (pick == 1 && !((u32)val & kReadyCombine) && (val - 1) / a.tl.NT2 >= n_rb && !MIXED))
            tq_next = -1;  // (cannot happen: no such tiles without mixed heights; nothing runs, nothing is drawn)
        if (pick == 2) {
            tile_stage<P, true, false>(kargs, lds, home, n_rb, n_rbs, lq, val, tq_next, caller_local);
        } else if (pick == 3) {
            if (MIXED) tile_stage<PS, true, true>(kargs, lds, home, n_rb, n_rbs, lq, val, tq_next, caller_local);
        } else if ((u32)val & kReadyCombine) {
            u32 next = 0x7fffffffu;
            if (tid == 0 && tq_next >= 0) next = atomicAdd(&c->rq_head[tq_next], 1u);
            combine_task<ET, true>(a, (int)((u32)val & ~kReadyCombine));
            __syncthreads();
            if (tid == 0) {
                mark_phase_end(c, 5, t0);
                sl->next = (int)next;
            }
        } else {
            const int code = val - 1, rb = code / a.tl.NT2, ct = code % a.tl.NT2;
            if (rb < n_rb)
                tile_stage<P, false, false>(kargs, lds, home, n_rb, n_rbs, rb, ct, tq_next, caller_local);
            else if (MIXED)
                tile_stage<PS, false, true>(kargs, lds, home, n_rb, n_rbs, rb - n_rb, ct, tq_next, caller_local);
        }
        __syncthreads();
        if (tq_next >= 0) {
            const int t = uniform(sl->next);
            if (t != 0x7fffffff) ticket = t;
        }
    }
    if (tid == 0 && idle_since != 0) atomicAdd(&c->stats[14], now_ticks() - idle_since);
}

}  // namespace moe

// Dispatch in its local form (paper section 2.1 step 2, section 2.3 "group
// tokens into tiles"): histogram -> exclusive scans -> stable permutation ->
// coalesced row gather, plus the tables the tile scheduler and the publish
// step read (row blocks per expert, flag numbering per destination).
#pragma once
#include "common.hpp"

namespace moe {

// LDS the plan needs, and whether its two tables are staged in LDS (they are
// unless the problem is unusually large; then the slow global-memory path runs).
constexpr size_t kPlanSegLds = 48 * 1024, kPlanHistLds = 32 * 1024;
__host__ __device__ inline bool plan_seg_in_lds(int E, int R) { return (size_t)3 * E * R * 4 <= kPlanSegLds; }
__host__ __device__ inline bool plan_hist_in_lds(int nPB, int E) { return (size_t)nPB * E * 4 <= kPlanHistLds; }
__host__ __device__ inline size_t plan_smem_bytes(int E, int R, int nPB) {
    size_t n = (size_t)(4 * E + 2 * R + 12) * 4;
    if (plan_seg_in_lds(E, R)) n += (size_t)3 * E * R * 4;
    if (plan_hist_in_lds(nPB, E)) n += (size_t)nPB * E * 4;
    return n;
}

// Exclusive prefix sum by ONE wavefront over n values src[0], src[stride], ... (LDS or global),
// written to dst at the same positions; returns the total.  src == dst is allowed.
__device__ __forceinline__ int wave_exclusive_scan(const int32_t *src, int32_t *dst, int n, int stride, int start) {
    const int lane = threadIdx.x & 63;
    int carry = start;
    for (int base = 0; base < n; base += 64) {
        const int i = base + lane;
        const int x = i < n ? src[(size_t)i * stride] : 0;
        int inc = x;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int o = __shfl_up(inc, off, 64);
            if (lane >= off) inc += o;
        }
        if (i < n) dst[(size_t)i * stride] = carry + inc - x;
        carry += __shfl(inc, 63, 64);
    }
    return carry;
}

// Single-workgroup task.  Reads blk_hist[nPB][E] and, unless it can be derived from it, seg_cnt[E][R]
// (complete),
// writes counts, offsets, blk_base, seg_begin, flag_base, dest_flag_begin, dest_group_begin,
// rb_base, rb_expert, rbs_base, rbs_expert, ctrl->n_rb, ctrl->n_rbs, ctrl->n_flags.  The inputs are first copied
// to LDS with coalesced loads; every scan then runs either one thread per
// sequence (many short sequences) or one wavefront per sequence with a shuffle
// scan (few long ones), so that nothing walks a long sequence serially.
__device__ __forceinline__ void plan_task(const KArgs &a, char *smem) {
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int E = a.E, R = a.R, nPB = a.nPB;
    int32_t *s_cnt = (int32_t *)smem;  // [E]
    int32_t *s_off = s_cnt + E;        // [E+1]
    int32_t *s_dest = s_off + E + 1;   // [R+1] flags per destination, then their scan
    int32_t *s_rb = s_dest + R + 1;    // [E+1] row blocks per expert, then their scan
    int32_t *s_grp = s_rb + E + 2;     // [R+1] fence groups per destination, then their scan
    int32_t *s_rbs = s_grp + R + 1;    // [E+1] small row blocks per expert (0 or 1), then their scan
    int32_t *s_free = s_cnt + ((4 * E + 2 * R + 7 + 3) & ~3);  // behind s_rbs, 16-byte aligned (inside the 12 spare words)
    MOE_TT_BEGIN();
    const bool seg_lds = plan_seg_in_lds(E, R), hist_lds = plan_hist_in_lds(nPB, E);
    int32_t *segc = a.seg_cnt, *segb = a.seg_begin, *hist = a.blk_base, *nfl = a.flag_base;
    // tile_m and the row-block height are powers of two
    const int lm = 31 - __clz(a.tile_m), lbm = 31 - __clz(a.tl.BM);
    if (seg_lds) {
        segc = s_free;
        segb = segc + E * R;
        nfl = segb + E * R;  // [R][E]
        s_free = nfl + E * R;
        if (!a.seg_from_blocks) {
#pragma unroll 8
            for (int q = tid; q < E * R; q += kThreads) segc[q] = a.seg_cnt[q];
        }
    }
    if (hist_lds) hist = s_free;
    // (independent loads, all of a thread's in flight together: nothing else runs on the GPU while
    // the plan does; blk_base <- blk_hist if not in LDS)
    if (((nPB * E) & 3) == 0 && (!hist_lds || !seg_lds || ((3 * E * R) & 3) == 0)) {  // 16-byte pieces
        const u32x4_t *src = (const u32x4_t *)a.blk_hist;
        u32x4_t *dst = (u32x4_t *)hist;
#pragma unroll 8
        for (int q = tid; q < nPB * E / 4; q += kThreads) dst[q] = src[q];
    } else {
#pragma unroll 8
        for (int q = tid; q < nPB * E; q += kThreads) hist[q] = a.blk_hist[q];
    }
    __syncthreads();
    if (a.seg_from_blocks) {  // a destination is a whole number of blocks: add up its blocks' histograms
        const int bpd = a.per_dest / kPermBlock;
        for (int q = tid; q < E * R; q += kThreads) {
            const int e = q / R, r = q - e * R;
            int c = 0;
            for (int b = r * bpd; b < (r + 1) * bpd; ++b) c += hist[b * E + e];
            segc[q] = c;
        }
        __syncthreads();
    }
    MOE_TT(a.ctrl, 34);
    // per expert: rows per destination -> first row of each (e, r) segment and the total
    if (R <= 16) {
        for (int e = tid; e < E; e += kThreads) {
            int sb = 0;
            for (int r = 0; r < R; ++r) {
                const int c = segc[e * R + r];
                segb[e * R + r] = sb;
                sb += c;
            }
            s_cnt[e] = sb;
        }
    } else {
        for (int e = wave; e < E; e += 4) {
            const int total = wave_exclusive_scan(segc + (size_t)e * R, segb + (size_t)e * R, R, 1, 0);
            if (lane == 0) s_cnt[e] = total;
        }
    }
    __syncthreads();
    // row blocks per expert.  One height: ceil(rows / BM).  Mixed heights: big blocks, and the last
    // rows of the expert in one small block when they fit into it.
    for (int e = tid; e < E; e += kThreads) {
        const int n = s_cnt[e];
        if (a.tl.BMS == 0) {
            s_rb[e] = (n + a.tl.BM - 1) >> lbm;
            s_rbs[e] = 0;
        } else {
            const int rem = n & (a.tl.BM - 1);
            // a short tail gets a small block; but where the layer is bound by streaming weights (tail_with_big),
            // an expert that has big blocks keeps its tail with them, as a padded big block: its weights are then
            // streamed once, while its tiles run side by side, and not a second time in the small-tile phase
            const bool small = rem > 0 && rem <= a.tl.BMS && (!a.tl.tail_with_big || (n >> lbm) == 0);
            s_rb[e] = (n >> lbm) + ((rem > 0 && !small) ? 1 : 0);
            s_rbs[e] = small ? 1 : 0;
        }
    }
    __syncthreads();
    if (wave == 0) {
        int rows = wave_exclusive_scan(s_cnt, s_off, E, 1, 0);
        if (a.capacity > 0) {  // padded layout: expert e owns the `capacity` rows from e * capacity
            for (int e = lane; e < E; e += 64) {
                s_off[e] = e * a.capacity;
                if (s_cnt[e] > a.capacity) set_error(a.ctrl, MOE_ERR_CAPACITY);
            }
            rows = E * a.capacity;
        }
        const int rb = wave_exclusive_scan(s_rb, s_rb, E, 1, 0);
        const int rbs = wave_exclusive_scan(s_rbs, s_rbs, E, 1, 0);
        if (lane == 0) {
            s_off[E] = rows;
            s_rb[E] = rb;
            s_rbs[E] = rbs;
            a.ctrl->n_rb = (u32)rb;
            a.ctrl->n_rbs = (u32)rbs;
        }
    }
    __syncthreads();
    for (int e = tid; e <= E; e += kThreads) {
        a.offsets[e] = s_off[e];
        a.rb_base[e] = s_rb[e];
        a.rbs_base[e] = s_rbs[e];
        if (e < E) {
            a.counts[e] = s_cnt[e];
            for (int i = s_rb[e]; i < s_rb[e + 1]; ++i) a.rb_expert[i] = e;
            if (s_rbs[e + 1] > s_rbs[e]) a.rbs_expert[s_rbs[e]] = e;
        }
    }
    // sorted position of each block's first slot of e: exclusive scan over blocks
    if (E >= 64) {
        for (int e = tid; e < E; e += kThreads) {
            int run = s_off[e];
            for (int b = 0; b < nPB; ++b) {
                const int c = hist[b * E + e];
                hist[b * E + e] = run;
                run += c;
            }
        }
    } else {
        for (int e = wave; e < E; e += 4) wave_exclusive_scan(hist + e, hist + e, nPB, E, s_off[e]);
    }
    MOE_TT(a.ctrl, 36);
    // flags: destination-major, then expert; a segment with expert-local rows
    // [b0, b0+c) touches row blocks b0/tile_m .. (b0+c-1)/tile_m.  All (r, e)
    // pairs in parallel, then one scan per destination.
    for (int q = tid; q < E * R; q += kThreads) {
        const int r = q / E, e = q - r * E;
        const int c = segc[e * R + r];
        int n = 0;
        if (c > 0) {
            const int b0 = segb[e * R + r];
            n = (((b0 + c - 1) >> lm) - (b0 >> lm) + 1) * a.ncb;
        }
        nfl[q] = n;
    }
    __syncthreads();
    if (R <= 16) {
        for (int r = wave; r < R; r += 4) {
            const int total = wave_exclusive_scan(nfl + (size_t)r * E, nfl + (size_t)r * E, E, 1, 0);
            if (lane == 0) s_dest[r] = total;
        }
    } else {
        for (int r = tid; r < R; r += kThreads) {
            int run = 0;
            for (int e = 0; e < E; ++e) {
                const int n = nfl[r * E + e];
                nfl[r * E + e] = run;  // exclusive within the destination
                run += n;
            }
            s_dest[r] = run;
        }
    }
    __syncthreads();
    // fence groups of the per-destination mode: all flags of a destination, or group_size at a time
    for (int r = tid; r < R; r += kThreads)
        s_grp[r] = a.group_size > 0 ? (s_dest[r] + a.group_size - 1) / a.group_size : 1;
    __syncthreads();
    if (wave == 0) {
        const int total = wave_exclusive_scan(s_dest, s_dest, R, 1, 0);
        const int groups = wave_exclusive_scan(s_grp, s_grp, R, 1, 0);
        if (lane == 0) {
            s_dest[R] = total;
            s_grp[R] = groups;
            a.ctrl->n_flags = (u32)total;
        }
    }
    __syncthreads();
    MOE_TT(a.ctrl, 37);
    if (hist_lds)
        for (int q = tid; q < nPB * E; q += kThreads) a.blk_base[q] = hist[q];
    if (seg_lds)
        for (int q = tid; q < E * R; q += kThreads) a.seg_begin[q] = segb[q];
    for (int q = tid; q < E * R; q += kThreads) a.flag_base[q] = nfl[q] + s_dest[q / E];
    for (int r = tid; r <= R; r += kThreads) {
        a.dest_flag_begin[r] = s_dest[r];
        a.dest_group_begin[r] = s_grp[r];
    }
    __syncthreads();
    MOE_TT(a.ctrl, 38);
}

// One permutation block: tokens [b*64, b*64+64).  The k experts of a token are
// distinct, so the rank of slot (t, e) among the block's slots of e is the
// number of earlier tokens of the block that chose e: a popcount on a 64-bit
// per-expert mask.  Deterministic, no arrival-order atomics.
// mask[e] = the tokens of block b (bit = token - b*64) that chose expert e
__device__ __forceinline__ void block_masks(const KArgs &a, int b, u64 *mask) {
    const int tid = threadIdx.x;
    const int E = a.E, k = a.k;
    const int t0 = b * kPermBlock;
    const int nt = min(kPermBlock, a.T - t0);
    for (int e = tid; e < E; e += kThreads) mask[e] = 0ull;
    __syncthreads();
    for (int q = tid; q < nt * k; q += kThreads) {
        int e = a.idx[(size_t)t0 * k + q];
        if (e >= 0 && e < E) atomicOr(&mask[e], 1ull << (q / k));
    }
    __syncthreads();
}

// base[e]: sorted position of the block's first slot of expert e; counts[e]: rows of expert e (E entries
// each, LDS or global; counts is read in the padded layout only)
template <typename ET>
__device__ __forceinline__ void perm_task(const KArgs &a, int b, char *smem, const int32_t *base,
                                          const int32_t *counts) {
    const int tid = threadIdx.x;
    const int E = a.E, k = a.k;
    u64 *mask = (u64 *)smem;  // [E]
    const int t0 = b * kPermBlock;
    const int nt = min(kPermBlock, a.T - t0);
    block_masks(a, b, mask);
    if (a.capacity > 0) {
        // padded layout: the unused entries of perm, experts dealt round-robin to the blocks (counts[] is
        // final: the plan, or the caller's own sums, came first)
        for (int e = b; e < E; e += a.nPB)
            for (int j = counts[e] + tid; j < a.capacity; j += kThreads) a.perm[(size_t)e * a.capacity + j] = -1;
    }
    for (int q = tid; q < nt * k; q += kThreads) {
        const int s = t0 * k + q;
        const int tl = q / k;
        const int e = a.idx[s];
        if (e < 0 || e >= E) continue;
        const int rank = __popcll(mask[e] & ((1ull << tl) - 1ull));
        const int p = base[e] + rank;
        a.perm[p] = s;
        a.inv_perm[s] = p;
        if (a.slot_flag) {
            const int r = (t0 + tl) / a.per_dest;
            const int ql = p - a.offsets[e];
            const int b0 = a.seg_begin[(size_t)e * a.R + r];
            a.slot_flag[s] = a.flag_base[(size_t)r * E + e] + (ql / a.tile_m - b0 / a.tile_m) * a.ncb;
        }
    }
    __syncthreads();
}

// Standalone dispatch without the single-workgroup plan (it needs none of the plan's tables for
// tiles and flags), in two steps that every permutation block runs in parallel.
// Step 1: the block's histogram = popcounts of its masks, to hist[b][.].
__device__ __forceinline__ void block_hist_task(const KArgs &a, int b, int32_t *hist, char *smem) {
    u64 *mask = (u64 *)smem;  // [E]
    block_masks(a, b, mask);
    for (int e = threadIdx.x; e < a.E; e += kThreads) hist[(size_t)b * a.E + e] = __popcll(mask[e]);
}
// LDS of step 2: all histograms, three tables of E + 1, the masks
__host__ __device__ inline size_t block_perm_smem_bytes(int E, int nPB) {
    return (((size_t)nPB * E + 3 * (E + 1)) * 4 + 15) / 16 * 16 + (size_t)E * 8;
}
// Step 2: every block reads all histograms (they are small), adds up the columns (counts), scans them
// (offsets), takes the part of each column above itself (its base), and writes its slots' positions.
// Block 0 also writes counts and offsets.
template <typename ET>
__device__ __forceinline__ void block_perm_task(const KArgs &a, int b, const int32_t *hist_g, char *smem) {
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int E = a.E, nPB = a.nPB;
    int32_t *hist = (int32_t *)smem;   // [nPB][E]
    int32_t *tot = hist + nPB * E;     // [E+1]
    int32_t *base = tot + E + 1;       // [E+1]
    int32_t *off = base + E + 1;       // [E+1]
    char *mask_smem = smem + (((size_t)nPB * E + 3 * (E + 1)) * 4 + 15) / 16 * 16;
    if (((nPB * E) & 3) == 0) {
        const u32x4_t *src = (const u32x4_t *)hist_g;
        u32x4_t *dst = (u32x4_t *)hist;
#pragma unroll 8
        for (int q = tid; q < nPB * E / 4; q += kThreads) dst[q] = src[q];
    } else {
#pragma unroll 8
        for (int q = tid; q < nPB * E; q += kThreads) hist[q] = hist_g[q];
    }
    __syncthreads();
    // column e, split over the four wavefronts' worth of threads when there are few experts
    for (int e = tid; e < E; e += kThreads) {
        int run = 0, mine = 0;
        for (int bb = 0; bb < nPB; ++bb) {
            if (bb == b) mine = run;
            run += hist[bb * E + e];
        }
        tot[e] = run;
        base[e] = mine;
    }
    __syncthreads();
    if (wave == 0) {
        const int total = wave_exclusive_scan(tot, off, E, 1, 0);
        if (lane == 0) off[E] = total;
    }
    __syncthreads();
    const int total_rows = off[E];
    __shared__ int s_over;
    if (tid == 0) s_over = 0;
    __syncthreads();
    if (a.capacity > 0) {  // padded layout: expert e owns the `capacity` rows from e * capacity
        for (int e = tid; e <= E; e += kThreads) {
            off[e] = e * a.capacity;
            if (e < E && tot[e] > a.capacity) s_over = 1;
        }
        __syncthreads();
    }
    for (int e = tid; e < E; e += kThreads) base[e] += off[e];
    // ids outside [0, E) are counted nowhere: the histogram then accounts for fewer than N slots
    const bool bad_ids = total_rows != a.N;
    if (b == 0) {
        for (int e = tid; e <= E; e += kThreads) {
            a.offsets[e] = off[e];
            if (e < E) a.counts[e] = tot[e];
        }
        if (tid == 0 && a.status_dev) {
            if (bad_ids)
                *a.status_dev = (int)MOE_ERR_BAD_ROUTING;
            else if (s_over)
                *a.status_dev = (int)MOE_ERR_CAPACITY;
        }
    }
    __syncthreads();
    // an expert has more rows than the capacity, or an id is invalid: counts and the status say so, nothing else
    // is written
    if (s_over || bad_ids) return;
    perm_task<ET>(a, b, mask_smem, base, tot);
}

// x_perm[p,:] = x[perm[p]/k,:] for sorted rows p = first, first+stride, ...: one
// wavefront per row, 16-byte pieces, up to four loads in flight per lane, so
// both the reads and the writes are whole contiguous rows.
__device__ void gather_rows(const KArgs &a, int first, int stride, size_t row_bytes) {
    const int lane = threadIdx.x & 63;
    const int pieces = (int)(row_bytes / 16);
    for (int p = first; p < a.NP; p += stride) {
        const int s = a.perm[p];
        uint4 *dst = (uint4 *)((char *)a.x_perm + (size_t)p * row_bytes);
        if (s < 0 || s >= a.N) {  // unused row of the padded layout (a slot number is never followed out of x)
            for (int c = lane; c < pieces; c += 64) dst[c] = make_uint4(0u, 0u, 0u, 0u);
            continue;
        }
        const uint4 *src = (const uint4 *)((const char *)a.x + (size_t)(s / a.k) * row_bytes);
        int c = lane;
        for (; c + 192 < pieces; c += 256) {
            uint4 v0 = src[c], v1 = src[c + 64], v2 = src[c + 128], v3 = src[c + 192];
            dst[c] = v0;
            dst[c + 64] = v1;
            dst[c + 128] = v2;
            dst[c + 192] = v3;
        }
        for (; c < pieces; c += 64) dst[c] = src[c];
    }
}

// ---- the standalone dispatch as one launch: every workgroup owns kScatterTokens tokens and derives, by itself,
// everything it needs to place them: it counts ALL N slots per expert (the ids are a few hundred KB that stay in
// the L2), split into those in front of its own first slot and the rest; the sums give counts and offsets, the
// front part gives the sorted position of its own first slot of every expert, and a popcount on per-expert
// token masks gives the rank inside the workgroup (the k experts of a token are distinct).  No histogram
// crosses workgroups, so there is no second launch and no grid-wide wait.  Then every token row is read ONCE and
// stored to its k sorted positions: the row movement writes N rows but reads only T (a gather by sorted
// position reads N rows, most of them from cache, and the chip then moves the written rows at barely half
// the rate).  Used while N x workgroups stays small enough for the redundant counting to hide behind the row
// movement of the other workgroups of a CU; larger problems take the histogram form.
constexpr int kScatterTokens = 16;  // at most; fewer when there are few tokens (see scatter_tokens)
// tokens per workgroup of the row movement: 16, or as many as still give about 256 workgroups
__host__ __device__ inline int scatter_tokens(int T) {
    int t = kScatterTokens;
    while (t > 1 && (T + t - 1) / t < 256) t >>= 1;
    return t;
}

// copies of the LDS counters that lanes are spread over, so that few experts do not serialise the LDS atomics
__host__ __device__ inline int count_copies(int E) {
    int c = 1;
    while (c < 16 && 2 * c * E <= 256) c *= 2;
    return c;
}

// 16-byte store of a row piece of x_perm: written through to memory (STORE 0; rows that fit the memory-side
// cache) or non-temporal (STORE 1; more rows than that cache holds)
template <int STORE>
__device__ __forceinline__ void store_row16(char *p, const uint4 &v) {
    const u32x4_t w = {v.x, v.y, v.z, v.w};
    if (STORE == 0)
        asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 1" ::"v"(p), "v"(w) : "memory");  // (s_nop: see store_tile16)
    else
        __builtin_nontemporal_store(w, (u32x4_t *)p);
}

// rows of tokens t0 .. t0+nt-1 to the sorted positions pos[tl*k + j] (LDS): a wavefront takes 4 KB of a token's row
// at a time (the four wavefronts share a row when the workgroup has fewer than four tokens), each piece loaded once
// and stored k times, four 16-byte loads in flight per lane
template <int STORE>
__device__ __forceinline__ void scatter_rows(const KArgs &a, int t0, int nt, const int *pos, size_t row_bytes) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int pieces = (int)(row_bytes / 16), k = a.k;
    char *xp = (char *)a.x_perm;
    // with four tokens or more a wavefront owns whole rows; with fewer the wavefronts share each row's chunks
    const int tstep = nt >= 4 ? 4 : 1, cstep = nt >= 4 ? 256 : 1024;
    for (int tl = nt >= 4 ? wave : 0; tl < nt; tl += tstep) {
        const uint4 *src = (const uint4 *)((const char *)a.x + (size_t)(t0 + tl) * row_bytes);
        for (int c = (nt >= 4 ? 0 : wave * 256) + lane; c < pieces; c += cstep) {
            uint4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (c + 64 * u < pieces) v[u] = src[c + 64 * u];
            for (int j = 0; j < k; ++j) {
                char *dst = xp + (size_t)pos[tl * k + j] * row_bytes;
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (c + 64 * u < pieces) store_row16<STORE>(dst + (size_t)(c + 64 * u) * 16, v[u]);
            }
        }
    }
}

template <int STORE>
__device__ __forceinline__ void dispatch_fused_task(const KArgs &a, int b, size_t row_bytes) {
    __shared__ int s_bef[256], s_aft[256], s_cnt[kMaxExperts], s_off[kMaxExperts + 1], s_base[kMaxExperts];
    __shared__ u64 s_mask[kMaxExperts];
    __shared__ int s_pos[kScatterTokens * 32];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int E = a.E, k = a.k, N = a.N;
    const int t0 = b * a.disp_tokens, nt = min(a.disp_tokens, a.T - t0), s0 = t0 * k;
    const int C = count_copies(E);
    s_bef[tid] = 0;
    s_aft[tid] = 0;
    for (int e = tid; e < E; e += kThreads) s_mask[e] = 0ull;
    __syncthreads();
    // ---- every slot, counted in front of / from this workgroup's first slot on
    int *my_bef = s_bef + (lane & (C - 1)) * E, *my_aft = s_aft + (lane & (C - 1)) * E;
    auto count = [&](int e, int s) {
        if ((unsigned)e < (unsigned)E) atomicAdd(s < s0 ? &my_bef[e] : &my_aft[e], 1);
    };
    if ((((uintptr_t)a.idx) & 15) == 0) {
        // 16 loads of four ids in flight per thread: the ids come from the L2, and one trip at a time would
        // cost more than the row movement that follows
        const int4 *idx4 = (const int4 *)a.idx;
        const int n4 = N >> 2;
        constexpr int U = 16;
        for (int q0 = tid; q0 < n4; q0 += kThreads * U) {
            int4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (q0 + u * kThreads < n4) v[u] = idx4[q0 + u * kThreads];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int q = q0 + u * kThreads;
                if (q < n4) count(v[u].x, 4 * q), count(v[u].y, 4 * q + 1), count(v[u].z, 4 * q + 2), count(v[u].w, 4 * q + 3);
            }
        }
        for (int s = (n4 << 2) + tid; s < N; s += kThreads) count(a.idx[s], s);
    } else {
#pragma unroll 4
        for (int s = tid; s < N; s += kThreads) count(a.idx[s], s);
    }
    __syncthreads();
    for (int e = tid; e < E; e += kThreads) {
        int bs = 0, as = 0;
        for (int c = 0; c < C; ++c) bs += s_bef[c * E + e], as += s_aft[c * E + e];
        s_base[e] = bs;
        s_cnt[e] = bs + as;
    }
    __syncthreads();
    if (wave == 0) {
        const int total = wave_exclusive_scan(s_cnt, s_off, E, 1, 0);
        if (lane == 0) s_off[E] = total;
    }
    __syncthreads();
    // ids outside [0, E) are counted nowhere: the histogram then accounts for fewer than N slots
    const bool bad_ids = s_off[E] != N;
    int over = 0;
    if (a.capacity > 0) {  // padded layout: expert e owns the `capacity` rows from e * capacity
        for (int e = tid; e < E; e += kThreads) over |= s_cnt[e] > a.capacity ? 1 : 0;
        over = __syncthreads_or(over);
        for (int e = tid; e <= E; e += kThreads) s_off[e] = e * a.capacity;
        __syncthreads();
    }
    if (b == 0) {
        for (int e = tid; e <= E; e += kThreads) {
            a.offsets[e] = s_off[e];
            if (e < E) a.counts[e] = s_cnt[e];
        }
        if (tid == 0 && a.status_dev) {
            if (bad_ids)
                *a.status_dev = (int)MOE_ERR_BAD_ROUTING;
            else if (over)
                *a.status_dev = (int)MOE_ERR_CAPACITY;
        }
    }
    if (bad_ids || over) return;  // counts and the status say so; nothing else is written
    // ---- this workgroup's slots: rank inside the workgroup from the per-expert token masks
    for (int q = tid; q < nt * k; q += kThreads) atomicOr(&s_mask[a.idx[s0 + q]], 1ull << (q / k));
    __syncthreads();
    for (int q = tid; q < nt * k; q += kThreads) {
        const int e = a.idx[s0 + q], tl = q / k;
        const int p = s_off[e] + s_base[e] + __popcll(s_mask[e] & ((1ull << tl) - 1ull));
        a.perm[p] = s0 + q;
        a.inv_perm[s0 + q] = p;
        s_pos[q] = p;
    }
    if (a.capacity > 0) {
        // padded layout: the unused entries of perm and rows of x_perm, experts dealt round-robin to the workgroups
        const int pieces = (int)(row_bytes / 16);
        for (int e = b; e < E; e += (int)gridDim.x) {
            const int first = e * a.capacity + s_cnt[e], n = a.capacity - s_cnt[e];
            for (int j = tid; j < n; j += kThreads) a.perm[first + j] = -1;
            if (a.x_perm) {
                uint4 *rows = (uint4 *)((char *)a.x_perm + (size_t)first * row_bytes);
                for (size_t q = tid; q < (size_t)n * pieces; q += kThreads) rows[q] = make_uint4(0u, 0u, 0u, 0u);
            }
        }
    }
    __syncthreads();
    if (a.x_perm) scatter_rows<STORE>(a, t0, nt, s_pos, row_bytes);
}

// The row movement of the histogram form for the ragged layout, as its own launch after the permutation: the
// sorted positions of the workgroup's tokens come from inv_perm.
template <int STORE>
__device__ __forceinline__ void scatter_task(const KArgs &a, int b, size_t row_bytes) {
    __shared__ int s_pos[kScatterTokens * 32];
    const int t0 = b * a.disp_tokens, nt = min(a.disp_tokens, a.T - t0);
    for (int q = threadIdx.x; q < nt * a.k; q += kThreads) {
        const int p = a.inv_perm[(size_t)t0 * a.k + q];
        s_pos[q] = min(max(p, 0), a.NP - 1);  // (a position is never followed out of x_perm)
    }
    __syncthreads();
    scatter_rows<STORE>(a, t0, nt, s_pos, row_bytes);
}

}  // namespace moe

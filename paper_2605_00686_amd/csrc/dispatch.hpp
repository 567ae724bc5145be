// Dispatch in its local form (paper section 2.1 step 2, section 2.3 "group
// tokens into tiles"): histogram -> exclusive scans -> stable permutation ->
// coalesced row gather, plus the tables the tile scheduler and the publish
// step read (row blocks per expert, flag numbering per destination).
#pragma once
#include "common.hpp"

namespace moe {

// Single-workgroup task.  Reads blk_hist[nPB][E] and seg_cnt[E][R] (complete),
// writes counts, offsets, blk_base, seg_begin, flag_base, dest_flag_begin,
// rb_base, rb_expert, ctrl->n_rb, ctrl->n_flags.
__device__ void plan_task(const KArgs &a, char *smem) {
    const int tid = threadIdx.x;
    const int E = a.E, R = a.R;
    int32_t *s_cnt = (int32_t *)smem;  // [E] counts, then reused
    int32_t *s_off = s_cnt + E;        // [E+1]
    int32_t *s_dest = s_off + E + 1;   // [R+1] flags per destination, then their scan
    int32_t *s_rb = s_dest + R + 1;    // [E+1]

    // per-expert totals and per-block running bases (expert-local)
    for (int e = tid; e < E; e += kThreads) {
        int run = 0;
        for (int b = 0; b < a.nPB; ++b) {
            int c = a.blk_hist[(size_t)b * E + e];
            a.blk_base[(size_t)b * E + e] = run;
            run += c;
        }
        s_cnt[e] = run;
        int sb = 0;
        for (int r = 0; r < R; ++r) {
            a.seg_begin[(size_t)e * R + r] = sb;
            sb += a.seg_cnt[(size_t)e * R + r];
        }
    }
    __syncthreads();
    if (tid == 0) {
        int run = 0, rb = 0;
        for (int e = 0; e < E; ++e) {
            s_off[e] = run;
            s_rb[e] = rb;
            run += s_cnt[e];
            rb += (s_cnt[e] + a.tl.BM - 1) / a.tl.BM;
        }
        s_off[E] = run;
        s_rb[E] = rb;
        a.ctrl->n_rb = (u32)rb;
    }
    __syncthreads();
    for (int e = tid; e <= E; e += kThreads) {
        a.offsets[e] = s_off[e];
        a.rb_base[e] = s_rb[e];
        if (e < E) {
            a.counts[e] = s_cnt[e];
            for (int i = s_rb[e]; i < s_rb[e + 1]; ++i) a.rb_expert[i] = e;
        }
    }
    for (int q = tid; q < a.nPB * E; q += kThreads) a.blk_base[q] += s_off[q % E];
    // flags: destination-major, then expert; a segment with expert-local rows
    // [b0, b0+c) touches row blocks b0/tile_m .. (b0+c-1)/tile_m
    for (int r = tid; r < R; r += kThreads) {
        int n = 0;
        for (int e = 0; e < E; ++e) {
            int c = a.seg_cnt[(size_t)e * R + r];
            if (c > 0) {
                int b0 = a.seg_begin[(size_t)e * R + r];
                n += ((b0 + c - 1) / a.tile_m - b0 / a.tile_m + 1) * a.ncb;
            }
        }
        s_dest[r] = n;
    }
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        for (int r = 0; r < R; ++r) {
            int n = s_dest[r];
            s_dest[r] = run;
            run += n;
        }
        s_dest[R] = run;
        a.ctrl->n_flags = (u32)run;
    }
    __syncthreads();
    for (int r = tid; r <= R; r += kThreads) {
        a.dest_flag_begin[r] = s_dest[r];
        if (r < R) {
            int run = s_dest[r];
            for (int e = 0; e < E; ++e) {
                a.flag_base[(size_t)r * E + e] = run;
                int c = a.seg_cnt[(size_t)e * R + r];
                if (c > 0) {
                    int b0 = a.seg_begin[(size_t)e * R + r];
                    run += ((b0 + c - 1) / a.tile_m - b0 / a.tile_m + 1) * a.ncb;
                }
            }
        }
    }
    __syncthreads();
}

// One permutation block: tokens [b*64, b*64+64).  The k experts of a token are
// distinct, so the rank of slot (t, e) among the block's slots of e is the
// number of earlier tokens of the block that chose e: a popcount on a 64-bit
// per-expert mask.  Deterministic, no arrival-order atomics.
template <typename ET>
__device__ void perm_task(const KArgs &a, int b, char *smem) {
    const int tid = threadIdx.x;
    const int E = a.E, k = a.k;
    u64 *mask = (u64 *)smem;  // [E]
    const int t0 = b * kPermBlock;
    const int nt = min(kPermBlock, a.T - t0);
    for (int e = tid; e < E; e += kThreads) mask[e] = 0ull;
    __syncthreads();
    for (int q = tid; q < nt * k; q += kThreads) {
        int e = a.idx[(size_t)t0 * k + q];
        if (e >= 0 && e < E) atomicOr(&mask[e], 1ull << (q / k));
    }
    __syncthreads();
    for (int q = tid; q < nt * k; q += kThreads) {
        const int s = t0 * k + q;
        const int tl = q / k;
        const int e = a.idx[s];
        if (e < 0 || e >= E) continue;
        const int rank = __popcll(mask[e] & ((1ull << tl) - 1ull));
        const int p = a.blk_base[(size_t)b * E + e] + rank;
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

// x_perm[p,:] = x[perm[p]/k,:] for sorted rows p = first, first+stride, ...: one
// wavefront per row, 16-byte pieces, up to four loads in flight per lane, so
// both the reads and the writes are whole contiguous rows.
__device__ void gather_rows(const KArgs &a, int first, int stride, size_t row_bytes) {
    const int lane = threadIdx.x & 63;
    const int pieces = (int)(row_bytes / 16);
    for (int p = first; p < a.N; p += stride) {
        const int s = a.perm[p];
        const uint4 *src = (const uint4 *)((const char *)a.x + (size_t)(s / a.k) * row_bytes);
        uint4 *dst = (uint4 *)((char *)a.x_perm + (size_t)p * row_bytes);
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

}  // namespace moe

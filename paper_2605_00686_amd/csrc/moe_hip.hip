// C ABI of the MoE hot path for MI355X (gfx950): argument validation, workspace
// layout, kernel selection and launches.  Declarations and contracts live in
// include/moe.h.
#include <hip/hip_runtime.h>

#include <cstring>
#include <mutex>
#include <type_traits>

#include "common.hpp"
#include "dispatch.hpp"
#include "expert.hpp"
#include "route.hpp"

namespace moe {

// ------------------------------------------------------------------ kernels
__global__ __launch_bounds__(kThreads) void k_zero(u32 *p, size_t n) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        p[i] = 0u;
}

template <typename ET>
__global__ __launch_bounds__(kThreads) void k_route(KArgs a, int do_hist) {
    extern __shared__ __align__(16) char smem[];
    route_task<ET>(a, blockIdx.x, smem, do_hist != 0);
}

__global__ __launch_bounds__(kThreads) void k_plan(KArgs a) {
    extern __shared__ __align__(16) char smem[];
    plan_task(a, smem);
}

template <typename ET>
__global__ __launch_bounds__(kThreads) void k_perm(KArgs a) {
    extern __shared__ __align__(16) char smem[];
    if (a.ctrl->error == 0) perm_task<ET>(a, blockIdx.x, smem, a.blk_base + (size_t)blockIdx.x * a.E, a.counts);
}

// standalone dispatch, short form (see block_hist_task): histograms go to blk_base, which nothing
// else reads in this form, and nothing that must be zero between calls is touched
__global__ __launch_bounds__(kThreads) void k_block_hist(KArgs a) {
    extern __shared__ __align__(16) char smem[];
    block_hist_task(a, blockIdx.x, a.blk_base, smem);
}
template <typename ET>
__global__ __launch_bounds__(kThreads) void k_block_perm(KArgs a) {
    extern __shared__ __align__(16) char smem[];
    block_perm_task<ET>(a, blockIdx.x, a.blk_base, smem);
}

__global__ __launch_bounds__(kThreads) void k_gather(KArgs a, size_t row_bytes) {
    if (a.ctrl && a.ctrl->error != 0) return;  // (no control block: the form without a workspace)
    // perm was not written if an expert is over its capacity (padded layout) or if the histogram does not account
    // for every slot (an expert id outside [0, E)): nothing is gathered then
    __shared__ int s_rows;
    if (threadIdx.x == 0) s_rows = 0;
    __syncthreads();
    int over = 0, mine = 0;
    for (int e = threadIdx.x; e < a.E; e += kThreads) {
        const int c = a.counts[e];
        mine += c;
        over |= (a.capacity > 0 && c > a.capacity) ? 1 : 0;
    }
    if (mine) atomicAdd(&s_rows, mine);
    if (__syncthreads_or(over)) return;
    if (s_rows != a.N) return;
    const int wave = (blockIdx.x * kThreads + threadIdx.x) >> 6;
    gather_rows(a, wave, (gridDim.x * kThreads) >> 6, row_bytes);
}

// Measurement aid (moe_probe_mfma): nothing but independent bf16 matrix-core instructions, one wavefront per SIMD,
// the 256 accumulator registers of the 256 x 256 GEMM tile (16 independent 32x32x16 products per round), operands
// read once from `frag` (128 bytes per lane of a wavefront, whatever the caller put there).  What this reaches is what
// the matrix cores deliver on this chip at the clock it holds under that load, with no LDS or memory traffic at all.
__global__ __launch_bounds__(kThreads, 1) void k_probe_mfma(const uint4 *frag, int iters, float *sink) {
    const int lane = threadIdx.x & 63;
    bf16x8_t fa[4], fb[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        fa[i] = __builtin_bit_cast(bf16x8_t, frag[(size_t)(i * 64 + lane)]);
        fb[i] = __builtin_bit_cast(bf16x8_t, frag[(size_t)((4 + i) * 64 + lane)]);
    }
    f32x16_t acc[4][4];
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int n = 0; n < 4; ++n)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[m][n][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int m = 0; m < 4; ++m)
#pragma unroll
            for (int n = 0; n < 4; ++n) acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[n], fa[m], acc[m][n], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int n = 0; n < 4; ++n)
#pragma unroll
            for (int v = 0; v < 16; ++v) s += acc[m][n][v];
    sink[(size_t)blockIdx.x * kThreads + threadIdx.x] = s;
}

// Measurement aid (moe_probe_stream): nothing but loads.  Every workgroup of NT threads reads `bytes_per_wg` bytes
// that start at byte (workgroup * stride) % span of `buf` and wrap inside its first `span` bytes, 1 KB per wavefront
// and instruction (16 bytes per lane, consecutive), kStreamDepth instructions per wavefront issued back to back and
// half of them awaited before the next batch.  LDS form: global_load_lds_dwordx4 into a per-wavefront ring in LDS,
// the way the GEMM main loop loads its stages; register form: global_load_dwordx4, the values folded into one word.
// What this reaches is what a CU can pull in with that many wavefronts, from HBM (span far beyond the caches), from
// the memory-side cache or from L2 (small span, stride 0), whatever else the kernel that is compared with it does.
constexpr int kStreamDepth = 8;
template <int NT, bool TO_LDS>
__global__ __launch_bounds__(NT, 1) void k_probe_stream(const char *buf, size_t span, size_t stride, size_t bytes_per_wg, u32 *sink) {
    extern __shared__ __align__(1024) char stream_lds[];
    constexpr int NW = NT / 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const size_t start = ((size_t)blockIdx.x * stride) % span;
    const size_t n_instr = bytes_per_wg / ((size_t)NW * 1024);
    u32x4_t acc = u32x4_t{0u, 0u, 0u, 0u};
    const size_t mine = (size_t)wave * 1024 + (size_t)lane * 16;
    if (TO_LDS) {
        const u32 ring = lds_offset(stream_lds) + (u32)wave * (kStreamDepth * 1024);
        for (size_t it = 0; it + kStreamDepth <= n_instr; it += kStreamDepth) {
#pragma unroll
            for (int u = 0; u < kStreamDepth; ++u) {
                const char *src = buf + (start + (it + u) * ((size_t)NW * 1024) + mine) % span;
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                             :
                             : "s"(__builtin_amdgcn_readfirstlane(ring + (u32)u * 1024)), "v"(src)
                             : "m0", "memory");
            }
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kStreamDepth / 2) : "memory");
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        acc = *(const u32x4_t *)(stream_lds + (size_t)tid * 16);
    } else {
        for (size_t it = 0; it + kStreamDepth <= n_instr; it += kStreamDepth) {
            u32x4_t r[kStreamDepth];
#pragma unroll
            for (int u = 0; u < kStreamDepth; ++u)
                r[u] = *(const u32x4_t *)(buf + (start + (it + u) * ((size_t)NW * 1024) + mine) % span);
#pragma unroll
            for (int u = 0; u < kStreamDepth; ++u) acc ^= r[u];
        }
    }
    sink[(size_t)blockIdx.x * NT + tid] = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
}

// standalone dispatch as one launch (see dispatch_fused_task); and the row movement of the histogram form by
// token (ragged layout), which moves nothing unless the histogram accounts for every slot
template <int STORE>
__global__ __launch_bounds__(kThreads) void k_dispatch_fused(KArgs a, size_t row_bytes) {
    dispatch_fused_task<STORE>(a, blockIdx.x, row_bytes);
}
template <int STORE>
__global__ __launch_bounds__(kThreads) void k_scatter(KArgs a, size_t row_bytes) {
    if (a.ctrl && a.ctrl->error != 0) return;
    if (a.offsets[a.E] != a.N) return;  // an expert id outside [0, E): perm and inv_perm were not written
    scatter_task<STORE>(a, blockIdx.x, row_bytes);
}

// standalone dispatch leaves the control block clean for the next call
__global__ __launch_bounds__(kThreads) void k_dispatch_finish(KArgs a) {
    // (one workgroup: the status must be read before the control block is cleared)
    if (threadIdx.x == 0 && a.status_dev && a.ctrl->error != 0) *a.status_dev = -(int)a.ctrl->error;
    __syncthreads();
    u32 *z = (u32 *)a.ctrl;
    const size_t n = a.zero_bytes / 4;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        z[i] = 0u;
}

template <typename ET, bool STREAM>
__global__ __launch_bounds__(kThreads) void k_combine(KArgs a) {
    combine_task<ET, false, STREAM>(a, blockIdx.x);
}

// Front tasks of the megakernel from their counter, in this order:
// [gate-weight transposition tiles | gate tasks | plan | permutation blocks].  Returns nonzero if a wait failed or
// the routing was found invalid.
template <typename ET>
__device__ __forceinline__ int front_stage(const KArgs &a, char *smem) {
    const int tid = threadIdx.x;
    Ctrl *c = a.ctrl;
    StageLds *sl = (StageLds *)(smem + a.sched_lds_off);
    const u64 t0 = kernel_start_ticks(c);
    __syncthreads();
    if (tid == 0) sl->next = (int)atomicAdd(&c->next_task, 1u);
    __syncthreads();
    int task = uniform(sl->next);
    bool seen_plan = false, seen_wgt = false, bad = false;
    // (the next task is only drawn when this one is done: there are about as many gate tasks
    // as workgroups, and drawing ahead would give the first workgroups two each)
    while (task < a.t_g1) {
        int phase;
        if (task < a.t_gate) {
            phase = 0;
            wgt_task(a, task, smem);
            sync_stores();
            if (tid == 0) {
                fence_release(0);
                atomicAdd(&c->wgt_done, 1u);
            }
#ifdef MOE_TILE_TIMING
            if (tid == 0) atomicMax(&c->dbg[46], now_ticks() - c->t0);
#endif
        } else if (task < a.t_plan) {
            phase = 0;
            if (a.t_gate > 0 && !seen_wgt) {  // the transposed gate weights are complete
                if (tid == 0) sl->ok = wait_ge(c, &c->wgt_done, (u32)a.t_gate, a.wait_ticks) ? 1 : 0;
                __syncthreads();
                seen_wgt = true;
                bad = bad || !sl->ok;
#ifdef MOE_TILE_TIMING
                if (tid == 0) atomicMax(&c->dbg[45], now_ticks() - c->t0);
#endif
            }
            if (!bad) route_task<ET>(a, task - a.t_gate, smem, true);
            sync_stores();
            if (tid == 0) {
                fence_release(0);
                atomicAdd(&c->route_done, 1u);
            }
        } else if (task < a.t_perm) {
            phase = 1;
            if (tid == 0) sl->ok = wait_ge(c, &c->route_done, (u32)a.nRT, a.wait_ticks) ? 1 : 0;
            __syncthreads();
#ifdef MOE_TILE_TIMING
            if (tid == 0) c->dbg[39] = now_ticks() - c->t0;
#endif
            if (sl->ok) plan_task(a, smem);
            sync_stores();
            if (tid == 0) {
                fence_release(0);
                __hip_atomic_store(&c->plan_done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        } else {
            phase = 2;
            if (!seen_plan) {
                if (tid == 0) sl->ok = (wait_ge(c, &c->plan_done, 1u, a.wait_ticks) && ld_relaxed_agent(&c->error) == 0) ? 1 : 0;
                __syncthreads();
                seen_plan = true;
                bad = bad || !sl->ok;
            }
            if (!bad) perm_task<ET>(a, task - a.t_perm, smem, a.blk_base + (size_t)(task - a.t_perm) * a.E, a.counts);
            sync_stores();
            if (tid == 0) {
                fence_release(0);
                atomicAdd(&c->perm_done, 1u);
            }
        }
        __syncthreads();
        if (tid == 0) {
            mark_phase_end(c, phase, t0);
            sl->next = (int)atomicAdd(&c->next_task, 1u);
        }
        __syncthreads();
        task = uniform(sl->next);
    }
    return bad ? 1 : 0;
}

// The whole layer in one persistent kernel.  Every workgroup walks through three
// stages, drawing work from counters in the control block:
//   1. front tasks, one counter, in this order: [gate tasks | plan | permutation blocks];
//   2. GEMM tiles, four kinds in turn (GEMM1 then GEMM2, big then small row blocks), each kind
//      from one list per XCD (see TileQueue): its own XCD's list first, then the others;
//   3. combine tasks, one counter.
// No wait can deadlock, whatever the grid size: a task only waits for tasks of an
// earlier kind (permutation <- plan <- gate, GEMM1 <- permutation, GEMM2 <- GEMM1,
// combine <- GEMM2), a workgroup only moves on to a later kind when every entry of the
// kinds before has been drawn, and whoever drew an entry is running it.  So the not yet finished entry of the earliest kind is always either
// running with everything it needs, or about to be drawn by a workgroup that is not
// waiting.  A workgroup draws its next entry while it works on the current one, which
// hides the counter's latency.  The kernel body itself only strings the stage
// functions together (see StageLds) and never hands out a reference to its argument
// block.
// P: tile policy (of the big tile when row blocks have two heights), PS: policy of the small tile
// (= P when there is one height).
template <class P, class PS>
__global__ __launch_bounds__(kThreads, P::MIN_WAVES) void k_megakernel(KArgs a) {
    using ET = typename P::ET;
    constexpr bool MIXED = !std::is_same<P, PS>::value;
    static_assert(P::MIN_WAVES == PS::MIN_WAVES, "one occupancy for both tile codes");
    extern __shared__ __align__(16) char smem[];
    __shared__ int s_task, s_ok, s_last;
    Ctrl *c = a.ctrl;
    const int tid = threadIdx.x;
    const KArgsAddr kargs = kernel_args_address();
    if (tid == 0) {
        atomicCAS(&c->t0, 0ull, now_ticks());
        atomicAdd(&c->stats[15], 1ull);
    }

    // ---- stage 1: gate, plan, permutation
    bool bad = front_stage<ET>(a, smem) != 0;

    // ---- wait for the plan and the permutation (and with them for every gate task); copy
    // the decode tables to LDS
    if (tid == 0) s_ok = (wait_ge(c, &c->plan_done, 1u, a.wait_ticks) && ld_relaxed_agent(&c->error) == 0) ? 1 : 0;
    __syncthreads();
    bad = bad || !s_ok;
    int n_rb = 0, n_rbs = 0;
    if (!bad) {
        n_rb = (int)c->n_rb;
        n_rbs = (int)c->n_rbs;
        if (a.tab_lds_off > 0) {  // [offsets | rb_base | rbs_base | counts | rb_expert | rbs_expert]
            int32_t *t_off = (int32_t *)(smem + a.tab_lds_off);
            int32_t *t_rbb = t_off + a.E + 1;
            int32_t *t_rsb = t_rbb + a.E + 1;
            int32_t *t_cnt = t_rsb + a.E + 1;
            int32_t *t_rbe = t_cnt + a.E + 1;
            int32_t *t_rse = t_rbe + n_rb;
            for (int i = tid; i <= a.E; i += kThreads) {
                t_off[i] = a.offsets[i];
                t_rbb[i] = a.rb_base[i];
                t_rsb[i] = a.rbs_base[i];
                t_cnt[i] = i < a.E ? a.counts[i] : 0;
            }
            for (int i = tid; i < n_rb; i += kThreads) t_rbe[i] = a.rb_expert[i];
            for (int i = tid; i < n_rbs; i += kThreads) t_rse[i] = a.rbs_expert[i];
        }
    }
    __syncthreads();
    if (tid == 0) s_ok = wait_ge(c, &c->perm_done, (u32)a.nPB, a.wait_ticks) ? 1 : 0;
    __syncthreads();
    bad = bad || !s_ok;

    if (!bad) {
        // ---- stage 2: GEMM tiles, one call per kind, this XCD's lists first
        const int home = xcd_id() % kTileQueues;
        const u32 lds = lds_offset_opaque(smem);
        // The stage functions get the address of a local of this kernel.  That keeps the compiler from
        // marking the calls as tail calls, which is what lets it drop the saving and restoring of
        // callee-saved registers in these functions (they have one caller, which keeps nothing in them):
        // some 270 registers per lane through scratch memory, per call, otherwise.
        volatile int stage_mark = 0;
        if constexpr (P::FUSED) {
            // ---- stage 2, fused: row blocks through both GEMMs, then combine
            fused_stage<P>(kargs, lds, home, n_rb, &stage_mark);
            combine_stage<ET>(a, smem);
        } else if (a.scheduler == MOE_SCHED_READY_QUEUE) {
            // ---- stages 2 and 3 from the ready queues
            ready_queue_stage<P, PS, MIXED>(a, kargs, smem, home, n_rb, n_rbs, &stage_mark);
        } else {
            MOE_TT_BEGIN();
            tile_stage<P, true, false>(kargs, lds, home, n_rb, n_rbs, -1, -1, -1, &stage_mark);
            MOE_TT(c, 20);
            if (MIXED && n_rbs > 0) tile_stage<PS, true, true>(kargs, lds, home, n_rb, n_rbs, -1, -1, -1, &stage_mark);
            MOE_TT(c, 21);
            tile_stage<P, false, false>(kargs, lds, home, n_rb, n_rbs, -1, -1, -1, &stage_mark);
            MOE_TT(c, 22);
            if (MIXED && n_rbs > 0) tile_stage<PS, false, true>(kargs, lds, home, n_rb, n_rbs, -1, -1, -1, &stage_mark);
            MOE_TT(c, 23);
#ifdef MOE_TILE_TIMING
            if (tid == 0) {
                const u64 t = now_ticks() - c->t0;
                atomicAdd(&c->dbg[14], t);
                atomicMax(&c->dbg[15], t);
            }
#endif
            // ---- stage 3: combine
            combine_stage<ET>(a, smem);
        }
    }
    // last workgroup out copies the statistics and clears the control block
    sync_stores();
    if (tid == 0) {
        fence_release(0);
        const u32 old = atomicAdd(&c->exit_count, 1u);
        s_last = (old == gridDim.x - 1) ? 1 : 0;
        if (s_last) fence_acquire(0);
    }
    __syncthreads();
    if (s_last) {
        if (a.stats) {
            if (tid < MOE_NUM_STATS) {
                u64 v = c->stats[tid];
                if (tid == 7) v = (u64)(long long)(-(int)c->error);
                if (tid >= 8 && tid <= 14) v *= 10ull;  // 100 MHz ticks -> ns
                a.stats[tid] = v;
            }
        }
        __syncthreads();
#ifdef MOE_TILE_TIMING
        // development build: the per-part tick sums follow the statistics (the caller's array has room for them)
        if (a.stats && tid < 48) a.stats[MOE_NUM_STATS + tid] = c->dbg[tid];
        __syncthreads();
#endif
        u32 *z = (u32 *)c;
        for (size_t i = tid; i < a.zero_bytes / 4; i += kThreads) z[i] = 0u;
    }
}

// --------------------------------------------------------------- host side
// The standalone dispatch runs as one launch while (slots) x (workgroups of 16 tokens) is at most this: every
// workgroup counts every slot, which hides behind the row movement up to about this much.
constexpr long long kFusedDispatchWork = 64ll << 20;
constexpr size_t kLdsBudget = 160 * 1024 - 256;  // dynamic LDS a kernel may ask for: the CU's 160 KB less the kernels' few static words
constexpr int kMaxDevices = 16;  // devices the host-side launch memo covers (others ask the runtime on every call)

static inline size_t align_up(size_t v, size_t al) { return (v + al - 1) / al * al; }

static int elem_size(int dtype) { return dtype == MOE_DT_F32 ? 4 : 2; }

// The gate is split over its reduction when there are at most kGateSplitBlocks blocks of 16 tokens,
// into at most kGateSplitTasks tasks in all.
constexpr int kGateSplitBlocks = 64, kGateSplitTasks = 256, kGateSplitMax = 16;

// LM: 256-row tiles plus a 128-row tile for short tails; FS / FM: row blocks of the fused FFN (32 / 64 rows)
enum TileKind { TK_F32 = 0, TK_LM = 1, TK_S = 3, TK_FS = 4, TK_FM = 5 };

struct Plan {
    moe_problem_t p;
    int tile_m, tile_n, N, NP, per_dest, ncb, nPB, nRT, nCT, comb_tokens, maxRB_layout;
    int kind;
    Tiling tl;
    // workspace byte offsets
    size_t o_ctrl, o_blk_hist, o_seg_cnt, o_group_counter, o_h_ready, o_dest_done, o_gate_parts, zero_bytes;
    size_t o_gate_partial;
    size_t o_rq_slots, init_zero_bytes;  // the ready queues empty themselves: zeroed by moe_workspace_init only
    int rq_cap;
    size_t o_blk_base, o_seg_begin, o_flag_base, o_dest_flag_begin, o_dest_group_begin, o_rb_base, o_rb_expert, o_rbs_base, o_rbs_expert, o_h, o_wgt, total;
};

static int make_plan(const moe_problem_t *p, Plan *pl) {
    if (!p) return MOE_ERR_INVALID_ARG;
    if (p->T < 1 || p->d < 1 || p->E < 1 || p->k < 1 || p->f < 1 || p->R < 1) return MOE_ERR_INVALID_ARG;
    if (p->k > p->E || p->T % p->R != 0) return MOE_ERR_INVALID_ARG;
    if (p->dtype != MOE_DT_F32 && p->dtype != MOE_DT_BF16) return MOE_ERR_INVALID_ARG;
    if (p->signal_mode != MOE_SIGNAL_PER_TILE && p->signal_mode != MOE_SIGNAL_PER_DEST) return MOE_ERR_INVALID_ARG;
    if (p->fence_scope != MOE_SCOPE_AGENT && p->fence_scope != MOE_SCOPE_SYSTEM) return MOE_ERR_INVALID_ARG;
    if (p->tile_m < 0 || p->tile_n < 0) return MOE_ERR_INVALID_ARG;
    if (p->group_size < 0 || (p->group_size != 0 && p->signal_mode != MOE_SIGNAL_PER_DEST)) return MOE_ERR_INVALID_ARG;
    if (p->scheduler != MOE_SCHED_STATIC && p->scheduler != MOE_SCHED_READY_QUEUE) return MOE_ERR_INVALID_ARG;
    if (p->capacity < 0) return MOE_ERR_INVALID_ARG;
    if (p->fuse_ffn != 0 && p->fuse_ffn != 1) return MOE_ERR_INVALID_ARG;
    if (p->fuse_ffn && p->scheduler != MOE_SCHED_STATIC) return MOE_ERR_INVALID_ARG;
    if ((long long)p->E * p->capacity > (1ll << 30)) return MOE_ERR_UNSUPPORTED;
    if (p->E > kMaxExperts || p->k > 32 || p->R > kMaxDest) return MOE_ERR_UNSUPPORTED;
    if ((long long)p->T * p->k > (1ll << 30)) return MOE_ERR_UNSUPPORTED;
    const int tm = p->tile_m ? p->tile_m : 128, tn = p->tile_n ? p->tile_n : 64;
    if (tm != 32 && tm != 64 && tm != 128) return MOE_ERR_UNSUPPORTED;
    if (tn != 64 && tn != 128) return MOE_ERR_UNSUPPORTED;
    // 16-byte pieces everywhere; the MFMA main loop steps K by 64, the fp32 one by 16
    const int kstep = (p->dtype == MOE_DT_BF16) ? 64 : 16;
    if (p->d % kstep != 0 || p->f % kstep != 0) return MOE_ERR_UNSUPPORTED;
    pl->p = *p;
    pl->tile_m = tm;
    pl->tile_n = tn;
    pl->N = p->T * p->k;
    pl->NP = p->capacity > 0 ? p->E * p->capacity : pl->N;  // rows of the sorted order (h, x_perm, perm)
    pl->per_dest = p->T / p->R;
    pl->ncb = (p->d + tn - 1) / tn;
    pl->nPB = (p->T + kPermBlock - 1) / kPermBlock;
    pl->nRT = (p->T + kRouteTokens - 1) / kRouteTokens;
    pl->comb_tokens = p->T >= 16384 ? 16 : p->T >= 8192 ? 8 : p->T >= 2048 ? 4 : 1;
    // the ready-queue scheduler enqueues combine tasks per destination: none may span two
    if (p->scheduler == MOE_SCHED_READY_QUEUE && pl->per_dest % pl->comb_tokens != 0) pl->comb_tokens = 1;
    pl->nCT = (p->T + pl->comb_tokens - 1) / pl->comb_tokens;
    // tile shape: the smallest row block that holds an average expert, never
    // smaller than the publish tile (a publish tile must not span two compute tiles)
    const int avg = pl->N / p->E;
    int bm;
    if (p->dtype == MOE_DT_F32) {
        pl->kind = TK_F32;
        bm = TileF32::BM;
        pl->tl.BN1 = TileF32::BN;
        pl->tl.BN2 = TileF32::BN;
    } else if (p->fuse_ffn) {
        // the fused FFN: row blocks of 32 rows for decode-sized experts, else 64; the block's h must fit the LDS
        // beside the stage buffers (checked at launch: MOE_ERR_UNSUPPORTED if it does not)
        pl->kind = (avg < 96 && tm == 32) ? TK_FS : TK_FM;
        bm = pl->kind == TK_FS ? CfgFS::BM : CfgFM::BM;
        pl->tl.BN1 = 128;
        pl->tl.BN2 = 256;
    } else {
        pl->kind = (avg >= 96 || tm > 32) ? TK_LM : TK_S;
        bm = pl->kind == TK_LM ? CfgL::BM : CfgS::BM;
        pl->tl.BN1 = 128;
        pl->tl.BN2 = 256;
    }
    if (p->fuse_ffn && p->dtype != MOE_DT_BF16) return MOE_ERR_UNSUPPORTED;
    pl->tl.BMS = pl->kind == TK_LM ? CfgM::BM : 0;
    // few rows per expert: the layer streams weights (measured: about -1 % on cfg2; +2 to 4 % on cfg3 and cfg4,
    // which have thousands of rows per expert and are bound by the matrix cores, if it were applied there)
    pl->tl.tail_with_big = avg < 512 ? 1 : 0;
    // a publish tile must lie inside one compute tile, in both directions (the fp32 tile is 64 columns wide)
    if (pl->tl.BN2 % tn != 0) return MOE_ERR_UNSUPPORTED;
    if (pl->tl.BMS % tm != 0) return MOE_ERR_UNSUPPORTED;
    if (bm % tm != 0) return MOE_ERR_UNSUPPORTED;
    pl->tl.BM = bm;
    pl->tl.NT1 = (p->f + pl->tl.BN1 - 1) / pl->tl.BN1;
    pl->tl.NT2 = (p->d + pl->tl.BN2 - 1) / pl->tl.BN2;
    pl->tl.maxRB = pl->N / bm + p->E;
    pl->maxRB_layout = pl->N / 32 + 2 * p->E;  // big plus small row blocks; the layout does not depend on the tile choice
    if ((long long)(pl->tl.maxRB + p->E) * (pl->tl.NT1 + pl->tl.NT2) > (1ll << 30)) return MOE_ERR_UNSUPPORTED;
    size_t o = 0;
    auto take = [&](size_t bytes) {
        size_t at = o;
        o = align_up(o + bytes, 256);
        return at;
    };
    pl->o_ctrl = take(sizeof(Ctrl));
    pl->o_blk_hist = take((size_t)pl->nPB * p->E * 4);
    pl->o_seg_cnt = take((size_t)p->E * p->R * 4);
    pl->o_h_ready = take((size_t)pl->maxRB_layout * 4);
    pl->o_dest_done = take((size_t)p->R * 4);
    pl->o_gate_parts = take((size_t)kGateSplitBlocks * 4);
    pl->zero_bytes = o;
    // What follows is zero between calls because its users leave it so (moe_workspace_init zeroes it
    // once).  Sizes are the largest any signal mode, group size or scheduler needs, so that the
    // layout depends on the shape of the problem only and these may change from call to call.
    // Fence groups: one counter per group, at most one group per flag (group_size 1) plus R.
    const size_t max_flags = ((size_t)(pl->N + tm - 1) / tm + (size_t)p->E * p->R) * pl->ncb;
    pl->o_group_counter = take((max_flags + p->R) * 4);
    // One ready queue per XCD, each able to hold every GEMM2 tile and every combine task (at most
    // one per token).
    pl->rq_cap = (pl->tl.maxRB + p->E) * pl->tl.NT2 + p->T;
    pl->o_rq_slots = take((size_t)kTileQueues * pl->rq_cap * 4);
    pl->init_zero_bytes = o;
    pl->o_blk_base = take((size_t)pl->nPB * p->E * 4);
    pl->o_seg_begin = take((size_t)p->E * p->R * 4);
    pl->o_flag_base = take((size_t)p->E * p->R * 4);
    pl->o_dest_flag_begin = take((size_t)(p->R + 1) * 4);
    pl->o_dest_group_begin = take((size_t)(p->R + 1) * 4);
    pl->o_rb_base = take((size_t)(p->E + 1) * 4);
    pl->o_rb_expert = take((size_t)pl->maxRB_layout * 4);
    pl->o_rbs_base = take((size_t)(p->E + 1) * 4);
    pl->o_rbs_expert = take((size_t)p->E * 4);
    pl->o_h = take((size_t)pl->NP * p->f * elem_size(p->dtype));
    // partial logits of a gate split over its reduction (few tokens only): at most kGateSplitTasks tasks
    pl->o_gate_partial = take((size_t)kGateSplitTasks * kRouteTokens * p->E * 8);
    // transposed gate weights (bf16 problems; unused when the routing is an input)
    pl->o_wgt = take(p->dtype == MOE_DT_BF16 ? (size_t)p->E * p->d * 2 : 0);
    pl->total = o;
    return MOE_OK;
}

static void fill_args(const Plan &pl, void *workspace, KArgs *a) {
    const moe_problem_t &p = pl.p;
    memset(a, 0, sizeof(*a));
    a->T = p.T; a->d = p.d; a->E = p.E; a->k = p.k; a->f = p.f; a->R = p.R;
    a->dtype = p.dtype; a->tile_m = pl.tile_m; a->tile_n = pl.tile_n;
    a->signal_mode = p.signal_mode; a->fence_scope = p.fence_scope; a->epoch = p.epoch;
    a->group_size = p.group_size;
    a->wait_ticks = p.wait_ticks ? (u64)p.wait_ticks : kWaitTicks;
    a->scheduler = p.scheduler;
    a->N = pl.N; a->NP = pl.NP; a->capacity = p.capacity; a->per_dest = pl.per_dest; a->ncb = pl.ncb;
    a->nPB = pl.nPB; a->nRT = pl.nRT; a->nCT = pl.nCT; a->comb_tokens = pl.comb_tokens;
    a->seg_from_blocks = (pl.per_dest % kPermBlock == 0) ? 1 : 0;
    a->disp_tokens = scatter_tokens(p.T);
    a->tl = pl.tl;
    a->t_gate = 0;  // the megakernel adds the transposition tasks when it has a gate to compute
    a->t_plan = pl.nRT;
    a->t_perm = a->t_plan + 1;
    a->t_g1 = a->t_perm + pl.nPB;
    a->t_end = a->t_g1 + (pl.tl.maxRB + p.E) * (pl.tl.NT1 + pl.tl.NT2) + pl.nCT;
    char *ws = (char *)workspace;
    if (ws) {
        a->ctrl = (Ctrl *)(ws + pl.o_ctrl);
        a->blk_hist = (int32_t *)(ws + pl.o_blk_hist);
        a->seg_cnt = (int32_t *)(ws + pl.o_seg_cnt);
        a->group_counter = (u32 *)(ws + pl.o_group_counter);
        a->h_ready = (u32 *)(ws + pl.o_h_ready);
        if (p.scheduler == MOE_SCHED_READY_QUEUE) {
            a->dest_done = (u32 *)(ws + pl.o_dest_done);
            a->rq_slots = (u32 *)(ws + pl.o_rq_slots);
            a->rq_cap = pl.rq_cap;
        }
        a->blk_base = (int32_t *)(ws + pl.o_blk_base);
        a->seg_begin = (int32_t *)(ws + pl.o_seg_begin);
        a->flag_base = (int32_t *)(ws + pl.o_flag_base);
        a->dest_flag_begin = (int32_t *)(ws + pl.o_dest_flag_begin);
        a->dest_group_begin = (int32_t *)(ws + pl.o_dest_group_begin);
        a->rb_base = (int32_t *)(ws + pl.o_rb_base);
        a->rb_expert = (int32_t *)(ws + pl.o_rb_expert);
        a->rbs_base = (int32_t *)(ws + pl.o_rbs_base);
        a->rbs_expert = (int32_t *)(ws + pl.o_rbs_expert);
        a->h = ws + pl.o_h;
        a->zero_bytes = pl.zero_bytes;
    }
}

static size_t plan_smem(const Plan &pl) { return plan_smem_bytes(pl.p.E, pl.p.R, pl.nPB); }

static int check_ws(const void *ws) {
    if (!ws || ((uintptr_t)ws & 255u)) return MOE_ERR_WORKSPACE;
    return MOE_OK;
}

static int hip_ok(hipError_t e) { return e == hipSuccess ? MOE_OK : MOE_ERR_HIP; }

// Allow `kernel` `bytes` of dynamic LDS on the current device.  The limit of a kernel is only ever raised, and
// what it was raised to is remembered per (device, kernel), so that a call which needs no more than an earlier
// one asks the runtime nothing (a host-side memo: no device state, nothing a call can observe).
static int set_smem_raw(const void *kernel, size_t bytes) {
    if (bytes > 160 * 1024) return MOE_ERR_UNSUPPORTED;
    if (bytes <= 48 * 1024) return MOE_OK;
    struct Entry {
        int dev;
        const void *kernel;
        size_t limit;
    };
    static std::mutex lock;
    static Entry table[64];
    static int n = 0;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return MOE_ERR_HIP;
    std::lock_guard<std::mutex> g(lock);
    Entry *hit = nullptr;
    for (int i = 0; i < n; ++i)
        if (table[i].dev == dev && table[i].kernel == kernel) hit = &table[i];
    if (hit && hit->limit >= bytes) return MOE_OK;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) return MOE_ERR_HIP;
    if (hit)
        hit->limit = bytes;
    else if (n < 64)
        table[n++] = Entry{dev, kernel, bytes};
    return MOE_OK;
}
template <class K>
static int set_smem(K kernel, size_t bytes) {
    return set_smem_raw((const void *)kernel, bytes);
}

template <class P, class PS>
static int launch_mega(const Plan &pl, const KArgs &a_in, hipStream_t st) {
    size_t smem = tile_smem_bytes<P>();
    if (tile_smem_bytes<PS>() > smem) smem = tile_smem_bytes<PS>();
    KArgs a = a_in;
    if (P::FUSED) {  // the row block's h, behind the GEMM region and the publish bookkeeping (the gate's LDS is free by then)
        a.fused = 1;
        a.fused_h_off = (int)align_up(smem, 16);
        smem = a.fused_h_off + (size_t)P::BM * pl.p.f * elem_size(pl.p.dtype);
        if (smem + sizeof(StageLds) + 16 > kLdsBudget) return MOE_ERR_UNSUPPORTED;
    }
    const size_t rsm = route_smem_bytes(pl.p.E, elem_size(pl.p.dtype));
    if (a_in.Wg && rsm > smem) smem = rsm;
    if (a_in.WgT && screen_smem_bytes(pl.p.E) > smem) smem = screen_smem_bytes(pl.p.E);
    if (plan_smem(pl) > smem) smem = plan_smem(pl);
    // decode tables live behind everything else, for the life of the workgroup
    const size_t tab_bytes = (size_t)(4 * (pl.p.E + 1) + pl.tl.maxRB + pl.p.E) * 4;
    a.tab_lds_off = 0;
    if (tab_bytes <= 6 * 1024 && smem + tab_bytes + sizeof(StageLds) + 16 <= kLdsBudget) {  // small enough that two workgroups of the 128-row tile still share a CU
        a.tab_lds_off = (int)align_up(smem, 16);
        smem = a.tab_lds_off + tab_bytes;
    }
    a.sched_lds_off = (int)align_up(smem, 16);
    smem = a.sched_lds_off + sizeof(StageLds);
    auto kern = k_megakernel<P, PS>;
    int rc = set_smem(kern, smem);
    if (rc) return rc;
    // The CU count and the occupancy of this kernel are asked for once per device and LDS size (a host-side memo
    // of what the runtime answered, like the one in set_smem_raw).
    struct Memo {
        size_t smem;
        int cus, per_cu;
    };
    static std::mutex memo_lock;
    static Memo memo[kMaxDevices][4];
    static int memo_n[kMaxDevices];
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess) return MOE_ERR_HIP;
    const bool memoised = dev >= 0 && dev < kMaxDevices;
    bool found = false;
    if (memoised) {
        std::lock_guard<std::mutex> g(memo_lock);
        for (int i = 0; i < memo_n[dev]; ++i)
            if (memo[dev][i].smem == smem) cus = memo[dev][i].cus, per_cu = memo[dev][i].per_cu, found = true;
    }
    if (!found) {
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return MOE_ERR_HIP;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, kThreads, smem) != hipSuccess) return MOE_ERR_HIP;
        std::lock_guard<std::mutex> g(memo_lock);
        if (memoised && memo_n[dev] < 4) memo[dev][memo_n[dev]++] = Memo{smem, cus, per_cu};
    }
    if (per_cu < 1) return MOE_ERR_UNSUPPORTED;
    if (per_cu > 2) per_cu = 2;
    long long grid = (long long)cus * per_cu;
    if (grid > a.t_end) grid = a.t_end;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kThreads), smem, st, a);
    return hip_ok(hipGetLastError());
}

}  // namespace moe

using namespace moe;

// ---- scratch for callers that cannot allocate (see moe_dispatch_noalloc): one array per GPU the library runs on,
// held until the process ends.  In host code the array's name is only a handle: the device address comes from
// hipGetSymbolAddress, once per device with that device current, and only that address is handed to kernels.
constexpr size_t kStaticScratchBytes = 64 * 1024;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

static int static_scratch_address(unsigned char **out) {
    static std::mutex lock;
    static unsigned char *addr[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return MOE_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return MOE_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> g(lock);
    if (!addr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return MOE_ERR_HIP;
        addr[dev] = (unsigned char *)ptr;
    }
    *out = addr[dev];
    return MOE_OK;
}

extern "C" {

const char *moe_status_string(int s) {
    switch (s) {
        case MOE_OK: return "ok";
        case MOE_ERR_INVALID_ARG: return "invalid argument";
        case MOE_ERR_UNSUPPORTED: return "unsupported problem";
        case MOE_ERR_WORKSPACE: return "workspace missing or misaligned";
        case MOE_ERR_NOT_READY: return "a ready flag was not at the expected epoch";
        case MOE_ERR_HIP: return "HIP runtime error";
        case MOE_ERR_TIMEOUT: return "a bounded in-kernel wait expired";
        case MOE_ERR_BAD_ROUTING: return "expert id outside [0, E)";
        case MOE_ERR_CAPACITY: return "an expert received more rows than the capacity";
        default: return "unknown status";
    }
}

size_t moe_workspace_bytes(const moe_problem_t *p) {
    Plan pl;
    if (make_plan(p, &pl) != MOE_OK) return 0;
    return pl.total;
}

size_t moe_num_flags(const moe_problem_t *p) {
    Plan pl;
    if (make_plan(p, &pl) != MOE_OK) return 0;
    // a segment of c rows touches at most c/tile_m + 1 row blocks; there are E*R segments
    return ((size_t)(pl.N + pl.tile_m - 1) / pl.tile_m + (size_t)p->E * p->R) * pl.ncb;  // (make_plan sizes the group counters with the same bound)
}

int moe_workspace_init(const moe_problem_t *p, void *workspace, void *stream) {
    Plan pl;
    int rc = make_plan(p, &pl);
    if (rc) return rc;
    if ((rc = check_ws(workspace))) return rc;
    hipLaunchKernelGGL(k_zero, dim3(64), dim3(kThreads), 0, (hipStream_t)stream, (u32 *)workspace, pl.init_zero_bytes / 4);
    return hip_ok(hipGetLastError());
}

int moe_route(const moe_problem_t *p, const void *x, const void *Wg, const float *gate_bias, int32_t *topk_idx,
              float *topk_w, void *stream) {
    Plan pl;
    int rc = make_plan(p, &pl);
    if (rc) return rc;
    if (!x || !Wg || !topk_idx || !topk_w) return MOE_ERR_INVALID_ARG;
    KArgs a;
    fill_args(pl, nullptr, &a);
    a.x = x; a.Wg = Wg; a.bias = gate_bias; a.idx = topk_idx; a.w = topk_w;
    const size_t smem = route_smem_bytes(p->E, elem_size(p->dtype));
    hipStream_t st = (hipStream_t)stream;
    if (p->dtype == MOE_DT_F32) {
        if ((rc = set_smem(k_route<float>, smem))) return rc;
        hipLaunchKernelGGL(k_route<float>, dim3(pl.nRT), dim3(kThreads), smem, st, a, 0);
    } else {
        if ((rc = set_smem(k_route<bf16_t>, smem))) return rc;
        hipLaunchKernelGGL(k_route<bf16_t>, dim3(pl.nRT), dim3(kThreads), smem, st, a, 0);
    }
    return hip_ok(hipGetLastError());
}

// The launches of a dispatch, shared by moe_dispatch (scratch in the caller's workspace) and
// moe_dispatch_noalloc (scratch in this library's static device array).  `short_only`: the form that needs the
// control block and the plan's tables is not available.
static int dispatch_launches(const Plan &pl, const KArgs &a, bool short_only, hipStream_t st) {
    const moe_problem_t *p = &pl.p;
    int rc;
    const size_t row_bytes = (size_t)p->d * elem_size(p->dtype);
    int ggrid = (pl.NP + 3) / 4;  // gather: one wavefront per row while rows last
    if (ggrid > 8192) ggrid = 8192;
    // rows that do not fit the 256 MB memory-side cache are stored past it; others are written through
    const bool past_cache = (size_t)pl.NP * row_bytes > ((size_t)192 << 20);
    const int sgrid = (p->T + a.disp_tokens - 1) / a.disp_tokens;
    // rows by token (read once, stored k times): ragged layout; the padded layout's histogram form keeps the gather
    // by sorted position, which also zeroes the unused rows
    auto move_rows = [&]() {
        if (!a.x_perm) return;
        if (p->capacity > 0)
            hipLaunchKernelGGL(k_gather, dim3(ggrid), dim3(kThreads), 0, st, a, row_bytes);
        else if (past_cache)
            hipLaunchKernelGGL(k_scatter<1>, dim3(sgrid), dim3(kThreads), 0, st, a, row_bytes);
        else
            hipLaunchKernelGGL(k_scatter<0>, dim3(sgrid), dim3(kThreads), 0, st, a, row_bytes);
    };
    if ((long long)pl.N * sgrid <= kFusedDispatchWork) {
        // one launch: every workgroup counts all N slots itself (no scratch at all)
        if (past_cache)
            hipLaunchKernelGGL(k_dispatch_fused<1>, dim3(sgrid), dim3(kThreads), 0, st, a, row_bytes);
        else
            hipLaunchKernelGGL(k_dispatch_fused<0>, dim3(sgrid), dim3(kThreads), 0, st, a, row_bytes);
        return hip_ok(hipGetLastError());
    }
    const size_t bsmem = block_perm_smem_bytes(p->E, pl.nPB);
    if (bsmem <= 64 * 1024) {
        // short form: per-block histograms, then every block derives its own base positions from all of
        // them (no single-workgroup plan, whose tile and flag tables a dispatch alone does not need)
        hipLaunchKernelGGL(k_block_hist, dim3(pl.nPB), dim3(kThreads), (size_t)p->E * 8, st, a);
        if (p->dtype == MOE_DT_F32) {
            if ((rc = set_smem(k_block_perm<float>, bsmem))) return rc;
            hipLaunchKernelGGL(k_block_perm<float>, dim3(pl.nPB), dim3(kThreads), bsmem, st, a);
        } else {
            if ((rc = set_smem(k_block_perm<bf16_t>, bsmem))) return rc;
            hipLaunchKernelGGL(k_block_perm<bf16_t>, dim3(pl.nPB), dim3(kThreads), bsmem, st, a);
        }
        move_rows();
        return hip_ok(hipGetLastError());
    }
    if (short_only) return MOE_ERR_UNSUPPORTED;
    const size_t psmem = plan_smem(pl);
    if ((rc = set_smem(k_plan, psmem))) return rc;
    // histogram (gate task without the gate), plan, permutation, row gather, clean-up
    if (p->dtype == MOE_DT_F32) {
        hipLaunchKernelGGL(k_route<float>, dim3(pl.nRT), dim3(kThreads), (size_t)p->E * 4, st, a, 1);
        hipLaunchKernelGGL(k_plan, dim3(1), dim3(kThreads), psmem, st, a);
        hipLaunchKernelGGL(k_perm<float>, dim3(pl.nPB), dim3(kThreads), (size_t)p->E * 8, st, a);
    } else {
        hipLaunchKernelGGL(k_route<bf16_t>, dim3(pl.nRT), dim3(kThreads), (size_t)p->E * 4, st, a, 1);
        hipLaunchKernelGGL(k_plan, dim3(1), dim3(kThreads), psmem, st, a);
        hipLaunchKernelGGL(k_perm<bf16_t>, dim3(pl.nPB), dim3(kThreads), (size_t)p->E * 8, st, a);
    }
    move_rows();
    hipLaunchKernelGGL(k_dispatch_finish, dim3(1), dim3(kThreads), 0, st, a);
    return hip_ok(hipGetLastError());
}

int moe_dispatch(const moe_problem_t *p, const void *x, const int32_t *topk_idx, int32_t *counts, int32_t *offsets,
                 int32_t *perm, int32_t *inv_perm, void *x_perm, int32_t *status_dev, void *workspace, void *stream) {
    Plan pl;
    int rc = make_plan(p, &pl);
    if (rc) return rc;
    if (!topk_idx || !counts || !offsets || !perm || !inv_perm) return MOE_ERR_INVALID_ARG;
    if (x_perm && !x) return MOE_ERR_INVALID_ARG;
    if ((rc = check_ws(workspace))) return rc;
    KArgs a;
    fill_args(pl, workspace, &a);
    a.x = x; a.idx = const_cast<int32_t *>(topk_idx);
    a.counts = counts; a.offsets = offsets; a.perm = perm; a.inv_perm = inv_perm; a.x_perm = x_perm;
    a.status_dev = status_dev;
    return dispatch_launches(pl, a, false, (hipStream_t)stream);
}

int moe_dispatch_noalloc(const moe_problem_t *p, const void *x, const int32_t *topk_idx, int32_t *counts,
                         int32_t *offsets, int32_t *perm, int32_t *inv_perm, void *x_perm, int32_t *status_dev,
                         void *stream) {
    Plan pl;
    int rc = make_plan(p, &pl);
    if (rc) return rc;
    if (!topk_idx || !counts || !offsets || !perm || !inv_perm) return MOE_ERR_INVALID_ARG;
    if (x_perm && !x) return MOE_ERR_INVALID_ARG;
    // the block histograms, the only scratch of the short form, must fit the static array
    if ((size_t)pl.nPB * p->E * 4 > kStaticScratchBytes) return MOE_ERR_UNSUPPORTED;
    unsigned char *scratch_dev = nullptr;
    if ((rc = static_scratch_address(&scratch_dev))) return rc;
    KArgs a;
    fill_args(pl, nullptr, &a);  // no workspace: no control block, no plan tables
    a.blk_base = (int32_t *)scratch_dev;
    a.x = x; a.idx = const_cast<int32_t *>(topk_idx);
    a.counts = counts; a.offsets = offsets; a.perm = perm; a.inv_perm = inv_perm; a.x_perm = x_perm;
    a.status_dev = status_dev;
    return dispatch_launches(pl, a, true, (hipStream_t)stream);
}

int moe_megakernel_forward(const moe_problem_t *p, const void *x, const void *Wg, const float *gate_bias,
                           const void *W1, const void *W3, const void *W2, int32_t *topk_idx, float *topk_w,
                           int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv_perm, int32_t *slot_flag,
                           void *staging, uint32_t *flags, void *out, uint64_t *stats, void *workspace,
                           void *stream) {
    Plan pl;
    int rc = make_plan(p, &pl);
    if (rc) return rc;
    if (!x || !W1 || !W3 || !W2 || !topk_idx || !topk_w || !counts || !offsets || !perm || !inv_perm || !slot_flag ||
        !staging || !flags || !out)
        return MOE_ERR_INVALID_ARG;
    if (p->epoch == 0) return MOE_ERR_INVALID_ARG;
    if ((rc = check_ws(workspace))) return rc;
    KArgs a;
    fill_args(pl, workspace, &a);
    a.x = x; a.Wg = Wg; a.bias = gate_bias; a.W1 = W1; a.W3 = W3; a.W2 = W2;
    a.idx = topk_idx; a.w = topk_w; a.counts = counts; a.offsets = offsets; a.perm = perm; a.inv_perm = inv_perm;
    a.slot_flag = slot_flag; a.staging = staging; a.flags = flags; a.out = out;
    a.stats = (u64 *)stats;
    // few tokens (at most kGateSplitBlocks blocks of 16): split every gate task over the reduction, so that
    // the gate runs on all workgroups instead of a handful
    int S = 1;
    if (Wg && pl.nRT <= kGateSplitBlocks) {
        S = kGateSplitTasks / pl.nRT;
        if (S > kGateSplitMax) S = kGateSplitMax;
        if (S > route_max_slices(p->d)) S = route_max_slices(p->d);
    }
    if (S > 1) {
        const int extra = pl.nRT * (S - 1);
        a.gate_split = S;
        a.nRT = pl.nRT * S;
        a.gate_partial = (double *)((char *)workspace + pl.o_gate_partial);
        a.gate_parts = (u32 *)((char *)workspace + pl.o_gate_parts);
        a.t_plan += extra; a.t_perm += extra; a.t_g1 += extra; a.t_end += extra;
    } else if (Wg && p->dtype == MOE_DT_BF16 && p->E >= 64) {
        // bf16 gate with one task or more per workgroup: screen on the bf16 matrix cores, exact fp64 logits for
        // the candidates only; this needs the gate weights transposed, which the first front tasks of the kernel write
        a.WgT = (char *)workspace + pl.o_wgt;
        const int ntt = wgt_tasks(p->d, p->E);
        a.t_gate = ntt;
        a.t_plan += ntt; a.t_perm += ntt; a.t_g1 += ntt; a.t_end += ntt;
    }
    hipStream_t st = (hipStream_t)stream;
    switch (pl.kind) {
        case TK_F32: return launch_mega<F32Policy, F32Policy>(pl, a, st);
        case TK_LM: return launch_mega<Bf16Policy<CfgL>, Bf16Policy<CfgM>>(pl, a, st);
        case TK_FS: return launch_mega<FusedPolicy<CfgFS>, FusedPolicy<CfgFS>>(pl, a, st);
        case TK_FM: return launch_mega<FusedPolicy<CfgFM>, FusedPolicy<CfgFM>>(pl, a, st);
        default: return launch_mega<Bf16Policy<CfgS>, Bf16Policy<CfgS>>(pl, a, st);
    }
}

int moe_probe_stream(const void *buf, size_t span_bytes, size_t stride_bytes, size_t bytes_per_workgroup, int32_t workgroups,
                     int32_t wavefronts, int32_t to_lds, uint32_t *sink, void *stream) {
    if (!buf || !sink || workgroups < 1 || workgroups > 65536) return MOE_ERR_INVALID_ARG;
    if (wavefronts != 4 && wavefronts != 8 && wavefronts != 16) return MOE_ERR_INVALID_ARG;
    if (to_lds != 0 && to_lds != 1) return MOE_ERR_INVALID_ARG;
    // every piece is 16 bytes at a multiple of 16 below span_bytes
    if (span_bytes < 16 * 1024 || span_bytes % 16 != 0 || stride_bytes % 16 != 0 || bytes_per_workgroup < 1) return MOE_ERR_INVALID_ARG;
    // the whole LDS of a CU minus a margin: one workgroup per CU, whatever its size
    const size_t smem = 128 * 1024;
    hipStream_t st = (hipStream_t)stream;
    const char *b = (const char *)buf;
    int rc;
#define MOE_STREAM_CASE(NT, L)                                                                                          \
    if (wavefronts * 64 == NT && to_lds == L) {                                                                         \
        if ((rc = set_smem(k_probe_stream<NT, L != 0>, smem))) return rc;                                               \
        hipLaunchKernelGGL((k_probe_stream<NT, L != 0>), dim3(workgroups), dim3(NT), smem, st, b, span_bytes, stride_bytes, \
                           bytes_per_workgroup, sink);                                                                  \
    }
    MOE_STREAM_CASE(256, 0) MOE_STREAM_CASE(256, 1) MOE_STREAM_CASE(512, 0) MOE_STREAM_CASE(512, 1)
    MOE_STREAM_CASE(1024, 0) MOE_STREAM_CASE(1024, 1)
#undef MOE_STREAM_CASE
    return hip_ok(hipGetLastError());
}

int moe_probe_mfma(const void *frag, int32_t iters, int32_t workgroups, float *sink, void *stream) {
    if (!frag || !sink || iters < 1 || workgroups < 1 || workgroups > 65536) return MOE_ERR_INVALID_ARG;
    hipLaunchKernelGGL(k_probe_mfma, dim3(workgroups), dim3(kThreads), 0, (hipStream_t)stream, (const uint4 *)frag, iters, sink);
    return hip_ok(hipGetLastError());
}

int moe_combine(const moe_problem_t *p, const void *staging, const uint32_t *flags, const int32_t *slot_flag,
                const float *topk_w, void *out, int32_t *status_dev, void *stream) {
    Plan pl;
    int rc = make_plan(p, &pl);
    if (rc) return rc;
    if (!staging || !topk_w || !out) return MOE_ERR_INVALID_ARG;
    if ((slot_flag != nullptr) != (flags != nullptr)) return MOE_ERR_INVALID_ARG;
    KArgs a;
    fill_args(pl, nullptr, &a);
    a.staging = const_cast<void *>(staging);
    a.flags = const_cast<uint32_t *>(flags);
    a.slot_flag = const_cast<int32_t *>(slot_flag);
    a.w = const_cast<float *>(topk_w);
    a.out = out;
    a.status_dev = status_dev;
    hipStream_t st = (hipStream_t)stream;
    // rows that do not fit the 256 MB last-level cache are streamed past it
    const bool past_cache = (size_t)pl.N * p->d * elem_size(p->dtype) > ((size_t)192 << 20);
    if (p->dtype == MOE_DT_F32) {
        if (past_cache)
            hipLaunchKernelGGL((k_combine<float, true>), dim3(pl.nCT), dim3(kThreads), 0, st, a);
        else
            hipLaunchKernelGGL((k_combine<float, false>), dim3(pl.nCT), dim3(kThreads), 0, st, a);
    } else {
        if (past_cache)
            hipLaunchKernelGGL((k_combine<bf16_t, true>), dim3(pl.nCT), dim3(kThreads), 0, st, a);
        else
            hipLaunchKernelGGL((k_combine<bf16_t, false>), dim3(pl.nCT), dim3(kThreads), 0, st, a);
    }
    return hip_ok(hipGetLastError());
}

}  // extern "C"

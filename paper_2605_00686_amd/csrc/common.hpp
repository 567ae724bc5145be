// Shared device-side definitions: kernel argument block, workspace layout,
// bounded waits and scoped fences.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/moe.h"

namespace moe {

typedef unsigned long long u64;
typedef uint32_t u32;
typedef unsigned short bf16_t;  // raw bf16 bits
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) u32 u32x4_t;  // 16 bytes in registers

constexpr int kThreads = 256;       // every kernel here runs 4 wavefronts per workgroup
constexpr int kPermBlock = 64;      // tokens per permutation block (one bit each in a 64-bit mask)
constexpr int kRouteTokens = 16;    // tokens per gate task
constexpr int kMaxExperts = 256;    // gate / plan limits
constexpr int kMaxDest = 1024;
constexpr u64 kWaitTicks = 400000000ull;  // 4 s of the 100 MHz wall clock: default bound of every in-kernel wait
// (the bound a call uses is KArgs::wait_ticks, from moe_problem_t::wait_ticks: tests of the time-out path set it to
// almost nothing, so that the waits give up, the error spreads and every workgroup leaves in the ordinary way)

// Control block at the start of the workspace.  All zero between calls: the
// last workgroup to leave a kernel clears what the kernel dirtied.
struct Ctrl {
    u32 next_task;   // persistent scheduler: next task to hand out
    u32 route_done;  // gate tasks finished
    u32 plan_done;   // 1 once offsets / tables are valid
    u32 perm_done;   // permutation blocks finished
    u32 exit_count;  // workgroups that left the kernel
    u32 error;       // first device status (moe_status_t as positive number), 0 = ok
    u32 n_rb;        // (big) row blocks in use, all experts
    u32 n_flags;     // publish tiles / flags in use
    u32 tile_next[4][8];  // tile queues, [GEMM1 big, GEMM1 small, GEMM2 big, GEMM2 small] x XCD: next entry to hand out
    u32 comb_next;     // next combine task
    u32 wgt_done;      // gate-weight transposition tasks finished
    u32 n_rbs;         // small row blocks in use (mixed tile heights), all experts
    u32 pad[5];
    u32 rq_head[8];    // ready queues, one per XCD: next entry to take ...
    u32 rq_tail[8];    // ... and next free entry
    u64 t0;          // wall-clock tick of the first task drawn
    u64 stats[MOE_NUM_STATS];
#ifdef MOE_TILE_TIMING
    u64 dbg[48];  // development build only: time spent in the parts of a tile, summed over tiles
#endif
};

// GEMM tiling chosen on the host.
struct Tiling {
    int BM;     // rows of a compute tile (multiple of tile_m); with mixed heights: of the big tile
    int BMS;    // mixed heights: rows of the small tile that takes an expert's last rows when they fit, 0 = one height
    int BN1;    // h columns per GEMM1 tile
    int BN2;    // y columns per GEMM2 tile
    int NT1;    // ceil(f / BN1)
    int NT2;    // ceil(d / BN2)
    int maxRB;  // upper bound on row blocks: N / BM + E
    int tail_with_big;  // mixed heights: only experts without a big block get a small one (see the plan)
};

// Everything a kernel needs, passed by value.
struct KArgs {
    int T, d, E, k, f, R;
    int dtype, tile_m, tile_n, signal_mode, fence_scope;
    int group_size;  // flags per fence group of the per-destination mode, 0 = all flags of a destination
    int scheduler;   // moe_scheduler_t
    int gate_split;  // gate tasks per block of 16 tokens: each takes a slice of the reduction (1 = the whole)
    int capacity;    // rows every expert owns in the sorted order, 0 = ragged layout (see moe_problem_t)
    int NP;          // rows of the sorted order: N (ragged) or E * capacity
    u32 epoch;
    u64 wait_ticks;  // bound of every in-kernel wait, in ticks of the 100 MHz wall clock
    int N, per_dest, ncb;  // slots, tokens per destination, column blocks per row
    int nPB, nRT, nCT;     // permutation blocks, gate tasks, combine tasks
    int comb_tokens;       // tokens per combine task
    int disp_tokens;       // tokens per workgroup of the standalone dispatch's row movement
    int fused;             // moe_problem_t::fuse_ffn: a workgroup takes a row block through both GEMMs, h in LDS
    int fused_h_off;       // ... LDS offset of that h buffer [row block rows][f]
    int seg_from_blocks;   // destinations are whole permutation blocks: the plan derives seg_cnt from blk_hist
    Tiling tl;
    // front task ranges of the persistent scheduler: [gate-weight transposition | route | plan |
    // perm), then the tile queues and the combine tasks; t_end bounds the useful number of
    // workgroups
    int t_gate, t_plan, t_perm, t_g1, t_end;
    // caller tensors
    const void *x, *Wg;
    const float *bias;
    const void *W1, *W3, *W2;
    int32_t *idx;
    float *w;
    int32_t *counts, *offsets, *perm, *inv_perm, *slot_flag;
    void *staging;
    u32 *flags;
    void *out;
    u64 *stats;
    void *x_perm;
    int32_t *status_dev;
    // workspace
    Ctrl *ctrl;
    int32_t *blk_hist;         // [nPB][E] slots of block b routed to e
    int32_t *blk_base;         // [nPB][E] sorted position of block b's first slot of e
    int32_t *seg_cnt;          // [E][R]
    int32_t *seg_begin;        // [E][R] expert-local first row of (e, r)
    int32_t *flag_base;        // [R][E]
    int32_t *dest_flag_begin;  // [R+1]
    int32_t *dest_group_begin; // [R+1] first fence group of destination r
    u32 *group_counter;        // [fence groups] publish tiles written so far (PER_DEST)
    int32_t *rb_base;          // [E+1] first row block of expert e
    int32_t *rb_expert;        // [maxRB]
    int32_t *rbs_base;         // [E+1] first small row block of expert e (each expert has at most one)
    int32_t *rbs_expert;       // [E]
    u32 *h_ready;              // [maxRB] GEMM1 tiles finished per row block
    void *h;                   // [N][f]
    void *WgT;                 // [E][d] transposed gate weights (bf16 problems with a gate), else NULL
    double *gate_partial;      // [blocks][gate_split][16][E] partial logits of the split gate
    u32 *gate_parts;           // [blocks] slices finished per block of 16 tokens
    u32 *dest_done;            // [R] flags stored so far per destination (ready-queue scheduler), else NULL
    u32 *rq_slots;             // [8][rq_cap] ready-queue entries, 0 = empty (ready-queue scheduler), else NULL
    int rq_cap;                // entries per ready queue: all GEMM2 tiles plus all combine tasks
    size_t zero_bytes;         // bytes from ctrl that must be zero between calls
    int tab_lds_off;           // megakernel: LDS offset of the cached decode tables, 0 = none
    int sched_lds_off;         // megakernel: LDS offset of the task loops' broadcast slots (StageLds)
};

__device__ __forceinline__ u64 now_ticks() { return wall_clock64(); }

__device__ __forceinline__ void set_error(Ctrl *c, int status) {
    atomicCAS(&c->error, 0u, (u32)(-status));
}

__device__ __forceinline__ u32 ld_relaxed_agent(const u32 *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ u32 ld_relaxed(const u32 *p, int system_scope) {
    return system_scope ? __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM)
                        : __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_relaxed(u32 *p, u32 v, int system_scope) {
    if (system_scope)
        __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    else
        __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void fence_release(int system_scope) {
    if (system_scope)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "");
    else
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
}
__device__ __forceinline__ void fence_acquire(int system_scope) {
    if (system_scope)
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "");
    else
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
}

// 16-byte store of tile results (h, staging) that workgroups on other XCDs will read: written
// through to memory.  An ordinary store would leave the line dirty in this XCD's L2 until the
// release fence that follows the tile writes back everything dirty in that L2 at once, the other
// workgroups' half-written tiles included; with write-through stores the fence finds little to do
// (measured: 1.5 % of the whole layer on the two large workloads).  The instruction is written out
// because no builtin sets these cache-policy bits on a 16-byte store; every caller follows its
// stores with sync_stores(), which waits for them.
// The s_nop belongs to the store: a vector store of more than 8 bytes reads its data registers for a few cycles
// after it issues, and a vector ALU instruction that overwrites one of them in the very next slots changes what
// the later lanes store.  For its own stores the compiler keeps that distance; it cannot see into this statement
// and may reuse the registers at once (seen in a variant that stored accumulators back to back: the upper lanes
// of a 16-byte piece stored the next piece's address bits).
__device__ __forceinline__ void store_tile16(char *p, const uint4 &v) {
    const u32x4_t w = {v.x, v.y, v.z, v.w};
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 1" ::"v"(p), "v"(w));
}

// Workgroup barrier that also waits for this wavefront's outstanding global
// stores.  __syncthreads() alone only drains LDS traffic; a store still in
// flight when ANOTHER wavefront of the workgroup issues the release fence would
// miss that fence's cache write-back and stay invisible to other XCDs.
__device__ __forceinline__ void sync_stores() {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
}

// Spin until *p >= target (agent scope), bounded by the wall clock and by the
// global error flag so that a broken dependency drains the grid instead of
// hanging it.  Called by one thread; returns false on time-out; `limit` is the
// bound in wall-clock ticks.  A successful wait ends with an agent-scope acquire
// (which invalidates this CU's and this XCD's non-coherent cache lines: what the
// memory model asks for data written on another XCD; an acquire that kept the L2
// measured within 0.6 % of this one on every workload).
__device__ __forceinline__ bool wait_ge(Ctrl *c, const u32 *p, u32 target, u64 limit) {
    if (ld_relaxed_agent(p) >= target) {
        fence_acquire(0);
        return true;
    }
    const u64 t0 = now_ticks();
    int spins = 0;
    bool ok = true;
    while (true) {
        if (ld_relaxed_agent(p) >= target) break;
        __builtin_amdgcn_s_sleep(2);
        if ((++spins & 63) == 0) {
            if (ld_relaxed_agent(&c->error) != 0) {
                ok = false;
                break;
            }
            if (now_ticks() - t0 > limit) {
                set_error(c, MOE_ERR_TIMEOUT);
                atomicAdd(&c->stats[6], 1ull);
                ok = false;
                break;
            }
        }
    }
    atomicAdd(&c->stats[14], now_ticks() - t0);
    if (ok) fence_acquire(0);
    return ok;
}

// phase bookkeeping for the in-kernel timeline (ticks since the first task)
__device__ __forceinline__ u64 kernel_start_ticks(Ctrl *c) {
    return __hip_atomic_load(&c->t0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// t0 = kernel_start_ticks(), read once per stage: it is final before any task is drawn, and
// reading it here would put a trip to memory between two workgroup barriers of every task
__device__ __forceinline__ void mark_phase_end(Ctrl *c, int phase, u64 t0) {
    atomicMax(&c->stats[8 + phase], now_ticks() - t0);
}

#ifdef MOE_TILE_TIMING
#define MOE_TT_BEGIN() u64 tt_prev_ = now_ticks()
#define MOE_TT(ctrl, slot)                                     \
    do {                                                       \
        const u64 tt_now_ = now_ticks();                       \
        if (threadIdx.x == 0) atomicAdd(&(ctrl)->dbg[slot], tt_now_ - tt_prev_); \
        tt_prev_ = tt_now_;                                    \
    } while (0)
#else
#define MOE_TT_BEGIN() do {} while (0)
#define MOE_TT(ctrl, slot) do {} while (0)
#endif

// Device functions that are real calls (not inlined) cannot see where a pointer
// they are handed points.  These helpers tell the compiler, so that it emits
// global_* / ds_* instead of the slower flat_* instructions.
template <typename T>
__device__ __forceinline__ T *as_global(T *p) {
    return (T *)(__attribute__((address_space(1))) T *)p;
}
__device__ __forceinline__ char *lds_at(u32 byte_offset) {
    return (char *)(__attribute__((address_space(3))) char *)(uintptr_t)byte_offset;
}
__device__ __forceinline__ u32 lds_offset(const void *p) {
    return (u32)(uintptr_t)(const __attribute__((address_space(3))) void *)p;
}
// The LDS offset of the kernel's dynamic LDS as a plain number in a scalar register, for handing to device
// functions that are real calls.  Without the empty asm the compiler sees that every caller passes the address
// of the same LDS variable, moves that variable into the callee, and (a non-kernel function cannot know where a
// kernel's dynamic LDS starts) looks its offset up in a table in memory: one scalar load plus a wait for ALL
// outstanding LDS traffic at every use, the GEMM main loop's stage switch included.
__device__ __forceinline__ u32 lds_offset_opaque(const void *p) {
    u32 v = (u32)__builtin_amdgcn_readfirstlane((int)lds_offset(p));
    asm volatile("" : "+s"(v));
    return v;
}
// The argument block of the running kernel sits in constant memory that scalar
// loads can read.  A kernel whose single parameter is a KArgs takes its address
// with kernel_args_address() (the compiler only knows it inside the kernel
// function itself) and hands it to device functions that are real calls; those
// read the block with load_kernel_args(): a handful of scalar loads instead of a
// copy through per-lane scratch memory.
typedef u64 KArgsAddr;
__device__ __forceinline__ KArgsAddr kernel_args_address() {
#if defined(__HIP_DEVICE_COMPILE__)
    return (KArgsAddr)(uintptr_t)__builtin_amdgcn_kernarg_segment_ptr();
#else
    return 0;
#endif
}
__device__ __forceinline__ KArgs load_kernel_args(KArgsAddr addr) {
    KArgs a;
#if defined(__HIP_DEVICE_COMPILE__)
    const u32 lo = __builtin_amdgcn_readfirstlane((u32)addr), hi = __builtin_amdgcn_readfirstlane((u32)(addr >> 32));
    // (an aligned pointer to constant memory at a uniform address: the copy becomes scalar loads)
    typedef const __attribute__((address_space(4))) KArgs *ConstArgs;
    __builtin_memcpy(&a, (ConstArgs)(uintptr_t)(((u64)hi << 32) | lo), sizeof(KArgs));
#endif
    return a;
}
// A value known to be the same in every lane, moved to a scalar register.
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

// Which of the chip's XCDs (accelerator dies, each with an L2 of its own) this
// wavefront runs on.
__device__ __forceinline__ int xcd_id() {
    u32 v;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(v));
    return (int)(v & 0xfu);
}
constexpr int kTileQueues = 8;  // one per XCD of an MI355X

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((u32)b) << 16); }
// round to nearest even; inputs here are finite
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    u32 u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}
__device__ __forceinline__ u32 pack_bf16x2(float lo, float hi) {
    return (u32)f32_to_bf16(lo) | ((u32)f32_to_bf16(hi) << 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float *p, size_t i) { return p[i]; }
};
template <> struct Elem<bf16_t> {
    static __device__ __forceinline__ float load(const bf16_t *p, size_t i) { return bf16_to_f32(p[i]); }
};

}  // namespace moe

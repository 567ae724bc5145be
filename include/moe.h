/*
 * C ABI of the MI355X (gfx950) MoE megakernel hot path.
 *
 * One GPU's share of a tile-granular Mixture-of-Experts layer (paper section
 * 2.1: gate -> dispatch -> expert compute -> combine; section 2.3: one
 * persistent kernel working on tiles; section 2.3 "put-with-signal" and
 * section 4.1 / Algorithm 1: how finished tiles are announced).
 *
 * Conventions
 *   - Every call returns a moe_status_t (0 = MOE_OK, negative = error).  The
 *     library never throws, aborts or prints.
 *   - Every pointer is a DEVICE pointer owned by the caller unless marked
 *     "host".  The library allocates nothing; scratch comes from a caller
 *     workspace of moe_workspace_bytes() bytes, 256-byte aligned, prepared once
 *     by moe_workspace_init().
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and the call returns without waiting for it.
 *   - Tensors are contiguous and row-major.  Element type of x, Wg, W1, W3,
 *     W2, staging and out is `dtype` (fp32, or bf16 as raw 16-bit patterns).
 *     Indices are int32, gate weights fp32.
 *   - Host-detectable misuse (NULL required pointer, k > E, R not dividing T,
 *     unsupported sizes) is reported before anything is launched.
 *
 * Notation: T tokens, d model dim, E local experts, k experts per token,
 * f FFN dim, R destinations.  Slot s = t*k + j is token t's j-th choice;
 * N = T*k slots.  Token t belongs to destination r = t / (T/R); destination
 * r's partition of `staging` is rows [r*(T/R)*k, (r+1)*(T/R)*k).
 */
#ifndef MOE_H
#define MOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MOE_OK = 0,
    MOE_ERR_INVALID_ARG = -1, /* NULL pointer, k > E, R does not divide T, ... */
    MOE_ERR_UNSUPPORTED = -2, /* legal problem this build has no kernel for    */
    MOE_ERR_WORKSPACE = -3,   /* workspace NULL or misaligned                  */
    MOE_ERR_NOT_READY = -4,   /* (device status) a flag was not at `epoch`     */
    MOE_ERR_HIP = -5,         /* a HIP runtime call failed                     */
    MOE_ERR_TIMEOUT = -6,     /* (device status) a bounded wait expired        */
    MOE_ERR_BAD_ROUTING = -7, /* (device status) expert id outside [0, E)      */
    MOE_ERR_CAPACITY = -8     /* (device status) an expert got more rows than  */
                              /* moe_problem_t.capacity                        */
} moe_status_t;

typedef enum { MOE_DT_F32 = 0, MOE_DT_BF16 = 1 } moe_dtype_t;

/* How a finished output tile is announced (section 2.3, section 4.1):
 *   PER_TILE  coupled put-with-signal: every published tile is written, then a
 *             release fence, then its flag (PUT -> FENCE -> SIGNAL per tile).
 *   PER_DEST  decoupled signaling (Algorithm 1) with one group per
 *             destination: tiles are written back to back and counted in a
 *             per-destination counter; whoever completes the count issues ONE
 *             fence and then stores all flags of that destination. */
typedef enum { MOE_SIGNAL_PER_TILE = 0, MOE_SIGNAL_PER_DEST = 1 } moe_signal_mode_t;

/* Memory scope of the fence that precedes flag stores and of the flag
 * accesses themselves: this GPU only, or GPU + host + peers. */
typedef enum { MOE_SCOPE_AGENT = 0, MOE_SCOPE_SYSTEM = 1 } moe_fence_scope_t;

/* How the persistent kernel orders the expert tiles and the combine tasks (section 2.3:
 * tasks run as soon as their inputs are there):
 *   STATIC       dependency-ordered lists: every GEMM1 tile is handed out before any
 *                GEMM2 tile, every GEMM2 tile before any combine task; a task that finds
 *                its input unfinished waits for it.
 *   READY_QUEUE  tasks are enqueued by the event that makes them runnable and taken in
 *                that order: the workgroup that finishes the last GEMM1 tile of a row
 *                block enqueues the block's GEMM2 tiles; the workgroup that stores the
 *                last flag of a destination enqueues the combine tasks of the
 *                destination's tokens.  Workgroups take ready tasks before new GEMM1
 *                tiles, so GEMM2 tiles and combine tasks start out of order and nothing
 *                that was taken ever waits.  Results are identical. */
typedef enum { MOE_SCHED_STATIC = 0, MOE_SCHED_READY_QUEUE = 1 } moe_scheduler_t;

typedef struct {
    int32_t T, d, E, k, f, R; /* R must divide T.  Limits (else MOE_ERR_UNSUPPORTED):  */
                              /* E <= 256, k <= min(E, 32), R <= 1024, T*k <= 2^30,  */
                              /* d and f multiples of 64 (bf16) or 16 (fp32)         */
    int32_t dtype;            /* moe_dtype_t                                        */
    int32_t tile_m, tile_n;   /* publish tile rows x cols; 0 = 128 x 64 (the tile   */
                              /* of section 2.3).  tile_m in {32,64,128}, tile_n in */
                              /* {64,128}; MOE_DT_F32 takes tile_n = 64 only (else  */
                              /* MOE_ERR_UNSUPPORTED)                               */
    int32_t signal_mode;      /* moe_signal_mode_t                                  */
    int32_t fence_scope;      /* moe_fence_scope_t                                  */
    uint32_t epoch;           /* value a flag takes when its tile is ready; nonzero */
                              /* and larger than that of every earlier call on the  */
                              /* same `flags` array since the array was last zeroed */
                              /* (a call only touches the flags of the tiles it     */
                              /* publishes, and how many those are depends on the   */
                              /* routing: a flag that an earlier call set and this  */
                              /* one does not publish keeps its old value, so a     */
                              /* reused value could read as ready).  To start over, */
                              /* zero `flags` first                                 */
    int32_t group_size;       /* MOE_SIGNAL_PER_DEST only: flags per fence group    */
                              /* (section 4.1, granularity of Algorithm 1).  0 = all */
                              /* flags of a destination form one group (the paper's */
                              /* per-destination default); g >= 1 = groups of g     */
                              /* consecutive flags of a destination, one fence per  */
                              /* group: fences = sum over r of ceil(n_r / g).  Must */
                              /* be 0 for MOE_SIGNAL_PER_TILE                       */
    int32_t scheduler;        /* moe_scheduler_t (moe_megakernel_forward only)      */
    int32_t capacity;         /* layout of the rows sorted by expert.  0: ragged    */
                              /* (dropless: expert e owns rows offsets[e] ..        */
                              /* offsets[e] + counts[e], back to back).  C > 0: the */
                              /* padded layout of balanced routing (section 6.1,    */
                              /* expert capacity EC = S*k/E): expert e owns the C   */
                              /* rows from e*C, of which the first counts[e] are    */
                              /* used; offsets[e] = e*C, perm has E*C entries with  */
                              /* -1 in unused ones, x_perm has E*C rows (unused:    */
                              /* zero).  Nothing is dropped: an expert with more    */
                              /* than C rows is an error (MOE_ERR_CAPACITY)         */
    uint32_t wait_ticks;      /* bound of every wait inside the kernels, in ticks   */
                              /* of the GPU's 100 MHz wall clock; 0 = 4 s.  When a  */
                              /* wait's bound expires the waiter records            */
                              /* MOE_ERR_TIMEOUT, every other wait sees the error   */
                              /* and gives up, and all workgroups leave in the      */
                              /* ordinary way; the status arrives in stats[7] and   */
                              /* the workspace must be initialised again.  (A tiny  */
                              /* value is how a test forces that path from the      */
                              /* host.)                                             */
    int32_t fuse_ffn;         /* moe_megakernel_forward only.  0: GEMM1 and GEMM2   */
                              /* are separate tile passes with h in the workspace.  */
                              /* 1: a workgroup takes a row block of 32 or 64 rows  */
                              /* through both GEMMs and keeps the block's h in LDS  */
                              /* (section 2.3: a tile traverses GEMM -> activation  */
                              /* -> GEMM).  bf16 only, MOE_SCHED_STATIC only,       */
                              /* tile_m <= 64, and rows * f * 2 bytes must fit the  */
                              /* LDS beside the stage buffers (f <= 768), else      */
                              /* MOE_ERR_UNSUPPORTED.  Same results                 */
} moe_problem_t;

/* number of 64-bit counters moe_megakernel_forward writes to `stats` */
#define MOE_NUM_STATS 20
/* stats[0] release fences issued right before flag stores (per tile, or per fence group:
 *          a destination, or group_size of its flags)
 * stats[1] flags stored                 stats[2] publish tiles written
 * stats[3] per-compute-tile releases that only feed a fence-group counter (PER_DEST)
 * stats[4] GEMM1 compute tiles          stats[5] GEMM2 compute tiles
 * stats[6] bounded waits that expired   stats[7] device status (a moe_status_t, 0 = ok)
 * stats[8..13] in-kernel timeline: nanoseconds from the first task drawn to the end of
 *   the last gate task [8], the plan [9], the last permutation block [10], the last
 *   GEMM1 tile [11], the last GEMM2 tile [12], the last combine task [13]
 * stats[14] nanoseconds workgroups spent waiting on dependencies (each wait counted once per
 *   workgroup, by its clock from the first poll to the last), summed over workgroups
 * stats[15] workgroups launched
 * stats[16..17] MOE_SCHED_READY_QUEUE only (else 0): tasks taken from the ready queues [16];
 *   GEMM2 tiles among them that a workgroup ran while GEMM1 tiles were still waiting to be
 *   handed out [17]
 * stats[18..19] reserved (0) */

/* Host, pure: bytes of workspace a problem needs / upper bound on the number
 * of flags (uint32 each) the caller must provide; 0 if the problem is invalid. */
size_t moe_workspace_bytes(const moe_problem_t *p);
size_t moe_num_flags(const moe_problem_t *p);

/* Host, pure: static string for a status code. */
const char *moe_status_string(int status);

/* Zero the control part of a fresh workspace.  Call once after allocating it
 * (and again after a call reported MOE_ERR_TIMEOUT); every other entry point
 * leaves the workspace ready for the next call.  Size and layout of the workspace
 * depend on T, d, E, k, f, R, dtype, tile_m, tile_n and capacity only: signal_mode,
 * fence_scope, epoch, group_size and scheduler may change from call to call. */
int moe_workspace_init(const moe_problem_t *p, void *workspace, void *stream);

/*
 * Gate (section 2.1 step 1).  logits[t,e] = sum_i x[t,i] Wg[i,e] + gate_bias[e]
 * accumulated in fp64; topk_idx[t,:] = the k largest in descending order
 * (equal scores: lower expert id first); topk_w[t,j] = softmax over the k
 * chosen logits (sums to 1).
 *   x [T,d], Wg [d,E] in, dtype; gate_bias [E] fp32 in, may be NULL.
 *   topk_idx [T,k] int32 out; topk_w [T,k] fp32 out.   E <= 256.
 */
int moe_route(const moe_problem_t *p, const void *x, const void *Wg, const float *gate_bias,
              int32_t *topk_idx, float *topk_w, void *stream);

/*
 * Dispatch in its local form (section 2.1 step 2; section 2.3 "group tokens
 * into tiles"): stable counting sort of the N slots by expert.
 *   topk_idx [T,k] in (every id in [0,E), the k ids of a token distinct).
 *   counts [E], offsets [E+1] out: histogram and its exclusive scan.
 *   perm [N] out: slot at sorted position p (slots of one expert ascending);
 *   inv_perm [N] out: inverse.  x_perm [N,d] out, may be NULL:
 *   x_perm[p,:] = x[perm[p]/k,:].  workspace as above.
 *   With p->capacity = C > 0, perm and x_perm have E*C entries / rows (see
 *   moe_problem_t) and inv_perm[s] = e*C + rank; counts are exact whatever C is,
 *   and when one exceeds C nothing else is written.
 *   status_dev: int32 on the device, may be NULL, written only on failure:
 *   MOE_ERR_BAD_ROUTING if an id lies outside [0,E) (such a slot is counted for
 *   no expert), MOE_ERR_CAPACITY if an expert has more than C rows.  In both
 *   cases counts (and offsets) are written, perm / inv_perm / x_perm are not,
 *   and no slot number is ever followed outside x.
 */
int moe_dispatch(const moe_problem_t *p, const void *x, const int32_t *topk_idx, int32_t *counts,
                 int32_t *offsets, int32_t *perm, int32_t *inv_perm, void *x_perm,
                 int32_t *status_dev, void *workspace, void *stream);

/*
 * moe_dispatch for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments (minus the workspace), same results, same
 * kernels; the one scratch buffer those kernels need (the per-block expert
 * histograms, ceil(T/64) * E int32) lives in a static array of 64 KB in device
 * memory that belongs to the library: one copy per GPU the library runs on, held
 * until the process ends.  The call allocates and frees nothing.
 *   (Small problems, T*k * ceil(T/16) <= 2^26, run as one launch that needs no
 *   scratch at all; the array serves the larger ones.)
 *   Limit (the form of the dispatch whose histograms fit one workgroup's LDS):
 *   4 * (ceil(T/64) * E + 3 * (E + 1)) + 8 * E <= 65536, e.g. T <= 7808 at
 *   E = 128 and T <= 130688 at E = 8; beyond it MOE_ERR_UNSUPPORTED is returned
 *   before anything is launched.
 *   Every call on a GPU uses that GPU's array, which keeps what the last call
 *   left (each call overwrites the part it reads, nothing has to start at
 *   zero): calls that overlap in time on one GPU, on whatever streams, race.
 */
int moe_dispatch_noalloc(const moe_problem_t *p, const void *x, const int32_t *topk_idx,
                         int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv_perm,
                         void *x_perm, int32_t *status_dev, void *stream);

/*
 * The whole layer in ONE persistent kernel (sections 2.1, 2.3, 4.1): gate,
 * dispatch, per-expert SwiGLU FFN  y = (silu(x W1[e]) * (x W3[e])) W2[e]
 * as a grouped GEMM, publication of every finished y tile into `staging`
 * (row s of staging = expert output for slot s) with a ready flag, and the
 * weighted combine out[t] = sum_j topk_w[t,j] * staging[t*k+j], which waits on
 * the flags.
 *   Wg == NULL: routing is precomputed; topk_idx / topk_w are inputs.
 *   W1, W3 [E,d,f], W2 [E,f,d] in.
 *   topk_idx, topk_w, counts, offsets, perm, inv_perm: as above (outputs).
 *   slot_flag [N] int32 out: index of the first flag (column block 0) of the
 *     publish tile that carries slot s; column block c is slot_flag[s] + c.
 *   staging [N,d] out; flags [moe_num_flags()] uint32 in/out: entries of
 *     tiles published by this call are set to p->epoch; out [T,d] out.
 *   stats [MOE_NUM_STATS] uint64 out, may be NULL.
 * Flags are numbered destination-major, then expert, then row block of tile_m
 * rows counted from the expert's first row, then column block of tile_n.
 */
int moe_megakernel_forward(const moe_problem_t *p, const void *x, const void *Wg,
                           const float *gate_bias, const void *W1, const void *W3, const void *W2,
                           int32_t *topk_idx, float *topk_w, int32_t *counts, int32_t *offsets,
                           int32_t *perm, int32_t *inv_perm, int32_t *slot_flag, void *staging,
                           uint32_t *flags, void *out, uint64_t *stats, void *workspace,
                           void *stream);

/*
 * Combine alone (section 2.1 step 4): out[t] = sum_j topk_w[t,j] *
 * staging[t*k+j] in fp32, rounded once to dtype.  Before reading slot s the
 * kernel checks, with acquire loads at p->fence_scope, that every flag
 * slot_flag[s] + c (c < ceil(d/tile_n)) equals p->epoch; if one does not,
 * *status_dev is set to MOE_ERR_NOT_READY (the row is still combined from
 * whatever staging holds).  slot_flag == NULL skips the check.
 *   status_dev: int32 on the device, written only on failure; may be NULL.
 */
int moe_combine(const moe_problem_t *p, const void *staging, const uint32_t *flags,
                const int32_t *slot_flag, const float *topk_w, void *out, int32_t *status_dev,
                void *stream);

/*
 * Measurement aid, no part of the layer: the rate at which this GPU's matrix cores retire bf16 work when nothing
 * else happens (what the grouped GEMM's "fraction of the MFMA peak" can be held against on a given box; the clock
 * a chip holds under matrix-core load depends on its power limit and on the operand bits).  `workgroups` workgroups
 * of 4 wavefronts each run `iters` rounds of 16 independent 32x32x16 bf16 products (16 * 32768 FLOP per wavefront
 * and round) on operands read once from `frag` (device, 8192 bytes: 8 fragments of 16 bytes per lane; any bf16
 * patterns) and write one float per thread to `sink` (device, workgroups * 256 floats) so that the work is kept.
 * Asynchronous on `stream`; the caller times it.  FLOPs = workgroups * 4 * iters * 16 * 32768.
 */
int moe_probe_mfma(const void *frag, int32_t iters, int32_t workgroups, float *sink, void *stream);

/*
 * Measurement aid, no part of the layer: the rate at which this GPU's CUs pull bytes in when they do nothing else
 * (what the weight-streaming phases of the layer, which run 4 wavefronts per CU, can be held against on a given
 * box, by source and by wavefronts per CU).  `workgroups` workgroups of
 * `wavefronts` (4, 8 or 16) wavefronts, one per CU (each takes 128 KB of LDS), read `bytes_per_workgroup` bytes each
 * (rounded down to a multiple of wavefronts * 8 KB) from `buf` (device, at least span_bytes): workgroup w starts at
 * byte (w * stride_bytes) mod span_bytes and wraps inside the first span_bytes, so that a span far beyond the caches
 * with stride = bytes_per_workgroup streams from HBM, and a small span with stride 0 streams from L2.  to_lds = 1:
 * loads that write straight into LDS, as the GEMM main loop's do; 0: loads into registers.  `sink` (device,
 * workgroups * wavefronts * 64 words) receives one word per thread so that the work is kept.  span_bytes >= 16 KB,
 * span_bytes and stride_bytes multiples of 16, else MOE_ERR_INVALID_ARG.  Asynchronous on `stream`; the caller
 * times it.  Bytes = workgroups * bytes_per_workgroup (rounded as above).
 */
int moe_probe_stream(const void *buf, size_t span_bytes, size_t stride_bytes, size_t bytes_per_workgroup,
                     int32_t workgroups, int32_t wavefronts, int32_t to_lds, uint32_t *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_H */

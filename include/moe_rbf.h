/*
 * moe_rbf -- relay-buffer-free MoE dispatch and combine for AMD MI355X (gfx950).
 *
 * One device's share of the paper's communication path: routing ids are turned
 * into counts, offsets and a stable row map; dispatch copies every token row
 * straight into its destination expert window; combine reads the k expert-output
 * rows of a token back out of the windows and reduces them with the gate weights,
 * writing in token order.  There is no staging, relay or un-permute buffer.
 *
 * Notation (paper, Section 5.1 and Table 1): T tokens, hidden size H, routing
 * degree k, E experts on R ranks, E_r = E/R experts per rank; X[T,H] hidden
 * states, K[T,k] routing ids, W[T,k] gate weights; c^exp, c^rank branch counts;
 * s small offset; o large offset; expert-window row = o + s.
 * The R rank windows are R contiguous row regions of ONE device buffer that
 * stands in for the remote windows of a pooled-HBM system.
 *
 * General conventions
 *   - Every pointer named "device" must be device memory of the current HIP
 *     device, owned by the caller, 16-byte aligned.  The library allocates and
 *     frees nothing, copies nothing between host and device and never
 *     synchronises: all work is enqueued on the caller's stream and results are
 *     valid once that stream reaches the end of the call's work.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - The shared library needs the HIP runtime by soname (libamdhip64.so.7) and uses whichever copy the
 *     process has loaded first.  A process that embeds PyTorch must load torch's copy before this library
 *     (the Python binding does), so that the caller's streams and device pointers belong to the same
 *     runtime as the library's launches.
 *   - moe_shape and moe_plan_t are read on the host during the call only.
 *   - All tensors are row-major and dense.  X, window, expert_out and Y share
 *     `dtype`; K is int32; W is float32; all counts and offsets are int32.
 *   - Return value: MOE_OK or a negative moe_status.  All error returns are
 *     decided on the host BEFORE anything is enqueued (so a failed call has no
 *     effect), except MOE_ERR_LAUNCH which reports that the HIP runtime refused a kernel launch.
 *   - Data-dependent problems cannot be returned without a synchronisation; they
 *     are recorded in the device words plan->status[0..1] (see moe_plan).
 */
#ifndef MOE_RBF_H
#define MOE_RBF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum moe_dtype { MOE_DTYPE_BF16 = 0, MOE_DTYPE_F32 = 1 };

/* Two schedules compute the same values (paper, Section 4):
 *   PREFILL: explicit Layout -> Notify -> Dispatch -> Combine; moe_plan must run before moe_dispatch.
 *   DECODE : counts, offsets and row map are produced inside the dispatch kernel.
 *   AUTO   : DECODE iff T*k <= MOE_AUTO_DECODE_MAX_BRANCHES. */
enum moe_schedule { MOE_SCHEDULE_AUTO = 0, MOE_SCHEDULE_PREFILL = 1, MOE_SCHEDULE_DECODE = 2 };

enum moe_status {
  MOE_OK = 0,
  MOE_ERR_NULL = -1,       /* a required pointer is NULL */
  MOE_ERR_SHAPE = -2,      /* T<0, H<1, k<1, E<1, R<1, E%R!=0, E>MOE_MAX_EXPERTS, rank_id outside [0,R), negative
                              stride, unknown dtype/schedule, or DECODE forced with T*k > MOE_DECODE_MAX_BRANCHES */
  MOE_ERR_ALIGN = -3,      /* H*elem_bytes not a multiple of 16, or a device pointer not 16-byte aligned */
  MOE_ERR_OVERFLOW = -4,   /* T*k or the window row count does not fit in int32, or a launch grid would not:
                              8*T*k and T*ceil(H*elem_bytes/1024) must also stay below 2^31 */
  MOE_ERR_WORKSPACE = -5,  /* plan->workspace missing or smaller than moe_workspace_bytes (only when moe_plan
                              uses it: batches of more than MOE_PLAN_SINGLE_LAUNCH_MAX_BRANCHES branches) */
  MOE_ERR_LAUNCH = -6,     /* the HIP runtime refused a kernel launch */
  MOE_ERR_OVERLAP = -7     /* x overlaps the window, or y overlaps expert_out (byte ranges known on the host) */
};

#define MOE_MAX_EXPERTS 1024
#define MOE_AUTO_DECODE_MAX_BRANCHES 5120
#define MOE_DECODE_MAX_BRANCHES 8192
#define MOE_PLAN_SINGLE_LAUNCH_MAX_BRANCHES 12288 /* up to here moe_plan is one launch and ignores plan->workspace */
#ifndef MOE_PREFETCH_MAX_BYTES
#define MOE_PREFETCH_MAX_BYTES (224u << 20)       /* what moe_plan reads of plan->prefetch at most (the Infinity Cache holds 256 MB) */
#endif
#define MOE_STATIC_SCRATCH_BYTES (1u << 20)       /* device scratch held by the library for moe_plan_static */

typedef struct moe_shape {
  int32_t T;                  /* tokens (0 is legal: counts are zeroed, nothing else happens) */
  int32_t H;                  /* hidden size, elements */
  int32_t k;                  /* routing degree; ids may repeat inside a token, so k > E is legal */
  int32_t E;                  /* experts, 1..MOE_MAX_EXPERTS */
  int32_t R;                  /* rank regions; E % R == 0 */
  int32_t dtype;              /* moe_dtype of X / window / expert_out / Y */
  int32_t schedule;           /* moe_schedule */
  int32_t rank_id;            /* which source rank this device is, 0..R-1; only used when plan->source_count is
                                 given (otherwise leave 0) */
  int64_t region_stride_rows; /* 0: tight windows, region r holds exactly c^rank[r] rows and the window has T*k rows.
                                 >0: symmetric windows, region r starts at row r*stride; branches that do not fit
                                 in their region are not placed (row_map = -1) and are counted in status[1]. */
} moe_shape;

/* Plan state (paper, Table 1).  All pointers are DEVICE pointers owned by the caller.
 * Written by moe_plan (PREFILL) or by moe_dispatch (DECODE); read by moe_dispatch (PREFILL) and moe_combine. */
typedef struct moe_plan_t {
  int32_t *expert_count;  /* [E]    c^exp: routed branches per expert (perExpertTokenNum; also the per-expert
                                    receive counts n^exp for the single source rank) */
  int32_t *rank_count;    /* [R]    c^rank: routed branches per destination rank (perRankTokenNum; n^recv of region r) */
  int32_t *expert_offset; /* [E+1]  o: first window row of expert e's block (putOffset / ep_recv_count);
                                    [E] = one past the last expert's block */
  int32_t *region_base;   /* [R+1]  first window row of rank region r; [R] = window row count */
  int32_t *send_idx;      /* [T*k]  s / delta: position of the branch inside its expert's stream, counting branches
                                    with smaller flat index t*k+j and the same expert (sendTokenIdx / expandIdx);
                                    -1 for skipped ids.  May be NULL: then it is not written. */
  int32_t *row_map;       /* [T*k]  window row of the branch = expert_offset[K] + send_idx; -1 = not placed */
  int32_t *status;        /* [3]    {number of ids outside [0,E) other than -1, number of branches dropped for
                                    region capacity, 1 if the rows of all source ranks together reach 2^31}.
                                    Id -1 marks an unused slot and is not an error.  When status[2] is set (possible
                                    only with source_count) no branch is placed: row_map is -1 everywhere, status[1] is
                                    0 and the offset tables are unspecified; counts and send_idx are valid. */
  void *workspace;        /* device scratch for moe_plan, >= moe_workspace_bytes(shape); unused by DECODE dispatch and
                             by moe_plan for T*k <= MOE_PLAN_SINGLE_LAUNCH_MAX_BRANCHES (may then be NULL) */
  size_t workspace_bytes;
  /* Several source ranks (paper, Section 5.2 "Prefill Notify": gathered count matrix M, recvData).  Optional. */
  const int32_t *source_count; /* [R*E] in: M[r*E+e] = branches source rank r sends to expert e.  Row shape->rank_id is
                                    ignored (this rank's counts are computed from its own ids).  NULL = this rank is the
                                    only source.  An expert's block then holds one sub-block per source rank, in rank
                                    order, and expert_offset[e] = o_{e,rank_id} = start of THIS rank's sub-block;
                                    expert_offset[E] = one past the last block.  The caller, who holds M, sizes tight
                                    windows to the sum of all counts (moe_window_rows cannot know it).  Counts are
                                    non-negative; a row total of 2^31 or more is reported in status[2]. */
  int32_t *recv_count;    /* [E]    out, may be NULL: rows of expert e's whole block over all sources (n^exp,
                                    recvTokenNumPerExpert); the rows a rank region receives (n^recv) are its segment sum */
  int32_t *recv_offset;   /* [E+1]  out, may be NULL: first row of expert e's whole block; [E] = one past the last block */
  int32_t *dispatch_order; /* [2*T*k] optional (NULL: not used): plan state for the PREFILL dispatch.  Where it pays
                                    (rows of 12 KB or more while x holds at most 96 MiB and the window at most 770 MiB; rows of 8 to 12 KB and of 2 to 4 KB with windows of up to 1100 MiB) the plan also lists the
                                    placed branches as (token, window row) pairs, sorted by window row inside stretches
                                    of about 28 MB of X, and moe_dispatch walks that list instead of the tokens: rows
                                    of one expert are then written together.  Entries of unplaced branches are -1.
                                    The result of moe_dispatch is the same with or without it.  Content and use are
                                    decided by the shape alone; a DECODE dispatch leaves a valid list too. */
  const void *prefetch;    /* optional (NULL: none), read by moe_plan / moe_plan_static only: device memory that the
                                    call should pull into the cache hierarchy while it plans, normally the x of the
                                    moe_dispatch that follows.  The plan kernels are latency-bound and leave the
                                    memory system idle; spare workgroups of the second plan launch read this range
                                    (nothing is written, no result depends on it).  A dispatch whose token rows are
                                    not cached runs 15-35 % slower (they are fetched in small pieces while the chip
                                    is saturated with writes), so a caller that cannot tell whether x is still
                                    cached from the operator that produced it passes it here.  16-byte aligned. */
  size_t prefetch_bytes;   /* bytes of `prefetch` that may be read (all of it readable device memory); a multiple
                                    of 16.  At most MOE_PREFETCH_MAX_BYTES of it are read. */
} moe_plan_t;

/* Bytes of plan->workspace that moe_plan needs for this shape (multiple of 256, never 0). */
int moe_workspace_bytes(const moe_shape *shape, size_t *out_bytes);

/* Rows the window / expert_out buffers must hold: T*k (tight) or R*region_stride_rows. */
int moe_window_rows(const moe_shape *shape, int64_t *out_rows);

/* Which schedule moe_dispatch will use for this shape (resolves AUTO). */
int moe_resolve_schedule(const moe_shape *shape, int32_t *out_schedule);

/* Prefill Layout + Notify (paper, Section 5.2; Algorithm 1 steps "Layout" and "Notify"; one source rank, or
 * one of several when plan->source_count carries the gathered count matrix).
 *   topk_idx : device, int32 [T*k], read only.
 *   Writes every array of `plan` (send_idx only if non-NULL) and zero-initialises status itself.
 *   Moves no payload.  Results do not depend on the launch configuration. */
int moe_plan(const moe_shape *shape, const int32_t *topk_idx, moe_plan_t *plan, void *stream);

/* moe_plan for callers that cannot allocate device memory or hand a workspace over: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same results and the same
 * kernels as moe_plan, but plan->workspace and plan->workspace_bytes are ignored: the scratch (per-tile
 * histograms) lives in a device array of MOE_STATIC_SCRATCH_BYTES that is part of the library image, one copy
 * per device, held until the process ends.  The call allocates and frees nothing.
 *   Limit: MOE_ERR_WORKSPACE if moe_workspace_bytes(shape) > MOE_STATIC_SCRATCH_BYTES (with E <= 510 every
 *   shape fits; E = 1024 fits up to 522240 branches); decided on the host before anything is enqueued.
 *   The first call on a device looks the array's device address up (hipGetSymbolAddress, no allocation);
 *   make that first call outside stream capture.  A failed lookup returns MOE_ERR_LAUNCH.
 *   Every call on a device shares that device's array.  Nothing in it has to start at zero (each call writes
 *   every word before reading it), but two calls that overlap in time on one device, on different streams,
 *   race on it: serialise them, or use moe_plan with separate workspaces. */
int moe_plan_static(const moe_shape *shape, const int32_t *topk_idx, moe_plan_t *plan, void *stream);

/* Dispatch (paper, Section 5.2 "Prefill Dispatch" / Section 5.3 "Decode Dispatch"; first loop of
 * Algorithms 1 and 2): window[row_map[t,j], :] = X[t, :] for every placed branch.
 *   x        : device, [T,H] of shape->dtype, read only.
 *   topk_idx : device, int32 [T*k]; read by the DECODE schedule only (may be NULL for PREFILL).
 *   plan     : PREFILL reads row_map; DECODE writes all of the plan exactly as moe_plan would.
 *   window   : device, [moe_window_rows, H]; only rows some branch maps to are written.
 *   x and window must not overlap: MOE_ERR_OVERLAP if the T*H elements of x share a byte with the window rows
 *   the host knows of (moe_window_rows; with plan->source_count and tight windows, the first T*k rows). */
int moe_dispatch(const moe_shape *shape, const void *x, const int32_t *topk_idx, moe_plan_t *plan,
                 void *window, void *stream);

/* Row-wise quantised dispatch (paper, Section 5.2, end of "Prefill Dispatch"; the "quant" rows of Table 2):
 * every token row is quantised once and its scale is kept in a separate float array indexed by window row.
 * The paper names no format; this library's format is OCP FP8 E4M3 codes plus one float32 scale per row:
 *   amax = max |x| over the token row, scale = amax / 448, code = e4m3(x * (448 / amax)) rounded to nearest
 *   even; an all-zero row has scale 1.  Every destination row of a token receives the same codes and scale.
 *   Non-finite inputs: a NaN element does not enter amax and yields a NaN code (S.1111.111, sign unspecified);
 *   a row with an infinite element has scale +Inf, signed-zero codes for its finite elements and NaN codes
 *   for the infinite ones.
 *   shape->dtype must be MOE_DTYPE_BF16 (type of x) and H <= 32768; schedules and plan as for moe_dispatch.
 *   window_q     : device, [moe_window_rows, H] bytes; only rows some branch maps to are written.
 *   window_scale : device, float32 [moe_window_rows]; same rows. */
int moe_dispatch_quant(const moe_shape *shape, const void *x, const int32_t *topk_idx, moe_plan_t *plan,
                       void *window_q, float *window_scale, void *stream);

/* Combine (paper, Section 5.2 "Prefill Combine" / Section 5.3 "Decode Combine"; second loop of
 * Algorithms 1 and 2): Y[t,:] = sum_j W[t,j] * expert_out[row_map[t,j], :].
 *   Accumulation is fp32 from +0 in ascending j with one fused multiply-add per placed branch and a single
 *   round-to-nearest-even to shape->dtype; unplaced branches (row_map = -1) are skipped.
 *   expert_out : device, window layout, read only (may be the window buffer itself).
 *   topk_w     : device, float32 [T*k].
 *   y          : device, [T,H], every row written; must not overlap expert_out (MOE_ERR_OVERLAP, same extent
 *                rule as for moe_dispatch). */
int moe_combine(const moe_shape *shape, const void *expert_out, const float *topk_w, const moe_plan_t *plan,
                void *y, void *stream);

/* HIP runtime's description of the most recent launch result on the calling thread (diagnostics for
 * MOE_ERR_LAUNCH; "no error" if the last launch succeeded). */
const char *moe_last_launch_error(void);

/* Static string for a moe_status value. */
const char *moe_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* MOE_RBF_H */

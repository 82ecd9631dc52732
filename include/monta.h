/*
 * monta.h -- C ABI of the MI355X (gfx950) MoE token dispatch / combine path of
 * MoNTA (arxiv 2411.00662).
 *
 * One GPU holds what the paper spreads over an expert-parallel (EP) x
 * tensor-parallel (TP) group: the `ep` destination ranks and the `tp` redundant
 * TP ranks are *virtual* -- partitions of buffers in one HBM allocation.  The
 * path is the source-side work of the paper's first AllToAll and its mirror:
 *
 *   route     gate logits -> top-k expert ids + probabilities          (section "Expert Parallel": Routing)
 *   plan      stable counting sort of (token, choice) pairs by expert   (same section: Permutation)
 *   dispatch  each virtual TP rank packs only its 1/tp of the tokens of (section "Pipelining": "Drop" split;
 *             slice j into its region of the send buffer STAGE           Eq. 4: chunks along the sequence)
 *   regather  every (unit, expert) block of STAGE is copied to its      (section "Pipelining": AllGather; paragraph
 *             place in the expert-major buffer FINAL                     "AllGather and D2D copy Pipelining")
 *   combine   out[t] = sum_j gate[t,j] * y[row of (t,j)]                (section "Expert Parallel": Combine, Unpermutation)
 *
 * FINAL is, byte for byte, what the plain (tp = 1, slices = 1) permutation
 * produces: the paper's claim that its transforms are exact rearrangements.
 *
 * Conventions
 *   - Every pointer except `cfg`, `layout` and output scalars is a DEVICE pointer
 *     owned by the caller.  The library allocates no user buffer and frees none.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls
 *     only enqueue work; none synchronises with the host.
 *   - Return value: MONTA_OK (0) or a negative monta_status.  Arguments are
 *     validated before the first HIP call, so bad arguments never reach the GPU.
 *     Nothing throws or aborts across this boundary.
 *   - Threads.  Entry points may be called from several host threads as long as
 *     calls that share a workspace or a buffer are ordered by the caller (same
 *     stream, or events).  The forms that use the library's side stream
 *     (pipeline mode 0, monta_route_dispatch_expert with overlap = 1) share one
 *     side stream and one set of events per device; such a call holds a per-device
 *     lock while it enqueues, so calls from several threads are safe and run one
 *     after the other on the side stream.  The monta_set_* switches are
 *     process-wide; every entry point reads them once, when it is called, and
 *     uses that snapshot for all of its work, so a switch changed by another
 *     thread takes effect at the next call, never in the middle of one.
 *     monta_shutdown() releases the side streams and events.
 *   - Limits: 1 <= top_k <= experts <= 256, top_k <= 32, experts % ep == 0,
 *     tokens % (slices * tp) == 0, tokens * top_k < 2^31,
 *     hidden * sizeof(element) % 16 == 0; activation base pointers 16-byte
 *     aligned, all others 4-byte aligned.  Logits must be finite (NaN is
 *     treated as -inf; the result is then unspecified but in bounds).
 *
 * Units.  U = slices * tp units of Tu = tokens / U consecutive tokens; unit u is
 * slice u / tp, virtual TP rank u % tp.  Expert e lives on virtual EP rank
 * e / (experts / ep), so expert order is (EP rank, local expert) order.
 *
 * Buffers.  STAGE and FINAL hold `max_rows` rows of hidden elements; only rows
 * below R (the number of kept pairs) are ever written -- except in the
 * capacity-padded layout (cfg->padded = 1), where FINAL is written up to row
 * E*C: kept rows first in every expert's block, zeros behind them.
 *   STAGE  [slice][tp rank][expert][kept rows of that unit, token order]
 *   FINAL  [expert][kept rows, token order]
 */
#ifndef MONTA_H
#define MONTA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum monta_dtype { MONTA_FP32 = 0, MONTA_BF16 = 1 };

enum monta_status {
    MONTA_OK = 0,
    MONTA_ERR_INVALID = -1,     /* a size or flag violates the preconditions above          */
    MONTA_ERR_UNSUPPORTED = -2, /* valid in principle, outside this library's limits        */
    MONTA_ERR_NULL = -3,        /* a required pointer is NULL                               */
    MONTA_ERR_HIP = -4,         /* a HIP runtime call failed; see monta_last_hip_error()    */
    MONTA_ERR_ALIGN = -5,       /* a pointer is not aligned as required                     */
    MONTA_ERR_TOO_LARGE = -6    /* monta_route_dispatch_combine_static: the plan tables exceed the static array */
};

/* The problem statement: tokens, hidden, experts, top-k, ep, tp, slices, capacity. */
typedef struct monta_cfg {
    int64_t tokens;          /* T = microbatch * sequence length (b*s of Eq. 3)               */
    int32_t hidden;          /* H, elements per token row                                       */
    int32_t dtype;           /* monta_dtype of activations; logits and gates are always fp32    */
    int32_t experts;         /* E                                                               */
    int32_t top_k;           /* k                                                               */
    int32_t ep;              /* virtual expert-parallel ranks (e of Eq. 8)                      */
    int32_t tp;              /* virtual tensor-parallel ranks (t of Eq. 8-9)                    */
    int32_t slices;          /* S chunks along the sequence (N of Eq. 4)                        */
    float capacity_factor;   /* 0: nothing is dropped; else C = min(T, ceil(cf*T*k/E)) per expert,
                                global over all tokens, lowest token indices survive            */
    int32_t renorm;          /* 1: gates renormalised over the k winners; 0: softmax over all E */
    int32_t padded;          /* 0: compact FINAL (expert segments back to back, R rows);
                                1: capacity-padded FINAL [E][C][H]: expert e owns rows [e*C, (e+1)*C), kept rows
                                   first, the padding zero-filled by the regather of slice 0 (or of all slices).
                                   STAGE stays compact.  With capacity_factor = 0, C = T. */
} monta_cfg;

/* Where the plan tables live inside the caller's workspace (byte offsets from
 * `ws`; every table is int32, row-major).  Filled by monta_ws_layout_query(). */
typedef struct monta_ws_layout {
    int64_t ws_bytes;        /* size the caller must allocate; the base must be 16-byte aligned (checked:
                                MONTA_ERR_ALIGN), tables inside start at multiples of 256 bytes */
    int64_t max_rows;        /* rows STAGE / FINAL / expert output must hold: min(T*k, E*C), or E*C if padded */
    int64_t capacity;        /* C                                                               */
    int32_t units;           /* U                                                               */
    int32_t tokens_per_unit; /* Tu                                                              */
    int32_t block_tokens;    /* tokens routed per workgroup (internal granularity)             */
    int32_t num_blocks;      /* workgroups of the route kernel                                  */
    int64_t off_meta;        /* [16]: [0] R (kept pairs)  [1] tokens with >= 1 kept pair  [2] C  [4] rows of FINAL */
    int64_t off_counts;      /* [E]     pairs that chose expert e                               */
    int64_t off_kept;        /* [E]     min(counts, C)                                          */
    int64_t off_offsets;     /* [E+1]   first FINAL row of expert e (exclusive scan of kept, or e*C if padded) */
    int64_t off_n;           /* [U][E]  kept pairs of expert e with token in unit u             */
    int64_t off_stage_off;   /* [U][E]  first STAGE row of block (u,e)                          */
    int64_t off_unit_base;   /* [U][E]  first FINAL row of block (u,e)                          */
    int64_t off_send_rows;   /* [U][ep] rows unit u addresses to virtual EP rank d              */
    int64_t off_unit_rows;   /* [U+1]   first STAGE row of unit u; [U] = R                      */
    int64_t off_pos_final;   /* [T][k]  FINAL row of pair (t,j), -1 if dropped                  */
    int64_t off_pos_stage;   /* [T][k]  STAGE row of pair (t,j), -1 if dropped                  */
    int64_t off_row_map;     /* [max_rows] FINAL row of STAGE row s (the per-row index offsets) */
    int64_t off_block_counts;/* [num_blocks][E] internal                                        */
    int64_t off_block_base;  /* [num_blocks][E] internal                                        */
    int64_t off_local_rank;  /* [T][k] internal: rank of a pair inside its route workgroup      */
    int64_t off_kept_prefix; /* [E+1] internal: exclusive scan of kept (= offsets when compact)    */
} monta_ws_layout;

/* Host only.  Validates cfg and reports the workspace size and the row capacity
 * the activation buffers need. */
int monta_workspace_bytes(const monta_cfg *cfg, size_t *ws_bytes, int64_t *max_rows);

/* Host only.  Same validation; fills the whole layout. */
int monta_ws_layout_query(const monta_cfg *cfg, monta_ws_layout *layout);

/* Puts a freshly allocated workspace into its initial state (a small fill kernel
 * on `stream`; zero-filling the workspace by any other means is equivalent).
 * Needed once per workspace, before its first monta_route. */
int monta_ws_init(const monta_cfg *cfg, void *ws, void *stream);

/* Gate projection (section "MoE": the gating network is a linear layer whose output goes through softmax
 * and TopK): logits[t][e] = sum_h x[t][h] * w_gate[e][h].  x [T][H] and w_gate [E][H] (one row per expert) in
 * cfg->dtype, device pointers, 16-byte aligned; logits [T][E] fp32, device, written in full.  bf16 inputs are
 * multiplied on the matrix cores with fp32 accumulation; the order of the additions is fixed for a given shape,
 * so two calls on the same inputs agree bit for bit, and it differs from a left-to-right sum by at most
 * H * 2^-24 * sum_h |x[t][h] * w_gate[e][h]|.  Uses only tokens, hidden, dtype and experts of cfg (all of it is
 * validated); needs no workspace.  Nothing is owned or kept; the work is enqueued on `stream`. */
int monta_gate(const monta_cfg *cfg, const void *x, const void *w_gate, float *logits, void *stream);

/* Expert computation on the expert-major buffer (section "Expert Parallel": between Dispatch and Combine every
 * expert processes the tokens grouped to it; section "Pipelining": the expert computation waits for the D2D
 * copies of the chunks it reads).  One linear layer per expert stands in for the expert network:
 *   y[r][n] = sum_h x_final[r][h] * w_exp[e][n][h]   for every kept row r of expert e,
 * x_final [max_rows][H] (the FINAL buffer, compact or padded layout), w_exp [E][out_features][H] (one row of H
 * inputs per output feature), y [max_rows][out_features], all in cfg->dtype, device pointers, 16-byte aligned;
 * out_features a multiple of 8 (bf16) or 4 (fp32).  slice = -1: all kept rows; slice = j: only the rows that
 * slice j's tokens fill (one contiguous run per expert), so the call can follow monta_regather(j) while later
 * slices are still being moved.  Rows of no expert (and padding rows) are not written.  bf16 runs on the matrix
 * cores with fp32 accumulation and one rounding to bf16; the order of the additions is fixed for a shape.
 * Needs the tables written by monta_route on `ws`; enqueued on `stream`. */
int monta_expert_linear(const monta_cfg *cfg, const void *x_final, const void *w_exp, int32_t out_features, void *y,
                        const void *ws, int slice, void *stream);

/* Routing, the slice pipeline and the expert layer in one call (section "Pipelining": the expert computation needs
 * the D2D copies of the chunks it reads; overlapping it with the remaining copies is what the paper leaves as future
 * work).  overlap = 0: monta_route_dispatch_regather, then monta_expert_linear on all rows, on `stream`.
 * overlap = 1: as soon as the regather of slice j is done, the expert layer of slice j's rows starts on a second
 * stream of the library (default priority) while `stream` goes on packing and regathering slice j+1; the call
 * returns with `stream` waiting for the last expert launch.  Either way y holds the same values (a row's result
 * does not depend on which launch computed it).  Arguments as in monta_route_dispatch_regather and
 * monta_expert_linear; y must not alias x, stage or final_. */
int monta_route_dispatch_expert(const monta_cfg *cfg, const float *logits, const void *x, int32_t *topk_idx, float *gates,
                                void *stage, void *final_, const void *w_exp, int32_t out_features, void *y, void *ws,
                                int overlap, void *stream);

/* Routing + Permutation plan.  logits [T][E] fp32 -> topk_idx [T][k] int32 (slot 0
 * = strongest choice; ties go to the lower expert index; selection is on the raw
 * logits), gates [T][k] fp32 (evaluated in fp64, rounded once), and every plan
 * table of monta_ws_layout in `ws`.  `ws` must be ws_bytes large and must have
 * been through monta_ws_init once (the library keeps it consistent from then on).  Calls on the same ws must not overlap in time. */
int monta_route(const monta_cfg *cfg, const float *logits, int32_t *topk_idx, float *gates,
                void *ws, void *stream);

/* Send-buffer packing with the TP-group split and the sequence chunks: for every
 * token of slice `slice` (all slices if -1) and every kept choice j the token's row
 * is copied, bit for bit, to STAGE row pos_stage[t][j].  x [T][H], stage
 * [max_rows][H] in cfg->dtype.  Needs the tables written by monta_route on `ws`.
 * Per virtual TP rank and slice this moves T*k*row/(S*tp) bytes when nothing is
 * dropped: the I/(N*t) of Eq. 8. */
int monta_dispatch(const monta_cfg *cfg, const void *x, void *stage, const void *ws, int slice,
                   void *stream);

/* Intra-node gather + D2D copy to index offsets, as one device copy pass:
 * STAGE row s of slice `slice` (all if -1) goes to FINAL row row_map[s].  After
 * all slices FINAL[pos_final[t][j]] == x[t] for every kept pair. */
int monta_regather(const monta_cfg *cfg, const void *stage, void *final_, const void *ws, int slice,
                   void *stream);

/* The gather as a pass of its own (the O2 order of section "Pipelining": AllGather first, D2D copy
 * after it): the STAGE rows of slice `slice` (all if -1), one contiguous range, are copied unchanged
 * into `gathered` [max_rows][H] -- what every TP rank of the group holds after the AllGather.
 * monta_regather(cfg, gathered, final_, ...) is then the D2D copy.  monta_regather straight from
 * STAGE fuses the two passes and moves half the bytes; this entry point exists to measure the
 * two-pass order against it. */
int monta_allgather(const monta_cfg *cfg, const void *stage, void *gathered, const void *ws, int slice, void *stream);

/* The two-pass order with the paper's third transform (paragraph "AllGather and D2D copy Pipelining", Fig. 8;
 * the stream picture of section "AllToAll performance", Implementation): for every chunk j the gather
 * (STAGE rows of slice j -> gathered) and then the D2D copy to index offsets (gathered -> FINAL), with the
 * copy of chunk j overlapping the gather of chunk j+1.  stage must hold every slice (after monta_dispatch).
 * schedule 0: chunk by chunk, gather then copy, nothing overlaps (the O2 order on one stream);
 *          1: S+1 launches on `stream`; launch j gathers chunk j and, in disjoint workgroups of the same
 *             grid, copies chunk j-1;
 *          2: gathers on `stream`, copies on the library's side stream (default priority), one event per
 *             chunk, joined back into `stream` before the call returns.
 * gathered [max_rows][H] ends up equal to stage below R; final_ equals what monta_regather produces.
 * MONTA_ERR_INVALID for another schedule or aliased buffers. */
int monta_allgather_regather(const monta_cfg *cfg, const void *stage, void *gathered, void *final_, const void *ws,
                             int schedule, void *stream);

/* The slice pipeline (the paper's multi-stream schedule, section "AllToAll
 * performance", Implementation): regather(j) runs after pack(j) and overlaps
 * pack(j+1); everything has finished, in stream order, when the call's work on
 * `stream` completes.  Equivalent to calling monta_dispatch and monta_regather
 * for j = 0..S-1.  How the overlap is realised is chosen by
 * monta_set_pipeline_mode(). */
int monta_dispatch_regather(const monta_cfg *cfg, const void *x, void *stage, void *final_,
                            const void *ws, void *stream);

/* monta_route followed by monta_dispatch_regather, as one call.  Same results and
 * same tables.  In pipeline mode 1, for shapes whose histogram table is small, the
 * kernel that finishes the plan also packs slice 0 (those workgroups derive their
 * rows themselves), so the first pack does not wait for the plan; otherwise the
 * call is exactly the two calls in sequence. */
int monta_route_dispatch_regather(const monta_cfg *cfg, const float *logits, const void *x, int32_t *topk_idx,
                                  float *gates, void *stage, void *final_, void *ws, void *stream);

/* Unpermutation with scale-add: out[t][:] = sum over kept j (ascending) of
 * gates[t][j] * y[pos_final[t][j]][:], accumulated in fp64 starting from +0 (every
 * product of an fp32 gate with an fp32 / bf16 element is exact there) and rounded
 * once, nearest-even, to cfg->dtype (bf16 through a round-to-odd fp32 step, so there
 * is no double rounding); a token with no kept pair gives a zero row.  y [max_rows][H] is the expert output in FINAL
 * layout (FINAL itself under identity experts), out [T][H]. */
int monta_combine(const monta_cfg *cfg, const void *y, const float *gates, void *out, const void *ws,
                  void *stream);

/* For callers that cannot allocate device memory or hand over a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  The whole step with identity experts --
 * monta_route_dispatch_regather followed by monta_combine(y = final_) -- with the plan tables kept in a
 * file-scope device array of the library (16 MiB per GPU, held until the process ends) instead of a caller
 * workspace.  The caller still passes every input and output: logits [T][E], x [T][H], topk_idx / gates [T][k],
 * stage / final_ [max_rows][H], out [T][H], all device pointers as in the calls above; results are bit-identical
 * to those calls.  Calls no hipMalloc / hipFree and creates no stream or event: pipeline mode 0 is replaced by
 * the size-chosen mode, and with event profiling enabled the call is refused (MONTA_ERR_INVALID).  Problems
 * whose tables (monta_ws_layout.ws_bytes) exceed 16 MiB are refused with MONTA_ERR_TOO_LARGE before any GPU
 * work; the five named workloads need at most 8.2 MiB.  Every call on one GPU shares that GPU's array: the
 * counters in it are cleared by a small kernel at the start of each call, the tables are overwritten, and two
 * calls that overlap in time on one GPU (different streams or threads) race -- the caller must order them.  The
 * first call on a device looks the array's address up (hipGetSymbolAddress): make one call before capturing the
 * entry point into a HIP graph; captured, it records kernel nodes only. */
int monta_route_dispatch_combine_static(const monta_cfg *cfg, const float *logits, const void *x, int32_t *topk_idx,
                                        float *gates, void *stage, void *final_, void *out, void *stream);

/* ---- the second AllToAll, mirrored (section "Pipelining", end of the paragraph on the Drop / AllGather
 * transform: the paper applies the same split to the second AllToAll) ----
 * The expert output y [max_rows][H] (FINAL layout) travels back the way the tokens came: block by
 * block into the unit-major layout of STAGE, so that every virtual TP rank again carries only 1/tp
 * of a slice, and from there into token order.  The result is bit-identical to monta_combine. */

/* Row row_map[s] of y goes to row s of y_stage, for the STAGE rows of slice `slice` (all if -1). */
int monta_unregather(const monta_cfg *cfg, const void *y, void *y_stage, const void *ws, int slice, void *stream);

/* Scale-add from the unit-major layout: out[t] = sum over kept j of gates[t][j] * y_stage[pos_stage[t][j]]
 * for the tokens of slice `slice` (all if -1); same arithmetic as monta_combine. */
int monta_combine_staged(const monta_cfg *cfg, const void *y_stage, const float *gates, void *out, const void *ws,
                         int slice, void *stream);

/* The return pipeline on one stream.  With pipeline mode 0 or 1, launch j fetches slice j back and, in disjoint
 * workgroups of the same grid, combines the tokens of slice j-1 (S+1 launches); with mode 2, fetch and combine of
 * every slice are two plain kernels; the default (-1) groups consecutive slices as the forward pipeline does
 * (groups of up to 256 MiB, two plain kernels per group once a group is that large or the problem is one group). */
int monta_unregather_combine(const monta_cfg *cfg, const void *y, void *y_stage, const float *gates, void *out,
                             const void *ws, void *stream);

/* Pipeline realisations for monta_dispatch_regather:
 *   0  two streams: packs on `stream`, regathers on a library-owned side stream
 *      (default priority), one event per slice, joined back into `stream`;
 *   1  one stream, co-scheduled grids: launch j does regather(j-1) and pack(j) in
 *      disjoint workgroups of one grid (S+1 launches, no events);
 *   2  one stream, strictly serial pack(0), regather(0), pack(1), ...
 *  -1  (default) chosen per call from the sizes, as the paper's planner picks its chunk count from
 *      the traffic: consecutive slices are grouped into one launch until a launch's share of STAGE
 *      reaches 256 MiB; the groups run as in 1 while their copies are short, as in 2 once a group
 *      moves 192 MiB or more.  A problem that fits one group runs in three launches: plan + pack of
 *      the first slices (about one round of workgroups), pack of the rest co-scheduled with the
 *      regather of the first, regather of the rest.
 * With 0, 1 or 2 every launch covers exactly one slice.  STAGE keeps its [slice][tp rank][expert]
 * layout in every case; only the launch grouping differs.
 * Returns MONTA_ERR_INVALID for other values.  Process-wide. */
int monta_set_pipeline_mode(int mode);
int monta_get_pipeline_mode(void);
/* Host only: what monta_route_dispatch_regather would do for cfg under the current switch: the realisation
 * (0, 1 or 2), the slices the first launch covers, the slices each later launch covers, and whether the kernel
 * that finishes the plan also packs the first launch's slices.  Benchmarks use it to attribute bytes to launches. */
int monta_pipeline_query(const monta_cfg *cfg, int32_t *mode, int32_t *first_slices, int32_t *slices_per_launch,
                         int32_t *plan_fused);

/* How monta_route builds the plan tables.  -1 (default): when the per-workgroup
 * histogram table is small (num_blocks * experts <= 65536) every workgroup of the
 * positions kernel rebuilds the scans it needs from that table (no serial tail);
 * otherwise, and always with mode 0, the last route workgroup to finish does the
 * scans once (ticket counter) and a separate kernel finishes the positions.  Both
 * produce identical tables.  Process-wide. */
int monta_set_plan_mode(int mode);
int monta_get_plan_mode(void);

/* Cache policy of the row movers: a bit mask saying which streams use non-temporal
 * (streaming) accesses: 1 pack loads, 2 pack stores, 4 regather loads, 8 regather
 * stores, 16 combine loads, 32 combine stores.  A clear bit leaves that stream
 * cacheable, which pays when the next kernel finds the data in the memory-side cache.
 * -1 (default) lets the library choose from the working-set size.  Process-wide. */
int monta_set_cache_policy(int policy);
int monta_get_cache_policy(void);

/* Plain device copy of `bytes` (multiple of 16, 16-byte aligned pointers) with the
 * same 16-byte-per-lane access pattern as the row movers.  It exists to measure
 * the achievable copy bandwidth and to calibrate profiler byte counters. */
int monta_copy(void *dst, const void *src, size_t bytes, void *stream);

/* Per-kernel timing with HIP events recorded on the launching stream.
 * After monta_profile_enable(1) every kernel launch is followed by an event; a
 * kernel's duration runs from the previous such event on its stream (the end of
 * the kernel before it) to its own, so back-to-back launches are timed without
 * gaps; a duration includes the kernel's launch latency and the stream time of
 * one event marker (a few microseconds, which a caller can estimate from the
 * slow-down of the whole sequence while profiling is on).  Only the library's
 * own launches are seen: other work put on the stream in between is charged to
 * the next kernel.  monta_profile_read synchronises with the recorded events and
 * returns the summed duration and the launch count of one kernel class since the
 * last reset.  Meant for benchmarks: it adds host work per launch. */
enum monta_kernel_id {
    MONTA_K_ROUTE = 0,      /* top-k + gates + histogram + scan               */
    MONTA_K_POSITIONS = 1,  /* per-pair positions and row map                 */
    MONTA_K_PACK = 2,
    MONTA_K_REGATHER = 3,
    MONTA_K_PACK_REGATHER = 4, /* co-scheduled grid of pipeline mode 1        */
    MONTA_K_COMBINE = 5,
    MONTA_K_COPY = 6,
    MONTA_K_PLAN_PACK = 7,  /* plan + positions + pack of slice 0 in one grid */
    MONTA_K_UNREGATHER = 8,
    MONTA_K_UNREGATHER_COMBINE = 9, /* co-scheduled grid of the return pipeline */
    MONTA_K_ALLGATHER = 10,
    MONTA_K_GATE = 11,      /* gate projection                                */
    MONTA_K_EXPERT = 12,    /* expert layer (grouped GEMM)                    */
    MONTA_K_ALLGATHER_REGATHER = 13, /* co-scheduled grid of the pipelined two-pass order */
    MONTA_K_COUNT = 14
};
int monta_profile_enable(int on);
int monta_profile_reset(void);
int monta_profile_read(int kernel_id, double *total_ms, int64_t *launches);

/* ---- planner: the paper's traffic-aware strategy choice (section "Network-traffic-aware") ----
 * Host only, no GPU work.  Per-chunk times AA_j, AG_j, D2D_j (Eq. 8-10), the O1 cost (Eq. 11),
 * the chunk-count searches (Algorithm 1 for O2, Algorithm 2 for O3) and the selection of the
 * cheapest strategy (Algorithm 3).  Where the printed algorithms are garbled the search keeps
 * the best (N, T) seen while N = 1, 2, ... runs until a chunk falls under i_minimal or n_max.
 * An efficiency curve is `n` points (volume in bytes ascending, efficiency in (0,1]),
 * interpolated linearly in the volume and held constant outside the sampled range. */
typedef struct monta_curve {
    const double *volume;   /* host pointer, n ascending volumes in bytes  */
    const double *eff;      /* host pointer, n efficiencies                */
    int32_t n;              /* >= 1                                        */
} monta_curve;

typedef struct monta_plan_in {
    double traffic;         /* I = b*s*h*BPE in bytes (Eq. 3)                                  */
    int32_t t, e;           /* tensor-parallel and expert-parallel degrees                     */
    double b1, b2, b3;      /* theoretical AllToAll, AllGather and memory bandwidth, bytes/s   */
    monta_curve r1, r2, r3; /* efficiency of AllToAll, AllGather, D2D copy against the volume  */
    double i_minimal;       /* chunks under this volume are not considered                     */
    int32_t n_max;          /* upper bound of the chunk search (>= 1)                          */
} monta_plan_in;

typedef struct monta_plan_out {
    double t_base;          /* untransformed AllToAll: I*(e-1)/e/(B1*r1(I))                    */
    double t_o1;            /* Eq. 11                                                          */
    double t_o2, t_o3;      /* best chunked times; +inf if no chunk count is admissible        */
    int32_t n_o2, n_o3;     /* their chunk counts; 0 if none                                   */
    int32_t strategy;       /* 1, 2 or 3: the cheapest (the lower number wins a tie)           */
    int32_t chunks;         /* chunk count of the chosen strategy (1 for O1)                   */
    double t_best;
} monta_plan_out;

/* Eq. 8-10 for one of n chunks; any of the outputs may be NULL. */
int monta_plan_chunk_times(const monta_plan_in *in, int n, double *aa, double *ag, double *d2d);
/* Algorithms 1-3. */
int monta_plan_strategy(const monta_plan_in *in, monta_plan_out *out);

/* Text for a monta_status; never NULL. */
const char *monta_strerror(int code);
/* The hipError_t (as int) behind the calling thread's last MONTA_ERR_HIP, 0 if none. */
int monta_last_hip_error(void);

/* Waits for the library's side streams, then destroys them, their events and any pending profiling
 * events, on every device that used them.  No other call of the library may be in flight.  The library
 * works again afterwards (the resources are created on demand). */
int monta_shutdown(void);

#ifdef __cplusplus
}
#endif
#endif /* MONTA_H */

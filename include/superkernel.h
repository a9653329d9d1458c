/*
 * superkernel.h -- C ABI of the coalesced "superkernel" library for MI355X (gfx950).
 *
 * The paper (arXiv 1901.10008, "The OoO VLIW JIT Compiler for GPU Inference")
 * proposes that callers hand the GPU runtime *operators, their inputs and a
 * latency constraint* instead of grids and blocks (Section 5.1, declarative
 * kernel dispatch), and that the runtime then (a) coalesces the mutually
 * independent operators of several inference streams into one large launch,
 * the superkernel (Sections 1 and 5.3), and (b) puts operators with tighter
 * latency budgets first (Section 5, item (a)).  This header is that interface
 * for one batch of operators: describe them (sk_problem), plan them
 * (sk_plan_create), run them as one launch (sk_launch) or, as the paper's
 * time-multiplexing baseline of Section 4.1, one launch per operator
 * (sk_launch_sequential).
 *
 * Operators are GEMMs and NHWC convolutions executed as the GEMM that backs
 * them (Section 5.3, Figure 6 caption).  Every operator has its own operands;
 * alpha = 1, beta = 0: C is overwritten and never read.
 *
 * General rules
 *   - Every function returns sk_status (0 = success, negative = error) unless
 *     stated otherwise.  No C++ exception crosses this boundary.  On error the
 *     output arguments are left untouched; sk_last_error() gives a thread-local
 *     detail string.
 *   - A, B and C pointers are DEVICE pointers borrowed from the caller, who
 *     keeps them alive and unmodified until the launches that use them have
 *     completed.  The sk_problem array itself is copied by sk_plan_create.
 *   - The plan owns its device-side tile table, operator descriptors and
 *     counters.  `hip_stream` arguments are hipStream_t handles owned by the
 *     caller (NULL = the default stream).  Launches are asynchronous.
 *   - A plan has one work counter: two launches of the SAME plan must not be in
 *     flight at the same time.  Launching it again on the same stream is fine
 *     (the stream orders them); on another stream the launch calls return
 *     SK_ERR_BUSY while the previous launch has not completed.  The check is best
 *     effort: launches recorded into a HIP graph are not tracked, and ordering a
 *     graph's replays against other launches of the plan is the caller's job.
 *   - Host threads: any number of threads may call into the library at the same
 *     time, each on plans of its own; calls that name the same plan are
 *     serialised by the caller.
 */
#ifndef SUPERKERNEL_H
#define SUPERKERNEL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SK_OK = 0,
  SK_ERR_INVALID_ARG = -1, /* null pointer, dimension < 1, bad struct field          */
  SK_ERR_UNSUPPORTED = -2, /* dtype / operator / dimension outside what is built      */
  SK_ERR_OVERLAP = -3,     /* two operators' C ranges overlap                        */
  SK_ERR_ALLOC = -4,       /* host or device allocation failed                       */
  SK_ERR_HIP = -5,         /* a HIP runtime call failed (no device, launch error...) */
  SK_ERR_BUSY = -6,        /* the plan's previous launch still runs on another stream */
  SK_ERR_STATE = -7        /* plan is host-only / stamps not enabled / ...           */
} sk_status;

/* A, B and C of one operator share the element type; accumulation is always fp32. */
typedef enum { SK_F32 = 0, SK_BF16 = 1, SK_F16 = 2 } sk_dtype;
typedef enum { SK_GEMM = 0, SK_CONV2D_NHWC = 1, SK_CONV2D_NCHW = 2 } sk_op;

/*
 * One operator: what it computes, where its operands live and its latency
 * budget, the three things Section 5.1 has the caller state instead of a launch
 * geometry.
 *
 * SK_GEMM:  C[M,N] = A[M,K] . B, with the K x N weight operand stored
 *   K-contiguous as Bs[N,K] (the layout of a linear layer's weight), i.e.
 *   C[m,n] = sum_k A[m*lda + k] * Bs[n*ldb + k].  A and C are row-major.
 *   lda, ldb, ldc are row strides in ELEMENTS; 0 means packed (K, K, N).
 *   The conv fields are ignored.
 *
 * SK_CONV2D_NHWC:  Y = conv(X, W), cross-correlation, dilation 1, one group,
 *   zero padding, no bias:  A = X[Nb,H,Wd,Cin],  B = W[Cout,R,S,Cin],
 *   Y[b,ho,wo,co] = sum_{r,s,c} X[b, ho*stride-pad_h+r, wo*stride-pad_w+s, c] * W[co,r,s,c],
 *   C = Y[Nb,Ho,Wo,Cout] with Ho = (H + 2*pad_h - R) / stride + 1 and
 *   Wo = (Wd + 2*pad_w - S) / stride + 1 (integer division), all dense.
 *   stride applies to both directions; 0 means 1 (the residual networks the
 *   paper serves in Section 5.3 have layers of stride 1 and 2).
 *   M, N, K and the row strides are ignored.  It is executed as the
 *   GEMM with rows (b*Ho+ho)*Wo+wo, columns co and reduction index
 *   (r*S+s)*Cin+c, without materialising the patch matrix.
 *
 * SK_CONV2D_NCHW:  the same operator on channel-major arrays, the other
 *   storage order inference frameworks hand over:  A = X[Nb,Cin,H,Wd],
 *   B = W[Cout,Cin,R,S],  C = Y[Nb,Cout,Ho,Wo], all dense,
 *   Y[b,co,ho,wo] = sum_{c,r,s} X[b, c, ho*stride-pad_h+r, wo*stride-pad_w+s] * W[co,c,r,s].
 *   Same fields and output size.  The reduction index is (c*R+r)*S+s, so the
 *   weights are still one contiguous row per output channel; activations and
 *   outputs are not contiguous along it, and the operator runs through the
 *   element-wise tile paths (correct for every shape, several times slower
 *   than the NHWC form).
 *
 * deadline_ms: latency budget measured from the start of the launch.  <= 0, NaN
 *   or +inf mean "none".  It only orders the operators (earliest first, ties by
 *   index); nothing is dropped or aborted when a deadline is missed.
 */
typedef struct {
  int32_t op;    /* sk_op    */
  int32_t dtype; /* sk_dtype */
  int32_t M, N, K;
  int64_t lda, ldb, ldc;
  int32_t Nb, H, Wd, Cin, Cout, R, S, pad_h, pad_w;
  int32_t stride;
  const void *A; /* device, read only */
  const void *B; /* device, read only */
  void *C;       /* device, written   */
  double deadline_ms;
} sk_problem;

/*
 * Planning parameters.  sk_plan_params_default() fills the defaults; a NULL
 * params pointer means the defaults.  The tile table is a pure integer
 * function of (problems, these fields); no device property enters it.
 */
typedef struct {
  int32_t edf;            /* 1: order operators by (deadline, index); 0: by index            */
  int32_t stamps;         /* 1: record a completion timestamp per operator (small cost)      */
  int32_t host_only;      /* 1: plan on the host only, touch no device (launches then fail)  */
  int32_t skinny_max_m;   /* operators with at most this many rows stream their weights      */
                          /* straight to registers ("skinny" classes); 0..64, default 64     */
  int64_t tile_bytes_max; /* upper/lower clamp of the target operand bytes per tile (defaults  */
  int64_t tile_bytes_min; /* 2 MiB, 32 KiB); the target is sum(bytes the operators' tiles      */
                          /* load) / balance_div: a streaming operator's weights, an LDS-tile  */
                          /* operator's 128 + BN operand rows per output tile                  */
  int32_t balance_div;    /* default 512                                                     */
  int32_t max_groups;     /* cap on 32-row weight groups per skinny tile, default 256        */
  int32_t grid_limit;     /* upper bound on persistent workgroups per launch;                */
                          /* 0 = 2 per compute unit of the current device                    */
  int32_t tail_div;       /* tiles shrink towards the end of the table: an operator's target */
                          /* is also capped by (such bytes of it and of all operators        */
                          /* after it in execution order) / tail_div, so that the launch     */
                          /* does not end on a few long tiles, but never below               */
                          /* 8 * tile_bytes_min; 0 = off, default 384                        */
  int32_t xcd_part;       /* LDS tiles that share operands go to the same accelerator die    */
                          /* (XCD: 32 compute units behind one L2): an operator's output     */
                          /* rectangles are cut into the fewest 1, 2, 4 or 8 two-dimensional */
                          /* parts of at most this many rectangles, one die per part         */
                          /* (sk_plan_get_xcd_lists); 0 = tiles are taken in table order by  */
                          /* whichever workgroup is free.  The lists halve the memory        */
                          /* traffic of compute-heavy plans and gain 0 to 10 percent there,  */
                          /* and cost plans with skinny tiles time.  Default -1: the planner */
                          /* decides: lists, with an eighth of the plan's rectangles per     */
                          /* part, if every operator is in the LDS-tile classes and the sum  */
                          /* of flops / peak exceeds the sum of operand bytes / bandwidth    */
                          /* (datasheet ratios, no device query); none otherwise             */
  int32_t reserved;       /* 0                                                               */
} sk_plan_params;

/*
 * One record of the flat tile table (32 bytes, little endian).  The table
 * lists, operator after operator in execution order, row blocks outer, column
 * blocks inner, reduction slices innermost.
 */
typedef struct {
  uint32_t problem;     /* index of the operator in the sk_problem array                    */
  uint16_t cls;         /* tile class: 0, 3, 6 skinny (1, 2, 4 blocks of 16 rows), 9: 128x128 and 10: 128x64 LDS tile */
  uint8_t ks_idx;       /* which reduction slice of the output rectangle this record is     */
  uint8_t S;            /* number of reduction slices of the rectangle (1 = not split)      */
  uint32_t m0, n0;      /* origin of the output rectangle in the operator's [Mg,Ng] GEMM view */
  uint16_t m_len, n_len;/* its extent, already clipped to the operator                      */
  uint32_t k0, k_len;   /* reduction range of this record                                   */
  uint32_t out_tile_id; /* running index of the output rectangle over the whole plan        */
} sk_tile;

typedef struct sk_plan sk_plan; /* opaque, owned by the library */

void sk_plan_params_default(sk_plan_params *params);

/*
 * Build the plan for n operators (the paper's runtime packing step, Section
 * 5.3): canonical GEMM view, tile class per operator, earliest-deadline-first
 * operator order, flat tile table; then upload table and descriptors to the
 * current HIP device (unless params->host_only).
 * n = 0 is a valid empty plan whose launches do nothing.
 * Errors: SK_ERR_INVALID_ARG (null pointers, dims < 1, negative strides,
 * strides smaller than a row), SK_ERR_UNSUPPORTED (unknown op/dtype, a
 * dimension that does not fit the table's fields), SK_ERR_OVERLAP (the C
 * ranges of two operators intersect; A and B may be shared freely),
 * SK_ERR_ALLOC, SK_ERR_HIP.
 */
sk_status sk_plan_create(const sk_problem *problems, int32_t n, const sk_plan_params *params,
                         sk_plan **out);
/*
 * Destroys the plan; NULL is accepted.  Waits first for the plan's launches
 * (they may still be reading its tables): for the latest one if all went to
 * one stream, for the whole device if they went to several streams or into a
 * stream capture.  Other plans' launches keep running.  Then hands the device
 * tables to a per-process pool from which later plans on the
 * same device are served: a runtime that plans once per launch (Section 5's
 * just-in-time coalescing) would otherwise pay a device allocation per launch.
 * The pool keeps at most 32 blocks and 512 MiB; older blocks are freed.
 */
sk_status sk_plan_destroy(sk_plan *plan);

/* Frees every pooled table block (all devices).  Plans that exist are not touched. */
sk_status sk_release_cached_memory(void);

/*
 * Run every operator of the plan in ONE kernel launch on `hip_stream`
 * (Sections 1 and 5.3: the superkernel).  Persistent workgroups take tiles
 * from the table in order, so operators with earlier deadlines start first:
 * workgroup b starts on tile b and takes further tiles through a single atomic
 * counter; a plan whose tiles are all short (at most 64 KB of operands each)
 * skips the counter and gives workgroup b the tiles b, b + grid, ...  With
 * per-die lists (params.xcd_part) a position of the table that holds an LDS tile only says
 * that one LDS tile is due: the workgroup runs the next tile of its die's list
 * (sk_plan_get_xcd_lists), so operators still start in table order, and every
 * tile runs exactly once with the same result bits.
 * Asynchronous.  Needs a device-resident plan (SK_ERR_STATE otherwise).
 * A plan has one tile queue and one set of split-reduction counters, which the
 * kernel re-arms itself when it ends: launches of ONE plan must not overlap
 * (order them on one stream or with events); different plans may.  SK_ERR_BUSY
 * if the plan's previous launch went to another stream and still runs.
 * The call makes no allocation, copy, memset or host synchronisation, so it may
 * be captured into a HIP graph; the plan must then outlive the graph's
 * replays.  (A plan with stamps enabled launches one more, one-thread kernel
 * that resets the start stamp.)
 */
sk_status sk_launch(sk_plan *plan, void *hip_stream);

/*
 * The time-multiplexing baseline (Section 4.1): the same device code, one
 * launch per operator, in submission (index) order, all on `hip_stream`.
 * Every operator is tiled as if it had been planned alone (the plan rule applied
 * to that operator by itself, what a caller who launches operators one by one
 * would get), not with the tiles of the coalesced table.  Reductions may
 * therefore be sliced differently: outputs agree with sk_launch up to the order
 * of summation, and bit for bit where the two tables coincide (a plan of one
 * operator).  SK_ERR_BUSY as for sk_launch.  The first call on a plan builds and uploads these tables
 * (SK_ERR_ALLOC / SK_ERR_HIP as for sk_plan_create); later calls only launch
 * (and may be captured into a HIP graph like sk_launch).
 */
sk_status sk_launch_sequential(sk_plan *plan, void *hip_stream);

/*
 * sk_launch for callers that cannot allocate device memory: code under HIP graph
 * capture set-ups, tight serving loops, harnesses that forbid hipMalloc.  Takes a
 * plan created with params->host_only = 1 (such a plan touches no device) and
 * runs it as sk_launch would, with the plan's device tables (work records, tile
 * queue, split-reduction counters and workspace) placed in a fixed array inside
 * the library's code object, SK_STATIC_SCRATCH_BYTES per GPU, instead of an
 * allocated block.  The call enqueues one copy of the plan's table image from
 * host memory to that array and one kernel launch on `hip_stream`, and calls no
 * hipMalloc, hipFree or other allocating routine; the first call on a device
 * looks up the array's address and the device's size.  Same results as
 * sk_launch, bit for bit (same table, same kernel).
 * SK_ERR_UNSUPPORTED if tables plus workspace exceed SK_STATIC_SCRATCH_BYTES,
 * SK_ERR_STATE for a plan that is not host-only or has stamps enabled.
 * Every call on a GPU uses that GPU's one array: calls that overlap on one GPU
 * (different streams, or different host threads without ordering) race and give
 * wrong results; calls on one stream are ordered by the stream.  The plan must
 * stay alive until the call has returned; A, B and C as for sk_launch.
 */
#define SK_STATIC_SCRATCH_BYTES (32u << 20)
sk_status sk_launch_static(sk_plan *plan, void *hip_stream);

/* Introspection of the packed plan (Section 5.3: what the runtime packing step produced; used to compare
 * the plan with a reference planner). */
int64_t sk_plan_num_tiles(const sk_plan *plan);    /* < 0 on error */
int32_t sk_plan_num_problems(const sk_plan *plan); /* < 0 on error */
/* Copies the flat table (num_tiles * 32 bytes) to host memory `dst`. */
sk_status sk_plan_get_tiles(const sk_plan *plan, void *dst, int64_t dst_bytes);
/* Execution order: order[i] = index of the i-th operator to start (n entries). */
sk_status sk_plan_get_order(const sk_plan *plan, int32_t *order);
/* Per operator (by index): first record and number of records in the table. */
sk_status sk_plan_get_ranges(const sk_plan *plan, int64_t *first_tile, int64_t *tile_count);
/* Persistent workgroups sk_launch uses for this plan (0 for an empty or host-only plan). */
int32_t sk_plan_grid(const sk_plan *plan);
/* Which die takes which LDS tile (sk_plan_params.xcd_part; Section 1 item (c): the shape of the execution
 * blocks is the runtime's to choose): offsets[9] and, if `tiles` is not null, at most `cap` table indices:
 * tiles[offsets[x] .. offsets[x+1]) are the records die x takes, in order.  offsets[8] is the number of
 * LDS tiles of the plan, 0 if the plan has no lists.  Host memory, caller-owned. */
sk_status sk_plan_get_xcd_lists(const sk_plan *plan, uint32_t *offsets, uint32_t *tiles, int64_t cap);

/*
 * Per-operator latency of the LAST completed launch of this plan (Section 5.2:
 * the runtime monitors inference latency per kernel); the caller must have
 * synchronised the stream.  done_ticks[i] is the device wall clock when
 * operator i's last tile retired, *start_tick the earliest clock at which any
 * workgroup of the launch (of the first launch, for sk_launch_sequential)
 * started; *ticks_per_ms converts.  Any pointer may be NULL.  SK_ERR_STATE
 * unless the plan was created with params->stamps = 1.
 */
sk_status sk_plan_get_stamps(sk_plan *plan, uint64_t *done_ticks, uint64_t *start_tick,
                             double *ticks_per_ms);

/*
 * Operators that arrive over time (Section 5, items (a) and (b); Section 5.2): a queue in front of the
 * planner that decides which of the operators submitted so far go into the next superkernel.
 *
 *   SK_QUEUE_SEQUENTIAL  one launch per operator in arrival order: the time multiplexing of Section 4.1
 *   SK_QUEUE_COALESCE    whenever the device is about to run dry, everything that has arrived and whose
 *                        output buffer is free goes into one plan, earliest deadline first
 *   SK_QUEUE_OOO         as COALESCE, but a launch is closed once its estimated duration reaches cap_ms:
 *                        operators are taken in deadline order and those with the most slack wait, so
 *                        that an urgent operator arriving meanwhile never sits behind a long launch
 *                        (the reordering in time of Section 5.2)
 *
 * The queue runs in the caller's thread: sk_queue_submit and sk_queue_poll both retire finished launches
 * and plan and launch the next one when it is due (shortly before the running launch is expected to end:
 * operand bytes / bytes_per_ms, corrected by a running ratio of measured to estimated durations), so the
 * caller keeps calling sk_queue_poll.  A queue belongs to one host thread at a time.  Launches go to
 * `hip_stream` (NULL = the default stream; a stream of its own keeps reading results from waiting for the
 * launch queued behind).  Two operators with the same C pointer are never in flight together: the later
 * one waits for a later launch.  Operand pointers as for sk_problem; they stay valid until the operator's
 * completion has been returned.
 *
 * sk_queue_submit: n operators arriving now, budget_ms[i] their latency budgets from now (NULL = none);
 *   tickets[i] (may be NULL) identify them in completions.  The problems are copied.
 * sk_queue_poll: up to `cap` completions into out[], *n_out of them.  wait = 0: never blocks; wait = 1:
 *   blocks until at least one completion can be returned or the queue is empty.  latency_ms runs from the
 *   submit call to the retirement of the operator's last tile (completion stamps of the launch, anchored at
 *   the host time at which the launch was seen complete); met = latency_ms <= budget_ms, or -1 for an
 *   operator whose batch could not be planned (the planner's status is then returned by the call that
 *   tried, and sk_last_error() has the detail).
 * sk_queue_destroy: waits for the launches in flight; operators not launched yet are dropped.
 */
typedef enum { SK_QUEUE_SEQUENTIAL = 0, SK_QUEUE_COALESCE = 1, SK_QUEUE_OOO = 2 } sk_queue_policy;

typedef struct {
  int32_t policy;         /* sk_queue_policy                                                              */
  int32_t depth;          /* launches queued on the device at once; 0 = 2 (16 for SK_QUEUE_SEQUENTIAL)    */
  double cap_ms;          /* SK_QUEUE_OOO: estimated duration at which a launch is closed, default 0.5    */
  double bytes_per_ms;    /* duration estimate of a launch: operand bytes / this, default 5.5e9           */
  double launch_floor_ms; /* no launch is estimated shorter than this, default 0.02                       */
} sk_queue_params;

typedef struct {
  uint64_t ticket;
  double latency_ms;
  double budget_ms; /* +inf if none was given */
  int32_t met;
  int32_t launch;   /* running number of the launch that served the operator */
} sk_completion;

typedef struct {
  int64_t submitted, completed, launches, met;
  double device_busy_ms; /* sum over coalesced launches of (last completion stamp - start stamp) */
  double span_ms;        /* first submit to the latest completion seen                           */
} sk_queue_stats;

typedef struct sk_queue sk_queue; /* opaque, owned by the library */

void sk_queue_params_default(sk_queue_params *params);
sk_status sk_queue_create(const sk_queue_params *params, void *hip_stream, sk_queue **out);
sk_status sk_queue_submit(sk_queue *queue, const sk_problem *ops, const double *budget_ms, int32_t n, uint64_t *tickets);
sk_status sk_queue_poll(sk_queue *queue, int32_t wait, sk_completion *out, int32_t cap, int32_t *n_out);
sk_status sk_queue_get_stats(const sk_queue *queue, sk_queue_stats *stats);
sk_status sk_queue_destroy(sk_queue *queue);

const char *sk_strerror(sk_status status);
const char *sk_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SUPERKERNEL_H */

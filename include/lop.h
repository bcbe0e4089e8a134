/* lop.h - C ABI of the banded local-operator chain library for AMD MI355X (gfx950).
 *
 * The library executes the data-parallel hot path of Local Operation Parallelism
 * (Intra-DP, arXiv 2507.05829, Sec. IV-A/IV-B): a chain of *local operators*
 * (block-wise: convolution, depthwise convolution, max pooling; element-wise: bias,
 * ReLU, ReLU6, residual add) is split into independent *row bands*. A band is a
 * contiguous interval of final output rows (the contiguous operation interval of
 * Sec. IV-C, "Computational Efficiency"); the rows of every earlier layer that the
 * band needs follow from kernel size, stride, padding and dilation (Sec. IV-A) and
 * are recomputed by neighbouring bands where they overlap (local-operation
 * replication, Sec. IV-C), so each band's output is final and can be copied to the
 * host while the next band computes (computation/transmission overlap, Sec. IV-B).
 *
 * Conventions
 *  - Every function returns LOP_OK (0) or a negative lop_status_t; nothing throws,
 *    aborts or prints.
 *  - Device tensors are NHWC, dense, in the storage type of the plan (float or
 *    bfloat16 bit patterns); accumulation is always fp32 and each layer output is
 *    rounded once (bfloat16: round to nearest even).
 *  - "host" / "device" in a parameter comment says where the pointer must point.
 *  - Row intervals are half-open [lo, hi) in rows of the tensor they refer to.
 */
#ifndef LOP_H_
#define LOP_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LOP_API __attribute__((visibility("default")))

typedef enum {
  LOP_OK = 0,
  LOP_ERR_INVALID_ARG = -1, /* null pointer, n_bands < 1, non-positive size, bad input_from */
  LOP_ERR_UNSUPPORTED = -2, /* operator / dtype / parameter combination without a kernel     */
  LOP_ERR_SHAPE = -3,       /* channel or residual shape mismatch, window larger than input  */
  LOP_ERR_BAND_RANGE = -4,  /* band or layer index outside the plan                          */
  LOP_ERR_OOM = -5,         /* host or device allocation failed                              */
  LOP_ERR_HIP = -6,         /* a HIP call failed; see lop_last_hip_error()                   */
  LOP_ERR_NOT_READY = -7,   /* plan was made with LOP_FLAG_PLAN_ONLY and cannot run          */
  LOP_ERR_TOO_LARGE = -8    /* lop_run_chain_static: scratch need above LOP_STATIC_SCRATCH_BYTES */
} lop_status_t;

/* Operator kinds (Sec. IV-A). Global operators (softmax, ...) are not local and are
 * rejected with LOP_ERR_UNSUPPORTED. */
typedef enum { LOP_CONV2D = 0, LOP_DWCONV2D = 1, LOP_MAXPOOL2D = 2, LOP_ELTWISE = 3 } lop_op_t;
typedef enum { LOP_ACT_NONE = 0, LOP_ACT_RELU = 1, LOP_ACT_RELU6 = 2 } lop_act_t;
typedef enum { LOP_F32 = 0, LOP_BF16 = 1 } lop_dtype_t;

#define LOP_INPUT (-1)       /* input_from / residual_from: the chain input */
#define LOP_NO_RESIDUAL (-2) /* residual_from: no residual                  */
#define LOP_MAX_BANDS 64

/* One vertex of the chain (the DAG of Sec. IV-C restricted to a chain with skip
 * edges). y = act(op(x) + bias + residual); for LOP_MAXPOOL2D bias, residual and act
 * must be absent. */
typedef struct {
  int op;                  /* lop_op_t                                                    */
  int c_in, c_out;         /* DWCONV / MAXPOOL / ELTWISE: c_out == c_in                   */
  int kh, kw, sh, sw, ph, pw, dh, dw; /* window, stride, padding, dilation (ELTWISE: ignored) */
  int act;                 /* lop_act_t                                                   */
  int input_from;          /* LOP_INPUT or the index of an earlier layer                  */
  int residual_from;       /* LOP_NO_RESIDUAL, LOP_INPUT or an earlier layer of the same
                              output shape; added before the activation                   */
  const void* weight;      /* host; OIHW in the plan's storage type (DWCONV: C x 1 x kh x kw);
                              copied by lop_plan, may be freed afterwards; NULL for MAXPOOL
                              and ELTWISE                                                 */
  const float* bias;       /* host; c_out fp32 values or NULL (= zero); copied by lop_plan */
} lop_layer_t;

typedef struct { int n, c, h, w; int dtype; /* lop_dtype_t */ } lop_tensor_desc_t;
typedef struct { int lo, hi; } lop_rows_t;
typedef struct lop_plan_s lop_plan_t; /* opaque */

typedef struct {
  int n_bands;
  float wall_ms;    /* host clock from first launch to the last byte arriving        */
  float compute_ms; /* first kernel start to last kernel end on the compute stream   */
  float copy_ms;    /* sum of the bands' device-to-host copy durations               */
  float band_compute_ms[LOP_MAX_BANDS];
  float band_copy_ms[LOP_MAX_BANDS];
  float band_ready_ms[LOP_MAX_BANDS]; /* from the start of the chain until the band's final rows
                                         are complete (on the host if copied, else on the device):
                                         when a consumer of that band could start (Sec. IV-B)   */
} lop_timing_t;

/* lop_plan flags */
#define LOP_FLAG_INDEPENDENT 0u /* the default mode, named: every band recomputes its halo rows
                                 (local-operation replication, Sec. IV-C), so bands are
                                 independent of one another and run in any order            */
#define LOP_FLAG_NO_D2H 1u    /* never copy to the host even if a host pointer is given  */
#define LOP_FLAG_PLAN_ONLY 2u /* integer planning only: touches no GPU, needs no weights;
                                 lop_run_* return LOP_ERR_NOT_READY                      */
#define LOP_FLAG_DMA_COPY 8u  /* always use hipMemcpyAsync for the band copies; by default the
                                 pinned host buffer is written by the kernel of the
                                 band's last layer itself (band outputs up to 256 KiB) or by
                                 a small copy kernel                                     */
#define LOP_FLAG_REUSE 16u    /* bands run in order and share per-layer buffers: a band computes,
                                 of every layer, only the rows no earlier band has produced
                                 (no halo recompute; data already on the device is reused,
                                 Sec. IV-B). A whole chain then runs on one lane and the
                                 chains of consecutive lop_run_chain calls rotate over the
                                 lanes. lop_run_band must be called for bands 0,1,2,... in
                                 order.                                                   */
#define LOP_DEFAULT_LANES 4
#define LOP_FLAG_BATCH_BANDS 128u /* independent bands (every halo row recomputed) whose launches are
                                 batched per operator (Sec. IV-D operation batching): all bands of
                                 a chain run on one lane, every layer is one launch that computes
                                 its rows for every band (each band on its own slabs), and chains
                                 of consecutive calls rotate over the lanes. The bands' rows leave
                                 behind the last layer's launch. Not with LOP_FLAG_REUSE; at most
                                 16 bands; LOP_ERR_UNSUPPORTED if an operator of the chain has no
                                 kernel form that takes several bands (the inverted-residual
                                 block, the 1x1 streaming and 3x3 depthwise kernels)      */
#define LOP_FLAG_NO_FUSE 32u  /* run every layer as a launch of its own. By default a 1x1 conv,
                                 a 3x3 depthwise conv and a 1x1 conv in a row whose middle
                                 tensors nobody else reads (an inverted-residual block) run as
                                 one launch that keeps the expanded tensor on chip; results
                                 agree with the layer-by-layer path to fp32 summation order */
#define LOP_FLAG_POISON_SCRATCH 64u /* debug aid: before a band's kernels (reuse mode: before a chain's
                                 first band) its scratch slabs and split-K workspace are filled
                                 with NaN bit patterns, so any read of a scratch row that the
                                 band's own launches did not write first poisons the output  */
#define LOP_FLAG_LANES(n) (((unsigned)(n) & 0xffu) << 8) /* bands are dealt round robin to n
                                 compute streams ("lanes", each with its own scratch) that run
                                 concurrently; 0 = LOP_DEFAULT_LANES, capped at the number of
                                 non-empty bands. With three or more lanes, independent
                                 bands whose copies are long (more than 256 KiB per band,
                                 at most 64 MiB per chain) leave one lane to the copies:
                                 n - 1 lanes compute, and a lop_run_chain without
                                 compute_stream and timing sends every band's copy to the
                                 last lane behind an event                                */
#define LOP_FLAG_GRAPH 4u     /* lop_run_chain (without timing) captures its launches and copies
                                 into a HIP graph on the first call for a given (d_in, d_out,
                                 h_out) and replays it afterwards; the graph joins the copies,
                                 so compute_stream then also waits for them              */

/* Build a plan: validate the chain, infer shapes, split the last layer's output rows
 * into n_bands intervals (first H mod B bands one row longer; trailing bands may be
 * empty when B > H), propagate each band backwards to the rows of every layer it needs
 * (hull over all consumers of a tensor, clamped to the image), size the scratch slabs,
 * and - unless LOP_FLAG_PLAN_ONLY - upload re-laid-out weights and biases to the
 * current HIP device.  (Sec. IV-A block size; Sec. IV-C partitioning and contiguity.)
 *   layers   host, n_layers entries, read only during the call
 *   in       host, shape and storage type of the chain input
 *   out_plan host; receives the handle, or NULL on error. Free with lop_plan_destroy. */
LOP_API int lop_plan(const lop_layer_t* layers, int n_layers, const lop_tensor_desc_t* in, int n_bands,
             unsigned flags, lop_plan_t** out_plan);

/* Shape queries (host only). */
LOP_API int lop_plan_out_desc(const lop_plan_t* plan, lop_tensor_desc_t* out);
LOP_API int lop_plan_layer_desc(const lop_plan_t* plan, int layer, lop_tensor_desc_t* out);
LOP_API int lop_plan_n_bands(const lop_plan_t* plan);
LOP_API int lop_plan_n_layers(const lop_plan_t* plan);

/* Row intervals of a band: final output rows, chain-input rows, rows of `layer`'s
 * output. An empty interval is reported as lo == hi. */
LOP_API int lop_plan_band_out_rows(const lop_plan_t* plan, int band, lop_rows_t* rows);
LOP_API int lop_plan_band_in_rows(const lop_plan_t* plan, int band, lop_rows_t* rows);
LOP_API int lop_plan_band_layer_rows(const lop_plan_t* plan, int band, int layer, lop_rows_t* rows);
/* Rows of `layer`'s output that the band's launch produces: all the rows it needs
 * (independent bands), or those of them no earlier band has produced (LOP_FLAG_REUSE). */
LOP_API int lop_plan_band_compute_rows(const lop_plan_t* plan, int band, int layer, lop_rows_t* rows);

/* Work counts: operations of the whole layers (useful) and summed over the bands'
 * intervals (executed; > useful where halos are recomputed); bytes of device scratch one lane
 * holds (the slabs of one band plus the largest split-K workspace of a launch). */
LOP_API int lop_plan_stats(const lop_plan_t* plan, double* useful_flop, double* executed_flop,
                   size_t* scratch_bytes);
/* Per layer and band: operations executed and algorithmic bytes moved (rows read of the
 * input and residual slabs, rows written, weights). */
LOP_API int lop_plan_layer_work(const lop_plan_t* plan, int band, int layer, double* flop, double* bytes);

/* Run one band (Alg. 1: compute on an operation interval, then send the finished
 * rows): enqueue one kernel per layer on compute_stream for the band's intervals,
 * then, if h_out is not NULL, enqueue on copy_stream the copy of the band's final rows
 * to h_out once the kernels are done. Asynchronous.
 *   d_in   device, whole chain input N x H x W x C; only band_in_rows(band) are read
 *   d_out  device, whole chain output; only band_out_rows(band) are written
 *   h_out  pinned host (hipHostMalloc or equivalent: memory the device can address), whole
 *          chain output, or NULL; host memory that is not pinned is refused with
 *          LOP_ERR_INVALID_ARG. What kind of memory h_out is is looked up once per address and
 *          plan and kept, and a
 *          captured graph (LOP_FLAG_GRAPH) holds the addresses it was captured with: a buffer
 *          passed here must stay allocated, and of the same kind, for as long as the plan lives.
 *   compute_stream, copy_stream  hipStream_t or NULL (= the plan's own streams)
 * d_in, d_out and h_out start on a 16-byte boundary (the kernels move 16-byte vectors), in this
 * and every other call that takes them; an address that does not is LOP_ERR_INVALID_ARG.
 * Bands b and b' with b = b' (mod lanes) share scratch memory: give them the same
 * compute stream (or NULL). Bands of different lanes may run concurrently. */
LOP_API int lop_run_band(lop_plan_t* plan, int band, const void* d_in, void* d_out, void* h_out,
                 void* compute_stream, void* copy_stream);

/* Run every band: the lanes fork from compute_stream, each runs its bands in order, band b's
 * copy overlaps the kernels of the bands after it (Sec. IV-B), and compute_stream waits for
 * all lanes' kernels (not for the copies: those are complete after lop_synchronize). With
 * compute_stream == NULL there is nothing to order against: d_in must be complete when the
 * call is made, every lane appends its bands to its own stream and the lanes are not joined,
 * so the chains of consecutive calls overlap (give each chain in flight its own d_out /
 * h_out); results are complete after lop_synchronize. With timing != NULL the call records
 * events, waits for completion and fills *timing; otherwise it is asynchronous. */
LOP_API int lop_run_chain(lop_plan_t* plan, const void* d_in, void* d_out, void* h_out,
                  void* compute_stream, lop_timing_t* timing);

/* lop_run_chain for callers that cannot allocate device memory or create streams and events
 * where they run: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc. Enqueues the kernels of every band, bands in order, on `stream` alone (NULL = the
 * null stream) and returns; no copy to the host, no event, no other stream. The band slabs and
 * the split-K partial sums do not live in the plan's allocations but in an array of
 * LOP_STATIC_SCRATCH_BYTES that is part of the library's code object: every GPU the library
 * is used on holds one such array from load until the process ends. The call allocates nothing,
 * frees nothing and calls no allocating routine. Its address on the plan's device was looked up
 * when the plan was made (lop_plan is the set-up call and does allocate).
 *   plan    made by lop_plan / lop_plan_rowwise on the current device, either mode
 *   d_in    device, whole chain input; d_out device, whole chain output (every row is written)
 * LOP_ERR_TOO_LARGE: the plan needs more scratch (lop_plan_stats: scratch_bytes) than the
 * array holds; nothing was enqueued. Results are those of lop_run_chain bit for bit (the same
 * kernels on the same intervals). All calls on one GPU, from any plan, share that GPU's array:
 * calls whose kernels can overlap on the GPU (different streams without an ordering between
 * them) race; order them on one stream or with events. The array is not cleared between calls
 * and need not be: every scratch row is written before it is read within a call. */
#define LOP_STATIC_SCRATCH_BYTES (64u << 20)
LOP_API int lop_run_chain_static(lop_plan_t* plan, const void* d_in, void* d_out, void* stream);

/* Wait for everything the plan has enqueued on its own and on the passed streams. */
LOP_API int lop_synchronize(lop_plan_t* plan);

/* Row-wise local operators (Sec. IV-A, Eq. 1): a chain of matrix products on a matrix of m
 * rows. A row of a layer's output depends on the same row of its input and on the whole
 * parameter matrix, which every band uses unpartitioned (replicated): row bands need no halo
 * and no exchange. Layer l computes y = act(x W^T + bias + residual) with x of m x k and W of
 * n x k (one row of W per output column, the layout of a fully connected layer's weight). */
typedef struct {
  int k, n;            /* columns of the input and of the output matrix                      */
  int act;             /* lop_act_t                                                          */
  int input_from;      /* LOP_INPUT or the index of an earlier layer (k must be its n)       */
  int residual_from;   /* LOP_NO_RESIDUAL, LOP_INPUT or an earlier layer with n columns      */
  const void* weight;  /* host; n x k row-major in the plan's storage type; copied           */
  const float* bias;   /* host; n fp32 values or NULL; copied                                */
} lop_rowwise_t;

/* Plan a chain of row-wise operators on an m x k matrix (row-major, storage type `dtype`),
 * its rows split into n_bands intervals as in lop_plan. The plan is used with every other
 * function of this header: d_in is the m x k matrix, d_out / h_out the m x n_last result, a
 * band's rows are matrix rows; lop_plan_out_desc reports {n = 1, c = n_last, h = m, w = 1}.
 * The matrix product runs on the kernels of the 1x1 convolution. Errors as lop_plan. */
LOP_API int lop_plan_rowwise(const lop_rowwise_t* layers, int n_layers, int m, int k, int dtype,
                             int n_bands, unsigned flags, lop_plan_t** out_plan);

/* ---- Local-operation scheduling model (Sec. IV-C): host arithmetic only, no GPU ----
 *
 * A vertex's operations are its output rows. A schedule gives every vertex two contiguous
 * row intervals, x_M on the mobile device and x_R on the server, that together cover all rows
 * (partitioning and operation-batching constraints); overlap is replication. The chain input
 * is whole on M, the result must be whole on M. */
typedef struct {
  int n_ops;          /* output rows                                                        */
  int input_from;     /* LOP_INPUT or an earlier vertex: the windowed edge                  */
  int residual_from;  /* LOP_NO_RESIDUAL, LOP_INPUT or an earlier vertex of n_ops rows: an
                         identity edge (row i needs row i)                                  */
  int k, s, p, d;     /* rows of the parent one output row reads: window, stride, padding,
                         dilation along the row axis                                        */
  double cm_fixed, cm_row; /* C_M(v) = cm_fixed + cm_row * |x_M(v)| seconds (0 if empty)    */
  double cr_fixed, cr_row; /* the same for the server                                       */
  double row_bytes;   /* bytes of one output row                                            */
} lop_loss_layer_t;

typedef struct { int m_lo, m_hi, r_lo, r_hi; } lop_loss_alloc_t; /* x_M = [m_lo, m_hi), x_R */

/* How transfers share the link in the model. INDEPENDENT: Eq. 3 as printed, every edge's rows
 * take latency + rows * row_bytes / bandwidth by themselves. QUEUED: as the runtime stage moves
 * them (Sec. IV-D, lop_run_two_party): after every vertex the rows its consumers on the other
 * device read travel as messages, a message occupies its direction of the link for latency +
 * bytes / bandwidth, messages of one direction queue in issue order, and rows a device already
 * holds are not sent again. */
#define LOP_LINK_INDEPENDENT 0
#define LOP_LINK_QUEUED 1

/* T = s_M(output) (Eq. 2) of a schedule under the dependency recurrence (Eq. 3): rows of a
 * parent that a device consumes but did not produce arrive from the peer latency + rows *
 * row_bytes / bandwidth seconds after the peer has finished that parent; several parents
 * combine by max; a device runs its vertices in index order. s_m (n_layers + 1 doubles, the
 * last is T) and s_r (n_layers) receive the start times if not NULL; *violations (optional)
 * the number of edges that carry rows out of a vertex whose output is larger than the raw
 * input (transmission-efficiency constraint). link_model: LOP_LINK_INDEPENDENT or
 * LOP_LINK_QUEUED. LOP_ERR_INVALID_ARG: malformed problem;
 * LOP_ERR_BAND_RANGE: an allocation that is not two intervals covering the vertex's rows. */
LOP_API int lop_loss_eval(const lop_loss_layer_t* layers, int n_layers, int in_rows, double in_row_bytes,
                          double bandwidth, double latency, const lop_loss_alloc_t* sched, double* T,
                          double* s_m, double* s_r, int* violations, int link_model);

/* Search a schedule of small T by differential evolution (DE/rand/1/bin, F 0.6, CR 0.9) over
 * x_M = [0, A), x_R = [B, n) with B <= A per vertex, seeded with the two one-device schedules;
 * schedules that break the transmission-efficiency constraint lose against all that keep it.
 * population <= 0: ten per decision variable. Deterministic for a given seed. Writes the best
 * schedule found (n_layers entries), its T and its violation count. */
LOP_API int lop_loss_solve(const lop_loss_layer_t* layers, int n_layers, int in_rows, double in_row_bytes,
                           double bandwidth, double latency, int population, int generations,
                           unsigned long long seed, lop_loss_alloc_t* best, double* T, int* violations,
                           int link_model);

/* Result of lop_run_two_party. */
typedef struct {
  float total_ms;      /* from the client's start until the whole result is on the client      */
  double bytes_to_m;   /* bytes the client received over the emulated link                      */
  double bytes_to_r;   /* bytes the server received                                             */
  int transfers;       /* messages (contiguous row ranges of one tensor) over the link, both ways */
} lop_two_party_stats_t;

/* Runtime stage with two parties (Sec. IV-D, Alg. 1 client / Alg. 2 server), emulated on the
 * one GPU: party M (client) holds the chain input and must end up with the whole result,
 * party R (server) starts with nothing. Each party is a stream with full-height buffers of its
 * own for every layer; for every layer, in chain order, a party computes its interval of
 * sched[layer] (x_M = [m_lo, m_hi), x_R = [r_lo, r_hi); one launch per party and layer,
 * operation batching), then for every edge out of that layer the rows its consumer on the other
 * party reads and does not hold yet are copied across (Send / Receive / combine: they land at
 * their position in the receiver's buffer). A consumer's launch waits only for its own
 * messages. The link is one stream per direction: a message is a device-to-device copy followed
 * by a wait of latency + bytes / bandwidth seconds (bandwidth in bytes per second), so messages
 * in one direction queue behind each other. If costs is not NULL (n_layers entries, only the
 * cm_ and cr_ fields are read) every launch is followed by a wait of its modelled time
 * C_D(v) = fixed + per_row * rows on that party's stream, which makes the party as slow as the
 * device it stands for. Fused launches are not used here. The plan's banding is ignored.
 *   d_in  device, whole input (N x H x W x C, the client's copy); d_out device, whole output.
 *   sched host, n_sched == number of layers, every entry two intervals covering the layer's
 *         rows, else LOP_ERR_BAND_RANGE. stats host, optional.
 * No single emulated wait may exceed 2 s (LOP_ERR_INVALID_ARG). Allocates and frees its
 * buffers and streams inside the call and returns when both parties are done (synchronous).
 * Values are those of the unpartitioned chain whatever the schedule (Sec. IV-B). */
LOP_API int lop_run_two_party(lop_plan_t* plan, const void* d_in, void* d_out, const lop_loss_alloc_t* sched,
                              int n_sched, const lop_loss_layer_t* costs, double bandwidth, double latency,
                              lop_two_party_stats_t* stats);

/* What this GPU sustains, measured: hbm_copy_gbs = bytes read + bytes written per second of a
 * plain 16-byte-vector copy between two 1 GiB device buffers; mfma_bf16_tflops / mfma_f32_tflops
 * = rate of a loop of nothing but independent 32x32x16 bf16 (32x32x2 fp32) MFMAs with two
 * wavefronts on every SIMD and operand bits that differ per lane (all-zero operands clock
 * higher than real data). Best of five launches each. launch_floor_us: mean duration, from
 * events attached to the dispatch, of a kernel of 128 workgroups that returns at once: what a
 * launch costs before it does anything. graph_node_floor_us: wall time per node of a graph of 200
 * such kernels, each depending on the one before, replayed on one stream. Allocates and frees 2 GiB of device
 * memory inside the call; synchronous; uses the null stream. Measurement aid: the roofline's
 * denominators stay the published peaks, these say how close any kernel can get here. */
typedef struct { double hbm_copy_gbs, mfma_bf16_tflops, mfma_f32_tflops, launch_floor_us, graph_node_floor_us; } lop_ceilings_t;
LOP_API int lop_measure_ceilings(lop_ceilings_t* out /* host */);

/* Time one layer's kernel of one band in isolation: `iters` launches on the plan's
 * compute stream between two events, on the plan's own scratch (contents are whatever
 * the last run left). Writes the mean milliseconds per launch. Measurement aid. */
LOP_API int lop_time_layer(lop_plan_t* plan, int band, int layer, const void* d_in, void* d_out,
                   int iters, float* ms_per_launch);

/* Name of the kernel instance that runs `layer` for `band`, as a profiler prints it without
 * namespace and argument list (empty string when the band computes no row of the layer),
 * copied into name[size]; *k_slices (optional) receives the number of slices its reduction
 * axis is cut into: 1 = one kernel, > 1 = that kernel followed by splitk_finish_kernel,
 * 0 = nothing to run. Measurement aid: lets a profile be grouped by kernel. */
LOP_API int lop_plan_layer_kernel(const lop_plan_t* plan, int band, int layer, char* name, size_t size,
                                  int* k_slices);

/* Run the whole chain `iters` times, bands in order on one stream, with a start and a stop
 * event attached to every kernel dispatch (the kernel's own duration, as a profiler's kernel
 * trace reports it), and write the mean milliseconds of each (band, layer) main kernel to
 * layer_ms[band * n_layers + layer] and of its splitk_finish_kernel (0 if none) to
 * finish_ms[...] (host, n_bands * n_layers floats each; finish_ms may be NULL, the finish
 * time is then not reported). No host copies. Synchronous. Measurement aid. */
LOP_API int lop_profile_chain(lop_plan_t* plan, const void* d_in, void* d_out, int iters, float* layer_ms,
                              float* finish_ms);

/* Enqueue only the bands' device-to-host copies, back to back on the plan's copy stream
 * (the transmission leg alone, to measure how much of it the pipelined run hides). */
LOP_API int lop_copy_chain(lop_plan_t* plan, const void* d_out, void* h_out);

/* Debug aid. With the environment variable LOP_GUARD_BYTES=<n> set when the library makes its
 * first device allocation, every device allocation of the library carries n bytes of a fixed
 * pattern in front and behind. Waits for the device, compares the guards of all live
 * allocations and returns the number of allocations (live, or freed since the process
 * started) whose guard was overwritten, i.e. that some kernel stored outside of; 0 when the
 * variable is not set; each finding is also reported on stderr. */
LOP_API int lop_debug_guard_check(void);

LOP_API void lop_plan_destroy(lop_plan_t* plan);
LOP_API const char* lop_strerror(int code);
LOP_API int lop_last_hip_error(void); /* raw hipError_t behind this thread's last LOP_ERR_HIP */

#ifdef __cplusplus
}
#endif
#endif /* LOP_H_ */

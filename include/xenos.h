/*
 * xenos.h -- C ABI of the MI355X (gfx950) linked-operator-chain CNN inference library.
 *
 * The interface follows the paper's problem statement (Section 6): the user hands over a
 * computation graph plus the hardware description (memory hierarchy, number of compute
 * units); an automatic optimiser (Sections 4.1-4.4) links adjacent operators and splits
 * them across the units; a runtime then executes the optimised model on input data
 * (Section 3).  Operator vocabulary: Table 3.
 *
 * Conventions
 *  - Opaque handles; every entry point returns a status and never throws.  On failure
 *    nothing is written through output pointers and xenos_last_error() holds a message.
 *  - HOST pointers: descriptors, operator parameters (fp32), hw info, options, JSON buffer.
 *    They are borrowed only for the duration of the call (parameters are copied).
 *  - DEVICE pointers: d_weights, d_workspace, d_input, d_output.  All device memory is owned
 *    by the caller (e.g. PyTorch tensors); the library never allocates device memory and
 *    never synchronises in xenos_run.
 *  - hip_stream is a hipStream_t passed as void* (NULL = the default stream).
 *  - One GPU; a plan may be run on one stream at a time.
 */
#ifndef XENOS_H
#define XENOS_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  XENOS_OK = 0,
  XENOS_EINVAL = 1,        /* NULL / out-of-range argument                     */
  XENOS_ESHAPE = 2,        /* operator shapes do not fit together              */
  XENOS_EUNSUPPORTED = 3,  /* valid graph, but outside what the kernels cover  */
  XENOS_ENOMEM = 4,        /* host allocation failed                           */
  XENOS_EDEVICE = 5        /* a HIP call failed                                */
} xenos_status;

typedef enum { XENOS_F32 = 0, XENOS_BF16 = 1 } xenos_dtype;
typedef enum { XENOS_NCHW = 0, XENOS_NHWC = 1 } xenos_layout;   /* graph I/O only */

/* Operator kinds: the members of the paper's operator library (Table 3) that a CNN graph
 * is built from before fusion.  Conv+Bn+Bias+Relu are fused to CBR by the optimiser
 * (Section 4.3); CBR followed by pooling is linked to CBRM / CBRA (Table 3). */
typedef enum {
  XENOS_OP_CONV = 0,            /* x.conv: cross-correlation, zero padding, floor output size, groups */
  XENOS_OP_BIAS = 1,            /* per-channel add                                                   */
  XENOS_OP_BN = 2,              /* inference batch-norm: gamma*(x-mean)/sqrt(var+eps)+beta            */
  XENOS_OP_RELU = 3,
  XENOS_OP_MAXPOOL = 4,         /* x.gampool                                                         */
  XENOS_OP_AVGPOOL = 5,
  XENOS_OP_GLOBAL_AVGPOOL = 6,
  XENOS_OP_ADD = 7,             /* x.add, two inputs of equal shape                                  */
  XENOS_OP_CONCAT = 8,          /* x.concat along channels, 2..4 inputs                              */
  XENOS_OP_FC = 9,              /* x.matmul as FullyConnected over the NCHW flattening of its input  */
  XENOS_OP_SLICE = 10,          /* channels [c_begin, c_begin + out_c) of the input (the inverse of x.concat) */
  XENOS_OP_SHUFFLE = 11,        /* channel shuffle of the ShuffleNet models (Section 7.1): with C = groups * m,
                                   output channel i * groups + j is input channel j * m + i                  */
  XENOS_OP_MATMUL = 12          /* x.matmul (Table 3; the MatmulX -> MatmulY row of Table 1): Y[M][N] = X[M][K] . W[N][K]^T (+ bias[N]).
                                   The rows are the tensor's first dimension: input M x K x 1 x 1, output M x out_c x 1 x 1,
                                   i.e. row-major [row][column] in memory under either layout name; any number of rows */
} xenos_op_kind;

typedef struct {
  int n, c, h, w;
  xenos_dtype dtype;            /* element type of the caller's buffer (graph input / output) */
  xenos_layout layout;
} xenos_tensor_desc;

/* One operator.  Tensor ids: 0 is the graph input, i + 1 is the output of ops[i]; ops must be
 * in topological order.  Parameter arrays are HOST fp32 and may be NULL where optional. */
typedef struct {
  xenos_op_kind kind;
  int n_inputs;
  int inputs[4];
  int out_c;                    /* conv, fc, matmul, slice                         */
  int kh, kw;                   /* conv, pool                                      */
  int stride_h, stride_w;       /* conv, pool (must be equal)                      */
  int pad_h, pad_w;             /* conv, pool (must be equal)                      */
  int groups;                   /* conv: 1 (dense) or == channels (depthwise); shuffle: number of groups */
  int ceil_mode;                /* pool                                            */
  int count_include_pad;        /* avgpool                                         */
  int c_begin;                  /* slice: first channel                            */
  float eps;                    /* bn                                              */
  const float* weight;          /* conv: [out_c][c/groups][kh][kw]; fc: [out_c][c*h*w]; matmul: [out_c][c] */
  const float* bias;            /* conv, fc (optional); bias op (required): [c]    */
  const float* gamma;           /* bn: [c] each                                    */
  const float* beta;
  const float* mean;
  const float* var;
} xenos_op_desc;

/* Hardware description the optimiser is given beside the graph (Section 6).  The planner sizes its partitions
 * from num_cu, lds_bytes_per_cu and l2_bytes; llc_bytes and hbm_bytes are informative.  Fixed for gfx950 and
 * not taken from here: 8 XCDs (workgroups are dealt to them round-robin) and the 160 KiB LDS limit of a launch. */
typedef struct {
  int num_cu;                   /* compute units that share the work (MI355X: 256)          */
  size_t lds_bytes_per_cu;      /* private memory per unit (MI355X: 160 KiB LDS)            */
  size_t l2_bytes;              /* shared cache per XCD (MI355X: 4 MiB)                     */
  size_t llc_bytes;             /* memory-side cache (MI355X: 256 MiB)                      */
  size_t hbm_bytes;             /* device memory                                           */
} xenos_hw_info;

/* link:  0 = operator by operator (the paper's Vanilla dataflow: every operator is one pass)
 *        1 = fused CBR only; pooling / add / concat stay separate passes (the "HO baseline")
 *        2 = operator linking on (Section 4.1): CBR + pool, shortcut add, concat-by-offset
 *        3 = 2 plus the chains whose intermediate tensor stays on chip (Table 1, ConvX -> ConvY): depthwise -> pointwise
 *            and pointwise -> depthwise (Section 2.2 example), a 1x1 squeeze convolution -> its 1x1 and 3x3 expand
 *            convolutions -> concat (-> max-pool), and, on the bf16 path, a first-layer 3x3 -> 3x3 convolution pair
 * split: 0 = every chain runs on ONE compute unit (no operator split; for tests)
 *        1 = DSP-aware operator split (Section 4.2): output channels first, then H/W, then (layers whose output tiles
 *            leave most units idle) the reduction, whose shares a summing pass adds in index order
 * compute: element type of activations and weights in HBM; accumulation is always fp32.
 * tile: 0 = planner's choice; 1..4 force a tile shape of the general conv kernel; 5 the halo-staged 3x3 kernel
 *       (7 / 8: with 128- / 64-channel tiles; 9 / 10: the same in its patch-linear form where one exists) and 6 the
 *       first-layer kernel for every chain they apply to, the other
 *       chains keep the planner's choice (tests, tuning). */
typedef struct {
  int link;
  int split;
  xenos_dtype compute;
  int tile;
} xenos_plan_opts;

typedef struct xenos_graph xenos_graph;
typedef struct xenos_plan xenos_plan;

/* Section 6 (the user supplies the computation graph): validates the operator list, infers
 * every tensor shape and copies descriptors and parameters.  output_tensor_id names the graph
 * output; output gives the dtype/layout the caller wants it in (n,c,h,w are checked if non-zero). */
xenos_status xenos_graph_create(const xenos_tensor_desc* input, const xenos_op_desc* ops, int n_ops,
                                int output_tensor_id, const xenos_tensor_desc* output,
                                xenos_graph** out);

/* Sections 4.1-4.4, the automatic optimiser: fusion pre-pass (Conv/Bn/Bias/Relu -> CBR), operator
 * linking (pattern table, Table 1) with per-edge layout assignment, then DSP-aware operator split
 * (feature-map partition over outC then H/W; parameter split K first, C/R/S as in-kernel reduction).
 * Host only; does not touch the device. */
xenos_status xenos_plan_link_split(const xenos_graph* graph, const xenos_hw_info* hw,
                                   const xenos_plan_opts* opts, xenos_plan** out);

/* Plan metadata (Section 4.1 "metadata"): sizes the caller must allocate, the output descriptor and
 * a JSON description of chains, tiles, layouts and algorithmic HBM bytes.  Any pointer may be NULL.
 * json_cap is the capacity of json in bytes; the text is truncated (and NUL-terminated) if larger;
 * *json_len receives the full length needed, NUL included. */
xenos_status xenos_plan_query(const xenos_plan* plan, size_t* weight_bytes, size_t* workspace_bytes,
                              xenos_tensor_desc* out_desc, char* json, size_t json_cap, size_t* json_len);

/* Packs the parameters in operand order (K-tile major, (r,s,c) contiguous; Section 4.2.2) into the
 * caller's device buffer d_weights (>= weight_bytes) and records d_workspace (>= workspace_bytes).
 * Both must be 256-byte aligned.  d_workspace may be NULL: the plan then runs through xenos_run_static only.
 * Synchronises hip_stream before returning. */
xenos_status xenos_plan_bind(xenos_plan* plan, void* d_weights, void* d_workspace, void* hip_stream);

/* Section 3, the runtime: enqueues the planned kernel sequence on hip_stream.  d_input / d_output
 * are device buffers in the dtype / layout of the graph's input / output descriptors.
 * Asynchronous; allocates nothing; returns XENOS_EDEVICE if a launch fails. */
xenos_status xenos_run(xenos_plan* plan, const void* d_input, void* d_output, void* hip_stream);

/* xenos_run with the intermediate tensors in d_workspace (256-byte aligned, at least workspace_bytes of
 * xenos_plan_query) instead of the workspace given to xenos_plan_bind, which is not touched.  A pass reads the plan and
 * the packed weights and writes only its workspace and its output, so several passes of ONE plan may be in flight at a
 * time, each on its own stream with its own workspace and output: kernels of one pass then fill the compute units that
 * the last round of tiles of another leaves idle (Section 4.2.1: no unit idle), and the gap behind a dependent launch of
 * one stream is covered by the other.  Passes that share a workspace or an output must follow each other on one
 * stream.  Same result as xenos_run, bit for bit; asynchronous; allocates nothing. */
xenos_status xenos_run_with(xenos_plan* plan, const void* d_input, void* d_output, void* d_workspace, void* hip_stream);

/* For callers that cannot allocate device memory or hand over a workspace (code under HIP-graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): xenos_run with the intermediate tensors in a workspace that is
 * part of the library's own device image, XENOS_STATIC_WORKSPACE_BYTES per GPU, held until the process ends.
 * Same arguments, same result and same asynchrony as xenos_run; the workspace given to xenos_plan_bind is not
 * touched.  Returns XENOS_EUNSUPPORTED when the plan needs a larger workspace (xenos_plan_query tells), and
 * XENOS_EDEVICE when the address of the static workspace cannot be obtained.  Calls no allocating routine.  The
 * first call on a device looks the workspace's address up (not to be made under stream capture).  All calls on one
 * GPU share the workspace, whatever the plan: calls that overlap in time on one GPU (two streams, two threads) race;
 * calls that follow each other on one stream do not.  Nothing is cleared between calls: every chain writes what a
 * later chain of the same pass reads. */
#define XENOS_STATIC_WORKSPACE_BYTES (32u << 20)
xenos_status xenos_run_static(xenos_plan* plan, const void* d_input, void* d_output, void* hip_stream);

/* Same result as xenos_run, for latency-bound (batch 1) use: the first call with a given (d_input, d_output)
 * pair captures the kernel sequence into a HIP graph (kernel nodes only; the runtime allocates host-side graph
 * objects on that call), later calls with the same pair replay it with one launch.  The pointers must stay
 * valid and the plan bound to the same buffers for as long as the pair is reused.  Asynchronous on hip_stream. */
xenos_status xenos_run_graph(xenos_plan* plan, const void* d_input, void* d_output, void* hip_stream);

/* Profiling-driven choice of the partition (the single-device form of Algorithm 1, Section 5: enumerate the legal
 * partition schemes of an operator, profile each, keep the fastest; a one-off search per model and platform).
 * For every convolution chain of a bound plan whose split planner found more than one legal tile shape / kernel,
 * each candidate is launched `reps` times on hip_stream and the fastest replaces the cost model's choice.  One full
 * pass runs first so that every buffer holds finite values of the real shapes; since workspace blocks are reused
 * along the pass, a chain is not guaranteed to be timed on its own input (the kernels' run time does not depend on
 * the values), and the call ends with a full pass that leaves d_output valid.  Chains whose plan structure depends on the choice (reduction
 * split, first-layer kernel, linked depthwise producer) keep it.  d_output is overwritten; the JSON of
 * xenos_plan_query reflects the result ("tuned":1); *n_changed (may be NULL) = chains whose choice changed.
 * Synchronises hip_stream.  Allocates no device memory. */
xenos_status xenos_plan_tune(xenos_plan* plan, const void* d_input, void* d_output, void* hip_stream,
                             int reps, int* n_changed);

/* Runs only chain `chain` of a bound plan (0 <= chain < number of chains in the JSON), reading and
 * writing the same buffers xenos_run would; used for per-chain timing. */
xenos_status xenos_run_chain(xenos_plan* plan, int chain, const void* d_input, void* d_output,
                             void* hip_stream);

/* Device probes for the measurement report (no part of the inference path): what this GPU attains, to put beside the
 * published peaks when a kernel's roofline fraction is quoted.  Both enqueue ONE kernel on hip_stream, asynchronously;
 * the caller times it (events on the same stream).  d_out is scratch of at least 8192 * hw->num_cu bytes.
 * xenos_probe_mfma: every compute unit runs `iters` rounds (rounded up to a multiple of four) of eight independent bf16
 * MFMA (32x32x16) accumulations with no memory instruction in the loop; *flops (host, may be NULL) receives the
 * floating-point operations of the launch.  `data` chooses the operand values, on which the sustained clock depends:
 * 0 = a few small values per lane, 1 = pseudo-random dense operands, 2 = pseudo-random with half of the pixel operand
 * zero (activations behind a ReLU); any other value is XENOS_EINVAL.
 * xenos_probe_read: streams `bytes` (a multiple of 16, 16-byte aligned) of device memory through 16-byte loads. */
xenos_status xenos_probe_mfma(const xenos_hw_info* hw, void* d_out, size_t out_bytes, int iters, int data, void* hip_stream, double* flops);
xenos_status xenos_probe_read(const xenos_hw_info* hw, const void* d_in, size_t bytes, void* d_out, size_t out_bytes, void* hip_stream);

/* Releases a graph or a plan (either handle type; NULL is ignored).  A plan holds a reference to
 * nothing of the graph after xenos_plan_link_split returns. */
void xenos_destroy(void* graph_or_plan);

/* Thread-local message of the last failing call on this thread ("" if none). */
const char* xenos_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* XENOS_H */

/*
 * libhap - per-device compute of HAP-style SPMD programs on one MI355X (gfx950).
 *
 * HAP (arXiv 2401.05965) shards every tensor of a training graph over m virtual
 * devices with UNEVEN ratios B_1..B_m chosen by a linear program (Sec. 5.1), and
 * each device executes its own slice of every instruction (Sec. 4.1, Fig.
 * "semantics"; Sec. 6).  This library is that per-device work:
 *
 *   host   hap_shard_ratios      the LP of Eq. (opt_B)
 *          hap_round_shards      integer sizes + ownership ranges (Sec. 5.1 rounding, Sec. 6 slicing)
 *   device hap_sharded_linear_*  the three MatMul sharding rules of Fig. "semantics" + the replicated rule
 *          hap_sharded_attn_*    softmax attention restricted to a head / batch slice
 *          hap_sfb_grad          sufficient-factor gradient rebuild (Sec. 2.3.2, Fig. "sfb"(c))
 *          hap_layernorm_*, hap_gelu_*, hap_add, hap_colsum   memory-bound row / element helpers
 *
 * Conventions
 *   - activations X[tokens x in], weights W[in x out], all row-major with an explicit leading
 *     dimension (elements);  Y = act(X W + b),  dX = dP W^T,  dW = X^T dP,  db = colsum(dP),
 *     dP = dY * act'(preact).
 *   - every function returns a hap_status (0 = OK); nothing throws or aborts.  Arguments are
 *     validated on the host before any launch.  hap_last_error() gives a thread-local detail string.
 *   - "device pointer" = memory of the current HIP device, owned by the caller, never freed or
 *     resized here.  The library allocates no device memory: scratch comes in through (ws, ws_bytes),
 *     sized by the matching hap_*_workspace() call; HAP_EWORKSPACE if too small.
 *   - device calls are asynchronous on `stream` (a hipStream_t passed as void*, NULL = default stream).
 *   - a shard of size 0 is legal (B_j >= 0 in Eq. (opt_B)): the call returns HAP_OK without launching.
 *   - outputs never alias inputs unless stated.
 */
#ifndef LIBHAP_H
#define LIBHAP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  HAP_OK = 0,
  HAP_EINVAL = 1,       /* NULL pointer, non-positive size, bad enum */
  HAP_ESHAPE = 2,       /* offsets not monotone / not ending at the dimension, ld too small, granule mismatch */
  HAP_EINFEASIBLE = 3,  /* LP has no feasible point (cannot happen for valid inputs) */
  HAP_EUNBOUNDED = 4,   /* LP unbounded (negative cost coefficients) */
  HAP_EWORKSPACE = 5,   /* ws NULL or ws_bytes below hap_*_workspace() */
  HAP_EDEVICE = 6,      /* HIP launch failed */
  HAP_EUNSUPPORTED = 7  /* valid request this build does not implement (e.g. head_dim other than 64 / 128) */
} hap_status;

const char* hap_strerror(int status);  /* static string */
const char* hap_last_error(void);      /* thread-local; valid until the next libhap call on this thread */
const char* hap_version(void);

/* ------------------------------------------------------------------ host: ratios and ranges --- */

/* One stage of the synthesized program (Sec. 3.2): a collective followed by computation.
 *   compute time on device j:  (flops_sharded * B_j + flops_fixed) / speed_j
 *   communication time:        comm_latency + comm_per_ratio * max_j B_j                         */
typedef struct {
  double flops_sharded;   /* flops of ops with a sharded dimension: scale with B_j (Sec. 3.2)      */
  double flops_fixed;     /* flops of ops without one: every device does all of them               */
  double comm_latency;    /* seconds                                                               */
  double comm_per_ratio;  /* seconds for the whole tensor; the largest shard decides (Sec. 5.1)    */
} hap_stage;

/* Eq. (opt_B):  min_B sum_i [ comm_i(B) + max_j comp_ij(B_j) ]  s.t. sum_j B_j = 1, B >= 0.
 * Solved as an LP in epigraph form by a dense two-phase simplex with Bland's rule (host, plain C).
 * speed[m] > 0 (flops/s), st[n_stages] with non-negative fields; ratios[m] out; objective (seconds)
 * out, may be NULL.  All host pointers.  m <= 256, n_stages <= 256.                              */
int hap_shard_ratios(int m, const double* speed, int n_stages, const hap_stage* st,
                     double* ratios, double* objective);

/* The cost model itself (Sec. 3.2): t(B) for given ratios; host pointers. */
int hap_iteration_time(int m, const double* speed, int n_stages, const hap_stage* st,
                       const double* ratios, double* seconds);

/* Different ratios across the model (Sec. 5.2): the stages are cut into g consecutive segments
 * [seg_offsets[k], seg_offsets[k+1]) (host array [g+1], 0 .. n_stages, no empty segment) and B becomes a
 * g x m matrix, row k for the tensors of segment k.  An All-To-All re-shards at every segment boundary
 * (its cost is the communication of the next segment's first stage), devices synchronise there, every
 * stage lies inside one segment, so each segment is Eq. (opt_B) by itself.  ratios: [g*m] out, row-major;
 * objective: sum of the segments' times (may be NULL).  hap_iteration_time_segments evaluates t for a
 * given g x m matrix.                                                                             */
int hap_shard_ratios_segments(int m, const double* speed, int n_stages, const hap_stage* st, int g, const int* seg_offsets,
                              double* ratios, double* objective);
int hap_iteration_time_segments(int m, const double* speed, int n_stages, const hap_stage* st, int g, const int* seg_offsets,
                                const double* ratios, double* seconds);

/* Sec. 5.1 rounding: sizes nearest to ratios[j]*dim_len, then +-1 on the shard whose size after the
 * move is closest to its target until they sum to dim_len (ties: .5 up, lowest device first, never
 * below 0).  Sizes are multiples of `granule` (>= 1, must divide dim_len).  offsets[j] = sum of the
 * sizes before j, offsets[m] = dim_len: device j owns [offsets[j], offsets[j+1])  (Sec. 6).
 * sizes[m] and offsets[m+1] are host output arrays.                                              */
int hap_round_shards(int m, const double* ratios, int64_t dim_len, int64_t granule,
                     int64_t* sizes, int64_t* offsets);

/* ------------------------------------------------------------------ host: program synthesis on small graphs --- */

/* Sec. 4: a distributed program is synthesized for a single-device graph so that it provably produces
 * the same loss.  Tensors are 2-D; node e's output is reference tensor e; inputs must be earlier nodes;
 * the last node is the loss (a Sum).  A property (e, form) states which collective turns the
 * distributed tensor into e on every device (Sec. 4.2); the theory holds the Hoare triples of
 * Fig. "semantics" for MatMul and the collectives, the Grouped-Broadcast and replicated-MatMul rules
 * of Sec. 4.4, and element-wise / transpose / sum rules of the same kind.  The search is the A* of
 * Fig. "a*" with its dominance pruning; the score adds to the time so far (Sec. 3.2) what every device
 * still has to compute with all remaining operations sharded and infinite bandwidth.  Restrictions: a
 * tensor is communicated at most once, loaded tensors never (Sec. 4.5); every tensor is computed once,
 * in graph order.  At most 16 nodes and 16 devices.                                                  */
typedef enum { HAP_OP_PLACEHOLDER = 0, HAP_OP_PARAMETER = 1, HAP_OP_MATMUL = 2, HAP_OP_UNARY = 3, HAP_OP_ADD = 4,
               HAP_OP_TRANSPOSE = 5, HAP_OP_SUM = 6 } hap_op;
typedef struct { int op; int a, b; int64_t rows, cols; } hap_graph_node;   /* a, b: input nodes (-1: none); rows x cols: output */
typedef enum { HAP_FORM_ID = 0, HAP_FORM_AG0 = 1, HAP_FORM_AG1 = 2, HAP_FORM_AR = 3 } hap_form;  /* replicated, sharded on 0 / 1, partial sums */
typedef enum { HAP_I_PLACEHOLDER = 0, HAP_I_PLACEHOLDER_SHARD = 1, HAP_I_PARAMETER = 2, HAP_I_PARAMETER_SHARD = 3,
               HAP_I_MATMUL = 4, HAP_I_UNARY = 5, HAP_I_ADD = 6, HAP_I_TRANSPOSE = 7, HAP_I_SUM = 8,
               HAP_I_ALL_REDUCE = 9, HAP_I_REDUCE_SCATTER = 10, HAP_I_ALL_GATHER = 11, HAP_I_GROUPED_BROADCAST = 12,
               HAP_I_ALL_TO_ALL = 13 } hap_instr_kind;
/* tensor: the reference tensor the instruction produces (computations, loads) or moves (collectives).
 * arg0, arg1: the sharded dimension of a *_SHARD load / Reduce-Scatter / All-Gather / Grouped-Broadcast,
 * (from, to) dimensions of an All-To-All, the forms (hap_form) of the inputs of a computation.        */
typedef struct { int kind; int tensor; int arg0, arg1; } hap_instr;
typedef struct { double latency, bandwidth; int elem_bytes; } hap_net;   /* seconds, bytes/s: the fitted linear model of Sec. 3.2 */
typedef struct { int placeholder_dims_mask, parameter_dims_mask;          /* bit d: the loads may shard dimension d       */
                 int grouped_broadcast, replicated_matmul, placeholder_replicated; } hap_synth_rules;   /* NULL = everything on */

/* The cheapest complete program for the given ratios (host pointers throughout).  program: room for
 * `capacity` instructions (HAP_EWORKSPACE if too few); seconds = t(Q, B); expanded (may be NULL) =
 * partial programs taken from the queue.  HAP_EINFEASIBLE if the rules admit no complete program.     */
int hap_synthesize(int n_nodes, const hap_graph_node* graph, int m, const double* ratios, const double* speed,
                   const hap_net* net, const hap_synth_rules* rules, hap_instr* program, int capacity, int* n_instr,
                   double* seconds, int64_t* expanded);
/* t(Q, B) of a given program (Sec. 3.2): a collective ends a stage; a stage costs its slowest device.  */
int hap_program_time(int n_nodes, const hap_graph_node* graph, int n_instr, const hap_instr* program, int m,
                     const double* ratios, const double* speed, const hap_net* net, double* seconds);

/* The stages of a program as Eq. (opt_B) takes them: stages[0] is the computation before the first
 * collective, every collective opens a new stage.  hap_iteration_time on the result equals
 * hap_program_time on the program.  stages: room for `capacity` (HAP_EWORKSPACE if too few).          */
int hap_program_stages(int n_nodes, const hap_graph_node* graph, int n_instr, const hap_instr* program, int m,
                       const hap_net* net, hap_stage* stages, int capacity, int* n_stages);
/* The iterative optimisation of Sec. 3.1: Q(s) = argmin_Q t(Q, B(s-1)), B(s) = argmin_B t(Q(s), B), from
 * ratios proportional to speed, until a step brings no gain or max_steps is reached; returns the best
 * (program, ratios[m], seconds) seen and the number of steps taken.                                   */
int hap_optimize(int n_nodes, const hap_graph_node* graph, int m, const double* speed, const hap_net* net,
                 const hap_synth_rules* rules, int max_steps, hap_instr* program, int capacity, int* n_instr,
                 double* ratios, double* seconds, int* steps);

/* ------------------------------------------------------------------ device: sharded linear --- */

typedef enum { HAP_F32 = 0, HAP_BF16 = 1 } hap_dtype;

/* Which MatMul rule of Fig. "semantics" the instruction follows (names: sharded axis of the layer). */
typedef enum {
  HAP_SHARD_BATCH = 0,      /* X rows sharded, W whole       -> Y rows sharded                     */
  HAP_SHARD_FEATURE = 1,    /* X whole, W columns sharded    -> Y columns sharded                  */
  HAP_SHARD_REDUCTION = 2,  /* X columns, W rows sharded     -> Y is a partial sum (to All-Reduce) */
  HAP_REPLICATED = 3        /* everything whole on every device (rule added for SFB, Sec. 4.3)     */
} hap_shard_mode;

typedef enum { HAP_ACT_NONE = 0, HAP_ACT_GELU_ERF = 1 } hap_act;

typedef struct {
  int64_t tokens, in_features, out_features; /* UNSHARDED logical sizes                              */
  int mode;                 /* hap_shard_mode                                                        */
  int m;                    /* number of virtual devices                                             */
  const int64_t* offsets;   /* host pointer, [m+1], from hap_round_shards over the sharded axis
                               (tokens / out_features / in_features); ignored for HAP_REPLICATED   */
  int io_dtype;             /* hap_dtype of X, W, bias, Y, preact, dY, dX.  Accumulation is fp32.   */
  int act;                  /* hap_act, applied after bias; must be NONE in REDUCTION mode          */
  int has_bias;             /* must be 0 in REDUCTION mode: bias belongs after the All-Reduce       */
  int64_t ldx, ldw, ldy;    /* leading dimensions (elements) of the X-like, W-like, Y-like buffers  */
  int operands_are_full;    /* 1: sharded tensors are passed whole; the library applies the range.
                               0: sharded tensors are passed as the device's compact slice
                                  (row 0 / column 0 of the buffer = first owned row / column).
                               Tensors the mode does not shard are always whole.                    */
} hap_linear_desc;

/* Y_j (and optionally the pre-activation) of device `shard_index`.
 *   BATCH:     Y[r_j,:]  = act(X[r_j,:] W + b)          X,Y(,preact) sharded on rows
 *   FEATURE:   Y[:,c_j]  = act(X W[:,c_j] + b[c_j])     W,bias,Y(,preact) sharded on columns
 *   REDUCTION: P_j       = X[:,k_j] W[k_j,:]            X sharded on columns, W on rows; Y whole [tokens x out]
 * X, W, bias (NULL iff !has_bias), Y, preact (NULL = do not save) are device pointers.
 * preact has Y's shape/ld and is required by the backward only when act != NONE.  The activation
 * is applied to the pre-activation as preact stores it (Y = act(round_to_io_dtype(XW + b))), the
 * point at which the backward evaluates act', whether or not the copy is kept.                     */
int hap_sharded_linear_fwd(const hap_linear_desc* d, int shard_index, const void* X, const void* W,
                           const void* bias, void* Y, void* preact, void* ws, size_t ws_bytes, void* stream);

/* Gradients of device `shard_index`.  dY has Y's layout, dX has X's, dW has W's (dtype dW_dtype,
 * leading dimension ldw), dbias has bias's layout but is always fp32.
 *   BATCH:     dX[r_j,:] exact;  dW, dbias are the device's partial sums over its rows
 *   FEATURE:   dX is a partial [tokens x in];  dW[:,c_j], dbias[c_j] exact
 *   REDUCTION: dX[:,k_j], dW[k_j,:] exact;  dbias must be NULL
 * Any of dX, dW, dbias may be NULL to skip it.  With act != NONE the call first forms
 * dP = dY * act'(preact) in ws (see hap_linear_bwd_workspace).                                    */
int hap_sharded_linear_bwd(const hap_linear_desc* d, int shard_index, const void* X, const void* W,
                           const void* preact, const void* dY, void* dX, void* dW, int dW_dtype,
                           float* dbias, void* ws, size_t ws_bytes, void* stream);

/* hap_sharded_linear_bwd with the activation backward of the layer that PRODUCED X folded into the dX product's
 * epilogue (Sec. 2.3.1: the chain fc1 -> GeLU -> fc2 of a transformer MLP; the backward of fc2 hands fc1 its dP):
 *     dX <- (dP W^T) * x_act'(x_preact)
 * x_preact (device, io_dtype) is that layer's saved pre-activation and has X's shape, layout and leading dimension
 * ldx (whole or compact exactly as X is); x_act is its hap_act.  The returned dX is then that layer's dP, and its own
 * backward is called with a descriptor whose act is NONE.  Defined only where dX is complete on the device (BATCH,
 * REDUCTION, REPLICATED): in FEATURE mode dX is a partial sum, the activation backward belongs after its All-Reduce,
 * and the call returns HAP_EINVAL.  x_act = HAP_ACT_NONE makes the call identical to hap_sharded_linear_bwd.
 * The result equals hap_sharded_linear_bwd followed by hap_gelu_bwd in place, rounding included (dX is rounded to
 * io_dtype before the multiplication in both); it saves that pass's read and write of dX.  Same workspace.          */
int hap_sharded_linear_bwd_dact(const hap_linear_desc* d, int shard_index, const void* X, const void* W,
                                const void* preact, const void* dY, void* dX, void* dW, int dW_dtype,
                                float* dbias, const void* x_preact, int x_act, void* ws, size_t ws_bytes, void* stream);

/* Workspace sizes.  The forward needs none; what hap_linear_fwd_workspace() reports (and the last 64 MiB of what
 * hap_linear_bwd_workspace() / hap_sfb_workspace() report) is OPTIONAL scratch that lets the GEMM engine split the
 * contracted axis over idle compute units when an output has too few tiles to fill the chip.  With a smaller
 * buffer, or ws = NULL in the forward / SFB calls, results are the same and only that optimisation is skipped.  */
size_t hap_linear_fwd_workspace(const hap_linear_desc* d, int shard_index);
size_t hap_linear_bwd_workspace(const hap_linear_desc* d, int shard_index);

/* ------------------------------------------------------------------ device: SFB rebuild --- */

/* dW[in x out] (+)= sum_i X_i[0:rows_i,:]^T dY_i[0:rows_i,:]      (Sec. 2.3.2, Fig. "sfb"(c))
 * One GEMM whose contracted axis is the concatenation of the m devices' gathered factors.
 *   X, dY   host arrays of m device pointers; X_i is [cap_i x in_features] with leading dimension ldx,
 *           dY_i is [cap_i x out_features] with ldy; cap_i >= rows_i (padded All-Gather layout) or
 *           cap_i == rows_i (grouped-Broadcast layout).  Rows >= rows_i are never read.
 *   rows    host array, rows_i >= 0 (0: that device contributes nothing)
 *   dW      device, fp32, leading dimension lddw; accumulate = 0 overwrites, 1 adds to the contents
 * m <= HAP_SFB_MAX_DEVICES.                                                                       */
#define HAP_SFB_MAX_DEVICES 64
int hap_sfb_grad(int m, const void* const* X, const void* const* dY, const int64_t* rows,
                 int64_t in_features, int64_t out_features, int64_t ldx, int64_t ldy, int in_dtype,
                 float* dW, int64_t lddw, int accumulate, void* ws, size_t ws_bytes, void* stream);
size_t hap_sfb_workspace(int m, const int64_t* rows, int64_t in_features, int64_t out_features);

/* hap_sfb_grad for callers that cannot allocate device memory or hand over a workspace: code under HIP graph capture,
 * tight serving / training loops, harnesses that forbid hipMalloc.  Same arguments and same results as hap_sfb_grad
 * given a workspace of HAP_SFB_STATIC_SCRATCH_BYTES, but the split-K partial tiles live in an array that is part of
 * the library's device image (each GPU the library runs on holds HAP_SFB_STATIC_SCRATCH_BYTES of it until the process
 * ends); the call allocates and frees nothing.  Limit: in_features * out_features <= HAP_SFB_STATIC_MAX_ELEMS
 * (HAP_EUNSUPPORTED beyond it, nothing launched).  All calls on one GPU share that GPU's array: calls that may run
 * concurrently on one GPU (different streams, different threads) race on it and must be serialised by the caller; the
 * array needs no clearing between calls (every partial tile is written before it is read).                          */
#define HAP_SFB_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
#define HAP_SFB_STATIC_MAX_ELEMS ((int64_t)8 << 20)
int hap_sfb_grad_static(int m, const void* const* X, const void* const* dY, const int64_t* rows,
                        int64_t in_features, int64_t out_features, int64_t ldx, int64_t ldy, int in_dtype,
                        float* dW, int64_t lddw, int accumulate, void* stream);

/* ------------------------------------------------------------------ device: MoE experts --- */

/* One fully-connected layer per expert of a Mixture-of-Experts layer whose EXPERT axis is sharded
 * unevenly (Sec. 7.6, "Uneven Placement of Experts"): device j owns the experts
 * [offsets[j], offsets[j+1]) - offsets from hap_round_shards over `experts`, any integer split,
 * a device may own none - and runs exactly those, all in one grouped launch; no expert is padded in.
 *   X     [experts x capacity x in_features]   tokens dispatched to each expert (row stride ldx)
 *   W     [experts x in_features x out_features] (row stride ldw),  bias [experts x out_features]
 *   Y     [experts x capacity x out_features]  (row stride ldy); preact and dY likewise, dX like X,
 *         dW like W (dtype dW_dtype), dbias [experts x out_features] fp32
 * Consecutive experts lie capacity*ldx, in_features*ldw, capacity*ldy, out_features elements apart.
 * operands_are_full = 1: pointers address expert 0 of the whole layer and the library steps to the
 * device's first expert; 0: they address the device's first expert (compact per-device buffers).
 * rows: DEVICE array of int32, one count per expert (indexed like the tensors), of the buffer rows
 * that hold a token, clamped to [0, capacity]; NULL = every row.  Rows at or beyond the count may
 * hold anything (NaN included): they influence no result, and the matching rows of Y, preact and dX
 * are left untouched; an expert with no token gets dW = 0 and dbias = 0.  The counts stay on the
 * device: no host synchronisation.                                                                */
typedef struct {
  int64_t experts, capacity, in_features, out_features;   /* UNSHARDED expert count                  */
  int m;
  const int64_t* offsets;   /* host, [m+1] over experts                                              */
  int io_dtype;             /* hap_dtype of X, W, bias, Y, preact, dY, dX; accumulation is fp32     */
  int act;                  /* hap_act, applied after the bias                                       */
  int has_bias;
  int64_t ldx, ldw, ldy;
  int operands_are_full;
} hap_moe_desc;

int hap_moe_linear_fwd(const hap_moe_desc* d, int shard_index, const void* X, const void* W, const void* bias,
                       const int32_t* rows, void* Y, void* preact, void* ws, size_t ws_bytes, void* stream);
/* Any of dX, dW, dbias may be NULL to skip it.  ws holds dP = dY * act'(preact) and column-sum partials
 * (required when act != NONE or dbias is given).  As for the linear layers, the forward's workspace and
 * the last 64 MiB of the backward's are OPTIONAL scratch that lets a device with few experts split the
 * contracted axis over idle compute units; results are the same without it.                         */
int hap_moe_linear_bwd(const hap_moe_desc* d, int shard_index, const void* X, const void* W, const void* preact,
                       const void* dY, const int32_t* rows, void* dX, void* dW, int dW_dtype, float* dbias,
                       void* ws, size_t ws_bytes, void* stream);
/* hap_moe_linear_bwd with the activation backward of the expert layer that PRODUCED X folded into the dX products' epilogue
 * (the experts' fc1 -> GeLU -> fc2 chain, Sec. 7.6): dX_e <- (dP_e W_e^T) * x_act'(x_preact_e) on the expert's token rows.
 * x_preact (device, io_dtype) has X's shape and layout [experts x capacity x ldx]; the returned dX is that layer's dP and its
 * own backward is called with a descriptor whose act is NONE.  Expert parallelism shards the expert axis, so dX is always
 * complete on the device.  x_act = HAP_ACT_NONE makes the call identical to hap_moe_linear_bwd.  Same workspace.              */
int hap_moe_linear_bwd_dact(const hap_moe_desc* d, int shard_index, const void* X, const void* W, const void* preact,
                            const void* dY, const int32_t* rows, void* dX, void* dW, int dW_dtype, float* dbias,
                            const void* x_preact, int x_act, void* ws, size_t ws_bytes, void* stream);
size_t hap_moe_linear_fwd_workspace(const hap_moe_desc* d, int shard_index);
size_t hap_moe_linear_bwd_workspace(const hap_moe_desc* d, int shard_index);

/* ------------------------------------------------------------------ device: attention slice --- */

/* Softmax attention per (batch, head): S = Q K^T / sqrt(head_dim), P = softmax_keys(S), O = P V;
 * no mask, no dropout.  The tensors passed are WHOLE [batch, seq, heads, head_dim] views addressed by
 * strides (elements; head_dim contiguous); the device computes only its heads (shard_over_heads = 1)
 * or its batch entries (0), i.e. the index range [offsets[j], offsets[j+1]).  With m = 1 and
 * offsets = {0, heads or batch} the whole tensor is computed (use this for compact slices).       */
typedef struct {
  int64_t batch, heads, seq, head_dim;     /* head_dim in {64, 128}                                   */
  int shard_over_heads;
  int m;
  const int64_t* offsets;                  /* host, [m+1] over heads or batch                          */
  int io_dtype;                            /* HAP_BF16                                                 */
  int64_t stride_b, stride_s, stride_h;    /* of Q, K, V and dQ, dK, dV                                */
  int64_t o_stride_b, o_stride_s, o_stride_h; /* of O and dO; all three 0 = same as above (e.g. Q|K|V
                                              are column blocks of one [tokens x 3*heads*d] buffer
                                              while O is [tokens x heads*d])                        */
} hap_attn_desc;

/* lse: device fp32 [batch x heads x seq] (whole-tensor indexing), log-sum-exp of each query row,
 * written for the slice; needed by the backward.  The forward uses no workspace (ws may be NULL).
 * The backward's workspace (hap_attn_bwd_workspace: two fp32 per (batch, head, query) of the whole
 * tensor) holds D = rowsum(dO * O) and lse * log2(e).  All tensor pointers 16-byte aligned, strides
 * multiples of 8 elements, (seq + 64) * stride_s below 2^30 elements (HAP_EUNSUPPORTED otherwise);
 * rows past the sequence end are never read (tile loads are bounded by a buffer descriptor that ends
 * with the last valid row of the (batch entry, head) being processed).                              */
int hap_sharded_attn_fwd(const hap_attn_desc* d, int shard_index, const void* Q, const void* K, const void* V,
                         void* O, float* lse, void* ws, size_t ws_bytes, void* stream);
int hap_sharded_attn_bwd(const hap_attn_desc* d, int shard_index, const void* Q, const void* K, const void* V,
                         const void* O, const float* lse, const void* dO, void* dQ, void* dK, void* dV,
                         void* ws, size_t ws_bytes, void* stream);
size_t hap_attn_bwd_workspace(const hap_attn_desc* d, int shard_index);

/* ------------------------------------------------------------------ device: row / element helpers --- */

/* LayerNorm over the last axis, biased variance, eps = 1e-5.  x,y [rows x n] (ld = n), gamma/beta [n]
 * in io_dtype; mean, rstd fp32 [rows] saved for the backward.  n <= 2048 (HAP_EUNSUPPORTED beyond);
 * 16-byte aligned pointers with n a multiple of 16 / sizeof(element) take the vector path.          */
int hap_layernorm_fwd(int64_t rows, int64_t n, int io_dtype, const void* x, const void* gamma, const void* beta,
                      void* y, float* mean, float* rstd, void* stream);
/* dx in io_dtype; dgamma, dbeta fp32 [n], overwritten (with zeros when rows == 0: the partial sums of a device
 * whose shard is empty).  ws from hap_layernorm_bwd_workspace.
 * dresidual: NULL, or [rows x n] in io_dtype that is added to dx before the one rounding to io_dtype (a
 * pre-LayerNorm layer's gradient on the residual path, which bypasses the normalisation); it may be dx
 * itself, no other aliasing.                                                                        */
int hap_layernorm_bwd(int64_t rows, int64_t n, int io_dtype, const void* x, const void* gamma, const float* mean,
                      const float* rstd, const void* dy, const void* dresidual, void* dx, float* dgamma, float* dbeta,
                      void* ws, size_t ws_bytes, void* stream);
size_t hap_layernorm_bwd_workspace(int64_t rows, int64_t n);

/* out[r,c] = dy[r,c] * gelu'(preact[r,c])   (erf form)                                            */
int hap_gelu_bwd(int64_t rows, int64_t cols, int io_dtype, const void* preact, int64_t ldp, const void* dy,
                 int64_t lddy, void* out, int64_t ldo, void* stream);
/* out = a + b (+ bias broadcast over rows if bias != NULL); out may alias a or b.                  */
int hap_add(int64_t rows, int64_t cols, int io_dtype, const void* a, int64_t lda, const void* b, int64_t ldb,
            const void* bias, void* out, int64_t ldo, void* stream);
/* out[c] = sum_r a[r,c], fp32 out, overwritten.  ws from hap_colsum_workspace.                     */
int hap_colsum(int64_t rows, int64_t cols, int io_dtype, const void* a, int64_t lda, float* out,
               void* ws, size_t ws_bytes, void* stream);
size_t hap_colsum_workspace(int64_t rows, int64_t cols);

/* ------------------------------------------------------------------ device: uneven All-Gather data movement --- */

/* The copies one device performs around an All-Gather of a tensor [rows x cols] that is sharded
 * unevenly along `dim` (Sec. 2.2; Sec. 2.3.1, Fig. "comm_opt").  Collective libraries gather
 * equal-size pieces, so either every shard is padded to capacity = max_j size_j along `dim` before the
 * exchange and trimmed after it (padded All-Gather), or every shard travels at its own size (grouped
 * Broadcast).  Either way piece j ends up at [offsets[j], offsets[j+1]) of the sharded axis of `out`.
 * The exchange itself is not part of this library.  Element type is opaque: elem_bytes in {1,2,4,8};
 * leading dimensions are in elements; no alignment is required (16-byte accesses when everything
 * allows, smaller powers of two otherwise).  Bit-exact by construction.                             */
typedef struct {
  int64_t rows, cols;       /* the FULL tensor                                                       */
  int dim;                  /* 0: sharded over rows, 1: over columns                                 */
  int m;                    /* devices, <= HAP_SFB_MAX_DEVICES                                       */
  const int64_t* offsets;   /* host, [m+1] over the sharded axis                                     */
  int elem_bytes;
} hap_gather_desc;

/* max_j size_j: the extent of a padded slot along `dim` (-1 on a bad descriptor).                   */
int64_t hap_allgather_capacity(const hap_gather_desc* d);
/* "Pad": copies device shard_index's shard ([size_j x cols] or [rows x size_j], ld_shard) to the front
 * of its send slot (ld_slot).  The rest of the slot is left as it is: what the padding holds is never
 * looked at.                                                                                        */
int hap_allgather_pad(const hap_gather_desc* d, int shard_index, const void* shard, int64_t ld_shard,
                      void* slot, int64_t ld_slot, void* stream);
/* "Trim" / place: out[range of j along dim] = first size_j rows (dim 0) or columns (dim 1) of pieces[j],
 * for all j in one launch.  pieces, ld_pieces: HOST arrays [m] (device pointers, leading dimensions);
 * padded layout: pieces[j] = slots + j * slot_extent, ld = cols (dim 0) or capacity (dim 1); grouped
 * layout: each shard's own buffer and width.  Empty shards may have NULL pieces.  out must not overlap
 * any piece.                                                                                        */
int hap_allgather_assemble(const hap_gather_desc* d, const void* const* pieces, const int64_t* ld_pieces,
                           void* out, int64_t ld_out, void* stream);
/* The collective libraries' Reduce-Scatter wants equal shards too (Sec. 2.3.1, first paragraph): before it, a device
 * cuts its full [rows x cols] partial tensor (device, ld_full elements) into m slots of capacity size along dim -
 * slot j = the range of shard j followed by zeros, which add nothing to the sums.  slots: host array of m device
 * pointers, slot j [capacity x cols] (dim 0) or [rows x capacity] (dim 1) with ld_slots[j] elements per row; columns
 * beyond the slot's width are not written.  One launch.  After the collective the device's own slot is trimmed with
 * hap_allgather_assemble on a one-piece descriptor.                                                             */
int hap_reducescatter_split(const hap_gather_desc* d, const void* full, int64_t ld_full, void* const* slots,
                            const int64_t* ld_slots, void* stream);

/* ------------------------------------------------------------------ diagnostics --- */

/* Issue-rate probe for the roofline report: 256 blocks x 8 waves run `iters` rounds of 8 independent
 * v_mfma_f32_32x32x16_bf16 on register operands (no memory traffic).  random_operands != 0 uses
 * pseudo-random operand values, which draw more power than constants and show the sustained clock a
 * real GEMM can expect.  scratch: device, >= 256*512 floats, overwritten.  *flops (host, may be NULL)
 * receives the floating-point operations of one launch; the caller times the launch.              */
int hap_probe_mfma_bf16(int random_operands, int iters, float* scratch, double* flops, void* stream);
/* Compute units and peak engine clock (kHz) of the current device, for the report's derivation of the roofline
 * (units x clock x 4096 bf16 flop per clock and unit).  Either pointer may be NULL.                        */
int hap_device_info(int* compute_units, int* clock_khz);

#ifdef __cplusplus
}
#endif
#endif /* LIBHAP_H */

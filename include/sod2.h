/*
 * sod2.h -- C ABI of the MI355X-native SoD2 hot path.
 *
 * The library executes a dynamic DNN whose tensor shapes are symbolic
 * expressions resolved by Rank and Dimension Propagation (RDP), as fused
 * operator groups over a pre-planned memory arena (Sections 4.1 - 4.4 of the
 * SoD2 paper).  Five calls form the path:
 *
 *   sod2_graph_build  extended computational graph G (Section 4.1, item G;
 *                     operator classes of Section 3, Table 2)
 *   sod2_rdp_infer    RDP fixed point (Alg. 1, Tables 3 and 4)
 *   sod2_plan         fusion groups (4.2), sub-graph partition and static
 *                     execution order (4.3), kernel-version rules (4.4.2)
 *   sod2_bind         per input: evaluate the symbols, peak-first arena
 *                     offsets (4.4.1), kernel version and launch geometry
 *   sod2_run          launch the fused HIP kernels on a stream
 *
 * Conventions
 *   - All handles are opaque, host side, owned by the library until the
 *     matching *_destroy.  Handles are not thread safe.
 *   - Every pointer named "host" is host memory read during the call only.
 *     Device pointers (arena, weights, inputs, outputs) are owned by the
 *     caller; the library never allocates or frees device memory in sod2_run.
 *   - Every function returns a sod2_status; on failure out-parameters are
 *     untouched and sod2_last_error() describes the failure (thread local).
 */
#ifndef SOD2_H
#define SOD2_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t sod2_status;
enum {
  SOD2_OK = 0,
  SOD2_ERR_INVALID_ARG = -1,
  SOD2_ERR_SYMBOL_OUT_OF_RANGE = -2,
  SOD2_ERR_SHAPE_MISMATCH = -3,   /* producer and consumer disagree on a known constant */
  SOD2_ERR_UNRESOLVED_SHAPE = -4, /* a nac dim reaches a point that needs its value */
  SOD2_ERR_ARENA_TOO_SMALL = -5,
  SOD2_ERR_UNSUPPORTED = -6,
  SOD2_ERR_HIP = -7,
  SOD2_ERR_BUFFER_TOO_SMALL = -8,
  SOD2_ERR_NONCAUSAL_PLAN = -9,   /* offsets used before a Switch differ from the final plan */
  SOD2_ERR_SCRATCH_TOO_SMALL = -10 /* sod2_run_static: a split-K contraction needs more than the static buffer */
};

enum { SOD2_F32 = 0, SOD2_BF16 = 1, SOD2_I64 = 2, SOD2_I32 = 3 };
enum { SOD2_INTER = 0, SOD2_INPUT = 1, SOD2_WEIGHT = 2, SOD2_HOSTCONST = 3 };

/* Operator kinds (ONNX names, Table 2, plus the <Switch, Combine> pair).  Inputs, where the ONNX
 * signature is narrowed:
 *   Slice: data, starts, ends, axes.  CacheAppend: cache (a session tensor), new rows; the result is
 *   the cache extended in place.  ScatterRows: data, row indices, rows (a copy of data with those rows
 *   replaced).  Resize: data, sizes (nearest neighbour, floor(i * D / S) per axis).  Upsample: data,
 *   whole-number factors (a float HOSTCONST, one per dim).  Range: start, limit, delta (one-element
 *   integer tensors).  Expand: data, shape.  ConstantOfShape: shape.  EyeLike: a matrix.  OneHot:
 *   indices, depth (one-element integer tensor), values = float HOSTCONST [off, on]; last axis.
 *   TopK: data, k (one-element integer tensor); two results, values then positions; last axis,
 *   largest first, of equal entries the lower position first.  MaxUnpool (channels last): data x, int64 indices of the
 *   same shape (positions in the flattened result, distinct; positions outside it are ignored), output_shape (a short
 *   int tensor whose values are the result's shape; Table 2: ISVDOS); the rest of the result is zero.
 *   GroupNorm (GroupNormalization, channels last): data
 *   [N, ..., C], scale [C], bias [C]; per sample and group of C / groups channels, mean and biased variance over the
 *   group's channels at every position.  AveragePool (channels last, like MaxPool): the mean over the window
 *   positions inside the input (padding is not counted; 0 <= pad < kernel).  Round: to the nearest integer, halves
 *   to the even one.  NMS (non-maximum suppression; Table 2: execution determined): scores [N] and boxes [N, 4]
 *   (x1, y1, x2, y2 with x1 <= x2, y1 <= y2), both f32, N <= 4096, no NaN; boxes are visited by decreasing score
 *   (equal scores: increasing index) and kept unless one already kept overlaps them by more than the threshold,
 *   decided in fp32 as intersection > threshold * ((area_a + area_b) - intersection); result: the kept boxes'
 *   indices in visiting order, int64, a vector whose length is known once the operator has run (handled like
 *   NonZero's count).  Switch: data, predicate (one float);
 *   two results: taken when predicate <= threshold, taken when predicate > threshold.  Switch and Combine forward
 *   storage and write none: their results must not be graph outputs (sod2_plan: SOD2_ERR_UNSUPPORTED; an operator
 *   behind the Combine, e.g. a Cast to its own type, makes the copy).                                          */
enum {
  SOD2_OP_SHAPE = 0, SOD2_OP_GATHER, SOD2_OP_CONCAT, SOD2_OP_RESHAPE, SOD2_OP_SLICE,
  SOD2_OP_TRANSPOSE, SOD2_OP_MATMUL, SOD2_OP_CONV, SOD2_OP_ADD, SOD2_OP_MUL, SOD2_OP_RELU,
  SOD2_OP_GELU, SOD2_OP_SIGMOID, SOD2_OP_CAST, SOD2_OP_SOFTMAX, SOD2_OP_LAYERNORM,
  SOD2_OP_REDUCEMEAN, SOD2_OP_MAXPOOL, SOD2_OP_ARGMAX, SOD2_OP_CACHEAPPEND, SOD2_OP_NONZERO,
  SOD2_OP_SWITCH, SOD2_OP_COMBINE, SOD2_OP_SCATTERROWS, SOD2_OP_RESIZE, SOD2_OP_RANGE, SOD2_OP_EXPAND,
  SOD2_OP_UPSAMPLE, SOD2_OP_CONSTANTOFSHAPE, SOD2_OP_EYELIKE, SOD2_OP_ONEHOT, SOD2_OP_TOPK, SOD2_OP_GROUPNORM, SOD2_OP_MAXUNPOOL,
  SOD2_OP_AVERAGEPOOL, SOD2_OP_ROUND, SOD2_OP_NMS, SOD2_OP_COUNT
};

#define SOD2_MAX_RANK 8

typedef struct {
  const char* name;          /* host, copied */
  int32_t dtype;             /* SOD2_F32 ... */
  int32_t role;              /* SOD2_INTER ... */
  int32_t rank;              /* -1: shape undeclared, to be inferred by RDP */
  const char* const* dims;   /* rank strings: an integer, a symbol name, or a '+' sum of those */
  const void* host_data;     /* HOSTCONST only: int64 / int32 / float32 values, copied */
  int64_t host_count;        /* number of elements of host_data */
  int32_t is_output;         /* written to the caller's output buffer instead of the arena */
  int32_t session;           /* persists across calls (a KV cache): placed first in the arena */
  const char* const* capacity_dims; /* session only: dims the storage is sized for, else NULL */
} sod2_tensor_desc;

/* Integer attributes per kind, in this order:
 *   Gather/Concat: axis.  Transpose: the permutation.  MatMul: transB.  Conv: stride, pad.
 *   Softmax: causal.  ReduceMean: keepdims, then the axes.  MaxPool, AveragePool: kernel, stride, pad.
 *   EyeLike: the diagonal k.  GroupNorm: the number of groups.  NMS: the largest number of boxes to keep (0: no limit).
 * Float attribute: LayerNorm and GroupNorm epsilon; Switch threshold; ConstantOfShape value; NMS overlap threshold. */
typedef struct {
  int32_t kind;
  int32_t n_inputs;
  const int32_t* inputs;     /* tensor ids */
  int32_t n_outputs;
  const int32_t* outputs;
  int32_t n_iattr;
  const int64_t* iattr;
  double fattr;
} sod2_op_desc;

typedef struct {
  int32_t n_symbols;
  const char* const* symbol_names;
  const int64_t* symbol_lo;  /* declared range of each symbol, both ends included */
  const int64_t* symbol_hi;
  int32_t n_tensors;
  const sod2_tensor_desc* tensors;
  int32_t n_ops;
  const sod2_op_desc* ops;
} sod2_graph_desc;

/* The four optimisation switches the paper's breakdown study names (Section 5.3), and in-place reuse. */
typedef struct {
  int32_t fusion;  /* RDP-enabled fusion; 0: one group per operator                       */
  int32_t sep;     /* static execution planning; 0: node order                            */
  int32_t dmp;     /* peak-first arena plan; 0: best-fit greedy in execution order        */
  int32_t mvc;     /* multi-version kernels; 0: one version (128 x 128 x 64 tile) for every shape  */
  int32_t inplace; /* a group's result may take over the storage of an operand that dies there */
  /* Limits of the fusion rules; 0 selects the default.  max_versions: most code versions a fused elementwise group
   * may need (Section 4.2, Fig. 4: two per dim pair that RDP can prove neither equal nor 1; default 8, the largest
   * bucket of Fig. 8; 1: only proven chains fuse).  The others state what the kernels behind the plan can fuse --
   * they shape the groups, never a value: the head size of the fused attention group (default 64), the most rows a
   * CacheAppend inside it may add (4), and for a LayerNorm run as the prologue of a contraction the most rows (8),
   * the largest normalised extent (1024) and the multiple it must be of (64). */
  int32_t max_versions;
  int32_t attn_head_dim, append_max_rows, prologue_max_rows, prologue_max_k, prologue_k_multiple;
  /* fold_ln = 1: a LayerNorm that reads the result of a contraction group and feeds one MatMul becomes that group's
   * second result (one kernel fewer per LayerNorm); its extent must be a multiple of fold_k_multiple (0: 64). */
  int32_t fold_ln, fold_k_multiple;
} sod2_plan_opts;

typedef struct sod2_graph_s sod2_graph_t;
typedef struct sod2_rdp_s sod2_rdp_t;
typedef struct sod2_plan_s sod2_plan_t;
typedef struct sod2_binding_s sod2_binding_t;

/* -- graph (Section 4.1, G; Section 3 classes) -------------------------------------------- */
/* Copies the description.  SOD2_ERR_INVALID_ARG for what no later stage could make sense of: tensor ids out of
 * range, a tensor written twice, a graph output that no operator produces, an operator on a cycle or unreachable
 * from the inputs (the operators must form a DAG), a wrong input / output count, attributes out of their range (a Transpose attribute that is no permutation,
 * a window with kernel < 1, stride < 1 or pad >= kernel, ...).  Shapes that contradict each other are found by
 * sod2_rdp_infer / sod2_plan (SOD2_ERR_SHAPE_MISMATCH); extents that are negative, or tensors beyond 2^44 bytes, at
 * the symbols of a call by sod2_bind (SOD2_ERR_SHAPE_MISMATCH). */
sod2_status sod2_graph_build(const sod2_graph_desc* desc_host, sod2_graph_t** out);
void sod2_graph_destroy(sod2_graph_t*);
/* class of operator op: 0 ISDO, 1 ISDOS, 2 ISVDOS, 3 EDO (Table 2) */
sod2_status sod2_graph_op_class(const sod2_graph_t*, int32_t op, int32_t* cls);
/* the same for an operator kind (sod2_op_kind), without a graph */
sod2_status sod2_op_kind_class(int32_t kind, int32_t* cls);

/* -- RDP (Alg. 1) ------------------------------------------------------------------------- */
sod2_status sod2_rdp_infer(const sod2_graph_t*, sod2_rdp_t** out);
/* same analysis visiting the operators in the given order (a permutation of 0..n_ops-1);
 * the fixed point must not depend on it (Section 4.1, lattice argument) */
sod2_status sod2_rdp_infer_ordered(const sod2_graph_t*, const int32_t* order_host, int32_t n, sod2_rdp_t** out);
void sod2_rdp_destroy(sod2_rdp_t*);
typedef struct {
  int32_t cls;        /* 0 known constant, 1 symbolic constant, 2 operation-inferred, 3 nac */
  int64_t value;      /* cls 0 only */
  char expr[120];     /* canonical expression text (truncated if longer) */
} sod2_dim_info;
/* rank = -1 when the whole shape is nac; dims must hold SOD2_MAX_RANK entries */
sod2_status sod2_rdp_query(const sod2_rdp_t*, int32_t tensor, int32_t* rank, sod2_dim_info* dims);
sod2_status sod2_rdp_sweeps(const sod2_rdp_t*, int32_t* sweeps);
/* canonical text of all S- and V-maps.  Writes at most cap bytes (NUL terminated), stores the
 * full length in *needed; returns SOD2_ERR_BUFFER_TOO_SMALL when cap was not enough. */
sod2_status sod2_rdp_dump(const sod2_rdp_t*, char* buf_host, size_t cap, size_t* needed);

/* -- plan (Sections 4.2, 4.3, 4.4.2) -------------------------------------------------------- */
sod2_status sod2_plan(const sod2_graph_t*, const sod2_rdp_t*, const sod2_plan_opts* opts_host /* NULL: all on */,
                      sod2_plan_t** out);
void sod2_plan_destroy(sod2_plan_t*);
sod2_status sod2_plan_counts(const sod2_plan_t*, int32_t* n_groups, int32_t* n_subgraphs, int32_t* n_switches);
sod2_status sod2_plan_dump(const sod2_plan_t*, char* buf_host, size_t cap, size_t* needed);
/* The plan as records (the text dump stays the canonical form for byte comparison).  Groups are numbered
 * 0 .. n_groups-1 in planned execution order (sub-graph by sub-graph, Section 4.3).  ops_host / ins_host receive up
 * to the given capacities of the member operators (Section 4.2: the operators fused into one kernel) and of the
 * tensors the group reads from outside itself; info->n_ops / n_ins always hold the full counts. */
enum { SOD2_G_GEMM = 0, SOD2_G_CONV, SOD2_G_LAYERNORM, SOD2_G_SOFTMAX, SOD2_G_MAXPOOL, SOD2_G_REDUCEMEAN, SOD2_G_ARGMAX,
       SOD2_G_CACHEAPPEND, SOD2_G_NONZERO, SOD2_G_GATHER, SOD2_G_ELTWISE, SOD2_G_ATTENTION, SOD2_G_SCATTER, SOD2_G_RESIZE,
       SOD2_G_CONCAT, SOD2_G_RANGE, SOD2_G_FILL, SOD2_G_ONEHOT, SOD2_G_TOPK, SOD2_G_GROUPNORM, SOD2_G_MAXUNPOOL, SOD2_G_AVGPOOL, SOD2_G_NMS, SOD2_G_COPY };
typedef struct {
  int32_t gid;        /* group id: the smallest operator id in the group */
  int32_t kind;       /* SOD2_G_* */
  int32_t out;        /* tensor the group writes */
  int32_t out2;       /* second result (TopK: the positions), or -1 */
  int32_t n_ops, n_ins;
  int32_t subgraph;   /* sub-graph the group is planned in */
  int32_t sg_class;   /* of that sub-graph: 0 every shape constant, 1 symbolic and constant, 2 execution determined (Fig. 8) */
  int32_t inplace_of; /* tensor whose storage the result takes over, or -1 */
  int32_t versions;   /* code versions of the fused loop nest (Fig. 4): 1 when every broadcast pair is proven */
} sod2_group_info;
sod2_status sod2_plan_query_group(const sod2_plan_t*, int32_t index, sod2_group_info* info_host,
                                  int32_t* ops_host, int32_t ops_cap, int32_t* ins_host, int32_t ins_cap);

/* -- bind (Section 4.4.1) ------------------------------------------------------------------- */
/* symbol_values_host: one value per declared symbol, in declaration order.  For graphs with
 * Switch operators the arena plan depends on the decisions; sod2_bind plans as if every branch
 * ran and sod2_run re-plans after each decision (Section 4.3: a sub-graph after an
 * execution-determined operator is planned once that operator has executed).  The size reported by
 * sod2_binding_arena_bytes is then that of the all-branches plan; a particular path usually needs
 * less but may need more, in which case sod2_run stops at the Switch with SOD2_ERR_ARENA_TOO_SMALL
 * (nothing after it launched), sod2_run_arena_bytes reports the size needed, and the call can be
 * repeated with a larger arena. */
sod2_status sod2_bind(const sod2_plan_t*, const int64_t* symbol_values_host, int32_t n_symbols, sod2_binding_t** out);
/* pure planning with a given decision vector (1 = the skip output of the Switch is taken); no run */
sod2_status sod2_bind_decided(const sod2_plan_t*, const int64_t* symbol_values_host, int32_t n_symbols,
                              const int32_t* decisions_host, int32_t n_decisions, sod2_binding_t** out);
/* The same for graphs with execution-determined extents (NonZero and NMS, Table 2's EDO class; Section 4.3):
 * exec_values_host = the counts found by the NonZero / NMS operators that have executed so far, in
 * execution order.  One still to run is planned at its upper bound, the element count of its first
 * input (this is also what sod2_bind does for all of them).  sod2_run reads each count back when the
 * operator has run and plans what follows with it; the exact plan usually needs less than the
 * upper-bound plan but may need more (first fit is not monotone in the sizes): then sod2_run stops
 * there with SOD2_ERR_ARENA_TOO_SMALL as described for Switch.  A count outside
 * [0, element count of the input] is SOD2_ERR_INVALID_ARG. */
sod2_status sod2_bind_executed(const sod2_plan_t*, const int64_t* symbol_values_host, int32_t n_symbols,
                               const int32_t* decisions_host, int32_t n_decisions,
                               const int64_t* exec_values_host, int32_t n_exec_values, sod2_binding_t** out);
void sod2_binding_destroy(sod2_binding_t*);
/* bytes the arena passed to sod2_run must have; peak of summed live tensor bytes */
sod2_status sod2_binding_arena_bytes(const sod2_binding_t*, size_t* arena_bytes, size_t* peak_live_bytes);
sod2_status sod2_binding_dump(const sod2_binding_t*, char* buf_host, size_t cap, size_t* needed);
/* One tensor of the bound plan (Section 4.4.1: sizes, lifetimes and offsets exist once the symbols are bound).
 * executed = 0: no executed group writes it in this binding (a skipped branch, a folded or fused-away tensor): the
 * other fields are then unset.  where: 0 planned in the arena (offset, bytes, life valid), 1 a session slot at the
 * arena's bottom (offset, bytes valid), 2 the storage of another tensor taken over in place (base = that tensor),
 * 3 caller memory (a graph output).  sod2_run_query_tensor answers for the plan the last run executed. */
typedef struct {
  int32_t executed, where, base, rank;
  int64_t dims[SOD2_MAX_RANK];
  int64_t offset, bytes;
  int32_t life_start, life_end;   /* first and last executed step that needs the storage */
} sod2_tensor_info;
sod2_status sod2_binding_query_tensor(const sod2_binding_t*, int32_t tensor, sod2_tensor_info* info_host);
sod2_status sod2_run_query_tensor(const sod2_binding_t*, int32_t tensor, sod2_tensor_info* info_host);
/* force the decisions of the next runs (replay of a reference decision vector); n = 0 clears */
sod2_status sod2_binding_force_decisions(sod2_binding_t*, const int32_t* decisions_host, int32_t n);
/* force one kernel version for every contraction: -1 automatic, 0 regular, 1 fat, 2 skinny,
 * 3 the plain FMA kernel (any dtype, any strides) */
sod2_status sod2_binding_force_variant(sod2_binding_t*, int32_t variant);

/* force the number of k ranges of every contraction that can split k (split-K: fp32 partial tiles
 * summed in a fixed order): 0 automatic, 1 never, n <= 16 that many where the workspace allows */
sod2_status sod2_binding_force_splits(sod2_binding_t*, int32_t n);
/* Optional workspace.  When the arena handed to sod2_run is at least this many bytes longer than
 * sod2_binding_arena_bytes (rounded up to 256), its last workspace_bytes are used for split-K partial
 * sums; with a shorter arena no contraction splits k.  Either way the same call is bit-reproducible. */
sod2_status sod2_binding_workspace_bytes(const sod2_binding_t*, size_t* workspace_bytes);

/* Constants derived from the weights, for the normalisations that the plan made the second result of a
 * contraction (Section 4.2: fusion across operators whose shapes RDP relates; sod2_plan_opts.fold_ln).  The
 * contraction that reads such a normalisation multiplies the un-normalised rows and finishes the normalisation
 * in its epilogue, which needs, per output column n, sum_k gamma[k] W[n][k] and sum_k beta[k] W[n][k] (+ bias[n])
 * in fp32.  They depend on the weights only:
 *   sod2_plan_constants_bytes    size of the buffer (0: the plan has no such pair)
 *   sod2_plan_prepare_constants  computes them into constants_dev (device memory of the caller, 256-byte aligned,
 *                                at least that size) from weights_dev (device pointers, one per weight tensor in
 *                                graph order) with kernels on hip_stream; call it again when the weights change
 *   sod2_binding_set_constants   runs of this binding use the buffer (it must stay valid and unchanged while runs
 *                                are in flight); NULL: back to the default
 * Without constants (the default, and always in replays) every such normalisation is
 * computed by its own kernel right behind the contraction that produces its input; with them, no kernel of its own
 * runs, whenever both contractions of the pair run tiled matrix-core kernels on dense operands.  The two ways round
 * differently (within the tolerance of the storage type), each is bit-reproducible. */
sod2_status sod2_plan_constants_bytes(const sod2_plan_t*, size_t* bytes);
sod2_status sod2_plan_prepare_constants(const sod2_plan_t*, const void* const* weights_dev, int32_t n_weights,
                                        void* constants_dev, size_t bytes, void* hip_stream);
sod2_status sod2_binding_set_constants(sod2_binding_t*, const void* constants_dev, size_t bytes);

/* -- run -------------------------------------------------------------------------------------- */
/* arena: device memory, 256-byte aligned, at least arena_bytes long.  weights / inputs / outputs:
 * host arrays of device pointers, one per tensor with that role, ordered by tensor id (the pointer of an input or
 * output that has no elements at the bound symbols may be NULL, any other NULL is SOD2_ERR_INVALID_ARG).
 * hip_stream: a hipStream_t (NULL = the null stream).  The first run of a graph with Switch, NonZero or NMS operators on
 * a host thread allocates one 64-byte slot of pinned, device-visible host memory (hipHostMalloc) for the read-backs;
 * it is kept until the process ends.  Nothing else is allocated by a run (launch records: events, created when
 * profiling is switched on).  Enqueues and returns; the host waits for the
 * GPU only at a Switch, whose predicate it needs, and after a NonZero or NMS, whose count (8 bytes) sizes
 * what follows: a one-thread kernel behind the producing kernel publishes the value into pinned host
 * memory and the host polls it (after 20 ms without it the stream is synchronised instead).  A run
 * with such a wait cannot be captured in a HIP graph (it returns SOD2_ERR_HIP under capture); runs
 * without Switch, NonZero and NMS only enqueue kernels and can be.  Kernel arguments are
 * prepared step by step while earlier kernels already execute: when a call fails (a group the
 * kernels do not support, an arena too small for the path taken) the groups before the failing one
 * may have run and the contents of the outputs and of the arena are unspecified. */
sod2_status sod2_run(sod2_binding_t*, void* arena_dev, size_t arena_bytes,
                     const void* const* weights_dev, int32_t n_weights,
                     const void* const* inputs_dev, int32_t n_inputs,
                     void* const* outputs_dev, int32_t n_outputs, void* hip_stream);
/* The same run for callers that cannot allocate device memory (code under HIP graph capture, serving
 * loops and harnesses that forbid hipMalloc) and therefore cannot lengthen the arena by the split-K
 * workspace: the fp32 partial tiles of split-K contractions go to a buffer of SOD2_STATIC_SCRATCH_BYTES
 * that is part of the library's device image (one copy per GPU, held until the process ends).  The call
 * allocates nothing, on the device or in pinned host memory, and creates no events.  arena_bytes is the
 * plan's size (sod2_binding_arena_bytes); anything behind it is ignored.  Results are bit-identical to
 * those of sod2_run with a workspace.
 *   SOD2_ERR_SCRATCH_TOO_SMALL  a contraction of the binding splits k into so many ranges that its
 *                               partial tiles exceed the buffer (checked for every launch before the
 *                               first one is enqueued: nothing has run); sod2_binding_force_splits(b, 1)
 *                               or sod2_run with a workspace avoid it
 *   SOD2_ERR_UNSUPPORTED        the graph has Switch, NonZero or NMS operators (their read-backs need a pinned
 *                               host slot), or profiling is on (launch records need events)
 * All calls on one GPU share the buffer: two calls that overlap in time on the same GPU (different
 * streams or threads) race on it; calls on one stream are ordered and safe.  Every partial tile is written
 * before it is read within a call, so nothing is cleared between calls. */
#define SOD2_STATIC_SCRATCH_BYTES (8u << 20)
sod2_status sod2_run_static(sod2_binding_t*, void* arena_dev, size_t arena_bytes,
                            const void* const* weights_dev, int32_t n_weights,
                            const void* const* inputs_dev, int32_t n_inputs,
                            void* const* outputs_dev, int32_t n_outputs, void* hip_stream);
/* decisions taken by the last run, in execution order; *n receives their count */
sod2_status sod2_run_decisions(const sod2_binding_t*, int32_t* decisions_host, int32_t cap, int32_t* n);
/* counts found by the NonZero / NMS operators of the last run, in execution order; *n receives their number */
sod2_status sod2_run_exec_values(const sod2_binding_t*, int64_t* values_host, int32_t cap, int32_t* n);

/* What the last run did, step by step (Section 4.3: with control flow only the taken path is launched; Section
 * 4.4.2: the kernel version is picked at run time).  One entry per executed step: a group with the kernel family
 * (numbering of sod2_launch_record.kernel; -1 for a group whose result was empty), version and split-K count it was
 * launched with, or a control operator with the decision taken (Switch: 1 = the skip output, else -1). */
typedef struct {
  int32_t is_group;   /* 1 a group (ref = group id), 0 a Switch / Combine (ref = operator id) */
  int32_t ref;
  int32_t kernel, variant, splits;
  int32_t decision;
  int32_t fold;       /* a contraction and a folded normalisation: 0 none; 1 its kernel also wrote the normalisation of
                         its result as a second result; 3 the normalisation's own kernel ran right behind it; 2 its first
                         operand was such a second result and its epilogue finished the normalisation */
} sod2_trace_entry;
sod2_status sod2_run_trace(const sod2_binding_t*, sod2_trace_entry* entries_host, int32_t cap, int32_t* n);

/* plan actually executed by the last run (differs from the bind-time plan only with Switches):
 * same text format as sod2_binding_dump; arena bytes and live peak of the executed path */
sod2_status sod2_run_plan_dump(const sod2_binding_t*, char* buf_host, size_t cap, size_t* needed);
sod2_status sod2_run_arena_bytes(const sod2_binding_t*, size_t* arena_bytes, size_t* peak_live_bytes);

/* per-launch records of the last run (filled when profiling is on: two events per launch).  The
 * first two records (kernel 7, groups -1 and -2) are one and two empty launches timed the same way:
 * twice the first minus the second is what the pair of events adds to every duration. */
typedef struct {
  int32_t group;       /* group id */
  int32_t kernel;      /* 0 gemm, 1 conv, 2 layernorm, 3 softmax, 4 eltwise, 5 pool, 6 reduce, 7 other,
                          8 gather, 9 cache append, 10 argmax, 11 fused attention, 12 nonzero,
                          13 scatter rows, 14 resize (nearest), 15 concat, 16 range, 17 fill (constant / identity),
                          18 one-hot, 19 top-k, 20 group normalisation, 21 max-unpool, 22 non-maximum suppression */
  int32_t variant;
  int32_t reserved;
  float ms;            /* event-to-event duration */
  double flops;        /* algorithmic floating-point operations of the group */
  double bytes;        /* algorithmic bytes: every operand read once, the result written once */
} sod2_launch_record;
sod2_status sod2_binding_set_profiling(sod2_binding_t*, int32_t on);
sod2_status sod2_binding_launch_records(const sod2_binding_t*, sod2_launch_record* recs_host, int32_t cap, int32_t* n);

/* -- replay of a step sequence ---------------------------------------------------------------- */
/* For a graph that is run step after step with one symbol growing by 1 per step (a decoder: the
 * length of its KV cache) and whose launch sequence depends on that symbol only through the row a
 * CacheAppend writes and the number of keys a few-query attention reads: the launches of one step are
 * captured once in a HIP graph; the kernels read the step from a counter in device memory, so each
 * further step costs one graph launch and no host planning.  symbols_host are the values of step 0;
 * inputs / outputs are the device pointers of step 0 and *_step_bytes (host, one per pointer, may be
 * NULL) the bytes each advances per step; step_counter_dev is one int32 of device memory the caller
 * keeps alive.  The arena must hold the plan of the last step.  hip_stream must not be the null stream.
 * Returns SOD2_ERR_UNSUPPORTED when anything else in the launch table depends on the step symbol. */
typedef struct sod2_replay_s sod2_replay_t;
sod2_status sod2_replay_create(const sod2_plan_t*, const int64_t* symbols_host, int32_t n_symbols, int32_t step_symbol,
                               int32_t max_steps, void* arena_dev, size_t arena_bytes,
                               const void* const* weights_dev, int32_t n_weights,
                               const void* const* inputs_dev, const int64_t* input_step_bytes_host, int32_t n_inputs,
                               void* const* outputs_dev, const int64_t* output_step_bytes_host, int32_t n_outputs,
                               int32_t* step_counter_dev, void* hip_stream, sod2_replay_t** out);
/* enqueues: counter = first_step, then n_steps graph launches (each ends by advancing the counter) */
sod2_status sod2_replay_launch(sod2_replay_t*, int32_t first_step, int32_t n_steps, void* hip_stream);
void sod2_replay_destroy(sod2_replay_t*);

const char* sod2_last_error(void);
const char* sod2_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SOD2_H */

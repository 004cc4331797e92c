/*
 * dnnf.h - C ABI of the MI355X (gfx950) fused-block executor.
 *
 * The calls follow the pipeline of the paper's Section 4.1 (overview figure):
 * a computational graph with weights is annotated into the Extended
 * Computational Graph (Sec. 3.2), rewritten with mathematical properties
 * (Sec. 4.2, Table 4), partitioned into fusion blocks (Sec. 4.3, Listing 1,
 * mapping-type table of Sec. 3.2), lowered block by block to one generated HIP
 * kernel each (Sec. 4.4), and run.
 *
 * Conventions
 *   - Every function returns a dnnf_status (0 = OK, negative = error); no
 *     exception crosses the boundary and nothing aborts.  dnnf_last_error()
 *     returns a thread-local, NUL-terminated description of the last failure.
 *   - "host" pointers are ordinary process memory; "device" pointers are HIP
 *     device memory of the current device.  The library never allocates or
 *     frees device memory: tensors and the workspace belong to the caller.
 *   - Tensors are dense, row-major, in the layout the operator definitions use
 *     (NCHW for Conv, [..., M, K] x [..., K, N] for MatMul).
 *   - Handles are created and destroyed by the library; all graph structure
 *     passed in is copied.
 */
#ifndef DNNF_H
#define DNNF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dnnf_graph dnnf_graph;
typedef struct dnnf_plan dnnf_plan;

typedef enum {
  DNNF_OK = 0,
  DNNF_INVALID_ARG = -1,
  DNNF_SHAPE_MISMATCH = -2,
  DNNF_UNSUPPORTED_OP = -3,
  DNNF_CYCLE = -4,
  DNNF_OUT_OF_MEMORY = -5,
  DNNF_COMPILE_FAILED = -6,
  DNNF_HIP_ERROR = -7,
  DNNF_NOT_FINALIZED = -8
} dnnf_status;

typedef enum { DNNF_F32 = 0, DNNF_F16 = 1, DNNF_BF16 = 2, DNNF_I32 = 3, DNNF_I64 = 4, DNNF_BOOL = 5 } dnnf_dtype;
typedef enum { DNNF_INPUT = 0, DNNF_WEIGHT = 1, DNNF_INTERMEDIATE = 2, DNNF_OUTPUT = 3 } dnnf_tensor_kind;

/* Mapping types of Sec. 3.1, numbered in the increasing order of complexity
 * given in that section's footnote. */
typedef enum {
  DNNF_ONE_TO_ONE = 0,
  DNNF_REORGANIZE = 1,
  DNNF_SHUFFLE = 2,
  DNNF_ONE_TO_MANY = 3,
  DNNF_MANY_TO_MANY = 4
} dnnf_mapping_type;

/* Cell colour of the mapping-type analysis table (Sec. 3.2): green = fuse,
 * yellow = decide by profiling, red = do not fuse. */
typedef enum { DNNF_GREEN = 0, DNNF_YELLOW = 1, DNNF_RED = 2 } dnnf_colour;

/* An operator attribute: a named array of doubles (integers are exact). */
typedef struct {
  const char* name;     /* host, NUL-terminated */
  int n;
  const double* values; /* host */
} dnnf_attr;

const char* dnnf_last_error(void);

/* ---- graph construction (Sec. 4.1: the computational graph that is the input) ---- */
dnnf_status dnnf_graph_create(dnnf_graph** g);
void dnnf_graph_destroy(dnnf_graph* g);

/* Declares a tensor.  dims: host array of `rank` extents (rank 0 = scalar).  tensor_id receives
 * the handle used by the other calls.  INPUT/WEIGHT/OUTPUT tensors are numbered, per kind, in the
 * order they are declared; that order indexes the pointer arrays of dnnf_plan_build/_run. */
dnnf_status dnnf_graph_add_tensor(dnnf_graph* g, const char* name, dnnf_dtype dtype, int rank,
                                  const int64_t* dims, dnnf_tensor_kind kind, int* tensor_id);

/* Gives the compiler host-readable values of a WEIGHT tensor (double, `count` = number of
 * elements).  Needed for scalar constants that rewrites fold or the generator inlines; large
 * weights need not be supplied. */
dnnf_status dnnf_graph_set_const(dnnf_graph* g, int tensor_id, const double* values, int64_t count);

/* Appends an operator of ONNX kind `op_kind` ("Conv", "MatMul", "Add", ...; Table 2 vocabulary).
 * in_ids/out_ids: host arrays of tensor handles.  op_id receives the operator handle. */
dnnf_status dnnf_graph_add_op(dnnf_graph* g, const char* op_kind, int n_in, const int* in_ids, int n_out,
                              const int* out_ids, const dnnf_attr* attrs, int n_attrs, int* op_id);

/* Validates, infers shapes (declared extents must agree), orders topologically, and annotates
 * every operator with its mapping type (Table 2 and the most-complex-pair rule of Sec. 3.1) and
 * mathematical properties (Sec. 3.2, ECG). */
dnnf_status dnnf_graph_finalize(dnnf_graph* g);

dnnf_status dnnf_graph_num_ops(const dnnf_graph* g, int* n);            /* live operators */
dnnf_status dnnf_graph_num_op_slots(const dnnf_graph* g, int* n);       /* handles 0..n-1, some may be dead */
/* kind_buf (host, cap bytes) receives the operator kind; alive = 0 if a rewrite removed it. */
dnnf_status dnnf_graph_op_info(const dnnf_graph* g, int op_id, char* kind_buf, int cap, int* alive,
                               int* mapping_type);
dnnf_status dnnf_op_mapping_type(const dnnf_graph* g, int op_id, int* type);
/* Table 2 lookup by operator name alone (no graph context). */
dnnf_status dnnf_op_kind_mapping_type(const char* op_kind, int* type);

/* Mapping-type analysis table (Sec. 3.2): type of the fused operator and the cell colour for a
 * first operator feeding a second one. */
dnnf_status dnnf_fuse_relation(int type_first, int type_second, int* fused_type, int* colour);

/* ---- mathematical-property graph rewriting (Sec. 4.2, Table 4) ---- */
typedef struct {
  int rules_fired;          /* applications of Table 4's rules, printed and derived */
  int canonicalisations;    /* decompositions recognised, constants folded */
  double flops_before, flops_after;
  int ops_before, ops_after;
  int derived_rules_fired;  /* of rules_fired: rules that are not printed in Table 4 but are instances of a printed row */
} dnnf_rewrite_stats;
dnnf_status dnnf_graph_rewrite(dnnf_graph* g, dnnf_rewrite_stats* stats /* host, may be NULL */);

/* The annotated graph (the ECG of Sec. 3.2) as JSON text: live tensors (id, name, dtype, kind,
 * shape, constant values if known) and live operators in topological order (kind, mapping type,
 * #FLOPS, operands, attributes).  buf: host, cap bytes; needed receives the size required. */
dnnf_status dnnf_graph_dump_json(const dnnf_graph* g, char* buf, size_t cap, size_t* needed);

/* ---- fusion plan (Sec. 4.3, Listing 1) and code generation (Sec. 4.4) ---- */
typedef struct {
  int fusion;            /* 0 = one block per operator (the unfused executor) */
  int profile;           /* 1 = time yellow candidates on the device, 0 = treat yellow as green */
  int intra_block;       /* 1 = fold Reorganize/Shuffle into index maps (Sec. 4.4.2) */
  int max_block_ops;     /* constraint check of Listing 1, step 2.2; <=0 selects the default (64) */
  int max_block_operands;/* distinct external tensors per block; <=0 selects the default (16) */
  void* profile_scratch; /* device; used only while building with profile = 1 */
  size_t profile_scratch_bytes;
  const char* cache_dir; /* host; directory for compiled kernels, NULL = in-memory only */
  int verbose;
  int successors_first;  /* 1 = explore a seed's successors before its predecessors (the order of the paper's
                            worked example, Fig. 3); 0 = predecessors first (Sec. 4.3 allows either) */
  int check_lowerable;   /* 1 = the constraint check also demands a kernel template for the candidate block;
                            0 = analysis only (plans for inspection, not for running) */
  int tune;              /* 1 = a block whose kernel template offers several tile configurations (MatMul) is
                            timed with each of them on the device while the plan is built (profile scratch
                            required) and keeps the fastest - the choice the paper leaves to its profiling
                            database (Sec. 4.3); dnnf_plan_precompile then compiles every configuration, so
                            that a tuned build on the device finds them in cache_dir.  0 = a cost model picks */
  int attention;         /* 1 = extension beyond the paper's table: MatMul -> One-to-One operators -> Softmax ->
                            MatMul (Many-to-Many after Many-to-Many, a red cell of Sec. 3.2) is formed as one
                            block and runs as a streaming-softmax kernel whose score matrix never reaches
                            memory.  0 (default) = the paper's table decides */
  int layout;            /* global data-format selection (Sec. 4.4.2): 1 = the activations between the blocks of a
                            convolutional graph are stored channels-last (the order its dominant operators, the
                            convolutions, run fastest on) and depthwise filters are re-laid to match when the
                            plan is prepared; graph inputs and outputs keep the declared order.  0 (default) =
                            every tensor in the declared order */
  int broadcast_prologue;/* 1 = second extension beyond the table: a multiply by a tensor that is constant over the image
                            plane (x * s[n, c, 1, 1], the squeeze-excite scaling; One-to-Many) directly in front of a
                            pointwise convolution joins the convolution's block and is applied to the operand vectors
                            as they are loaded (One-to-Many before Many-to-Many is a red cell of Sec. 3.2).  With
                            profile = 1 the fused kernel is timed against the two separate ones first.  0 (default)
                            = the paper's table decides */
  int graphs;            /* 1 = dnnf_plan_run replays its launch sequence as a HIP graph from the second call with the
                            same input / output / workspace pointers on (one graph per pointer set, at most 16);
                            0 (default) = always launch kernel by kernel.  Results are the same either way; on
                            MI355X the five benchmark graphs run no faster as graphs (the launches are already hidden
                            behind the kernels) and the one-kernel ones slower, hence the default */
  int gemm_norm;         /* third extension beyond the table: MatMul -> One-to-One operators -> normalisation of the last axis
                            (LayerNorm behind a linear layer: Many-to-Many after Many-to-Many, a red cell of Sec. 3.2) as one
                            block whose workgroups own whole rows of the product (at most 768 columns), so that the row
                            statistics are taken from the accumulators before they leave the chip.  1 = with profile = 1
                            the fused kernel is timed against the two separate ones first (without profiling it is
                            taken); 2 = always taken.  0 (default) = the paper's table decides.  On MI355X the separate
                            kernels win at 768 columns: a row-owning tile re-reads the whole weight matrix per 32 rows */
  int squeeze_excite;    /* fourth extension beyond the table: [GlobalAveragePool ->] 1x1 Conv -> One-to-One operators ->
                            1x1 Conv -> One-to-One operators on [n, c, 1, 1] vectors (the squeeze-excite tail of a mobile
                            network block; three Many-to-Many operators in a row) as one kernel, one workgroup per image,
                            the pooled and the hidden vector in LDS.  The pool joins when its map has at most 256 positions
                            (larger maps keep their own, multi-workgroup pooling kernel).  Where the map comes out of a depthwise
                            convolution whose kernel sees a whole image plane per workgroup, the pool is taken inside that
                            kernel instead and the tail holds the two layers.  1 = with profile = 1 timed
                            against the separate kernels first; 2 = always taken; 0 (default) = the paper's table decides */
} dnnf_plan_opts;
void dnnf_plan_default_opts(dnnf_plan_opts* o);
/* Developer switches read from the environment when a plan is built (none is needed in normal use):
 *   DNNF_GEMM_TILE=BM,BN,BK,WAVES_M,WAVES_N,NBUF[,PF[,DMA]]  forces one tile configuration of the GEMM template on every
 *       MatMul block (the parity tests walk through all of them this way);
 *   DNNF_GEMM_NO_DMA=1     leaves the tile configurations that load operand tiles straight into LDS out of the tuning;
 *   DNNF_GEMM_NO_ROW_ALIGN=1  stores results whose rows do not start on 16-byte boundaries element by element instead
 *       of row by row from each row's first aligned column;
 *   DNNF_NO_WEIGHT_PREFETCH=1 / DNNF_CONV_PREFETCH_KB=n  switch off the up-front touch of a MatMul block's weight
 *       matrix (256 KiB to 16 MiB) / set the smallest convolution filter that is touched that way (default 64, 0 = none);
 *   DNNF_STREAM_MB=n       smallest result, in MiB, that a MatMul / convolution block writes with non-temporal vector
 *       stores (default 48: more than the L2 caches hold together; measured on the decoder workload, streaming results
 *       of 4 MiB and more costs 10 % end to end because their readers then miss). */

/* weight_dev_ptrs: host array, one device pointer per WEIGHT tensor in declaration order; the
 * buffers stay caller-owned and must outlive the plan.  stream: a hipStream_t (as void*) used for
 * profiling launches.  The graph must be finalized; it is not modified. */
dnnf_status dnnf_plan_build(const dnnf_graph* g, const dnnf_plan_opts* opts, const void* const* weight_dev_ptrs,
                            void* stream, dnnf_plan** plan);
void dnnf_plan_destroy(dnnf_plan* p);

typedef struct {
  int n_ops;
  int fused_type;          /* dnnf_mapping_type of the block */
  int family;              /* kernel family of the block's generated operator (Sec. 4.4.1): 0 elementwise chain (also
                              Gather, Resize, Expand, Concat parts and window pooling kernels' One-to-One neighbours),
                              1 row reduction (Softmax, Normalize, Reduce*, GlobalAveragePool, CumSum, MaxPool /
                              AveragePool), 2 MFMA GEMM (MatMul / Gemm / Einsum), 3 convolution as implicit GEMM
                              (Conv 2-d / 3-d, ConvTranspose), 4 depthwise convolution, 5 alias (a lone contiguous
                              Reshape or a stacking Concat: no kernel, the result shares its operands' storage), 6 streaming-softmax
                              attention (opts.attention), 7 squeeze-excite tail (opts.squeeze_excite) */
  double bytes;            /* algorithmic HBM bytes: external inputs read once + outputs written once */
  double flops;
  double irs_bytes_removed;/* intermediate results that never reach HBM (Table 5's IRS statistic) */
  int n_kernel_launches;
  char kernel_name[96];
} dnnf_block_info;

dnnf_status dnnf_plan_num_blocks(const dnnf_plan* p, int* n);
dnnf_status dnnf_plan_block_info(const dnnf_plan* p, int block, dnnf_block_info* info);
/* op_ids (host, cap entries) receives the operators of `block` in topological order. */
dnnf_status dnnf_plan_block_ops(const dnnf_plan* p, int block, int* op_ids, int cap, int* n);
/* Kind of operator `op_id` of the plan (host buffer).  Ids below the graph's slot count are the graph's
 * operators; data-format selection (layout = 1) may append operators of its own after them. */
dnnf_status dnnf_plan_op_kind(const dnnf_plan* p, int op_id, char* kind_buf, int cap);
/* Generated HIP source of a block's kernel (host buffer). */
dnnf_status dnnf_plan_block_source(const dnnf_plan* p, int block, char* buf, size_t cap, size_t* needed);

/* The plan as JSON text: per block its operators, kernel family and variant, and its external
 * input / output tensors (id, name, name of the original-graph tensor it equals after rewriting,
 * dtype, shape, where it lives: caller pointer index or workspace offset); plus the planner's log
 * (seeds, fusions, profiling decisions).  Used for per-block parity checks and reporting. */
dnnf_status dnnf_plan_dump_json(const dnnf_plan* p, char* buf, size_t cap, size_t* needed);

/* Compiles every kernel of the plan into the in-memory cache (and cache_dir, if one was given).
 * Needs no GPU: used to build kernels ahead of time. */
dnnf_status dnnf_plan_precompile(dnnf_plan* p);

/* Device bytes the caller must provide as `workspace`: the results of fusion blocks that other blocks read (the
 * intermediate results Sec. 4.4 / Table 5 counts - the ones fusion could not remove), the tensors the plan pre-computes
 * from weights, and the partial results of split reductions.  256-byte aligned base required. */
dnnf_status dnnf_plan_workspace_bytes(const dnnf_plan* p, size_t* bytes);
/* Loads every kernel of the plan onto the current device and runs the weight-only blocks (folded constants)
 * once into `workspace`.  Call before the first dnnf_plan_run with a given workspace.  With workspace == NULL
 * only the kernels are loaded (enough for a plan that runs through dnnf_plan_run_static). */
dnnf_status dnnf_plan_prepare(dnnf_plan* p, void* workspace, void* stream);

/* Runs the fusion plan (Sec. 4.4: one generated operator per fusion block, in an order that respects the graph's data
 * dependences).  Enqueues every block on `stream` (asynchronous; returns after the launches).
 * input_dev_ptrs / output_dev_ptrs: host arrays of device pointers, one per INPUT / OUTPUT tensor
 * in declaration order.  With opts.graphs = 1 the second call with the same pointers records the
 * launches into a HIP graph (on a stream the plan owns) and that call and later ones enqueue the graph
 * on `stream` instead; the buffers' contents are read when the graph runs, as with plain launches. */
dnnf_status dnnf_plan_run(dnnf_plan* p, const void* const* input_dev_ptrs, void* const* output_dev_ptrs,
                          void* workspace, void* stream);
/* dnnf_plan_run for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The workspace (intermediates between blocks,
 * tensors the plan pre-computes, partial results of split reductions) is a file-scope device array of
 * DNNF_STATIC_WORKSPACE_BYTES inside the library; each GPU the library runs on holds its own copy until the process
 * ends.  The call allocates and frees nothing, on the device or through the runtime: it only enqueues kernel launches
 * on `stream`.  For that the plan's kernels must be resident already - call dnnf_plan_prepare once beforehand
 * (a NULL workspace is enough); otherwise DNNF_NOT_FINALIZED.  A plan whose dnnf_plan_workspace_bytes exceeds
 * DNNF_STATIC_WORKSPACE_BYTES is refused with DNNF_OUT_OF_MEMORY and a message that names both sizes.  All plans
 * share a device's array, which keeps the last call's contents: when another plan ran there last, this call first
 * puts the plan's pre-computed tensors back (extra launches on `stream`); everything else is written before it is
 * read.  Calls that overlap on one GPU (two streams, two threads) race on the array: serialise them.  Inputs and
 * outputs stay caller-owned as in dnnf_plan_run; opts.graphs is ignored here (always kernel-by-kernel launches,
 * which a caller may itself capture). */
#define DNNF_STATIC_WORKSPACE_BYTES (64u << 20)
dnnf_status dnnf_plan_run_static(dnnf_plan* p, const void* const* input_dev_ptrs, void* const* output_dev_ptrs,
                                 void* stream);
/* Same, for one fusion block only (Sec. 4.3's profiling measures blocks one at a time; so do per-block parity and
 * rocprofv3 runs). */
dnnf_status dnnf_plan_run_block(dnnf_plan* p, int block, const void* const* input_dev_ptrs,
                                void* const* output_dev_ptrs, void* workspace, void* stream);
/* Latency of one fusion block as Listing 1 (step 2.3) measures it: average device time of `block` over `iters`
 * launches after `warmup`, taken with HIP events on `stream`; microseconds. */
dnnf_status dnnf_plan_time_block(dnnf_plan* p, int block, const void* const* input_dev_ptrs,
                                 void* const* output_dev_ptrs, void* workspace, void* stream, int warmup,
                                 int iters, double* usec);

#ifdef __cplusplus
}
#endif
#endif /* DNNF_H */

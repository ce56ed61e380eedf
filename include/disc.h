/*
 * disc.h -- C ABI of the shape-generic fusion-kernel library for MI355X (gfx950).
 *
 * The library implements the hot path that the DISC dynamic-shape compiler
 * (arXiv 2103.05288) speeds up: a fusion pattern of memory-bound ops is
 * registered ONCE, without shape values, and is then launched at any runtime
 * shape without recompiling (Section 2: the fused kernels are generated for
 * shapes that are not known yet; static rank only).
 *
 *   register:  op list + shape constraints  ->  constraint closure (Section
 *              4.2.1), fusion decision from shape propagation + constraints
 *              (Section 4.3, the paragraph on shape hints), kernel template choice
 *              (loop fusion / input fusion with a reduce root, Section 4.3,
 *              the paragraph on fusion configuration), ONE device compile that
 *              holds every kernel version, and a launch plan with everything
 *              that does not depend on shape values precomputed.
 *   launch:    runtime dims -> host shape calculation (Section 4.2.1),
 *              version + launch-dimension selection (Section 4.3), kernel
 *              launch (Section 4.2.3, host-side control).
 *              No op of the pattern is walked at launch time.
 *
 * Conventions
 *  - Every function returns 0 (DISC_OK) or a negative disc_status; nothing
 *    throws, aborts or prints.  disc_last_error() returns a context-owned,
 *    NUL-terminated message that stays valid until the next call on that
 *    context.
 *  - A context is not thread-safe: one context per host thread.
 *  - All tensor pointers passed to disc_launch / disc_plan are DEVICE pointers
 *    owned by the caller (the paper takes its buffers from the framework's
 *    cached allocator, Section 4.2.2); tensors are dense, row-major, without
 *    strides.  `ops`, `cs`, `dims` and the pointer arrays themselves are HOST
 *    memory, read during the call only.
 *  - The library never allocates or frees device memory in disc_launch and
 *    never synchronises: the launch is asynchronous on `hip_stream`.
 *  - Outputs must not overlap inputs or each other.
 */
#ifndef DISC_H_
#define DISC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct disc_ctx disc_ctx;

typedef enum {
  DISC_OK = 0,
  DISC_ERR_INVALID_ARG = -1, /* null pointer, bad id, n_dims / n_in / n_out mismatch          */
  DISC_ERR_BAD_PATTERN = -2, /* malformed op list: bad opcode / dtype / rank, forward reference,
                                contradictory static sizes, rank > DISC_MAX_RANK               */
  DISC_ERR_UNFUSIBLE = -3,   /* the checker cannot prove that all ops share one iteration space */
  DISC_ERR_CONSTRAINT = -4,  /* runtime dims contradict a registered equality or a static size  */
  DISC_ERR_WORKSPACE = -5,   /* workspace missing or smaller than disc_workspace_bytes()        */
  DISC_ERR_COMPILE = -6,     /* device compile failed; the compiler log is in disc_last_error   */
  DISC_ERR_HIP = -7,         /* a HIP runtime call failed                                       */
  DISC_ERR_SHAPE = -8,       /* negative dim, element count overflow, row too long              */
  DISC_ERR_EMPTY_REDUCE = -9,/* reduction over an axis of runtime size 0                        */
  DISC_ERR_INTERNAL = -10    /* an exception inside the library (out of host memory, ...); caught
                                at the boundary, never propagated                               */
} disc_status;

enum { DISC_MAX_RANK = 4, DISC_MAX_OPS = 256, DISC_MAX_DIMS = 16 };

typedef enum {
  DISC_F32 = 0, DISC_F16 = 1, DISC_BF16 = 2, DISC_I32 = 3, DISC_I64 = 4,
  DISC_BOOL = 5 /* one byte per element, nonzero = true */
} disc_dtype;

/* Op set: the element-wise / broadcast / cast / select / reduce family with HLO meaning
 * (the paper names Add, Sub, Mul, Broadcast, ... by example: Sections 4.1, 4.2.1, 4.3). */
typedef enum {
  /* leaves */
  DISC_PARAM = 0,  /* k-th PARAM = k-th input pointer of disc_launch                           */
  DISC_CONST,      /* rank-0 constant `fconst`                                                 */
  DISC_DIM_SIZE,   /* rank-0 scalar: runtime size of symbolic dim axis_map[0] (shape value
                      computed on the host and handed to the device, Section 4.2.1)            */
  /* unary */
  DISC_NEG, DISC_ABS, DISC_EXP, DISC_LOG, DISC_TANH, DISC_SQRT, DISC_RSQRT, DISC_RCP,
  DISC_SIGMOID, DISC_ERF,
  /* binary */
  DISC_ADD, DISC_SUB, DISC_MUL, DISC_DIV, DISC_MAX, DISC_MIN, DISC_POW,
  /* compare: result dtype DISC_BOOL */
  DISC_LT, DISC_LE, DISC_GT, DISC_GE, DISC_EQ, DISC_NE,
  DISC_SELECT,     /* in = (pred, on_true, on_false); pred != 0 picks on_true                  */
  DISC_CAST,       /* to `dtype`; float->int truncates toward zero                             */
  DISC_BROADCAST,  /* HLO broadcast_in_dim: axis_map[k] = result axis of operand axis k,
                      strictly increasing; an operand axis of static size 1 may expand         */
  DISC_REDUCE_SUM, DISC_REDUCE_MAX, DISC_REDUCE_MIN,
  DISC_REDUCE_ARGMAX, /* lowest index among the maxima; dtype DISC_I32 or DISC_I64             */
  DISC_OUTPUT,     /* k-th OUTPUT = k-th output pointer; in[0] = the value, same dtype.  Rank 0
                      (one element) only for a reduction of per-row values over the rows, see
                      DISC_TEMPLATE_ROW_REDUCE                                                  */
  DISC_SLICE,      /* dynamic slice of a PARAM, stride 1 (Section 4.1: start indices are runtime
                      values, not attributes): result[i0,i1,..] = in[s0+i0, s1+i1, ..]; dim[] = sizes
                      of the result; axis_map[k] = start along axis k: >= 0 the symbolic dim id whose
                      runtime value is the start, < 0 the static start -1 - axis_map[k].  in[0] must
                      be a PARAM (the slice is an indexing function on the input, never a copy; one
                      PARAM may be sliced several times).  A launch whose slice leaves the operand
                      fails with DISC_ERR_SHAPE.                                               */
  DISC_PAD,        /* dynamic pad of a PARAM (named beside slice in Section 4.1), no interior padding:
                      result[i] = in[i - low] where that exists, else `fconst` rounded to the operand's dtype
                      (the padding value is a scalar of the operand's element type); dim[] = sizes of the
                      result, axis_map[k] = padding in front of axis k, encoded like a SLICE start.
                      in[0] must be a PARAM; the padding is produced in registers, never written to
                      memory on its own.  A launch whose operand does not fit the result fails with
                      DISC_ERR_SHAPE.                                                          */
  DISC_TRANSPOSE,  /* HLO transpose of a PARAM: result axis k = operand axis axis_map[k] (a permutation).
                      in[0] must be a PARAM; an indexing function like SLICE, never a copy.  The
                      operand's innermost axis must stay the innermost axis of the pattern's
                      iteration space (accesses stay contiguous along rows); a transpose that moves
                      it cannot be fused with anything (DISC_ERR_UNFUSIBLE), but is a pattern on its
                      own (PARAM, TRANSPOSE, OUTPUT: DISC_TEMPLATE_TRANSPOSE) when it collapses to a
                      batched 2-D transpose; disc_register_graph cuts it out that way.          */
  /* ---- outputs whose size depends on the input VALUES (Section 2 names Unique as the op whose
   * output shape is only known once the data is: the other source of dynamic shapes besides varying
   * input shapes).  All four live in a pattern of rank-1 values of one length N
   * (DISC_TEMPLATE_COMPACT); the results of the last three may only feed OUTPUTs. */
  DISC_NE_PREV,       /* in[0] = a PARAM x of rank 1; DISC_BOOL result[i] = (i == 0) || x[i] != x[i-1]: marks
                         the first element of every run of equal values                              */
  DISC_COMPACT,       /* in = (value, keep); rank 1, dim = N (the upper bound), dtype of value:
                         result[k] = value[i_k], where i_0 < i_1 < ... are the positions with keep != 0.
                         Only the first n = COMPACT_COUNT(keep) elements of the OUTPUT buffer are written;
                         the caller sizes it for N.  COMPACT(x, NE_PREV(x)) is Unique of a sorted x
                         (distinct values in order of first occurrence)                              */
  DISC_COMPACT_COUNT, /* in[0] = keep; rank 0, DISC_I32 or DISC_I64: the number n of positions kept -- the
                         data-dependent size, delivered in device memory (nothing is synchronised)   */
  DISC_COMPACT_RANK,  /* in[0] = keep; rank 1, dim = N, DISC_I32 or DISC_I64: result[i] = (number of kept
                         positions <= i) - 1.  For keep = NE_PREV(x) this is Unique's second result: the
                         index in the compacted output of the value at position i                    */
  DISC_OPCODE_COUNT
} disc_opcode;

/* One op.  A value is named by the index of the op producing it; `in[]` refers to earlier ops.
 * dim[i] >= 0 : symbolic dim id (size given at launch as dims[id]);  dim[i] < 0 : static size
 * -dim[i].  Rank-0 values (CONST, DIM_SIZE) may be operands of element-wise ops as scalars.
 * Float values are computed in fp32 registers whatever their storage dtype and rounded once,
 * to nearest even, when stored. */
typedef struct {
  int32_t opcode;                  /* disc_opcode                                              */
  int32_t dtype;                   /* disc_dtype of the result                                 */
  int32_t in[3];                   /* operand value ids, unused = -1                           */
  int32_t rank;                    /* 0..DISC_MAX_RANK                                         */
  int32_t dim[DISC_MAX_RANK];
  int32_t axis_map[DISC_MAX_RANK]; /* BROADCAST: map; REDUCE_*: [0] = axis; DIM_SIZE: [0] = id */
  double fconst;                   /* CONST only                                               */
} disc_op;

/* Caller-supplied shape constraints: what the paper's bridging layer injects when lowering loses
 * shape information (Section 4.2.1, the Split example). */
typedef enum {
  DISC_DIM_EQ = 0,   /* dim a_axis of value a_value == dim b_axis of value b_value             */
  DISC_NUMEL_EQ = 1  /* values a_value and b_value have the same number of elements            */
} disc_constraint_kind;

typedef struct {
  int32_t kind, a_value, a_axis, b_value, b_axis;
} disc_constraint;

typedef enum {
  DISC_TEMPLATE_LOOP = 0,       /* loop fusion: element-wise / broadcast chain                  */
  DISC_TEMPLATE_ROW_REDUCE = 1, /* input fusion, reduce over the innermost axis (+ epilogue).  One
                                   extension beyond Section 4.3's one reduction kind per kernel:
                                   REDUCE_SUM of a float value over the outer axis of a
                                   two-dimensional iteration space whose result feeds OUTPUTs only
                                   (weight gradients next to an input gradient) is carried along
                                   by the row kernels as per-block partial sums in the workspace
                                   and finished by a second launch, in a fixed order.  Likewise
                                   REDUCE_SUM / MAX / MIN of a per-row float value over the rows,
                                   down to one number (a rank-0 OUTPUT: the total of per-row
                                   losses, the amax of a tensor): one partial result per block,
                                   folded by a last launch of one block                         */
  DISC_TEMPLATE_COL_REDUCE = 2, /* input fusion, reduce over an outer axis (+ epilogue)         */
  DISC_TEMPLATE_TRANSPOSE = 3,  /* not a fusion: PARAM -> TRANSPOSE -> OUTPUT alone, a permutation
                                   that moves the innermost axis, run as a batched 2-D tile
                                   transpose (what an op graph falls back to for such an op)    */
  DISC_TEMPLATE_COMPACT = 4     /* loop fusion over rank-1 values whose outputs are compacted by a
                                   predicate computed in the same pattern (DISC_COMPACT and
                                   friends): per-block counts, a fixed-order scan of the counts, a
                                   scatter -- three launches, no atomics, the element count written
                                   to device memory                                              */
} disc_template;

typedef struct {
  int32_t template_kind;   /* disc_template                                                    */
  int32_t n_dims;          /* symbolic dims expected by disc_launch                            */
  int32_t n_inputs, n_outputs;
  int32_t compile_events;  /* device compiles spent on this pattern so far (target: 1)         */
  int32_t n_variants;      /* kernel versions held by the pattern's single module              */
  int32_t n_phases;        /* row/col reduce: number of dependent reduction levels             */
  int32_t vec_width;       /* elements per vector access of the vectorised versions            */
  int32_t n_collapsed;     /* iteration-space rank after merging dims with identical roles     */
  int32_t n_dim_classes;   /* number of dimension-equality classes after closure               */
  int32_t dim_class[DISC_MAX_DIMS]; /* class id of every symbolic dim (equal id = proved equal) */
  double compile_ms;       /* wall time of the one device compile                              */
} disc_pattern_info_t;

/* Kernel versions (Section 4.3: several versions per pattern, selected on the host). */
typedef enum {
  DISC_V_LOOP_VEC = 0,      /* loop fusion, vector accesses, 32-bit slot index                 */
  DISC_V_LOOP_VEC_I64,      /* ... 64-bit index                                                */
  DISC_V_LOOP_SCALAR,       /* loop fusion, one element per access                             */
  DISC_V_LOOP_SCALAR_I64,
  DISC_V_ROW_REG_VEC,       /* row reduce, row resident in registers of a lane group, vector   */
  DISC_V_ROW_REG_SCALAR,    /* same, one element per access                                    */
  DISC_V_ROW_STREAM_VEC,    /* row reduce, one block per row, row re-read per phase            */
  DISC_V_ROW_STREAM_SCALAR,
  DISC_V_COL_3STAGE_VEC,    /* column reduce: partial -> combine -> epilogue (<= 3 launches)   */
  DISC_V_COL_3STAGE_SCALAR,
  DISC_V_COL_STRIP_VEC,     /* column reduce, one block per column strip, single launch        */
  DISC_V_COL_STRIP_SCALAR,
  DISC_V_TRANSPOSE_TILE,    /* batched 2-D transpose through a 64 x 64 tile in LDS              */
  DISC_V_COL_2STAGE_VEC,    /* column reduce: partial -> finish + epilogue in one kernel (2 launches) */
  DISC_V_COL_2STAGE_SCALAR,
  DISC_V_COMPACT_VEC,       /* compaction: count -> scan -> scatter, vector loads               */
  DISC_V_COMPACT_SCALAR,
  DISC_V_COUNT
} disc_variant;

typedef struct {
  int32_t variant;          /* disc_variant                                                    */
  int32_t n_launches;       /* device launches this call makes (0 when an output is empty)     */
  int32_t index_bits;       /* 32 or 64                                                        */
  int32_t vec_width;        /* elements per access of the chosen version                       */
  int32_t lanes_per_row;    /* row reduce: lanes that own one row (1..1024); column reduce:
                               lanes along the columns per block; else 0                       */
  int32_t slots_per_lane;   /* row reduce: vector slots held per lane, else unroll factor      */
  int32_t reg_slots;        /* compile-time slot capacity of the chosen instantiation          */
  uint32_t grid[3][3];      /* per launch                                                      */
  uint32_t block[3][3];
  uint32_t lds_bytes[3];
  char kernel[3][48];       /* entry-point symbol of each launch, as a profiler shows it        */
  int64_t rows, inner;      /* canonical iteration space [rows, inner] ([outer,mid,inner] for
                               column reduce: rows = outer * mid)                              */
  int64_t mid;              /* column reduce: reduced extent, else 0                           */
  int64_t algorithmic_bytes;/* inputs read once + outputs written once at these dims           */
  size_t workspace_bytes;
} disc_plan_t;

typedef struct {
  int64_t patterns_registered;  /* distinct patterns                                           */
  int64_t pattern_cache_hits;   /* re-registrations answered from the pattern cache            */
  int64_t compile_events;       /* device compiles, all patterns                               */
  int64_t launch_calls;         /* successful disc_launch calls                                */
  int64_t device_launches;      /* kernels enqueued                                            */
  int64_t variant_count[DISC_V_COUNT];
  int64_t host_plan_ns;         /* total wall time in shape calculation + selection            */
  int64_t host_launch_ns;       /* total wall time in disc_launch (plan + enqueue)             */
} disc_stats_t;

/* Create a context bound to HIP device `hip_device`.  hip_device = -1 makes a host-only context:
 * registration (checker, classifier, code generation, device compile for gfx950) and disc_plan
 * work, disc_launch returns DISC_ERR_INVALID_ARG.  The caller frees it with disc_destroy. */
int disc_create(disc_ctx** out, int hip_device);
void disc_destroy(disc_ctx* ctx);
const char* disc_last_error(const disc_ctx* ctx);

/* Register a fusion pattern (op sequence without shape values + constraints) and compile it
 * once (Section 2: fused kernels are generated for shapes that are not known yet; Section 4.2.1:
 * shape constraints collected without shape values; Section 4.3: they decide what may share a
 * kernel and which template it gets).  `ops` / `cs` are copied.  Registering an identical op list
 * + constraints again returns the same id without compiling (pattern cache keyed on the op
 * sequence, never on sizes). */
int disc_register_pattern(disc_ctx* ctx, const disc_op* ops, int n_ops, const disc_constraint* cs,
                          int n_cs, int32_t* pattern_id_out);
/* The same pattern compiled for ONE shape, the way a static-shape compiler would (Section 1 and
 * Section 5.3: the recompile-per-shape alternative, and the gap of the shape-generic kernels to
 * it).  `dims` (host, n_dims values, copied) are planned with the same host rules as any launch;
 * the module then holds only the kernel versions that plan launches, with every extent, stride,
 * division constant and launch-plan member a compile-time constant.  The result is a pattern of
 * its own (one per shape, cached on op sequence + constraints + dims): disc_plan / disc_launch
 * with any other dims return DISC_ERR_SHAPE, forcing a version returns DISC_ERR_INVALID_ARG.
 * disc_pattern_info(...).compile_ms is the per-shape compile cost. */
int disc_register_pattern_static(disc_ctx* ctx, const disc_op* ops, int n_ops, const disc_constraint* cs,
                                 int n_cs, const int64_t* dims, int n_dims, int32_t* pattern_id_out);
int disc_pattern_info(disc_ctx* ctx, int32_t id, disc_pattern_info_t* out);
/* Generated device source of the pattern (context-owned, valid until disc_destroy). */
const char* disc_pattern_source(disc_ctx* ctx, int32_t id);

/* Bytes of device workspace disc_launch needs at these dims (0 for loop patterns and for row
 * patterns without sums over the rows).  Buffer sizes are a result of the host-side shape
 * calculation (Section 4.2.1) and the buffers come from the caller (Section 4.2.2: the framework's
 * allocator owns the memory). */
int disc_workspace_bytes(disc_ctx* ctx, int32_t id, const int64_t* dims, int n_dims, size_t* out);

/* Pure host: the runtime flow of one launch without enqueueing anything: shape calculation and
 * constraint check (Section 4.2.1), selection of one of the pattern's kernel versions and of the
 * launch dimensions from the runtime shape (Section 4.3, the paragraph on the versions).  `inputs` / `outputs` may be NULL
 * (then buffers are assumed 16-byte aligned); pointers are only inspected, never dereferenced.
 * force_variant = -1 lets the host choose. */
int disc_plan(disc_ctx* ctx, int32_t id, const int64_t* dims, int n_dims, const void* const* inputs,
              void* const* outputs, int force_variant, disc_plan_t* out);

/* Launch the pattern at runtime sizes dims[0..n_dims): the generated runtime flow of Sections
 * 4.2.1 and 4.2.3 (shape calculation, kernel launch with host-chosen launch dimensions) followed
 * by the enqueue; a dims vector that contradicts a registered dimension-size or tensor-size
 * equality is refused with DISC_ERR_CONSTRAINT before anything runs.  Asynchronous on `hip_stream` (a
 * hipStream_t, NULL = default stream).  Any output with zero elements and no reduction over an
 * empty axis: success, nothing launched. */
int disc_launch(disc_ctx* ctx, int32_t id, const int64_t* dims, int n_dims,
                const void* const* inputs, int n_in, void* const* outputs, int n_out,
                void* workspace, size_t workspace_bytes, void* hip_stream);

/* For callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): disc_launch without a workspace argument.  The kernels that exchange
 * partial results through device memory (column reduces; row reduces that carry sums over the
 * rows) use a fixed array of DISC_STATIC_SCRATCH_BYTES that is part of the library's code object
 * -- one copy per GPU, held until the process ends -- instead of a caller's workspace.  The call
 * allocates nothing and frees nothing, on the device or through any library.  A shape whose
 * partial results need more than the array holds is refused with DISC_ERR_WORKSPACE before
 * anything runs (use disc_launch with a workspace then).  Same kernels, same launch plan and same
 * results, bit for bit, as disc_launch.  Every call on one GPU shares that GPU's array: calls
 * that overlap in time on one GPU (two streams, two contexts, two threads) race on it -- keep
 * them on one stream, or give all but one of them a workspace through disc_launch.  Nothing in the
 * array has to be cleared between calls (each call writes every cell it later reads).
 * disc_create asks the array's device address once per device; disc_static_scratch_init repeats
 * that (idempotent) for a caller that wants the failure, if any, up front. */
enum { DISC_STATIC_SCRATCH_BYTES = 16 << 20 };
int disc_static_scratch_init(disc_ctx* ctx);
int disc_launch_static_scratch(disc_ctx* ctx, int32_t id, const int64_t* dims, int n_dims,
                               const void* const* inputs, int n_in, void* const* outputs, int n_out,
                               void* hip_stream);

/* Tests only: make the next launches of this context use `variant` when it is legal for the
 * pattern and the shape (else DISC_ERR_INVALID_ARG at launch); -1 restores host selection. */
int disc_force_variant(disc_ctx* ctx, int variant);
/* Tests only: override one host rule of the context, so that kernel versions the rule would not
 * pick at small test sizes still run against the oracle.  Results never depend on these. */
typedef enum {
  DISC_OPT_NON_TEMPORAL = 0,      /* -1 host rule (default), 0 never, 1 wherever the version exists   */
  DISC_OPT_STAGE_ROW_VECTORS = 1, /* 1 host rule (default), 0 row vectors are never staged in LDS     */
  DISC_OPT_ROW_ROUNDS = 2,        /* 0 host rule (default), n > 0: row-kernel grid = n rounds of the
                                     blocks the chip holds at once                                    */
  DISC_OPT_ALIGN_ROW_SLOTS = 3    /* 1 host rule (default), 0: the vector slots of ragged rows are never
                                     shifted to the 16-byte boundaries of the tensor                  */
} disc_test_option_id;
int disc_test_option(disc_ctx* ctx, int option, int value);

/* ---- op graphs larger than one fusion pattern --------------------------------------------------
 * The fusion decision over a graph (Section 4.3: whether ops may share a kernel follows from how
 * shapes propagate through them and from the collected shape constraints) and the planning of the
 * buffers between kernels (Section 4.2.2).  `ops` is an op list in the format above that need not
 * be fusible as a whole.  The library cuts it, in list order, into consecutive fusion patterns: an
 * op joins the current pattern as long as the pattern checker still accepts the result; an op
 * that only feeds one later pattern moves there when that saves a buffer; each pattern is
 * registered (and compiled once) through the pattern cache.  Values that cross a cut and are not
 * graph outputs live in workspace buffers; a buffer is reused by a later value of the same element
 * size and the same symbolic shape once its previous tenant has been read for the last time.
 * Graph OUTPUTs must name computed values, each at most once (DISC_ERR_BAD_PATTERN otherwise).
 * DISC_ERR_UNFUSIBLE when a single op is not a pattern by itself, DISC_ERR_BAD_PATTERN when the
 * cut needs more than DISC_MAX_GRAPH_PATTERNS patterns.  All arrays are host memory, read during
 * the call only.
 *
 * disc_graph_launch: `inputs` / `outputs` are host arrays of DEVICE pointers in the order of the
 * graph's PARAM / OUTPUT ops; `workspace` is DEVICE memory of at least disc_graph_workspace_bytes
 * (256-byte aligned), owned by the caller, free to reuse once the stream has passed the launch
 * (DISC_ERR_WORKSPACE when missing or too small).  The patterns run in order on `hip_stream`; the
 * call returns once they are enqueued.  A failure of one pattern's launch-time shape check returns
 * that status with the earlier patterns already enqueued. */
enum { DISC_MAX_GRAPH_PATTERNS = 64 };
typedef struct {
  int32_t n_dims, n_inputs, n_outputs;
  int32_t n_patterns;                               /* kernels-worth of fused patterns         */
  int32_t n_intermediates;                          /* values crossing a cut                   */
  int32_t n_buffers;                                /* workspace buffers after reuse           */
  int32_t pattern_id[DISC_MAX_GRAPH_PATTERNS];      /* ids usable with disc_pattern_info       */
  int32_t pattern_ops[DISC_MAX_GRAPH_PATTERNS];     /* graph ops fused into each               */
  int32_t group_of_op[DISC_MAX_OPS];                /* pattern index of each graph op, -1 for
                                                       leaves, OUTPUT ops and dead code        */
} disc_graph_info_t;
int disc_register_graph(disc_ctx* ctx, const disc_op* ops, int n_ops, const disc_constraint* cs, int n_cs,
                        int32_t* graph_id_out);
int disc_graph_info(disc_ctx* ctx, int32_t graph_id, disc_graph_info_t* out);
/* Bytes of DEVICE workspace disc_graph_launch needs at these dims: the planned buffers plus the
 * largest workspace of any of its patterns. */
int disc_graph_workspace_bytes(disc_ctx* ctx, int32_t graph_id, const int64_t* dims, int n_dims, size_t* out);
/* Launches the patterns in order on `hip_stream`; same pointer conventions as disc_launch. */
int disc_graph_launch(disc_ctx* ctx, int32_t graph_id, const int64_t* dims, int n_dims, const void* const* inputs,
                      int n_in, void* const* outputs, int n_out, void* workspace, size_t workspace_bytes,
                      void* hip_stream);


int disc_get_stats(disc_ctx* ctx, disc_stats_t* out);

/* Measurement helpers (not part of the method): a plain 16-byte-vector device copy used as the
 * practical bandwidth ceiling, and an empty kernel used as the launch-latency floor.
 * dst / src are device pointers, 16-byte aligned; bytes a multiple of 16. */
int disc_util_copy(disc_ctx* ctx, void* dst, const void* src, size_t bytes, void* hip_stream);
/* The same copy with non-temporal loads and stores (the faster of the two on large buffers). */
int disc_util_copy_nt(disc_ctx* ctx, void* dst, const void* src, size_t bytes, void* hip_stream);
int disc_util_empty_launch(disc_ctx* ctx, void* hip_stream);
/* A streaming probe with the traffic mix of the row kernels and next to no arithmetic: the practical
 * ceiling those kernels are measured against.  Per element of 2 bytes: kind 0 reads 2 bytes of `a` and
 * 1 byte of `b_or_mask` and writes 2 bytes of `out` (3 read : 2 written, the 12-op pattern's mix);
 * kind 1 reads 2 bytes each of `a` and `b_or_mask` and writes 2 (4 : 2, residual + LayerNorm).  Device
 * pointers, 16-byte aligned; n_elems a multiple of 8; slots_in_flight in {1, 2, 4, 8} (16-byte slots
 * per lane in flight); blocks_per_cu 1..64 (grid = that x CUs, grid-stride). */
int disc_util_mix(disc_ctx* ctx, int kind, int non_temporal, int slots_in_flight, int blocks_per_cu, void* out, const void* a,
                  const void* b_or_mask, size_t n_elems, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* DISC_H_ */

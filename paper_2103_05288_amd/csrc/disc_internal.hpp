// Internal data structures of the host side: pattern IR, constraint classes, the resolved
// node graph, collapsed iteration space, launch recipes.  Nothing here touches the GPU.
#pragma once

#include <cstdint>
#include <map>
#include <string>
#include <vector>

#include "disc.h"

namespace disc {

// Register kind a value is computed in (storage dtype only matters at loads / stores).
enum RegKind { RK_F32 = 0, RK_I32 = 1, RK_I64 = 2, RK_BOOL = 3 };

inline RegKind reg_kind(int dtype) {
  switch (dtype) {
    case DISC_I32: return RK_I32;
    case DISC_I64: return RK_I64;
    case DISC_BOOL: return RK_BOOL;
    default: return RK_F32;
  }
}
inline int dtype_bytes(int dtype) {
  switch (dtype) {
    case DISC_F32: case DISC_I32: return 4;
    case DISC_F16: case DISC_BF16: return 2;
    case DISC_I64: return 8;
    default: return 1;
  }
}
inline bool is_float_dtype(int d) { return d == DISC_F32 || d == DISC_F16 || d == DISC_BF16; }
const char* dtype_ctype(int dtype);   // storage type name in device code
const char* reg_ctype(RegKind k);     // register type name in device code
const char* opcode_name(int opcode);

// ---------------------------------------------------------------------------------------
// Dimension-size equality classes (Section 4.2.1): union-find over "atoms".  Atoms
// [0, n_sym) are the symbolic dims, further atoms are distinct static sizes.
// ---------------------------------------------------------------------------------------
struct DimClasses {
  int n_sym = 0;
  std::vector<int> parent;
  std::vector<int64_t> static_val;      // per atom; -1 = unknown (symbolic)
  std::map<int64_t, int> static_atom;   // static size -> atom

  void init(int n_symbolic);
  int atom(int32_t dim);                 // dim as stored in disc_op::dim
  int find(int a);
  int64_t static_of(int a) { return static_val[find(a)]; }
  // false + message when two different static sizes would become equal
  bool unite(int a, int b, std::string* err);
  bool same(int a, int b) { return find(a) == find(b); }
};

// A value seen from the iteration space: for each axis of the value the root axis it is
// indexed by, or -1 when the axis has static size 1 (contributes nothing to the offset).
typedef std::vector<int> Ctx;

enum Domain { DOM_SCALAR = 0, DOM_ROW = 1, DOM_ELEM = 2 };

// Where an operand / result lives relative to the canonical [outer groups..., inner] space.
enum AccessKind {
  ACC_FULL = 0,     // all outer groups + inner, contiguous: offset = row * inner + col
  ACC_ROWVEC = 1,   // inner only:                            offset = col
  ACC_PERROW = 2,   // all outer groups, no inner:            offset = row
  ACC_SCALAR = 3,   // no group at all:                       offset = 0
  ACC_PARTIAL = 4   // a strict subset of the outer groups (+ inner or not): strided
};

struct Access {
  int value = -1;          // op index of the PARAM / OUTPUT
  int slot = -1;           // k-th input or k-th output pointer
  bool is_output = false;
  int dtype = 0;
  Ctx ctx;
  std::vector<int> groups; // collapsed groups it spans, increasing
  bool has_inner = false;
  AccessKind kind = ACC_FULL;
  // ACC_PARTIAL: index (into Recipe::products) of the stride of each spanned outer group
  std::vector<int> stride_prod;
  // SLICE of a PARAM: `value` is the SLICE op (its dims are what is read), `src_value` the PARAM;
  // the strides are products of the PARAM's own dims and the base offset (index into
  // Analysis::offsets, -1 = none) is the sum of start * stride over the sliced axes
  int src_value = -1;
  int offset_index = -1;
  bool all_outer = false;  // spans every outer group: full-size data, loaded once per row like ACC_FULL
  // PAD of a PARAM: as for SLICE, with the offset negative; `window[t]` (parallel to `groups`, -1 =
  // none) names a pair of shape-calculation values [lo, hi): the operand exists where the index
  // of that group lies inside, the rest of the result is `pad_value`
  bool padded = false;
  double pad_value = 0.0;
  std::vector<int> window;
  // output of a row-reduce pattern that is a sum over the rows (a column sum beside the row
  // reductions): one element per column, accumulated next to the epilogue
  bool col_sum = false;
  // output of a row-reduce pattern that reduces per-row values over the rows to one number
  bool row_red = false;
  // compaction pattern: an input read one element earlier (NE_PREV); outputs that are the kept
  // values (compact), the slot of every element (compact_rank), the number kept (compact_count)
  bool prev = false;
  bool compact = false, compact_rank = false, compact_count = false;
};

// Resolved graph: one node per (value, context) pair actually needed.
struct Node {
  int opcode = 0;
  int dtype = 0;
  RegKind rk = RK_F32;
  int value = -1;           // originating op
  Ctx ctx;
  int in[3] = {-1, -1, -1}; // node ids
  int n_in = 0;
  Domain dom = DOM_SCALAR;
  int phase = 0;            // number of dependent reductions before this value is known
  int access = -1;          // PARAM: index into accesses
  double fconst = 0.0;
  int sym_dim = -1;         // DIM_SIZE
  int reduce_slot = -1;     // REDUCE_*: index of the reduction within its phase
};

struct OutputRef {
  int node = -1;      // the value stored; for a column sum beside row reductions, the value summed
  int access = -1;
  bool col_sum = false;
  bool row_red = false;   // a reduction (red_opcode) of the per-row value `node` over the rows
  int red_opcode = 0;
};

// A product of runtime dims the host evaluates at launch (shape calculation).
struct DimProduct {
  std::vector<int> sym;     // symbolic dim ids
  int64_t stat = 1;         // static factor
};
// Base offset of a sliced operand: sum of start * stride; a start is a symbolic dim id (>= 0) or
// the static value -1 - start.
struct OffsetRecipe {
  std::vector<std::pair<int32_t, DimProduct>> terms;
  bool negative = false;   // PAD: the operand starts `low` elements late, the offset is subtracted
};
// [lo, hi) of a padded operand in the index space of one collapsed group:
// lo = low * inner_sizes, hi = (low + extent) * inner_sizes
struct WindowRecipe {
  int32_t low;             // encoded like a slice start
  int32_t extent_dim;      // the operand's extent along the padded axis (symbolic id or -static)
  DimProduct inner_sizes;  // product of the sizes of the group's axes behind the padded one
};
// Launch-time check of one sliced axis: 0 <= start and start + size <= extent of the operand
struct SliceCheck {
  int32_t start, size_dim, src_dim;   // start: as above; the dims: symbolic id or -static
  int op;
  int axis;
};

struct Analysis {
  int tmpl = DISC_TEMPLATE_LOOP;
  int n_sym = 0;
  std::vector<disc_op> ops;
  std::vector<disc_constraint> cs;
  DimClasses classes;

  // iteration space
  int root_rank = 0;
  std::vector<int32_t> root_dims;        // dim entries (symbolic id or -static) of the root shape
  int reduce_axis = -1;                  // root axis, -1 for loop fusion
  bool flat = false;                     // loop fusion over values that only agree in element count
  std::vector<std::vector<int>> groups;  // collapsed groups of consecutive root axes
  int inner_group = -1;                  // index of the innermost group
  int mid_group = -1;                    // column reduce: the reduced group

  std::vector<Node> nodes;               // topological order
  std::vector<Access> accesses;
  std::vector<OutputRef> outputs;        // in OUTPUT-op order
  std::vector<int> reduces[8];           // reduce nodes per phase
  int n_phases = 0;
  int n_col_sums = 0;                    // row reduce: outputs that are sums over the rows
  int n_row_reds = 0;                    // row reduce: outputs that reduce per-row values over the rows to one number
  int compact_keep = -1;                 // compaction pattern: node of the predicate
  int n_inputs = 0, n_outputs = 0;
  bool needs_decomp = false;             // some access is ACC_PARTIAL

  // launch recipes
  std::vector<DimProduct> group_size;    // per collapsed group
  std::vector<DimProduct> products;      // strides of partial accesses
  std::vector<OffsetRecipe> offsets;     // base offsets of sliced operands (kernel argument st<products.size() + i>)
  std::vector<SliceCheck> slice_checks;
  // flat loop fusion: element counts of the operands and results, each of which must equal the
  // element count of the iteration space at launch (the tensor-size equalities the decision used)
  std::vector<std::pair<int, DimProduct>> numel_checks;   // (op index, its element count)
  std::vector<WindowRecipe> windows;     // kernel arguments st<products + offsets + 2 i> (lo) and + 1 (hi)
  std::vector<int> dim_size_syms;        // symbolic dims referenced by DIM_SIZE nodes
  int vec_width = 1;                     // elements per vector slot
};

// Kernel-argument block layout shared by the code generator and the launcher.
struct ArgField {
  enum Kind { ROWS, INNER, NSLOTS, SPR, SPR_DIV, GROUP_DIV, GROUP_SIZE, IN_PTR, OUT_PTR, STRIDE,
              DIMF, DIMI, MID, WS_PTR, AUX } kind;
  int index = 0;       // group / pointer / product / dim index
  int offset = 0;
  int size = 0;
};
struct ArgLayout {
  std::vector<ArgField> fields;
  int size = 0;
};

struct Generated {
  std::string source;
  ArgLayout args;
  std::string prefix;                 // per-pattern prefix of the entry-point symbols (profilers tell patterns apart)
  std::vector<std::string> kernels;   // entry-point names present in the module, without the prefix
  int n_acc_cells = 0;                // column reduce: 8-byte cells per partial accumulator
  int n_red_planes = 0;               // column reduce: reduce-result planes in the workspace
  bool has_epilogue = true;           // column reduce: some output keeps the reduced axis
  int n_col_sums = 0;                 // row reduce: outputs summed over the rows (second launch combines the partial sums)
  int n_row_reds = 0;                 // row reduce: per-row values reduced over the rows to one number (last launch)
  std::vector<int> staged_elem_bytes; // row reduce: element size of each row vector that can be staged in LDS
  bool row_tail_ok = false;           // row reduce: there are versions that take a ragged end of a row as single elements (_t)
  bool row_shift_ok = false;          // ... and their vector slots may be shifted to the 16-byte boundaries of the tensor
  std::vector<std::string> field_names;   // member name of each args.fields entry in Pat::Args
};

// Every entry point a pattern module can hold has a fixed number, so that the launch path
// indexes arrays (function handles, residency) and never looks a name up.  The row kernels are
// numbered by their five version bits: K_ROW_BASE + row_kernel_index(...).
enum KernelId {
  K_LOOP_VEC = 0, K_LOOP_VEC_I64, K_LOOP_SCALAR, K_LOOP_SCALAR_I64, K_LOOP_VEC_NT,
  K_ROW_STREAM_VEC, K_ROW_STREAM_SCALAR, K_COLSUM_FINISH, K_ROWRED_FINISH,
  K_COL_PARTIAL_VEC, K_COL_PARTIAL_SCALAR, K_COL_FINISH, K_COL_STRIP_VEC, K_COL_STRIP_SCALAR,
  K_COL_EPI_VEC, K_COL_EPI_VEC_I64, K_COL_EPI_SCALAR, K_COL_EPI_SCALAR_I64, K_COL_EPI_VEC_NT,
  K_TRANSPOSE_TILE,
  K_COL_EPI2_VEC, K_COL_EPI2_VEC_NT, K_COL_EPI2_SCALAR,
  K_COMPACT_COUNT_VEC, K_COMPACT_COUNT_SCALAR, K_COMPACT_SCAN, K_COMPACT_SCATTER_VEC, K_COMPACT_SCATTER_SCALAR,
  K_ROW_BASE,
  K_COUNT = K_ROW_BASE + 96
};
// k_row_{vec|scalar}_nv{1|2|3}[w][_s][_nt|_e|_t]: scalar access, instantiated slots per lane, block above
// 256 threads, row vectors staged in LDS, then the access flavour: 0 = any row length, 1 (_nt) = rows
// of whole slots with non-temporal accesses of the full-size operands, 2 (_e) = rows of whole slots,
// 3 (_t) = whole slots + the ragged end of the row as single elements
inline int row_kernel_index(bool scalar, int inst, bool wide, bool staged, int flavour) {
  return ((((scalar ? 1 : 0) * 3 + (inst - 1)) * 2 + (wide ? 1 : 0)) * 2 + (staged ? 1 : 0)) * 4 + flavour;
}
const char* kernel_name(int kid);            // entry-point name without the pattern prefix
int kernel_id(const std::string& name);      // -1 when unknown (registration time only)

// Optional restriction of the generated module: only the named entry points (without prefix).
struct GenOptions {
  std::vector<std::string> only_kernels;
};

// checker.cpp: validate, close constraints, decide fusion, resolve contexts, collapse.
// number of operands (`in[]` entries that mean something) of an opcode
int operand_count(int opcode);

int analyze(const disc_op* ops, int n_ops, const disc_constraint* cs, int n_cs, Analysis* out,
            std::string* err);

// codegen.cpp
int generate(const Analysis& an, const std::string& prefix, Generated* out, std::string* err,
             const GenOptions* opt = nullptr);

}  // namespace disc

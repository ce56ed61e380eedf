// Registration-time analysis of a fusion pattern (host only, no GPU).
//
//  1. validate the op list (static rank, Section 2);
//  2. close the shape constraints: dimension-size equality classes from op semantics and
//     from the caller, tensor-size equality from the caller (Section 4.2.1);
//  3. fusion decision: prove from shape propagation + constraints that every op shares one
//     iteration space, and pick the template (Section 4.3);
//  4. resolve every value to the root axes it is indexed by (implicit broadcast: a broadcast
//     is an indexing function on the small operand, never materialised);
//  5. merge root axes that play identical roles for every operand, so index arithmetic is
//     done once per group instead of once per axis (the index-calculation
//     simplification of Section 4.2.1);
//  6. write the shape-calculation recipes the launch path evaluates.
#include <algorithm>
#include <cstdio>
#include <cstring>
#include <set>
#include <functional>

#include "disc_internal.hpp"

namespace disc {

const char* dtype_ctype(int d) {
  switch (d) {
    case DISC_F32: return "float";
    case DISC_F16: return "_Float16";
    case DISC_BF16: return "__bf16";
    case DISC_I32: return "int";
    case DISC_I64: return "disc::i64";
    default: return "disc::u8";
  }
}
const char* reg_ctype(RegKind k) {
  switch (k) {
    case RK_I32: return "int";
    case RK_I64: return "disc::i64";
    case RK_BOOL: return "bool";
    default: return "float";
  }
}
const char* opcode_name(int oc) {
  static const char* names[] = {"param", "const", "dim_size", "neg", "abs", "exp", "log", "tanh",
    "sqrt", "rsqrt", "rcp", "sigmoid", "erf", "add", "sub", "mul", "div", "max", "min", "pow",
    "lt", "le", "gt", "ge", "eq", "ne", "select", "cast", "broadcast", "reduce_sum", "reduce_max",
    "reduce_min", "reduce_argmax", "output", "slice", "pad", "transpose", "ne_prev", "compact", "compact_count",
    "compact_rank"};
  if (oc < 0 || oc >= DISC_OPCODE_COUNT) return "?";
  return names[oc];
}

// ------------------------------------------------------------------ DimClasses
void DimClasses::init(int n_symbolic) {
  n_sym = n_symbolic;
  parent.resize(n_sym);
  static_val.assign(n_sym, -1);
  for (int i = 0; i < n_sym; ++i) parent[i] = i;
  static_atom.clear();
}
int DimClasses::atom(int32_t dim) {
  if (dim >= 0) return dim;
  int64_t sz = -(int64_t)dim;
  auto it = static_atom.find(sz);
  if (it != static_atom.end()) return it->second;
  int a = (int)parent.size();
  parent.push_back(a);
  static_val.push_back(sz);
  static_atom[sz] = a;
  return a;
}
int DimClasses::find(int a) {
  while (parent[a] != a) {
    parent[a] = parent[parent[a]];
    a = parent[a];
  }
  return a;
}
bool DimClasses::unite(int a, int b, std::string* err) {
  a = find(a);
  b = find(b);
  if (a == b) return true;
  if (static_val[a] >= 0 && static_val[b] >= 0 && static_val[a] != static_val[b]) {
    if (err) {
      char buf[128];
      snprintf(buf, sizeof buf, "static sizes %lld and %lld would have to be equal",
               (long long)static_val[a], (long long)static_val[b]);
      *err = buf;
    }
    return false;
  }
  // keep the smaller atom id as representative so class ids are stable
  if (b < a) std::swap(a, b);
  parent[b] = a;
  if (static_val[a] < 0) static_val[a] = static_val[b];
  return true;
}

namespace {

bool is_unary(int oc) { return oc >= DISC_NEG && oc <= DISC_ERF; }
bool is_binary(int oc) { return oc >= DISC_ADD && oc <= DISC_POW; }
bool is_compare(int oc) { return oc >= DISC_LT && oc <= DISC_NE; }
bool is_reduce(int oc) { return oc >= DISC_REDUCE_SUM && oc <= DISC_REDUCE_ARGMAX; }
bool is_elementwise(int oc) {
  return is_unary(oc) || is_binary(oc) || is_compare(oc) || oc == DISC_SELECT || oc == DISC_CAST;
}
int n_operands(int oc) {
  if (oc <= DISC_DIM_SIZE) return 0;
  if (is_unary(oc) || oc == DISC_CAST || oc == DISC_BROADCAST || is_reduce(oc) || oc == DISC_OUTPUT || oc == DISC_SLICE || oc == DISC_PAD || oc == DISC_TRANSPOSE ||
      oc == DISC_NE_PREV || oc == DISC_COMPACT_COUNT || oc == DISC_COMPACT_RANK)
    return 1;
  if (oc == DISC_COMPACT) return 2;
  if (oc == DISC_SELECT) return 3;
  return 2;
}

struct Builder {
  Analysis& an;
  std::string& err;
  std::map<std::pair<int, Ctx>, int> memo;
  int status = DISC_OK;

  Builder(Analysis& a, std::string& e) : an(a), err(e) {}

  int fail(int code, const std::string& msg) {
    if (status == DISC_OK) {
      status = code;
      err = msg;
    }
    return -1;
  }
  std::string opdesc(int v) {
    char buf[64];
    snprintf(buf, sizeof buf, "op %d (%s)", v, opcode_name(an.ops[v].opcode));
    return buf;
  }
  bool dim_is_one(int32_t d) { return an.classes.static_of(an.classes.atom(d)) == 1; }
  bool shapes_match_root(const disc_op& op) {
    if (op.rank != an.root_rank) return false;
    for (int k = 0; k < op.rank; ++k)
      if (!an.classes.same(an.classes.atom(op.dim[k]), an.classes.atom(an.root_dims[k]))) return false;
    return true;
  }
  // axis k of a SLICE / PAD op covers the whole axis of its operand: static start 0 and provably
  // the same size (a TRANSPOSE covers every axis)
  bool slice_axis_full(const disc_op& op, int k) {
    if (op.opcode == DISC_TRANSPOSE) return true;
    const disc_op& src = an.ops[op.in[0]];
    return op.axis_map[k] == -1 && an.classes.same(an.classes.atom(op.dim[k]), an.classes.atom(src.dim[k]));
  }
  // drop axes of static size 1 from a context (they contribute offset 0)
  Ctx normalise(const disc_op& op, Ctx c) {
    for (int k = 0; k < op.rank; ++k)
      if (dim_is_one(op.dim[k])) c[k] = -1;
    return c;
  }

  // Resolve value v as seen through context c; returns node id.
  int demand(int v, Ctx c) {
    const disc_op& op = an.ops[v];
    c = normalise(op, c);
    auto key = std::make_pair(v, c);
    auto it = memo.find(key);
    if (it != memo.end()) return it->second;
    Node n;
    n.opcode = op.opcode;
    n.dtype = op.dtype;
    n.rk = reg_kind(op.dtype);
    n.value = v;
    n.ctx = c;
    const int oc = op.opcode;
    if (oc == DISC_PARAM) {
      Access a;
      a.value = v;
      a.is_output = false;
      a.dtype = op.dtype;
      a.ctx = c;
      int slot = 0;
      for (int i = 0; i < v; ++i)
        if (an.ops[i].opcode == DISC_PARAM) ++slot;
      a.slot = slot;
      n.access = (int)an.accesses.size();
      an.accesses.push_back(a);
    } else if (oc == DISC_SLICE || oc == DISC_PAD || oc == DISC_TRANSPOSE) {
      // an indexing function on the sliced / padded / transposed PARAM: the node is a PARAM node
      // whose access carries the PARAM's own extents and the offsets.  The context of the access
      // is kept in the order of the PARAM's axes.
      n.opcode = DISC_PARAM;
      Access a;
      a.value = v;
      a.src_value = op.in[0];
      a.padded = oc == DISC_PAD;
      a.pad_value = op.fconst;
      if (oc == DISC_TRANSPOSE) {
        Ctx pc(c.size(), -1);
        for (int k = 0; k < op.rank; ++k) pc[op.axis_map[k]] = c[k];
        c = pc;
      }
      a.is_output = false;
      a.dtype = op.dtype;
      a.ctx = c;
      int slot = 0;
      for (int i = 0; i < op.in[0]; ++i)
        if (an.ops[i].opcode == DISC_PARAM) ++slot;
      a.slot = slot;
      n.access = (int)an.accesses.size();
      an.accesses.push_back(a);
    } else if (oc == DISC_NE_PREV) {
      // two reads of the same PARAM: the element itself and its predecessor (an access of its own,
      // one element earlier)
      n.in[0] = demand(op.in[0], c);
      if (n.in[0] < 0) return -1;
      Node pn;
      const disc_op& src = an.ops[op.in[0]];
      pn.opcode = DISC_PARAM;
      pn.dtype = src.dtype;
      pn.rk = reg_kind(src.dtype);
      pn.value = op.in[0];
      pn.ctx = c;
      Access a = an.accesses[an.nodes[n.in[0]].access];
      a.prev = true;
      pn.access = (int)an.accesses.size();
      an.accesses.push_back(a);
      n.in[1] = (int)an.nodes.size();
      an.nodes.push_back(pn);
      n.n_in = 2;
    } else if (oc == DISC_COMPACT) {
      // the kept values are the value itself; where they go is decided by the kernel
      int id = demand(op.in[0], c);
      memo[key] = id;
      return id;
    } else if (oc == DISC_CONST) {
      n.fconst = op.fconst;
    } else if (oc == DISC_DIM_SIZE) {
      n.sym_dim = op.axis_map[0];
    } else if (oc == DISC_BROADCAST || oc == DISC_OUTPUT) {
      // no computation: alias of the operand seen through the composed context
      const disc_op& src = an.ops[op.in[0]];
      Ctx sc(src.rank, -1);
      if (oc == DISC_OUTPUT) {
        sc = c;
      } else {
        for (int k = 0; k < src.rank; ++k) sc[k] = c[op.axis_map[k]];
      }
      int id = demand(op.in[0], sc);
      memo[key] = id;
      return id;
    } else if (is_reduce(oc)) {
      if (an.reduce_axis < 0) return fail(DISC_ERR_UNFUSIBLE, opdesc(v) + ": reduction in a loop-fusion pattern");
      Ctx natural;
      for (int k = 0; k < an.root_rank; ++k)
        if (k != an.reduce_axis) natural.push_back(k);
      Ctx nn = normalise(op, natural);
      if (c != nn)
        return fail(DISC_ERR_UNFUSIBLE, opdesc(v) + ": reduction result is consumed along other axes than "
                    "the ones it was produced on; the iteration spaces cannot be proved compatible");
      Ctx ident(an.root_rank);
      for (int k = 0; k < an.root_rank; ++k) ident[k] = k;
      n.in[0] = demand(op.in[0], ident);
      n.n_in = 1;
      if (n.in[0] < 0) return -1;
    } else {
      const int no = n_operands(oc);
      for (int k = 0; k < no; ++k) {
        const disc_op& src = an.ops[op.in[k]];
        Ctx sc = src.rank == 0 ? Ctx() : c;
        n.in[k] = demand(op.in[k], sc);
        if (n.in[k] < 0) return -1;
      }
      n.n_in = no;
    }
    int id = (int)an.nodes.size();
    an.nodes.push_back(n);
    memo[key] = id;
    return id;
  }
};

void mul_into(DimProduct& p, const DimClasses&, int32_t dim) {
  if (dim >= 0) p.sym.push_back(dim); else p.stat *= -(int64_t)dim;
}

}  // namespace

int operand_count(int opcode) { return n_operands(opcode); }

namespace {
struct KernelNames {
  std::string name[K_COUNT];
  KernelNames() {
    static const char* const fixed[K_ROW_BASE] = {
        "k_loop_vec", "k_loop_vec_i64", "k_loop_scalar", "k_loop_scalar_i64", "k_loop_vec_nt",
        "k_row_stream_vec", "k_row_stream_scalar", "k_colsum_finish", "k_rowred_finish",
        "k_col_partial_vec", "k_col_partial_scalar", "k_col_finish", "k_col_strip_vec", "k_col_strip_scalar",
        "k_col_epi_vec", "k_col_epi_vec_i64", "k_col_epi_scalar", "k_col_epi_scalar_i64", "k_col_epi_vec_nt",
        "k_transpose_tile", "k_col_epi2_vec", "k_col_epi2_vec_nt", "k_col_epi2_scalar",
        "k_compact_count_vec", "k_compact_count_scalar", "k_compact_scan", "k_compact_scatter_vec", "k_compact_scatter_scalar"};
    for (int i = 0; i < K_ROW_BASE; ++i) name[i] = fixed[i];
    for (int sc = 0; sc < 2; ++sc)
      for (int n = 1; n <= 3; ++n)
        for (int w = 0; w < 2; ++w)
          for (int st = 0; st < 2; ++st)
            for (int fl = 0; fl < 4; ++fl)
              name[K_ROW_BASE + row_kernel_index(sc, n, w, st, fl)] = std::string("k_row_") + (sc ? "scalar" : "vec") + "_nv" +
                                                                      std::to_string(n) + (w ? "w" : "") + (st ? "_s" : "") +
                                                                      (fl == 1 ? "_nt" : fl == 2 ? "_e" : fl == 3 ? "_t" : "");
  }
};
const KernelNames& kernel_names() {
  static const KernelNames t;
  return t;
}
}  // namespace

const char* kernel_name(int kid) { return kid >= 0 && kid < K_COUNT ? kernel_names().name[kid].c_str() : "?"; }
int kernel_id(const std::string& name) {
  const KernelNames& t = kernel_names();
  for (int i = 0; i < K_COUNT; ++i)
    if (t.name[i] == name) return i;
  return -1;
}

// A pattern with DISC_COMPACT / COMPACT_COUNT / COMPACT_RANK outputs (Section 2: Unique-style ops,
// whose output size depends on the input values): a loop fusion over rank-1 values of one length N
// that computes the values and ONE predicate; what is kept goes to the outputs in order.
// Called after validation and constraint closure.
static int analyze_compact(Analysis& an, std::string& err) {
  const std::vector<disc_op>& ops = an.ops;
  const int n_ops = (int)ops.size();
  char buf[256];
  auto fail = [&](int code, int i, const char* what) {
    snprintf(buf, sizeof buf, "op %d (%s): %s", i, opcode_name(ops[i].opcode), what);
    err = buf;
    return code;
  };
  int keep = -1, root = -1;
  for (int i = 0; i < n_ops; ++i) {
    const disc_op& op = ops[i];
    const int oc = op.opcode;
    if (oc == DISC_BROADCAST || is_reduce(oc) || oc == DISC_SLICE || oc == DISC_PAD || oc == DISC_TRANSPOSE)
      return fail(DISC_ERR_UNFUSIBLE, i, "a pattern with compacted outputs is a loop fusion over rank-1 values of one length: "
                                         "no broadcast, reduction, slice, pad or transpose");
    if (op.rank > 1) return fail(DISC_ERR_UNFUSIBLE, i, "a pattern with compacted outputs works on rank-1 values");
    if (oc == DISC_COMPACT || oc == DISC_COMPACT_COUNT || oc == DISC_COMPACT_RANK) {
      const int k = oc == DISC_COMPACT ? op.in[1] : op.in[0];
      if (keep >= 0 && k != keep) return fail(DISC_ERR_UNFUSIBLE, i, "all compactions of one pattern share one predicate");
      keep = k;
      if (oc == DISC_COMPACT && ops[op.in[0]].opcode >= DISC_COMPACT && ops[op.in[0]].opcode <= DISC_COMPACT_RANK)
        return fail(DISC_ERR_UNFUSIBLE, i, "a compaction result cannot be compacted again in the same pattern");
    } else if (oc != DISC_OUTPUT) {
      for (int k = 0; k < n_operands(oc); ++k)
        if (ops[op.in[k]].opcode >= DISC_COMPACT && ops[op.in[k]].opcode <= DISC_COMPACT_RANK)
          return fail(DISC_ERR_UNFUSIBLE, i, "a compaction result may only feed OUTPUTs (its size is not known to the host)");
    } else if (ops[op.in[0]].opcode < DISC_COMPACT || ops[op.in[0]].opcode > DISC_COMPACT_RANK) {
      return fail(DISC_ERR_UNFUSIBLE, i, "every OUTPUT of a pattern with compacted outputs is a COMPACT, COMPACT_COUNT or COMPACT_RANK result");
    }
    if (op.rank == 1 && root < 0) root = i;
  }
  if (keep < 0) { err = "NE_PREV is supported in patterns whose outputs are compacted (COMPACT / COMPACT_COUNT / COMPACT_RANK)"; return DISC_ERR_UNFUSIBLE; }
  DimClasses& dc = an.classes;
  for (int i = 0; i < n_ops; ++i)
    if (ops[i].rank == 1 && !dc.same(dc.atom(ops[i].dim[0]), dc.atom(ops[root].dim[0])))
      return fail(DISC_ERR_UNFUSIBLE, i, "its length cannot be proved equal to that of the other values; add a DIM_EQ constraint");
  an.tmpl = DISC_TEMPLATE_COMPACT;
  an.root_rank = 1;
  an.root_dims.assign(1, ops[root].dim[0]);
  an.reduce_axis = -1;
  an.groups.assign(1, std::vector<int>(1, 0));
  an.inner_group = 0;
  Builder b(an, err);
  const Ctx ident(1, 0);
  an.compact_keep = b.demand(keep, ident);
  if (an.compact_keep < 0) return b.status;
  for (int i = 0; i < n_ops; ++i) {
    if (ops[i].opcode != DISC_OUTPUT) continue;
    const disc_op& src = ops[ops[i].in[0]];
    OutputRef o;
    Access a;
    a.value = i;
    a.is_output = true;
    a.dtype = ops[i].dtype;
    a.slot = (int)an.outputs.size();
    if (src.opcode == DISC_COMPACT) {
      o.node = b.demand(src.in[0], ident);
      if (o.node < 0) return b.status;
      a.compact = true;
      a.ctx = ident;
    } else {
      o.node = an.compact_keep;
      a.compact_rank = src.opcode == DISC_COMPACT_RANK;
      a.compact_count = src.opcode == DISC_COMPACT_COUNT;
      if (a.compact_rank) a.ctx = ident;
    }
    o.access = (int)an.accesses.size();
    an.accesses.push_back(a);
    an.outputs.push_back(o);
  }
  if (b.status != DISC_OK) return b.status;
  for (auto& a : an.accesses) {
    a.groups.clear();
    if (!a.ctx.empty()) a.groups.push_back(0);
    a.has_inner = !a.ctx.empty();
    a.kind = a.has_inner ? ACC_FULL : ACC_SCALAR;
  }
  for (auto& n : an.nodes) {
    n.dom = (n.opcode == DISC_CONST || n.opcode == DISC_DIM_SIZE || n.ctx.empty()) ? DOM_SCALAR : DOM_ELEM;
    n.phase = 0;
  }
  an.n_phases = 0;
  an.group_size.assign(1, DimProduct());
  mul_into(an.group_size[0], dc, ops[root].dim[0]);
  for (auto& n : an.nodes)
    if (n.opcode == DISC_DIM_SIZE &&
        std::find(an.dim_size_syms.begin(), an.dim_size_syms.end(), n.sym_dim) == an.dim_size_syms.end())
      an.dim_size_syms.push_back(n.sym_dim);
  int min_bytes = 8;
  for (const auto& a : an.accesses)
    if (a.has_inner && a.dtype != DISC_BOOL && !a.compact_rank) min_bytes = std::min(min_bytes, dtype_bytes(a.dtype));
  an.vec_width = std::min(8, 16 / min_bytes);
  return DISC_OK;
}

// loop_sides: sums over the rows next to a loop fusion may ride along in a row template without
// reduction phases; *used_loop_sides tells whether that rule decided the template
static int analyze_impl(const disc_op* ops, int n_ops, const disc_constraint* cs, int n_cs, Analysis* out,
                        std::string* errp, bool loop_sides, bool* used_loop_sides) {
  Analysis& an = *out;
  std::string& err = *errp;
  char buf[400];
  if (!ops || n_ops <= 0) { err = "empty op list"; return DISC_ERR_INVALID_ARG; }
  if (n_ops > DISC_MAX_OPS) { err = "too many ops"; return DISC_ERR_BAD_PATTERN; }
  if (n_cs < 0 || (n_cs > 0 && !cs)) { err = "bad constraint list"; return DISC_ERR_INVALID_ARG; }
  an.ops.assign(ops, ops + n_ops);
  an.cs.assign(cs, cs + n_cs);

  // ---- 1. structural validation ---------------------------------------------------------
  int n_sym = 0, n_out = 0, n_in = 0;
  std::vector<char> is_output_src(n_ops, 0);
  for (int i = 0; i < n_ops; ++i) {
    const disc_op& op = ops[i];
    auto bad = [&](const char* what) {
      snprintf(buf, sizeof buf, "op %d (%s): %s", i, opcode_name(op.opcode), what);
      err = buf;
      return DISC_ERR_BAD_PATTERN;
    };
    if (op.opcode < 0 || op.opcode >= DISC_OPCODE_COUNT) return bad("unknown opcode");
    if (op.dtype < DISC_F32 || op.dtype > DISC_BOOL) return bad("unknown dtype");
    if (op.rank < 0 || op.rank > DISC_MAX_RANK) return bad("rank outside 0..4 (static rank only)");
    for (int k = 0; k < op.rank; ++k) {
      if (op.dim[k] >= DISC_MAX_DIMS) return bad("symbolic dim id too large");
      if (op.dim[k] >= 0) n_sym = std::max(n_sym, op.dim[k] + 1);
    }
    const int no = n_operands(op.opcode);
    for (int k = 0; k < no; ++k) {
      if (op.in[k] < 0 || op.in[k] >= i) return bad("operand must name an earlier op");
      if (ops[op.in[k]].opcode == DISC_OUTPUT) return bad("an OUTPUT op is not a value");
    }
    const int oc = op.opcode;
    if (oc == DISC_CONST && op.rank != 0) return bad("CONST must have rank 0");
    if (oc == DISC_DIM_SIZE) {
      if (op.rank != 0) return bad("DIM_SIZE must have rank 0");
      if (op.axis_map[0] < 0 || op.axis_map[0] >= DISC_MAX_DIMS) return bad("DIM_SIZE of an unknown dim");
      n_sym = std::max(n_sym, op.axis_map[0] + 1);
      if (op.dtype == DISC_BOOL) return bad("DIM_SIZE cannot be bool");
    }
    if (oc == DISC_PARAM) ++n_in;
    if (oc == DISC_OUTPUT) {
      ++n_out;
      if (op.dtype != ops[op.in[0]].dtype) return bad("OUTPUT dtype differs from its value");
      if (op.rank != ops[op.in[0]].rank) return bad("OUTPUT rank differs from its value");
      if (op.rank == 0 && !is_reduce(ops[op.in[0]].opcode) && ops[op.in[0]].opcode != DISC_COMPACT_COUNT)
        return bad("rank-0 outputs are supported only for reductions of per-row values over the rows and for COMPACT_COUNT");
    }
    if (is_unary(oc) && oc != DISC_NEG && oc != DISC_ABS && !is_float_dtype(op.dtype))
      return bad("transcendental op needs a float dtype");
    if (is_unary(oc) && reg_kind(op.dtype) == RK_BOOL) return bad("arithmetic on bool");
    if (is_binary(oc)) {
      if (reg_kind(op.dtype) == RK_BOOL) return bad("arithmetic result cannot be bool");
      for (int k = 0; k < 2; ++k)
        if (reg_kind(ops[op.in[k]].dtype) == RK_BOOL) return bad("arithmetic on bool (cast first)");
      if (!is_float_dtype(op.dtype))
        for (int k = 0; k < 2; ++k)
          if (is_float_dtype(ops[op.in[k]].dtype)) return bad("float operand of an integer op (cast first)");
      if (oc == DISC_POW && !is_float_dtype(op.dtype)) return bad("POW needs a float dtype");
    }
    if (is_compare(oc) && op.dtype != DISC_BOOL) return bad("comparison result must be DISC_BOOL");
    if (oc == DISC_SELECT) {
      for (int k = 1; k < 3; ++k)
        if (is_float_dtype(ops[op.in[k]].dtype) != is_float_dtype(op.dtype) ||
            (reg_kind(op.dtype) == RK_BOOL) != (reg_kind(ops[op.in[k]].dtype) == RK_BOOL))
          return bad("SELECT branches must have the kind of the result");
    }
    if (is_reduce(oc)) {
      const disc_op& src = ops[op.in[0]];
      if (reg_kind(src.dtype) == RK_BOOL) return bad("reduction over bool (cast first)");
      if (oc == DISC_REDUCE_ARGMAX) {
        if (op.dtype != DISC_I32 && op.dtype != DISC_I64) return bad("ARGMAX result must be I32 or I64");
      } else if (is_float_dtype(src.dtype) != is_float_dtype(op.dtype) || reg_kind(op.dtype) == RK_BOOL) {
        return bad("reduction result must have the kind of its operand");
      }
      if (src.rank < 1 || op.rank != src.rank - 1) return bad("reduce result must drop exactly one axis");
      if (op.axis_map[0] < 0 || op.axis_map[0] >= src.rank) return bad("reduce axis out of range");
    }
    if (oc == DISC_SLICE || oc == DISC_PAD) {
      const disc_op& src = ops[op.in[0]];
      if (src.opcode != DISC_PARAM) return bad("SLICE / PAD apply to a PARAM (slice or pad the input, then compute)");
      if (src.dtype != op.dtype) return bad("SLICE / PAD change dtype");
      if (src.rank != op.rank || op.rank < 1) return bad("SLICE / PAD keep the rank of their operand (>= 1)");
      for (int k = 0; k < op.rank; ++k) {
        if (op.axis_map[k] >= DISC_MAX_DIMS) return bad("SLICE start / PAD low names an unknown dim");
        if (op.axis_map[k] >= 0) n_sym = std::max(n_sym, op.axis_map[k] + 1);
      }
    }
    if (oc == DISC_TRANSPOSE) {
      const disc_op& src = ops[op.in[0]];
      if (src.opcode != DISC_PARAM) return bad("TRANSPOSE applies to a PARAM (transpose the input, then compute)");
      if (src.dtype != op.dtype) return bad("TRANSPOSE changes dtype");
      if (src.rank != op.rank || op.rank < 1) return bad("TRANSPOSE keeps the rank of its operand (>= 1)");
      int seen = 0;
      for (int k = 0; k < op.rank; ++k) {
        if (op.axis_map[k] < 0 || op.axis_map[k] >= op.rank || (seen >> op.axis_map[k] & 1)) return bad("TRANSPOSE needs a permutation");
        seen |= 1 << op.axis_map[k];
      }
    }
    if (oc == DISC_NE_PREV) {
      const disc_op& src = ops[op.in[0]];
      if (src.opcode != DISC_PARAM || src.rank != 1) return bad("NE_PREV applies to a PARAM of rank 1");
      if (op.dtype != DISC_BOOL || op.rank != 1) return bad("NE_PREV gives a DISC_BOOL value of rank 1");
    }
    if (oc == DISC_COMPACT) {
      if (op.rank != 1 || ops[op.in[0]].rank != 1 || ops[op.in[1]].rank != 1) return bad("COMPACT takes and gives rank-1 values");
      if (ops[op.in[1]].dtype != DISC_BOOL) return bad("COMPACT's second operand is the DISC_BOOL predicate");
      if (ops[op.in[0]].dtype != op.dtype) return bad("COMPACT changes dtype");
    }
    if (oc == DISC_COMPACT_COUNT || oc == DISC_COMPACT_RANK) {
      if (ops[op.in[0]].dtype != DISC_BOOL || ops[op.in[0]].rank != 1) return bad("operand must be a DISC_BOOL predicate of rank 1");
      if (op.dtype != DISC_I32 && op.dtype != DISC_I64) return bad("result must be DISC_I32 or DISC_I64");
      if (op.rank != (oc == DISC_COMPACT_RANK ? 1 : 0)) return bad("COMPACT_COUNT has rank 0, COMPACT_RANK rank 1");
    }
    if (oc == DISC_BROADCAST) {
      const disc_op& src = ops[op.in[0]];
      if (src.dtype != op.dtype) return bad("BROADCAST changes dtype");
      if (src.rank > op.rank) return bad("BROADCAST to a lower rank");
      for (int k = 0; k < src.rank; ++k) {
        if (op.axis_map[k] < 0 || op.axis_map[k] >= op.rank) return bad("BROADCAST axis_map out of range");
        if (k > 0 && op.axis_map[k] <= op.axis_map[k - 1]) return bad("BROADCAST axis_map must be strictly increasing");
      }
    }
    if (is_elementwise(oc)) {
      for (int k = 0; k < no; ++k) {
        const disc_op& src = ops[op.in[k]];
        if (src.rank != 0 && src.rank != op.rank) return bad("element-wise operand rank differs from result rank");
      }
    }
  }
  if (n_out == 0) { err = "pattern has no OUTPUT"; return DISC_ERR_BAD_PATTERN; }
  an.n_sym = n_sym;
  an.n_inputs = n_in;
  an.n_outputs = n_out;

  // ---- 2. constraint closure ------------------------------------------------------------
  DimClasses& dc = an.classes;
  dc.init(n_sym);
  auto unite = [&](int i, int32_t a, int32_t b) -> bool {
    std::string e;
    if (!dc.unite(dc.atom(a), dc.atom(b), &e)) {
      snprintf(buf, sizeof buf, "op %d (%s): %s", i, opcode_name(ops[i].opcode), e.c_str());
      err = buf;
      return false;
    }
    return true;
  };
  for (int i = 0; i < n_ops; ++i) {
    const disc_op& op = ops[i];
    const int oc = op.opcode;
    if (is_elementwise(oc) || oc == DISC_OUTPUT) {
      // shape propagation class "same shape": every non-scalar operand has the result's shape
      for (int k = 0; k < n_operands(oc); ++k) {
        const disc_op& src = ops[op.in[k]];
        if (src.rank == 0) continue;
        for (int a = 0; a < op.rank; ++a)
          if (!unite(i, src.dim[a], op.dim[a])) return DISC_ERR_BAD_PATTERN;
      }
    } else if (oc == DISC_TRANSPOSE) {
      const disc_op& src = ops[op.in[0]];
      for (int k = 0; k < op.rank; ++k)
        if (!unite(i, src.dim[op.axis_map[k]], op.dim[k])) return DISC_ERR_BAD_PATTERN;
    } else if (oc == DISC_BROADCAST) {
      const disc_op& src = ops[op.in[0]];
      for (int k = 0; k < src.rank; ++k) {
        if (src.dim[k] == -1) continue;   // static 1 expands (or stays 1)
        if (!unite(i, src.dim[k], op.dim[op.axis_map[k]])) return DISC_ERR_BAD_PATTERN;
      }
    } else if (is_reduce(oc)) {
      const disc_op& src = ops[op.in[0]];
      for (int k = 0, r = 0; k < src.rank; ++k) {
        if (k == op.axis_map[0]) continue;
        if (!unite(i, src.dim[k], op.dim[r])) return DISC_ERR_BAD_PATTERN;
        ++r;
      }
    } else if (oc == DISC_NE_PREV || oc == DISC_COMPACT || oc == DISC_COMPACT_RANK) {
      // shape propagation: one length N for operands and result (a COMPACT result's dim is the
      // upper bound of its data-dependent length)
      for (int k = 0; k < n_operands(oc); ++k)
        if (!unite(i, ops[op.in[k]].dim[0], op.dim[0])) return DISC_ERR_BAD_PATTERN;
    }
  }
  // caller-supplied constraints (what the framework bridging would inject)
  std::vector<std::pair<int, int>> numel_eq;
  for (int c = 0; c < n_cs; ++c) {
    const disc_constraint& k = cs[c];
    auto badc = [&](const char* what) {
      snprintf(buf, sizeof buf, "constraint %d: %s", c, what);
      err = buf;
      return DISC_ERR_BAD_PATTERN;
    };
    if (k.a_value < 0 || k.a_value >= n_ops || k.b_value < 0 || k.b_value >= n_ops) return badc("unknown value");
    if (k.kind == DISC_DIM_EQ) {
      if (k.a_axis < 0 || k.a_axis >= ops[k.a_value].rank || k.b_axis < 0 || k.b_axis >= ops[k.b_value].rank)
        return badc("axis out of range");
      std::string e;
      if (!dc.unite(dc.atom(ops[k.a_value].dim[k.a_axis]), dc.atom(ops[k.b_value].dim[k.b_axis]), &e))
        return badc(e.c_str());
    } else if (k.kind == DISC_NUMEL_EQ) {
      numel_eq.push_back({k.a_value, k.b_value});
    } else {
      return badc("unknown kind");
    }
  }

  // ---- outputs whose size depends on the data ---------------------------------------------------
  for (int i = 0; i < n_ops; ++i)
    if (ops[i].opcode >= DISC_NE_PREV && ops[i].opcode <= DISC_COMPACT_RANK) return analyze_compact(an, err);

  // ---- a transpose on its own -----------------------------------------------------------------
  // PARAM -> TRANSPOSE -> OUTPUT with a permutation that moves the innermost axis is not a fusion
  // pattern (every access of a fused kernel would be strided by a whole row); alone it is a
  // batched 2-D transpose when its axes collapse to [batch,] P, Q <- [batch,] Q, P.
  if (n_ops == 3 && ops[0].opcode == DISC_PARAM && ops[1].opcode == DISC_TRANSPOSE && ops[1].in[0] == 0 &&
      ops[2].opcode == DISC_OUTPUT && ops[2].in[0] == 1) {
    const disc_op& tr = ops[1];
    // result axes that carry an index (size not statically 1), with the operand axis each comes from
    std::vector<int> res_ax, src_ax;
    for (int k = 0; k < tr.rank; ++k)
      if (dc.static_of(dc.atom(tr.dim[k])) != 1) { res_ax.push_back(k); src_ax.push_back(tr.axis_map[k]); }
    bool moves_inner = false;
    if (!src_ax.empty()) {
      int last_src = -1;
      for (int a : src_ax) last_src = std::max(last_src, a);
      moves_inner = src_ax.back() != last_src;
    }
    if (moves_inner) {
      // merge result axes that are neighbours, in order, in the operand too
      std::vector<std::vector<int>> grp;   // result axes per group
      std::vector<int> first_src;          // operand axis of the first member
      for (size_t t = 0; t < res_ax.size(); ++t) {
        bool join = false;
        if (!grp.empty()) {
          const int prev = src_ax[t - 1], cur = src_ax[t];
          join = cur > prev;
          for (int a = prev + 1; a < cur && join; ++a)       // only unit axes may lie between them
            if (dc.static_of(dc.atom(ops[0].dim[a])) != 1) join = false;
        }
        if (join) grp.back().push_back(res_ax[t]);
        else { grp.push_back({res_ax[t]}); first_src.push_back(src_ax[t]); }
      }
      const size_t ng2 = grp.size();
      const bool two = ng2 == 2 && first_src[0] > first_src[1];
      const bool three = ng2 == 3 && first_src[0] < first_src[2] && first_src[2] < first_src[1];
      if (!two && !three) {
        err = "op 1 (transpose): the permutation does not collapse to a batched 2-D transpose";
        return DISC_ERR_UNFUSIBLE;
      }
      an.tmpl = DISC_TEMPLATE_TRANSPOSE;
      an.root_rank = tr.rank;
      an.root_dims.assign(tr.dim, tr.dim + tr.rank);
      an.reduce_axis = -1;
      an.groups = grp;
      an.inner_group = (int)ng2 - 1;
      an.group_size.assign(ng2, DimProduct());
      for (size_t g2 = 0; g2 < ng2; ++g2)
        for (int ax : grp[g2]) mul_into(an.group_size[g2], dc, tr.dim[ax]);
      Access in_a, out_a;
      in_a.value = 0; in_a.slot = 0; in_a.dtype = ops[0].dtype; in_a.kind = ACC_FULL; in_a.has_inner = true;
      out_a.value = 2; out_a.slot = 0; out_a.dtype = ops[2].dtype; out_a.kind = ACC_FULL; out_a.has_inner = true; out_a.is_output = true;
      an.accesses = {in_a, out_a};
      OutputRef o;
      o.node = -1;
      o.access = 1;
      an.outputs = {o};
      an.n_phases = 0;
      an.vec_width = 1;
      return DISC_OK;
    }
  }

  // ---- 3. fusion decision + template -----------------------------------------------------
  // tensor-size classes: two values have provably the same element count when the multisets of
  // their (non-unit) dimension classes agree, or when the caller says so
  auto numel_key = [&](const disc_op& op) {
    std::vector<int> k;
    for (int a = 0; a < op.rank; ++a) {
      int c = dc.find(dc.atom(op.dim[a]));
      if (dc.static_val[c] == 1) continue;
      k.push_back(c);
    }
    std::sort(k.begin(), k.end());
    return k;
  };
  std::vector<int> numel_parent(n_ops);
  for (int i = 0; i < n_ops; ++i) numel_parent[i] = i;
  std::function<int(int)> nfind = [&](int a) {
    while (numel_parent[a] != a) a = numel_parent[a] = numel_parent[numel_parent[a]];
    return a;
  };
  {
    std::map<std::vector<int>, int> first;
    for (int i = 0; i < n_ops; ++i) {
      auto k = numel_key(ops[i]);
      auto it = first.find(k);
      if (it == first.end()) first[k] = i; else numel_parent[nfind(i)] = nfind(it->second);
    }
    for (auto& p : numel_eq) numel_parent[nfind(p.first)] = nfind(p.second);
  }

  int first_reduce = -1;
  for (int i = 0; i < n_ops; ++i)
    if (is_reduce(ops[i].opcode)) { first_reduce = i; break; }
  // Sums over the rows next to reductions over the innermost axis (the weight gradients of a
  // normalisation beside its input gradient): the row template carries them along as per-column
  // partial sums that a second launch combines.  Accepted for a two-dimensional iteration space
  // (other axes of size 1), floating-point sums, results that go straight to outputs.
  std::vector<char> side(n_ops, 0);
  int rows_axis_override = -1;
  if (first_reduce >= 0) {
    auto unit = [&](int32_t d) { return dc.static_val[dc.find(dc.atom(d))] == 1; };
    auto inner_axis = [&](const disc_op& t) {
      for (int k = t.rank - 1; k >= 0; --k) if (!unit(t.dim[k])) return k;
      return t.rank - 1;
    };
    bool mixed = false;
    for (int i = 0; i < n_ops; ++i)
      if (is_reduce(ops[i].opcode) && ops[i].axis_map[0] != ops[first_reduce].axis_map[0]) mixed = true;
    // may reduction i ride along with rows whose innermost axis is a1?
    auto side_ok = [&](int i, int a1) {
      const disc_op& src = ops[ops[i].in[0]];
      const int a2 = ops[i].axis_map[0];
      bool ok = ops[i].opcode == DISC_REDUCE_SUM && a2 < a1 && reg_kind(src.dtype) == RK_F32;
      for (int k = 0; k < src.rank; ++k)
        if (k != a1 && k != a2 && !unit(src.dim[k])) ok = false;
      for (int j = 0; j < n_ops; ++j)
        for (int k = 0; k < operand_count(ops[j].opcode); ++k)
          if (ops[j].in[k] == i && ops[j].opcode != DISC_OUTPUT) ok = false;
      return ok;
    };
    auto non_unit = [&](const disc_op& t) {
      int n = 0;
      for (int k = 0; k < t.rank; ++k) n += unit(t.dim[k]) ? 0 : 1;
      return n;
    };
    int primary = -1;
    if (mixed)
      for (int i = 0; i < n_ops && primary < 0; ++i)
        if (is_reduce(ops[i].opcode) && non_unit(ops[ops[i].in[0]]) >= 2 &&
            ops[i].axis_map[0] == inner_axis(ops[ops[i].in[0]])) primary = i;
    // A reduction of PER-ROW values over the rows, down to one number (the sum of per-row losses,
    // the maximum of per-row maxima): rides along too, one partial result per block.  The source
    // has the rows' axis alone; sum, maximum or minimum of float values; result to outputs only.
    auto scalar_side_ok = [&](int i, int primary_op) {
      const disc_op& src = ops[ops[i].in[0]];
      const disc_op& root = ops[ops[primary_op].in[0]];
      const int a1 = ops[primary_op].axis_map[0];
      if (non_unit(src) != 1 || non_unit(ops[i]) != 0 || non_unit(root) != 2) return false;
      if (ops[i].opcode != DISC_REDUCE_SUM && ops[i].opcode != DISC_REDUCE_MAX && ops[i].opcode != DISC_REDUCE_MIN) return false;
      if (reg_kind(src.dtype) != RK_F32) return false;
      int rows_class = -1, inner_class = dc.find(dc.atom(root.dim[a1])), src_class = -1;
      for (int k = 0; k < root.rank; ++k)
        if (k != a1 && !unit(root.dim[k])) rows_class = dc.find(dc.atom(root.dim[k]));
      for (int k = 0; k < src.rank; ++k)
        if (!unit(src.dim[k])) {
          src_class = dc.find(dc.atom(src.dim[k]));
          if (ops[i].axis_map[0] != k) return false;       // it must be the rows' axis that is reduced
        }
      if (src_class != rows_class || src_class == inner_class) return false;
      for (int j = 0; j < n_ops; ++j)
        for (int k = 0; k < operand_count(ops[j].opcode); ++k)
          if (ops[j].in[k] == i && ops[j].opcode != DISC_OUTPUT) return false;
      return true;
    };
    if (!mixed && loop_sides) {
      // Sums over the rows next to a LOOP fusion (a bias gradient beside an element-wise backward):
      // when every reduction qualifies and some output keeps the full shape, the pattern runs in
      // the row template without reduction phases -- the operands are read once, where a column
      // reduce would read them again for its epilogue.
      const disc_op& src0 = ops[ops[first_reduce].in[0]];
      const int a1 = inner_axis(src0);
      bool ok = ops[first_reduce].axis_map[0] != a1, elem_out = false;
      for (int i = 0; i < n_ops && ok; ++i) {
        if (is_reduce(ops[i].opcode)) ok = side_ok(i, a1);
        if (ops[i].opcode == DISC_OUTPUT && !is_reduce(ops[ops[i].in[0]].opcode) && ops[i].rank == src0.rank) elem_out = true;
      }
      if (ok && elem_out) {
        for (int i = 0; i < n_ops; ++i)
          if (is_reduce(ops[i].opcode)) side[i] = 1;
        rows_axis_override = a1;
        *used_loop_sides = true;
      }
    }
    if (primary >= 0) {
      const int a1 = ops[primary].axis_map[0];
      for (int i = 0; i < n_ops; ++i) {
        if (!is_reduce(ops[i].opcode) || i == primary) continue;
        if (non_unit(ops[ops[i].in[0]]) == 1 && scalar_side_ok(i, primary)) { side[i] = 2; continue; }
        if (ops[i].axis_map[0] == a1) continue;
        const int a2 = ops[i].axis_map[0];
        const bool ok = side_ok(i, a1);
        if (!ok) {
          snprintf(buf, sizeof buf, "op %d (%s) reduces over axis %d while op %d reduces over the innermost axis: a "
                   "reduction over the rows is fused with row reductions only as a floating-point sum over the "
                   "outer axis of a two-dimensional iteration space that feeds outputs alone", i,
                   opcode_name(ops[i].opcode), a2, primary);
          err = buf;
          return DISC_ERR_UNFUSIBLE;
        }
        side[i] = 1;
      }
      first_reduce = primary;
    }
  }
  for (int i = 0; i < n_ops; ++i)
    if (ops[i].opcode == DISC_OUTPUT && ops[i].rank == 0 && side[ops[i].in[0]] != 2) {
      snprintf(buf, sizeof buf, "op %d (output): a rank-0 result is fused only as a sum, maximum or minimum of "
               "per-row float values over the rows of a two-dimensional row-reduce pattern", i);
      err = buf;
      return DISC_ERR_UNFUSIBLE;
    }
  int root_value;
  if (first_reduce >= 0) {
    root_value = ops[first_reduce].in[0];
    an.reduce_axis = rows_axis_override >= 0 ? rows_axis_override : ops[first_reduce].axis_map[0];
  } else {
    root_value = -1;
    for (int i = 0; i < n_ops; ++i)
      if (ops[i].opcode == DISC_OUTPUT) { root_value = ops[i].in[0]; break; }
    an.reduce_axis = -1;
  }
  an.root_rank = ops[root_value].rank;
  an.root_dims.assign(ops[root_value].dim, ops[root_value].dim + an.root_rank);

  Builder b(an, err);
  // every reduction must run over the same axis of the same iteration space
  for (int i = 0; i < n_ops; ++i) {
    if (!is_reduce(ops[i].opcode) || side[i] == 2) continue;
    const disc_op& src = ops[ops[i].in[0]];
    if (!b.shapes_match_root(src)) {
      snprintf(buf, sizeof buf, "op %d (%s) and op %d (%s): the reduced tensors cannot be proved to have "
               "the same shape", first_reduce, opcode_name(ops[first_reduce].opcode), i, opcode_name(ops[i].opcode));
      err = buf;
      return DISC_ERR_UNFUSIBLE;
    }
    if (ops[i].axis_map[0] != an.reduce_axis && !side[i]) {
      snprintf(buf, sizeof buf, "op %d and op %d reduce over different axes (%d vs %d)", first_reduce, i,
               an.reduce_axis, ops[i].axis_map[0]);
      err = buf;
      return DISC_ERR_UNFUSIBLE;
    }
  }

  // "natural" context of values that are not full-shaped: defined through reductions
  std::vector<Ctx> nat(n_ops);
  std::vector<char> has_nat(n_ops, 0);
  Ctx ident(an.root_rank);
  for (int k = 0; k < an.root_rank; ++k) ident[k] = k;
  for (int i = 0; i < n_ops; ++i) {
    const disc_op& op = ops[i];
    if (op.rank > 0 && b.shapes_match_root(op)) { nat[i] = ident; has_nat[i] = 1; continue; }
    if (is_reduce(op.opcode)) {
      const int ax = side[i] ? op.axis_map[0] : an.reduce_axis;
      if (side[i] != 2)
        for (int k = 0; k < an.root_rank; ++k) if (k != ax) nat[i].push_back(k);
      has_nat[i] = 1;
    } else if (is_elementwise(op.opcode) || op.opcode == DISC_OUTPUT) {
      for (int k = 0; k < n_operands(op.opcode); ++k) {
        int s = op.in[k];
        if (ops[s].rank == op.rank && has_nat[s]) { nat[i] = nat[s]; has_nat[i] = 1; break; }
      }
    }
  }

  // flat loop fusion: outputs agree only in element count (tensor-size equality)
  if (an.reduce_axis < 0) {
    bool all_match = true, all_numel = true;
    for (int i = 0; i < n_ops; ++i) {
      if (ops[i].opcode != DISC_OUTPUT) continue;
      if (!b.shapes_match_root(ops[i])) all_match = false;
      if (nfind(i) != nfind(root_value)) all_numel = false;
    }
    if (!all_match) {
      if (!all_numel) {
        int o1 = -1, o2 = -1;
        for (int i = 0; i < n_ops; ++i)
          if (ops[i].opcode == DISC_OUTPUT) { if (o1 < 0) o1 = i; else if (!b.shapes_match_root(ops[i]) && o2 < 0) o2 = i; }
        snprintf(buf, sizeof buf, "op %d (output) and op %d (output): neither equal shapes nor equal element "
                 "counts can be proved; add a DIM_EQ or NUMEL_EQ constraint or register two patterns", o1, o2);
        err = buf;
        return DISC_ERR_UNFUSIBLE;
      }
      an.flat = true;
    }
  }

  // ---- 4. contexts ---------------------------------------------------------------------
  if (an.flat) {
    // Every tensor is walked with one linear index: legal only when each operand is a full
    // (non-broadcast) tensor of the common element count or a scalar.
    for (int i = 0; i < n_ops; ++i) {
      const disc_op& op = ops[i];
      if (op.opcode == DISC_BROADCAST || op.opcode == DISC_SLICE || op.opcode == DISC_PAD || op.opcode == DISC_TRANSPOSE) {
        snprintf(buf, sizeof buf, "op %d (%s): outputs agree only in element count, so the pattern is "
                 "fused over a flat index and cannot contain a broadcast, a slice, a pad or a transpose", i, opcode_name(op.opcode));
        err = buf;
        return DISC_ERR_UNFUSIBLE;
      }
      if (op.rank > 0 && nfind(i) != nfind(root_value)) {
        snprintf(buf, sizeof buf, "op %d (%s): element count cannot be proved equal to that of op %d", i,
                 opcode_name(op.opcode), root_value);
        err = buf;
        return DISC_ERR_UNFUSIBLE;
      }
      // the proof may rest on a caller's tensor-size equality: the host-side shape calculation
      // carries it (Section 4.2.1) and refuses a launch whose dims contradict it
      if ((op.opcode == DISC_PARAM || op.opcode == DISC_OUTPUT) && op.rank > 0 && numel_key(op) != numel_key(ops[root_value])) {
        DimProduct prod;
        for (int k = 0; k < op.rank; ++k) mul_into(prod, dc, op.dim[k]);
        an.numel_checks.push_back({i, prod});
      }
    }
  }
  for (int i = 0; i < n_ops; ++i) {
    if (ops[i].opcode != DISC_OUTPUT) continue;
    Ctx c;
    if (an.flat) {
      c.assign(ops[i].rank, 0);   // placeholder, flat accesses ignore contexts
    } else if (b.shapes_match_root(ops[i])) {
      c = ident;
    } else if (has_nat[i]) {
      c = nat[i];
    } else {
      snprintf(buf, sizeof buf, "op %d (output): its shape is neither the iteration space of the pattern nor "
               "derived from a reduction over it", i);
      err = buf;
      return DISC_ERR_UNFUSIBLE;
    }
    OutputRef o;
    Access a;
    if (side[ops[i].in[0]] == 2) {
      // a reduction of per-row values over the rows: the node is the per-row value
      const disc_op& src = ops[ops[ops[i].in[0]].in[0]];
      int rows_axis = -1;
      for (int k = 0; k < an.root_rank; ++k)
        if (k != an.reduce_axis && !b.dim_is_one(an.root_dims[k])) rows_axis = k;
      Ctx sc(src.rank, -1);
      for (int k = 0; k < src.rank; ++k)
        if (!b.dim_is_one(src.dim[k])) sc[k] = rows_axis;
      o.row_red = a.row_red = true;
      o.red_opcode = ops[ops[i].in[0]].opcode;
      o.node = b.demand(ops[ops[i].in[0]].in[0], sc);
      ++an.n_row_reds;
    } else if (side[ops[i].in[0]]) {
      // a sum over the rows: the node is the value summed, seen over the whole iteration space
      o.col_sum = a.col_sum = true;
      o.node = b.demand(ops[ops[i].in[0]].in[0], ident);
      ++an.n_col_sums;
    } else {
      o.node = b.demand(i, c);
    }
    if (o.node < 0) return b.status;
    a.value = i;
    a.is_output = true;
    a.dtype = ops[i].dtype;
    a.ctx = b.normalise(ops[i], c);
    a.slot = (int)an.outputs.size();
    o.access = (int)an.accesses.size();
    an.accesses.push_back(a);
    an.outputs.push_back(o);
  }
  if (b.status != DISC_OK) return b.status;
  if (an.n_col_sums > 4 || an.n_row_reds > 4) {
    // (registers per lane for the column sums, LDS of the last launch for the rank-0 results)
    err = "more than four reductions over the rows of one kind in a row-reduce pattern";
    return DISC_ERR_UNFUSIBLE;
  }

  // ---- 5. collapse root axes with identical roles ------------------------------------------
  an.groups.clear();
  if (an.flat) {
    an.root_rank = ops[root_value].rank;
    std::vector<int> g;
    for (int k = 0; k < an.root_rank; ++k) g.push_back(k);
    an.groups.push_back(g);
    for (auto& a : an.accesses) {
      a.ctx.assign(ops[a.value].rank, 0);
      a.groups = {0};
    }
  } else {
    auto mergeable = [&](int i) {   // may root axes i and i+1 form one group?
      if (i == an.reduce_axis || i + 1 == an.reduce_axis) return false;
      for (const auto& a : an.accesses) {
        int pi = -1, pj = -1;
        for (int k = 0; k < (int)a.ctx.size(); ++k) {
          if (a.ctx[k] == i) pi = k;
          if (a.ctx[k] == i + 1) pj = k;
        }
        if (pi < 0 && pj < 0) continue;
        if (pi < 0 || pj < 0) return false;
        // both present: must be adjacent in the operand too (axes of size 1 in between are fine)
        for (int k = pi + 1; k < pj; ++k)
          if (a.ctx[k] != -1) return false;
      }
      return true;
    };
    // root axes of static size 1 carry no index: drop them from the iteration space
    std::vector<int> live;
    for (int k = 0; k < an.root_rank; ++k)
      if (!b.dim_is_one(an.root_dims[k]) || k == an.reduce_axis) live.push_back(k);
    if (live.empty()) live.push_back(an.root_rank - 1);
    std::vector<int> cur;
    for (size_t t = 0; t < live.size(); ++t) {
      cur.push_back(live[t]);
      bool join = false;
      if (t + 1 < live.size()) {
        // axes between live[t] and live[t+1] are unit axes; merge only direct neighbours in the live list
        join = true;
        int i = live[t], j = live[t + 1];
        if (i == an.reduce_axis || j == an.reduce_axis) join = false;
        if (join) {
          for (const auto& a : an.accesses) {
            int pi = -1, pj = -1;
            for (int k = 0; k < (int)a.ctx.size(); ++k) {
              if (a.ctx[k] == i) pi = k;
              if (a.ctx[k] == j) pj = k;
            }
            if (pi < 0 && pj < 0) continue;
            if (pi < 0 || pj < 0 || pj < pi) { join = false; break; }   // (pj < pi: a transposed operand)
            for (int k = pi + 1; k < pj; ++k)
              if (a.ctx[k] != -1) { join = false; break; }
            // a sliced operand is contiguous across the two axes only if the inner one is whole
            if (a.src_value >= 0)
              for (int k = pi + 1; k <= pj; ++k)
                if (!b.slice_axis_full(ops[a.value], k)) { join = false; break; }
            if (!join) break;
          }
        }
      }
      if (!join) {
        an.groups.push_back(cur);
        cur.clear();
      }
    }
    (void)mergeable;
    // group membership of every access
    for (auto& a : an.accesses) {
      a.groups.clear();
      for (int g = 0; g < (int)an.groups.size(); ++g) {
        bool has = false;
        for (int ax : an.groups[g])
          for (int c : a.ctx) if (c == ax) has = true;
        if (has) a.groups.push_back(g);
      }
    }
  }
  const int ng = (int)an.groups.size();
  if (an.reduce_axis >= 0) {
    int rg = -1;
    for (int g = 0; g < ng; ++g)
      for (int ax : an.groups[g]) if (ax == an.reduce_axis) rg = g;
    if (rg == ng - 1) {
      an.tmpl = DISC_TEMPLATE_ROW_REDUCE;
      an.inner_group = ng - 1;
    } else {
      an.tmpl = DISC_TEMPLATE_COL_REDUCE;
      an.mid_group = rg;
      an.inner_group = ng - 1;
      if (rg + 2 != ng) {
        err = "column reduction: the axes after the reduced one do not collapse into one contiguous group";
        return DISC_ERR_UNFUSIBLE;
      }
      if (rg > 1) {
        err = "column reduction: the axes before the reduced one do not collapse into one group";
        return DISC_ERR_UNFUSIBLE;
      }
    }
  } else {
    an.tmpl = DISC_TEMPLATE_LOOP;
    an.inner_group = ng - 1;
  }
  if (ng > 4) { err = "iteration space does not collapse to <= 4 groups"; return DISC_ERR_UNFUSIBLE; }

  // ---- 6. domains and phases --------------------------------------------------------------
  auto ctx_has_group = [&](const Ctx& c, int g) {
    for (int ax : an.groups[g]) for (int x : c) if (x == ax) return true;
    return false;
  };
  int max_phase = 0;
  for (auto& n : an.nodes) {
    if (n.opcode == DISC_CONST || n.opcode == DISC_DIM_SIZE) {
      n.dom = DOM_SCALAR;
      n.phase = 0;
      continue;
    }
    if (an.flat) {
      n.dom = DOM_ELEM;
    } else if (an.tmpl == DISC_TEMPLATE_COL_REDUCE) {
      // "row" domain of a column reduction = values without the reduced (mid) axis
      n.dom = ctx_has_group(n.ctx, an.mid_group) ? DOM_ELEM : DOM_ROW;
    } else {
      n.dom = ctx_has_group(n.ctx, an.inner_group) ? DOM_ELEM : DOM_ROW;
    }
    int ph = 0;
    for (int k = 0; k < n.n_in; ++k) ph = std::max(ph, an.nodes[n.in[k]].phase);
    if (is_reduce(n.opcode)) {
      n.reduce_slot = (int)an.reduces[ph].size();
      if (ph >= 7) { err = "too many dependent reduction levels"; return DISC_ERR_UNFUSIBLE; }
      an.reduces[ph].push_back((int)(&n - &an.nodes[0]));
      n.phase = ph + 1;
      n.dom = DOM_ROW;
    } else {
      n.phase = ph;
    }
    max_phase = std::max(max_phase, n.phase);
  }
  an.n_phases = max_phase;
  if (an.tmpl == DISC_TEMPLATE_COL_REDUCE && an.n_phases > 1) {
    err = "column reduction feeding another reduction: needs a second pass over the tensor, not one fusion";
    return DISC_ERR_UNFUSIBLE;
  }

  // ---- 7. access kinds and shape-calculation recipes ---------------------------------------
  an.group_size.assign(ng, DimProduct());
  for (int g = 0; g < ng; ++g)
    for (int ax : an.groups[g]) mul_into(an.group_size[g], dc, an.root_dims[ax]);
  const int n_outer = an.inner_group;   // groups before the inner one
  an.needs_decomp = false;
  for (auto& a : an.accesses) {
    a.has_inner = !a.groups.empty() && a.groups.back() == an.inner_group;
    int outer_cnt = (int)a.groups.size() - (a.has_inner ? 1 : 0);
    if (outer_cnt == n_outer) a.kind = a.has_inner ? ACC_FULL : (n_outer == 0 ? ACC_SCALAR : ACC_PERROW);
    else if (outer_cnt == 0) a.kind = a.has_inner ? ACC_ROWVEC : ACC_SCALAR;
    else a.kind = ACC_PARTIAL;
    if (a.src_value >= 0) {
      // sliced / padded PARAM: strided like a partial access, with the PARAM's own extents as strides
      const disc_op& sl = ops[a.value];
      const disc_op& src = ops[a.src_value];
      a.all_outer = outer_cnt == n_outer && a.has_inner;
      a.kind = ACC_PARTIAL;
      an.needs_decomp = true;
      if (a.padded && !a.has_inner) {
        snprintf(buf, sizeof buf, "op %d (pad): a padded operand without the innermost axis is not supported", a.value);
        err = buf;
        return DISC_ERR_UNFUSIBLE;
      }
      auto tail_product = [&](int after) {       // product of the operand's extents of the axes behind `after`
        DimProduct p;
        for (int k = after + 1; k < src.rank; ++k) mul_into(p, dc, src.dim[k]);
        return p;
      };
      for (size_t t = 0; t < a.groups.size(); ++t) {
        int first = DISC_MAX_RANK, last = -1;
        for (int k = 0; k < (int)a.ctx.size(); ++k)
          for (int ax : an.groups[a.groups[t]])
            if (a.ctx[k] == ax) { last = std::max(last, k); first = std::min(first, k); }
        // the operand is only present inside a window of this group's index when the group's
        // outermost axis is padded (the axes behind it in the group are whole, or they would
        // not have been merged with it)
        int win = -1;
        if (a.padded && last >= 0 && !b.slice_axis_full(sl, first)) {
          WindowRecipe w;
          w.low = sl.axis_map[first];
          w.extent_dim = src.dim[first];
          for (int k = first + 1; k <= last; ++k) mul_into(w.inner_sizes, dc, src.dim[k]);
          win = (int)an.windows.size();
          an.windows.push_back(w);
        }
        a.window.push_back(win);
        if (a.groups[t] == an.inner_group) {
          // rows must stay contiguous in the operand: nothing but unit axes behind the inner group
          for (int k = last + 1; k < src.rank; ++k)
            if (!b.dim_is_one(src.dim[k])) {
              snprintf(buf, sizeof buf, "op %d (%s): the operand's innermost axis is not the innermost axis of the "
                       "iteration space; a transpose that moves it needs a tile transpose and is not fused", a.value,
                       opcode_name(sl.opcode));
              err = buf;
              return DISC_ERR_UNFUSIBLE;
            }
          continue;
        }
        a.stride_prod.push_back((int)an.products.size());
        an.products.push_back(tail_product(last));
      }
      OffsetRecipe off;
      off.negative = a.padded;
      for (int k = 0; k < sl.rank && sl.opcode != DISC_TRANSPOSE; ++k) {
        if (sl.axis_map[k] != -1) off.terms.push_back({sl.axis_map[k], tail_product(k)});
        if (!b.slice_axis_full(sl, k)) {
          if (a.padded && b.dim_is_one(sl.dim[k])) {
            snprintf(buf, sizeof buf, "op %d (pad): axis %d has result size 1 and cannot be padded", a.value, k);
            err = buf;
            return DISC_ERR_BAD_PATTERN;
          }
          SliceCheck sc;
          sc.start = sl.axis_map[k];
          // slice: start + result size <= operand extent; pad: low + operand extent <= result size
          sc.size_dim = a.padded ? src.dim[k] : sl.dim[k];
          sc.src_dim = a.padded ? sl.dim[k] : src.dim[k];
          sc.op = a.value;
          sc.axis = k;
          an.slice_checks.push_back(sc);
        }
      }
      if (!off.terms.empty()) {
        a.offset_index = (int)an.offsets.size();
        an.offsets.push_back(off);
      }
      continue;
    }
    if (a.kind == ACC_PARTIAL) {
      an.needs_decomp = true;
      // stride of spanned outer group g = product of the later groups this access spans
      for (size_t t = 0; t < a.groups.size(); ++t) {
        if (a.groups[t] == an.inner_group) continue;
        DimProduct p;
        for (size_t u = t + 1; u < a.groups.size(); ++u) {
          const DimProduct& gs = an.group_size[a.groups[u]];
          p.sym.insert(p.sym.end(), gs.sym.begin(), gs.sym.end());
          p.stat *= gs.stat;
        }
        a.stride_prod.push_back((int)an.products.size());
        an.products.push_back(p);
      }
    }
  }
  for (auto& n : an.nodes)
    if (n.opcode == DISC_DIM_SIZE &&
        std::find(an.dim_size_syms.begin(), an.dim_size_syms.end(), n.sym_dim) == an.dim_size_syms.end())
      an.dim_size_syms.push_back(n.sym_dim);

  // vector width: 16 bytes of the narrowest per-element tensor, at most 8 elements
  int min_bytes = 8;
  bool any = false;
  for (const auto& a : an.accesses) {
    if (!a.has_inner) continue;
    if (a.dtype == DISC_BOOL) continue;      // masks ride along at whatever width the data needs
    min_bytes = std::min(min_bytes, dtype_bytes(a.dtype));
    any = true;
  }
  if (!any) min_bytes = 2;
  an.vec_width = std::min(8, 16 / min_bytes);
  return DISC_OK;
}

int analyze(const disc_op* ops, int n_ops, const disc_constraint* cs, int n_cs, Analysis* out,
            std::string* errp) {
  bool used = false;
  int rc = analyze_impl(ops, n_ops, cs, n_cs, out, errp, true, &used);
  if (rc != DISC_OK && used) {
    // the pattern is not a loop fusion with sums riding along after all: judge it as before
    *out = Analysis();
    errp->clear();
    rc = analyze_impl(ops, n_ops, cs, n_cs, out, errp, false, &used);
  }
  return rc;
}

}  // namespace disc

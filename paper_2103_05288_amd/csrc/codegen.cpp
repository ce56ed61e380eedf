// Device-code generation: turns the resolved node graph of a pattern into ONE `struct Pat`
// (the fused per-element expression, operand addressing and reduction bookkeeping) that the
// hand-written schedules of disc_device.h are instantiated with.  All kernel versions of a
// pattern come out of this one translation unit, so a pattern costs exactly one device
// compile whatever shapes it later runs at (Section 2 / Section 4.3 of the paper).
//
// Decisions taken here, per pattern and independent of any shape value:
//  * which operands stream from HBM and are loaded up front into the slot (tensors that span
//    the whole iteration space) and which are small, cached operands loaded where they are
//    used (row vectors, row-group operands): keeps registers free across reduction phases;
//  * which intermediate values are carried in registers from one reduction phase to the next
//    and which are recomputed from the raw slot (a cast or one add is cheaper than 8 registers);
//  * division by a per-row value becomes a multiplication by a reciprocal computed once per row;
//    per-element transcendental ops use the hardware approximations (1 ulp exp2 / log2 / rcp /
//    rsq); so do per-row reciprocals and roots; per-row exp / log / tanh and per-column math stay
//    IEEE-correct.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <functional>
#include <map>
#include <set>
#include <sstream>

#include "disc_internal.hpp"

namespace disc {
namespace {

std::string fmt(const char* f, ...) __attribute__((format(printf, 1, 2)));
std::string fmt(const char* f, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, f);
  vsnprintf(buf, sizeof buf, f, ap);
  va_end(ap);
  return buf;
}

std::string float_lit(double v) {
  float f = (float)v;
  if (std::isnan(f)) return "__builtin_nanf(\"\")";
  if (std::isinf(f)) return f > 0 ? "__builtin_inff()" : "(-__builtin_inff())";
  char buf[64];
  snprintf(buf, sizeof buf, "%.9gf", (double)f);
  std::string s = buf;
  if (s.find('.') == std::string::npos && s.find('e') == std::string::npos) s.insert(s.size() - 1, ".0");
  if (std::signbit(f)) s = "(" + s + ")";   // a literal that starts with '-' must survive a prefix operator
  return s;
}

bool heavy_op(int oc) {
  switch (oc) {
    case DISC_EXP: case DISC_LOG: case DISC_TANH: case DISC_SQRT: case DISC_RSQRT: case DISC_RCP:
    case DISC_SIGMOID: case DISC_ERF: case DISC_DIV: case DISC_POW: return true;
    default: return false;
  }
}

struct Gen {
  const Analysis& an;
  ArgLayout layout;
  std::ostringstream os;
  int acc_bytes = 8;
  int n_acc_cells = 0;
  // row template: values carried in registers across phases, and the function that makes them
  std::set<int> keep_nodes;
  std::map<int, int> produced_phase;
  std::set<int> need_rinv;     // per-row values whose reciprocal is precomputed
  std::set<int> need_nl2e;     // per-row values r for which -r*log2(e) is precomputed (exp(x - r))
  const GenOptions* opt = nullptr;
  std::set<int> read_on;       // ops whose value something other than an OUTPUT reads
  explicit Gen(const Analysis& a) : an(a) {
    for (const auto& op : an.ops)
      if (op.opcode != DISC_OUTPUT)
        for (int k = 0; k < operand_count(op.opcode); ++k) read_on.insert(op.in[k]);
  }

  static bool is_reduce(int oc) { return oc >= DISC_REDUCE_SUM && oc <= DISC_REDUCE_ARGMAX; }
  bool col_tmpl() const { return an.tmpl == DISC_TEMPLATE_COL_REDUCE; }
  bool row_tmpl() const { return an.tmpl == DISC_TEMPLATE_ROW_REDUCE; }
  bool compact_tmpl() const { return an.tmpl == DISC_TEMPLATE_COMPACT; }
  // small cached operands of a row reduce are loaded at their point of use, not into the slot
  bool late(const Access& a) const { return row_tmpl() && !a.is_output && a.has_inner && a.kind != ACC_FULL && !a.all_outer; }

  // ---- kernel-argument block ------------------------------------------------------------
  void add_field(ArgField::Kind k, int index, int size) {
    ArgField f;
    f.kind = k;
    f.index = index;
    f.size = size;
    f.offset = layout.size;
    layout.size += size;
    layout.fields.push_back(f);
  }
  void build_layout() {
    add_field(ArgField::ROWS, 0, 8);
    add_field(ArgField::INNER, 0, 8);
    add_field(ArgField::NSLOTS, 0, 8);
    add_field(ArgField::SPR, 0, 8);
    add_field(ArgField::MID, 0, 8);
    for (int g = 0; g < 3; ++g) add_field(ArgField::GROUP_SIZE, g, 8);
    for (int i = 0; i < an.n_inputs; ++i) add_field(ArgField::IN_PTR, i, 8);
    for (int i = 0; i < an.n_outputs; ++i) add_field(ArgField::OUT_PTR, i, 8);
    for (int i = 0; i < 2; ++i) add_field(ArgField::WS_PTR, i, 8);
    for (int i = 0; i < 4; ++i) add_field(ArgField::AUX, i, 8);
    // strides, then base offsets of sliced / padded operands, then [lo, hi) of every padding window
    for (size_t i = 0; i < an.products.size() + an.offsets.size() + 2 * an.windows.size(); ++i) add_field(ArgField::STRIDE, (int)i, 8);
    for (size_t i = 0; i < an.dim_size_syms.size(); ++i) add_field(ArgField::DIMI, (int)i, 8);
    add_field(ArgField::SPR_DIV, 0, 16);
    for (int g = 0; g < 3; ++g) add_field(ArgField::GROUP_DIV, g, 16);
    for (size_t i = 0; i < an.dim_size_syms.size(); ++i) add_field(ArgField::DIMF, (int)i, 4);
    if (layout.size % 8) layout.size += 8 - layout.size % 8;
  }
  int io_dtype(int opcode, int index) const {
    int k = 0;
    for (const auto& op : an.ops)
      if (op.opcode == opcode && k++ == index) return op.dtype;
    return DISC_F32;
  }
  std::string field_name(const ArgField& f) const {
    switch (f.kind) {
      case ArgField::ROWS: return "rows";
      case ArgField::INNER: return "inner";
      case ArgField::NSLOTS: return "nslots";
      case ArgField::SPR: return "spr";
      case ArgField::MID: return "mid";
      case ArgField::GROUP_SIZE: return fmt("gs%d", f.index);
      case ArgField::IN_PTR: return fmt("p%d", f.index);
      case ArgField::OUT_PTR: return fmt("o%d", f.index);
      case ArgField::WS_PTR: return fmt("ws%d", f.index);
      case ArgField::AUX: return fmt("aux%d", f.index);
      case ArgField::STRIDE: return fmt("st%d", f.index);
      case ArgField::DIMI: return fmt("dimi%d", f.index);
      case ArgField::SPR_DIV: return "spr_div";
      case ArgField::GROUP_DIV: return fmt("gd%d", f.index);
      case ArgField::DIMF: return fmt("dimf%d", f.index);
    }
    return "";
  }
  std::string field_decl(const ArgField& f) const {
    const std::string n = field_name(f);
    switch (f.kind) {
      case ArgField::IN_PTR: return fmt("const %s* __restrict__ %s;", dtype_ctype(io_dtype(DISC_PARAM, f.index)), n.c_str());
      case ArgField::OUT_PTR: return fmt("%s* __restrict__ %s;", dtype_ctype(io_dtype(DISC_OUTPUT, f.index)), n.c_str());
      case ArgField::WS_PTR: return "void* " + n + ";";
      case ArgField::SPR_DIV: case ArgField::GROUP_DIV: return "disc::FastDiv " + n + ";";
      case ArgField::DIMF: return "float " + n + ";";
      default: return "disc::i64 " + n + ";";
    }
  }

  // ---- conversions -------------------------------------------------------------------------
  int dim_index(int sym) const {
    for (size_t i = 0; i < an.dim_size_syms.size(); ++i)
      if (an.dim_size_syms[i] == sym) return (int)i;
    return 0;
  }
  static std::string convert(const std::string& x, RegKind from, RegKind to) {
    if (from == to) return x;
    switch (to) {
      case RK_F32: return from == RK_BOOL ? "(" + x + " ? 1.0f : 0.0f)" : "(float)(" + x + ")";
      case RK_I32: return from == RK_BOOL ? "(" + x + " ? 1 : 0)" : "(int)(" + x + ")";
      case RK_I64: return from == RK_BOOL ? "(" + x + " ? 1LL : 0LL)" : "(disc::i64)(" + x + ")";
      default: return "((" + x + ") != 0)";
    }
  }
  static std::string from_storage(const std::string& x, int dtype) {
    switch (reg_kind(dtype)) {
      case RK_F32: return "disc::to_f32(" + x + ")";
      case RK_I32: return "(int)(" + x + ")";
      case RK_I64: return "(disc::i64)(" + x + ")";
      default: return "((" + x + ") != 0)";
    }
  }
  static std::string to_storage(const std::string& x, RegKind rk, int dtype) {
    if (is_float_dtype(dtype)) return fmt("disc::from_f32<%s>(%s)", dtype_ctype(dtype), convert(x, rk, RK_F32).c_str());
    if (dtype == DISC_BOOL) return "(disc::u8)(" + convert(x, rk, RK_BOOL) + " ? 1 : 0)";
    return fmt("(%s)(%s)", dtype_ctype(dtype), x.c_str());
  }

  // accumulator field names of reduce `slot` in a phase
  static std::string accf(int slot) { return fmt("f%d", slot); }
  static std::string acci(int slot) { return fmt("i%d", slot); }
  // accumulator C type of a reduction: long column sums of fp32 data run in fp64 (values near
  // zero must still meet the absolute part of the fp32 tolerance after cancellation)
  std::string acc_ctype(const Node& n) const {
    RegKind ok = an.nodes[n.in[0]].rk;
    if (col_tmpl() && n.opcode == DISC_REDUCE_SUM && ok == RK_F32) return "double";
    return reg_ctype(ok);
  }
  // reduce result as a register value of the node's kind, read from accumulator `acc`
  std::string acc_value(const Node& n, const std::string& acc) const {
    RegKind ok = an.nodes[n.in[0]].rk;
    if (n.opcode == DISC_REDUCE_ARGMAX) return convert(acc + "." + acci(n.reduce_slot), RK_I32, n.rk);
    std::string f = acc + "." + accf(n.reduce_slot);
    if (acc_ctype(n) == "double") f = "(float)" + f;
    return convert(f, ok, n.rk);
  }

  // Where a piece of generated code runs; decides where each kind of value is read from.
  enum Mode {
    M_ELEM,        // row / loop templates, per element: slot `s`, element `e`, per-row values in `rc`
    M_ROWLOCAL,    // row / loop templates, per row: row_begin / row_after compute per-row values
    M_COL_ACCUM,   // column reduce stage 1, per element: values without the reduced axis are inlined
    M_COL_FINISH,  // column reduce stage 2, per (outer, column): scalars `o`, `c`, accumulator `acc`
    M_COL_EPI      // column reduce stage 3, per element: reduce results arrive in the slot
  };

  // Emits straight-line code computing nodes inside one device function.
  struct Fn {
    Gen& g;
    std::ostringstream body;
    std::map<int, std::string> names;
    Mode mode;
    int P = 0;            // M_ELEM: index of the phase function being emitted (n_phases = epilogue)
    bool keep = false;    // M_ELEM: values may be read from / written to the Keep registers
    std::set<int> late_used;
    Fn(Gen& gg, Mode m) : g(gg), mode(m) {}
    bool fast() const { return mode == M_ELEM || mode == M_COL_ACCUM || mode == M_COL_EPI; }

    std::string val(int id) {
      auto it = names.find(id);
      if (it != names.end()) return it->second;
      const Node& n = g.an.nodes[id];
      std::string r;
      const bool col = mode == M_COL_ACCUM || mode == M_COL_FINISH || mode == M_COL_EPI;
      if (n.opcode == DISC_CONST) {
        if (n.rk == RK_F32) r = float_lit(n.fconst);
        else if (n.rk == RK_BOOL) r = n.fconst != 0 ? "true" : "false";
        else r = fmt("(%lld%s)", (long long)n.fconst, n.rk == RK_I64 ? "LL" : "");
      } else if (n.opcode == DISC_DIM_SIZE) {
        if (n.rk == RK_F32) r = fmt("A.dimf%d", g.dim_index(n.sym_dim));
        else r = fmt("(%s)A.dimi%d", reg_ctype(n.rk), g.dim_index(n.sym_dim));
      } else if (n.opcode == DISC_PARAM) {
        const Access& a = g.an.accesses[n.access];
        if (mode == M_COL_FINISH) {
          // a scalar load at (outer index o, column c); the operand has no reduced axis here
          std::string off = a.has_inner ? (a.groups.size() > 1 ? "o * A.inner + c" : "c")
                                        : (a.groups.empty() ? "0" : "o");
          r = from_storage(fmt("A.p%d[%s]", a.slot, off.c_str()), a.dtype);
        } else if (a.has_inner) {
          if (g.late(a)) {
            late_used.insert(n.access);
            r = from_storage(fmt("l%d.get(e)", n.access), a.dtype);
          } else {
            r = from_storage(fmt("s.a%d.get(e)", n.access), a.dtype);
          }
        } else {
          r = fmt("rc.r%d", id);   // loaded by row_begin
        }
      } else if (is_reduce(n.opcode)) {
        if (mode == M_COL_FINISH) r = g.acc_value(n, "acc");
        else if (mode == M_COL_EPI) r = fmt("s.red%d.get(e)", n.reduce_slot);
        else r = fmt("rc.r%d", id);
      } else if (!col && n.dom == DOM_ROW && mode == M_ELEM) {
        r = fmt("rc.r%d", id);
      } else if (mode == M_ELEM && keep && g.keep_nodes.count(id) && g.produced_phase[id] < P) {
        r = fmt("k.k%d[e]", id);
      } else {
        r = fmt("t%d", id);
        const std::string rhs = expr(n);   // emits the operands first
        body << "        const " << reg_ctype(n.rk) << " " << r << " = " << rhs << ";\n";
        if (mode == M_ELEM && keep && g.keep_nodes.count(id) && g.produced_phase[id] == P)
          body << "        k.k" << id << "[e] = " << r << ";\n";
      }
      names[id] = r;
      return r;
    }
    std::string as(int id, RegKind k) { return convert(val(id), g.an.nodes[id].rk, k); }
    static std::string wrap_arith(RegKind k, const std::string& x, const char* op, const std::string& y) {
      const char* u = k == RK_I64 ? "disc::u64" : "disc::u32";
      return fmt("(%s)((%s)(%s) %s (%s)(%s))", reg_ctype(k), u, x.c_str(), op, u, y.c_str());
    }
    std::string expr(const Node& n) {
      const RegKind k = n.rk;
      auto a = [&](int i) { return as(n.in[i], k); };
      const bool f = fast();
      switch (n.opcode) {
        case DISC_NEG: return k == RK_F32 ? "-(" + a(0) + ")" : wrap_arith(k, "0", "-", a(0));
        case DISC_ABS: return k == RK_F32 ? "fabsf(" + a(0) + ")" : "((" + a(0) + ") < 0 ? " + wrap_arith(k, "0", "-", a(0)) + " : (" + a(0) + "))";
        case DISC_EXP: {
          // exp(x - r) with r a per-row value: exp2(fma(x, log2e, -r*log2e)), the product with r
          // is made once per row
          const Node& s0 = g.an.nodes[n.in[0]];
          if (f && mode == M_ELEM && s0.opcode == DISC_SUB && s0.rk == RK_F32 && g.need_nl2e.count(s0.in[1]))
            return "disc::fast_exp2(__builtin_fmaf(" + as(s0.in[0], RK_F32) + ", 1.44269504088896341f, " + fmt("rc.n%d", s0.in[1]) + "))";
          return (f ? "disc::fast_exp(" : "expf(") + a(0) + ")";
        }
        case DISC_LOG: return (f ? "disc::fast_log(" : "logf(") + a(0) + ")";
        case DISC_TANH: return (f ? "disc::fast_tanh(" : "tanhf(") + a(0) + ")";
        // square roots and reciprocals use the approximation units per row as well (1 ulp: far inside
        // the fp32 bar): the IEEE expansions cost 6-10 instructions each, per row and lane, and a
        // lane of a long row only has 16-24 elements to spread them over
        case DISC_SQRT: return (f || mode == M_ROWLOCAL ? "disc::fast_sqrt(" : "sqrtf(") + a(0) + ")";
        case DISC_RSQRT: return (f || mode == M_ROWLOCAL ? "disc::fast_rsqrt(" : "rsqrtf(") + a(0) + ")";
        case DISC_RCP: return f || mode == M_ROWLOCAL ? "disc::fast_rcp(" + a(0) + ")" : "(1.0f / " + a(0) + ")";
        case DISC_SIGMOID: return f ? "disc::fast_sigmoid(" + a(0) + ")" : "(1.0f / (1.0f + expf(-" + a(0) + ")))";
        case DISC_ERF: return "erff(" + a(0) + ")";
        // integers wrap (two's complement of the declared width): computed on the unsigned type
        case DISC_ADD: return k == RK_F32 ? a(0) + " + " + a(1) : wrap_arith(k, a(0), "+", a(1));
        case DISC_SUB: return k == RK_F32 ? a(0) + " - " + a(1) : wrap_arith(k, a(0), "-", a(1));
        case DISC_MUL: return k == RK_F32 ? a(0) + " * " + a(1) : wrap_arith(k, a(0), "*", a(1));
        case DISC_DIV: {
          if (k == RK_F32 && mode == M_ROWLOCAL) {
            // per-row quotients: by a launch-wide scalar (a dimension size) it is a product with the
            // reciprocal, which the compiler computes once per kernel; by a per-row value a product
            // with its approximate reciprocal
            const Node& dr = g.an.nodes[n.in[1]];
            if (dr.dom == DOM_SCALAR) return a(0) + " * (1.0f / " + a(1) + ")";
            return a(0) + " * disc::fast_rcp(" + a(1) + ")";
          }
          if (k != RK_F32 || !f) return a(0) + " / " + a(1);
          const Node& d = g.an.nodes[n.in[1]];
          if (mode == M_ELEM && g.need_rinv.count(n.in[1])) return a(0) + " * " + fmt("rc.q%d", n.in[1]);
          if (d.dom == DOM_SCALAR) return a(0) + " * (1.0f / " + a(1) + ")";
          return a(0) + " * disc::fast_rcp(" + a(1) + ")";
        }
        case DISC_MAX: return k == RK_F32 ? "fmaxf(" + a(0) + ", " + a(1) + ")" : "(" + a(0) + " > " + a(1) + " ? " + a(0) + " : " + a(1) + ")";
        case DISC_MIN: return k == RK_F32 ? "fminf(" + a(0) + ", " + a(1) + ")" : "(" + a(0) + " < " + a(1) + " ? " + a(0) + " : " + a(1) + ")";
        case DISC_POW: return "powf(" + a(0) + ", " + a(1) + ")";
        case DISC_LT: case DISC_LE: case DISC_GT: case DISC_GE: case DISC_EQ: case DISC_NE: {
          // compare in the wider kind of the two operands
          RegKind ka = g.an.nodes[n.in[0]].rk, kb = g.an.nodes[n.in[1]].rk;
          RegKind kc = (ka == RK_F32 || kb == RK_F32) ? RK_F32 : (ka == RK_I64 || kb == RK_I64) ? RK_I64 : RK_I32;
          static const char* sym[] = {"<", "<=", ">", ">=", "==", "!="};
          return as(n.in[0], kc) + " " + sym[n.opcode - DISC_LT] + " " + as(n.in[1], kc);
        }
        case DISC_NE_PREV: {
          // the first element of the tensor opens the first run; in[1] is the same operand read one
          // element earlier
          const RegKind kc = g.an.nodes[n.in[0]].rk;
          return "((disc::i64)col + e == 0) || (" + as(n.in[0], kc) + " != " + as(n.in[1], kc) + ")";
        }
        case DISC_SELECT: return as(n.in[0], RK_BOOL) + " ? " + a(1) + " : " + a(2);
        case DISC_CAST:
          // float -> int truncates toward zero in C.  A cast to a 16-bit float type whose value is
          // read by further ops rounds it to that type, as the unfused sequence would hand it on;
          // one that only feeds outputs is rounded by the store
          if ((n.dtype == DISC_F16 || n.dtype == DISC_BF16) && g.read_on.count(n.value))
            return fmt("disc::to_f32(disc::from_f32<%s>(%s))", dtype_ctype(n.dtype), a(0).c_str());
          return a(0);
        default: return "0 /* unexpected opcode */";
      }
    }
  };

  // ---- planning of cross-phase registers (row template) -----------------------------------------
  std::vector<int> phase_roots(int P) const {
    std::vector<int> r;
    if (P < an.n_phases) {
      for (int id : an.reduces[P]) r.push_back(an.nodes[id].in[0]);
    } else {
      for (const auto& out : an.outputs)
        if (elem_output(an.accesses[out.access]) || out.col_sum) r.push_back(out.node);
    }
    return r;
  }
  double recompute_cost(int id, int P, std::map<int, double>& memo) const {
    auto it = memo.find(id);
    if (it != memo.end()) return it->second;
    const Node& n = an.nodes[id];
    double c;
    if (n.dom != DOM_ELEM) c = 0;
    else if (n.opcode == DISC_PARAM) c = late(an.accesses[n.access]) ? 1e9 : 0;
    else if (keep_nodes.count(id) && produced_phase.at(id) < P) c = 0;
    else {
      c = heavy_op(n.opcode) ? 4 : 1;
      for (int k = 0; k < n.n_in; ++k) c += recompute_cost(n.in[k], P, memo);
    }
    memo[id] = c;
    return c;
  }
  void plan_keeps() {
    keep_nodes.clear();
    produced_phase.clear();
    if (!row_tmpl()) return;
    for (int P = 0; P <= an.n_phases; ++P) {
      std::set<int> seen;
      std::function<void(int)> visit = [&](int id) {
        const Node& n = an.nodes[id];
        if (n.dom != DOM_ELEM || n.opcode == DISC_PARAM || seen.count(id)) return;
        seen.insert(id);
        auto pp = produced_phase.find(id);
        if (pp != produced_phase.end() && pp->second < P) {
          std::map<int, double> memo;
          if (keep_nodes.count(id) || recompute_cost(id, P, memo) > 2.0) {
            keep_nodes.insert(id);
            return;
          }
        }
        if (pp == produced_phase.end()) produced_phase[id] = P;
        for (int k = 0; k < n.n_in; ++k) visit(n.in[k]);
      };
      for (int r : phase_roots(P)) visit(r);
    }
  }
  void plan_rinv() {
    need_rinv.clear();
    need_nl2e.clear();
    if (col_tmpl()) return;
    for (const Node& n : an.nodes)
      if (n.opcode == DISC_EXP && n.dom == DOM_ELEM) {
        const Node& s0 = an.nodes[n.in[0]];
        if (s0.opcode == DISC_SUB && s0.rk == RK_F32 && an.nodes[s0.in[1]].dom == DOM_ROW && an.nodes[s0.in[1]].rk == RK_F32)
          need_nl2e.insert(s0.in[1]);
      }
    for (const Node& n : an.nodes)
      if (n.opcode == DISC_DIV && n.rk == RK_F32 && n.dom == DOM_ELEM) {
        const Node& d = an.nodes[n.in[1]];
        if (d.dom == DOM_ROW && d.rk == RK_F32) need_rinv.insert(n.in[1]);
      }
  }

  // ---- per-row context -------------------------------------------------------------------------
  std::string row_fields() {
    std::ostringstream o;
    for (size_t i = 0; i < an.accesses.size(); ++i) {
      const Access& a = an.accesses[i];
      if (a.has_inner && a.kind == ACC_PARTIAL) o << "    disc::i64 b" << i << ";\n";
      if (has_outer_window(a)) o << "    bool v" << i << ";\n";
      if (!a.has_inner && a.is_output && a.kind == ACC_PARTIAL) o << "    disc::i64 b" << i << ";\n";
    }
    // full-size operands: element offset of the row = sb + lb.  sb is the offset of the first row
    // of the wavefront (uniform when the caller passes a uniform base row, so it lives in scalar
    // registers and the accesses use scalar base + 32-bit lane offset), lb the lane's share.
    o << "    disc::i64 sb;\n    int lb;\n    bool tail_ok;\n";
    for (size_t i = 0; i < an.nodes.size(); ++i) {
      const Node& n = an.nodes[i];
      const bool perrow_param = n.opcode == DISC_PARAM && !an.accesses[n.access].has_inner;
      if ((!col_tmpl() && n.dom == DOM_ROW) || perrow_param) o << "    " << reg_ctype(n.rk) << " r" << i << ";\n";
      if (need_rinv.count((int)i)) o << "    float q" << i << ";\n";
      if (need_nl2e.count((int)i)) o << "    float n" << i << ";\n";
    }
    if (col_tmpl()) o << "    disc::i64 ob;\n";   // offset of this row's outer slice in the reduce-result planes
    o << "    const char* sl;\n";                 // staged row vectors in LDS (row reduce), or null
    o << "    int unused_;\n";
    return o.str();
  }
  void assign_row(Fn& fn, size_t i, const std::string& v) {
    fn.body << "    rc.r" << i << " = " << v << ";\n";
    if (need_rinv.count((int)i)) fn.body << "    rc.q" << i << " = disc::fast_rcp(rc.r" << i << ");\n";
    if (need_nl2e.count((int)i)) fn.body << "    rc.n" << i << " = -1.44269504088896341f * rc.r" << i << ";\n";
    fn.names[(int)i] = fmt("rc.r%zu", i);
  }

  bool has_outer_window(const Access& a) const {
    if (!a.padded) return false;
    for (size_t t = 0; t < a.groups.size(); ++t)
      if (a.groups[t] != an.inner_group && a.window[t] >= 0) return true;
    return false;
  }
  int window_arg(int w) const { return (int)(an.products.size() + an.offsets.size()) + 2 * w; }
  // load of a slot of an operand; a padded one takes the padding value wherever the operand is not
  std::string load_call(const Access& a, size_t i, const std::string& dst, const std::string& ld_tmpl, const std::string& extra) {
    const std::string ptr = elem_ptr(a, fmt("A.p%d", a.slot));
    if (a.prev) return "disc::ld_prev(" + dst + ", " + ptr + ", (disc::i64)" + elem_base(a, i) + ", sp);";
    if (!a.padded) return "disc::ld" + ld_tmpl + "(" + dst + ", " + ptr + ", " + elem_base(a, i) + ", sp" + extra + ");";
    std::string lo = "0", hi = "0x7fffffffffffffffLL";
    for (size_t t = 0; t < a.groups.size(); ++t)
      if (a.groups[t] == an.inner_group && a.window[t] >= 0) {
        lo = fmt("A.st%d", window_arg(a.window[t]));
        hi = fmt("A.st%d", window_arg(a.window[t]) + 1);
      }
    const std::string ok = has_outer_window(a) ? fmt("rc.v%zu", i) : std::string("true");
    return "disc::ld_win(" + dst + ", " + ptr + ", " + elem_base(a, i) + ", sp, (disc::i64)col, " + ok + ", " + lo + ", " + hi +
           ", disc::pad_const<" + dtype_ctype(a.dtype) + ">(" + float_lit(a.pad_value) + "));";
  }

  // offset expression of an access without the inner group, for row `row`
  std::string perrow_offset(const Access& a, size_t idx) {
    switch (a.kind) {
      case ACC_PERROW: return "row";
      case ACC_SCALAR: return "0";
      default: return fmt("pb%zu", idx);
    }
  }

  void emit_row_begin() {
    os << "  static DISC_DEV void row_begin(const Args& A, disc::i64 row, RowCtx& rc) { row_begin2(A, row, 0, rc); }\n";
    os << "  static DISC_DEV void row_begin2(const Args& A, disc::i64 row_base, int row_delta, RowCtx& rc) {"
          " row_begin3(A, row_base, row_delta, row_base * A.inner, rc); }\n";
    // row = row_base + row_delta; base_off = row_base * inner, handed in by callers that keep it running
    os << "  static DISC_DEV void row_begin3(const Args& A, disc::i64 row_base, int row_delta, disc::i64 base_off, RowCtx& rc) {\n";
    os << "    const disc::i64 row = row_base + row_delta;\n";
    // tail_ok: a ragged slot of this row may read its whole vector, because the rows after it hold
    // the surplus elements (at most 15; one more row does when rows are that long, 16 rows always do)
    os << "    rc.sb = base_off;\n    rc.lb = row_delta * (int)A.inner;\n"
       << "    rc.tail_ok = A.rows - 1 - row >= (A.inner >= 15 ? 1 : 16);\n";
    const int n_outer = an.inner_group;
    const bool decomp = an.needs_decomp || (col_tmpl() && an.mid_group == 1);
    if (decomp) {
      os << "    disc::i64 ig[4] = {0, 0, 0, 0};\n";
      os << "    if (A.rows < 2147483648LL) {\n      disc::u32 t = (disc::u32)row;\n";
      for (int g = n_outer - 1; g >= 1; --g)
        os << fmt("      { disc::u32 q = disc::fdiv(t, A.gd%d); ig[%d] = t - q * A.gd%d.d; t = q; }\n", g, g, g);
      os << "      ig[0] = t;\n    } else {\n      disc::i64 t = row;\n";
      for (int g = n_outer - 1; g >= 1; --g)
        os << fmt("      { disc::i64 q = t / A.gs%d; ig[%d] = t - q * A.gs%d; t = q; }\n", g, g, g);
      os << "      ig[0] = t;\n    }\n";
    }
    if (col_tmpl()) os << (an.mid_group == 1 ? "    rc.ob = ig[0] * A.inner;\n" : "    rc.ob = 0;\n");
    for (size_t i = 0; i < an.accesses.size(); ++i) {
      const Access& a = an.accesses[i];
      if (a.kind == ACC_PARTIAL) {
        std::string e;
        size_t sp = 0;
        if (a.offset_index >= 0)
          e = fmt("%sA.st%d", an.offsets[a.offset_index].negative ? "-" : "", (int)an.products.size() + a.offset_index);
        for (size_t t = 0; t < a.groups.size(); ++t) {
          if (a.groups[t] == an.inner_group) continue;
          if (!e.empty()) e += " + ";
          e += fmt("ig[%d] * A.st%d", a.groups[t], a.stride_prod[sp++]);
        }
        if (e.empty()) e = "0";
        if (a.has_inner || a.is_output) os << "    rc.b" << i << " = " << e << ";\n";
        else os << "    const disc::i64 pb" << i << " = " << e << ";\n";
        if (has_outer_window(a)) {
          // the row lies inside the operand along every padded outer group
          std::string v;
          for (size_t t = 0; t < a.groups.size(); ++t) {
            if (a.groups[t] == an.inner_group || a.window[t] < 0) continue;
            if (!v.empty()) v += " && ";
            v += fmt("ig[%d] >= A.st%d && ig[%d] < A.st%d", a.groups[t], window_arg(a.window[t]), a.groups[t], window_arg(a.window[t]) + 1);
          }
          os << "    rc.v" << i << " = " << v << ";\n";
        }
      }
    }
    Fn fn(*this, M_ROWLOCAL);
    for (size_t i = 0; i < an.nodes.size(); ++i) {
      const Node& n = an.nodes[i];
      if (n.opcode == DISC_PARAM) {
        const Access& a = an.accesses[n.access];
        if (a.has_inner) continue;
        std::string off = perrow_offset(a, n.access);
        assign_row(fn, i, from_storage(fmt("A.p%d[%s]", a.slot, off.c_str()), a.dtype));
      } else if (!col_tmpl() && n.dom == DOM_ROW && n.phase == 0) {
        std::string v = fn.val((int)i);
        assign_row(fn, i, v);
      }
    }
    os << fn.body.str();
    os << "    (void)A; (void)row; (void)rc;\n  }\n";
  }

  // Which operand accesses a stage needs: those reachable from the values the stage computes.
  std::vector<char> accesses_needed(const std::vector<int>& roots, bool stop_at_reduce) {
    std::vector<char> need(an.accesses.size(), 0), seen(an.nodes.size(), 0);
    std::vector<int> stack(roots);
    while (!stack.empty()) {
      int id = stack.back();
      stack.pop_back();
      if (seen[id]) continue;
      seen[id] = 1;
      const Node& n = an.nodes[id];
      if (n.opcode == DISC_PARAM) need[n.access] = 1;
      if (stop_at_reduce && is_reduce(n.opcode)) continue;
      for (int k = 0; k < n.n_in; ++k) stack.push_back(n.in[k]);
    }
    return need;
  }

  // outputs written per element by the epilogue (column reduce: only those that keep the reduced axis)
  bool elem_output(const Access& a) const {
    if (!a.has_inner || a.col_sum || a.compact_rank) return false;
    if (!col_tmpl()) return true;
    for (int g : a.groups) if (g == an.mid_group) return true;
    return false;
  }

  void emit_slots(const std::vector<char>& need, bool with_red, bool with_keep) {
    os << "  template <int V> struct Slot {\n";
    for (size_t i = 0; i < an.accesses.size(); ++i) {
      const Access& a = an.accesses[i];
      if (!a.is_output && a.has_inner && need[i] && !late(a)) os << "    disc::Vec<" << dtype_ctype(a.dtype) << ", V> a" << i << ";\n";
    }
    if (with_red)
      for (int id : an.reduces[0])
        os << "    disc::Vec<" << reg_ctype(an.nodes[id].rk) << ", V> red" << an.nodes[id].reduce_slot << ";\n";
    os << "    int unused_;\n  };\n";
    os << "  template <int V> struct Keep {\n";
    if (with_keep)
      for (int id : keep_nodes)   // native vectors: always registers, never a stack array
        os << "    typename disc::Vec<" << reg_ctype(an.nodes[id].rk) << ", V>::vec_t k" << id << ";\n";
    os << "    int unused_;\n  };\n";
    os << "  template <int V> struct OutSlot {\n";
    for (size_t i = 0; i < an.accesses.size(); ++i) {
      const Access& a = an.accesses[i];
      if (a.is_output && elem_output(a)) os << "    disc::Vec<" << dtype_ctype(a.dtype) << ", V> o" << a.slot << ";\n";
    }
    if (compact_tmpl()) os << "    bool keep[V];\n";   // the predicate of every element of the slot
    os << "    int unused_;\n  };\n";
  }

  // pointer and element offset of slot `col` of an access that spans the inner group
  std::string elem_ptr(const Access& a, const std::string& p) {
    return a.kind == ACC_FULL ? "(" + p + " + rc.sb)" : p;
  }
  std::string elem_base(const Access& a, size_t i) {
    if (a.kind == ACC_ROWVEC) return "col";
    if (a.kind == ACC_FULL) return "disc::off(rc.lb, col)";
    return fmt("rc.b%zu + col", i);
  }

  void emit_load_store(const std::vector<char>& need, bool with_red) {
    if (with_red) emit_load(need, false, "load_x");   // operands only: the caller holds the reduce results
    emit_load(need, with_red, "load");
    emit_store();
  }
  void emit_load(const std::vector<char>& need, bool with_red, const char* name) {
    os << "  template <int V, int NT = 0, class C, class SP> static DISC_DEV void " << name << "(const Args& A, const RowCtx& rc, C col, SP sp, Slot<V>& s) {\n";
    for (size_t i = 0; i < an.accesses.size(); ++i) {
      const Access& a = an.accesses[i];
      if (a.is_output || !a.has_inner || !need[i] || late(a)) continue;
      os << "    " << load_call(a, i, fmt("s.a%zu", i), a.kind == ACC_FULL ? "<(NT & 1) != 0>" : "",
                            a.kind == ACC_FULL ? ", rc.tail_ok" : "") << "\n";
    }
    if (with_red) {
      int k = 0;
      for (int id : an.reduces[0]) {
        const Node& n = an.nodes[id];
        os << "    disc::ld(s.red" << n.reduce_slot << ", reinterpret_cast<const " << reg_ctype(n.rk)
           << "*>(reinterpret_cast<const char*>(A.ws1) + " << k << " * A.aux1), rc.ob + col, sp);\n";
        ++k;
      }
    }
    os << "    (void)A; (void)rc; (void)col; (void)sp; (void)s;\n  }\n";
  }
  void emit_store() {
    os << "  template <int V, int NT = 0, class C, class SP> static DISC_DEV void store(const Args& A, const RowCtx& rc, C col, SP sp, const OutSlot<V>& o) {\n";
    for (size_t i = 0; i < an.accesses.size(); ++i) {
      const Access& a = an.accesses[i];
      if (!a.is_output || !elem_output(a)) continue;
      os << "    disc::st" << (a.kind == ACC_FULL ? "<(NT & 2) != 0>" : "") << "(" << elem_ptr(a, fmt("A.o%d", a.slot)) << ", " << elem_base(a, i)
         << ", o.o" << a.slot << ", sp);\n";
    }
    os << "    (void)A; (void)rc; (void)col; (void)sp; (void)o;\n  }\n";
  }

  void emit_acc_types() {
    int max_bytes = 8;
    for (int p = 0; p < an.n_phases; ++p) {
      os << "struct PatAcc" << p << " {\n";
      int bytes = 0;
      for (int id : an.reduces[p]) {
        const Node& n = an.nodes[id];
        const std::string ct = acc_ctype(n);
        os << "  " << ct << " " << accf(n.reduce_slot) << ";\n";
        bytes += (ct == "double" || ct == "disc::i64") ? 8 : 4;
        if (n.opcode == DISC_REDUCE_ARGMAX) { os << "  int " << acci(n.reduce_slot) << ";\n"; bytes += 4; }
      }
      os << "};\n";
      max_bytes = std::max(max_bytes, (bytes + 7) / 8 * 8 + 8);
    }
    os << "template <int P> struct PatAccSel { typedef int type; };\n";
    for (int p = 0; p < an.n_phases; ++p)
      os << "template <> struct PatAccSel<" << p << "> { typedef PatAcc" << p << " type; };\n";
    acc_bytes = max_bytes;
  }

  std::string identity(const Node& n) {
    RegKind ok = an.nodes[n.in[0]].rk;
    switch (n.opcode) {
      case DISC_REDUCE_SUM: return acc_ctype(n) == "double" ? "0.0" : ok == RK_F32 ? "0.0f" : "0";
      case DISC_REDUCE_MIN: return ok == RK_F32 ? "__builtin_inff()" : ok == RK_I64 ? "9223372036854775807LL" : "2147483647";
      default: return ok == RK_F32 ? "(-__builtin_inff())" : ok == RK_I64 ? "(-9223372036854775807LL - 1)" : "(-2147483647 - 1)";
    }
  }

  // statement folding value `x` of one element into accumulator field(s) of reduce node n
  std::string fold_stmt(const Node& n, const std::string& x, const std::string& idx) {
    RegKind ok = an.nodes[n.in[0]].rk;
    std::string f = "acc." + accf(n.reduce_slot), i = "acc." + acci(n.reduce_slot);
    switch (n.opcode) {
      case DISC_REDUCE_SUM:
        if (ok == RK_I32 || ok == RK_I64) return f + " = " + Fn::wrap_arith(ok, f, "+", x) + ";";   // integer sums wrap
        return f + " += " + x + ";";
      case DISC_REDUCE_MAX:
        return ok == RK_F32 ? f + " = fmaxf(" + f + ", " + x + ");" : f + " = " + f + " > " + x + " ? " + f + " : " + x + ";";
      case DISC_REDUCE_MIN:
        return ok == RK_F32 ? f + " = fminf(" + f + ", " + x + ");" : f + " = " + f + " < " + x + " ? " + f + " : " + x + ";";
      default:
        return "if (" + x + " > " + f + ") { " + f + " = " + x + "; " + i + " = " + idx + "; }";
    }
  }

  void emit_acc_basic() {
    os << "  template <int P> static DISC_DEV void acc_init(Acc<P>& a) {\n";
    for (int p = 0; p < an.n_phases; ++p) {
      os << "    if constexpr (P == " << p << ") {\n";
      for (int id : an.reduces[p]) {
        const Node& n = an.nodes[id];
        os << "      a." << accf(n.reduce_slot) << " = " << identity(n) << ";\n";
        if (n.opcode == DISC_REDUCE_ARGMAX) os << "      a." << acci(n.reduce_slot) << " = 2147483647;\n";
      }
      os << "    }\n";
    }
    os << "    (void)a;\n  }\n";
    os << "  template <int P> static DISC_DEV void acc_merge(Acc<P>& a, const Acc<P>& b) {\n";
    for (int p = 0; p < an.n_phases; ++p) {
      os << "    if constexpr (P == " << p << ") {\n";
      for (int id : an.reduces[p]) {
        const Node& n = an.nodes[id];
        RegKind ok = an.nodes[n.in[0]].rk;
        std::string f = accf(n.reduce_slot), i = acci(n.reduce_slot);
        switch (n.opcode) {
          case DISC_REDUCE_SUM:
            if (ok == RK_I32 || ok == RK_I64) os << "      a." << f << " = " << Fn::wrap_arith(ok, "a." + f, "+", "b." + f) << ";\n";
            else os << "      a." << f << " += b." << f << ";\n";
            break;
          case DISC_REDUCE_MAX:   // compare-select: partner values arrive through lane exchanges / LDS
            os << "      a." << f << " = b." << f << " > a." << f << " ? b." << f << " : a." << f << ";\n";
            break;
          case DISC_REDUCE_MIN:
            os << "      a." << f << " = b." << f << " < a." << f << " ? b." << f << " : a." << f << ";\n";
            break;
          default:
            os << "      if (b." << f << " > a." << f << " || (b." << f << " == a." << f << " && b." << i << " < a." << i
               << ")) { a." << f << " = b." << f << "; a." << i << " = b." << i << "; }\n";
        }
      }
      os << "    }\n";
    }
    os << "    (void)a; (void)b;\n  }\n";
    os << "  template <int P, int S> static DISC_DEV void acc_xchg(Acc<P>& a) {\n";
    for (int p = 0; p < an.n_phases; ++p) {
      os << "    if constexpr (P == " << p << ") {\n";
      for (int id : an.reduces[p]) {
        const Node& n = an.nodes[id];
        os << "      a." << accf(n.reduce_slot) << " = disc::lane_xchg<S>(a." << accf(n.reduce_slot) << ");\n";
        if (n.opcode == DISC_REDUCE_ARGMAX)
          os << "      a." << acci(n.reduce_slot) << " = disc::lane_xchg<S>(a." << acci(n.reduce_slot) << ");\n";
      }
      os << "    }\n";
    }
    os << "    (void)a;\n  }\n";
  }

  // May the vector slots of a row start at any column (the _t versions shift them to the 16-byte
  // boundaries of the tensor)?  The copies of row vectors in LDS are then read with element
  // alignment, which is only as fast as an aligned read for elements of 4 bytes and more.
  bool row_shift_ok() const {
    if (!row_tmpl() || an.n_col_sums > 0) return false;
    for (int ai : staged_accesses())
      if (dtype_bytes(an.accesses[ai].dtype) < 4) return false;
    return true;
  }
  // row-vector operands of a row reduce that can be staged in LDS, in access order
  std::vector<int> staged_accesses() const {
    std::vector<int> r;
    if (!row_tmpl()) return r;
    for (size_t i = 0; i < an.accesses.size(); ++i)
      if (late(an.accesses[i]) && an.accesses[i].kind == ACC_ROWVEC) r.push_back((int)i);
    return r;
  }
  int staged_index(int access) const {
    std::vector<int> st = staged_accesses();
    for (size_t k = 0; k < st.size(); ++k)
      if (st[k] == access) return (int)k;
    return -1;
  }
  // byte offset of staged operand k: operands are laid out one after the other, each
  // (inner + vector width) elements long (zero padding behind), rounded up to 16 bytes.  The
  // padding is that of the pattern's vector width whatever the width of the slot that reads the
  // copy (the single elements at the end of a row read it too).
  void emit_stage_fns() {
    std::vector<int> st = staged_accesses();
    const int pad = an.vec_width;
    os << "  static constexpr int N_STAGED = " << st.size() << ";\n";
    os << "  static DISC_DEV int stage_offset(const Args& A, int k) {\n    int off = 0;\n";
    for (size_t k = 0; k < st.size(); ++k)
      os << "    if (k > " << k << ") off += (((int)A.inner + " << pad << ") * " << dtype_bytes(an.accesses[st[k]].dtype) << " + 15) & ~15;\n";
    os << "    (void)A; (void)k;\n    return off;\n  }\n";
    os << "  template <int V> static DISC_DEV void stage(const Args& A, char* lds, int tid, int nthreads) {\n";
    for (size_t k = 0; k < st.size(); ++k) {
      const Access& a = an.accesses[st[k]];
      os << "    {\n      " << dtype_ctype(a.dtype) << "* dst = reinterpret_cast<" << dtype_ctype(a.dtype)
         << "*>(lds + stage_offset(A, " << k << "));\n";
      os << "      const int n = (int)A.inner;\n";
      os << "      disc::stage_copy<" << pad << ">(dst, A.p" << a.slot << ", n, tid, nthreads);\n    }\n";
    }
    os << "    (void)A; (void)lds; (void)tid; (void)nthreads;\n  }\n";
  }

  void emit_late_loads(std::ostream& o, const Fn& fn, const char* ind) {
    for (int ai : fn.late_used) {
      const Access& a = an.accesses[ai];
      o << ind << "disc::Vec<" << dtype_ctype(a.dtype) << ", V> l" << ai << ";\n";
      const int st = staged_index(ai);
      if (st >= 0) {
        // a compile-time choice: behind a run-time branch the wait for the operand would cover both
        // the LDS and the global counter, and so also the row loads that are in flight for later
        o << ind << "if constexpr (STAGED) disc::ld_lds<SP::kAnyColumn && " << (row_shift_ok() ? "true" : "false") << ">(l" << ai << ", rc.sl, stage_offset(A, " << st << "), (int)col);\n";
        o << ind << "else " << load_call(a, ai, fmt("l%d", ai), "", "") << "\n";
      } else {
        o << ind << load_call(a, ai, fmt("l%d", ai), "", "") << "\n";
      }
    }
  }

  // one flavour (with or without cross-phase registers) of reduction phase p, slot granularity
  void emit_phase_flavour(int p, bool keep) {
    Fn fn(*this, M_ELEM);
    fn.P = p;
    fn.keep = keep;
    std::string tail, tail_pred;
    for (int id : an.reduces[p]) {
      const Node& n = an.nodes[id];
      const std::string x = fn.val(n.in[0]);
      const std::string st = fold_stmt(n, x, "col + e");
      tail += "        " + st + "\n";
      // elements outside the row contribute the identity; selecting the value (not the update)
      // keeps the accumulation itself the same instruction sequence as in the full body
      if (n.opcode == DISC_REDUCE_ARGMAX) tail_pred += "        if (sp.has(e)) { " + st + " }\n";
      else tail_pred += "        " + fold_stmt(n, "(sp.has(e) ? " + x + " : " + identity(n) + ")", "col + e") + "\n";
    }
    emit_late_loads(os, fn, "      ");
    // wave-uniform choice: the unpredicated body only when every lane of the wavefront has a
    // full slot; otherwise the whole wavefront takes the predicated body once (a per-lane branch
    // would make wavefronts with one ragged lane execute both bodies)
    os << "      if (disc::wave_all(sp.full(V))) {\n#pragma unroll\n      for (int e = 0; e < V; ++e) {\n" << fn.body.str() << tail << "      }\n";
    os << "      } else {\n#pragma unroll\n      for (int e = 0; e < V; ++e) {\n" << fn.body.str() << tail_pred << "      }\n      }\n";
  }

  void emit_row_phase_fns() {
    os << "  template <int P, int V, bool KEEP, class SP> static DISC_DEV void phase(const Args& A, Acc<P>& acc, const Slot<V>& s, Keep<V>& k, SP sp, int col, const RowCtx& rc) {\n";
    for (int p = 0; p < an.n_phases; ++p) {
      os << "    if constexpr (P == " << p << ") {\n";
      os << "      if constexpr (KEEP) {\n";
      emit_phase_flavour(p, true);
      os << "      } else {\n";
      emit_phase_flavour(p, false);
      os << "      }\n    }\n";
    }
    os << "    (void)A; (void)acc; (void)s; (void)k; (void)sp; (void)col; (void)rc;\n  }\n";
    // per-row values known after phase P
    os << "  template <int P> static DISC_DEV void row_after(const Args& A, RowCtx& rc, const Acc<P>& acc) {\n";
    for (int p = 0; p < an.n_phases; ++p) {
      os << "    if constexpr (P == " << p << ") {\n";
      Fn fn(*this, M_ROWLOCAL);
      // earlier per-row values are read back from rc
      for (size_t i = 0; i < an.nodes.size(); ++i) {
        const Node& n = an.nodes[i];
        if (n.dom != DOM_ROW) continue;
        if (n.phase <= p && !(is_reduce(n.opcode) && n.phase == p + 1)) fn.names[(int)i] = fmt("rc.r%zu", i);
      }
      for (int id : an.reduces[p]) assign_row(fn, id, acc_value(an.nodes[id], "acc"));
      for (size_t i = 0; i < an.nodes.size(); ++i) {
        const Node& n = an.nodes[i];
        if (n.dom != DOM_ROW || n.phase != p + 1 || is_reduce(n.opcode)) continue;
        std::string v = fn.val((int)i);
        assign_row(fn, i, v);
      }
      os << fn.body.str() << "    }\n";
    }
    os << "    (void)A; (void)rc; (void)acc;\n  }\n";
  }

  // column reduce stage 1: element granularity (one accumulator per column element)
  void emit_col_accum() {
    os << "  template <int P, int V> static DISC_DEV void accum(const Args& A, Acc<P>& acc, const Slot<V>& s, int e, int col, const RowCtx& rc) {\n";
    Fn fn(*this, M_COL_ACCUM);
    std::string tail;
    for (int id : an.reduces[0]) {
      const Node& n = an.nodes[id];
      tail += "        " + fold_stmt(n, fn.val(n.in[0]), "col") + "\n";
    }
    os << fn.body.str() << tail;
    os << "    (void)A; (void)acc; (void)s; (void)e; (void)col; (void)rc;\n  }\n";
  }

  void emit_epilogue(Mode mode) {
    os << "  template <int V, bool KEEP, class C, class SP> static DISC_DEV void epilogue(const Args& A, const RowCtx& rc, const Slot<V>& s, const Keep<V>& k, C col, SP sp, OutSlot<V>& o) {\n";
    auto flavour = [&](bool keep) {
      Fn fn(*this, mode);
      fn.P = an.n_phases;
      fn.keep = keep;
      std::ostringstream tail, decl, pack;
      for (const auto& out : an.outputs) {
        const Access& a = an.accesses[out.access];
        if (!elem_output(a)) continue;
        const Node& n = an.nodes[out.node];
        if (is_float_dtype(a.dtype)) {
          // float results are collected in fp32 and rounded to the storage type two at a time
          decl << "      float y" << a.slot << "[V];\n";
          tail << "        y" << a.slot << "[e] = " << convert(fn.val(out.node), n.rk, RK_F32) << ";\n";
          pack << "      disc::cvt_vec(o.o" << a.slot << ", y" << a.slot << ");\n";
        } else {
          decl << "      o.o" << a.slot << ".clear();\n";
          tail << "        o.o" << a.slot << ".set(e, " << to_storage(fn.val(out.node), n.rk, a.dtype) << ");\n";
        }
      }
      if (compact_tmpl()) tail << "        o.keep[e] = " << convert(fn.val(an.compact_keep), an.nodes[an.compact_keep].rk, RK_BOOL) << ";\n";
      emit_late_loads(os, fn, "      ");
      os << decl.str();
      os << "#pragma unroll\n      for (int e = 0; e < V; ++e) {\n" << fn.body.str() << tail.str() << "      }\n" << pack.str();
    };
    if (row_tmpl() && mode == M_ELEM) {
      os << "    if constexpr (KEEP) {\n";
      flavour(true);
      os << "    } else {\n";
      flavour(false);
      os << "    }\n";
    } else {
      os << "    {\n";
      flavour(false);
      os << "    }\n";
    }
    os << "    (void)A; (void)rc; (void)s; (void)k; (void)col; (void)sp; (void)o;\n  }\n";
    os << "  static DISC_DEV void row_store(const Args& A, disc::i64 row, const RowCtx& rc) {\n";
    if (!col_tmpl()) {
      for (const auto& out : an.outputs) {
        const Access& a = an.accesses[out.access];
        if (a.has_inner || a.row_red || a.compact_count) continue;
        const Node& n = an.nodes[out.node];
        std::string off = a.kind == ACC_PERROW ? "row" : a.kind == ACC_SCALAR ? "0" : fmt("rc.b%d", out.access);
        Fn fn2(*this, M_ELEM);
        os << "    A.o" << a.slot << "[" << off << "] = " << to_storage(fn2.val(out.node), n.rk, a.dtype) << ";\n";
      }
    }
    os << "    (void)A; (void)row; (void)rc;\n  }\n";
  }

  // ---- row reduce with sums over the rows: per-column partial sums next to the epilogue --------
  // ColAcc holds one fp32 vector per summed output; col_sums adds one slot of one row to it;
  // colsum_store rounds the finished sums of one column to the outputs' types.
  void emit_col_sums() {
    const int nq = an.n_col_sums;
    os << "  static constexpr int NCOLSUM = " << nq << ";\n";
    os << "  template <int V> struct ColAcc { typename disc::Vec<float, V>::vec_t c[" << std::max(nq, 1) << "]; };\n";
    if (nq == 0) return;
    os << "  template <int V, bool KEEP, class C, class SP> static DISC_DEV void col_sums(const Args& A, const RowCtx& rc, const Slot<V>& s, const Keep<V>& k, C col, SP sp, ColAcc<V>& ca) {\n";
    auto flavour = [&](bool keep) {
      Fn fn(*this, M_ELEM);
      fn.P = an.n_phases;
      fn.keep = keep;
      std::ostringstream tail;
      int q = 0;
      for (const auto& out : an.outputs) {
        if (!out.col_sum) continue;
        tail << "        ca.c[" << q++ << "][e] += " << convert(fn.val(out.node), an.nodes[out.node].rk, RK_F32) << ";\n";
      }
      emit_late_loads(os, fn, "      ");
      os << "#pragma unroll\n      for (int e = 0; e < V; ++e) {\n" << fn.body.str() << tail.str() << "      }\n";
    };
    os << "    if constexpr (KEEP) {\n";
    flavour(true);
    os << "    } else {\n";
    flavour(false);
    os << "    }\n";
    os << "    (void)A; (void)rc; (void)s; (void)k; (void)col; (void)sp; (void)ca;\n  }\n";
    os << "  static DISC_DEV void colsum_store(const Args& A, disc::i64 col, const float (&v)[" << nq << "]) {\n";
    int q = 0;
    for (const auto& out : an.outputs) {
      if (!out.col_sum) continue;
      const Access& a = an.accesses[out.access];
      os << "    A.o" << a.slot << "[col] = " << to_storage(fmt("v[%d]", q++), RK_F32, a.dtype) << ";\n";
    }
    os << "  }\n";
  }

  // ---- row reduce with reductions of per-row values over the rows (to one number each) ----------
  // rr_identity / rr_merge: the reduction of output q; row_reds folds one finished row into a
  // lane's running values; rowred_store rounds the results to the outputs' types.
  void emit_row_reds() {
    const int nq = an.n_row_reds;
    os << "  static constexpr int NROWRED = " << nq << ";\n";
    if (nq == 0) return;
    std::vector<const OutputRef*> outs;
    for (const auto& out : an.outputs) if (out.row_red) outs.push_back(&out);
    os << "  static DISC_DEV float rr_identity(int q) {\n    switch (q) {\n";
    for (int q = 0; q < nq; ++q)
      os << "      case " << q << ": return " << (outs[q]->red_opcode == DISC_REDUCE_SUM ? "0.0f" : outs[q]->red_opcode == DISC_REDUCE_MAX ? "-__builtin_inff()" : "__builtin_inff()") << ";\n";
    os << "    }\n    return 0.0f;\n  }\n";
    for (const char* ty : {"float", "double"}) {
      os << "  static DISC_DEV " << ty << " rr_merge(int q, " << ty << " a, " << ty << " b) {\n    switch (q) {\n";
      for (int q = 0; q < nq; ++q) {
        const int oc = outs[q]->red_opcode;
        const std::string f = std::string(oc == DISC_REDUCE_MAX ? "fmax" : "fmin") + (ty[0] == 'f' ? "f" : "");
        os << "      case " << q << ": return " << (oc == DISC_REDUCE_SUM ? std::string("a + b") : f + "(a, b)") << ";\n";
      }
      os << "    }\n    return a;\n  }\n";
    }
    os << "  static DISC_DEV void row_reds(const Args& A, const RowCtx& rc, float (&r)[" << nq << "]) {\n";
    for (int q = 0; q < nq; ++q) {
      const Node& n = an.nodes[outs[q]->node];
      os << "    r[" << q << "] = rr_merge(" << q << ", r[" << q << "], " << convert(fmt("rc.r%d", outs[q]->node), n.rk, RK_F32) << ");\n";
    }
    os << "    (void)A;\n  }\n";
    os << "  static DISC_DEV void rowred_store(const Args& A, const float (&v)[" << nq << "]) {\n";
    for (int q = 0; q < nq; ++q) {
      const Access& a = an.accesses[outs[q]->access];
      os << "    A.o" << a.slot << "[0] = " << to_storage(fmt("v[%d]", q), RK_F32, a.dtype) << ";\n";
    }
    os << "  }\n";
  }

  // ---- column reduce: partial-accumulator planes and the finish step -------------------------
  // Workspace ws0 holds one 8-byte cell per (accumulator field, outer, chunk, column); ws1 holds
  // the final reduce results, one plane per reduction, typed as the reduce result's register kind.
  void emit_col_extras() {
    int k = 0;
    auto cell = [&](const std::string& ct, const std::string& field, bool store) {
      std::string wide = (ct == "float" || ct == "double") ? "double" : "disc::i64";
      if (store) os << "    reinterpret_cast<" << wide << "*>(A.ws0)[" << k << " * A.aux0 + idx] = (" << wide << ")a." << field << ";\n";
      else os << "    a." << field << " = (" << ct << ")reinterpret_cast<const " << wide << "*>(A.ws0)[" << k << " * A.aux0 + idx];\n";
      ++k;
    };
    os << "  static DISC_DEV void acc_st(const Args& A, disc::i64 idx, const Acc<0>& a) {\n";
    for (int id : an.reduces[0]) {
      const Node& n = an.nodes[id];
      cell(acc_ctype(n), accf(n.reduce_slot), true);
      if (n.opcode == DISC_REDUCE_ARGMAX) cell("int", acci(n.reduce_slot), true);
    }
    os << "    (void)A; (void)idx; (void)a;\n  }\n";
    n_acc_cells = k;
    k = 0;
    os << "  static DISC_DEV void acc_ld(const Args& A, disc::i64 idx, Acc<0>& a) {\n";
    for (int id : an.reduces[0]) {
      const Node& n = an.nodes[id];
      cell(acc_ctype(n), accf(n.reduce_slot), false);
      if (n.opcode == DISC_REDUCE_ARGMAX) cell("int", acci(n.reduce_slot), false);
    }
    os << "    (void)A; (void)idx; (void)a;\n  }\n";
    // finish: one (outer index o, column c); writes the reduce-result planes and every output that
    // has lost the reduced axis
    os << "  static DISC_DEV void col_finish(const Args& A, disc::i64 o, disc::i64 c, const Acc<0>& acc) {\n";
    Fn fn(*this, M_COL_FINISH);
    std::ostringstream tail;
    k = 0;
    for (int id : an.reduces[0]) {
      const Node& n = an.nodes[id];
      tail << "    reinterpret_cast<" << reg_ctype(n.rk) << "*>(reinterpret_cast<char*>(A.ws1) + " << k
           << " * A.aux1)[o * A.inner + c] = " << fn.val(id) << ";\n";
      ++k;
    }
    for (const auto& out : an.outputs) {
      const Access& a = an.accesses[out.access];
      if (elem_output(a)) continue;
      const Node& n = an.nodes[out.node];
      std::string off = a.groups.size() > 1 ? "o * A.inner + c" : "c";
      tail << "    A.o" << a.slot << "[" << off << "] = " << to_storage(fn.val(out.node), n.rk, a.dtype) << ";\n";
    }
    os << fn.body.str() << tail.str();
    os << "    (void)A; (void)o; (void)c; (void)acc;\n  }\n";
  }

  // column reduce, two-launch version: the finish step of one (outer index o, column c) with the
  // reduce results delivered into element e of a slot (registers) instead of the workspace planes;
  // `write` (one block per column tile) also stores the outputs that lost the reduced axis
  void emit_finish_elem() {
    os << "  template <int V> static DISC_DEV void clear_red(Slot<V>& s) {\n";
    for (int id : an.reduces[0]) os << "    s.red" << an.nodes[id].reduce_slot << ".clear();\n";
    os << "    (void)s;\n  }\n";
    os << "  template <int V> static DISC_DEV void finish_elem(const Args& A, disc::i64 o, disc::i64 c, const Pat::Acc<0>& acc, Slot<V>& s, int e, bool write) {\n";
    Fn fn(*this, M_COL_FINISH);
    std::ostringstream tail;
    for (int id : an.reduces[0]) {
      const Node& n = an.nodes[id];
      tail << "    s.red" << n.reduce_slot << ".set(e, " << fn.val(id) << ");\n";
    }
    tail << "    if (write) {\n";
    for (const auto& out : an.outputs) {
      const Access& a = an.accesses[out.access];
      if (elem_output(a)) continue;
      const Node& n = an.nodes[out.node];
      std::string off = a.groups.size() > 1 ? "o * A.inner + c" : "c";
      tail << "      A.o" << a.slot << "[" << off << "] = " << to_storage(fn.val(out.node), n.rk, a.dtype) << ";\n";
    }
    tail << "    }\n";
    os << fn.body.str() << tail.str();
    os << "    (void)A; (void)o; (void)c; (void)acc; (void)s; (void)e; (void)write;\n  }\n";
  }

  // compaction pattern: where the kept values, the slots and the count go
  void emit_compact_fns() {
    os << "  template <int V> static DISC_DEV void compact_store(const Args& A, const OutSlot<V>& o, int e, disc::i64 pos) {\n";
    for (const auto& out : an.outputs) {
      const Access& a = an.accesses[out.access];
      if (a.compact) os << "    A.o" << a.slot << "[pos] = o.o" << a.slot << ".get(e);\n";
    }
    os << "    (void)A; (void)o; (void)e; (void)pos;\n  }\n";
    // the slots of the V elements of one slot of the tile, stored as one vector
    os << "  template <int V> static DISC_DEV void rank_store(const Args& A, disc::i64 col, const disc::i64 (&rank)[V], disc::Span sp) {\n";
    for (const auto& out : an.outputs) {
      const Access& a = an.accesses[out.access];
      if (!a.compact_rank) continue;
      os << "    {\n      disc::Vec<" << dtype_ctype(a.dtype) << ", V> t;\n#pragma unroll\n      for (int e = 0; e < V; ++e) t.v[e] = ("
         << dtype_ctype(a.dtype) << ")rank[e];\n      disc::st(A.o" << a.slot << ", col, t, sp);\n    }\n";
    }
    os << "    (void)A; (void)col; (void)rank; (void)sp;\n  }\n";
    bool has_rank = false;
    for (const auto& out : an.outputs) has_rank = has_rank || an.accesses[out.access].compact_rank;
    os << "  static constexpr bool HAS_RANK = " << (has_rank ? "true" : "false") << ";\n";
    os << "  static DISC_DEV void count_store(const Args& A, disc::i64 total) {\n";
    for (const auto& out : an.outputs) {
      const Access& a = an.accesses[out.access];
      if (a.compact_count) os << "    A.o" << a.slot << "[0] = (" << dtype_ctype(a.dtype) << ")total;\n";
    }
    os << "    (void)A; (void)total;\n  }\n";
  }

  void emit_args() {
    os << "  struct Args {\n";
    for (const auto& f : layout.fields) os << "    " << field_decl(f) << "\n";
    os << "  };\n";
  }

  bool has_elem_outputs() const {
    for (const auto& out : an.outputs)
      if (elem_output(an.accesses[out.access])) return true;
    return false;
  }

  void emit_kernels(Generated* out) {
    const int V = an.vec_width;
    int max_threads = 256;   // largest block the entry point may be launched with
    // DISC_STATIC_ARGS / DISC_STATIC_PLAN expand to nothing in the shape-generic module; the
    // single-shape module defines them to overwrite every extent with its constant
    auto k = [&](const std::string& name, const std::string& body, const char* plan, const char* pat = "Pat") {
      if (opt && !opt->only_kernels.empty() &&
          std::find(opt->only_kernels.begin(), opt->only_kernels.end(), name) == opt->only_kernels.end())
        return;
      os << "extern \"C\" __global__ void __launch_bounds__(" << max_threads << ") " << out->prefix << name << "(" << pat
         << "::Args A" << (plan ? std::string(", disc::") + plan + " rp" : std::string()) << ") { DISC_STATIC_ARGS(A) "
         << (plan ? "DISC_STATIC_PLAN(rp) " : "") << body << " }\n";
      out->kernels.push_back(name);
    };
    // the wide register-resident row kernels come in a second version (suffix _s) that reads
    // the row-vector operands from their LDS copy
    const bool staged = !staged_accesses().empty();
    auto krow = [&](const std::string& name, int v, int nv) {
      // the two-slot version for blocks above 256 threads runs without the software pipeline: the
      // registers it saves let a CU hold three 8-wavefront blocks instead of two (+10 % measured);
      // with three slots the residency is the same either way and the pipeline wins
      const char* pipe = max_threads > 256 && nv == 2 ? "false" : "true";
      k(name, fmt("disc::row_reg_body<Pat, %d, %d, %s>(A, rp);", v, nv, pipe), "RowPlan");
      if (staged && v > 1)
        k(name + "_s", fmt("disc::row_reg_body<PatT<true>, %d, %d, %s>(A, rp);", v, nv, pipe), "RowPlan", "PatT<true>");
      // blocks of one wavefront quad, vector width: versions whose vector slots are all whole (no
      // ragged-tail path anywhere in them).  _e: rows that are a whole number of slots; _nt: the
      // same with non-temporal accesses of the full-size operands, for large launches of rows that
      // start and end on 16-byte boundaries; _t: the elements behind the last whole slot of a row
      // are taken one per lane as slots of ONE element (not with sums over the rows: there a
      // lane's columns are laid out by slot).
      const bool tail = an.n_col_sums == 0;
      if (v > 1 && max_threads <= 256) {
        k(name + "_e", fmt("disc::row_reg_body<Pat, %d, %d, %s, 0, true>(A, rp);", v, nv, pipe), "RowPlan");
        if (tail) k(name + "_t", fmt("disc::row_reg_body<Pat, %d, %d, %s, 0, true, true>(A, rp);", v, nv, pipe), "RowPlan");
        k(name + "_nt", fmt("disc::row_reg_body<Pat, %d, %d, %s, 3, true>(A, rp);", v, nv, pipe), "RowPlan");
        if (staged) {
          k(name + "_s_e", fmt("disc::row_reg_body<PatT<true>, %d, %d, %s, 0, true>(A, rp);", v, nv, pipe), "RowPlan", "PatT<true>");
          if (tail) k(name + "_s_t", fmt("disc::row_reg_body<PatT<true>, %d, %d, %s, 0, true, true>(A, rp);", v, nv, pipe), "RowPlan", "PatT<true>");
          k(name + "_s_nt", fmt("disc::row_reg_body<PatT<true>, %d, %d, %s, 3, true>(A, rp);", v, nv, pipe), "RowPlan", "PatT<true>");
        }
      }
      // blocks above 256 threads: the _t version of the two-slot kernel only (the three-slot one
      // has no registers to spare under its 128-register cap)
      if (v > 1 && max_threads > 256 && nv == 2 && tail) {
        k(name + "_t", fmt("disc::row_reg_body<Pat, %d, %d, %s, 0, true, true>(A, rp);", v, nv, pipe), "RowPlan");
        if (staged) k(name + "_s_t", fmt("disc::row_reg_body<PatT<true>, %d, %d, %s, 0, true, true>(A, rp);", v, nv, pipe), "RowPlan", "PatT<true>");
      }
    };
    if (an.tmpl == DISC_TEMPLATE_COMPACT) {
      k("k_compact_count_vec", fmt("disc::compact_count_body<Pat, %d>(A);", V), nullptr);
      k("k_compact_count_scalar", "disc::compact_count_body<Pat, 1>(A);", nullptr);
      k("k_compact_scatter_vec", fmt("disc::compact_scatter_body<Pat, %d>(A);", V), nullptr);
      k("k_compact_scatter_scalar", "disc::compact_scatter_body<Pat, 1>(A);", nullptr);
      max_threads = 1024;
      k("k_compact_scan", "disc::compact_scan_body<Pat>(A);", nullptr);
      max_threads = 256;
    } else if (an.tmpl == DISC_TEMPLATE_LOOP) {
      k("k_loop_vec", fmt("disc::kloop_body<Pat, %d, 4, false>(A);", V), nullptr);
      if (V > 1) k("k_loop_vec_nt", fmt("disc::kloop_body<Pat, %d, 4, false, 3>(A);", V), nullptr);
      k("k_loop_vec_i64", fmt("disc::kloop_body<Pat, %d, 1, true>(A);", V), nullptr);
      k("k_loop_scalar", "disc::kloop_body<Pat, 1, 4, false>(A);", nullptr);
      k("k_loop_scalar_i64", "disc::kloop_body<Pat, 1, 1, true>(A);", nullptr);
    } else if (an.tmpl == DISC_TEMPLATE_ROW_REDUCE) {
      // two slots per lane keep the register footprint near 100 VGPRs (4-5 waves per SIMD); longer
      // rows get more lanes (blocks of up to 1024 threads) rather than more slots per lane.  The
      // three-slot versions exist for the row lengths that would leave a third of the lanes of the
      // next power of two without work
      // (a row of a single slot runs in the two-slot version: no version of its own)
      krow("k_row_vec_nv2", V, 2);
      krow("k_row_scalar_nv2", 1, 2);
      krow("k_row_vec_nv3", V, 3);
      max_threads = 1024;
      krow("k_row_vec_nv2w", V, 2);
      krow("k_row_vec_nv3w", V, 3);
      krow("k_row_scalar_nv2w", 1, 2);
      max_threads = 256;
      k("k_row_stream_vec", fmt("disc::row_stream_body<Pat, %d>(A);", V), nullptr);
      k("k_row_stream_scalar", "disc::row_stream_body<Pat, 1>(A);", nullptr);
      if (an.n_col_sums > 0) k("k_colsum_finish", "disc::colsum_finish_body<Pat>(A);", nullptr);
      if (an.n_row_reds > 0) {
        max_threads = 1024;
        k("k_rowred_finish", "disc::rowred_finish_body<Pat>(A);", nullptr);
        max_threads = 256;
      }
    } else {
      k("k_col_partial_vec", fmt("disc::col_partial_body<Pat, %d>(A, rp);", V), "ColPlan");
      k("k_col_partial_scalar", "disc::col_partial_body<Pat, 1>(A, rp);", "ColPlan");
      k("k_col_finish", "disc::col_finish_body<Pat>(A, rp);", "ColPlan");
      const char* epi = has_elem_outputs() ? "PatE" : "void";
      k("k_col_strip_vec", fmt("disc::col_strip_body<Pat, %s, %d>(A, rp);", epi, V), "ColPlan");
      k("k_col_strip_scalar", fmt("disc::col_strip_body<Pat, %s, 1>(A, rp);", epi), "ColPlan");
      if (has_elem_outputs()) {
        k("k_col_epi_vec", fmt("disc::kloop_body<PatE, %d, 4, false>(A);", V), nullptr);
        if (V > 1) k("k_col_epi_vec_nt", fmt("disc::kloop_body<PatE, %d, 4, false, 3>(A);", V), nullptr);
        k("k_col_epi_vec_i64", fmt("disc::kloop_body<PatE, %d, 1, true>(A);", V), nullptr);
        k("k_col_epi_scalar", "disc::kloop_body<PatE, 1, 4, false>(A);", nullptr);
        k("k_col_epi_scalar_i64", "disc::kloop_body<PatE, 1, 1, true>(A);", nullptr);
        // two-launch version: finish + epilogue in one kernel (plain; non-temporal stores)
        k("k_col_epi2_vec", fmt("disc::col_epi2_body<Pat, PatE, %d, 0>(A, rp);", V), "ColPlan");
        if (V > 1) k("k_col_epi2_vec_nt", fmt("disc::col_epi2_body<Pat, PatE, %d, 2>(A, rp);", V), "ColPlan");
        k("k_col_epi2_scalar", "disc::col_epi2_body<Pat, PatE, 1, 0>(A, rp);", "ColPlan");
      }
    }
  }

  int run(Generated* out, std::string* err) {
    (void)err;
    build_layout();
    if (an.tmpl == DISC_TEMPLATE_TRANSPOSE) {
      // no fused expression: the argument block and one hand-written tile-transpose kernel
      os << "// generated: a transpose on its own\nstruct Pat {\n";
      emit_args();
      os << "};\n";
      const int ng = (int)an.groups.size();
      const std::string batch = ng == 3 ? "A.gs0" : "1";
      auto k = [&](const std::string& name, const std::string& body) {
        if (opt && !opt->only_kernels.empty() &&
            std::find(opt->only_kernels.begin(), opt->only_kernels.end(), name) == opt->only_kernels.end())
          return;
        os << "extern \"C\" __global__ void __launch_bounds__(256) " << out->prefix << name
           << "(Pat::Args A) { DISC_STATIC_ARGS(A) " << body << " }\n";
        out->kernels.push_back(name);
      };
      k("k_transpose_tile", fmt("disc::ktranspose_body(A.p0, A.o0, %s, A.gs%d, A.gs%d);", batch.c_str(), ng - 2, ng - 1));
      out->source = os.str();
      out->args = layout;
      out->field_names.clear();
      for (const auto& f : layout.fields) out->field_names.push_back(field_name(f));
      out->has_epilogue = false;
      return DISC_OK;
    }
    plan_keeps();
    plan_rinv();
    os << "// generated: one fused pattern, every kernel version\n";
    emit_acc_types();
    std::vector<char> all(an.accesses.size(), 1);
    const bool staged_versions = !staged_accesses().empty();
    if (staged_versions) os << "template <bool ST> struct PatT {\n  static constexpr bool STAGED = ST;\n";
    else os << "struct Pat {\n  static constexpr bool STAGED = false;\n";
    os << "  static constexpr int NPHASE = " << an.n_phases << ";\n";
    os << "  static constexpr int MAX_ACC_BYTES = " << acc_bytes << ";\n";
    os << "  template <int P> using Acc = typename PatAccSel<P>::type;\n";
    emit_args();
    os << "  struct RowCtx {\n" << row_fields() << "  };\n";
    if (!col_tmpl()) {
      emit_slots(all, false, true);
      emit_row_begin();
      emit_load_store(all, false);
      emit_acc_basic();
      if (row_tmpl()) {
        emit_stage_fns();
        emit_row_phase_fns();
      }
      emit_epilogue(M_ELEM);
      emit_col_sums();
      emit_row_reds();
      if (compact_tmpl()) emit_compact_fns();
      os << "};\n";
      if (staged_versions) os << "typedef PatT<false> Pat;\n";
    } else {
      // stage 1 + 2: operands that feed the reductions
      std::vector<int> roots;
      for (int id : an.reduces[0]) roots.push_back(an.nodes[id].in[0]);
      std::vector<char> need1 = accesses_needed(roots, true);
      emit_slots(need1, false, false);
      emit_row_begin();
      emit_load_store(need1, false);
      emit_acc_basic();
      emit_col_accum();
      emit_col_extras();
      os << "  static constexpr int N_ACC_CELLS = " << n_acc_cells << ";\n";
      os << "};\n";
      if (has_elem_outputs()) {
        // stage 3: the epilogue as a loop fusion that reads the reduce results as column vectors
        std::vector<int> eroots;
        for (const auto& o2 : an.outputs)
          if (elem_output(an.accesses[o2.access])) eroots.push_back(o2.node);
        std::vector<char> need3 = accesses_needed(eroots, true);
        os << "struct PatE {\n";
        os << "  static constexpr int NPHASE = 0;\n  static constexpr int MAX_ACC_BYTES = 8;\n";
        os << "  template <int P> using Acc = int;\n";
        os << "  typedef Pat::Args Args;\n  typedef Pat::RowCtx RowCtx;\n";
        emit_slots(need3, true, false);
        os << "  static DISC_DEV void row_begin(const Args& A, disc::i64 row, RowCtx& rc) { Pat::row_begin(A, row, rc); }\n";
        emit_load_store(need3, true);
        emit_epilogue(M_COL_EPI);
        emit_finish_elem();
        os << "};\n";
      }
    }
    os << "static_assert(sizeof(Pat::Args) == " << layout.size << ", \"argument block layout\");\n";
    for (const auto& f : layout.fields)
      os << "static_assert(__builtin_offsetof(Pat::Args, " << field_name(f) << ") == " << f.offset << ", \"argument block layout\");\n";
    emit_kernels(out);
    out->source = os.str();
    out->args = layout;
    out->field_names.clear();
    for (const auto& f : layout.fields) out->field_names.push_back(field_name(f));
    out->n_acc_cells = n_acc_cells;
    out->n_red_planes = col_tmpl() ? (int)an.reduces[0].size() : 0;
    out->has_epilogue = col_tmpl() ? has_elem_outputs() : true;
    out->n_col_sums = row_tmpl() ? an.n_col_sums : 0;
    out->n_row_reds = row_tmpl() ? an.n_row_reds : 0;
    out->row_tail_ok = an.n_col_sums == 0;
    out->row_shift_ok = row_shift_ok();
    out->staged_elem_bytes.clear();
    for (int ai : staged_accesses()) out->staged_elem_bytes.push_back(dtype_bytes(an.accesses[ai].dtype));
    return DISC_OK;
  }
};

}  // namespace

int generate(const Analysis& an, const std::string& prefix, Generated* out, std::string* err, const GenOptions* opt) {
  out->prefix = prefix;
  Gen g(an);
  g.opt = opt;
  return g.run(out, err);
}

}  // namespace disc

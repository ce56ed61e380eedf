// Device-code generation: turns the resolved node graph of a pattern into ONE `struct Pat`
// (the fused per-element expression, operand addressing and reduction bookkeeping) that the
// hand-written schedules of disc_device.h are instantiated with.  All kernel versions of a
// pattern come out of this one translation unit, so a pattern costs exactly one device
// compile whatever shapes it later runs at (Section 2 / Section 4.3 of the paper).
#include <cmath>
#include <cstdarg>
#include <map>
#include <cstdio>
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
  if (s.find('.') == std::string::npos && s.find('e') == std::string::npos && s.find("inf") == std::string::npos)
    s.insert(s.size() - 1, ".0");
  return s;
}

struct Gen {
  const Analysis& an;
  ArgLayout layout;
  std::ostringstream os;
  explicit Gen(const Analysis& a) : an(a) {}

  bool is_reduce(int oc) const { return oc >= DISC_REDUCE_SUM && oc <= DISC_REDUCE_ARGMAX; }

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
    for (size_t i = 0; i < an.products.size(); ++i) add_field(ArgField::STRIDE, (int)i, 8);
    for (size_t i = 0; i < an.dim_size_syms.size(); ++i) add_field(ArgField::DIMI, (int)i, 8);
    add_field(ArgField::SPR_DIV, 0, 16);
    for (int g = 0; g < 3; ++g) add_field(ArgField::GROUP_DIV, g, 16);
    for (size_t i = 0; i < an.dim_size_syms.size(); ++i) add_field(ArgField::DIMF, (int)i, 4);
    if (layout.size % 8) layout.size += 8 - layout.size % 8;
  }
  std::string field_decl(const ArgField& f) const {
    switch (f.kind) {
      case ArgField::ROWS: return "disc::i64 rows;";
      case ArgField::INNER: return "disc::i64 inner;";
      case ArgField::NSLOTS: return "disc::i64 nslots;";
      case ArgField::SPR: return "disc::i64 spr;";
      case ArgField::MID: return "disc::i64 mid;";
      case ArgField::GROUP_SIZE: return fmt("disc::i64 gs%d;", f.index);
      case ArgField::IN_PTR: {
        int dt = DISC_F32;
        int k = 0;
        for (const auto& op : an.ops)
          if (op.opcode == DISC_PARAM && k++ == f.index) dt = op.dtype;
        return fmt("const %s* __restrict__ p%d;", dtype_ctype(dt), f.index);
      }
      case ArgField::OUT_PTR: {
        int dt = DISC_F32;
        int k = 0;
        for (const auto& op : an.ops)
          if (op.opcode == DISC_OUTPUT && k++ == f.index) dt = op.dtype;
        return fmt("%s* __restrict__ o%d;", dtype_ctype(dt), f.index);
      }
      case ArgField::WS_PTR: return fmt("void* ws%d;", f.index);
      case ArgField::AUX: return fmt("disc::i64 aux%d;", f.index);
      case ArgField::STRIDE: return fmt("disc::i64 st%d;", f.index);
      case ArgField::DIMI: return fmt("disc::i64 dimi%d;", f.index);
      case ArgField::SPR_DIV: return "disc::FastDiv spr_div;";
      case ArgField::GROUP_DIV: return fmt("disc::FastDiv gd%d;", f.index);
      case ArgField::DIMF: return fmt("float dimf%d;", f.index);
    }
    return "";
  }
  std::string field_name(const ArgField& f) const {
    std::string d = field_decl(f);
    size_t e = d.rfind(';');
    size_t b = d.find_last_of(" *_", e);   // crude but all names end the declaration
    (void)b;
    size_t sp = d.find_last_of(' ', e);
    return d.substr(sp + 1, e - sp - 1);
  }

  // ---- expression emission ---------------------------------------------------------------
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

  // Emits straight-line code computing nodes inside one device function.  `elem_ok` says
  // whether per-element values may be computed here (slot `s`, element `e` in scope);
  // per-row values are read from `rc` unless `row_define` lists them as being defined here.
  struct Fn {
    Gen& g;
    std::ostringstream body;
    std::map<int, std::string> names;
    bool elem_ok;
    bool row_local;     // compute per-row values locally instead of reading rc (row_begin / row_after)
    Fn(Gen& gg, bool e, bool rl) : g(gg), elem_ok(e), row_local(rl) {}

    std::string val(int id) {
      auto it = names.find(id);
      if (it != names.end()) return it->second;
      const Node& n = g.an.nodes[id];
      std::string r;
      if (n.opcode == DISC_CONST) {
        if (n.rk == RK_F32) r = float_lit(n.fconst);
        else if (n.rk == RK_BOOL) r = n.fconst != 0 ? "true" : "false";
        else r = fmt("%lld%s", (long long)n.fconst, n.rk == RK_I64 ? "LL" : "");
      } else if (n.opcode == DISC_DIM_SIZE) {
        if (n.rk == RK_F32) r = fmt("A.dimf%d", g.dim_index(n.sym_dim));
        else r = fmt("(%s)A.dimi%d", reg_ctype(n.rk), g.dim_index(n.sym_dim));
      } else if (n.dom == DOM_ROW && !row_local) {
        r = fmt("rc.r%d", id);
      } else if (n.opcode == DISC_PARAM) {
        const Access& a = g.an.accesses[n.access];
        if (n.dom == DOM_ELEM) r = from_storage(fmt("s.a%d.v[e]", n.access), a.dtype);
        else r = fmt("rc.r%d", id);   // loaded by row_begin
      } else if (g.is_reduce(n.opcode)) {
        r = fmt("rc.r%d", id);
      } else {
        r = fmt("t%d", id);
        const std::string rhs = expr(n);   // emits the operands first
        body << "    const " << reg_ctype(n.rk) << " " << r << " = " << rhs << ";\n";
      }
      names[id] = r;
      return r;
    }
    std::string as(int id, RegKind k) { return convert(val(id), g.an.nodes[id].rk, k); }
    std::string expr(const Node& n) {
      const RegKind k = n.rk;
      auto a = [&](int i) { return as(n.in[i], k); };
      switch (n.opcode) {
        case DISC_NEG: return "-" + a(0);
        case DISC_ABS: return k == RK_F32 ? "fabsf(" + a(0) + ")" : "(" + a(0) + " < 0 ? -" + a(0) + " : " + a(0) + ")";
        case DISC_EXP: return "expf(" + a(0) + ")";
        case DISC_LOG: return "logf(" + a(0) + ")";
        case DISC_TANH: return "tanhf(" + a(0) + ")";
        case DISC_SQRT: return "sqrtf(" + a(0) + ")";
        case DISC_RSQRT: return "rsqrtf(" + a(0) + ")";
        case DISC_RCP: return "(1.0f / " + a(0) + ")";
        case DISC_SIGMOID: return "(1.0f / (1.0f + expf(-" + a(0) + ")))";
        case DISC_ERF: return "erff(" + a(0) + ")";
        case DISC_ADD: return a(0) + " + " + a(1);
        case DISC_SUB: return a(0) + " - " + a(1);
        case DISC_MUL: return a(0) + " * " + a(1);
        case DISC_DIV: return a(0) + " / " + a(1);
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
        case DISC_SELECT: return as(n.in[0], RK_BOOL) + " ? " + a(1) + " : " + a(2);
        case DISC_CAST: return a(0);   // float->int conversion truncates toward zero in C
        default: return "0 /* unexpected opcode */";
      }
    }
  };

  std::string row_fields() {
    std::ostringstream o;
    for (size_t i = 0; i < an.accesses.size(); ++i) {
      const Access& a = an.accesses[i];
      if (a.has_inner && (a.kind == ACC_FULL || a.kind == ACC_PARTIAL)) o << "    disc::i64 b" << i << ";\n";
      if (!a.has_inner && a.is_output && a.kind == ACC_PARTIAL) o << "    disc::i64 b" << i << ";\n";
    }
    for (size_t i = 0; i < an.nodes.size(); ++i) {
      const Node& n = an.nodes[i];
      if (n.dom == DOM_ROW) o << "    " << reg_ctype(n.rk) << " r" << i << ";\n";
    }
    o << "    int unused_;\n";
    return o.str();
  }

  // offset expression of a per-row (no inner) access for row `row`
  std::string perrow_offset(const Access& a, size_t idx) {
    switch (a.kind) {
      case ACC_PERROW: return "row";
      case ACC_SCALAR: return "0";
      default: return fmt("pb%zu", idx);
    }
  }

  void emit_row_begin() {
    os << "  static DISC_DEV void row_begin(const Args& A, disc::i64 row, RowCtx& rc) {\n";
    const int n_outer = an.inner_group;
    if (an.needs_decomp) {
      os << "    disc::i64 ig[4] = {0, 0, 0, 0};\n";
      os << "    if (A.rows < 2147483648LL) {\n      disc::u32 t = (disc::u32)row;\n";
      for (int g = n_outer - 1; g >= 1; --g)
        os << fmt("      { disc::u32 q = disc::fdiv(t, A.gd%d); ig[%d] = t - q * A.gd%d.d; t = q; }\n", g, g, g);
      os << "      ig[0] = t;\n    } else {\n      disc::i64 t = row;\n";
      for (int g = n_outer - 1; g >= 1; --g)
        os << fmt("      { disc::i64 q = t / A.gs%d; ig[%d] = t - q * A.gs%d; t = q; }\n", g, g, g);
      os << "      ig[0] = t;\n    }\n";
    }
    for (size_t i = 0; i < an.accesses.size(); ++i) {
      const Access& a = an.accesses[i];
      if (a.kind == ACC_PARTIAL) {
        std::string e;
        size_t sp = 0;
        for (size_t t = 0; t < a.groups.size(); ++t) {
          if (a.groups[t] == an.inner_group) continue;
          if (!e.empty()) e += " + ";
          e += fmt("ig[%d] * A.st%d", a.groups[t], a.stride_prod[sp++]);
        }
        if (a.has_inner || a.is_output) os << "    rc.b" << i << " = " << e << ";\n";
        else os << "    const disc::i64 pb" << i << " = " << e << ";\n";
      } else if (a.kind == ACC_FULL && a.has_inner) {
        os << "    rc.b" << i << " = row * A.inner;\n";
      }
    }
    Fn fn(*this, false, true);
    for (size_t i = 0; i < an.nodes.size(); ++i) {
      const Node& n = an.nodes[i];
      if (n.dom != DOM_ROW || n.phase != 0) continue;
      if (n.opcode == DISC_PARAM) {
        const Access& a = an.accesses[n.access];
        std::string off = perrow_offset(a, n.access);
        fn.body << "    rc.r" << i << " = " << from_storage(fmt("A.p%d[%s]", a.slot, off.c_str()), a.dtype) << ";\n";
        fn.names[(int)i] = fmt("rc.r%zu", i);
      } else {
        std::string v = fn.val((int)i);
        fn.body << "    rc.r" << i << " = " << v << ";\n";
        fn.names[(int)i] = fmt("rc.r%zu", i);
      }
    }
    os << fn.body.str();
    os << "    (void)A; (void)row; (void)rc;\n  }\n";
  }

  void emit_slots() {
    os << "  template <int V> struct Slot {\n";
    for (size_t i = 0; i < an.accesses.size(); ++i) {
      const Access& a = an.accesses[i];
      if (!a.is_output && a.has_inner) os << "    disc::Vec<" << dtype_ctype(a.dtype) << ", V> a" << i << ";\n";
    }
    os << "    int unused_;\n  };\n";
    os << "  template <int V> struct OutSlot {\n";
    for (size_t i = 0; i < an.accesses.size(); ++i) {
      const Access& a = an.accesses[i];
      if (a.is_output && a.has_inner) os << "    disc::Vec<" << dtype_ctype(a.dtype) << ", V> o" << a.slot << ";\n";
    }
    os << "    int unused_;\n  };\n";
  }

  std::string elem_base(const Access& a, size_t i) {
    if (a.kind == ACC_ROWVEC) return "col";
    return fmt("rc.b%zu + col", i);
  }

  void emit_load_store() {
    os << "  template <int V, class C> static DISC_DEV void load(const Args& A, const RowCtx& rc, C col, int nvalid, Slot<V>& s) {\n";
    for (size_t i = 0; i < an.accesses.size(); ++i) {
      const Access& a = an.accesses[i];
      if (a.is_output || !a.has_inner) continue;
      os << "    disc::ld(s.a" << i << ", A.p" << a.slot << ", " << elem_base(a, i) << ", nvalid);\n";
    }
    os << "    (void)A; (void)rc; (void)col; (void)nvalid; (void)s;\n  }\n";
    os << "  template <int V, class C> static DISC_DEV void store(const Args& A, const RowCtx& rc, C col, int nvalid, const OutSlot<V>& o) {\n";
    for (size_t i = 0; i < an.accesses.size(); ++i) {
      const Access& a = an.accesses[i];
      if (!a.is_output || !a.has_inner) continue;
      os << "    disc::st(A.o" << a.slot << ", " << elem_base(a, i) << ", o.o" << a.slot << ", nvalid);\n";
    }
    os << "    (void)A; (void)rc; (void)col; (void)nvalid; (void)o;\n  }\n";
  }

  // accumulator field names of reduce `slot` in a phase
  static std::string accf(int slot) { return fmt("f%d", slot); }
  static std::string acci(int slot) { return fmt("i%d", slot); }

  void emit_acc_types() {
    int max_bytes = 8;
    for (int p = 0; p < an.n_phases; ++p) {
      os << "struct PatAcc" << p << " {\n";
      int bytes = 0;
      for (int id : an.reduces[p]) {
        const Node& n = an.nodes[id];
        RegKind ok = an.nodes[n.in[0]].rk;
        os << "  " << reg_ctype(ok) << " " << accf(n.reduce_slot) << ";\n";
        bytes += ok == RK_I64 ? 8 : 4;
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
  int acc_bytes = 8;

  std::string identity(const Node& n) {
    RegKind ok = an.nodes[n.in[0]].rk;
    switch (n.opcode) {
      case DISC_REDUCE_SUM: return ok == RK_F32 ? "0.0f" : "0";
      case DISC_REDUCE_MIN: return ok == RK_F32 ? "__builtin_inff()" : ok == RK_I64 ? "9223372036854775807LL" : "2147483647";
      default: return ok == RK_F32 ? "(-__builtin_inff())" : ok == RK_I64 ? "(-9223372036854775807LL - 1)" : "(-2147483647 - 1)";
    }
  }

  void emit_acc_fns() {
    // init
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
    // merge
    os << "  template <int P> static DISC_DEV void acc_merge(Acc<P>& a, const Acc<P>& b) {\n";
    for (int p = 0; p < an.n_phases; ++p) {
      os << "    if constexpr (P == " << p << ") {\n";
      for (int id : an.reduces[p]) {
        const Node& n = an.nodes[id];
        RegKind ok = an.nodes[n.in[0]].rk;
        std::string f = accf(n.reduce_slot), i = acci(n.reduce_slot);
        switch (n.opcode) {
          case DISC_REDUCE_SUM: os << "      a." << f << " += b." << f << ";\n"; break;
          case DISC_REDUCE_MAX:
            if (ok == RK_F32) os << "      a." << f << " = fmaxf(a." << f << ", b." << f << ");\n";
            else os << "      a." << f << " = a." << f << " > b." << f << " ? a." << f << " : b." << f << ";\n";
            break;
          case DISC_REDUCE_MIN:
            if (ok == RK_F32) os << "      a." << f << " = fminf(a." << f << ", b." << f << ");\n";
            else os << "      a." << f << " = a." << f << " < b." << f << " ? a." << f << " : b." << f << ";\n";
            break;
          default:
            os << "      if (b." << f << " > a." << f << " || (b." << f << " == a." << f << " && b." << i << " < a." << i
               << ")) { a." << f << " = b." << f << "; a." << i << " = b." << i << "; }\n";
        }
      }
      os << "    }\n";
    }
    os << "    (void)a; (void)b;\n  }\n";
    // shuffle
    os << "  template <int P> static DISC_DEV void acc_shfl(Acc<P>& a, int m) {\n";
    for (int p = 0; p < an.n_phases; ++p) {
      os << "    if constexpr (P == " << p << ") {\n";
      for (int id : an.reduces[p]) {
        const Node& n = an.nodes[id];
        os << "      a." << accf(n.reduce_slot) << " = disc::shfl_xor(a." << accf(n.reduce_slot) << ", m);\n";
        if (n.opcode == DISC_REDUCE_ARGMAX)
          os << "      a." << acci(n.reduce_slot) << " = disc::shfl_xor(a." << acci(n.reduce_slot) << ", m);\n";
      }
      os << "    }\n";
    }
    os << "    (void)a; (void)m;\n  }\n";
    // accumulate one element
    os << "  template <int P, int V> static DISC_DEV void accum(const Args& A, Acc<P>& acc, const Slot<V>& s, int e, int col, const RowCtx& rc) {\n";
    for (int p = 0; p < an.n_phases; ++p) {
      os << "    if constexpr (P == " << p << ") {\n";
      Fn fn(*this, true, false);
      std::ostringstream tail;
      for (int id : an.reduces[p]) {
        const Node& n = an.nodes[id];
        RegKind ok = an.nodes[n.in[0]].rk;
        std::string x = fn.val(n.in[0]);
        std::string f = "acc." + accf(n.reduce_slot), i = "acc." + acci(n.reduce_slot);
        switch (n.opcode) {
          case DISC_REDUCE_SUM: tail << "    " << f << " += " << x << ";\n"; break;
          case DISC_REDUCE_MAX:
            if (ok == RK_F32) tail << "    " << f << " = fmaxf(" << f << ", " << x << ");\n";
            else tail << "    " << f << " = " << f << " > " << x << " ? " << f << " : " << x << ";\n";
            break;
          case DISC_REDUCE_MIN:
            if (ok == RK_F32) tail << "    " << f << " = fminf(" << f << ", " << x << ");\n";
            else tail << "    " << f << " = " << f << " < " << x << " ? " << f << " : " << x << ";\n";
            break;
          default:
            tail << "    if (" << x << " > " << f << ") { " << f << " = " << x << "; " << i << " = col; }\n";
        }
      }
      os << fn.body.str() << tail.str() << "    }\n";
    }
    os << "    (void)A; (void)acc; (void)s; (void)e; (void)col; (void)rc;\n  }\n";
    // per-row values known after phase P
    os << "  template <int P> static DISC_DEV void row_after(const Args& A, RowCtx& rc, const Acc<P>& acc) {\n";
    for (int p = 0; p < an.n_phases; ++p) {
      os << "    if constexpr (P == " << p << ") {\n";
      Fn fn(*this, false, true);
      for (int id : an.reduces[p]) {
        const Node& n = an.nodes[id];
        RegKind ok = an.nodes[n.in[0]].rk;
        std::string src = n.opcode == DISC_REDUCE_ARGMAX ? "acc." + acci(n.reduce_slot) : "acc." + accf(n.reduce_slot);
        RegKind sk = n.opcode == DISC_REDUCE_ARGMAX ? RK_I32 : ok;
        fn.body << "    rc.r" << id << " = " << convert(src, sk, n.rk) << ";\n";
      }
      // earlier per-row values are read back from rc
      for (size_t i = 0; i < an.nodes.size(); ++i) {
        const Node& n = an.nodes[i];
        if (n.dom != DOM_ROW) continue;
        if (n.phase <= p || is_reduce(n.opcode)) fn.names[(int)i] = fmt("rc.r%zu", i);
      }
      for (size_t i = 0; i < an.nodes.size(); ++i) {
        const Node& n = an.nodes[i];
        if (n.dom != DOM_ROW || n.phase != p + 1 || is_reduce(n.opcode)) continue;
        std::string v = fn.val((int)i);
        fn.body << "    rc.r" << i << " = " << v << ";\n";
        fn.names[(int)i] = fmt("rc.r%zu", i);
      }
      os << fn.body.str() << "    }\n";
    }
    os << "    (void)A; (void)rc; (void)acc;\n  }\n";
  }

  void emit_epilogue() {
    os << "  template <int V, class C> static DISC_DEV void epilogue(const Args& A, const RowCtx& rc, const Slot<V>& s, C col, OutSlot<V>& o) {\n";
    os << "#pragma unroll\n    for (int e = 0; e < V; ++e) {\n";
    Fn fn(*this, true, false);
    std::ostringstream tail;
    for (const auto& out : an.outputs) {
      const Access& a = an.accesses[out.access];
      if (!a.has_inner) continue;
      const Node& n = an.nodes[out.node];
      tail << "    o.o" << a.slot << ".v[e] = " << to_storage(fn.val(out.node), n.rk, a.dtype) << ";\n";
    }
    os << fn.body.str() << tail.str();
    os << "    }\n    (void)A; (void)rc; (void)s; (void)col; (void)o;\n  }\n";
    os << "  static DISC_DEV void row_store(const Args& A, disc::i64 row, const RowCtx& rc) {\n";
    for (const auto& out : an.outputs) {
      const Access& a = an.accesses[out.access];
      if (a.has_inner) continue;
      const Node& n = an.nodes[out.node];
      std::string off = a.kind == ACC_PERROW ? "row" : a.kind == ACC_SCALAR ? "0" : fmt("rc.b%d", out.access);
      Fn fn2(*this, false, false);
      os << "    A.o" << a.slot << "[" << off << "] = " << to_storage(fn2.val(out.node), n.rk, a.dtype) << ";\n";
    }
    os << "    (void)A; (void)row; (void)rc;\n  }\n";
  }

  void emit_args() {
    os << "  struct Args {\n";
    for (const auto& f : layout.fields) os << "    " << field_decl(f) << "\n";
    os << "  };\n";
  }

  void emit_kernels(Generated* out) {
    const int V = an.vec_width;
    auto k = [&](const std::string& name, const std::string& body, bool rowplan) {
      os << "extern \"C\" __global__ void __launch_bounds__(256) " << name << "(Pat::Args A"
         << (rowplan ? ", disc::RowPlan rp" : "") << ") { " << body << " }\n";
      out->kernels.push_back(name);
    };
    if (an.tmpl == DISC_TEMPLATE_LOOP) {
      k("k_loop_vec", fmt("disc::kloop_body<Pat, %d, 4, false>(A);", V), false);
      k("k_loop_vec_i64", fmt("disc::kloop_body<Pat, %d, 1, true>(A);", V), false);
      k("k_loop_scalar", "disc::kloop_body<Pat, 1, 4, false>(A);", false);
      k("k_loop_scalar_i64", "disc::kloop_body<Pat, 1, 1, true>(A);", false);
    } else if (an.tmpl == DISC_TEMPLATE_ROW_REDUCE) {
      for (int nv : {1, 2, 4, 8}) {
        k(fmt("k_row_vec_nv%d", nv), fmt("disc::row_reg_body<Pat, %d, %d>(A, rp);", V, nv), true);
        k(fmt("k_row_scalar_nv%d", nv), fmt("disc::row_reg_body<Pat, 1, %d>(A, rp);", nv), true);
      }
      k("k_row_stream_vec", fmt("disc::row_stream_body<Pat, %d>(A);", V), false);
      k("k_row_stream_scalar", "disc::row_stream_body<Pat, 1>(A);", false);
    }
  }

  int run(Generated* out, std::string* err) {
    if (an.tmpl == DISC_TEMPLATE_COL_REDUCE) {
      *err = "column-reduction code generation is not available in this build";
      return DISC_ERR_UNFUSIBLE;
    }
    build_layout();
    os << "// generated: one fused pattern, every kernel version\n";
    emit_acc_types();
    os << "struct Pat {\n";
    os << "  static constexpr int NPHASE = " << an.n_phases << ";\n";
    os << "  static constexpr int MAX_ACC_BYTES = " << acc_bytes << ";\n";
    os << "  template <int P> using Acc = typename PatAccSel<P>::type;\n";
    emit_args();
    os << "  struct RowCtx {\n" << row_fields() << "  };\n";
    emit_slots();
    emit_row_begin();
    emit_load_store();
    emit_acc_fns();
    emit_epilogue();
    os << "};\n";
    os << "static_assert(sizeof(Pat::Args) == " << layout.size << ", \"argument block layout\");\n";
    for (const auto& f : layout.fields)
      os << "static_assert(__builtin_offsetof(Pat::Args, " << field_name(f) << ") == " << f.offset << ", \"argument block layout\");\n";
    emit_kernels(out);
    out->source = os.str();
    out->args = layout;
    return DISC_OK;
  }
};

}  // namespace

int generate(const Analysis& an, Generated* out, std::string* err) {
  Gen g(an);
  return g.run(out, err);
}

}  // namespace disc

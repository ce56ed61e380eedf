// Context, pattern cache, the one device compile per pattern, and the launch path.
//
// The launch path is the "generated runtime flow" of the paper (Section 4.2) in the form of a
// closure specialised at registration: shape calculation from the runtime dims, the check of
// the registered equalities, version and launch-dimension selection (Section 4.3), filling of
// the kernel-argument block, one enqueue.  It walks recipes made of a handful of integer
// products and comparisons; the op list of the pattern is never visited at launch time.
#include <hip/hip_runtime_api.h>
#include <hip/hiprtc.h>

#include <chrono>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <memory>
#include <numeric>
#include <set>
#include <sstream>

#include "disc_internal.hpp"

namespace disc {

extern const char* const kDeviceHeader;   // disc_device.h, embedded at build time

namespace {

struct DeviceRowPlan {   // mirrors disc::RowPlan of the device header
  int32_t G, log2G, nv, flags, rpb;
};
struct DeviceColPlan {   // mirrors disc::ColPlan of the device header
  int32_t GC, log2GC, nchunk, pad;
  int64_t chunk_rows, outer, epi_rows;
};
constexpr int kLdsStep = 512, kLdsSteps = 48 * 1024 / kLdsStep + 2;
constexpr int kArgBufBytes = 4096;    // kernel-argument block + launch-plan struct
constexpr int kMaxShapeValues = 64;   // strides + base offsets + padding windows of one pattern
struct FastDivHost {
  uint32_t d, m, s, pad;
};

FastDivHost make_fastdiv(uint64_t d) {
  FastDivHost f{1, 1, 0, 0};
  if (d == 0 || d > 0x7fffffffull) { f.d = (uint32_t)(d > 0xffffffffull ? 0xffffffffu : d); return f; }
  uint32_t s = 0;
  while ((1ull << s) < d) ++s;
  f.d = (uint32_t)d;
  f.s = s;
  f.m = (uint32_t)((((1ull << s) - d) << 32) / d + 1);
  return f;
}

struct Pattern {
  Analysis an;
  Generated gen;
  std::string key;
  int compile_events = 0;
  double compile_ms = 0;
  hipModule_t module = nullptr;
  // Launch-time tables, indexed by kernel number: nothing on the launch path looks up a name.
  hipFunction_t fn[K_COUNT] = {};
  // blocks resident per CU by (kernel, block-size class, dynamic LDS in steps of kLdsStep bytes),
  // asked from the runtime on first use (0 = not asked yet)
  mutable int16_t resident[K_COUNT][3][kLdsSteps] = {};
  bool is_static = false;                             // module specialised for static_dims only
  std::vector<int64_t> static_dims;
  // constraint recipes
  std::vector<std::pair<int, int>> eq_checks;         // symbolic dims that must be equal
  std::vector<std::pair<int, int64_t>> static_checks; // symbolic dim that must equal a static size
  std::vector<int> class_of_dim;
  int n_classes = 0;
  // element count recipes for algorithmic bytes
  std::vector<std::pair<DimProduct, int>> io_numel;   // (numel product, bytes per element)
};

struct ShapeVals {
  int64_t group[4] = {1, 1, 1, 1};
  int64_t rows = 1, inner = 1, mid = 0;
  int64_t products[kMaxShapeValues];   // strides, base offsets, padding windows (no allocation at launch)
  int64_t alg_bytes = 0;
};

bool mul_ovf(int64_t a, int64_t b, int64_t* r) { return __builtin_mul_overflow(a, b, r); }

bool eval_product(const DimProduct& p, const int64_t* dims, int64_t* out) {
  int64_t v = p.stat;
  for (int s : p.sym)
    if (mul_ovf(v, dims[s], &v)) return false;
  *out = v;
  return true;
}

int64_t now_ns() {
  return std::chrono::duration_cast<std::chrono::nanoseconds>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

}  // namespace
}  // namespace disc

using namespace disc;

// ---- op graphs larger than one fusion pattern (Section 4.3, fusion decision over a graph) -------
struct GraphGroup {
  std::vector<int> ops;          // graph op ids fused into this pattern, in graph order
  int pattern_id = -1;
  std::vector<int> in_values;    // graph value ids bound to the pattern's PARAMs, in order
  std::vector<int> out_values;   // graph value ids produced by the pattern's OUTPUTs, in order
  // where each of those values lives at launch, resolved at registration: (kind, index) with kind
  // 0 = graph input, 1 = graph output, 2 = planned buffer
  std::vector<std::pair<int, int>> in_place, out_place;
};
struct GraphIntermediate {
  int value = -1;                // produced by group `first`, last read by group `last`
  int first = 0, last = 0;
  int buffer = -1;
};
struct Graph {
  std::vector<disc_op> ops;
  std::vector<disc_constraint> cs;
  std::vector<int> group_of_op;  // -1 for leaves and OUTPUT ops
  std::vector<char> remat;       // value is recomputed by the patterns that read it instead of crossing a cut
  std::vector<char> needed;      // some graph output depends on the op (the others are dead code)
  std::vector<GraphGroup> groups;
  std::vector<GraphIntermediate> inter;
  std::map<int, int> inter_of_value;
  std::vector<int> buffer_value;         // a value whose size every tenant of the buffer shares
  std::map<int, int> param_index;        // PARAM op id -> input index
  std::map<int, int> output_index;       // value id -> output index (graph OUTPUT ops)
  int n_sym = 0, n_inputs = 0, n_outputs = 0;
};

struct disc_ctx {
  std::vector<std::unique_ptr<Graph>> graphs;
  int device = -1;
  int n_cus = 256;
  std::string err;
  std::vector<std::unique_ptr<Pattern>> patterns;
  std::map<std::string, int> cache;
  disc_stats_t stats{};
  int force_variant = -1;
  hipModule_t util_module = nullptr;
  hipFunction_t util_copy = nullptr, util_copy_nt = nullptr, util_empty = nullptr;
  hipFunction_t util_mix[2][2][4] = {};   // [kind][non-temporal][log2 slots in flight]
  // test overrides (disc_test_option); the defaults are the host rules
  int row_nt = -1;           // non-temporal versions: -1 = host rule, 0 = never, 1 = wherever the version exists
  int row_rounds = 0;        // row kernels: grid = this many rounds of resident blocks (0: host rule)
  int row_stage = 1;         // 0: row vectors are never staged in LDS
  int row_shift = 1;         // 0: vector slots of ragged rows are never shifted to the tensor's 16-byte boundaries
};
constexpr int kGridMult = 8;     // loop / column kernels: grid capped at this many blocks per CU
constexpr int kLoopUnroll = 4;   // loop kernels: slots in flight per lane

namespace {

int set_err(disc_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg;
  return code;
}

int hip_fail(disc_ctx* c, hipError_t e, const char* what) {
  return set_err(c, DISC_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

int compile_source(disc_ctx* c, const std::string& src, std::vector<char>* code, double* ms) {
  hiprtcProgram prog;
  if (hiprtcCreateProgram(&prog, src.c_str(), "disc_pattern.hip", 0, nullptr, nullptr) != HIPRTC_SUCCESS)
    return set_err(c, DISC_ERR_COMPILE, "hiprtcCreateProgram failed");
  std::vector<const char*> opts = {"--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                                   "-packed-fp32-ops", "-Wno-unused-value",
                                   // the fused expressions are scalar per element on purpose: no packed-fp32 pairs
                                   "-fno-slp-vectorize", "-fno-vectorize"};
  auto t0 = std::chrono::steady_clock::now();
  hiprtcResult r = hiprtcCompileProgram(prog, (int)opts.size(), opts.data());
  *ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
  if (r != HIPRTC_SUCCESS) {
    size_t n = 0;
    hiprtcGetProgramLogSize(prog, &n);
    std::string log(n, '\0');
    if (n) hiprtcGetProgramLog(prog, &log[0]);
    hiprtcDestroyProgram(&prog);
    return set_err(c, DISC_ERR_COMPILE, "device compile failed:\n" + log);
  }
  size_t n = 0;
  hiprtcGetCodeSize(prog, &n);
  code->resize(n);
  hiprtcGetCode(prog, code->data());
  hiprtcDestroyProgram(&prog);
  return DISC_OK;
}

Pattern* get_pattern(disc_ctx* c, int32_t id) {
  if (!c || id < 0 || id >= (int)c->patterns.size()) return nullptr;
  return c->patterns[id].get();
}

// ---- shape calculation (host) -------------------------------------------------------------
int shape_calc(disc_ctx* c, const Pattern& p, const int64_t* dims, int n_dims, ShapeVals* sv) {
  if (!dims && p.an.n_sym > 0) return set_err(c, DISC_ERR_INVALID_ARG, "dims is null");
  if (n_dims != p.an.n_sym) {
    char buf[96];
    snprintf(buf, sizeof buf, "pattern has %d symbolic dims, %d given", p.an.n_sym, n_dims);
    return set_err(c, DISC_ERR_INVALID_ARG, buf);
  }
  for (int i = 0; i < n_dims; ++i)
    if (dims[i] < 0) return set_err(c, DISC_ERR_SHAPE, "negative dimension");
  char buf[160];
  for (const auto& e : p.eq_checks)
    if (dims[e.first] != dims[e.second]) {
      snprintf(buf, sizeof buf, "dims[%d] = %lld and dims[%d] = %lld were registered as equal", e.first,
               (long long)dims[e.first], e.second, (long long)dims[e.second]);
      return set_err(c, DISC_ERR_CONSTRAINT, buf);
    }
  for (const auto& e : p.static_checks)
    if (dims[e.first] != e.second) {
      snprintf(buf, sizeof buf, "dims[%d] = %lld must equal the static size %lld", e.first, (long long)dims[e.first],
               (long long)e.second);
      return set_err(c, DISC_ERR_CONSTRAINT, buf);
    }
  const Analysis& an = p.an;
  const int ng = (int)an.groups.size();
  int64_t total = 1;
  for (int g = 0; g < ng; ++g) {
    if (!eval_product(an.group_size[g], dims, &sv->group[g]) || mul_ovf(total, sv->group[g], &total))
      return set_err(c, DISC_ERR_SHAPE, "element count overflows int64");
  }
  for (const auto& nc : an.numel_checks) {
    int64_t n = 0;
    if (!eval_product(nc.second, dims, &n)) return set_err(c, DISC_ERR_SHAPE, "element count overflows int64");
    if (n != total) {
      snprintf(buf, sizeof buf, "op %d has %lld elements, the iteration space %lld: they were registered as equal in size",
               nc.first, (long long)n, (long long)total);
      return set_err(c, DISC_ERR_CONSTRAINT, buf);
    }
  }
  sv->inner = sv->group[an.inner_group];
  sv->rows = 1;
  for (int g = 0; g < an.inner_group; ++g) sv->rows *= sv->group[g];
  sv->mid = an.mid_group >= 0 ? sv->group[an.mid_group] : 0;
  for (size_t i = 0; i < an.products.size(); ++i)
    if (!eval_product(an.products[i], dims, &sv->products[i]))
      return set_err(c, DISC_ERR_SHAPE, "stride overflows int64");
  // sliced operands (Section 4.1: slice starts are runtime values): bounds, then base offsets
  auto dim_val = [&](int32_t d) { return d >= 0 ? dims[d] : -(int64_t)d; };
  auto start_val = [&](int32_t s) { return s >= 0 ? dims[s] : (int64_t)(-1 - s); };
  for (const auto& sc : an.slice_checks) {
    const int64_t st = start_val(sc.start), n = dim_val(sc.size_dim), ext = dim_val(sc.src_dim);
    if (st < 0 || n > ext || st > ext - n) {
      snprintf(buf, sizeof buf, "op %d (%s), axis %d: [%lld, %lld) does not fit the extent %lld", sc.op,
               an.ops[sc.op].opcode == DISC_PAD ? "pad" : "slice", sc.axis, (long long)st, (long long)(st + n), (long long)ext);
      return set_err(c, DISC_ERR_SHAPE, buf);
    }
  }
  for (size_t i = 0; i < an.offsets.size(); ++i) {
    int64_t sum = 0;
    for (const auto& t : an.offsets[i].terms) {
      int64_t stride = 0, term = 0;
      if (!eval_product(t.second, dims, &stride) || mul_ovf(stride, start_val(t.first), &term) ||
          __builtin_add_overflow(sum, term, &sum))
        return set_err(c, DISC_ERR_SHAPE, "slice offset overflows int64");
    }
    sv->products[an.products.size() + i] = sum;
  }
  for (size_t i = 0; i < an.windows.size(); ++i) {
    const WindowRecipe& w = an.windows[i];
    int64_t inner = 0, lo = 0, hi = 0;
    if (!eval_product(w.inner_sizes, dims, &inner) || mul_ovf(start_val(w.low), inner, &lo) ||
        mul_ovf(start_val(w.low) + dim_val(w.extent_dim), inner, &hi))
      return set_err(c, DISC_ERR_SHAPE, "padding window overflows int64");
    sv->products[an.products.size() + an.offsets.size() + 2 * i] = lo;
    sv->products[an.products.size() + an.offsets.size() + 2 * i + 1] = hi;
  }
  sv->alg_bytes = 0;
  for (const auto& io : p.io_numel) {
    int64_t n = 0;
    if (!eval_product(io.first, dims, &n) || mul_ovf(n, io.second, &n))
      return set_err(c, DISC_ERR_SHAPE, "tensor size overflows int64");
    sv->alg_bytes += n;
  }
  return DISC_OK;
}

int ilog2_ceil(int64_t v) {
  int l = 0;
  while ((1ll << l) < v) ++l;
  return l;
}

struct LaunchRec {
  int kid = -1;              // KernelId
  uint32_t grid[3] = {1, 1, 1};
  uint32_t block = 256;
  int plan_kind = 0;         // 0 none, 1 RowPlan, 2 ColPlan
  uint32_t dyn_lds = 0;      // dynamic LDS bytes
  DeviceRowPlan rp{};
  DeviceColPlan cp{};
};

struct FullPlan {
  disc_plan_t pub{};
  ShapeVals sv;
  LaunchRec launches[3];
  int64_t nslots = 0, spr = 0;
  int64_t aux[4] = {0, 0, 0, 0};
  size_t ws_off[2] = {0, 0};
};

// Loop-fusion launch geometry for an iteration space [rows, inner]; shared by loop patterns and
// by the epilogue stage of column reduces.  want_vec / want_i64: -1 = let the shape decide.
// Launches that move less than this may be read back from the memory-side cache (256 MB) by
// whatever kernel consumes the result; the non-temporal versions are kept for larger ones, which
// stream through the caches anyway.
constexpr int64_t kNonTemporalMinBytes = 64ll << 20;

// nt_name: the non-temporal sibling of names[0] (vector width, 32-bit index), taken for large
// launches (`big`) whose rows start on 16-byte boundaries (`aligned`: the full-size operands are;
// inner a multiple of the width).
int plan_loop(disc_ctx* c, int64_t rows, int64_t inner, int V, int want_vec, int want_i64, const int names[4],
              int nt_name, bool aligned, bool big, FullPlan* fp, LaunchRec* L, bool* vec_out, bool* i64_out) {
  bool vec;
  {
    const int64_t spr_v = (inner + V - 1) / V;
    const double waste = 1.0 - (double)inner / (double)(spr_v * V);
    vec = waste <= 0.25;
  }
  if (want_vec >= 0) vec = want_vec != 0;
  const int v = vec ? V : 1;
  int64_t spr = (inner + v - 1) / v, nslots;
  if (mul_ovf(spr, rows, &nslots)) return set_err(c, DISC_ERR_SHAPE, "slot count overflows int64");
  bool i64 = nslots >= (1ll << 31) - (1ll << 24) || inner >= (1ll << 31) - 16 || rows >= (1ll << 31);
  if (want_i64 == 1) i64 = true;
  else if (want_i64 == 0 && i64) return set_err(c, DISC_ERR_INVALID_ARG, "forced 32-bit version cannot index this shape");
  const int U = i64 ? 1 : kLoopUnroll;
  const int64_t max_grid = (int64_t)c->n_cus * kGridMult;
  int64_t blocks = (nslots + 256ll * U - 1) / (256ll * U);
  blocks = std::min(blocks, i64 ? max_grid * 4 : max_grid);
  L->kid = names[(vec ? 0 : 2) + (i64 ? 1 : 0)];
  if (nt_name >= 0 && vec && v > 1 && !i64 && aligned && inner % v == 0 && c->row_nt != 0 &&
      (c->row_nt > 0 || big))
    L->kid = nt_name;
  L->grid[0] = (uint32_t)blocks;
  L->block = 256;
  fp->nslots = nslots;
  fp->spr = spr;
  fp->pub.index_bits = i64 ? 64 : 32;
  fp->pub.vec_width = v;
  fp->pub.slots_per_lane = U;
  *vec_out = vec;
  *i64_out = i64;
  return DISC_OK;
}

// Blocks of a kernel that one CU holds at a given block size and dynamic LDS size, as the
// runtime computes it from the compiled kernel's register and LDS use (asked once per
// combination).  Without a device: an estimate from a 16-wavefront budget.
int resident_blocks(const disc_ctx* c, const Pattern& p, int kid, uint32_t block, uint32_t dyn_lds);

// ---- version + launch-dimension selection (host) ---------------------------------------------
int make_plan(disc_ctx* c, const Pattern& p, const int64_t* dims, int n_dims, int force, const void* const* inputs,
              void* const* outputs, FullPlan* fp) {
  // pointer values: wide accesses need element alignment only; the non-temporal row versions are
  // picked for 16-byte aligned full-size operands (null arrays: assumed aligned)
  if (p.is_static) {
    if (force >= 0) return set_err(c, DISC_ERR_INVALID_ARG, "a single-shape pattern has one kernel version");
    if (n_dims != (int)p.static_dims.size() || !std::equal(dims, dims + n_dims, p.static_dims.begin()))
      return set_err(c, DISC_ERR_SHAPE, "pattern was compiled for one shape and is launched with another");
  }
  int rc = shape_calc(c, p, dims, n_dims, &fp->sv);
  if (rc) return rc;
  // every full-size operand on a 16-byte boundary (null pointer arrays: assumed)
  auto full_aligned = [&]() {
    for (const Access& a : p.an.accesses) {
      if (a.kind != ACC_FULL) continue;
      const void* ptr = a.is_output ? (outputs ? outputs[a.slot] : nullptr) : (inputs ? inputs[a.slot] : nullptr);
      if (reinterpret_cast<uintptr_t>(ptr) % 16 != 0) return false;
    }
    return true;
  };
  const Analysis& an = p.an;
  const ShapeVals& sv = fp->sv;
  disc_plan_t& pub = fp->pub;
  pub.rows = sv.rows;
  pub.inner = sv.inner;
  pub.mid = sv.mid;
  pub.algorithmic_bytes = sv.alg_bytes;
  pub.workspace_bytes = 0;
  pub.n_launches = 0;
  pub.variant = -1;
  const int V = an.vec_width;
  const int64_t max_grid = (int64_t)c->n_cus * kGridMult;

  if (an.tmpl == DISC_TEMPLATE_TRANSPOSE) {
    if (sv.rows == 0 || sv.inner == 0) return DISC_OK;
    if (force >= 0 && force != DISC_V_TRANSPOSE_TILE)
      return set_err(c, DISC_ERR_INVALID_ARG, "forced version does not belong to a transpose pattern");
    const int ng = (int)an.groups.size();
    const int64_t P = sv.group[ng - 2], Q = sv.group[ng - 1], batch = ng == 3 ? sv.group[0] : 1;
    // tiles of 256 bytes per row: 128 x 128 elements of one or two bytes, 64 x 64 wider ones
    const int64_t ts = dtype_bytes(an.accesses[0].dtype) <= 2 ? 128 : 64;
    const int64_t ntiles = batch * ((P + ts - 1) / ts) * ((Q + ts - 1) / ts);
    LaunchRec& L = fp->launches[0];
    L.kid = K_TRANSPOSE_TILE;
    L.block = 256;
    L.grid[0] = (uint32_t)std::min<int64_t>(ntiles, (int64_t)c->n_cus * 8);
    pub.variant = DISC_V_TRANSPOSE_TILE;
    pub.n_launches = 1;
    pub.vec_width = 1;
    pub.index_bits = 64;
  } else if (an.tmpl == DISC_TEMPLATE_COMPACT) {
    // count -> scan -> scatter over tiles of 256 lanes x kCompactSlots slots; the workspace holds one
    // 8-byte count / offset per tile.  An empty input still runs the scan launch: it stores the
    // count (zero) that the caller reads from device memory.
    if (force >= 0 && force != DISC_V_COMPACT_VEC && force != DISC_V_COMPACT_SCALAR)
      return set_err(c, DISC_ERR_INVALID_ARG, "forced version does not belong to a compaction pattern");
    constexpr int kCompactSlots = 4;   // (mirrors the device header)
    bool vec = V > 1;
    if (force >= 0) vec = force == DISC_V_COMPACT_VEC;
    const int v = vec ? V : 1;
    const int64_t tile = 256ll * kCompactSlots * v;
    const int64_t nb = (sv.inner + tile - 1) / tile;
    fp->aux[0] = nb;
    fp->ws_off[0] = 0;
    pub.workspace_bytes = (size_t)std::max<int64_t>(nb, 1) * 8;
    pub.variant = vec ? DISC_V_COMPACT_VEC : DISC_V_COMPACT_SCALAR;
    pub.vec_width = v;
    pub.index_bits = 64;
    pub.slots_per_lane = kCompactSlots;
    const uint32_t grid = (uint32_t)std::min<int64_t>(nb, max_grid * 4);
    int l = 0;
    if (nb > 0) {
      fp->launches[l].kid = vec ? K_COMPACT_COUNT_VEC : K_COMPACT_COUNT_SCALAR;
      fp->launches[l].grid[0] = grid;
      ++l;
    }
    fp->launches[l].kid = K_COMPACT_SCAN;
    fp->launches[l].block = 1024;
    fp->launches[l].grid[0] = 1;
    ++l;
    if (nb > 0) {
      fp->launches[l].kid = vec ? K_COMPACT_SCATTER_VEC : K_COMPACT_SCATTER_SCALAR;
      fp->launches[l].grid[0] = grid;
      ++l;
    }
    pub.n_launches = l;
  } else if (an.tmpl == DISC_TEMPLATE_LOOP) {
    if (sv.rows == 0 || sv.inner == 0) return DISC_OK;
    int want_vec = -1, want_i64 = -1;
    if (force >= 0) {
      if (force > DISC_V_LOOP_SCALAR_I64)
        return set_err(c, DISC_ERR_INVALID_ARG, "forced version does not belong to a loop-fusion pattern");
      want_vec = force == DISC_V_LOOP_VEC || force == DISC_V_LOOP_VEC_I64;
      want_i64 = force == DISC_V_LOOP_VEC_I64 || force == DISC_V_LOOP_SCALAR_I64;
    }
    static const int names[] = {K_LOOP_VEC, K_LOOP_VEC_I64, K_LOOP_SCALAR, K_LOOP_SCALAR_I64};
    bool vec, i64;
    rc = plan_loop(c, sv.rows, sv.inner, V, want_vec, want_i64, names, K_LOOP_VEC_NT, full_aligned(), sv.alg_bytes >= kNonTemporalMinBytes, fp, &fp->launches[0], &vec, &i64);
    if (rc) return rc;
    pub.variant = vec ? (i64 ? DISC_V_LOOP_VEC_I64 : DISC_V_LOOP_VEC) : (i64 ? DISC_V_LOOP_SCALAR_I64 : DISC_V_LOOP_SCALAR);
    pub.n_launches = 1;
  } else if (an.tmpl == DISC_TEMPLATE_ROW_REDUCE) {
    const int n_col_sums = p.gen.n_col_sums;   // outputs summed over the rows, carried along by the row kernels
    const int n_row_reds = p.gen.n_row_reds;   // per-row values reduced over the rows to one number each
    if (sv.rows == 0 && n_row_reds > 0) return set_err(c, DISC_ERR_EMPTY_REDUCE, "reduction over an axis of size 0");
    if (sv.rows == 0 && n_col_sums > 0 && sv.inner > 0)
      return set_err(c, DISC_ERR_EMPTY_REDUCE, "reduction over an axis of size 0");
    if (sv.rows == 0) return DISC_OK;
    if (sv.inner == 0 && an.n_phases == 0) return DISC_OK;   // (no reduction over the rows' axis: nothing to do)
    if (sv.inner == 0) return set_err(c, DISC_ERR_EMPTY_REDUCE, "reduction over an axis of size 0");
    if (sv.inner >= (1ll << 31) - 4096) return set_err(c, DISC_ERR_SHAPE, "row longer than 2^31 elements");
    bool vec = sv.inner >= V / 2 || V == 1;
    bool stream;
    if (force >= 0) {
      if (force < DISC_V_ROW_REG_VEC || force > DISC_V_ROW_STREAM_SCALAR)
        return set_err(c, DISC_ERR_INVALID_ARG, "forced version does not belong to a row-reduce pattern");
      vec = force == DISC_V_ROW_REG_VEC || force == DISC_V_ROW_STREAM_VEC;
    }
    const int v = vec ? V : 1;
    int64_t spr = (sv.inner + v - 1) / v;
    stream = spr > 1024 * (vec ? 3 : 2);
    if (force == DISC_V_ROW_STREAM_VEC || force == DISC_V_ROW_STREAM_SCALAR) stream = true;
    else if (force >= 0 && stream) return set_err(c, DISC_ERR_INVALID_ARG, "row too long for the forced register-resident version");
    pub.vec_width = v;
    pub.index_bits = 64;
    fp->spr = spr;
    fp->nslots = 0;
    LaunchRec& L = fp->launches[0];
    L.block = 256;
    if (stream) {
      pub.variant = vec ? DISC_V_ROW_STREAM_VEC : DISC_V_ROW_STREAM_SCALAR;
      L.kid = vec ? K_ROW_STREAM_VEC : K_ROW_STREAM_SCALAR;
      // (sums over the rows: a row of partial sums per block in the workspace, so fewer blocks)
      L.grid[0] = (uint32_t)std::min<int64_t>(sv.rows, n_col_sums > 0 ? (int64_t)c->n_cus * 2 : max_grid * 2);
      fp->aux[0] = L.grid[0];   // rows of partial sums: one per block
      pub.lanes_per_row = 256;
      pub.slots_per_lane = (int)((spr + 255) / 256);
      pub.reg_slots = 1;
    } else {
      // Lanes per row G and slots per lane nv (<= 2): the pair with the least capacity G * nv that
      // holds the row, two slots per lane on a tie.  G is a power of two.  The kernels accept any
      // multiple of 64 above a wavefront, but the finer steps measured slower: 6-wavefront blocks
      // load the four SIMDs of a CU unevenly (-25 %), 12-wavefront blocks (192 x 4 rows, 384 x 2)
      // leave a CU with one resident block (-10 %), and one slot per lane on more lanes loses to two
      // slots on fewer.  Wavefronts that hold no slot of the row skip the arithmetic anyway.
      struct Shape { int G, block; };
      static const Shape shapes[] = {{1, 256},  {2, 256},  {4, 256},   {8, 256},   {16, 256},  {32, 256},
                                     {64, 256}, {128, 256}, {256, 256}, {512, 512}, {1024, 1024}};
      const int max_nv = vec ? 3 : 2;   // three slots: vector versions only
      int G = 1024, nv = 2, block = 1024;
      auto choose = [&](int64_t slots) {
        int64_t best_cap = -1;
        for (const Shape& s : shapes)
          for (int k = max_nv; k >= 1; --k) {
            const int64_t cap = (int64_t)s.G * k;
            if (cap >= slots && (best_cap < 0 || cap < best_cap)) { best_cap = cap; G = s.G; nv = k; block = s.block; }
          }
      };
      // A ragged end (row length not a multiple of the vector width) as single elements: the row
      // then needs lanes for its WHOLE slots only, and the elements behind them go one each to the
      // first lanes of the row -- in the versions for rows of whole slots, when the pattern has
      // them for this case (no sums over the rows), the row has at least as many lanes as a slot
      // has elements, and the block is a wavefront quad.  Otherwise the ragged end is a slot.
      const bool tail_ok = vec && v > 1 && p.gen.row_tail_ok && sv.inner % v != 0 && sv.inner / v >= 1;
      bool tail = false;
      // (blocks above 256 threads have such a version for two slots per lane only)
      auto tail_fits = [&](int64_t slots) { return G >= v && (block <= 256 || (slots + G - 1) / G <= 2); };
      if (tail_ok) {
        choose(sv.inner / v);
        tail = tail_fits(sv.inner / v);
      }
      if (!tail) {
        choose(spr);
        tail = tail_ok && tail_fits(sv.inner / v);   // (the whole slots alone would have fitted fewer lanes than a slot has elements)
      }
      if (tail) spr = sv.inner / v;
      nv = (int)((spr + G - 1) / G);
      // Vector slots on the 16-byte boundaries of the tensor (the elements of a row in front of the
      // first boundary become single elements too): when the bases of the full-size operands are
      // aligned to a slot, the row has lanes for up to 2 (V - 1) single elements, and the grid can
      // be cut so that a lane group only meets rows of one alignment (see below).
      // Measured (rows of 2047 .. 4104 bf16 elements, plain accesses): rows that start on dword
      // boundaries run as fast unshifted as rows of whole 16-byte slots (5.14-5.20 against 5.15
      // TB/s) and lose 1-6 % when shifted (more single elements); rows that start off a dword
      // boundary (odd lengths of 2-byte elements) run at 4.90 unshifted and 4.95-5.01 shifted.
      // So the shift is for rows that start off dword boundaries only.
      bool shift = tail && p.gen.row_shift_ok && G >= 2 * v - 2 && c->row_shift != 0;
      if (shift) {
        bool off_dword = false;
        for (const Access& a : an.accesses) {
          if (a.kind != ACC_FULL || a.src_value >= 0) continue;
          const void* ptr = a.is_output ? (outputs ? outputs[a.slot] : nullptr) : (inputs ? inputs[a.slot] : nullptr);
          if (reinterpret_cast<uintptr_t>(ptr) % (uintptr_t)(v * dtype_bytes(a.dtype)) != 0) shift = false;
          if (dtype_bytes(a.dtype) >= 2 && (sv.inner * dtype_bytes(a.dtype)) % 4 != 0) off_dword = true;
        }
        shift = shift && off_dword;
      }
      int inst = std::max(nv, 2);   // instantiated slots per lane: 2 or 3
      pub.variant = vec ? DISC_V_ROW_REG_VEC : DISC_V_ROW_REG_SCALAR;
      L.block = (uint32_t)block;
      L.plan_kind = 1;
      L.rp.G = G;
      L.rp.log2G = ilog2_ceil(G);
      L.rp.nv = nv;
      L.rp.rpb = block / G;
      // stage row vectors in LDS when they fit a modest budget (keeps >= 3 blocks per CU resident)
      {
        int64_t bytes = 0;
        for (int eb : p.gen.staged_elem_bytes) bytes += ((sv.inner + v) * eb + 15) & ~15ll;
        const bool stage = vec && V > 1 && c->row_stage && bytes > 0 && bytes <= 48 * 1024;
        L.rp.flags = (stage ? 1 : 0) | (n_col_sums == 0 ? 0 : 2);
        L.dyn_lds = stage ? (uint32_t)bytes : 0;
        const bool wide_version = block > 256;
        // Non-temporal version (blocks of 256 threads, vector width only).  Host rule, measured on
        // softmax and LayerNorm sweeps: the hint gains 5-15 % when every row starts and ends on a
        // 16-byte boundary (row length a multiple of the vector width, aligned bases) and either
        // every row is a whole number of 128-byte cache lines (from 128 elements on) or the row has
        // at least 512 elements.  Rows whose first and last cache lines are shared with their
        // neighbours lose with it (-25 % for 360- or 464-element rows, -30 % for short odd rows),
        // as do operands that are read more than once, which never get the hint.  Small launches
        // (kNonTemporalMinBytes) keep the plain version: their results may be consumed from cache.
        // rows of whole slots (row length a multiple of the vector width) take the versions without
        // any ragged-tail path: _e, or _nt under the rule above
        const bool even = vec && V > 1 && !wide_version && (sv.inner % V == 0 || tail);
        bool nt = false;
        if (even && !tail && c->row_nt != 0) {
          nt = c->row_nt > 0;
          if (c->row_nt < 0 && sv.inner >= 128 && sv.alg_bytes >= kNonTemporalMinBytes) {
            nt = true;
            bool whole_lines = true;
            for (const Access& a : an.accesses) {
              if (a.kind != ACC_FULL) continue;
              const void* ptr = a.is_output ? (outputs ? outputs[a.slot] : nullptr) : (inputs ? inputs[a.slot] : nullptr);
              if (reinterpret_cast<uintptr_t>(ptr) % 16 != 0) nt = false;
              if ((sv.inner * dtype_bytes(a.dtype)) % 128 != 0) whole_lines = false;
            }
            if (!whole_lines && sv.inner < 512) nt = false;
          }
        }
        L.kid = K_ROW_BASE + row_kernel_index(!vec, inst, wide_version, stage, nt ? 1 : tail ? 3 : even ? 2 : 0);
      }
      // grid-stride over row groups: a small whole number of rounds of the blocks the chip holds
      // at once.  Measured: with plenty of rows, blocks of one wavefront-quad do best with three
      // rounds (the hardware does not fill every CU to the computed residency in the first round;
      // later blocks even that out); the wide blocks, and any launch that would leave a block
      // fewer than four row groups, with one (each new block pays an unpipelined first row and
      // the staging of the row vectors)
      const int rpb = (int)L.block / G;
      const int64_t ngroups = (sv.rows + rpb - 1) / rpb;
      const int64_t held = (int64_t)c->n_cus * resident_blocks(c, p, L.kid, L.block, L.dyn_lds);
      // (with sums over the rows every block writes a row of partial sums per wavefront: one round)
      const int rounds = c->row_rounds > 0 ? c->row_rounds
                         : (L.block > 256 || n_col_sums > 0 ? 1 : (int)std::max<int64_t>(1, std::min<int64_t>(3, ngroups / (held * 4))));
      int64_t grid = std::min<int64_t>(ngroups, held * rounds);
      // An odd grid: with an even one a block of one row per iteration would only ever see even or
      // only odd rows, and when the row length is odd every other row starts two bytes off a
      // dword -- half of the blocks would run ~20 % slower all the time and set the kernel's time
      // (measured: +14-18 % on 4095- and 5739-wide rows).  With an odd grid every block walks
      // through all alignments of its rows, whatever the rows per block.
      if (shift) {
        // rows of one alignment per lane group: (distance between its rows) x (row length) must be a
        // multiple of the vector width
        int64_t m = v / std::gcd<int64_t>(sv.inner % v, v);
        m /= std::gcd<int64_t>(m, rpb);
        if (grid >= m) grid -= grid % m;
        else shift = false;
      }
      if (shift) L.rp.flags |= 4;
      else if (grid > 2 && grid % 2 == 0 && grid < ngroups) grid -= 1;
      L.grid[0] = (uint32_t)grid;
      // rows of partial sums: one per block of 256 threads, one per lane group of a wider block
      fp->aux[0] = grid * (L.block <= 256 ? 1 : (int64_t)L.block / std::max(G, 64));
      pub.lanes_per_row = G;
      pub.slots_per_lane = nv;
      pub.reg_slots = inst;
    }
    pub.n_launches = 1;
    if (n_col_sums > 0) {
      // workspace: n_col_sums planes of [partial rows, inner] fp32; the second launch adds the rows up
      int64_t cells, bytes;
      if (mul_ovf(fp->aux[0], sv.inner, &cells) || mul_ovf(cells, 4ll * n_col_sums, &bytes))
        return set_err(c, DISC_ERR_SHAPE, "workspace size overflows int64");
      pub.workspace_bytes = (size_t)bytes;
      fp->ws_off[0] = 0;
      LaunchRec& L1 = fp->launches[1];
      L1.kid = K_COLSUM_FINISH;
      L1.block = 256;
      L1.grid[0] = (uint32_t)std::min<int64_t>((sv.inner + 15) / 16, max_grid * 4);   // 16 columns per block
      pub.n_launches = 2;
    } else {
      fp->aux[0] = 0;
    }
    if (n_row_reds > 0) {
      // one partial result per block and reduction behind the column-sum planes; a last launch of
      // one block folds them
      fp->aux[1] = L.grid[0];
      fp->ws_off[1] = (pub.workspace_bytes + 255) / 256 * 256;
      pub.workspace_bytes = fp->ws_off[1] + (size_t)n_row_reds * (size_t)L.grid[0] * 4;
      LaunchRec& Lr = fp->launches[pub.n_launches++];
      Lr.kid = K_ROWRED_FINISH;
      Lr.block = 1024;
      Lr.grid[0] = 1;
    }
  } else {
    // column reduce: canonical [outer, mid, inner], rows = outer * mid
    const int64_t outer = an.mid_group == 1 ? sv.group[0] : 1;
    const int64_t mid = sv.mid, inner = sv.inner;
    if (outer == 0 || inner == 0) return DISC_OK;
    if (mid == 0) return set_err(c, DISC_ERR_EMPTY_REDUCE, "reduction over an axis of size 0");
    if (mid >= (1ll << 31) - 1) return set_err(c, DISC_ERR_SHAPE, "reduced axis longer than 2^31");
    // the column tiles are the x dimension of the grids (no grid stride across columns)
    if (inner >= (1ll << 31) - 4096) return set_err(c, DISC_ERR_SHAPE, "column reduce: more than 2^31 columns");
    int want_vec = -1, want_strip = -1, want_two = -1;
    if (force >= 0) {
      const bool two = force == DISC_V_COL_2STAGE_VEC || force == DISC_V_COL_2STAGE_SCALAR;
      if ((force < DISC_V_COL_3STAGE_VEC || force > DISC_V_COL_STRIP_SCALAR) && !two)
        return set_err(c, DISC_ERR_INVALID_ARG, "forced version does not belong to a column-reduce pattern");
      if (two && !p.gen.has_epilogue)
        return set_err(c, DISC_ERR_INVALID_ARG, "the two-launch version needs an output that keeps the reduced axis");
      want_vec = force == DISC_V_COL_3STAGE_VEC || force == DISC_V_COL_STRIP_VEC || force == DISC_V_COL_2STAGE_VEC;
      want_strip = force == DISC_V_COL_STRIP_VEC || force == DISC_V_COL_STRIP_SCALAR;
      want_two = two;
    }
    bool vec;
    {
      const int64_t spr_v = (inner + V - 1) / V;
      vec = 1.0 - (double)inner / (double)(spr_v * V) <= 0.25;
      if (want_vec >= 0) vec = want_vec != 0;
    }
    const int v = vec ? V : 1;
    const int64_t spr = (inner + v - 1) / v;
    // Small problems: one launch, a block per strip of columns (reduce, finish and epilogue in the
    // same kernel).  A launch that makes a round trip to memory costs 5-6 us whatever it moves; up
    // to about a million elements one such launch (4.5-10 us measured on 1024 fp32 columns) beats
    // two (12 us).  Measured alternatives: the strip version up to two million elements (17 us at
    // 1500 rows: too few blocks) and 128 narrower strips instead of 64 (no gain).
    int64_t total;
    const bool small = !mul_ovf(outer * mid, inner, &total) && total <= (1ll << 20);
    const bool strip = want_strip >= 0 ? want_strip != 0 : small;
    if (strip) {
      // strips of >= 32 bytes per row keep the accesses coalesced; narrower strips = more blocks
      int GC = 1;
      while (GC < 64 && (GC * (vec ? 16 : 4) < 32 || spr / (GC * 2) >= 64)) GC *= 2;
      GC = std::min<int>(GC, 1 << ilog2_ceil(std::min<int64_t>(spr, 64)));
      const int64_t col_tiles = (spr + GC - 1) / GC;
      DeviceColPlan cp{GC, ilog2_ceil(GC), 1, 0, mid, outer, 0};
      fp->aux[0] = 0;
      fp->aux[1] = outer * inner * 8;
      fp->ws_off[0] = 0;
      fp->ws_off[1] = 0;
      // (with an epilogue the reduce results stay in registers; without, they go to the planes)
      pub.workspace_bytes = p.gen.has_epilogue ? 0 : (size_t)p.gen.n_red_planes * (size_t)fp->aux[1];
      pub.variant = vec ? DISC_V_COL_STRIP_VEC : DISC_V_COL_STRIP_SCALAR;
      pub.lanes_per_row = GC;
      pub.vec_width = v;
      pub.index_bits = 64;
      LaunchRec& L0 = fp->launches[0];
      L0.kid = vec ? K_COL_STRIP_VEC : K_COL_STRIP_SCALAR;
      L0.grid[0] = (uint32_t)col_tiles;
      L0.grid[1] = (uint32_t)std::min<int64_t>(outer, 65535);
      L0.plan_kind = 2;
      L0.cp = cp;
      pub.n_launches = 1;
      for (int k2 = 0; k2 < 3; ++k2) pub.grid[0][k2] = L0.grid[k2];
      pub.block[0][0] = L0.block;
      pub.block[0][1] = pub.block[0][2] = 1;
      pub.lds_bytes[0] = 0;
      snprintf(pub.kernel[0], sizeof pub.kernel[0], "%s%s", p.gen.prefix.c_str(), kernel_name(L0.kid));
      return DISC_OK;
    }
    // Lanes along the columns per block: 16 lanes of one vector each (256 bytes of a row: two
    // whole cache lines) unless the rows are narrower; the other lanes of the block run down the
    // rows.  Narrow column tiles give the grid its width: with 64 lanes across, 1024 fp32 columns
    // are only 4 tiles, and the chunks of the reduced axis would have to supply all the parallelism.
    constexpr int64_t kTwoLaunchChunks = 32;
    // (narrow tensors: 8 or 4 lanes across when that yields more blocks, down to 64-byte row pieces)
    int GC = 1 << ilog2_ceil(std::min<int64_t>(spr, 16));
    {
      auto blocks_at = [&](int gc) {
        const int64_t t = (spr + gc - 1) / gc * std::min<int64_t>(outer, 65535);
        const int64_t maxc = std::max<int64_t>(1, mid / (4ll * (256 / gc)));
        return std::min<int64_t>(t * std::min<int64_t>(kTwoLaunchChunks, maxc), (int64_t)c->n_cus * 2);
      };
      int best = GC;
      for (int gc = GC >> 1; gc >= 4; gc >>= 1)
        if (blocks_at(gc) > blocks_at(best)) best = gc;
      GC = best;
    }
    const int TY = 256 / GC;
    const int64_t col_tiles = (spr + GC - 1) / GC;
    const int64_t tiles = col_tiles * std::min<int64_t>(outer, 65535);
    // Chunks of the reduced axis: enough blocks for two per CU, at least four rows per row-lane.
    // Up to kTwoLaunchChunks chunks the second launch can afford to merge the partials of its own
    // columns in every block (a few loads per lane), which saves the finish launch and the round
    // trip of the reduce results through memory: the two-launch version.  A reduced axis so long
    // and narrow that it needs more chunks than that keeps the separate finish launch.
    const int64_t max_chunks = std::max<int64_t>(1, mid / (4ll * TY));
    int64_t nchunk = ((int64_t)c->n_cus * 2 + tiles - 1) / tiles;
    nchunk = std::max<int64_t>(1, std::min<int64_t>(nchunk, max_chunks));
    bool two = p.gen.has_epilogue && nchunk <= kTwoLaunchChunks;
    if (want_two >= 0) two = want_two != 0;
    if (two) nchunk = std::min<int64_t>(nchunk, kTwoLaunchChunks);
    else nchunk = std::min<int64_t>(std::max<int64_t>(1, std::min<int64_t>(((int64_t)c->n_cus * 4 + tiles - 1) / tiles, max_chunks)), 1024);
    const int64_t chunk_rows = (mid + nchunk - 1) / nchunk;
    nchunk = (mid + chunk_rows - 1) / chunk_rows;
    DeviceColPlan cp{GC, ilog2_ceil(GC), (int32_t)nchunk, 0, chunk_rows, outer, 0};
    int64_t cells, red_bytes;
    if (mul_ovf(outer * nchunk, inner, &cells) || mul_ovf(cells, (int64_t)p.gen.n_acc_cells * 8, &red_bytes))
      return set_err(c, DISC_ERR_SHAPE, "workspace size overflows int64");
    fp->aux[0] = cells;                 // cells per accumulator-field plane
    fp->aux[1] = outer * inner * 8;     // bytes per reduce-result plane
    fp->ws_off[0] = 0;
    fp->ws_off[1] = ((size_t)red_bytes + 255) / 256 * 256;
    pub.lanes_per_row = GC;
    LaunchRec& L0 = fp->launches[0];
    L0.kid = vec ? K_COL_PARTIAL_VEC : K_COL_PARTIAL_SCALAR;
    L0.grid[0] = (uint32_t)col_tiles;
    L0.grid[1] = (uint32_t)nchunk;
    L0.grid[2] = (uint32_t)std::min<int64_t>(outer, 65535);
    L0.plan_kind = 2;
    if (two) {
      // second launch: column tiles x row ranges, about eight blocks per CU; every lane gets at
      // least four rows so that the merge of the partials stays a small part of the block's work
      int64_t row_blocks = std::max<int64_t>(1, ((int64_t)c->n_cus * 8 + tiles - 1) / tiles);
      row_blocks = std::min<int64_t>(std::min<int64_t>(row_blocks, max_chunks), 65535);
      cp.epi_rows = (mid + row_blocks - 1) / row_blocks;
      row_blocks = (mid + cp.epi_rows - 1) / cp.epi_rows;
      pub.workspace_bytes = (size_t)red_bytes;   // partials only: the reduce results stay in registers
      pub.variant = vec ? DISC_V_COL_2STAGE_VEC : DISC_V_COL_2STAGE_SCALAR;
      pub.vec_width = v;
      pub.index_bits = 64;
      L0.cp = cp;
      LaunchRec& L1 = fp->launches[1];
      // non-temporal stores for large launches with aligned rows: the results then do not push the
      // operand, which the second launch reads again, out of the memory-side cache
      const bool nt = vec && v > 1 && inner % v == 0 && c->row_nt != 0 &&
                      (c->row_nt > 0 || (sv.alg_bytes >= kNonTemporalMinBytes && full_aligned()));
      L1.kid = vec ? (nt ? K_COL_EPI2_VEC_NT : K_COL_EPI2_VEC) : K_COL_EPI2_SCALAR;
      L1.grid[0] = (uint32_t)col_tiles;
      L1.grid[1] = (uint32_t)row_blocks;
      L1.grid[2] = (uint32_t)std::min<int64_t>(outer, 65535);
      L1.plan_kind = 2;
      L1.cp = cp;
      pub.n_launches = 2;
    } else {
      pub.workspace_bytes = fp->ws_off[1] + (size_t)p.gen.n_red_planes * (size_t)fp->aux[1];
      pub.variant = vec ? DISC_V_COL_3STAGE_VEC : DISC_V_COL_3STAGE_SCALAR;
      L0.cp = cp;
      LaunchRec& L1 = fp->launches[1];
      L1.kid = K_COL_FINISH;
      L1.grid[0] = (uint32_t)((inner + 15) / 16);   // 16 columns per block
      L1.grid[1] = (uint32_t)std::min<int64_t>(outer, 65535);
      L1.plan_kind = 2;
      L1.cp = cp;
      pub.n_launches = 2;
      if (p.gen.has_epilogue) {
        static const int names[] = {K_COL_EPI_VEC, K_COL_EPI_VEC_I64, K_COL_EPI_SCALAR, K_COL_EPI_SCALAR_I64};
        bool v2, i64;
        rc = plan_loop(c, sv.rows, inner, V, vec ? 1 : 0, -1, names, K_COL_EPI_VEC_NT, full_aligned(), sv.alg_bytes >= kNonTemporalMinBytes, fp, &fp->launches[2], &v2, &i64);
        if (rc) return rc;
        pub.n_launches = 3;
      } else {
        pub.vec_width = v;
        pub.index_bits = 64;
      }
    }
  }
  for (int l = 0; l < pub.n_launches; ++l) {
    for (int k = 0; k < 3; ++k) pub.grid[l][k] = fp->launches[l].grid[k];
    pub.block[l][0] = fp->launches[l].block;
    pub.block[l][1] = pub.block[l][2] = 1;
    pub.lds_bytes[l] = fp->launches[l].dyn_lds;
    snprintf(pub.kernel[l], sizeof pub.kernel[l], "%s%s", p.gen.prefix.c_str(), kernel_name(fp->launches[l].kid));
  }
  return DISC_OK;
}

int resident_blocks(const disc_ctx* c, const Pattern& p, int kid, uint32_t block, uint32_t dyn_lds) {
  const int estimate = std::max(1, 16 / (int)((block + 63) / 64));
  if (c->device < 0 || kid < 0 || kid >= K_COUNT || !p.fn[kid]) return estimate;
  // the table is stepped in dynamic LDS: the question is asked for the upper end of the step
  const int bc = block <= 256 ? 0 : block <= 512 ? 1 : 2;
  const int step = (int)std::min<uint32_t>((dyn_lds + kLdsStep - 1) / kLdsStep, kLdsSteps - 1);
  int16_t& cell = p.resident[kid][bc][step];
  if (cell > 0) return cell;
  int nb = 0;
  if (hipModuleOccupancyMaxActiveBlocksPerMultiprocessor(&nb, p.fn[kid], (int)block, (size_t)step * kLdsStep) != hipSuccess || nb < 1)
    nb = estimate;
  cell = (int16_t)nb;
  return nb;
}

void fill_args(const Pattern& p, const FullPlan& fp, const int64_t* dims, const void* const* in, void* const* outp,
               void* ws, unsigned char* buf) {
  const ShapeVals& sv = fp.sv;
  for (const auto& f : p.gen.args.fields) {
    unsigned char* dst = buf + f.offset;
    int64_t v = 0;
    switch (f.kind) {
      case ArgField::ROWS: v = sv.rows; memcpy(dst, &v, 8); break;
      case ArgField::INNER: v = sv.inner; memcpy(dst, &v, 8); break;
      case ArgField::NSLOTS: v = fp.nslots; memcpy(dst, &v, 8); break;
      case ArgField::SPR: v = fp.spr; memcpy(dst, &v, 8); break;
      case ArgField::MID: v = sv.mid; memcpy(dst, &v, 8); break;
      case ArgField::GROUP_SIZE: v = sv.group[f.index]; memcpy(dst, &v, 8); break;
      case ArgField::IN_PTR: memcpy(dst, &in[f.index], 8); break;
      case ArgField::OUT_PTR: memcpy(dst, &outp[f.index], 8); break;
      case ArgField::WS_PTR: { void* w = ws ? (char*)ws + fp.ws_off[f.index] : nullptr; memcpy(dst, &w, 8); break; }
      case ArgField::AUX: v = fp.aux[f.index]; memcpy(dst, &v, 8); break;
      case ArgField::STRIDE: v = sv.products[f.index]; memcpy(dst, &v, 8); break;
      case ArgField::DIMI: v = dims[p.an.dim_size_syms[f.index]]; memcpy(dst, &v, 8); break;
      case ArgField::SPR_DIV: { FastDivHost d = make_fastdiv((uint64_t)fp.spr); memcpy(dst, &d, 16); break; }
      case ArgField::GROUP_DIV: { FastDivHost d = make_fastdiv((uint64_t)sv.group[f.index]); memcpy(dst, &d, 16); break; }
      case ArgField::DIMF: { float x = (float)dims[p.an.dim_size_syms[f.index]]; memcpy(dst, &x, 4); break; }
    }
  }
}

const char* kUtilSource = R"SRC(
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
template <bool NT>
__device__ __forceinline__ void copy_body(u32x4* __restrict__ dst, const u32x4* __restrict__ src, long long n) {
  const long long stride = (long long)gridDim.x * blockDim.x;
  long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  for (; i + 3 * stride < n; i += 4 * stride) {
    u32x4 a, b, c, d;
    if constexpr (NT) {
      a = __builtin_nontemporal_load(src + i); b = __builtin_nontemporal_load(src + i + stride);
      c = __builtin_nontemporal_load(src + i + 2 * stride); d = __builtin_nontemporal_load(src + i + 3 * stride);
      __builtin_nontemporal_store(a, dst + i); __builtin_nontemporal_store(b, dst + i + stride);
      __builtin_nontemporal_store(c, dst + i + 2 * stride); __builtin_nontemporal_store(d, dst + i + 3 * stride);
    } else {
      a = src[i]; b = src[i + stride]; c = src[i + 2 * stride]; d = src[i + 3 * stride];
      dst[i] = a; dst[i + stride] = b; dst[i + 2 * stride] = c; dst[i + 3 * stride] = d;
    }
  }
  for (; i < n; i += stride) dst[i] = src[i];
}
extern "C" __global__ void __launch_bounds__(256) disc_util_copy_k(u32x4* __restrict__ dst, const u32x4* __restrict__ src, long long n) {
  copy_body<false>(dst, src, n);
}
extern "C" __global__ void __launch_bounds__(256) disc_util_copy_nt_k(u32x4* __restrict__ dst, const u32x4* __restrict__ src, long long n) {
  copy_body<true>(dst, src, n);
}
extern "C" __global__ void disc_util_empty_k() {}

// Streaming probes with the traffic mix of the row kernels and no arithmetic to speak of: per slot of
// eight 2-byte elements, KIND 0 reads 16 bytes + 8 bytes of a 1-byte stream and writes 16 bytes (3 bytes
// read : 2 written per element, the mix of the 12-op pattern), KIND 1 reads 16 + 16 bytes and writes 16
// (4 : 2, residual + LayerNorm).  NT = non-temporal accesses, U = slots in flight per lane.
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
template <int KIND, bool NT, int U>
__device__ __forceinline__ void mix_body(u32x4* __restrict__ out, const u32x4* __restrict__ a, const u32x4* __restrict__ b,
                                         const u32x2* __restrict__ m, long long n) {
  const long long stride = (long long)gridDim.x * blockDim.x;
  for (long long i0 = (long long)blockIdx.x * blockDim.x + threadIdx.x; i0 < n; i0 += stride * U) {
    u32x4 x[U], y[U];
    u32x2 k[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const long long i = i0 + u * stride;
      if (i < n) {
        if constexpr (NT) x[u] = __builtin_nontemporal_load(a + i); else x[u] = a[i];
        if constexpr (KIND == 0) { if constexpr (NT) k[u] = __builtin_nontemporal_load(m + i); else k[u] = m[i]; }
        else { if constexpr (NT) y[u] = __builtin_nontemporal_load(b + i); else y[u] = b[i]; }
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const long long i = i0 + u * stride;
      if (i < n) {
        u32x4 r = x[u];
        if constexpr (KIND == 0) { r.x ^= k[u].x; r.z ^= k[u].y; } else { r ^= y[u]; }
        if constexpr (NT) __builtin_nontemporal_store(r, out + i); else out[i] = r;
      }
    }
  }
}
#define DISC_MIX(KIND, NT, U)                                                                                        \
  extern "C" __global__ void __launch_bounds__(256) disc_util_mix_##KIND##_##NT##_##U(                               \
      u32x4* __restrict__ out, const u32x4* __restrict__ a, const u32x4* __restrict__ b, const u32x2* __restrict__ m, \
      long long n) {                                                                                                 \
    mix_body<KIND, NT != 0, U>(out, a, b, m, n);                                                                     \
  }
DISC_MIX(0, 0, 1) DISC_MIX(0, 0, 2) DISC_MIX(0, 0, 4) DISC_MIX(0, 0, 8)
DISC_MIX(0, 1, 1) DISC_MIX(0, 1, 2) DISC_MIX(0, 1, 4) DISC_MIX(0, 1, 8)
DISC_MIX(1, 0, 1) DISC_MIX(1, 0, 2) DISC_MIX(1, 0, 4) DISC_MIX(1, 0, 8)
DISC_MIX(1, 1, 1) DISC_MIX(1, 1, 2) DISC_MIX(1, 1, 4) DISC_MIX(1, 1, 8)
)SRC";

int ensure_util(disc_ctx* c) {
  if (c->util_module) return DISC_OK;
  if (c->device < 0) return set_err(c, DISC_ERR_INVALID_ARG, "host-only context");
  std::vector<char> code;
  double ms;
  int rc = compile_source(c, kUtilSource, &code, &ms);
  if (rc) return rc;
  hipError_t e = hipModuleLoadData(&c->util_module, code.data());
  if (e != hipSuccess) return hip_fail(c, e, "hipModuleLoadData");
  if ((e = hipModuleGetFunction(&c->util_copy, c->util_module, "disc_util_copy_k")) != hipSuccess) return hip_fail(c, e, "hipModuleGetFunction");
  if ((e = hipModuleGetFunction(&c->util_copy_nt, c->util_module, "disc_util_copy_nt_k")) != hipSuccess) return hip_fail(c, e, "hipModuleGetFunction");
  if ((e = hipModuleGetFunction(&c->util_empty, c->util_module, "disc_util_empty_k")) != hipSuccess) return hip_fail(c, e, "hipModuleGetFunction");
  for (int kind = 0; kind < 2; ++kind)
    for (int nt = 0; nt < 2; ++nt)
      for (int lu = 0; lu < 4; ++lu) {
        char name[48];
        snprintf(name, sizeof name, "disc_util_mix_%d_%d_%d", kind, nt, 1 << lu);
        if ((e = hipModuleGetFunction(&c->util_mix[kind][nt][lu], c->util_module, name)) != hipSuccess) return hip_fail(c, e, "hipModuleGetFunction");
      }
  return DISC_OK;
}

}  // namespace

// accessors for scratch.hip (the one source file compiled as HIP: it owns the static device array)
namespace disc {
int context_device(const disc_ctx* ctx) { return ctx ? ctx->device : -1; }
int context_fail(disc_ctx* ctx, int code, const char* msg) {
  try {
    return set_err(ctx, code, msg);
  } catch (...) {
    return code;
  }
}
}  // namespace disc
extern "C" int disc_static_scratch_init(disc_ctx* ctx);

// ============================================================================================
// C ABI
// ============================================================================================
// Nothing may leave an extern "C" function by exception: registration allocates (strings, vectors,
// maps), and an allocation failure there must come back as a status like everything else.
static int guard_fail(disc_ctx* c, const char* what) noexcept {
  if (c) {
    try {
      c->err = std::string("internal error: ") + what;
    } catch (...) {
    }
  }
  return DISC_ERR_INTERNAL;
}
#define DISC_TRY try {
#define DISC_CATCH(c)                                                          \
  }                                                                            \
  catch (const std::bad_alloc&) { return guard_fail(c, "out of host memory"); } \
  catch (const std::exception& e) { return guard_fail(c, e.what()); }          \
  catch (...) { return guard_fail(c, "unknown exception"); }

extern "C" {

int disc_create(disc_ctx** out, int hip_device) {
  DISC_TRY
  if (!out) return DISC_ERR_INVALID_ARG;
  *out = nullptr;
  std::unique_ptr<disc_ctx> c(new (std::nothrow) disc_ctx);
  if (!c) return DISC_ERR_INVALID_ARG;
  c->device = hip_device;
  if (hip_device >= 0) {
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || hip_device >= n) return DISC_ERR_HIP;
    if (hipSetDevice(hip_device) != hipSuccess) return DISC_ERR_HIP;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, hip_device) != hipSuccess) return DISC_ERR_HIP;
    c->n_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    // the device address of the static scratch array (disc_launch_static_scratch), once per device
    if (disc_static_scratch_init(c.get()) != DISC_OK) return DISC_ERR_HIP;
  }
  *out = c.release();
  return DISC_OK;
  DISC_CATCH(nullptr)
}

void disc_destroy(disc_ctx* ctx) {
  if (!ctx) return;
  if (ctx->device >= 0) {
    for (auto& p : ctx->patterns)
      if (p->module) (void)hipModuleUnload(p->module);
    if (ctx->util_module) (void)hipModuleUnload(ctx->util_module);
  }
  delete ctx;
}

const char* disc_last_error(const disc_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

// Text of the DISC_STATIC_ARGS / DISC_STATIC_PLAN macros for one shape: every non-pointer member
// of the argument block and of the launch-plan struct becomes an assignment of its constant.
static std::string static_macros(const Pattern& p, const FullPlan& fp, const int64_t* dims) {
  alignas(16) unsigned char buf[kArgBufBytes] = {0};
  std::vector<const void*> in(std::max(1, p.an.n_inputs), nullptr);
  std::vector<void*> outp(std::max(1, p.an.n_outputs), nullptr);
  fill_args(p, fp, dims, in.data(), outp.data(), nullptr, buf);
  std::ostringstream a;
  a << "#define DISC_STATIC_ARGS(A)";
  for (size_t i = 0; i < p.gen.args.fields.size(); ++i) {
    const ArgField& f = p.gen.args.fields[i];
    const std::string& n = p.gen.field_names[i];
    const unsigned char* src = buf + f.offset;
    switch (f.kind) {
      case ArgField::IN_PTR: case ArgField::OUT_PTR: case ArgField::WS_PTR: break;
      case ArgField::AUX:
        // the number of partial-sum rows follows the grid, which is chosen again at every launch
        // from the loaded kernel's residency: it stays a run-time argument
        if (p.gen.n_col_sums > 0 || p.gen.n_row_reds > 0) break;
        [[fallthrough]];
      default: {
        int64_t v;
        memcpy(&v, src, 8);
        a << " A." << n << " = " << v << "LL;";
        break;
      }
      case ArgField::SPR_DIV: case ArgField::GROUP_DIV: {
        uint32_t w[4];
        memcpy(w, src, 16);
        a << " A." << n << " = disc::FastDiv{" << w[0] << "u, " << w[1] << "u, " << w[2] << "u, 0u};";
        break;
      }
      case ArgField::DIMF: {
        uint32_t w;
        memcpy(&w, src, 4);
        a << " A." << n << " = __builtin_bit_cast(float, " << w << "u);";
        break;
      }
    }
  }
  a << "\n#define DISC_STATIC_PLAN(rp)";
  const LaunchRec& L = fp.launches[0];
  if (L.plan_kind == 1)
    a << " rp.G = " << L.rp.G << "; rp.log2G = " << L.rp.log2G << "; rp.nv = " << L.rp.nv << "; rp.flags = " << L.rp.flags
      << "; rp.rpb = " << L.rp.rpb << ";";
  else if (L.plan_kind == 2)
    a << " rp.GC = " << L.cp.GC << "; rp.log2GC = " << L.cp.log2GC << "; rp.nchunk = " << L.cp.nchunk << "; rp.chunk_rows = "
      << L.cp.chunk_rows << "LL; rp.outer = " << L.cp.outer << "LL; rp.epi_rows = " << L.cp.epi_rows << "LL;";
  a << "\n";
  return a.str();
}

static int register_impl(disc_ctx* ctx, const disc_op* ops, int n_ops, const disc_constraint* cs, int n_cs,
                         const int64_t* static_dims, int n_static_dims, int32_t* pattern_id_out) {
  if (!ctx) return DISC_ERR_INVALID_ARG;
  if (!pattern_id_out) return set_err(ctx, DISC_ERR_INVALID_ARG, "pattern_id_out is null");
  *pattern_id_out = -1;
  if (!ops || n_ops <= 0) return set_err(ctx, DISC_ERR_INVALID_ARG, "empty op list");
  if (n_cs < 0 || (n_cs > 0 && !cs)) return set_err(ctx, DISC_ERR_INVALID_ARG, "bad constraint list");
  if (n_ops > DISC_MAX_OPS) return set_err(ctx, DISC_ERR_BAD_PATTERN, "too many ops");
  // pattern cache: the key is the op sequence and the constraints -- no sizes (Section 2)
  std::string key;
  for (int i = 0; i < n_ops; ++i) {
    disc_op o = ops[i];
    const int rank = std::max(0, std::min<int>(o.rank, DISC_MAX_RANK));
    for (int k = rank; k < DISC_MAX_RANK; ++k) o.dim[k] = 0;
    const bool uses_map = o.opcode == DISC_BROADCAST || o.opcode == DISC_DIM_SIZE ||
                          (o.opcode >= DISC_REDUCE_SUM && o.opcode <= DISC_REDUCE_ARGMAX);
    if (!uses_map) memset(o.axis_map, 0, sizeof o.axis_map);
    if (o.opcode != DISC_CONST) o.fconst = 0;
    key.append(reinterpret_cast<const char*>(&o.opcode), sizeof(int32_t) * 2);
    key.append(reinterpret_cast<const char*>(o.in), sizeof o.in);
    key.append(reinterpret_cast<const char*>(&o.rank), sizeof(int32_t));
    key.append(reinterpret_cast<const char*>(o.dim), sizeof o.dim);
    key.append(reinterpret_cast<const char*>(o.axis_map), sizeof o.axis_map);
    key.append(reinterpret_cast<const char*>(&o.fconst), sizeof o.fconst);
  }
  key.append("|");
  for (int i = 0; i < n_cs; ++i) key.append(reinterpret_cast<const char*>(&cs[i]), sizeof(disc_constraint));
  if (static_dims) {   // a single-shape module is a pattern of its own, one per shape
    key.append("|static");
    key.append(reinterpret_cast<const char*>(static_dims), sizeof(int64_t) * (size_t)n_static_dims);
  }
  auto hit = ctx->cache.find(key);
  if (hit != ctx->cache.end()) {
    *pattern_id_out = hit->second;
    ctx->stats.pattern_cache_hits++;
    return DISC_OK;
  }

  std::unique_ptr<Pattern> p(new Pattern);
  p->key = key;
  std::string err;
  int rc = analyze(ops, n_ops, cs, n_cs, &p->an, &err);
  if (rc) return set_err(ctx, rc, err);
  const std::string prefix = "disc_p" + std::to_string(ctx->patterns.size()) + "_";
  rc = generate(p->an, prefix, &p->gen, &err);
  if (rc) return set_err(ctx, rc, err);
  p->gen.source = std::string(kDeviceHeader) + "\n" + p->gen.source;
  // the launch path works in fixed-size buffers (nothing is allocated per launch)
  if (p->an.products.size() + p->an.offsets.size() + 2 * p->an.windows.size() > (size_t)kMaxShapeValues)
    return set_err(ctx, DISC_ERR_UNFUSIBLE, "too many strided, sliced or padded operands in one pattern");
  if (p->gen.args.size + 48 > kArgBufBytes) return set_err(ctx, DISC_ERR_UNFUSIBLE, "kernel-argument block too large");

  // launch-time constraint recipes
  DimClasses& dc = p->an.classes;
  p->class_of_dim.assign(p->an.n_sym, 0);
  {
    std::map<int, int> rep_to_class;
    std::map<int, int> first_member;
    for (int d = 0; d < p->an.n_sym; ++d) {
      int r = dc.find(d);
      if (!rep_to_class.count(r)) rep_to_class[r] = (int)rep_to_class.size();
      p->class_of_dim[d] = rep_to_class[r];
      if (first_member.count(r)) p->eq_checks.push_back({first_member[r], d});
      else first_member[r] = d;
      if (dc.static_val[r] >= 0 && first_member[r] == d) p->static_checks.push_back({d, dc.static_val[r]});
    }
    p->n_classes = (int)rep_to_class.size();
  }
  // algorithmic bytes: every operand and result once; an input that is only read through slices
  // counts with the elements its slices read
  std::vector<char> read_whole(p->an.ops.size(), 0);
  for (const auto& op : p->an.ops) {
    if (op.opcode == DISC_SLICE || op.opcode <= DISC_DIM_SIZE) continue;   // (a PAD reads its operand whole)
    for (int k = 0; k < 3; ++k)
      if (op.in[k] >= 0 && (k == 0 || op.opcode == DISC_SELECT || (op.opcode >= DISC_ADD && op.opcode <= DISC_NE)))
        read_whole[op.in[k]] = 1;
  }
  for (size_t i = 0; i < p->an.ops.size(); ++i) {
    const disc_op& op = p->an.ops[i];
    if (op.opcode == DISC_PARAM && !read_whole[i]) continue;
    if (op.opcode == DISC_SLICE && read_whole[op.in[0]]) continue;
    if (op.opcode != DISC_PARAM && op.opcode != DISC_OUTPUT && op.opcode != DISC_SLICE) continue;
    DimProduct prod;
    for (int k = 0; k < op.rank; ++k) {
      if (op.dim[k] >= 0) prod.sym.push_back(op.dim[k]); else prod.stat *= -(int64_t)op.dim[k];
    }
    p->io_numel.push_back({prod, dtype_bytes(op.dtype)});
  }

  if (static_dims) {
    // plan the one shape with the generic rules, then regenerate the module with only the kernel
    // versions that plan launches and with every extent and plan member as a constant
    FullPlan fp;
    rc = make_plan(ctx, *p, static_dims, n_static_dims, -1, nullptr, nullptr, &fp);
    if (rc) return rc;
    GenOptions opt;
    for (int l = 0; l < fp.pub.n_launches; ++l) {
      const std::string k = kernel_name(fp.launches[l].kid);
      opt.only_kernels.push_back(k);
      // planned without pointers, i.e. for aligned operands: keep the plain sibling of a
      // non-temporal version for launches whose operands turn out not to be 16-byte aligned
      // (for a row kernel that sibling is the version for rows of whole slots, _e)
      if (k.size() > 3 && k.compare(k.size() - 3, 3, "_nt") == 0)
        opt.only_kernels.push_back(k.substr(0, k.size() - 3) + (k.compare(0, 6, "k_row_") == 0 ? "_e" : ""));
    }
    if (opt.only_kernels.empty()) return set_err(ctx, DISC_ERR_SHAPE, "a single-shape pattern needs a shape that launches something");
    const std::string macros = static_macros(*p, fp, static_dims);
    Generated g2;
    rc = generate(p->an, prefix, &g2, &err, &opt);
    if (rc) return set_err(ctx, rc, err);
    g2.source = macros + std::string(kDeviceHeader) + "\n" + g2.source;
    p->gen = g2;
    p->is_static = true;
    p->static_dims.assign(static_dims, static_dims + n_static_dims);
  }
  std::vector<char> code;
  rc = compile_source(ctx, p->gen.source, &code, &p->compile_ms);
  p->compile_events = 1;
  ctx->stats.compile_events++;
  if (rc) return rc;
  if (ctx->device >= 0) {
    hipError_t e = hipModuleLoadData(&p->module, code.data());
    if (e != hipSuccess) return hip_fail(ctx, e, "hipModuleLoadData");
    for (const auto& name : p->gen.kernels) {
      hipFunction_t f;
      e = hipModuleGetFunction(&f, p->module, (p->gen.prefix + name).c_str());
      if (e != hipSuccess) return hip_fail(ctx, e, ("hipModuleGetFunction " + name).c_str());
      const int kid = kernel_id(name);
      if (kid < 0) return set_err(ctx, DISC_ERR_COMPILE, "generated module holds an unnumbered kernel: " + name);
      p->fn[kid] = f;
    }
  }
  const int id = (int)ctx->patterns.size();
  ctx->cache[key] = id;
  ctx->patterns.push_back(std::move(p));
  ctx->stats.patterns_registered++;
  *pattern_id_out = id;
  return DISC_OK;
}

int disc_register_pattern(disc_ctx* ctx, const disc_op* ops, int n_ops, const disc_constraint* cs, int n_cs,
                          int32_t* pattern_id_out) {
  DISC_TRY
  return register_impl(ctx, ops, n_ops, cs, n_cs, nullptr, 0, pattern_id_out);
  DISC_CATCH(ctx)
}

int disc_register_pattern_static(disc_ctx* ctx, const disc_op* ops, int n_ops, const disc_constraint* cs, int n_cs,
                                 const int64_t* dims, int n_dims, int32_t* pattern_id_out) {
  DISC_TRY
  if (!ctx) return DISC_ERR_INVALID_ARG;
  if (!dims || n_dims <= 0) return set_err(ctx, DISC_ERR_INVALID_ARG, "a single-shape pattern needs its dims");
  return register_impl(ctx, ops, n_ops, cs, n_cs, dims, n_dims, pattern_id_out);
  DISC_CATCH(ctx)
}

int disc_pattern_info(disc_ctx* ctx, int32_t id, disc_pattern_info_t* out) {
  DISC_TRY
  Pattern* p = get_pattern(ctx, id);
  if (!p || !out) return set_err(ctx, DISC_ERR_INVALID_ARG, "bad pattern id or null output");
  memset(out, 0, sizeof *out);
  out->template_kind = p->an.tmpl;
  out->n_dims = p->an.n_sym;
  out->n_inputs = p->an.n_inputs;
  out->n_outputs = p->an.n_outputs;
  out->compile_events = p->compile_events;
  out->n_variants = (int)p->gen.kernels.size();
  out->n_phases = p->an.n_phases;
  out->vec_width = p->an.vec_width;
  out->n_collapsed = (int)p->an.groups.size();
  out->n_dim_classes = p->n_classes;
  for (int d = 0; d < p->an.n_sym && d < DISC_MAX_DIMS; ++d) out->dim_class[d] = p->class_of_dim[d];
  out->compile_ms = p->compile_ms;
  return DISC_OK;
  DISC_CATCH(ctx)
}

const char* disc_pattern_source(disc_ctx* ctx, int32_t id) {
  Pattern* p = get_pattern(ctx, id);
  return p ? p->gen.source.c_str() : nullptr;
}

int disc_workspace_bytes(disc_ctx* ctx, int32_t id, const int64_t* dims, int n_dims, size_t* out) {
  DISC_TRY
  Pattern* p = get_pattern(ctx, id);
  if (!p || !out) return set_err(ctx, DISC_ERR_INVALID_ARG, "bad pattern id or null output");
  FullPlan fp;
  int rc = make_plan(ctx, *p, dims, n_dims, ctx->force_variant, nullptr, nullptr, &fp);   // same selection disc_launch will make
  if (rc) return rc;
  *out = fp.pub.workspace_bytes;
  return DISC_OK;
  DISC_CATCH(ctx)
}

int disc_plan(disc_ctx* ctx, int32_t id, const int64_t* dims, int n_dims, const void* const* inputs,
              void* const* outputs, int force_variant, disc_plan_t* out) {
  DISC_TRY
  Pattern* p = get_pattern(ctx, id);
  if (!p || !out) return set_err(ctx, DISC_ERR_INVALID_ARG, "bad pattern id or null output");
  FullPlan fp;
  int rc = make_plan(ctx, *p, dims, n_dims, force_variant, inputs, outputs, &fp);
  if (rc) return rc;
  *out = fp.pub;
  return DISC_OK;
  DISC_CATCH(ctx)
}

int disc_force_variant(disc_ctx* ctx, int variant) {
  DISC_TRY
  if (!ctx || variant < -1 || variant >= DISC_V_COUNT) return set_err(ctx, DISC_ERR_INVALID_ARG, "unknown version");
  ctx->force_variant = variant;
  return DISC_OK;
  DISC_CATCH(ctx)
}

int disc_test_option(disc_ctx* ctx, int option, int value) {
  DISC_TRY
  if (!ctx) return DISC_ERR_INVALID_ARG;
  switch (option) {
    case DISC_OPT_NON_TEMPORAL: ctx->row_nt = value < 0 ? -1 : value > 0 ? 1 : 0; return DISC_OK;
    case DISC_OPT_STAGE_ROW_VECTORS: ctx->row_stage = value != 0; return DISC_OK;
    case DISC_OPT_ROW_ROUNDS: ctx->row_rounds = std::max(0, value); return DISC_OK;
    case DISC_OPT_ALIGN_ROW_SLOTS: ctx->row_shift = value != 0; return DISC_OK;
    default: return set_err(ctx, DISC_ERR_INVALID_ARG, "unknown option");
  }
  DISC_CATCH(ctx)
}

int disc_launch(disc_ctx* ctx, int32_t id, const int64_t* dims, int n_dims, const void* const* inputs, int n_in,
                void* const* outputs, int n_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  DISC_TRY
  const int64_t t0 = now_ns();
  Pattern* p = get_pattern(ctx, id);
  if (!p) return set_err(ctx, DISC_ERR_INVALID_ARG, "bad pattern id");
  if (ctx->device < 0) return set_err(ctx, DISC_ERR_INVALID_ARG, "host-only context cannot launch");
  if (n_in != p->an.n_inputs || n_out != p->an.n_outputs) {
    char buf[96];
    snprintf(buf, sizeof buf, "pattern takes %d inputs and %d outputs, got %d and %d", p->an.n_inputs, p->an.n_outputs, n_in, n_out);
    return set_err(ctx, DISC_ERR_INVALID_ARG, buf);
  }
  if ((n_in > 0 && !inputs) || !outputs) return set_err(ctx, DISC_ERR_INVALID_ARG, "null pointer array");
  FullPlan fp;
  int rc = make_plan(ctx, *p, dims, n_dims, ctx->force_variant, inputs, outputs, &fp);
  const int64_t t1 = now_ns();
  ctx->stats.host_plan_ns += t1 - t0;
  if (rc) return rc;
  if (fp.pub.n_launches == 0) {
    ctx->stats.launch_calls++;
    ctx->stats.host_launch_ns += now_ns() - t0;
    return DISC_OK;
  }
  for (int i = 0; i < n_in; ++i)
    if (!inputs[i]) return set_err(ctx, DISC_ERR_INVALID_ARG, "null input pointer");
  for (int i = 0; i < n_out; ++i)
    if (!outputs[i]) return set_err(ctx, DISC_ERR_INVALID_ARG, "null output pointer");
  if (fp.pub.workspace_bytes > 0 && (!workspace || workspace_bytes < fp.pub.workspace_bytes))
    return set_err(ctx, DISC_ERR_WORKSPACE, "workspace missing or too small");

  alignas(16) unsigned char buf[kArgBufBytes];
  const int asz = p->gen.args.size;   // (fits: checked at registration)
  fill_args(*p, fp, dims, inputs, outputs, workspace, buf);
  for (int l = 0; l < fp.pub.n_launches; ++l) {
    const LaunchRec& L = fp.launches[l];
    const hipFunction_t fn = L.kid >= 0 && L.kid < K_COUNT ? p->fn[L.kid] : nullptr;
    if (!fn) return set_err(ctx, DISC_ERR_HIP, std::string("kernel version missing: ") + kernel_name(L.kid));
    size_t size = (size_t)asz;
    if (L.plan_kind == 1) {
      memcpy(buf + asz, &L.rp, sizeof L.rp);
      size += sizeof L.rp;
    } else if (L.plan_kind == 2) {
      memcpy(buf + asz, &L.cp, sizeof L.cp);
      size += sizeof L.cp;
    }
    void* extra[] = {HIP_LAUNCH_PARAM_BUFFER_POINTER, buf, HIP_LAUNCH_PARAM_BUFFER_SIZE, &size, HIP_LAUNCH_PARAM_END};
    hipError_t e = hipModuleLaunchKernel(fn, L.grid[0], L.grid[1], L.grid[2], L.block, 1, 1, L.dyn_lds,
                                         (hipStream_t)hip_stream, nullptr, extra);
    if (e != hipSuccess) return hip_fail(ctx, e, "hipModuleLaunchKernel");
    ctx->stats.device_launches++;
  }
  ctx->stats.launch_calls++;
  if (fp.pub.variant >= 0 && fp.pub.variant < DISC_V_COUNT) ctx->stats.variant_count[fp.pub.variant]++;
  ctx->stats.host_launch_ns += now_ns() - t0;
  return DISC_OK;
  DISC_CATCH(ctx)
}

int disc_get_stats(disc_ctx* ctx, disc_stats_t* out) {
  DISC_TRY
  if (!ctx || !out) return DISC_ERR_INVALID_ARG;
  *out = ctx->stats;
  return DISC_OK;
  DISC_CATCH(ctx)
}

static int util_copy_impl(disc_ctx* ctx, void* dst, const void* src, size_t bytes, void* hip_stream, bool nt) {
  if (!ctx || !dst || !src || (bytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15))
    return set_err(ctx, DISC_ERR_INVALID_ARG, "copy needs 16-byte aligned pointers and size");
  int rc = ensure_util(ctx);
  if (rc) return rc;
  long long n = (long long)(bytes / 16);
  if (n == 0) return DISC_OK;
  void* args[] = {&dst, &src, &n};
  long long blocks = std::min<long long>((n + 1023) / 1024, (long long)ctx->n_cus * 2);
  hipError_t e = hipModuleLaunchKernel(nt ? ctx->util_copy_nt : ctx->util_copy, (uint32_t)blocks, 1, 1, 256, 1, 1, 0,
                                       (hipStream_t)hip_stream, args, nullptr);
  return e == hipSuccess ? DISC_OK : hip_fail(ctx, e, "hipModuleLaunchKernel");
}

int disc_util_copy(disc_ctx* ctx, void* dst, const void* src, size_t bytes, void* hip_stream) {
  DISC_TRY
  return util_copy_impl(ctx, dst, src, bytes, hip_stream, false);
  DISC_CATCH(ctx)
}

int disc_util_copy_nt(disc_ctx* ctx, void* dst, const void* src, size_t bytes, void* hip_stream) {
  DISC_TRY
  return util_copy_impl(ctx, dst, src, bytes, hip_stream, true);
  DISC_CATCH(ctx)
}

int disc_util_mix(disc_ctx* ctx, int kind, int non_temporal, int slots_in_flight, int blocks_per_cu, void* out, const void* a,
                  const void* b_or_mask, size_t n_elems, void* hip_stream) {
  DISC_TRY
  if (!ctx || !out || !a || !b_or_mask || (n_elems & 7) || kind < 0 || kind > 1 || blocks_per_cu < 1 || blocks_per_cu > 64 ||
      (((uintptr_t)out | (uintptr_t)a | (uintptr_t)b_or_mask) & 15))
    return set_err(ctx, DISC_ERR_INVALID_ARG, "mix probe: 16-byte aligned pointers, n_elems a multiple of 8, kind 0 or 1");
  int lu = 0;
  while (lu < 4 && (1 << lu) != slots_in_flight) ++lu;
  if (lu == 4) return set_err(ctx, DISC_ERR_INVALID_ARG, "mix probe: slots in flight must be 1, 2, 4 or 8");
  int rc = ensure_util(ctx);
  if (rc) return rc;
  long long n = (long long)(n_elems / 8);
  if (n == 0) return DISC_OK;
  const void* bp = kind == 1 ? b_or_mask : nullptr;
  const void* mp = kind == 0 ? b_or_mask : nullptr;
  void* args[] = {&out, &a, &bp, &mp, &n};
  const long long blocks = std::min<long long>((n + 255) / 256, (long long)ctx->n_cus * blocks_per_cu);
  hipError_t e = hipModuleLaunchKernel(ctx->util_mix[kind][non_temporal ? 1 : 0][lu], (uint32_t)blocks, 1, 1, 256, 1, 1, 0,
                                       (hipStream_t)hip_stream, args, nullptr);
  return e == hipSuccess ? DISC_OK : hip_fail(ctx, e, "hipModuleLaunchKernel");
  DISC_CATCH(ctx)
}

int disc_util_empty_launch(disc_ctx* ctx, void* hip_stream) {
  DISC_TRY
  if (!ctx) return DISC_ERR_INVALID_ARG;
  int rc = ensure_util(ctx);
  if (rc) return rc;
  hipError_t e = hipModuleLaunchKernel(ctx->util_empty, 1, 1, 1, 64, 1, 1, 0, (hipStream_t)hip_stream, nullptr, nullptr);
  return e == hipSuccess ? DISC_OK : hip_fail(ctx, e, "hipModuleLaunchKernel");
  DISC_CATCH(ctx)
}

}  // extern "C"

// =================================================================================================
// Op graphs (Section 4.3: fusion decision; Section 4.2.2: buffer management): a list of ops that
// need not be one fusible pattern is cut into consecutive fusion patterns with the SAME test the
// single-pattern path uses (the checker's shape propagation + constraints), and the values that
// cross pattern boundaries get buffers planned by lifetime, shared between values whose shapes
// are the same symbolic expression.
// =================================================================================================
namespace {

bool is_leaf(int opcode) { return opcode == DISC_PARAM || opcode == DISC_CONST || opcode == DISC_DIM_SIZE; }

int op_arity(const disc_op& o) { return operand_count(o.opcode); }

// The op list of the pattern that computes the graph ops `S` (ascending ids): operands produced
// outside S become PARAMs (scalar leaves are copied instead), values of S read outside S (by ops
// of other groups or by graph OUTPUTs) become OUTPUTs, constraints between values that both
// appear are carried over.
// `wanted` null (while the cut is still growing): every value read outside S counts as an output,
// also those that readers will recompute, so that a candidate always has an output.  For the
// patterns as registered, `wanted` marks the values other patterns really take in (their
// in_values, which includes what their recomputed cones read) and the graph outputs.
void build_sub_pattern(const Graph& g, const std::vector<int>& S, const std::vector<char>& in_S,
                       std::vector<disc_op>* sub, std::vector<disc_constraint>* sub_cs, std::vector<int>* in_values,
                       std::vector<int>* out_values, const std::vector<char>* wanted) {
  const bool final_cut = wanted != nullptr;
  std::map<int, int> id_of;   // graph value -> sub-pattern value
  sub->clear();
  sub_cs->clear();
  in_values->clear();
  out_values->clear();
  std::function<int(int)> operand = [&](int v) -> int {
    auto it = id_of.find(v);
    if (it != id_of.end()) return it->second;
    const disc_op& src = g.ops[v];
    disc_op o = src;
    if (src.opcode == DISC_CONST || src.opcode == DISC_DIM_SIZE) {
      for (int k = 0; k < 3; ++k) o.in[k] = -1;
    } else if (!is_leaf(src.opcode) && g.remat[v]) {
      // a cheap element-wise function of graph inputs computed by another pattern: computed again
      // here, from the inputs, instead of being written out and read back
      const int n = op_arity(src);
      for (int k = 0; k < n; ++k) o.in[k] = operand(src.in[k]);
    } else {               // a graph input or a value of another group: a PARAM of its type and shape
      o.opcode = DISC_PARAM;
      for (int k = 0; k < 3; ++k) o.in[k] = -1;
      for (int k = 0; k < DISC_MAX_RANK; ++k) o.axis_map[k] = 0;
      o.fconst = 0;
      in_values->push_back(v);
    }
    sub->push_back(o);
    id_of[v] = (int)sub->size() - 1;
    return id_of[v];
  };
  // consumers outside S
  std::vector<char> read_outside(g.ops.size(), 0);
  for (size_t i = 0; i < g.ops.size(); ++i) {
    if (in_S[i] || !g.needed[i]) continue;
    const disc_op& o = g.ops[i];
    if (is_leaf(o.opcode)) continue;
    const int n = op_arity(o);
    for (int k = 0; k < n; ++k)
      if (o.in[k] >= 0 && in_S[o.in[k]] && !final_cut) read_outside[o.in[k]] = 1;
  }
  if (final_cut)
    for (int v : S)
      if ((*wanted)[v]) read_outside[v] = 1;
  // ops of S that only fed readers which now recompute them are left out of the final pattern
  std::vector<char> live(g.ops.size(), final_cut ? 0 : 1);
  if (final_cut)
    for (size_t r = S.size(); r-- > 0;) {
      const int v = S[r];
      if (read_outside[v]) live[v] = 1;
      if (!live[v]) continue;
      const int n = op_arity(g.ops[v]);
      for (int k = 0; k < n; ++k)
        if (in_S[g.ops[v].in[k]]) live[g.ops[v].in[k]] = 1;
    }
  for (int v : S) {
    if (!live[v]) continue;
    disc_op o = g.ops[v];
    const int n = op_arity(o);
    for (int k = 0; k < n; ++k) o.in[k] = operand(g.ops[v].in[k]);
    sub->push_back(o);
    id_of[v] = (int)sub->size() - 1;
  }
  for (int v : S)
    if (read_outside[v]) {
      disc_op o = g.ops[v];
      o.opcode = DISC_OUTPUT;
      o.in[0] = id_of[v];
      o.in[1] = o.in[2] = -1;
      for (int k = 0; k < DISC_MAX_RANK; ++k) o.axis_map[k] = 0;
      o.fconst = 0;
      sub->push_back(o);
      out_values->push_back(v);
    }
  for (const auto& c : g.cs) {
    auto a = id_of.find(c.a_value), b = id_of.find(c.b_value);
    if (a == id_of.end() || b == id_of.end()) continue;
    disc_constraint t = c;
    t.a_value = a->second;
    t.b_value = b->second;
    sub_cs->push_back(t);
  }
}

// bytes of value v at these dims; false when the product does not fit 2^62
bool value_bytes(const Graph& g, int v, const int64_t* dims, int64_t* out) {
  const disc_op& o = g.ops[v];
  int64_t n = dtype_bytes(o.dtype);
  for (int k = 0; k < o.rank; ++k)
    if (mul_ovf(n, o.dim[k] >= 0 ? dims[o.dim[k]] : -(int64_t)o.dim[k], &n)) return false;
  *out = n;
  return n < (1ll << 62);
}

Graph* get_graph(disc_ctx* ctx, int32_t id) {
  if (!ctx || id < 0 || id >= (int)ctx->graphs.size()) return nullptr;
  return ctx->graphs[id].get();
}

// byte offset of every buffer and of the shared pattern-workspace region for one set of dims
// buf_off: room for one offset per buffer (at most DISC_MAX_OPS)
int graph_layout(disc_ctx* ctx, const Graph& g, const int64_t* dims, int n_dims, size_t* buf_off,
                 size_t* pattern_ws_off, size_t* total) {
  if (!dims || n_dims != g.n_sym) return set_err(ctx, DISC_ERR_INVALID_ARG, "wrong number of dims for this graph");
  for (int i = 0; i < n_dims; ++i)
    if (dims[i] < 0) return set_err(ctx, DISC_ERR_SHAPE, "negative dim");
  size_t off = 0;
  for (size_t b = 0; b < g.buffer_value.size(); ++b) {
    buf_off[b] = off;
    int64_t bytes = 0;
    if (!value_bytes(g, g.buffer_value[b], dims, &bytes) || off + (size_t)bytes + 256 < off)
      return set_err(ctx, DISC_ERR_SHAPE, "buffer size overflows");
    off += ((size_t)bytes + 255) / 256 * 256;
  }
  *pattern_ws_off = off;
  size_t need = 0;
  for (const auto& gr : g.groups) {
    size_t w = 0;
    const int ns = ctx->patterns[gr.pattern_id]->an.n_sym;
    int rc = disc_workspace_bytes(ctx, gr.pattern_id, dims, ns, &w);
    if (rc) return rc;
    need = std::max(need, w);
  }
  *total = off + need;
  return DISC_OK;
}

}  // namespace

int disc_register_graph(disc_ctx* ctx, const disc_op* ops, int n_ops, const disc_constraint* cs, int n_cs,
                        int32_t* graph_id_out) {
  DISC_TRY
  if (!ctx) return DISC_ERR_INVALID_ARG;
  if (!graph_id_out) return set_err(ctx, DISC_ERR_INVALID_ARG, "graph_id_out is null");
  *graph_id_out = -1;
  if (!ops || n_ops <= 0) return set_err(ctx, DISC_ERR_INVALID_ARG, "empty op list");
  if (n_cs < 0 || (n_cs > 0 && !cs)) return set_err(ctx, DISC_ERR_INVALID_ARG, "bad constraint list");
  if (n_ops > DISC_MAX_OPS) return set_err(ctx, DISC_ERR_BAD_PATTERN, "too many ops");
  std::unique_ptr<Graph> g(new Graph);
  g->ops.assign(ops, ops + n_ops);
  if (n_cs) g->cs.assign(cs, cs + n_cs);
  g->group_of_op.assign(n_ops, -1);
  // structure checks the per-pattern checker cannot make on a cut-up list
  std::vector<int> compute;
  for (int i = 0; i < n_ops; ++i) {
    const disc_op& o = g->ops[i];
    if (o.opcode < 0 || o.opcode >= DISC_OPCODE_COUNT) return set_err(ctx, DISC_ERR_BAD_PATTERN, "unknown opcode");
    if (o.rank < 0 || o.rank > DISC_MAX_RANK) return set_err(ctx, DISC_ERR_BAD_PATTERN, "rank out of range");
    const int n = op_arity(o);
    for (int k = 0; k < n; ++k)
      if (o.in[k] < 0 || o.in[k] >= i || g->ops[o.in[k]].opcode == DISC_OUTPUT)
        return set_err(ctx, DISC_ERR_BAD_PATTERN, "operand does not name an earlier value");
    for (int k = 0; k < o.rank; ++k)
      if (o.dim[k] >= 0) g->n_sym = std::max(g->n_sym, o.dim[k] + 1);
    if (o.opcode == DISC_DIM_SIZE) g->n_sym = std::max(g->n_sym, o.axis_map[0] + 1);
    if (o.opcode == DISC_SLICE || o.opcode == DISC_PAD)       // starts / low paddings that are runtime values
      for (int k = 0; k < o.rank; ++k) g->n_sym = std::max(g->n_sym, o.axis_map[k] + 1);
    if (o.opcode == DISC_PARAM) g->param_index[i] = g->n_inputs++;
    else if (o.opcode == DISC_OUTPUT) {
      if (n < 1 || is_leaf(g->ops[o.in[0]].opcode))
        return set_err(ctx, DISC_ERR_BAD_PATTERN, "a graph output must be a computed value");
      if (g->output_index.count(o.in[0])) return set_err(ctx, DISC_ERR_BAD_PATTERN, "a value is output twice");
      g->output_index[o.in[0]] = g->n_outputs++;
    } else if (!is_leaf(o.opcode)) compute.push_back(i);
  }
  if (g->n_sym > DISC_MAX_DIMS) return set_err(ctx, DISC_ERR_BAD_PATTERN, "too many symbolic dims");
  // dead code: ops that no graph output depends on belong to no pattern
  {
    std::vector<char>& needed = g->needed;
    needed.assign(n_ops, 0);
    for (int i = n_ops - 1; i >= 0; --i) {
      const disc_op& o = g->ops[i];
      if (o.opcode == DISC_OUTPUT) needed[i] = 1;
      if (!needed[i]) continue;
      const int n = op_arity(o);
      for (int k = 0; k < n; ++k) needed[o.in[k]] = 1;
    }
    std::vector<int> kept;
    for (int v : compute)
      if (needed[v]) kept.push_back(v);
    compute.swap(kept);
  }
  if (compute.empty() || g->n_outputs == 0) return set_err(ctx, DISC_ERR_BAD_PATTERN, "nothing to compute");

  // Recomputing instead of buffering.  A value that is a cheap element-wise function of at most
  // two graph inputs (a cast of an input, an input plus a broadcast bias, ...) does not cross
  // cuts: a pattern that reads it computes it again from the inputs, which costs no more traffic
  // than reading the stored result and saves writing it.  At level 2 the function may also use
  // reduction results (per-row or per-column values: small), so that e.g. normalised activations
  // are recomputed from the input and the row statistics instead of being stored in full; the
  // reduction results themselves then cross the cut as small buffers.  Level 1: inputs only.
  // Level 0: nothing is recomputed.  The highest level whose cut passes the checker is taken.
  auto compute_remat = [&](int level) {
    g->remat.assign(n_ops, 0);
    if (level == 0) return;
    std::vector<std::set<int>> cone_params(n_ops), cone_anchors(n_ops);
    std::vector<int> cone_ops(n_ops, 0);
    const size_t max_ops = level == 2 ? 16 : 8;
    for (int i = 0; i < n_ops; ++i) {
      const disc_op& o = g->ops[i];
      if (o.opcode == DISC_PARAM) { cone_params[i].insert(i); continue; }
      if (is_leaf(o.opcode) || o.opcode == DISC_OUTPUT) continue;
      if (o.opcode >= DISC_REDUCE_SUM && o.opcode <= DISC_REDUCE_ARGMAX) {
        if (level == 2) cone_anchors[i].insert(i);
        continue;
      }
      // a transpose that moves the innermost axis fuses with nothing: it stays a kernel of its own
      if (o.opcode == DISC_TRANSPOSE && o.rank > 0 && o.axis_map[o.rank - 1] != o.rank - 1) continue;
      bool ok = true;
      int nops = 1;
      const int n = op_arity(o);
      for (int k = 0; k < n && ok; ++k) {
        const int a = o.in[k];
        const bool anchor = level == 2 && g->ops[a].opcode >= DISC_REDUCE_SUM && g->ops[a].opcode <= DISC_REDUCE_ARGMAX;
        if (!is_leaf(g->ops[a].opcode) && !g->remat[a] && !anchor) ok = false;
        cone_params[i].insert(cone_params[a].begin(), cone_params[a].end());
        cone_anchors[i].insert(cone_anchors[a].begin(), cone_anchors[a].end());
        nops += cone_ops[a];
      }
      cone_ops[i] = nops;
      if (ok && cone_params[i].size() <= 2 && cone_anchors[i].size() <= 4 && (size_t)nops <= max_ops) g->remat[i] = 1;
    }
  };

  // greedy cut in list order: an op joins the current pattern when the checker still accepts the
  // pattern with it (one provable iteration space, one template); otherwise it opens the next one
  std::vector<disc_op> sub;
  std::vector<disc_constraint> sub_cs;
  std::vector<int> ins, outs;
  auto fusible = [&](const std::vector<int>& S, std::string* why) {
    std::vector<char> in_S(n_ops, 0);
    for (int v : S) in_S[v] = 1;
    build_sub_pattern(*g, S, in_S, &sub, &sub_cs, &ins, &outs, nullptr);
    Analysis an;
    return analyze(sub.data(), (int)sub.size(), sub_cs.empty() ? nullptr : sub_cs.data(), (int)sub_cs.size(), &an, why);
  };
  // The patterns as they will be registered, last to first: a pattern's outputs are the graph
  // outputs it computes and what later patterns take in -- directly or through the cones they
  // recompute.  `each` gets every pattern that has an output; returns the first failure.
  struct FinalPattern {
    std::vector<disc_op> ops;
    std::vector<disc_constraint> cs;
    std::vector<int> in_values, out_values;
  };
  auto finalize = [&](const std::vector<std::vector<int>>& cs_, std::vector<FinalPattern>* each, std::string* why) {
    std::vector<char> wanted(n_ops, 0);
    for (const auto& kv : g->output_index) wanted[kv.first] = 1;
    each->assign(cs_.size(), FinalPattern());
    for (size_t gi = cs_.size(); gi-- > 0;) {
      std::vector<char> in_S(n_ops, 0);
      for (int v : cs_[gi]) in_S[v] = 1;
      FinalPattern& fp = (*each)[gi];
      build_sub_pattern(*g, cs_[gi], in_S, &fp.ops, &fp.cs, &fp.in_values, &fp.out_values, &wanted);
      if (fp.out_values.empty()) { fp.in_values.clear(); continue; }      // nothing reads it: dropped
      for (int v : fp.in_values) wanted[v] = 1;
      Analysis an;
      const int rc = analyze(fp.ops.data(), (int)fp.ops.size(), fp.cs.empty() ? nullptr : fp.cs.data(), (int)fp.cs.size(), &an, why);
      if (rc) return rc;
    }
    return (int)DISC_OK;
  };
  std::vector<std::vector<int>> cuts;
  std::string why;
  int cut_rc = DISC_OK;
  for (int level = 2; level >= 0; --level) {
    compute_remat(level);
    cuts.clear();
    cut_rc = DISC_OK;
    std::vector<int> cur;
    for (int v : compute) {
      cur.push_back(v);
      if (fusible(cur, &why) == DISC_OK) continue;
      cur.pop_back();
      if (cur.empty()) {
        cut_rc = set_err(ctx, DISC_ERR_UNFUSIBLE, "op " + std::to_string(v) + " is not a pattern on its own: " + why);
        break;
      }
      cuts.push_back(cur);
      cur.assign(1, v);
      const int rc = fusible(cur, &why);
      if (rc) {
        cut_rc = set_err(ctx, rc, "op " + std::to_string(v) + " is not a pattern on its own: " + why);
        break;
      }
    }
    if (cut_rc == DISC_OK) {
      cuts.push_back(cur);
      std::vector<FinalPattern> probe;
      const int rc = finalize(cuts, &probe, &why);
      if (rc) cut_rc = set_err(ctx, rc, "a cut of the graph is not a pattern: " + why);
    }
    if (cut_rc == DISC_OK) break;
  }
  if (cut_rc != DISC_OK) return cut_rc;

  // Sinking: the greedy cut also pulls in ops that only feed the NEXT pattern (say the |x| ahead of
  // a reduction the current pattern cannot hold), which turns their result into one more buffer.
  // Such an op moves to the pattern of its users when nothing of its own pattern and no graph
  // output reads it, all its users sit in one later pattern, that pattern still passes the checker
  // with it, and each of its computed operands crosses a pattern boundary anyway -- then the move
  // saves one write and one read of the op's result and adds at most one read of an operand.
  {
    std::vector<int> grp(n_ops, -1);
    for (size_t gi = 0; gi < cuts.size(); ++gi)
      for (int v : cuts[gi]) grp[v] = (int)gi;
    std::vector<std::vector<int>> users(n_ops);
    for (int i = 0; i < n_ops; ++i) {
      if (is_leaf(g->ops[i].opcode) || !g->needed[i]) continue;
      const int n = op_arity(g->ops[i]);
      for (int k = 0; k < n; ++k) users[g->ops[i].in[k]].push_back(i);
    }
    auto read_elsewhere = [&](int v, int except) {       // graph output, or read outside its pattern by another op
      for (int u : users[v]) {
        if (u == except) continue;
        if (g->ops[u].opcode == DISC_OUTPUT || grp[u] != grp[v]) return true;
      }
      return false;
    };
    bool moved = true;
    while (moved) {
      moved = false;
      for (size_t gi = 0; gi + 1 < cuts.size(); ++gi) {
        for (size_t pos = cuts[gi].size(); pos-- > 0;) {
          const int x = cuts[gi][pos];
          if (users[x].empty()) continue;
          // a reduction stays where its operand is computed: moved, it would read the operand again
          if (g->ops[x].opcode >= DISC_REDUCE_SUM && g->ops[x].opcode <= DISC_REDUCE_ARGMAX) continue;
          int to = -1;
          bool ok = true;
          for (int u : users[x]) {
            if (g->ops[u].opcode == DISC_OUTPUT || grp[u] <= (int)gi) { ok = false; break; }
            if (to >= 0 && grp[u] != to) { ok = false; break; }
            to = grp[u];
          }
          if (!ok || to < 0) continue;
          const int n = op_arity(g->ops[x]);
          for (int k = 0; k < n && ok; ++k) {
            const int a = g->ops[x].in[k];
            if (!is_leaf(g->ops[a].opcode) && grp[a] == (int)gi && !read_elsewhere(a, x)) ok = false;
          }
          if (!ok) continue;
          std::vector<int> bigger = cuts[to];
          bigger.insert(std::lower_bound(bigger.begin(), bigger.end(), x), x);
          if (fusible(bigger, &why) != DISC_OK) continue;
          std::vector<int> smaller = cuts[gi];
          smaller.erase(smaller.begin() + (long)pos);
          if (!smaller.empty() && fusible(smaller, &why) != DISC_OK) continue;
          cuts[to].swap(bigger);
          cuts[gi].swap(smaller);
          grp[x] = to;
          moved = true;
        }
      }
    }
    std::vector<std::vector<int>> kept;
    for (auto& c : cuts)
      if (!c.empty()) kept.push_back(c);
    cuts.swap(kept);
  }
  if (cuts.size() > (size_t)DISC_MAX_GRAPH_PATTERNS) return set_err(ctx, DISC_ERR_BAD_PATTERN, "the graph needs too many patterns");

  std::vector<FinalPattern> finals;
  {
    const int rc = finalize(cuts, &finals, &why);
    if (rc) return set_err(ctx, rc, "a cut of the graph is not a pattern: " + why);
  }
  for (size_t gi = 0; gi < cuts.size(); ++gi) {
    GraphGroup gr;
    gr.ops = cuts[gi];
    for (int v : gr.ops) g->group_of_op[v] = (int)gi;
    gr.in_values = finals[gi].in_values;
    gr.out_values = finals[gi].out_values;
    if (gr.out_values.empty()) { gr.pattern_id = -1; g->groups.push_back(gr); continue; }   // dead code: nothing reads it
    int32_t pid = -1;
    int rc = disc_register_pattern(ctx, finals[gi].ops.data(), (int)finals[gi].ops.size(),
                                   finals[gi].cs.empty() ? nullptr : finals[gi].cs.data(), (int)finals[gi].cs.size(), &pid);
    if (rc) return rc;
    gr.pattern_id = pid;
    g->groups.push_back(gr);
  }
  // drop groups nothing reads
  {
    std::vector<GraphGroup> kept;
    std::vector<int> renum(g->groups.size(), -1);
    for (size_t gi = 0; gi < g->groups.size(); ++gi)
      if (g->groups[gi].pattern_id >= 0) { renum[gi] = (int)kept.size(); kept.push_back(g->groups[gi]); }
    for (int& x : g->group_of_op)
      if (x >= 0) x = renum[x];
    g->groups.swap(kept);
  }
  if (g->groups.empty()) return set_err(ctx, DISC_ERR_BAD_PATTERN, "no output depends on a computed value");

  // values that cross pattern boundaries and are not graph outputs live in planned buffers
  for (size_t gi = 0; gi < g->groups.size(); ++gi)
    for (int v : g->groups[gi].out_values) {
      if (g->output_index.count(v)) continue;
      GraphIntermediate it;
      it.value = v;
      it.first = it.last = (int)gi;
      g->inter_of_value[v] = (int)g->inter.size();
      g->inter.push_back(it);
    }
  for (size_t gi = 0; gi < g->groups.size(); ++gi)
    for (int v : g->groups[gi].in_values) {
      auto it = g->inter_of_value.find(v);
      if (it != g->inter_of_value.end()) g->inter[it->second].last = std::max(g->inter[it->second].last, (int)gi);
    }
  // a buffer is reused by a later value of the same dtype size and the same symbolic shape once
  // its previous tenant has been read for the last time (Section 4.2.2: reuse by shape compatibility)
  {
    std::vector<int> free_after;          // per buffer: last group that reads its tenant
    std::vector<std::string> key_of;      // per buffer
    for (auto& it : g->inter) {
      const disc_op& o = g->ops[it.value];
      std::string key(1, (char)dtype_bytes(o.dtype));
      key.append(reinterpret_cast<const char*>(o.dim), sizeof(int32_t) * (size_t)o.rank);
      int pick = -1;
      for (size_t b = 0; b < key_of.size() && pick < 0; ++b)
        if (key_of[b] == key && free_after[b] < it.first) pick = (int)b;
      if (pick < 0) {
        pick = (int)key_of.size();
        key_of.push_back(key);
        free_after.push_back(it.last);
        g->buffer_value.push_back(it.value);
      } else {
        free_after[pick] = it.last;
      }
      it.buffer = pick;
    }
  }
  // the launch path looks nothing up: every operand of every pattern gets its place now
  for (auto& gr : g->groups) {
    auto place_of = [&](int v) -> std::pair<int, int> {
      auto pi = g->param_index.find(v);
      if (pi != g->param_index.end()) return {0, pi->second};
      auto oi = g->output_index.find(v);
      if (oi != g->output_index.end()) return {1, oi->second};
      auto it = g->inter_of_value.find(v);
      if (it != g->inter_of_value.end()) return {2, g->inter[it->second].buffer};
      return {-1, 0};
    };
    for (int v : gr.in_values) gr.in_place.push_back(place_of(v));
    for (int v : gr.out_values) gr.out_place.push_back(place_of(v));
    for (const auto& pl : gr.in_place)
      if (pl.first < 0) return set_err(ctx, DISC_ERR_INTERNAL, "a value of the graph has no place");
    for (const auto& pl : gr.out_place)
      if (pl.first < 0) return set_err(ctx, DISC_ERR_INTERNAL, "a value of the graph has no place");
    if (gr.in_place.size() > (size_t)DISC_MAX_OPS || gr.out_place.size() > (size_t)DISC_MAX_OPS)
      return set_err(ctx, DISC_ERR_BAD_PATTERN, "too many operands in one pattern of the graph");
  }
  if (g->buffer_value.size() > (size_t)DISC_MAX_OPS) return set_err(ctx, DISC_ERR_BAD_PATTERN, "too many buffers");
  const int id = (int)ctx->graphs.size();
  ctx->graphs.push_back(std::move(g));
  *graph_id_out = id;
  return DISC_OK;
  DISC_CATCH(ctx)
}

int disc_graph_info(disc_ctx* ctx, int32_t id, disc_graph_info_t* out) {
  DISC_TRY
  Graph* g = get_graph(ctx, id);
  if (!g || !out) return set_err(ctx, DISC_ERR_INVALID_ARG, "bad graph id or null output");
  memset(out, 0, sizeof *out);
  out->n_dims = g->n_sym;
  out->n_inputs = g->n_inputs;
  out->n_outputs = g->n_outputs;
  out->n_patterns = (int)g->groups.size();
  out->n_intermediates = (int)g->inter.size();
  out->n_buffers = (int)g->buffer_value.size();
  for (size_t i = 0; i < g->groups.size() && i < DISC_MAX_GRAPH_PATTERNS; ++i) {
    out->pattern_id[i] = g->groups[i].pattern_id;
    out->pattern_ops[i] = (int)g->groups[i].ops.size();
  }
  for (size_t i = 0; i < g->group_of_op.size() && i < DISC_MAX_OPS; ++i) out->group_of_op[i] = g->group_of_op[i];
  return DISC_OK;
  DISC_CATCH(ctx)
}

int disc_graph_workspace_bytes(disc_ctx* ctx, int32_t id, const int64_t* dims, int n_dims, size_t* out) {
  DISC_TRY
  Graph* g = get_graph(ctx, id);
  if (!g || !out) return set_err(ctx, DISC_ERR_INVALID_ARG, "bad graph id or null output");
  size_t off[DISC_MAX_OPS];
  size_t pws = 0;
  return graph_layout(ctx, *g, dims, n_dims, off, &pws, out);
  DISC_CATCH(ctx)
}

int disc_graph_launch(disc_ctx* ctx, int32_t id, const int64_t* dims, int n_dims, const void* const* inputs, int n_in,
                      void* const* outputs, int n_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  DISC_TRY
  Graph* g = get_graph(ctx, id);
  if (!g) return set_err(ctx, DISC_ERR_INVALID_ARG, "bad graph id");
  if (n_in != g->n_inputs || n_out != g->n_outputs) return set_err(ctx, DISC_ERR_INVALID_ARG, "wrong number of inputs or outputs");
  if ((n_in > 0 && !inputs) || !outputs) return set_err(ctx, DISC_ERR_INVALID_ARG, "null pointer array");
  // nothing is allocated and nothing looked up here: offsets and pointer arrays live on the stack,
  // the place of every operand was resolved at registration
  size_t off[DISC_MAX_OPS];
  size_t pws = 0, total = 0;
  int rc = graph_layout(ctx, *g, dims, n_dims, off, &pws, &total);
  if (rc) return rc;
  if (total > 0 && (!workspace || workspace_bytes < total)) return set_err(ctx, DISC_ERR_WORKSPACE, "workspace missing or too small");
  char* ws = static_cast<char*>(workspace);
  const void* in[DISC_MAX_OPS];
  void* outp[DISC_MAX_OPS];
  auto where = [&](const std::pair<int, int>& pl) -> void* {
    return pl.first == 0 ? const_cast<void*>(inputs[pl.second]) : pl.first == 1 ? outputs[pl.second] : ws + off[pl.second];
  };
  for (const auto& gr : g->groups) {
    const int ni = (int)gr.in_place.size(), no = (int)gr.out_place.size();
    for (int k = 0; k < ni; ++k) {
      in[k] = where(gr.in_place[k]);
      if (!in[k]) return set_err(ctx, DISC_ERR_INVALID_ARG, "null input pointer");
    }
    for (int k = 0; k < no; ++k) {
      outp[k] = where(gr.out_place[k]);
      if (!outp[k]) return set_err(ctx, DISC_ERR_INVALID_ARG, "null output pointer");
    }
    const int ns = ctx->patterns[gr.pattern_id]->an.n_sym;
    rc = disc_launch(ctx, gr.pattern_id, dims, ns, in, ni, outp, no, ws ? ws + pws : nullptr, total - pws, hip_stream);
    if (rc) return rc;
  }
  return DISC_OK;
  DISC_CATCH(ctx)
}

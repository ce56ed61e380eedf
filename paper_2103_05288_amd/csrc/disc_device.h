// disc_device.h -- hand-written, shape-generic kernel schedules for gfx950 (CDNA4).
//
// This header is compiled at pattern-registration time together with ONE generated
// `struct Pat` that holds the fused per-element expression of the pattern.  Everything
// that decides performance lives here and is written by hand: how rows are mapped to
// lanes, how data moves through registers / LDS, how reductions are combined.  The
// schedules never see a shape as a compile-time constant; every extent arrives in the
// kernel-argument block that the host fills at launch (the paper's host-side shape
// calculation and launch-dimension selection, Sections 4.2.1 and 4.3).  (The one exception is
// the single-shape module built for the gap-to-static comparison, see DISC_STATIC_ARGS.)
//
// The two templates of Section 4.3 -- loop fusion, and input fusion rooted at a reduction -- are
// kloop_kernel and the row_* / col_* kernels; each exists in
// several versions (vector / scalar access, 32 / 64-bit index, register-resident / streamed
// row, ...) which the host selects per incoming shape.
//
// Interface expected from the generated `Pat` (all members static, __device__, inlined):
//   struct Args            kernel-argument block (pointers, extents, fast-division constants)
//   struct RowCtx          per-row state: operand base offsets and per-row values
//   template<int V> struct Slot      V consecutive elements of every per-element operand
//   template<int V> struct OutSlot   V consecutive elements of every per-element output
//   row_begin(A,row,rc)                        fill RowCtx for `row` (loads per-row operands)
//   load<V>(A,rc,col,span,slot)                load a slot (span: elements of the slot inside the row)
//   template<int P> struct Acc                 accumulator of reduction phase P
//   acc_init<P>(acc)  acc_merge<P>(a,b)  acc_xchg<P,S>(acc)   (S: lane_xchg step)
//   template<int V> struct Keep                per-element values carried between phases
//   phase<P,V,KEEP>(A,acc,slot,keep,span,col,rc)   fold one slot into acc (row reduce);
//                                              KEEP=false recomputes instead of using `keep`
//   accum<P,V>(A,acc,slot,e,col,rc)            fold element e of a slot into acc (column reduce)
//   row_after<P>(A,rc,acc)                     per-row values that become known after phase P
//   epilogue<V,KEEP>(A,rc,slot,keep,col,span,out)  per-element results of all outputs
//   store<V>(A,rc,col,span,out)                store a slot of outputs
//   row_store(A,row,rc)                        store per-row outputs (one lane per row calls it)
//   NPHASE, MAX_ACC_BYTES
#pragma once

// A module specialised for one shape defines these before this header: they assign the shape's
// constants to the by-value kernel arguments, and the compiler folds them through the kernel.
#ifndef DISC_STATIC_ARGS
#define DISC_STATIC_ARGS(A)
#define DISC_STATIC_PLAN(rp)
#endif

namespace disc {

typedef unsigned char u8;
typedef unsigned short u16;
typedef unsigned int u32;
typedef long long i64;
typedef unsigned long long u64;

#define DISC_DEV __device__ __forceinline__

// ---------------------------------------------------------------------------------------
// Vectors of N storage elements, loaded and stored with ELEMENT alignment only.  gfx950
// runs with unaligned global access enabled, so the compiler still emits one wide access
// (global_load_dwordx4 for 16 bytes) and the hardware serves rows that start at any element.
// This is why no separate "aligned" kernel version is needed for rows whose length is not a
// multiple of the vector width.  The payload is a native vector value (never a byte copy
// into a struct), so it always lives in registers.
// ---------------------------------------------------------------------------------------
template <class T, int N, bool PACKED = (sizeof(T) == 1 && N >= 4)>
struct Vec {
  typedef T vec_t __attribute__((ext_vector_type(N)));
  typedef vec_t unaligned_t __attribute__((aligned(alignof(T))));
  vec_t v;
  DISC_DEV void clear() { v = vec_t(T(0)); }
  DISC_DEV T get(int e) const { return v[e]; }
  DISC_DEV void set(int e, T x) { v[e] = x; }
};
// One-byte elements are kept as whole 32-bit words: a vector of bytes is not a register type, and
// the compiler would carry it around loops one byte per register, packing and unpacking each time.
template <class T, int N>
struct Vec<T, N, true> {
  typedef unsigned vec_t __attribute__((ext_vector_type(N / 4)));
  typedef vec_t unaligned_t __attribute__((aligned(1)));
  vec_t v;
  DISC_DEV void clear() { v = vec_t(0u); }
  DISC_DEV T get(int e) const { return (T)((v[e / 4] >> (8 * (e % 4))) & 0xffu); }
  DISC_DEV void set(int e, T x) {   // the byte must still be zero (clear() first)
    v[e / 4] |= (unsigned)(unsigned char)x << (8 * (e % 4));
  }
};

// The first n elements of a slot belong to the row (n = N everywhere but at the end of a row).
// The per-element test e < n is made where it is used: keeping the 8 or 16 lane masks of every
// slot alive across the phases was measured slower -- they do not fit the scalar registers next
// to the kernel arguments and were spilled to vector-register lanes on every path.
struct Span {
  static constexpr bool kAnyColumn = false;
  int n;
  static DISC_DEV Span upto(int n) {
    Span s;
    s.n = n;
    return s;
  }
  DISC_DEV bool full(int N) const { return n >= N; }
  DISC_DEV bool has(int e) const { return e < n; }
  DISC_DEV bool any() const { return n > 0; }
};
// The span of a slot in a launch whose rows are a whole number of slots (row length a multiple of
// the vector width): a slot is either all inside the row or not there at all, which the compiler
// knows -- every ragged-tail path (predicated bodies, piecewise loads and stores, the wave-wide
// "all full?" vote) drops out of the kernel versions built on it.
struct EvenSpan {
  static constexpr bool kAnyColumn = false;
  int n;
  static DISC_DEV EvenSpan upto(int n) {
    EvenSpan s;
    s.n = n;
    return s;
  }
  DISC_DEV bool full(int) const { return true; }
  DISC_DEV bool has(int) const { return true; }
  DISC_DEV bool any() const { return n > 0; }
};

// Element offset of a slot relative to the base row of the access.  A caller that passes the
// column as `unsigned` promises that lane_base + col, scaled to bytes, fits 32 bits (the
// register-resident row kernels: a wavefront's rows span at most 3 * 1024 slots); the access can
// then use a scalar base register plus a 32-bit lane offset.  Any other column type: 64 bits.
DISC_DEV unsigned off(int lane_base, unsigned col) { return (unsigned)lane_base + col; }
DISC_DEV i64 off(int lane_base, int col) { return (i64)lane_base + col; }
DISC_DEV i64 off(int lane_base, i64 col) { return lane_base + col; }

// A ragged slot (n < N elements) moves as the power-of-two pieces of n's binary expansion: the
// piece of width W covers [(q-1)W, qW) when n / W == q is odd.  Every lane of a launch has the
// same ragged length, so a wavefront issues at most log2(N) narrow accesses per ragged slot.
template <int W, class T, int N, class I>
DISC_DEV void ld_pieces(Vec<T, N>& d, const T* __restrict__ p, I off, int n) {
  if constexpr (W >= 1) {
#pragma unroll
    for (int q = 1; q * W < N; q += 2)
      if (n / W == q) {
        Vec<T, W> piece;
        piece.v = *reinterpret_cast<const typename Vec<T, W>::unaligned_t*>(p + off + (q - 1) * W);
#pragma unroll
        for (int i = 0; i < W; ++i) d.set((q - 1) * W + i, piece.get(i));
      }
    ld_pieces<W / 2>(d, p, off, n);
  }
}
template <int W, class T, int N, class I>
DISC_DEV void st_pieces(T* __restrict__ p, I off, const Vec<T, N>& s, int n) {
  if constexpr (W >= 1) {
#pragma unroll
    for (int q = 1; q * W < N; q += 2)
      if (n / W == q) {
        Vec<T, W> piece;
        piece.clear();
#pragma unroll
        for (int i = 0; i < W; ++i) piece.set(i, s.get((q - 1) * W + i));
        *reinterpret_cast<typename Vec<T, W>::unaligned_t*>(p + off + (q - 1) * W) = piece.v;
      }
    st_pieces<W / 2>(p, off, s, n);
  }
}

// `whole_ok`: all N elements lie inside the tensor even though only part of them belong to this
// row (the rest are the tail of the previous / head of the next row).  Then the wide load is
// still taken and the caller ignores the surplus elements; only a slot that would leave the
// tensor is read element by element.  This keeps ragged rows on the wide-load path.
// address of element `off` of p; a 32-bit unsigned offset is scaled in 32 bits, so that the
// address is base + zero-extended byte offset -- the form that takes a scalar base register
template <class T, class I>
DISC_DEV const T* at(const T* p, I off) {
  if constexpr (__is_same(I, unsigned))
    return reinterpret_cast<const T*>(reinterpret_cast<const char*>(p) + (unsigned)(off * (unsigned)sizeof(T)));
  else
    return p + off;
}
template <class T, class I>
DISC_DEV T* at(T* p, I off) {
  return const_cast<T*>(at(const_cast<const T*>(p), off));
}

// NT: non-temporal access, a compile-time constant of the kernel version (a run-time choice
// between the two accesses is merged into one plain access by the optimiser).  For operands
// and results that are touched exactly once the hint keeps them from displacing each other in the
// L2 and the memory-side cache; the host picks the version per launch (the hint hurts short or
// misaligned rows, whose cache lines are shared by neighbouring rows and so ARE touched twice).
template <bool NT = false, class T, int N, class I, class SP>
DISC_DEV void ld(Vec<T, N>& d, const T* __restrict__ p, I off, SP sp, bool whole_ok = false) {
  if (sp.full(N) || whole_ok) {
    const auto* q = reinterpret_cast<const typename Vec<T, N>::unaligned_t*>(at(p, off));
    if constexpr (NT) d.v = __builtin_nontemporal_load(q);
    else d.v = *q;
  } else {
    d.clear();
    ld_pieces<N / 2>(d, p, off, sp.n);
    // s_waitcnt vmcnt(0): the pieces are complete before the branches rejoin.  Otherwise the
    // compiler has to assume a piece may still be in flight into d's registers and makes the
    // wide load above wait for every earlier load of the wavefront -- on the path where no
    // lane took this branch at all, serialising the loads of full slots.
    __builtin_amdgcn_s_waitcnt(0x0F70);
  }
}

template <bool NT = false, class T, int N, class I, class SP>
DISC_DEV void st(T* __restrict__ p, I off, const Vec<T, N>& s, SP sp) {
  if (sp.full(N)) {
    auto* q = reinterpret_cast<typename Vec<T, N>::unaligned_t*>(at(p, off));
    if constexpr (NT) __builtin_nontemporal_store(s.v, q);
    else *q = s.v;
  } else {
    st_pieces<N / 2>(p, off, s, sp.n);
  }
}

// Slot of a padded operand: elements whose column lies in [wlo, whi) of a row that lies inside the
// operand (row_ok) come from memory, the others are the padding value.  A slot wholly inside
// takes the ordinary wide load; one that straddles an edge of the operand is read element by
// element (two slots per row at most).
template <class T>
DISC_DEV T pad_const(float x) {
  if constexpr (sizeof(T) == 1) return (T)(x != 0.0f);
  else return (T)x;
}
template <class T, int N, class I, class SP>
DISC_DEV void ld_win(Vec<T, N>& d, const T* __restrict__ p, I off, SP sp, i64 col, bool row_ok, i64 wlo, i64 whi, T padv) {
  const i64 lo = wlo - col, hi = whi - col;        // the operand's columns in slot coordinates
  if (row_ok && lo <= 0 && hi >= sp.n) {
    ld(d, p, off, sp);
  } else {
    d.clear();
#pragma unroll
    for (int e = 0; e < N; ++e) {
      T x = padv;
      if (row_ok && sp.has(e) && e >= lo && e < hi) x = at(p, off)[e];
      d.set(e, x);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
  }
}

// Slot of an operand read one element earlier: d[e] = p[off + e - 1].  The very first slot of the
// tensor (off == 0) has no element in front of it: its element 0 stays zero (the caller never looks
// at it) and the rest is read one by one.
template <class T, int N, class SP>
DISC_DEV void ld_prev(Vec<T, N>& d, const T* __restrict__ p, i64 off, SP sp) {
  if (off > 0) {
    ld(d, p, off - 1, sp);
  } else {
    d.clear();
#pragma unroll
    for (int e = 1; e < N; ++e)
      if (sp.has(e)) d.set(e, p[e - 1]);
    __builtin_amdgcn_s_waitcnt(0x0F70);
  }
}

// storage <-> register conversions (float values live in fp32 registers; one rounding,
// to nearest even, at the store)
DISC_DEV float to_f32(float x) { return x; }
DISC_DEV float to_f32(_Float16 x) { return (float)x; }
DISC_DEV float to_f32(__bf16 x) { return (float)x; }
DISC_DEV float to_f32(int x) { return (float)x; }
DISC_DEV float to_f32(i64 x) { return (float)x; }
DISC_DEV float to_f32(bool x) { return x ? 1.f : 0.f; }
template <class T> DISC_DEV T from_f32(float x);
template <> DISC_DEV float from_f32<float>(float x) { return x; }
template <> DISC_DEV _Float16 from_f32<_Float16>(float x) { return (_Float16)x; }
template <> DISC_DEV __bf16 from_f32<__bf16>(float x) { return (__bf16)x; }

// fp32 results -> storage vector, two elements per conversion where the type has a packed
// convert (v_cvt_pk_bf16_f32 on gfx950 rounds to nearest even and delivers the packed pair)
template <class T, int N>
DISC_DEV void cvt_vec(Vec<T, N>& d, const float (&y)[N]) {
  if constexpr (N % 2 == 0 && sizeof(T) == 2) {
    typedef float f2 __attribute__((ext_vector_type(2)));
    typedef T t2 __attribute__((ext_vector_type(2)));
#pragma unroll
    for (int e = 0; e < N; e += 2) {
      const f2 p = {y[e], y[e + 1]};
      const t2 q = __builtin_convertvector(p, t2);
      d.v[e] = q[0];
      d.v[e + 1] = q[1];
    }
  } else {
#pragma unroll
    for (int e = 0; e < N; ++e) d.v[e] = from_f32<T>(y[e]);
  }
}

// Per-element transcendental math on the hardware approximation units (about 1 ulp each):
// the fused kernels have roughly 40 VALU lane-operations per element to spend before they stop
// being HBM-bound, which IEEE-correct expf / division would use up several times over.
DISC_DEV float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }
DISC_DEV float fast_rsqrt(float x) { return __builtin_amdgcn_rsqf(x); }
DISC_DEV float fast_sqrt(float x) { return __builtin_amdgcn_sqrtf(x); }
DISC_DEV float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
DISC_DEV float fast_exp(float x) { return __builtin_amdgcn_exp2f(x * 1.44269504088896341f); }
DISC_DEV float fast_log(float x) { return __builtin_amdgcn_logf(x) * 0.693147180559945309f; }
DISC_DEV float fast_sigmoid(float x) { return fast_rcp(1.0f + fast_exp(-x)); }
// tanh(x) = 1 - 2 / (exp(2x) + 1): exact limits at +-inf, absolute error ~1e-7 everywhere
DISC_DEV float fast_tanh(float x) { return 1.0f - 2.0f * fast_rcp(fast_exp(2.0f * x) + 1.0f); }

// ---------------------------------------------------------------------------------------
// Division by a runtime extent with constants the host precomputes from the shape
// (round-up multiply-shift method of Granlund & Montgomery): for 0 <= n < 2^31,
//   n / d == (umulhi(n, m) + n) >> s   with s = ceil(log2 d), m = floor(2^32 (2^s - d) / d) + 1.
// ---------------------------------------------------------------------------------------
struct FastDiv {
  u32 d, m, s, pad;
};
DISC_DEV u32 fdiv(u32 n, const FastDiv& f) { return (__umulhi(n, f.m) + n) >> f.s; }

// ---------------------------------------------------------------------------------------
// Cross-lane exchange inside a 64-wide wavefront, all on the VALU (no LDS crossbar):
// lane_xchg<S>(v) returns v of a partner lane such that combining a value with its partner
// for S = 1, 2, 4, 8, 16, 32 in turn leaves every lane of each aligned 2S-lane group with
// the combination of the whole group.  S = 1, 2: DPP quad permutes; S = 4, 8: DPP mirror
// within 8 / 16 lanes (after the quad steps every quad is uniform, so mirroring pairs the
// right quads); S = 16, 32: gfx950's permlane16 / permlane32 swaps, called with both operands
// equal, which hand back the partner row / half as the second result.
// ---------------------------------------------------------------------------------------
template <int S>
DISC_DEV u32 lane_xchg_u32(u32 v) {
  if constexpr (S == 1) return (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xf, 0xf, true);        // quad_perm [1,0,3,2]
  else if constexpr (S == 2) return (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xf, 0xf, true);   // quad_perm [2,3,0,1]
  else if constexpr (S == 4) return (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xf, 0xf, true);  // row_half_mirror
  else if constexpr (S == 8) return (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xf, 0xf, true);  // row_mirror
  else if constexpr (S == 16) {
    auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    const bool odd_row = (threadIdx.x >> 4) & 1;
    return odd_row ? r[0] : r[1];
  } else {
    auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    const bool upper = (threadIdx.x >> 5) & 1;
    return upper ? r[0] : r[1];
  }
}
template <int S> DISC_DEV float lane_xchg(float v) { return __builtin_bit_cast(float, lane_xchg_u32<S>(__builtin_bit_cast(u32, v))); }
template <int S> DISC_DEV int lane_xchg(int v) { return (int)lane_xchg_u32<S>((u32)v); }
template <int S> DISC_DEV i64 lane_xchg(i64 v) {
  const u32 lo = lane_xchg_u32<S>((u32)(u64)v), hi = lane_xchg_u32<S>((u32)((u64)v >> 32));
  return (i64)(((u64)hi << 32) | lo);
}
template <int S> DISC_DEV double lane_xchg(double v) { return __builtin_bit_cast(double, lane_xchg<S>(__builtin_bit_cast(i64, v))); }

// true when the predicate holds in every active lane of the wavefront (scalar result)
DISC_DEV bool wave_all(bool p) { return __builtin_amdgcn_ballot_w64(!p) == 0; }

// all-reduce of an accumulator over aligned groups of G lanes (G a power of two, <= 64)
template <class Pat, int P, int S>
DISC_DEV void group_step(typename Pat::template Acc<P>& acc) {
  typename Pat::template Acc<P> o = acc;
  Pat::template acc_xchg<P, S>(o);
  Pat::template acc_merge<P>(acc, o);
}
// nested on purpose: one scalar test per level, nothing re-derived after the branches rejoin.
// The empty asm makes G opaque at each call: the tests are then scalar compares at the point of
// use; otherwise the compiler evaluates all six once per kernel and keeps them as lane masks in
// twelve scalar registers across the row loop, which does not have them to spare.
template <class Pat, int P>
DISC_DEV void group_allreduce(typename Pat::template Acc<P>& acc, int G) {
  asm volatile("" : "+s"(G));
  if (G > 1) {
    group_step<Pat, P, 1>(acc);
    if (G > 2) {
      group_step<Pat, P, 2>(acc);
      if (G > 4) {
        group_step<Pat, P, 4>(acc);
        if (G > 8) {
          group_step<Pat, P, 8>(acc);
          if (G > 16) {
            group_step<Pat, P, 16>(acc);
            if (G > 32) group_step<Pat, P, 32>(acc);
          }
        }
      }
    }
  }
}

// =======================================================================================
// Loop fusion (kLoop).  The iteration space is [rows, inner]; it is cut into slots of V
// consecutive elements of one row.  Consecutive lanes take consecutive slots, so every wave
// reads and writes one contiguous stretch of memory whatever `inner` is; a block walks the
// slot list with a grid stride, U slots in flight per lane to keep enough bytes in flight
// for HBM.  (row, col) of a slot come from one multiply-shift division per slot.
// =======================================================================================
// NT: bit 0 = non-temporal loads of the full-size operands, bit 1 = non-temporal stores
template <class Pat, int V, int U, bool I64, int NT = 0>
DISC_DEV void kloop_body(const typename Pat::Args& A) {
  if constexpr (!I64) {
    const u32 nslots = (u32)A.nslots;
    const u32 stride = gridDim.x * blockDim.x;
    const u32 inner = (u32)A.inner;
    for (u32 s0 = blockIdx.x * blockDim.x + threadIdx.x; s0 < nslots; s0 += stride * U) {
      typename Pat::template Slot<V> slot[U];
      typename Pat::RowCtx rc[U];
      int col[U], nv[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const u32 s = s0 + u * stride;
        nv[u] = 0;
        if (s < nslots) {
          const u32 row = fdiv(s, A.spr_div);
          col[u] = (int)((s - row * A.spr_div.d) * V);
          nv[u] = min((int)V, (int)(inner - (u32)col[u]));
          Pat::row_begin(A, (i64)row, rc[u]);
          Pat::template load<V, NT>(A, rc[u], col[u], Span::upto(nv[u]), slot[u]);
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (nv[u] > 0) {
          typename Pat::template OutSlot<V> o;
          typename Pat::template Keep<V> kp;
          Pat::template epilogue<V, false>(A, rc[u], slot[u], kp, col[u], Span::upto(nv[u]), o);
          Pat::template store<V, NT>(A, rc[u], col[u], Span::upto(nv[u]), o);
        }
      }
    }
  } else {
    const i64 nslots = A.nslots;
    const i64 stride = (i64)gridDim.x * blockDim.x;
    const i64 spr = A.spr;
    for (i64 s = (i64)blockIdx.x * blockDim.x + threadIdx.x; s < nslots; s += stride) {
      const i64 row = s / spr;
      const i64 col = (s - row * spr) * V;
      const i64 rem = A.inner - col;
      const int nv = rem < (i64)V ? (int)rem : V;
      typename Pat::template Slot<V> slot;
      typename Pat::RowCtx rc;
      Pat::row_begin(A, row, rc);
      Pat::template load<V, NT>(A, rc, col, Span::upto(nv), slot);
      typename Pat::template OutSlot<V> o;
      typename Pat::template Keep<V> kp;
      Pat::template epilogue<V, false>(A, rc, slot, kp, col, Span::upto(nv), o);
      Pat::template store<V, NT>(A, rc, col, Span::upto(nv), o);
    }
  }
}

// =======================================================================================
// Input fusion with a row reduction as root (kInput, reduce over the innermost axis).
//
// Register-resident version: a row is owned by a group of G lanes chosen by the host per shape:
// a power of two 1..32 = several rows per wavefront for short rows, 64 = a wavefront per row,
// a multiple of 64 up to 1024 = G/64 wavefronts per row (the host picks block sizes whose
// wavefront count is a multiple of four, so the four SIMDs of a CU get equal shares).  Lane l of the group holds
// slots l, l+G, l+2G, ... (NV of them, V elements each), loaded ONCE; every reduction phase
// and the epilogue run out of registers, so the row makes exactly one trip from HBM and one
// back.  Within a wavefront partial results are combined with xor-shuffles; across the
// wavefronts of a row through a double-buffered LDS exchange (one barrier per phase).
// =======================================================================================
// The span of a slot in the kernel versions that take the ragged ends of a row as single elements:
// whole like EvenSpan, but the slot may start at ANY column (the vector slots of a row may be
// shifted to 16-byte boundaries of memory, and single elements sit anywhere), so copies of row
// vectors in LDS are read with element alignment only.
struct TailSpan : EvenSpan {
  static constexpr bool kAnyColumn = true;
  static DISC_DEV TailSpan upto(int n) {
    TailSpan s;
    s.n = n;
    return s;
  }
};
template <bool EVEN, bool TAIL = false> struct SpanSel { typedef Span type; };
template <> struct SpanSel<true, false> { typedef EvenSpan type; };
template <> struct SpanSel<true, true> { typedef TailSpan type; };
struct RowPlan {
  int G;        // lanes per row: a power of two <= 64, or a multiple of 64 (whole wavefronts)
  int log2G;    // meaningful for G <= 64
  int nv;       // slots per lane actually needed at this shape (<= NV of the instantiation)
  int flags;    // bit 0: the launched kernel is the version that stages row-vector operands in LDS
                // bit 1: the slot grid is not turned from row to row
                // bit 2: (_t versions) vector slots on the V-element boundaries of the tensor
  int rpb;      // rows per block = blockDim.x / G
};

// Row-vector operands (bias, gamma, beta, ...) are the same for every row a block processes:
// when the host grants the LDS, each block copies them once into dynamic LDS, padded with V
// zero elements, and every slot reads them from there with one aligned LDS vector read --
// no per-slot trip through the vector memory pipeline and no ragged-tail path for them.
extern __shared__ __attribute__((aligned(16))) char disc_stage_lds[];

// cooperative copy of n elements (+ pad zero elements) into LDS: 16-byte pieces, then the tail
template <int PAD, class T>
DISC_DEV void stage_copy(T* dst, const T* __restrict__ src, int n, int tid, int nthreads) {
  constexpr int E = 16 / (int)sizeof(T);
  const int nvec = n / E;
  for (int i = tid; i < nvec; i += nthreads)
    reinterpret_cast<typename Vec<T, E>::vec_t*>(dst)[i] =
        *reinterpret_cast<const typename Vec<T, E>::unaligned_t*>(src + (i64)i * E);
  for (int i = nvec * E + tid; i < n + PAD; i += nthreads) dst[i] = i < n ? src[i] : T(0);
}

// each staged operand is stored as [inner elements | zeros]; col is a multiple of N, or (ANY) any
// column, read with element alignment
template <bool ANY = false, class T, int N>
DISC_DEV void ld_lds(Vec<T, N>& d, const char* base, int byte_off, int col) {
  const char* q = base + byte_off + col * (int)sizeof(T);
  if constexpr (ANY) d.v = *reinterpret_cast<const typename Vec<T, N>::unaligned_t*>(q);
  else d.v = *reinterpret_cast<const typename Vec<T, N>::vec_t*>(q);
}

// Sums over the rows carried along by a row reduce (Pat::NCOLSUM of them): every lane adds the
// values of its own columns, row after row, into fp32 registers; at the end of the kernel each
// wavefront (rows of at most a wavefront) or lane group (longer rows) writes one row of partial
// sums per summed output into the workspace, plane q at ws + q * n_partial_rows * inner, and a
// second launch adds the partial rows up in a fixed order.
DISC_DEV float lane_xor_f32(float v, int s) {
  const int lane = (int)threadIdx.x & 63;
  return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((lane ^ s) << 2, __builtin_bit_cast(int, v)));
}

// The end of a row behind its last whole slot, taken as slots of ONE element by the first lanes of
// the row (TAIL versions of the row kernels): the lane's element, what it keeps between the
// phases, and its column (-1: this lane has none).
template <class Pat>
struct TailSlot {
  typename Pat::template Slot<1> s;
  typename Pat::template Keep<1> k;
  int col;
};
struct NoTail {
  int col;
};
template <class Pat, bool TAIL>
struct TailSel {
  typedef NoTail type;
};
template <class Pat>
struct TailSel<Pat, true> {
  typedef TailSlot<Pat> type;
};

// `after_first` runs once, after the slots have been folded into the accumulator of phase 0 and
// before the lanes combine: the place where the caller issues the loads of the next row.
template <class Pat, int P, int V, int NV, class Hook, class SP, class TS>
DISC_DEV void row_phases(const typename Pat::Args& A, const RowPlan& rp, typename Pat::RowCtx& rc,
                         const typename Pat::template Slot<V> (&slot)[NV],
                         typename Pat::template Keep<V> (&keep)[NV], const SP (&span)[NV],
                         int col0, char* lds, int& parity, Hook& after_first, TS& ts) {
  if constexpr (P < Pat::NPHASE) {
    typename Pat::template Acc<P> acc;
    Pat::template acc_init<P>(acc);
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int col = col0 + j * rp.G * V;
      if (span[j].any()) Pat::template phase<P, V, true>(A, acc, slot[j], keep[j], span[j], col, rc);
    }
    if constexpr (!__is_same(TS, NoTail)) {
      if (ts.col >= 0) Pat::template phase<P, 1, true>(A, acc, ts.s, ts.k, TailSpan::upto(1), ts.col, rc);
    }
    if constexpr (P == 0) after_first();
    // lanes of one wavefront
    group_allreduce<Pat, P>(acc, rp.G < 64 ? rp.G : 64);
    // wavefronts of one row
    if (rp.G > 64) {
      typedef typename Pat::template Acc<P> AccT;
      AccT* ex = reinterpret_cast<AccT*>(lds + parity * 16 * Pat::MAX_ACC_BYTES);
      parity ^= 1;
      const int wave = threadIdx.x >> 6;
      if ((threadIdx.x & 63) == 0) ex[wave] = acc;
      __syncthreads();
      const int wpr = rp.G >> 6;               // wavefronts per row
      const int w0 = (wave / wpr) * wpr;       // first wavefront of this row
      if ((wpr & (wpr - 1)) == 0) {
        // every lane fetches one partial (lane i the one of wavefront i mod wpr) and the lanes
        // combine them with the butterfly: one LDS read instead of a chain of wpr dependent ones
        acc = ex[w0 + ((int)threadIdx.x & (wpr - 1))];
        group_allreduce<Pat, P>(acc, wpr);
      } else {
        acc = ex[w0];
        for (int w = 1; w < wpr; ++w) {
          AccT o = ex[w0 + w];
          Pat::template acc_merge<P>(acc, o);
        }
      }
    }
    Pat::template row_after<P>(A, rc, acc);
    row_phases<Pat, P + 1, V, NV>(A, rp, rc, slot, keep, span, col0, lds, parity, after_first, ts);
  }
}

// NT: bit 0 = non-temporal loads of the full-size operands, bit 1 = non-temporal stores
// EVEN: every vector slot is whole -- the host promises that the row length is a multiple of V, or
// TAIL: (with EVEN) the elements behind the last whole slot of a row, inner % V of them, are taken
//       one per lane by the lanes that hold the row's first columns, as slots of ONE element that
//       go through the same phases, the same accumulators and the same epilogue.  Against a
//       ragged last slot this costs one element's work in one wavefront of the row instead of a
//       predicated pass over a whole slot in every lane of that wavefront, no access moves in
//       pieces, and the row needs capacity for its whole slots only.  Needs G >= V lanes per row.
template <class Pat, int V, int NV, bool PIPE = true, int NT = 0, bool EVEN = false, bool TAIL = false>
DISC_DEV void row_reg_body(const typename Pat::Args& A, const RowPlan& rp) {
  static_assert(!TAIL || (EVEN && Pat::NCOLSUM == 0), "single-element tails: whole vector slots, no sums over the rows");
  typedef typename SpanSel<EVEN, TAIL>::type SP;
  __shared__ __attribute__((aligned(16))) char lds[2 * 16 * Pat::MAX_ACC_BYTES];
  // G <= 64: a power of two; G > 64: a multiple of 64
  const int grp = rp.G <= 64 ? (int)threadIdx.x >> rp.log2G : ((int)threadIdx.x >> 6) / (rp.G >> 6);
  const int lane = (int)threadIdx.x - grp * rp.G;
  const int rpb = rp.rpb;
  const i64 rows = A.rows;
  const int inner = (int)A.inner;
  int parity = 0;
  const char* staged = nullptr;
  if constexpr (Pat::STAGED) {
    Pat::template stage<V>(A, disc_stage_lds, threadIdx.x, blockDim.x);
    __syncthreads();
    staged = disc_stage_lds;
  }
  // A group past the last row (last block, several rows per block) works on the last row again
  // and stores nothing, so that no branch depends on it.
  //
  // Rows of several wavefronts: the wavefront that gets the ragged extra slots of a row does up
  // to twice the work of the others, and it would always be the first one -- on the same SIMD
  // of the CU for every row.  The slot grid is therefore turned by one wavefront from row to
  // row (lane l takes the columns of lane l + rot), which spreads the extra work evenly.
  // (a lane that sums its columns over the rows keeps its columns: no turning then)
  const int wpr = (Pat::NCOLSUM == 0 && rp.G > 64 && !(rp.flags & 2)) ? rp.G >> 6 : 1;   // flags bit 1: grid not turned (experiments)
  int rot = wpr > 1 ? (int)(blockIdx.x % (unsigned)wpr) * 64 : 0;
  // Row bookkeeping in scalar registers: rw = row of the first lane group of this wavefront in
  // the current row group, sbw = its element offset; both advance by a constant per iteration
  // (no 64-bit products in the loop).  A lane's row is rw + dgrp.
  const int grp_w = __builtin_amdgcn_readfirstlane(grp);
  const int dgrp = grp - grp_w;
  const i64 rstep = (i64)gridDim.x * rpb;
  const i64 sbstep = rstep * A.inner;
  i64 rw = (i64)blockIdx.x * rpb + grp_w;
  i64 sbw = rw * A.inner;
  // TAIL versions, flags bit 2: the vector slots of a row are shifted to the V-element boundaries
  // of the TENSOR (row * inner + column a multiple of V), so that every wide access of a full-size
  // operand whose base is aligned is aligned itself, whatever the row length: the `head` elements
  // in front of the first boundary are single elements like those behind the last whole slot.
  // The host launches a grid that puts rows of equal alignment on a lane group (the distance
  // between its rows times the row length is a multiple of V), so `head` is worked out once.  It is
  // an alignment matter only: any value 0 .. V-1 addresses the row correctly.
  int head = 0;
  if constexpr (TAIL) {
    if (rp.flags & 4) {
      const i64 r = rw + dgrp < rows ? rw + dgrp : rows - 1;
      const int e0 = (int)(((r & (V - 1)) * (i64)(inner & (V - 1))) & (V - 1));   // (row * inner) mod V
      head = (V - e0) & (V - 1);
    }
  }
  int col0 = lane * V;
  int nvalid[NV];
  int tcol = -1;                        // column of this lane's single element (TAIL versions), -1: none
  auto place = [&](int r, int& c0, int (&n)[NV], int& tc) {
    int l = lane + r;
    if (l >= rp.G) l -= rp.G;
    if constexpr (TAIL) {
      // [head single elements | whole slots | single elements behind them]
      const int whole = (inner - head) / V;
      const int behind = head + whole * V;         // first column behind the whole slots
      c0 = head + l * V;
#pragma unroll
      for (int j = 0; j < NV; ++j) n[j] = (j < rp.nv && l + j * rp.G < whole) ? V : 0;
      tc = l < head ? (l < inner ? l : -1) : (behind + (l - head) < inner ? behind + (l - head) : -1);
    } else {
      c0 = l * V;
      tc = -1;
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        const int col = c0 + j * rp.G * V;
        const int hi = inner - col > V ? V : inner - col;
        n[j] = (j < rp.nv && hi > 0) ? hi : 0;
      }
    }
  };
  place(rot, col0, nvalid, tcol);
  // Software pipeline over the rows of a block: the loads of the next row are issued as soon as
  // the first reduction phase has consumed the current row's slots (every load issued so far
  // has landed by then, so no wait in the rest of the iteration touches the new loads); they
  // complete behind the lane reductions, the later phases, the epilogue and the stores.
  typename Pat::RowCtx rc{};
  typename Pat::template Slot<V> slot[NV];
  typedef typename TailSel<Pat, TAIL>::type TS;
  TS ts, tsn;
  typename Pat::template ColAcc<V> cacc[NV]{};
  // reductions of per-row values over the rows: every lane of a lane group keeps the running values
  // of the group's rows
  float racc[Pat::NROWRED > 0 ? Pat::NROWRED : 1];
  if constexpr (Pat::NROWRED > 0) {
#pragma unroll
    for (int q = 0; q < Pat::NROWRED; ++q) racc[q] = Pat::rr_identity(q);
  }
  // rows past the end (last row group only) are replaced by the last row; their lanes compute
  // along and store nothing
  auto begin_row = [&](i64 rwv, i64 sbv, typename Pat::RowCtx& c) {
    if (rwv + (rpb - grp_w) <= rows) {
      Pat::row_begin3(A, rwv, dgrp, sbv, c);
    } else {
      const i64 last = rows - 1;
      const i64 b = rwv < last ? rwv : last;
      const i64 r = rwv + dgrp < last ? rwv + dgrp : last;
      Pat::row_begin3(A, b, (int)(r - b), b * A.inner, c);
    }
  };
  auto load_row = [&]() {
    begin_row(rw, sbw, rc);
    rc.sl = staged;
#pragma unroll
    for (int j = 0; j < NV; ++j)
      if (nvalid[j] > 0) Pat::template load<V, NT>(A, rc, (unsigned)(col0 + j * rp.G * V), SP::upto(nvalid[j]), slot[j]);
    if constexpr (TAIL) {
      ts.col = tcol;
      if (tcol >= 0) Pat::template load<1, 0>(A, rc, (unsigned)tcol, TailSpan::upto(1), ts.s);
    }
  };
  // the row group of the block starts at row rw - grp_w; the block is done when that is past the end
  if (PIPE && rw - grp_w < rows) load_row();
  while (rw - grp_w < rows) {
    if constexpr (!PIPE) load_row();
    SP span[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) span[j] = SP::upto(nvalid[j]);
    const i64 row = rw + dgrp;
    const bool active = row < rows;
    typename Pat::RowCtx rcn{};
    typename Pat::template Slot<V> nxt[NV];
    int col0n = col0, tcoln = tcol;
    int nvalidn[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) nvalidn[j] = nvalid[j];
    auto prefetch = [&]() {
      if (PIPE && rw + rstep - grp_w < rows) {
        if (wpr > 1) {
          rot = rot + 64 < rp.G ? rot + 64 : 0;
          place(rot, col0n, nvalidn, tcoln);
        }
        begin_row(rw + rstep, sbw + sbstep, rcn);
        rcn.sl = staged;
#pragma unroll
        for (int j = 0; j < NV; ++j)
          if (nvalidn[j] > 0) {
            SP sn;              // the loads look at the element count only
            sn.n = nvalidn[j];
            Pat::template load<V, NT>(A, rcn, (unsigned)(col0n + j * rp.G * V), sn, nxt[j]);
          }
        if constexpr (TAIL) {
          tsn.col = tcoln;
          if (tcoln >= 0) Pat::template load<1, 0>(A, rcn, (unsigned)tcoln, TailSpan::upto(1), tsn.s);
        }
      }
      // keep the loads here: without a fence the compiler is free to sink them below the
      // stores of this row (to save registers), which undoes the pipeline
      asm volatile("" ::: "memory");
    };
    typename Pat::template Keep<V> keep[NV];
    row_phases<Pat, 0, V, NV>(A, rp, rc, slot, keep, span, col0, lds, parity, prefetch, ts);
    if constexpr (Pat::NPHASE == 0) prefetch();   // (no reduction phase to hide the next row's loads behind)
    if constexpr (Pat::NROWRED > 0) {
      if (active) Pat::row_reds(A, rc, racc);
    }
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      if (span[j].any()) {
        const int col = col0 + j * rp.G * V;
        typename Pat::template OutSlot<V> o;
        Pat::template epilogue<V, true>(A, rc, slot[j], keep[j], col, span[j], o);
        // Loads and stores share one in-order counter, and with both kinds in flight the only
        // wait the compiler can express is "all of them".  Waiting for the next row's loads HERE,
        // before the first store of this row (they were issued a reduction phase ago and have
        // landed), means the first use of those loads in the next iteration needs no wait at all
        // -- otherwise that wait sits right behind these stores and exposes their full latency
        // in every iteration.  The stores then have a whole iteration to drain.
        if (PIPE && j == 0) __builtin_amdgcn_s_waitcnt(0x0F70);
        if (active) Pat::template store<V, NT>(A, rc, (unsigned)col, span[j], o);
        if constexpr (Pat::NCOLSUM > 0) {
          if (active) Pat::template col_sums<V, true>(A, rc, slot[j], keep[j], col, span[j], cacc[j]);
        }
      }
    }
    if constexpr (TAIL) {
      if (ts.col >= 0) {
        typename Pat::template OutSlot<1> o;
        Pat::template epilogue<1, true>(A, rc, ts.s, ts.k, ts.col, TailSpan::upto(1), o);
        if (active) Pat::template store<1, 0>(A, rc, (unsigned)ts.col, TailSpan::upto(1), o);
      }
    }
    if (active && lane == 0) Pat::row_store(A, row, rc);
    rw += rstep;
    sbw += sbstep;
    if constexpr (PIPE) {
      rc = rcn;
#pragma unroll
      for (int j = 0; j < NV; ++j) slot[j] = nxt[j];
      if constexpr (TAIL) ts = tsn;
      if (wpr > 1) {
        col0 = col0n;
        tcol = tcoln;
#pragma unroll
        for (int j = 0; j < NV; ++j) nvalid[j] = nvalidn[j];
      }
    } else if (wpr > 1) {
      rot = rot + 64 < rp.G ? rot + 64 : 0;
      place(rot, col0, nvalid, tcol);
    }
  }
  if constexpr (Pat::NCOLSUM > 0) {
    // lane groups of one wavefront hold the same columns: add them up across the groups
    if (rp.G < 64) {
#pragma unroll
      for (int j = 0; j < NV; ++j)
#pragma unroll
        for (int q = 0; q < Pat::NCOLSUM; ++q)
#pragma unroll
          for (int e = 0; e < V; ++e) {
            float x = cacc[j].c[q][e];
            for (int sft = rp.G; sft < 64; sft <<= 1) x += lane_xor_f32(x, sft);
            cacc[j].c[q][e] = x;
          }
    }
    // lane sets of the block that hold the same columns (the wavefronts of short rows, the lane
    // groups of rows of two wavefronts): in blocks of 256 threads they meet in LDS, one slot of
    // one sum at a time, so that a block writes a single row of partial sums
    const int period = rp.G > 64 ? rp.G : 64;
    const int copies = (int)blockDim.x / period;
    const int copy = (int)threadIdx.x / period;
    const bool merge = copies > 1 && blockDim.x <= 256;
    if (merge) {
      __shared__ typename Vec<float, V>::vec_t cbuf[256];
#pragma unroll
      for (int j = 0; j < NV; ++j)
#pragma unroll
        for (int q = 0; q < Pat::NCOLSUM; ++q) {
          if (copy > 0) cbuf[threadIdx.x] = cacc[j].c[q];
          __syncthreads();
          if (copy == 0)
            for (int k = 1; k < copies; ++k) cacc[j].c[q] += cbuf[(int)threadIdx.x + k * period];
          __syncthreads();
        }
    }
    const int ppb = merge ? 1 : copies;                                 // rows of partial sums per block
    const bool writer = (merge ? copy == 0 : true) && (rp.G >= 64 || ((int)threadIdx.x & 63) < rp.G);
    float* ws = reinterpret_cast<float*>(A.ws0);
    const i64 prow = (i64)blockIdx.x * ppb + (merge ? 0 : copy);
    if (writer) {
#pragma unroll
      for (int j = 0; j < NV; ++j)
        if (nvalid[j] > 0) {
#pragma unroll
          for (int q = 0; q < Pat::NCOLSUM; ++q) {
            Vec<float, V> t;
            t.v = cacc[j].c[q];
            st(ws + ((i64)q * A.aux0 + prow) * A.inner, (i64)(col0 + j * rp.G * V), t, SP::upto(nvalid[j]));
          }
        }
    }
  }
  if constexpr (Pat::NROWRED > 0) {
    // The lanes of a lane group hold the same values, the groups of a wavefront different rows:
    // combine across the groups, then across the wavefronts of the block through LDS (the
    // wavefronts of one lane group of a long row hold the same rows: one of them counts), and
    // write one partial result per block and reduction: ws1[q * blocks + block].
    if (rp.G < 64) {
#pragma unroll
      for (int q = 0; q < Pat::NROWRED; ++q)
        for (int sft = rp.G; sft < 64; sft <<= 1) racc[q] = Pat::rr_merge(q, racc[q], lane_xor_f32(racc[q], sft));
    }
    __shared__ float rbuf[16][Pat::NROWRED];
    const int wave = (int)threadIdx.x >> 6, nw = (int)blockDim.x >> 6;
    const int wpg = rp.G > 64 ? rp.G >> 6 : 1;
    if (((int)threadIdx.x & 63) == 0) {
#pragma unroll
      for (int q = 0; q < Pat::NROWRED; ++q) rbuf[wave][q] = racc[q];
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      float* ws = reinterpret_cast<float*>(A.ws1);
#pragma unroll
      for (int q = 0; q < Pat::NROWRED; ++q) {
        float t = rbuf[0][q];
        for (int w = wpg; w < nw; w += wpg) t = Pat::rr_merge(q, t, rbuf[w][q]);
        ws[(i64)q * A.aux1 + blockIdx.x] = t;
      }
    }
  }
}

// Streaming version for rows that do not fit the register budget: one block per row, the
// row is re-read (from L2 / Infinity Cache when it fits) once per reduction phase and once
// for the epilogue.  Any row length below 2^31 works.
template <class Pat, int P, int V>
DISC_DEV void row_stream_phases(const typename Pat::Args& A, typename Pat::RowCtx& rc, int inner,
                                char* lds, int& parity) {
  if constexpr (P < Pat::NPHASE) {
    typedef typename Pat::template Acc<P> AccT;
    AccT acc;
    Pat::template acc_init<P>(acc);
    for (int col = threadIdx.x * V; col < inner; col += blockDim.x * V) {
      int n = inner - col;
      n = n > V ? V : n;
      typename Pat::template Slot<V> slot;
      Pat::template load<V>(A, rc, col, Span::upto(n), slot);
      typename Pat::template Keep<V> kp;
      Pat::template phase<P, V, false>(A, acc, slot, kp, Span::upto(n), col, rc);
    }
    group_allreduce<Pat, P>(acc, 64);
    AccT* ex = reinterpret_cast<AccT*>(lds + parity * 16 * Pat::MAX_ACC_BYTES);
    parity ^= 1;
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) ex[wave] = acc;
    __syncthreads();
    const int nw = blockDim.x >> 6;
    acc = ex[0];
    for (int w = 1; w < nw; ++w) {
      AccT o = ex[w];
      Pat::template acc_merge<P>(acc, o);
    }
    Pat::template row_after<P>(A, rc, acc);
    row_stream_phases<Pat, P + 1, V>(A, rc, inner, lds, parity);
  }
}

template <class Pat, int V>
DISC_DEV void row_stream_body(const typename Pat::Args& A) {
  __shared__ __attribute__((aligned(16))) char lds[2 * 16 * Pat::MAX_ACC_BYTES];
  const int inner = (int)A.inner;
  int parity = 0;
  bool first = true;
  float racc[Pat::NROWRED > 0 ? Pat::NROWRED : 1];
  if constexpr (Pat::NROWRED > 0) {
#pragma unroll
    for (int q = 0; q < Pat::NROWRED; ++q) racc[q] = Pat::rr_identity(q);
  }
  for (i64 row = blockIdx.x; row < A.rows; row += gridDim.x) {
    typename Pat::RowCtx rc;
    Pat::row_begin(A, row, rc);
    rc.sl = nullptr;
    row_stream_phases<Pat, 0, V>(A, rc, inner, lds, parity);
    if constexpr (Pat::NROWRED > 0) Pat::row_reds(A, rc, racc);   // (every lane holds the row's values)
    for (int col = threadIdx.x * V; col < inner; col += blockDim.x * V) {
      int n = inner - col;
      n = n > V ? V : n;
      typename Pat::template Slot<V> slot;
      Pat::template load<V>(A, rc, col, Span::upto(n), slot);
      typename Pat::template OutSlot<V> o;
      typename Pat::template Keep<V> kp;
      Pat::template epilogue<V, false>(A, rc, slot, kp, col, Span::upto(n), o);
      Pat::template store<V>(A, rc, col, Span::upto(n), o);
      if constexpr (Pat::NCOLSUM > 0) {
        // sums over the rows: the block's row of partial sums lives in the workspace (the rows are
        // too long for registers); every lane owns its columns there, so no other lane touches them
        typename Pat::template ColAcc<V> ca{};
        Pat::template col_sums<V, false>(A, rc, slot, kp, col, Span::upto(n), ca);
#pragma unroll
        for (int q = 0; q < Pat::NCOLSUM; ++q) {
          float* dst = reinterpret_cast<float*>(A.ws0) + ((i64)q * A.aux0 + blockIdx.x) * A.inner;
          Vec<float, V> t;
          t.v = ca.c[q];
          if (!first) {
            Vec<float, V> old;
            ld(old, dst, (i64)col, Span::upto(n));
            t.v += old.v;
          }
          st(dst, (i64)col, t, Span::upto(n));
        }
      }
    }
    if (threadIdx.x == 0) Pat::row_store(A, row, rc);
    first = false;
  }
  if constexpr (Pat::NROWRED > 0) {
    if (threadIdx.x == 0) {
#pragma unroll
      for (int q = 0; q < Pat::NROWRED; ++q) reinterpret_cast<float*>(A.ws1)[(i64)q * A.aux1 + blockIdx.x] = racc[q];
    }
  }
}

// Last launch of a row reduce with reductions of per-row values over the rows: one block of 1024
// threads folds the per-block partial results of every reduction in a fixed order (sums in fp64)
// and stores them.  All reductions advance together and two strides are in flight per lane, so a
// lane makes one or two dependent trips to memory for the couple of thousand partial results of a
// large launch (a 256-thread block that took the reductions one after the other needed 14 us).
template <class Pat>
DISC_DEV void rowred_finish_body(const typename Pat::Args& A) {
  constexpr int NQ = Pat::NROWRED;
  __shared__ double red[NQ][1024];
  const float* ws = reinterpret_cast<const float*>(A.ws1);
  const i64 P = A.aux1;
  const int nt = (int)blockDim.x, tid = (int)threadIdx.x;      // nt: a power of two <= 1024
  double t0[NQ], t1[NQ];
#pragma unroll
  for (int q = 0; q < NQ; ++q) t0[q] = t1[q] = (double)Pat::rr_identity(q);
  i64 i = tid;
  for (; i + nt < P; i += 2 * nt) {
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
      const float a = ws[(i64)q * P + i], b = ws[(i64)q * P + i + nt];
      t0[q] = Pat::rr_merge(q, t0[q], (double)a);
      t1[q] = Pat::rr_merge(q, t1[q], (double)b);
    }
  }
  for (; i < P; i += nt) {
#pragma unroll
    for (int q = 0; q < NQ; ++q) t0[q] = Pat::rr_merge(q, t0[q], (double)ws[(i64)q * P + i]);
  }
#pragma unroll
  for (int q = 0; q < NQ; ++q) red[q][tid] = Pat::rr_merge(q, t0[q], t1[q]);
  __syncthreads();
  for (int s = nt >> 1; s > 0; s >>= 1) {
    if (tid < s) {
#pragma unroll
      for (int q = 0; q < NQ; ++q) red[q][tid] = Pat::rr_merge(q, red[q][tid], red[q][tid + s]);
    }
    __syncthreads();
  }
  if (tid == 0) {
    float v[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) v[q] = (float)red[q][0];
    Pat::rowred_store(A, v);
  }
}

// Second launch of a row reduce with sums over the rows: adds up the P rows of partial sums of
// every summed output, in a fixed order (the result does not depend on timing) and in fp64 (the
// fp32 partial sums each cover the rows of one block only).  A block takes 16 columns; its 256
// lanes are 16 columns x 16 lanes that each walk every 16th partial row of all sums together,
// eight loads in flight; the 16 lane totals of a column meet in LDS.  (Measured at 1023 partial
// rows x 1024 columns x 2 sums: 8.7 us, 12.6 with one sum after the other; 8 columns x 32 lanes,
// and blocks of 1024 threads covering whole 128-byte lines, both took 19 us.)
constexpr int kColsumCols = 16, kColsumLanes = 16;
template <class Pat>
DISC_DEV void colsum_finish_body(const typename Pat::Args& A) {
  constexpr int NQ = Pat::NCOLSUM, CL = kColsumCols, PL = kColsumLanes;
  __shared__ double red[NQ][PL][CL + 1];
  const int cl = (int)threadIdx.x % CL, pl = (int)threadIdx.x / CL;
  const i64 inner = A.inner, P = A.aux0;
  const float* ws = reinterpret_cast<const float*>(A.ws0);
  for (i64 c0 = (i64)blockIdx.x * CL; c0 < inner; c0 += (i64)gridDim.x * CL) {
    const i64 col = c0 + cl;
    constexpr int U = NQ >= 2 ? 4 : 8;            // partial rows in flight per lane and sum
    double acc[NQ][U];
#pragma unroll
    for (int q = 0; q < NQ; ++q)
#pragma unroll
      for (int u = 0; u < U; ++u) acc[q][u] = 0.0;
    if (col < inner) {
      const float* src = ws + col;
      const i64 plane = P * inner;
      i64 p = pl;
      for (; p + (U - 1) * PL < P; p += U * PL) {
        float x[NQ][U];
#pragma unroll
        for (int q = 0; q < NQ; ++q)
#pragma unroll
          for (int u = 0; u < U; ++u) x[q][u] = src[q * plane + (p + u * PL) * inner];
#pragma unroll
        for (int q = 0; q < NQ; ++q)
#pragma unroll
          for (int u = 0; u < U; ++u) acc[q][u] += x[q][u];
      }
      for (; p < P; p += PL) {
#pragma unroll
        for (int q = 0; q < NQ; ++q) acc[q][0] += src[q * plane + p * inner];
      }
    }
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
      double t = 0.0;
#pragma unroll
      for (int u = 0; u < U; ++u) t += acc[q][u];
      red[q][pl][cl] = t;
    }
    __syncthreads();
    if (pl == 0 && col < inner) {
      float v[NQ];
#pragma unroll
      for (int q = 0; q < NQ; ++q) {
        double t = 0.0;
#pragma unroll
        for (int k = 0; k < PL; ++k) t += red[q][k][cl];
        v[q] = (float)t;
      }
      Pat::colsum_store(A, col, v);
    }
    __syncthreads();
  }
}

// =======================================================================================
// A transpose on its own (not a fusion): out[b][p][q] = in[b][q][p], any element type.  A block
// moves square tiles through LDS so that both the reads (along p, the operand's innermost axis)
// and the writes (along q) are contiguous.  Every global access is 16 bytes wide (8 two-byte
// elements), and a tile row is 256 bytes of the operand -- two whole cache lines per row on both
// sides: 128 x 128 tiles for one- and two-byte elements, 64 x 64 for wider ones (with 64 x 64
// tiles and one element per lane, two-byte elements moved 128 bytes per row and reached 2.5 TB/s
// where four-byte elements reached 4.3).  A lane issues all its loads of a tile before the first
// LDS write.  The LDS row pitch is an odd number of dwords, so the column-wise element reads of
// the second half spread over the banks.
// =======================================================================================
template <class T>
DISC_DEV void ktranspose_body(const T* __restrict__ in, T* __restrict__ out, i64 batch, i64 P, i64 Q) {
  constexpr int VE = 16 / (int)sizeof(T);                    // elements per 16-byte access
  constexpr int TS = sizeof(T) <= 2 ? 128 : 64;
  constexpr int PAD = sizeof(T) >= 4 ? 1 : 4 / (int)sizeof(T);
  constexpr int VPR = TS / VE;                               // 16-byte pieces per tile row
  constexpr int NVEC = TS * VPR / 256;                       // pieces per lane and tile
  __shared__ __attribute__((aligned(16))) T tile[TS][TS + PAD];
  const i64 tiles_p = (P + TS - 1) / TS, tiles_q = (Q + TS - 1) / TS;
  const i64 per_batch = tiles_p * tiles_q;
  const i64 ntiles = batch * per_batch;
  for (i64 t = blockIdx.x; t < ntiles; t += gridDim.x) {
    const i64 b = t / per_batch;
    const i64 r = t - b * per_batch;
    // consecutive blocks walk a diagonal of the tile grid: with a power-of-two row pitch the tiles
    // of one tile row (or column) would otherwise queue up on the same memory channels
    const i64 tq = r / tiles_p;
    i64 tp = r - tq * tiles_p + tq;
    if (tp >= tiles_p) tp %= tiles_p;
    const i64 p0 = tp * TS, q0 = tq * TS;
    const T* src = in + b * P * Q;
    T* dst = out + b * P * Q;
    Vec<T, VE> piece[NVEC];
#pragma unroll
    for (int k = 0; k < NVEC; ++k) {              // row q0 + row of the operand, elements p0 + v * VE ...
      const int idx = (int)threadIdx.x + k * 256;
      const int row = idx / VPR, v = idx % VPR;
      const i64 q = q0 + row, p = p0 + v * VE;
      piece[k].clear();
      if (q < Q) {
        if (p + VE <= P) {
          piece[k].v = *reinterpret_cast<const typename Vec<T, VE>::unaligned_t*>(src + q * P + p);
        } else {
#pragma unroll
          for (int e = 0; e < VE; ++e)
            if (p + e < P) piece[k].set(e, src[q * P + p + e]);
        }
      }
    }
#pragma unroll
    for (int k = 0; k < NVEC; ++k) {
      const int idx = (int)threadIdx.x + k * 256;
      const int row = idx / VPR, v = idx % VPR;
#pragma unroll
      for (int e = 0; e < VE; ++e) tile[row][v * VE + e] = piece[k].get(e);
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < NVEC; ++k) {              // row p0 + row of the result, elements q0 + v * VE ...
      const int idx = (int)threadIdx.x + k * 256;
      const int row = idx / VPR, v = idx % VPR;
      const i64 p = p0 + row, q = q0 + v * VE;
      Vec<T, VE> o;
      o.clear();
#pragma unroll
      for (int e = 0; e < VE; ++e) o.set(e, tile[v * VE + e][row]);
      if (p < P) {
        if (q + VE <= Q) {
          *reinterpret_cast<typename Vec<T, VE>::unaligned_t*>(dst + p * Q + q) = o.v;
        } else {
#pragma unroll
          for (int e = 0; e < VE; ++e)
            if (q + e < Q) dst[p * Q + q + e] = o.get(e);
        }
      }
    }
    __syncthreads();
  }
}

// =======================================================================================
// Input fusion with a column reduction as root (reduce over an outer axis).  Canonical
// space [outer, mid, inner], `mid` reduced.  Three stages, no atomics, so results are
// bit-identical from run to run:
//   1. col_partial: the reduced axis is cut into chunks; a block owns one chunk of one column
//      tile.  Lanes run along `inner` (coalesced, V elements each), the block's row-lanes
//      stride over the rows of the chunk with four rows in flight; every lane keeps V column
//      accumulators (fp64 for fp32 sums).  The row-lanes of a column are combined through an
//      LDS transpose in fixed order and one partial per (chunk, column) goes to the workspace.
//   2. col_finish:  per column, partials are merged in fixed order; values and outputs that
//      no longer have the reduced axis (sum, mean, ...) are produced here.
//   3. the epilogue is a loop fusion (kloop_body) that reads the reduce results as column
//      vectors -- the tensor is read a second time, from Infinity Cache when it fits.
// =======================================================================================
struct ColPlan {
  int GC;          // lanes along inner per block, power of two <= 64
  int log2GC;
  int nchunk;      // chunks of the reduced axis
  int pad;
  i64 chunk_rows;  // rows per chunk
  i64 outer;
  i64 epi_rows;    // two-launch version: rows of the reduced axis per block of the second launch
};

// V column accumulators of one lane over rows [m0 + ty, m1) with stride TY of outer slice o,
// four rows in flight
template <class Pat, int V>
DISC_DEV void col_accumulate(const typename Pat::Args& A, i64 o, i64 col, int nvalid, i64 m0, i64 m1, int ty, int TY,
                             typename Pat::template Acc<0> (&acc)[V]) {
#pragma unroll
  for (int e = 0; e < V; ++e) Pat::template acc_init<0>(acc[e]);
  if (nvalid <= 0) return;
  i64 m = m0 + ty;
  for (; m + 3 * TY < m1; m += 4 * TY) {
    typename Pat::template Slot<V> s[4];
    typename Pat::RowCtx rc[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      Pat::row_begin(A, o * A.mid + m + u * TY, rc[u]);
      Pat::template load<V>(A, rc[u], col, Span::upto(nvalid), s[u]);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int e = 0; e < V; ++e)
        if (e < nvalid) Pat::template accum<0, V>(A, acc[e], s[u], e, (int)(m + u * TY), rc[u]);
  }
  for (; m < m1; m += TY) {
    typename Pat::template Slot<V> s;
    typename Pat::RowCtx rc;
    Pat::row_begin(A, o * A.mid + m, rc);
    Pat::template load<V>(A, rc, col, Span::upto(nvalid), s);
#pragma unroll
    for (int e = 0; e < V; ++e)
      if (e < nvalid) Pat::template accum<0, V>(A, acc[e], s, e, (int)m, rc);
  }
}

// Exchange with the lane whose number differs in bit S (a true xor exchange, unlike lane_xchg whose
// middle steps assume that earlier steps have run): DPP quad permutes, the swizzle unit for 4 and 8,
// the permlane swaps for 16 and 32.
template <int S>
DISC_DEV u32 lane_xor_u32(u32 v) {
  if constexpr (S == 1 || S == 2 || S == 16 || S == 32) return lane_xchg_u32<S>(v);
  else return (u32)__builtin_amdgcn_ds_swizzle((int)v, (S << 10) | 0x1f);   // bit mode: and 0x1f, or 0, xor S
}
template <int S, class T>
DISC_DEV T lane_xor_pod(const T& v) {
  static_assert(sizeof(T) % 4 == 0, "accumulators are made of 4- and 8-byte fields");
  u32 w[sizeof(T) / 4];
  __builtin_memcpy(w, &v, sizeof(T));
#pragma unroll
  for (int i = 0; i < (int)(sizeof(T) / 4); ++i) w[i] = lane_xor_u32<S>(w[i]);
  T r;
  __builtin_memcpy(&r, w, sizeof(T));
  return r;
}
template <class Pat, int S, int V>
DISC_DEV void col_lane_step(typename Pat::template Acc<0> (&acc)[V]) {
#pragma unroll
  for (int e = 0; e < V; ++e) {
    const typename Pat::template Acc<0> o = lane_xor_pod<S>(acc[e]);
    Pat::template acc_merge<0>(acc[e], o);
  }
}

// The row-lanes of a block each hold accumulators of the same GC * V columns (thread = ty * GC + tx).
// Combines them column by column in a fixed order and leaves the block's result in EVERY lane:
// the lanes of a wavefront that hold the same columns meet through xor exchanges over the lane
// distances GC .. 32 (both partners compute the same commutative merge, so they agree bit for bit),
// then the wavefronts meet through one LDS cell per wavefront and column.  (One lane per column
// walking all row-lanes' cells in LDS, as before, cost up to 2 us per block with 128 row-lanes.)
// `lds` holds 4 * 64 * V accumulators; ends with a barrier, so the caller may reuse it at once.
template <class Pat, int V>
DISC_DEV void col_block_merge(typename Pat::template Acc<0> (&acc)[V], typename Pat::template Acc<0>* lds, int GC, int tx) {
  int g = GC;
  asm volatile("" : "+s"(g));
  if (g <= 1) col_lane_step<Pat, 1, V>(acc);
  if (g <= 2) col_lane_step<Pat, 2, V>(acc);
  if (g <= 4) col_lane_step<Pat, 4, V>(acc);
  if (g <= 8) col_lane_step<Pat, 8, V>(acc);
  if (g <= 16) col_lane_step<Pat, 16, V>(acc);
  if (g <= 32) col_lane_step<Pat, 32, V>(acc);
  const int wave = (int)threadIdx.x >> 6, lane = (int)threadIdx.x & 63, nw = (int)blockDim.x >> 6;
  const int gw = GC < 64 ? GC : 64;          // columns-lanes per wavefront
  if (lane < gw) {
#pragma unroll
    for (int e = 0; e < V; ++e) lds[(wave * gw + lane) * V + e] = acc[e];
  }
  __syncthreads();
#pragma unroll
  for (int e = 0; e < V; ++e) {
    acc[e] = lds[tx * V + e];
    for (int w = 1; w < nw; ++w) Pat::template acc_merge<0>(acc[e], lds[(w * gw + tx) * V + e]);
  }
  __syncthreads();
}

template <class Pat, int V>
DISC_DEV void col_partial_body(const typename Pat::Args& A, const ColPlan& cp) {
  typedef typename Pat::template Acc<0> AccT;
  __shared__ AccT lds[256 * V];
  const int tx = threadIdx.x & (cp.GC - 1);
  const int ty = threadIdx.x >> cp.log2GC;
  const int TY = blockDim.x >> cp.log2GC;
  const i64 col = ((i64)blockIdx.x * cp.GC + tx) * V;
  const i64 rem = A.inner - col;
  const int nvalid = rem <= 0 ? 0 : (rem < (i64)V ? (int)rem : V);
  const i64 chunk = blockIdx.y;
  const i64 m0 = chunk * cp.chunk_rows;
  const i64 m1 = m0 + cp.chunk_rows < A.mid ? m0 + cp.chunk_rows : A.mid;
  for (i64 o = blockIdx.z; o < cp.outer; o += gridDim.z) {
    AccT acc[V];
    col_accumulate<Pat, V>(A, o, col, nvalid, m0, m1, ty, TY, acc);
    col_block_merge<Pat, V>(acc, lds, cp.GC, tx);
    if (ty == 0) {
#pragma unroll
      for (int e = 0; e < V; ++e)
        if (e < nvalid) Pat::acc_st(A, (o * cp.nchunk + chunk) * A.inner + col + e, acc[e]);
    }
  }
}

// The rows [m0, m1) of outer slice o, a block's share of them, through the epilogue: `base` holds
// the reduce results of the lane's columns (the same for every row), the operands are loaded into
// copies of it, four rows in flight per lane.
template <class Pat, class PatE, int V, int NT>
DISC_DEV void col_rows_epilogue(const typename Pat::Args& A, const typename PatE::template Slot<V>& base, i64 o, i64 col,
                                Span sp, i64 m0, i64 m1, int ty, int TY) {
  i64 m = m0 + ty;
  for (; m + 3 * TY < m1; m += 4 * TY) {
    typename PatE::template Slot<V> s[4];
    typename PatE::RowCtx rc[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      s[u] = base;
      PatE::row_begin(A, o * A.mid + m + u * TY, rc[u]);
      PatE::template load_x<V, NT>(A, rc[u], col, sp, s[u]);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      typename PatE::template OutSlot<V> out;
      typename PatE::template Keep<V> kp;
      PatE::template epilogue<V, false>(A, rc[u], s[u], kp, col, sp, out);
      PatE::template store<V, NT>(A, rc[u], col, sp, out);
    }
  }
  for (; m < m1; m += TY) {
    typename PatE::template Slot<V> s1 = base;
    typename PatE::RowCtx rc;
    PatE::row_begin(A, o * A.mid + m, rc);
    PatE::template load_x<V, NT>(A, rc, col, sp, s1);
    typename PatE::template OutSlot<V> out;
    typename PatE::template Keep<V> kp;
    PatE::template epilogue<V, false>(A, rc, s1, kp, col, sp, out);
    PatE::template store<V, NT>(A, rc, col, sp, out);
  }
}

// Single-launch version for small problems, where every further launch costs more than the work
// (a kernel that makes one round trip to memory takes 5-6 us on this part whatever it moves): a
// block owns a strip of GC * V columns and ALL rows of it.  It reduces the strip, every lane ends up
// with the results of its own columns in registers (col_block_merge), the lanes of the first row
// write the outputs that lost the reduced axis, and -- when the pattern has per-element outputs --
// the block walks its strip a second time for the epilogue, reading the tensor from cache.  Nothing
// goes through memory between the two passes.  PatE = void: no epilogue; the reduce results go to
// the workspace planes as in the three-launch version.
template <class Pat, class PatE, int V>
DISC_DEV void col_strip_body(const typename Pat::Args& A, const ColPlan& cp) {
  typedef typename Pat::template Acc<0> AccT;
  __shared__ AccT lds[256 * V];
  const int tx = threadIdx.x & (cp.GC - 1);
  const int ty = threadIdx.x >> cp.log2GC;
  const int TY = blockDim.x >> cp.log2GC;
  const i64 col = ((i64)blockIdx.x * cp.GC + tx) * V;
  const i64 rem = A.inner - col;
  const int nvalid = rem <= 0 ? 0 : (rem < (i64)V ? (int)rem : V);
  for (i64 o = blockIdx.y; o < cp.outer; o += gridDim.y) {
    AccT acc[V];
    col_accumulate<Pat, V>(A, o, col, nvalid, 0, A.mid, ty, TY, acc);
    col_block_merge<Pat, V>(acc, lds, cp.GC, tx);
    if constexpr (__is_same(PatE, void)) {
      if (ty == 0) {
#pragma unroll
        for (int e = 0; e < V; ++e)
          if (e < nvalid) Pat::col_finish(A, o, col + e, acc[e]);
      }
    } else {
      if (nvalid > 0) {
        typename PatE::template Slot<V> base;
        PatE::template clear_red<V>(base);
#pragma unroll
        for (int e = 0; e < V; ++e)
          if (e < nvalid) PatE::template finish_elem<V>(A, o, col + e, acc[e], base, e, ty == 0);
        col_rows_epilogue<Pat, PatE, V, 0>(A, base, o, col, Span::upto(nvalid), 0, A.mid, ty, TY);
      }
    }
  }
}

// Second of three launches: per column, the partials of all chunks merged in a fixed order.  A
// block takes 16 columns; its 256 lanes are 16 columns x 16 lanes that each walk every 16th chunk
// with four loads in flight, and the 16 lane results of a column meet in LDS.  (One lane per
// column walking the chunks one dependent load at a time, on inner / 64 blocks, took 18 us for
// 256 chunks x 1024 columns.)
template <class Pat>
DISC_DEV void col_finish_body(const typename Pat::Args& A, const ColPlan& cp) {
  typedef typename Pat::template Acc<0> AccT;
  constexpr int CL = 16, PL = 16;
  __shared__ AccT lds[PL][CL + 1];
  const int cl = (int)threadIdx.x % CL, pl = (int)threadIdx.x / CL;
  const i64 c = (i64)blockIdx.x * CL + cl;
  for (i64 o = blockIdx.y; o < cp.outer; o += gridDim.y) {
    AccT acc[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) Pat::template acc_init<0>(acc[u]);
    if (c < A.inner) {
      const i64 base = o * cp.nchunk * A.inner + c;
      int j = pl;
      for (; j + 3 * PL < cp.nchunk; j += 4 * PL) {
        AccT t[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) Pat::acc_ld(A, base + (i64)(j + u * PL) * A.inner, t[u]);
#pragma unroll
        for (int u = 0; u < 4; ++u) Pat::template acc_merge<0>(acc[u], t[u]);
      }
      for (; j < cp.nchunk; j += PL) {
        AccT t;
        Pat::acc_ld(A, base + (i64)j * A.inner, t);
        Pat::template acc_merge<0>(acc[0], t);
      }
    }
#pragma unroll
    for (int u = 1; u < 4; ++u) Pat::template acc_merge<0>(acc[0], acc[u]);
    lds[pl][cl] = acc[0];
    __syncthreads();
    if (pl == 0 && c < A.inner) {
      AccT tot = lds[0][cl];
      for (int k = 1; k < PL; ++k) Pat::template acc_merge<0>(tot, lds[k][cl]);
      Pat::col_finish(A, o, c, tot);
    }
    __syncthreads();
  }
}

// Two-launch version: the second launch both finishes and applies the epilogue.  A block owns a
// column tile (the same GC * V columns as in the partial pass) and a range of rows.  It first merges
// the few chunk partials of its own columns (every block of a column tile repeats this small piece
// of work, in the same fixed order, so all of them hold the same results; the block of the first
// row range also writes the outputs that lost the reduced axis), keeps the reduce results in
// registers -- they are the same for every row -- and then streams its rows through the epilogue.
// No finish launch, no reduce-result planes in memory, no per-slot loads of them.
// The row ranges are handed out in reverse: the first blocks to start take the rows that the
// partial pass read last and that are most likely still in the memory-side cache.
// NT: bit 0 = non-temporal loads of the full-size operands, bit 1 = non-temporal stores.
template <class Pat, class PatE, int V, int NT>
DISC_DEV void col_epi2_body(const typename Pat::Args& A, const ColPlan& cp) {
  typedef typename Pat::template Acc<0> AccT;
  __shared__ AccT lds[256 * V];
  const int tx = threadIdx.x & (cp.GC - 1);
  const int ty = threadIdx.x >> cp.log2GC;
  const int TY = blockDim.x >> cp.log2GC;
  const i64 col = ((i64)blockIdx.x * cp.GC + tx) * V;
  const i64 rem = A.inner - col;
  const int nvalid = rem <= 0 ? 0 : (rem < (i64)V ? (int)rem : V);
  const i64 rb = (i64)gridDim.y - 1 - blockIdx.y;
  const i64 m0 = rb * cp.epi_rows;
  const i64 m1 = m0 + cp.epi_rows < A.mid ? m0 + cp.epi_rows : A.mid;
  for (i64 o = blockIdx.z; o < cp.outer; o += gridDim.z) {
    AccT acc[V];
#pragma unroll
    for (int e = 0; e < V; ++e) Pat::template acc_init<0>(acc[e]);
    if (nvalid > 0) {
      for (int j = ty; j < cp.nchunk; j += TY) {
        AccT t[V];
#pragma unroll
        for (int e = 0; e < V; ++e)
          if (e < nvalid) Pat::acc_ld(A, (o * cp.nchunk + j) * A.inner + col + e, t[e]);
#pragma unroll
        for (int e = 0; e < V; ++e)
          if (e < nvalid) Pat::template acc_merge<0>(acc[e], t[e]);
      }
    }
    col_block_merge<Pat, V>(acc, lds, cp.GC, tx);
    if (nvalid > 0) {
      typename PatE::template Slot<V> base;
      PatE::template clear_red<V>(base);
#pragma unroll
      for (int e = 0; e < V; ++e)
        if (e < nvalid) PatE::template finish_elem<V>(A, o, col + e, acc[e], base, e, rb == 0 && ty == 0);
      col_rows_epilogue<Pat, PatE, V, NT>(A, base, o, col, Span::upto(nvalid), m0, m1, ty, TY);
    }
  }
}

// =======================================================================================
// Outputs whose size depends on the data (compaction by a predicate computed in the pattern; Unique
// of a sorted tensor is the case keep[i] = x[i] != x[i-1]).  Rank-1 values of length N = A.inner.
// Three launches, no atomics, nothing read back by the host:
//   1. compact_count:   a block owns a tile of 256 * kCompactSlots * V consecutive elements (a lane
//                       owns kCompactSlots consecutive slots), evaluates the fused chain and counts
//                       what is kept; one count per block to the workspace.
//   2. compact_scan:    one block turns the counts into exclusive offsets, in a fixed order, and
//                       stores the total -- the data-dependent size -- in the COMPACT_COUNT outputs.
//   3. compact_scatter: the blocks evaluate their tiles again (the inputs are read twice; nothing
//                       but the counts is kept between the launches), rank what they keep with a
//                       scan over the lanes, and store the kept values at offset + rank, in order;
//                       COMPACT_RANK outputs get the slot of every element.
// =======================================================================================
constexpr int kCompactSlots = 4;

// inclusive scan over the 64 lanes of a wavefront
DISC_DEV int wave_inclusive_scan(int x) {
  const int lane = (int)threadIdx.x & 63;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int t = __builtin_amdgcn_ds_bpermute(((lane - d) & 63) << 2, x);
    if (lane >= d) x += t;
  }
  return x;
}

// evaluates the tile of the calling lane: kept flags and values of its kCompactSlots slots
template <class Pat, int V>
DISC_DEV int compact_eval(const typename Pat::Args& A, i64 first, typename Pat::template OutSlot<V> (&o)[kCompactSlots],
                          int (&nvalid)[kCompactSlots]) {
  int cnt = 0;
  typename Pat::RowCtx rc;
  Pat::row_begin(A, 0, rc);
#pragma unroll
  for (int u = 0; u < kCompactSlots; ++u) {
    const i64 col = first + (i64)u * V;
    const i64 rem = A.inner - col;
    nvalid[u] = rem <= 0 ? 0 : (rem < (i64)V ? (int)rem : V);
    if (nvalid[u] > 0) {
      typename Pat::template Slot<V> slot;
      typename Pat::template Keep<V> kp;
      Pat::template load<V>(A, rc, col, Span::upto(nvalid[u]), slot);
      Pat::template epilogue<V, false>(A, rc, slot, kp, col, Span::upto(nvalid[u]), o[u]);
#pragma unroll
      for (int e = 0; e < V; ++e) cnt += (e < nvalid[u] && o[u].keep[e]) ? 1 : 0;
    }
  }
  return cnt;
}

template <class Pat, int V>
DISC_DEV void compact_count_body(const typename Pat::Args& A) {
  __shared__ int wsum[4];
  const i64 tile = (i64)blockDim.x * kCompactSlots * V;
  i64* counts = reinterpret_cast<i64*>(A.ws0);
  for (i64 b = blockIdx.x; b < A.aux0; b += gridDim.x) {
    typename Pat::template OutSlot<V> o[kCompactSlots];
    int nvalid[kCompactSlots];
    const int cnt = compact_eval<Pat, V>(A, b * tile + (i64)threadIdx.x * kCompactSlots * V, o, nvalid);
    const int incl = wave_inclusive_scan(cnt);
    if (((int)threadIdx.x & 63) == 63) wsum[threadIdx.x >> 6] = incl;
    __syncthreads();
    if (threadIdx.x == 0) counts[b] = (i64)wsum[0] + wsum[1] + wsum[2] + wsum[3];
    __syncthreads();
  }
}

// one block of 1024 threads: exclusive scan of the A.aux0 block counts, in place
template <class Pat>
DISC_DEV void compact_scan_body(const typename Pat::Args& A) {
  __shared__ i64 part[1024];
  i64* counts = reinterpret_cast<i64*>(A.ws0);
  const i64 nb = A.aux0;
  const int nt = (int)blockDim.x, tid = (int)threadIdx.x;
  const i64 per = (nb + nt - 1) / nt;
  const i64 lo = (i64)tid * per, hi = lo + per < nb ? lo + per : nb;
  i64 sum = 0;
  for (i64 i = lo; i < hi; ++i) sum += counts[i];
  part[tid] = sum;
  __syncthreads();
  for (int d = 1; d < nt; d <<= 1) {          // inclusive scan of the per-thread sums
    const i64 t = tid >= d ? part[tid - d] : 0;
    __syncthreads();
    part[tid] += t;
    __syncthreads();
  }
  i64 run = part[tid] - sum;                   // exclusive prefix of this thread's stretch
  for (i64 i = lo; i < hi; ++i) {
    const i64 c = counts[i];
    counts[i] = run;
    run += c;
  }
  if (tid == nt - 1) Pat::count_store(A, part[nt - 1]);
}

template <class Pat, int V>
DISC_DEV void compact_scatter_body(const typename Pat::Args& A) {
  __shared__ int wsum[4];
  const i64 tile = (i64)blockDim.x * kCompactSlots * V;
  const i64* offsets = reinterpret_cast<const i64*>(A.ws0);
  for (i64 b = blockIdx.x; b < A.aux0; b += gridDim.x) {
    typename Pat::template OutSlot<V> o[kCompactSlots];
    int nvalid[kCompactSlots];
    const i64 first = b * tile + (i64)threadIdx.x * kCompactSlots * V;
    const int cnt = compact_eval<Pat, V>(A, first, o, nvalid);
    const int incl = wave_inclusive_scan(cnt);
    const int wave = (int)threadIdx.x >> 6;
    if (((int)threadIdx.x & 63) == 63) wsum[wave] = incl;
    __syncthreads();
    i64 pos = offsets[b] + (incl - cnt);
    for (int w = 0; w < wave; ++w) pos += wsum[w];
#pragma unroll
    for (int u = 0; u < kCompactSlots; ++u) {
      i64 rank[V];
#pragma unroll
      for (int e = 0; e < V; ++e) {
        if (e < nvalid[u] && o[u].keep[e]) {
          Pat::template compact_store<V>(A, o[u], e, pos);
          ++pos;
        }
        rank[e] = pos - 1;
      }
      if constexpr (Pat::HAS_RANK) {
        if (nvalid[u] > 0) Pat::template rank_store<V>(A, first + (i64)u * V, rank, Span::upto(nvalid[u]));
      }
    }
    __syncthreads();
  }
}

}  // namespace disc

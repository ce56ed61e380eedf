// Counts heap allocations made while the launch path of the library runs (shape calculation,
// checks, version and launch-dimension selection: disc_plan, which is disc_launch without the
// enqueue).  The host flow of a registered pattern is meant to be "compiled": a handful of integer
// products and comparisons over tables built at registration (Section 4.2.3), so it must not
// allocate, build strings or search maps per call.
//
// usage: plan_alloc_count <pattern file>...   each file: int32 n_ops, int32 n_cs, int32 n_dims,
//        n_ops disc_op records, n_cs disc_constraint records, then int32 n_shapes and n_shapes rows
//        of n_dims int64 values.  Prints one line per pattern: "<file> plans=<n> allocations=<k>".
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "disc.h"

// Built with -DDISC_NO_INTERPOSE for the sanitizer run (AddressSanitizer brings its own allocator):
// then nothing is counted and the program only drives the host code.
#ifndef DISC_NO_INTERPOSE
extern "C" void* __libc_malloc(size_t);
extern "C" void* __libc_calloc(size_t, size_t);
extern "C" void* __libc_realloc(void*, size_t);
extern "C" void __libc_free(void*);

static volatile long g_count = 0;
static volatile int g_on = 0;
// every route to the heap of this process: the C allocator entry points (operator new of
// libstdc++ ends up in malloc, and is counted there)
extern "C" void* malloc(size_t n) {
  if (g_on) ++g_count;
  return __libc_malloc(n);
}
extern "C" void* calloc(size_t a, size_t b) {
  if (g_on) ++g_count;
  return __libc_calloc(a, b);
}
extern "C" void* realloc(void* p, size_t n) {
  if (g_on) ++g_count;
  return __libc_realloc(p, n);
}
extern "C" void free(void* p) { __libc_free(p); }
#else
static volatile long g_count = 0;
static volatile int g_on = 0;
#endif

int main(int argc, char** argv) {
  disc_ctx* ctx = nullptr;
  if (disc_create(&ctx, -1) != DISC_OK) return 2;
  // the counter itself must work: a vector growth is seen
  g_on = 1;
  { std::vector<int> v(1000, 1); if (v[999] != 1) return 3; }
  g_on = 0;
#ifndef DISC_NO_INTERPOSE
  if (g_count == 0) { fprintf(stderr, "allocation counter does not see the heap\n"); return 4; }
#endif
  int rc_all = 0;
  for (int a = 1; a < argc; ++a) {
    FILE* f = fopen(argv[a], "rb");
    if (!f) return 5;
    int32_t hdr[3];
    if (fread(hdr, 4, 3, f) != 3) return 6;
    std::vector<disc_op> ops(hdr[0]);
    std::vector<disc_constraint> cs(hdr[1] > 0 ? hdr[1] : 1);
    if (fread(ops.data(), sizeof(disc_op), hdr[0], f) != (size_t)hdr[0]) return 6;
    if (hdr[1] > 0 && fread(cs.data(), sizeof(disc_constraint), hdr[1], f) != (size_t)hdr[1]) return 6;
    int32_t n_shapes = 0;
    if (fread(&n_shapes, 4, 1, f) != 1) return 6;
    std::vector<int64_t> shapes((size_t)n_shapes * hdr[2]);
    if (fread(shapes.data(), 8, shapes.size(), f) != shapes.size()) return 6;
    fclose(f);
    int32_t id = -1;
    if (disc_register_pattern(ctx, ops.data(), hdr[0], cs.data(), hdr[1], &id) != DISC_OK) {
      fprintf(stderr, "%s: %s\n", argv[a], disc_last_error(ctx));
      return 7;
    }
    disc_plan_t plan;
    size_t ws = 0;
    // a dims vector the pattern refuses (negative size) and a wrong count: error paths run too
    {
      std::vector<int64_t> neg(shapes.begin(), shapes.begin() + hdr[2]);
      neg[0] = -1;
      if (disc_plan(ctx, id, neg.data(), hdr[2], nullptr, nullptr, -1, &plan) != DISC_ERR_SHAPE) return 8;
      if (disc_plan(ctx, id, neg.data(), hdr[2] + 1, nullptr, nullptr, -1, &plan) != DISC_ERR_INVALID_ARG) return 8;
    }
    // one call outside the count (function-local statics of the library are built on first use)
    disc_plan(ctx, id, shapes.data(), hdr[2], nullptr, nullptr, -1, &plan);
    g_count = 0;
    g_on = 1;
    int bad = 0;
    long launches = 0;
    for (int s = 0; s < n_shapes; ++s) {
      const int64_t* d = shapes.data() + (size_t)s * hdr[2];
      if (disc_plan(ctx, id, d, hdr[2], nullptr, nullptr, -1, &plan) != DISC_OK) ++bad;
      if (disc_workspace_bytes(ctx, id, d, hdr[2], &ws) != DISC_OK) ++bad;
      launches += plan.n_launches;
    }
    g_on = 0;
    printf("%s plans=%d launches=%ld failed=%d allocations=%ld\n", argv[a], n_shapes, launches, bad, (long)g_count);
    if (bad || g_count) rc_all = 1;
  }
  disc_destroy(ctx);
  return rc_all;
}

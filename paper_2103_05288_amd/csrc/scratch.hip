// disc_launch_static_scratch: disc_launch for callers that cannot provide (or allocate) a workspace.
//
// The patterns whose kernels exchange partial results through device memory (column reduces, row
// reduces that carry sums over the rows) take that memory from a caller-supplied workspace in
// disc_launch.  Code under HIP graph capture, tight serving loops and harnesses that forbid
// allocation have none to give, so this entry point lends the kernels a fixed array that lives in
// the library's own code object: nothing is allocated, here or in any call below.
//
// The array exists once per GPU (every device that loads the code object holds its own copy at its
// own address).  Host code never uses the array's name as an address: the device address is asked
// once per device with hipGetSymbolAddress and that pointer is what the kernels get, exactly as
// they get the caller's workspace in disc_launch.
#include <hip/hip_runtime.h>

#include "disc.h"

namespace disc {
// runtime.cpp
int context_device(const disc_ctx* ctx);
int context_fail(disc_ctx* ctx, int code, const char* msg);
}  // namespace disc

namespace {

static __device__ __align__(256) __attribute__((used)) unsigned char scratch[DISC_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];          // device address of `scratch` on each GPU, once asked
bool g_scratch_known[kMaxDevices];

// Device address of the array on `device`.  Asked once per device, with that device current (the
// address belongs to the copy of the array on the device that is current during the call).
int scratch_address(disc_ctx* ctx, int device, void** out) {
  if (device < 0 || device >= kMaxDevices) return disc::context_fail(ctx, DISC_ERR_INVALID_ARG, "device number out of range");
  if (!g_scratch_known[device]) {
    int cur = -1;
    if (hipGetDevice(&cur) != hipSuccess) return disc::context_fail(ctx, DISC_ERR_HIP, "hipGetDevice failed");
    if (cur != device && hipSetDevice(device) != hipSuccess) return disc::context_fail(ctx, DISC_ERR_HIP, "hipSetDevice failed");
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (cur != device && cur >= 0) (void)hipSetDevice(cur);
    if (e != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return disc::context_fail(ctx, DISC_ERR_HIP, "hipGetSymbolAddress of the static scratch array failed");
    }
    g_scratch_ptr[device] = ptr;
    g_scratch_known[device] = true;
  }
  *out = g_scratch_ptr[device];
  return DISC_OK;
}

}  // namespace

extern "C" int disc_static_scratch_init(disc_ctx* ctx) {
  if (!ctx) return DISC_ERR_INVALID_ARG;
  const int device = disc::context_device(ctx);
  if (device < 0) return disc::context_fail(ctx, DISC_ERR_INVALID_ARG, "host-only context has no device scratch");
  void* p = nullptr;
  return scratch_address(ctx, device, &p);
}

extern "C" int disc_launch_static_scratch(disc_ctx* ctx, int32_t id, const int64_t* dims, int n_dims,
                                          const void* const* inputs, int n_in, void* const* outputs, int n_out,
                                          void* hip_stream) {
  if (!ctx) return DISC_ERR_INVALID_ARG;
  const int device = disc::context_device(ctx);
  if (device < 0) return disc::context_fail(ctx, DISC_ERR_INVALID_ARG, "host-only context cannot launch");
  // what the call needs, from the same host planning disc_launch does (no allocation in there)
  size_t need = 0;
  int rc = disc_workspace_bytes(ctx, id, dims, n_dims, &need);
  if (rc != DISC_OK) return rc;
  if (need > (size_t)DISC_STATIC_SCRATCH_BYTES)
    return disc::context_fail(ctx, DISC_ERR_WORKSPACE,
                              "this shape needs more scratch memory than the static array holds "
                              "(DISC_STATIC_SCRATCH_BYTES); use disc_launch with a workspace");
  void* ptr = nullptr;
  if (need > 0) {
    // (the array is only touched by calls that need it; its address is known after disc_create)
    rc = scratch_address(ctx, device, &ptr);
    if (rc != DISC_OK) return rc;
  }
  // The kernels take `ptr` as their workspace argument.  Nothing in the array has to start at zero:
  // every cell a kernel reads was written earlier in the same call (no atomics, no counters), so
  // what an earlier call left behind is never seen.
  return disc_launch(ctx, id, dims, n_dims, inputs, n_in, outputs, n_out, ptr, need > 0 ? (size_t)DISC_STATIC_SCRATCH_BYTES : 0,
                     hip_stream);
}

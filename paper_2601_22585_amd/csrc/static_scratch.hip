// Reduce-Scatter for callers that cannot allocate device memory: the partial
// sums of the out-of-place STEPWISE schedule live in a fixed array that is part
// of the library's code object instead of a caller-supplied workspace.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <mutex>

#include "hcl.h"
#include "internal.h"
#include "ring_sched.h"

// Every GPU the process uses holds its own copy of this array, at its own
// address, from the moment the code object is loaded there until the process ends.
static __device__ __align__(256) unsigned char scratch[HCL_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
void* g_scratch_of_device[kMaxDevices];  // device address of `scratch` on each device, once looked up
std::mutex g_scratch_mutex;

// Device address of the array on the current device.  In host code the name
// `scratch` is only a handle for the runtime's symbol table, never a device
// address: the address is asked for once per device and kept.
hcl_status_t scratch_of_current_device(void** out) {
  int dev = -1;
  hipError_t rc = hipGetDevice(&dev);
  if (rc != hipSuccess) return hcl::fail(HCL_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(rc));
  if (dev < 0 || dev >= kMaxDevices) return hcl::fail(HCL_ERR_UNSUPPORTED, "device index %d beyond %d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_of_device[dev]) {
    void* p = nullptr;
    rc = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (rc != hipSuccess || !p) return hcl::fail(HCL_ERR_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(rc));
    g_scratch_of_device[dev] = p;
  }
  *out = g_scratch_of_device[dev];
  return HCL_OK;
}

}  // namespace

extern "C" size_t hcl_static_scratch_bytes(void) { return (size_t)HCL_STATIC_SCRATCH_BYTES; }

extern "C" hcl_status_t hcl_reduce_scatter_sim_static(const void* const* send, void* const* recv, int W,
                                                      size_t recvcount, hcl_dtype_t dtype, hcl_op_t op,
                                                      size_t chunk_bytes, const hcl_opts_t* opts, void* stream) {
  hcl_opts_t o{};
  if (opts) o = *opts;
  o.workspace = nullptr;
  o.workspace_bytes = 0;
  // what the schedule would ask of a caller-supplied workspace (0: it needs none, or the
  // arguments are invalid and the call below says why); the in-place form keeps its
  // partial sums in send[] and needs none either
  size_t need = hcl_workspace_bytes(HCL_KIND_REDUCE_SCATTER, W, recvcount, dtype, chunk_bytes, &o);
  if (need && send && recv) {
    const uint64_t stride = (uint64_t)recvcount * hcl::elem_size(dtype);
    int same = 0;
    for (int r = 0; r < W; ++r) same += send[r] && (const char*)recv[r] == (const char*)send[r] + (uint64_t)r * stride;
    if (same == W) need = 0;
  }
  if (need > (size_t)HCL_STATIC_SCRATCH_BYTES) {
    return hcl::fail(HCL_ERR_WORKSPACE,
                     "this Reduce-Scatter keeps %zu bytes of partial sums, the library's fixed scratch holds %zu: "
                     "use hcl_reduce_scatter_sim with a workspace, the in-place form or the FUSED schedule",
                     need, (size_t)HCL_STATIC_SCRATCH_BYTES);
  }
  if (need) {
    void* p = nullptr;
    hcl_status_t st = scratch_of_current_device(&p);
    if (st) return st;
    o.workspace = p;
    o.workspace_bytes = (size_t)HCL_STATIC_SCRATCH_BYTES;
  }
  // every partial is written by one step before the next step reads it: nothing in the
  // array has to start at zero, whatever an earlier call left there
  return hcl_reduce_scatter_sim(send, recv, W, recvcount, dtype, op, chunk_bytes, &o, stream);
}

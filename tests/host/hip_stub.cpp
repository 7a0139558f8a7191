// TEST INFRASTRUCTURE: host stand-ins for the HIP runtime calls and the kernel
// launchers that hcl_api.cpp uses, so that the whole host side of the library
// (validation, ring chunk scheduler, launch plans, stream fork / join) can be
// compiled with g++ and run under AddressSanitizer / UBSan without a GPU.
// Nothing is computed here: a "launch" only records its arguments.
#include <hip/hip_runtime_api.h>

#include <cstdint>
#include <vector>

#include "reduce_copy.h"
#include "ring_sched.h"
#include "shim.h"

static std::vector<shim::Launch> g_launches;
static std::vector<shim::StreamOp> g_stream_ops;

namespace shim {
std::vector<Launch>& launches() { return g_launches; }
std::vector<StreamOp>& stream_ops() { return g_stream_ops; }
void reset() {
  g_launches.clear();
  g_stream_ops.clear();
}
}  // namespace shim

namespace hcl {
// the tile a launch shape covers, as the device side defines it: threads x (16 / element size) x unroll
uint64_t tile_elems(int dtype, const Tuning& t) { return (uint64_t)t.threads * (16 / elem_size(dtype)) * t.unroll; }

int launch_step(const StepArgs& a, int dtype, int nsrc, int ndst, const Tuning& t, void* stream) {
  shim::Launch l{};
  l.fused = false;
  l.step = a;
  l.dtype = dtype;
  l.nsrc = nsrc;
  l.ndst = ndst;
  l.tune = t;
  l.stream = stream;
  g_launches.push_back(l);
  return 0;
}
int launch_fused(const FusedArgs& a, int dtype, const Tuning& t, void* stream) {
  shim::Launch l{};
  l.fused = true;
  l.fusedargs = a;
  l.dtype = dtype;
  l.tune = t;
  l.stream = stream;
  g_launches.push_back(l);
  return 0;
}
}  // namespace hcl

extern "C" {
hipError_t hipGetDevice(int* d) { *d = 0; return hipSuccess; }
hipError_t hipGetLastError(void) { return hipSuccess; }
hipError_t hipDeviceGetAttribute(int* v, hipDeviceAttribute_t, int) { *v = 256; return hipSuccess; }
const char* hipGetErrorString(hipError_t) { return "stub"; }
hipError_t hipEventCreate(hipEvent_t* e) { *e = (hipEvent_t) new int(0); return hipSuccess; }
hipError_t hipEventDestroy(hipEvent_t e) { delete (int*)e; return hipSuccess; }
hipError_t hipEventRecord(hipEvent_t e, hipStream_t s) {
  g_stream_ops.push_back({shim::StreamOp::RECORD, (void*)s, (void*)e, g_launches.size()});
  return hipSuccess;
}
hipError_t hipStreamWaitEvent(hipStream_t s, hipEvent_t e, unsigned) {
  g_stream_ops.push_back({shim::StreamOp::WAIT, (void*)s, (void*)e, g_launches.size()});
  return hipSuccess;
}
hipError_t hipEventElapsedTime(float* ms, hipEvent_t, hipEvent_t) { *ms = 0.f; return hipSuccess; }
}

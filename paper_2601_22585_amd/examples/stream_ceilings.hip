// stream_ceilings.hip -- what plain streaming kernels reach on this GPU, for
// comparison with the library's kernels: R read streams and D write streams,
// every thread touching the same offset in each (the access pattern of a ring
// step: R = 2, D = 1; of an All-Gather step: R = D = 1; of the fused schedules
// over W ranks: R = W with D = 1 or D = W, and R = 1 with D = W), 128-bit
// non-temporal accesses, one tile per workgroup, pseudo-random data.  No part
// of the library is used: this is the yardstick, not the product.
//
//   stream_ceilings [total GiB moved per launch = 8] [launches timed = 5]
//   stream_ceilings host [MiB per stream = 512] [launches timed = 3]
//
// Prints, per pattern, the best of a few launch shapes in GB/s and as a share
// of 8 TB/s.  The `host` form puts streams in pinned host memory instead and
// prints what kernels reach over the host link: reading it, writing it, and
// both at once (the access pattern of a ring step whose blocks travel through
// host memory: incoming block read from the host, outgoing block written to it).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
  fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(1); } } while (0)

constexpr int kMaxStreams = 16;
struct Streams { const u32x4* src[kMaxStreams]; u32x4* dst[kMaxStreams]; };

__global__ void fill_random(uint32_t* p, size_t n) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    uint32_t x = (uint32_t)i * 2654435761u ^ (uint32_t)(i >> 32);
    x ^= x >> 15; x *= 2246822519u; x ^= x >> 13;
    p[i] = (x & 0x807F807Fu) | 0x3A803A80u;   // two bf16 of magnitude about 1e-3, random sign and mantissa
  }
}

template <int R, int D, int U>
__global__ void __launch_bounds__(256) stream_kernel(const Streams s, size_t nvec) {
  const size_t first = (size_t)blockIdx.x * blockDim.x * U + threadIdx.x;
  u32x4 acc[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    acc[u] = u32x4{1u, 2u, (uint32_t)u, blockIdx.x};
    const size_t i = first + (size_t)u * blockDim.x;
    if (i < nvec) {
      u32x4 v[R > 0 ? R : 1];
#pragma unroll
      for (int k = 0; k < R; ++k) v[k] = __builtin_nontemporal_load(s.src[k] + i);
#pragma unroll
      for (int k = 0; k < R; ++k) acc[u] += v[k];
    }
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const size_t i = first + (size_t)u * blockDim.x;
    if (i < nvec) {
#pragma unroll
      for (int k = 0; k < D; ++k) __builtin_nontemporal_store(acc[u], s.dst[k] + i);
      // read-only patterns: a store that practically never happens keeps the loads alive
      if (D == 0 && acc[u].x == 0x12345678u && acc[u].y == 0x9abcdef0u) s.dst[0][i] = acc[u];
    }
  }
}

template <int R, int D, int U>
static double time_shape(const Streams& s, size_t stream_bytes, int threads, int reps) {
  const size_t nvec = stream_bytes / 16, tile = (size_t)threads * U;
  const size_t tiles = (nvec + tile - 1) / tile;
  if (tiles * threads > 0xFFFFFFFFull) return 0.0;   // the runtime refuses launches of 2^32 threads or more
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  for (int it = -2; it < reps; ++it) {
    if (it == 0) CK(hipEventRecord(e0, 0));
    stream_kernel<R, D, U><<<(uint32_t)tiles, threads>>>(s, nvec);
  }
  CK(hipEventRecord(e1, 0));
  CK(hipEventSynchronize(e1));
  CK(hipGetLastError());
  float ms;
  CK(hipEventElapsedTime(&ms, e0, e1));
  CK(hipEventDestroy(e0));
  CK(hipEventDestroy(e1));
  return (double)(R + D) * stream_bytes / (ms / reps) / 1e6;
}

template <int R, int D>
static void pattern(char* arena, size_t total_bytes, int reps) {
  // the arena cut into R + D equal streams, sources first
  const size_t stream_bytes = (total_bytes / (R + D)) & ~(size_t)4095;
  Streams s = {};
  for (int k = 0; k < R; ++k) s.src[k] = (const u32x4*)(arena + stream_bytes * k);
  for (int k = 0; k < D; ++k) s.dst[k] = (u32x4*)(arena + stream_bytes * (R + k));
  if (D == 0) s.dst[0] = (u32x4*)arena;   // a read-only pattern's never-taken store stays inside the stream it reads
  const struct { int threads, unroll; } shapes[] = {{64, 1}, {128, 1}, {256, 1}, {64, 2}, {128, 2}, {64, 4}};
  double best = 0.0;
  int best_shape = 0;
  for (int i = 0; i < 6; ++i) {
    const int t = shapes[i].threads, u = shapes[i].unroll;
    const double g = u == 1 ? time_shape<R, D, 1>(s, stream_bytes, t, reps)
                   : u == 2 ? time_shape<R, D, 2>(s, stream_bytes, t, reps) : time_shape<R, D, 4>(s, stream_bytes, t, reps);
    if (g > best) { best = g; best_shape = i; }
  }
  printf("%2d read, %2d write streams of %5zu MiB: %6.0f GB/s = %4.1f %% of 8 TB/s (%d threads x %d vectors)\n", R, D,
         stream_bytes >> 20, best, best / 80.0, shapes[best_shape].threads, shapes[best_shape].unroll);
  fflush(stdout);
}

// Streams in pinned host memory: GB/s each way over the host link.
template <int R, int D>
static void host_pattern(const char* what, const Streams& s, size_t stream_bytes, int reps, int host_reads, int host_writes) {
  const struct { int threads, unroll; } shapes[] = {{64, 1}, {128, 1}, {256, 1}, {64, 2}, {128, 2}, {64, 4}};
  double best = 0.0;
  int best_shape = 0;
  for (int i = 0; i < 6; ++i) {
    const int t = shapes[i].threads, u = shapes[i].unroll;
    const double g = u == 1 ? time_shape<R, D, 1>(s, stream_bytes, t, reps)
                   : u == 2 ? time_shape<R, D, 2>(s, stream_bytes, t, reps) : time_shape<R, D, 4>(s, stream_bytes, t, reps);
    if (g > best) { best = g; best_shape = i; }
  }
  const double per_stream = best / (R + D);   // every stream moves stream_bytes in the same time
  printf("%-44s host to device %5.1f GB/s, device to host %5.1f GB/s (%d threads x %d vectors)\n", what,
         per_stream * host_reads, per_stream * host_writes, shapes[best_shape].threads, shapes[best_shape].unroll);
  fflush(stdout);
}

static int host_link(size_t stream_bytes, int reps) {
  char *h0, *h1, *dev;
  CK(hipHostMalloc((void**)&h0, stream_bytes, hipHostMallocDefault));
  CK(hipHostMalloc((void**)&h1, stream_bytes, hipHostMallocDefault));
  CK(hipMalloc(&dev, 2 * stream_bytes));
  fill_random<<<8192, 256>>>((uint32_t*)dev, 2 * stream_bytes / 4);
  CK(hipDeviceSynchronize());
  CK(hipMemcpy(h0, dev, stream_bytes, hipMemcpyDeviceToHost));
  Streams s = {};
  s.src[0] = (const u32x4*)h0; s.dst[0] = (u32x4*)dev;
  host_pattern<1, 1>("read from host, write to device:", s, stream_bytes, reps, 1, 0);
  s.src[0] = (const u32x4*)dev; s.dst[0] = (u32x4*)h1;
  host_pattern<1, 1>("read from device, write to host:", s, stream_bytes, reps, 0, 1);
  // both ways at once: sum of a host stream and a device stream, written to the device and to the host
  s.src[0] = (const u32x4*)h0; s.src[1] = (const u32x4*)dev;
  s.dst[0] = (u32x4*)(dev + stream_bytes); s.dst[1] = (u32x4*)h1;
  host_pattern<2, 2>("read host + device, write device + host:", s, stream_bytes, reps, 1, 1);
  CK(hipFree(dev));
  CK(hipHostFree(h0));
  CK(hipHostFree(h1));
  return 0;
}

int main(int argc, char** argv) {
  if (argc > 1 && !strcmp(argv[1], "host")) {
    const size_t mib = argc > 2 ? (size_t)atol(argv[2]) : 512;
    const int reps = argc > 3 ? atoi(argv[3]) : 3;
    if (mib < 1 || mib > 8192 || reps < 1 || reps > 100) {
      fprintf(stderr, "usage: %s host [MiB per stream 1..8192] [launches timed 1..100]\n", argv[0]);
      return 2;
    }
    return host_link(mib << 20, reps);
  }
  const size_t total = (size_t)(argc > 1 ? atol(argv[1]) : 8) << 30;
  const int reps = argc > 2 ? atoi(argv[2]) : 5;
  if (total < ((size_t)1 << 30) || total > ((size_t)64 << 30) || reps < 1 || reps > 1000) {
    fprintf(stderr, "usage: %s [total GiB per launch 1..64] [launches timed 1..1000]\n", argv[0]);
    return 2;
  }
  char* arena;
  CK(hipMalloc(&arena, total));
  fill_random<<<8192, 256>>>((uint32_t*)arena, total / 4);
  CK(hipDeviceSynchronize());
  pattern<1, 0>(arena, total, reps);
  pattern<0, 1>(arena, total, reps);
  pattern<1, 1>(arena, total, reps);
  pattern<2, 1>(arena, total, reps);
  pattern<8, 1>(arena, total, reps);
  pattern<16, 1>(arena, total, reps);
  pattern<0, 8>(arena, total, reps);
  pattern<1, 8>(arena, total, reps);
  pattern<1, 16>(arena, total, reps);
  pattern<8, 8>(arena, total, reps);
  pattern<16, 16>(arena, total, reps);
  CK(hipFree(arena));
  return 0;
}

/*
 * allreduce_latency.c -- calling libhcl from plain C, and the latency-regime
 * figures of the message-size sweep without a binding in the way (the paper
 * separates a latency plot for small messages from the bandwidth plots,
 * Appendix E.4).
 *
 * For each message size it times, for the STEPWISE and the FUSED schedule:
 *   issue  : K back-to-back calls, one synchronisation at the end, per call
 *   single : one call followed by a synchronisation, median of K
 * Buffers come from hipMalloc; nothing else of HIP is used.
 *
 * Build (the library's build script does it):
 *   gcc -O2 -D__HIP_PLATFORM_AMD__ -I/opt/rocm/include -I<repo>/include allreduce_latency.c \
 *       <libdir>/libhcl.so -L/opt/rocm/lib -lamdhip64 -o allreduce_latency
 * Run:
 *   ./allreduce_latency [W=16] [dtype=2 (fp16)] [K=200]
 */
#include <hip/hip_runtime_api.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <time.h>

#include "hcl.h"

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
  fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 1; } } while (0)
#define HK(x) do { hcl_status_t s_ = (x); if (s_ != HCL_OK) { \
  fprintf(stderr, "%s: %s (line %d)\n", hcl_status_string(s_), hcl_last_error(), __LINE__); return 1; } } while (0)

static double now_us(void) {
  struct timespec t;
  clock_gettime(CLOCK_MONOTONIC, &t);
  return t.tv_sec * 1e6 + t.tv_nsec * 1e-3;
}
static int cmp_double(const void *a, const void *b) {
  double x = *(const double *)a, y = *(const double *)b;
  return x < y ? -1 : x > y;
}

int main(int argc, char **argv) {
  const int W = argc > 1 ? atoi(argv[1]) : 16;
  const int dtype = argc > 2 ? atoi(argv[2]) : HCL_FP16;
  const int K = argc > 3 ? atoi(argv[3]) : 200;
  if (W < 1 || W > HCL_MAX_RANKS || dtype < 0 || dtype > 3 || K < 1 || K > 100000) {
    fprintf(stderr, "usage: %s [W 1..16] [dtype 0..3] [K]\n", argv[0]);
    return 2;
  }
  const size_t es = (dtype == HCL_BF16 || dtype == HCL_FP16) ? 2 : 4;
  const size_t max_bytes = (size_t)4 << 20;
  void *send[HCL_MAX_RANKS], *recv[HCL_MAX_RANKS];
  for (int r = 0; r < W; ++r) {
    CK(hipMalloc(&send[r], max_bytes));
    CK(hipMalloc(&recv[r], max_bytes));
    CK(hipMemset(send[r], 0, max_bytes));   /* zeros: every sum stays finite */
  }
  hipStream_t stream;
  CK(hipStreamCreate(&stream));
  double *lat = (double *)malloc(sizeof(double) * (size_t)K);
  if (!lat) return 1;

  printf("W=%d dtype=%d K=%d  (times in microseconds)\n", W, dtype, K);
  printf("%12s | %14s %14s | %14s %14s\n", "bytes/rank", "stepwise issue", "stepwise single", "fused issue", "fused single");
  for (size_t bytes = 8192; bytes <= max_bytes; bytes *= 4) {
    const size_t count = bytes / es;
    size_t block_bytes = (count + W - 1) / W * es;
    const size_t chunk = block_bytes < ((size_t)4 << 20) ? 0 : (size_t)4 << 20;
    double res[2][2];
    for (int sched = 0; sched < 2; ++sched) {
      hcl_opts_t o;
      memset(&o, 0, sizeof o);
      o.sched = sched ? HCL_SCHED_FUSED : HCL_SCHED_STEPWISE;
      for (int i = 0; i < 10; ++i)
        HK(hcl_allreduce_sim((const void *const *)send, recv, W, count, (hcl_dtype_t)dtype, HCL_SUM, chunk, &o, stream));
      CK(hipStreamSynchronize(stream));
      double t0 = now_us();
      for (int i = 0; i < K; ++i)
        HK(hcl_allreduce_sim((const void *const *)send, recv, W, count, (hcl_dtype_t)dtype, HCL_SUM, chunk, &o, stream));
      CK(hipStreamSynchronize(stream));
      res[sched][0] = (now_us() - t0) / K;
      for (int i = 0; i < K; ++i) {
        t0 = now_us();
        HK(hcl_allreduce_sim((const void *const *)send, recv, W, count, (hcl_dtype_t)dtype, HCL_SUM, chunk, &o, stream));
        CK(hipStreamSynchronize(stream));
        lat[i] = now_us() - t0;
      }
      qsort(lat, (size_t)K, sizeof(double), cmp_double);
      res[sched][1] = lat[K / 2];
    }
    printf("%12zu | %14.1f %14.1f | %14.1f %14.1f\n", bytes, res[0][0], res[0][1], res[1][0], res[1][1]);
    fflush(stdout);
  }
  for (int r = 0; r < W; ++r) {
    CK(hipFree(send[r]));
    CK(hipFree(recv[r]));
  }
  CK(hipStreamDestroy(stream));
  free(lat);
  return 0;
}

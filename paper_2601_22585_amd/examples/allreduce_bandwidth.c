/*
 * allreduce_bandwidth.c -- the bandwidth regime of the message-size sweep
 * (Appendix E.4: large messages are reported as bandwidth) measured from plain
 * C, without a binding between the caller and the library: for every size, K
 * All-Reduce calls issued back to back on one stream, one synchronisation at
 * the end.  Buffers hold pseudo-random values of gradient-like magnitude
 * (bandwidth on zero-filled buffers is up to 3 % higher on MI355X and would
 * flatter the figures).
 *
 *   allreduce_bandwidth [W=8] [dtype=1 (bf16)] [min MiB per rank=16] [max MiB per rank=1024]
 *
 * Prints, per size and schedule: ms per call, S / t in GB/s, and the schedule's
 * own bytes (STEPWISE 5 (W - 1) S, FUSED 2 W S) per second as a share of 8 TB/s.
 *
 * Build (the library's build script does it):
 *   gcc -O2 -D__HIP_PLATFORM_AMD__ -I/opt/rocm/include -I<repo>/include allreduce_bandwidth.c \
 *       -L<libdir> -lhcl -L/opt/rocm/lib -lamdhip64 -o allreduce_bandwidth
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <time.h>

#include "hcl.h"

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
  fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 1; } } while (0)
#define HK(x) do { hcl_status_t s_ = (x); if (s_ != HCL_OK) { \
  fprintf(stderr, "%s: %s (line %d)\n", hcl_status_string(s_), hcl_last_error(), __LINE__); return 1; } } while (0)

static double now_ms(void) {
  struct timespec t;
  clock_gettime(CLOCK_MONOTONIC, &t);
  return t.tv_sec * 1e3 + t.tv_nsec * 1e-6;
}

int main(int argc, char **argv) {
  const int W = argc > 1 ? atoi(argv[1]) : 8;
  const int dtype = argc > 2 ? atoi(argv[2]) : HCL_BF16;
  const size_t lo_mib = argc > 3 ? (size_t)atol(argv[3]) : 16, hi_mib = argc > 4 ? (size_t)atol(argv[4]) : 1024;
  if (W < 2 || W > HCL_MAX_RANKS || dtype < HCL_FP32 || dtype > HCL_INT32 || lo_mib < 1 || hi_mib < lo_mib || hi_mib > 4096) {
    fprintf(stderr, "usage: %s [W 2..16] [dtype 0..3] [min MiB per rank] [max MiB per rank <= 4096]\n", argv[0]);
    return 2;
  }
  const size_t es = (dtype == HCL_BF16 || dtype == HCL_FP16) ? 2 : 4, max_bytes = hi_mib << 20;
  /* one host block of pseudo-random values, copied over every buffer at shifting offsets */
  const size_t blk = (size_t)16 << 20;
  uint32_t *host = (uint32_t *)malloc(blk);
  if (!host) return 1;
  uint64_t x = 88172645463325252ull;
  for (size_t i = 0; i < blk / 4; ++i) {
    x ^= x << 13; x ^= x >> 7; x ^= x << 17;
    const uint32_t w = (uint32_t)(x >> 16);
    /* random sign and mantissa under a fixed small exponent (about 1e-3); int32: small integers */
    host[i] = dtype == HCL_BF16 ? ((w & 0x807F807Fu) | 0x3A803A80u)
            : dtype == HCL_FP16 ? ((w & 0x83FF83FFu) | 0x14001400u)
            : dtype == HCL_FP32 ? ((w & 0x807FFFFFu) | 0x3A800000u) : (w & 0x3FFu);
  }
  void *send[HCL_MAX_RANKS], *recv[HCL_MAX_RANKS];
  for (int r = 0; r < W; ++r) {
    CK(hipMalloc(&send[r], max_bytes));
    CK(hipMalloc(&recv[r], max_bytes));
    for (size_t off = 0; off < max_bytes; off += blk) {
      const size_t n = max_bytes - off < blk ? max_bytes - off : blk;
      const size_t shift = ((size_t)r * 4099 + off / blk * 257) % 1024 * 4;   /* so that ranks and blocks differ */
      CK(hipMemcpy((char *)send[r] + off, (char *)host + shift, n - shift, hipMemcpyHostToDevice));
      CK(hipMemcpy((char *)send[r] + off + n - shift, host, shift, hipMemcpyHostToDevice));
    }
  }
  hipStream_t stream;
  CK(hipStreamCreate(&stream));
  printf("W=%d dtype=%d; ms per call | S/t GB/s | own bytes as %% of 8 TB/s\n", W, dtype);
  printf("%10s | %28s | %28s\n", "MiB/rank", "stepwise", "fused");
  for (size_t mib = lo_mib; mib <= hi_mib; mib *= 2) {
    const size_t bytes = mib << 20, count = bytes / es;
    int K = (int)(((size_t)8192 + mib - 1) / mib);
    if (K < 3) K = 3;
    if (K > 100) K = 100;
    printf("%10zu |", mib);
    for (int sched = 0; sched < 2; ++sched) {
      hcl_opts_t o;
      memset(&o, 0, sizeof o);
      o.sched = sched ? HCL_SCHED_FUSED : HCL_SCHED_STEPWISE;
      for (int i = 0; i < 3; ++i)
        HK(hcl_allreduce_sim((const void *const *)send, recv, W, count, (hcl_dtype_t)dtype, HCL_SUM, (size_t)4 << 20, &o, stream));
      CK(hipStreamSynchronize(stream));
      const double t0 = now_ms();
      for (int i = 0; i < K; ++i)
        HK(hcl_allreduce_sim((const void *const *)send, recv, W, count, (hcl_dtype_t)dtype, HCL_SUM, (size_t)4 << 20, &o, stream));
      CK(hipStreamSynchronize(stream));
      const double ms = (now_ms() - t0) / K;
      const double own = (sched ? 2.0 * W : 5.0 * (W - 1)) * (double)bytes;
      printf(" %9.4f %8.1f %7.1f %% %s", ms, bytes / ms / 1e6, own / ms / 1e6 / 80.0, sched ? "\n" : "|");
    }
    fflush(stdout);
  }
  for (int r = 0; r < W; ++r) {
    CK(hipFree(send[r]));
    CK(hipFree(recv[r]));
  }
  CK(hipStreamDestroy(stream));
  free(host);
  return 0;
}

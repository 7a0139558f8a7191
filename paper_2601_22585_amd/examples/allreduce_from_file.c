/*
 * allreduce_from_file.c -- the library driven from plain C, end to end: rank
 * buffers read from a file, one ring All-Reduce per schedule through the call
 * shape the paper's library shows to frameworks (send buffer, receive buffer,
 * count, datatype, operator, stream -- Section 4.4), every rank's result
 * written back to a file.  No binding, no Python: hipMalloc, hipMemcpy, the C
 * ABI of include/hcl.h.
 *
 *   allreduce_from_file W count dtype chunk_bytes in.bin out.bin
 *
 * in.bin : W * count elements, rank 0's vector first (raw little-endian wire
 *          elements of hcl_dtype_t `dtype`)
 * out.bin: for the STEPWISE schedule, then the STEPWISE schedule in place with
 *          the last Reduce-Scatter step forwarding its result, then the FUSED
 *          schedule: the W receive buffers, rank 0 first -- 3 * W * count elements
 *
 * Build (the library's build script does it):
 *   gcc -O2 -D__HIP_PLATFORM_AMD__ -I/opt/rocm/include -I<repo>/include allreduce_from_file.c \
 *       <libdir>/libhcl.so -L/opt/rocm/lib -lamdhip64 -o allreduce_from_file
 */
#include <hip/hip_runtime_api.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "hcl.h"

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
  fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 1; } } while (0)
#define HK(x) do { hcl_status_t s_ = (x); if (s_ != HCL_OK) { \
  fprintf(stderr, "%s: %s (line %d)\n", hcl_status_string(s_), hcl_last_error(), __LINE__); return 1; } } while (0)

static size_t elem_bytes(int dtype) {
  switch (dtype) {
    case HCL_BF16: case HCL_FP16: return 2;
    case HCL_FP64: case HCL_INT64: return 8;
    case HCL_UINT8: return 1;
    default: return 4;
  }
}

int main(int argc, char **argv) {
  if (argc != 7) {
    fprintf(stderr, "usage: %s W count dtype chunk_bytes in.bin out.bin\n", argv[0]);
    return 2;
  }
  const int W = atoi(argv[1]);
  const size_t count = (size_t)strtoull(argv[2], NULL, 10);
  const int dtype = atoi(argv[3]);
  const size_t chunk_bytes = (size_t)strtoull(argv[4], NULL, 10);
  if (W < 1 || W > HCL_MAX_RANKS || count == 0) { fprintf(stderr, "bad W or count\n"); return 2; }
  const size_t bytes = count * elem_bytes(dtype);

  void *host = malloc(bytes);
  const void *send[HCL_MAX_RANKS];
  void *recv[HCL_MAX_RANKS], *work[HCL_MAX_RANKS];
  FILE *in = fopen(argv[5], "rb");
  if (!host || !in) { fprintf(stderr, "cannot open %s\n", argv[5]); return 1; }
  for (int r = 0; r < W; ++r) {
    void *s;
    if (fread(host, 1, bytes, in) != bytes) { fprintf(stderr, "%s is too short\n", argv[5]); return 1; }
    CK(hipMalloc(&s, bytes));
    CK(hipMalloc(&recv[r], bytes));
    CK(hipMalloc(&work[r], bytes));
    CK(hipMemcpy(s, host, bytes, hipMemcpyHostToDevice));
    send[r] = s;
  }
  fclose(in);
  hipStream_t stream;
  CK(hipStreamCreateWithFlags(&stream, hipStreamNonBlocking));

  FILE *out = fopen(argv[6], "wb");
  if (!out) { fprintf(stderr, "cannot open %s\n", argv[6]); return 1; }
  for (int variant = 0; variant < 3; ++variant) {
    hcl_opts_t o;
    memset(&o, 0, sizeof o);
    void *const *dst = recv;
    if (variant == 1) {  /* in place on a copy of the inputs, last Reduce-Scatter step forwarding */
      o.fuse_rs_ag = 1;
      for (int r = 0; r < W; ++r) CK(hipMemcpyAsync(work[r], send[r], bytes, hipMemcpyDeviceToDevice, stream));
      dst = work;
    } else {
      o.sched = variant == 2 ? HCL_SCHED_FUSED : HCL_SCHED_STEPWISE;
      for (int r = 0; r < W; ++r) CK(hipMemsetAsync(recv[r], 0, bytes, stream));
    }
    HK(hcl_allreduce_sim(variant == 1 ? (const void *const *)work : send, dst, W, count, (hcl_dtype_t)dtype, HCL_SUM,
                         chunk_bytes, &o, stream));
    CK(hipStreamSynchronize(stream));
    for (int r = 0; r < W; ++r) {
      CK(hipMemcpy(host, dst[r], bytes, hipMemcpyDeviceToHost));
      if (fwrite(host, 1, bytes, out) != bytes) { fprintf(stderr, "short write\n"); return 1; }
    }
  }
  fclose(out);
  for (int r = 0; r < W; ++r) {
    CK(hipFree((void *)send[r]));
    CK(hipFree(recv[r]));
    CK(hipFree(work[r]));
  }
  CK(hipStreamDestroy(stream));
  free(host);
  printf("allreduce_from_file: W=%d count=%zu dtype=%d: three schedules written to %s\n", W, count, dtype, argv[6]);
  return 0;
}

/* TEST INFRASTRUCTURE: drives the CPU oracle (oracle/ring_oracle.c, linked in)
 * under AddressSanitizer and UBSan: exact-size heap buffers around every
 * argument, ragged counts, every wire type, operator, order and rounding.  The
 * sanitizers watch the memory accesses; the driver itself checks what needs no
 * second implementation: integer results against plain wrapped sums, every rank
 * identical after All-Reduce, All-Gather blocks equal to their sources. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

size_t orc_esize(int dtype);
int orc_allreduce_op(void *const *work, int W, size_t count, int dtype, int op, const int *ring, size_t chunk_elems);
int orc_reduce_scatter_op(void *const *work, void *const *out, int W, size_t recvcount, int dtype, int op, const int *ring, size_t chunk_elems);
int orc_all_gather(const void *const *in, void *const *out, int W, size_t sendcount, int dtype, const int *ring, size_t chunk_elems);
int orc_reduce_op(const void *const *in, void *out, int W, size_t count, int dtype, int op, const int *ring, int root, size_t chunk_elems);
int orc_broadcast(const void *in, void *const *out, int W, size_t count, int dtype, const int *ring, int root);
int orc_alltoall(const void *const *in, void *const *out, int W, size_t n, int dtype);
int orc_allreduce_var(const void *const *in, void *const *out, int W, size_t count, int dtype, int op, const int *ring, int order, int rounding);
int orc_reduce_scatter_var(const void *const *in, void *const *out, int W, size_t n, int dtype, int op, const int *ring, int order, int rounding);
int orc_reduce_var(const void *const *in, void *out, int W, size_t count, int dtype, int op, const int *ring, int root, int order, int rounding);
int orc_ring_step(int W, const int *ring, int phase, int step, int rank, int *send_block, int *recv_block);

enum { FP32, BF16, FP16, INT32, FP64, INT64, UINT8 };

static uint64_t state = 88172645463325252ull;
static uint64_t rnd(void) { state ^= state << 13; state ^= state >> 7; state ^= state << 17; return state; }
static int fails = 0;
#define CHECK(c, ...) do { if (!(c)) { fprintf(stderr, "oracle_check FAILED: " __VA_ARGS__); fprintf(stderr, "\n"); ++fails; } } while (0)

/* random bits for the float types would hit NaN payloads whose bits may differ between ranks;
 * small integers are exact in every wire type */
static void fill(void *p, size_t n, int dtype) {
  for (size_t i = 0; i < n; ++i) {
    const int v = (int)(rnd() % 7) - 3;
    switch (dtype) {
      case FP32: ((float *)p)[i] = (float)v; break;
      case BF16: { float f = (float)v; uint32_t u; memcpy(&u, &f, 4); ((uint16_t *)p)[i] = (uint16_t)(u >> 16); break; }
      case FP16: { static const uint16_t t[7] = {0xC200, 0xC000, 0xBC00, 0x0000, 0x3C00, 0x4000, 0x4200}; ((uint16_t *)p)[i] = t[v + 3]; break; }
      case INT32: ((int32_t *)p)[i] = (int32_t)rnd(); break;
      case FP64: ((double *)p)[i] = (double)v; break;
      case INT64: ((int64_t *)p)[i] = (int64_t)rnd(); break;
      default: ((uint8_t *)p)[i] = (uint8_t)rnd(); break;
    }
  }
}

int main(void) {
  static const int Ws[] = {1, 2, 3, 5, 8, 16};
  static const size_t counts[] = {1, 2, 7, 64, 1001};
  int runs = 0;
  for (unsigned wi = 0; wi < sizeof Ws / sizeof *Ws; ++wi)
    for (unsigned ci = 0; ci < sizeof counts / sizeof *counts; ++ci)
      for (int dtype = FP32; dtype <= UINT8; ++dtype) {
        const int W = Ws[wi];
        const size_t n = counts[ci], es = orc_esize(dtype);
        const size_t chunk = (size_t[]){0, 1, 3, 64}[rnd() % 4];
        int ring[16];
        for (int k = 0; k < W; ++k) ring[k] = k;
        for (int k = W - 1; k > 0; --k) { int j = (int)(rnd() % (unsigned)(k + 1)), t = ring[k]; ring[k] = ring[j]; ring[j] = t; }
        const int op = (int)(rnd() % 4), root = (int)(rnd() % (unsigned)W);
        void *in[16], *work[16], *out[16], *big[16];
        for (int r = 0; r < W; ++r) {
          in[r] = malloc(n * W * es);        /* exact sizes: one byte too far is a sanitizer report */
          work[r] = malloc(n * W * es);
          out[r] = malloc(n * es);
          big[r] = malloc(n * W * es);
          fill(in[r], n * W, dtype);
        }
        /* All-Reduce on the leading n elements (ragged blocks), in place on copies */
        for (int r = 0; r < W; ++r) memcpy(work[r], in[r], n * es);
        CHECK(orc_allreduce_op(work, W, n, dtype, op, ring, chunk) == 0, "allreduce rc");
        for (int r = 1; r < W; ++r) CHECK(!memcmp(work[r], work[0], n * es), "ranks differ after all-reduce W=%d n=%zu dtype=%d", W, n, dtype);
        if (dtype == INT32 && op == 0)
          for (size_t i = 0; i < n; ++i) {
            uint32_t s = 0;
            for (int r = 0; r < W; ++r) s += ((uint32_t *)in[r])[i];
            CHECK(((uint32_t *)work[0])[i] == s, "int32 sum W=%d n=%zu i=%zu", W, n, i);
          }
        /* Reduce-Scatter of W * n elements, then All-Gather of the shards */
        for (int r = 0; r < W; ++r) memcpy(work[r], in[r], n * W * es);
        CHECK(orc_reduce_scatter_op(work, out, W, n, dtype, op, ring, chunk) == 0, "reduce_scatter rc");
        CHECK(orc_all_gather((const void *const *)out, big, W, n, dtype, ring, chunk) == 0, "all_gather rc");
        for (int r = 0; r < W; ++r)
          for (int q = 0; q < W; ++q) CHECK(!memcmp((char *)big[r] + (size_t)q * n * es, out[q], n * es), "all-gather block W=%d", W);
        /* the closed-form variants agree with the message-passing replay in ring order, each rounding */
        CHECK(orc_reduce_scatter_var((const void *const *)in, big, W, n, dtype, op, ring, 0, 0) == 0, "reduce_scatter_var rc");
        for (int r = 0; r < W; ++r) CHECK(!memcmp(big[r], out[r], n * es), "variant replay differs from the ring W=%d n=%zu dtype=%d op=%d", W, n, dtype, op);
        for (int order = 0; order < 2; ++order)
          for (int rounding = 0; rounding < 2; ++rounding) {
            CHECK(orc_allreduce_var((const void *const *)in, big, W, n, dtype, op, ring, order, rounding) == 0, "allreduce_var rc");
            CHECK(orc_reduce_var((const void *const *)in, work[0], W, n, dtype, op, ring, root, order, rounding) == 0, "reduce_var rc");
          }
        CHECK(orc_reduce_op((const void *const *)in, work[0], W, n, dtype, op, ring, root, chunk) == 0, "reduce rc");
        CHECK(orc_broadcast(in[root], big, W, n, dtype, ring, root) == 0, "broadcast rc");
        for (int r = 0; r < W; ++r) CHECK(!memcmp(big[r], in[root], n * es), "broadcast copy");
        CHECK(orc_alltoall((const void *const *)in, big, W, n, dtype) == 0, "alltoall rc");
        for (int r = 0; r < W; ++r)
          for (int q = 0; q < W; ++q)
            CHECK(!memcmp((char *)big[r] + (size_t)q * n * es, (char *)in[q] + (size_t)r * n * es, n * es), "all-to-all block");
        for (int s = 0; s + 2 <= W; ++s)
          for (int r = 0; r < W; ++r) {
            int a, b;
            CHECK(orc_ring_step(W, ring, s & 1, s, r, &a, &b) == 0 && a >= 0 && a < W && b >= 0 && b < W, "ring_step");
          }
        for (int r = 0; r < W; ++r) { free(in[r]); free(work[r]); free(out[r]); free(big[r]); }
        ++runs;
      }
  if (fails) { fprintf(stderr, "oracle_check: %d failure(s)\n", fails); return 1; }
  printf("oracle_check: ok (%d configurations)\n", runs);
  return 0;
}

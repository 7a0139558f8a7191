/*
 * ring_oracle.c -- CPU oracle for ring Reduce-Scatter / All-Gather / All-Reduce
 * over W simulated ranks.  TEST INFRASTRUCTURE ONLY: nothing in the product
 * library links, includes or calls this file; it shares no code with the HIP
 * path.  It is deliberately plain and slow so that it can be checked against
 * the definitions by eye.
 *
 * What is replayed.  The paper names All-Reduce, All-Gather and Reduce-Scatter
 * as the collectives of data-parallel training (Section 1; Appendix B.1,
 * "Communication patterns in DL"; Appendix D.4 and Table "Communication
 * patterns across DeepSpeed ZeRO stages") and says that reductions run on the
 * GPU (Appendix E.3), but leaves the inside of the collectives to the vendor
 * libraries (Section 4.1 "Key Approach", Section 4.2).  The algorithm below is
 * therefore the textbook ring: W-1 Reduce-Scatter steps followed by W-1
 * All-Gather steps, written as literal message passing -- in every step each
 * rank first puts one block into its successor's inbox, then every rank
 * consumes its own inbox.  Because all sends of a step complete before any
 * receive of that step is applied, "all ranks act simultaneously" holds by
 * construction.
 *
 * Conventions (the paper is silent on them; they are the readings this
 * project fixes):
 *   - ring[] is a permutation of 0..W-1; next(r) is the entry after r in
 *     ring[], cyclically; pos(r) is r's index in ring[].
 *   - All-Reduce splits the count-element vector into W blocks of
 *     B = ceil(count / W) elements; block c covers
 *     [min(c*B, count), min((c+1)*B, count)).  Trailing blocks may be short or
 *     empty.  Reduce-Scatter / All-Gather take B = recvcount / sendcount.
 *   - Reduce-Scatter step s (0 <= s <= W-2): rank r sends block
 *     ring[(pos(r) - s - 1) mod W] and receives block ring[(pos(r) - s - 2) mod W].
 *     After the last step rank r holds the finished block r.
 *   - All-Gather step s: rank r sends block ring[(pos(r) - s) mod W] and
 *     receives block ring[(pos(r) - s - 1) mod W].
 *   - One hop of the reduction, per element:
 *         partial = round_T( f32(incoming) + f32(local) )
 *     incoming operand on the left, one IEEE binary32 addition (round to
 *     nearest even), then one conversion to the wire type T with round to
 *     nearest even.  Subnormals are kept, overflow gives infinity, NaN
 *     propagates.  int32 adds modulo 2^32.
 *   - A chunk is a contiguous run of chunk_elems elements inside a block.  It
 *     only orders the element loop; it never changes a value.
 *
 *   - Reduction operators other than the sum (the call shape carries a
 *     reduction operator, Section 4.4): one hop is
 *         partial = round_T( op(f32(incoming), f32(local)) )
 *     for the product (the product of two bf16 / fp16 values is exact in
 *     binary32, so the hop is the correctly rounded product), and
 *         partial = op(incoming, local)
 *     for maximum / minimum, which follow IEEE 754-2019 clause 9.6: a NaN
 *     operand gives NaN, and -0 orders below +0.  int32: the product wraps
 *     modulo 2^32, maximum / minimum compare as signed integers.
 *   - Further wire types: fp64 (one IEEE binary64 operation per hop, no
 *     widening, nothing to round afterwards), int64 (wraps modulo 2^64, signed
 *     comparisons) and uint8 (wraps modulo 2^8, unsigned comparisons).
 *   - Tree order (a reordered-class variant, like binary32 accumulation): the
 *     ranks' values are taken in ring order ring[0], ring[1], ..., ring[W-1] --
 *     the same order for every block -- and combined level by level, neighbours
 *     first: (v0 op v1), (v2 op v3), ...; an odd value at the end of a level
 *     moves up unchanged.  Every node is rounded to the wire type (per-node
 *     rounding) or the whole tree is evaluated in binary32 and rounded once.
 *
 *   - Reduce / Broadcast travel along the same ring as chains that end
 *     (Reduce) or start (Broadcast) at the root; Reduce therefore sums in the
 *     order next(root), ..., root.  All-to-All is the plain block transpose.
 *
 * Pins (tests/, marker "not gpu"): exact-rational brute force of the closed
 * form fold on tiny inputs; the hand-derived cancellation example under
 * tests/golden/; W = 2 against numpy / torch elementwise adds; integer-valued
 * inputs against exact integer sums; conversions against numpy float16 and
 * torch bfloat16 over all 2^16 patterns and sampled fp32 patterns; set-based
 * simulation of the block tables for every W <= 16.  Operators, tree order and
 * single rounding: exact-rational brute force of every combination; the
 * hand-derived overflow / underflow product example and the tree-order
 * cancellation example under tests/golden/; IEEE 754-2019 maximum / minimum of
 * special operands written out there; two ranks against numpy / torch multiply,
 * maximum, minimum on random bit patterns; order independence of maximum /
 * minimum and of the integer types; the pairwise-summation and 2-ulp bounds.
 * fp64 / int64 / uint8: the same brute force at binary64 width and in big
 * integers with explicit wrap.  The paper prints no value for this path, so
 * parity against the paper itself is unpinned; every pin is derived from the
 * arithmetic.
 *
 * Build: gcc -O2 -std=c11 -fopenmp -ffp-contract=off -fPIC -shared
 */
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_FP32 = 0, ORC_BF16 = 1, ORC_FP16 = 2, ORC_INT32 = 3, ORC_FP64 = 4, ORC_INT64 = 5, ORC_UINT8 = 6 };
enum { ORC_OK = 0, ORC_BAD_ARG = 1, ORC_NO_MEM = 2 };
enum { ORC_PHASE_RS = 0, ORC_PHASE_AG = 1 };
enum { ORC_SUM = 0, ORC_PROD = 1, ORC_MAX = 2, ORC_MIN = 3 };
enum { ORC_ORDER_RING = 0, ORC_ORDER_TREE = 1 };
enum { ORC_ROUND_EACH = 0, ORC_ROUND_ONCE = 1 };

/* ------------------------------------------------------------------ */
/* bit views                                                           */
/* ------------------------------------------------------------------ */
static uint32_t f32_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static float bits_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

/* ------------------------------------------------------------------ */
/* bfloat16: 1 sign, 8 exponent, 7 fraction bits = top half of binary32 */
/* ------------------------------------------------------------------ */
float orc_bf16_to_f32(uint16_t h) { return bits_f32((uint32_t)h << 16); }

uint16_t orc_f32_to_bf16(float f)
{
    uint32_t u = f32_bits(f);
    uint32_t keep = u >> 16;         /* the 16 bits that survive          */
    uint32_t drop = u & 0xFFFFu;     /* the 16 bits that are rounded away */
    if ((u & 0x7FFFFFFFu) > 0x7F800000u)        /* NaN stays NaN (quiet)   */
        return (uint16_t)(keep | 0x0040u);
    if (drop > 0x8000u) keep += 1;              /* above half: up          */
    else if (drop == 0x8000u && (keep & 1u)) keep += 1; /* tie: to even    */
    /* a carry out of the fraction moves into the exponent, and the largest
       finite value carries into the infinity pattern: both are what IEEE
       round-to-nearest-even prescribes */
    return (uint16_t)keep;
}

/* ------------------------------------------------------------------ */
/* binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits            */
/* ------------------------------------------------------------------ */
float orc_f16_to_f32(uint16_t h)
{
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t e = (h >> 10) & 0x1Fu;
    uint32_t m = h & 0x3FFu;
    if (e == 0x1Fu)                               /* inf / NaN */
        return bits_f32(sign | 0x7F800000u | (m << 13));
    if (e == 0) {                                 /* zero / subnormal: m * 2^-24 */
        float mag = ldexpf((float)m, -24);
        return sign ? -mag : mag;
    }
    return bits_f32(sign | ((e + 112u) << 23) | (m << 13));
}

uint16_t orc_f32_to_f16(float f)
{
    uint32_t u = f32_bits(f);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t e = (u >> 23) & 0xFFu;
    uint32_t m = u & 0x7FFFFFu;
    if (e == 0xFFu)
        return (uint16_t)(sign | (m ? 0x7E00u : 0x7C00u));
    if (e == 0)            /* |f| < 2^-126, far below half of 2^-24 */
        return sign;
    int E = (int)e - 127;                 /* f = sig * 2^(E-23)            */
    uint32_t sig = 0x800000u | m;         /* 24-bit significand            */
    if (E > 15)
        return (uint16_t)(sign | 0x7C00u);
    uint32_t q, rem, half;
    uint16_t mag;
    if (E >= -14) {                       /* normal range of binary16      */
        q = sig >> 13;                    /* 11 bits, leading one included */
        rem = sig & 0x1FFFu;
        half = 0x1000u;
        mag = (uint16_t)((((uint32_t)(E + 15)) << 10) | (q & 0x3FFu));
    } else {                              /* subnormal: multiples of 2^-24 */
        int s = -(E + 1);                 /* q = sig / 2^s                 */
        if (s > 24)                       /* below half an ulp             */
            return sign;
        q = sig >> s;
        rem = sig & ((1u << s) - 1u);
        half = 1u << (s - 1);
        mag = (uint16_t)q;
    }
    if (rem > half || (rem == half && (mag & 1u)))
        mag = (uint16_t)(mag + 1);        /* carry may reach exponent / inf */
    return (uint16_t)(sign | mag);
}

/* ------------------------------------------------------------------ */
/* one hop: partial = round_T(f32(incoming) + f32(local))              */
/* ------------------------------------------------------------------ */
float    orc_hop_f32 (float incoming, float local)       { return incoming + local; }
uint16_t orc_hop_bf16(uint16_t incoming, uint16_t local)
{ return orc_f32_to_bf16(orc_bf16_to_f32(incoming) + orc_bf16_to_f32(local)); }
uint16_t orc_hop_f16 (uint16_t incoming, uint16_t local)
{ return orc_f32_to_f16(orc_f16_to_f32(incoming) + orc_f16_to_f32(local)); }
int32_t  orc_hop_i32 (int32_t incoming, int32_t local)
{ return (int32_t)((uint32_t)incoming + (uint32_t)local); }

/* ------------------------------------------------------------------ */
/* the other reduction operators                                       */
/* ------------------------------------------------------------------ */
/* IEEE 754-2019 maximum / minimum on binary32 values: NaN if either operand
   is NaN; of two zeros with different signs the maximum is +0, the minimum -0 */
static float f32_maximum(float a, float b)
{
    if (isnan(a) || isnan(b)) return NAN;
    if (a > b) return a;
    if (b > a) return b;
    return signbit(a) ? b : a;      /* equal values: differ at most in the sign of zero */
}
static float f32_minimum(float a, float b)
{
    if (isnan(a) || isnan(b)) return NAN;
    if (a < b) return a;
    if (b < a) return b;
    return signbit(a) ? a : b;
}
/* op on two binary32 values, one IEEE operation, no rounding to a wire type */
static float f32_apply(int op, float a, float b)
{
    switch (op) {
    case ORC_PROD: return a * b;
    case ORC_MAX:  return f32_maximum(a, b);
    case ORC_MIN:  return f32_minimum(a, b);
    default:       return a + b;
    }
}
static int32_t i32_apply(int op, int32_t a, int32_t b)
{
    switch (op) {
    case ORC_PROD: return (int32_t)((uint32_t)a * (uint32_t)b);
    case ORC_MAX:  return a > b ? a : b;
    case ORC_MIN:  return a < b ? a : b;
    default:       return (int32_t)((uint32_t)a + (uint32_t)b);
    }
}
/* the same operators on the wider and narrower wire types */
static double f64_apply(int op, double a, double b)
{
    switch (op) {
    case ORC_PROD: return a * b;
    case ORC_MAX:
        if (isnan(a) || isnan(b)) return (double)NAN;
        if (a > b) return a;
        if (b > a) return b;
        return signbit(a) ? b : a;
    case ORC_MIN:
        if (isnan(a) || isnan(b)) return (double)NAN;
        if (a < b) return a;
        if (b < a) return b;
        return signbit(a) ? a : b;
    default: return a + b;
    }
}
static int64_t i64_apply(int op, int64_t a, int64_t b)
{
    switch (op) {
    case ORC_PROD: return (int64_t)((uint64_t)a * (uint64_t)b);
    case ORC_MAX:  return a > b ? a : b;
    case ORC_MIN:  return a < b ? a : b;
    default:       return (int64_t)((uint64_t)a + (uint64_t)b);
    }
}
static uint8_t u8_apply(int op, uint8_t a, uint8_t b)
{
    switch (op) {
    case ORC_PROD: return (uint8_t)(((unsigned)a * (unsigned)b) & 0xFFu);
    case ORC_MAX:  return a > b ? a : b;
    case ORC_MIN:  return a < b ? a : b;
    default:       return (uint8_t)(((unsigned)a + (unsigned)b) & 0xFFu);
    }
}

/* widen a wire element to binary32 (exact) and round binary32 to the wire type */
static float wire_to_f32(const void *p, size_t i, int dtype)
{
    if (dtype == ORC_FP32) return ((const float *)p)[i];
    uint16_t h = ((const uint16_t *)p)[i];
    return dtype == ORC_BF16 ? orc_bf16_to_f32(h) : orc_f16_to_f32(h);
}
static void f32_to_wire(void *p, size_t i, int dtype, float v)
{
    if (dtype == ORC_FP32) ((float *)p)[i] = v;
    else ((uint16_t *)p)[i] = dtype == ORC_BF16 ? orc_f32_to_bf16(v) : orc_f32_to_f16(v);
}
/* round a binary32 value to the wire type and widen it again: the value a
   partial has after it travelled in the wire type */
static float through_wire(float v, int dtype)
{
    if (dtype == ORC_BF16) return orc_bf16_to_f32(orc_f32_to_bf16(v));
    if (dtype == ORC_FP16) return orc_f16_to_f32(orc_f32_to_f16(v));
    return v;
}

/* one hop with operator `op`, element-wise over a run: local[i] = round_T(op(inbox[i], local[i])) */
static void hop_run_op(void *local, const void *inbox, size_t n, int dtype, int op)
{
    ptrdiff_t i, nn = (ptrdiff_t)n;
    if (dtype == ORC_INT32) {
        int32_t *l = (int32_t *)local; const int32_t *in = (const int32_t *)inbox;
        #pragma omp parallel for schedule(static) if (nn > 32768)
        for (i = 0; i < nn; ++i) l[i] = i32_apply(op, in[i], l[i]);
        return;
    }
    if (dtype == ORC_FP64) {
        double *l = (double *)local; const double *in = (const double *)inbox;
        #pragma omp parallel for schedule(static) if (nn > 32768)
        for (i = 0; i < nn; ++i) l[i] = f64_apply(op, in[i], l[i]);
        return;
    }
    if (dtype == ORC_INT64) {
        int64_t *l = (int64_t *)local; const int64_t *in = (const int64_t *)inbox;
        #pragma omp parallel for schedule(static) if (nn > 32768)
        for (i = 0; i < nn; ++i) l[i] = i64_apply(op, in[i], l[i]);
        return;
    }
    if (dtype == ORC_UINT8) {
        uint8_t *l = (uint8_t *)local; const uint8_t *in = (const uint8_t *)inbox;
        #pragma omp parallel for schedule(static) if (nn > 32768)
        for (i = 0; i < nn; ++i) l[i] = u8_apply(op, in[i], l[i]);
        return;
    }
    #pragma omp parallel for schedule(static) if (nn > 32768)
    for (i = 0; i < nn; ++i) {
        float a = wire_to_f32(inbox, (size_t)i, dtype), b = wire_to_f32(local, (size_t)i, dtype);
        f32_to_wire(local, (size_t)i, dtype, f32_apply(op, a, b));
    }
}

/* element-wise hop over a run: local[i] = hop(inbox[i], local[i]) */
static void hop_run(void *local, const void *inbox, size_t n, int dtype)
{
    ptrdiff_t i, nn = (ptrdiff_t)n;
    if (dtype >= ORC_FP64) { hop_run_op(local, inbox, n, dtype, ORC_SUM); return; }
    switch (dtype) {
    case ORC_FP32: {
        float *l = (float *)local; const float *in = (const float *)inbox;
        #pragma omp parallel for schedule(static) if (nn > 32768)
        for (i = 0; i < nn; ++i) l[i] = orc_hop_f32(in[i], l[i]);
    } break;
    case ORC_BF16: {
        uint16_t *l = (uint16_t *)local; const uint16_t *in = (const uint16_t *)inbox;
        #pragma omp parallel for schedule(static) if (nn > 32768)
        for (i = 0; i < nn; ++i) l[i] = orc_hop_bf16(in[i], l[i]);
    } break;
    case ORC_FP16: {
        uint16_t *l = (uint16_t *)local; const uint16_t *in = (const uint16_t *)inbox;
        #pragma omp parallel for schedule(static) if (nn > 32768)
        for (i = 0; i < nn; ++i) l[i] = orc_hop_f16(in[i], l[i]);
    } break;
    default: {
        int32_t *l = (int32_t *)local; const int32_t *in = (const int32_t *)inbox;
        #pragma omp parallel for schedule(static) if (nn > 32768)
        for (i = 0; i < nn; ++i) l[i] = orc_hop_i32(in[i], l[i]);
    } break;
    }
}

/* plain copy of a run (the All-Gather hop) */
static void copy_run(void *dst, const void *src, size_t nbytes)
{
    ptrdiff_t i, nn = (ptrdiff_t)nbytes;
    unsigned char *d = (unsigned char *)dst; const unsigned char *s = (const unsigned char *)src;
    #pragma omp parallel for schedule(static) if (nn > 262144)
    for (i = 0; i < nn; ++i) d[i] = s[i];
}

/* ------------------------------------------------------------------ */
/* ring tables                                                         */
/* ------------------------------------------------------------------ */
static int wrap(int a, int W) { a %= W; return a < 0 ? a + W : a; }

size_t orc_esize(int dtype)
{
    switch (dtype) {
    case ORC_BF16: case ORC_FP16: return 2u;
    case ORC_FP64: case ORC_INT64: return 8u;
    case ORC_UINT8: return 1u;
    default: return 4u;
    }
}

static int ring_ok(int W, const int *ring, int *pos)
{
    int k;
    for (k = 0; k < W; ++k) pos[k] = -1;
    for (k = 0; k < W; ++k) {
        int r = ring ? ring[k] : k;
        if (r < 0 || r >= W || pos[r] != -1) return 0;
        pos[r] = k;
    }
    return 1;
}
static int ring_at(const int *ring, int k) { return ring ? ring[k] : k; }

/* which block rank `rank` sends and which it receives at (phase, step) */
int orc_ring_step(int W, const int *ring, int phase, int step, int rank,
                  int *send_block, int *recv_block)
{
    int pos[64];
    if (W < 1 || W > 64 || rank < 0 || rank >= W || step < 0 || step > W - 2) return ORC_BAD_ARG;
    if (phase != ORC_PHASE_RS && phase != ORC_PHASE_AG) return ORC_BAD_ARG;
    if (!ring_ok(W, ring, pos)) return ORC_BAD_ARG;
    int p = pos[rank];
    if (phase == ORC_PHASE_RS) {
        *send_block = ring_at(ring, wrap(p - step - 1, W));
        *recv_block = ring_at(ring, wrap(p - step - 2, W));
    } else {
        *send_block = ring_at(ring, wrap(p - step, W));
        *recv_block = ring_at(ring, wrap(p - step - 1, W));
    }
    return ORC_OK;
}

/* block c of a vector cut into pieces of B elements */
static void block_range(size_t count, size_t B, int c, size_t *lo, size_t *hi)
{
    size_t a = (size_t)c * B, b = a + B;
    if (a > count) a = count;
    if (b > count) b = count;
    *lo = a; *hi = b;
}

/* ------------------------------------------------------------------ */
/* the ring, as message passing over work[r] (count elements each)     */
/* ------------------------------------------------------------------ */
static int ring_phase(void *const *work, int W, size_t count, size_t B, int dtype,
                      const int *ring, size_t chunk_elems, int phase, int op)
{
    int pos[64], r, s;
    size_t es = orc_esize(dtype);
    if (!ring_ok(W, ring, pos)) return ORC_BAD_ARG;
    if (W == 1 || count == 0 || B == 0) return ORC_OK;

    /* one inbox per rank, one block wide */
    unsigned char **inbox = (unsigned char **)calloc((size_t)W, sizeof *inbox);
    if (!inbox) return ORC_NO_MEM;
    for (r = 0; r < W; ++r) {
        inbox[r] = (unsigned char *)malloc(B * es);
        if (!inbox[r]) { for (s = 0; s < r; ++s) free(inbox[s]); free(inbox); return ORC_NO_MEM; }
    }

    for (s = 0; s <= W - 2; ++s) {
        /* every rank sends one block to its successor ... */
        for (r = 0; r < W; ++r) {
            int sb, rb; size_t lo, hi;
            orc_ring_step(W, ring, phase, s, r, &sb, &rb);
            int nxt = ring_at(ring, wrap(pos[r] + 1, W));
            block_range(count, B, sb, &lo, &hi);
            copy_run(inbox[nxt], (const unsigned char *)work[r] + lo * es, (hi - lo) * es);
        }
        /* ... then every rank consumes what arrived, chunk by chunk */
        for (r = 0; r < W; ++r) {
            int sb, rb; size_t lo, hi, c0;
            orc_ring_step(W, ring, phase, s, r, &sb, &rb);
            block_range(count, B, rb, &lo, &hi);
            size_t len = hi - lo, C = chunk_elems ? chunk_elems : len;
            for (c0 = 0; c0 < len; c0 += C) {
                size_t n = (len - c0 < C) ? len - c0 : C;
                unsigned char *mine = (unsigned char *)work[r] + (lo + c0) * es;
                const unsigned char *got = inbox[r] + c0 * es;
                if (phase == ORC_PHASE_AG)   copy_run(mine, got, n * es);
                else if (op == ORC_SUM)      hop_run(mine, got, n, dtype);
                else                         hop_run_op(mine, got, n, dtype, op);
            }
        }
    }
    for (r = 0; r < W; ++r) free(inbox[r]);
    free(inbox);
    return ORC_OK;
}

static int args_ok(int W, int dtype) { return W >= 1 && W <= 64 && dtype >= 0 && dtype <= ORC_UINT8; }
static int op_ok(int op) { return op >= ORC_SUM && op <= ORC_MIN; }

/* All-Reduce with operator `op`, in place on work[r]: on entry rank r's input,
   on exit the ring-order reduction in every work[r]. */
int orc_allreduce_op(void *const *work, int W, size_t count, int dtype, int op,
                     const int *ring, size_t chunk_elems)
{
    if (!args_ok(W, dtype) || !op_ok(op)) return ORC_BAD_ARG;
    size_t B = (count + (size_t)W - 1) / (size_t)W;
    int rc = ring_phase(work, W, count, B, dtype, ring, chunk_elems, ORC_PHASE_RS, op);
    if (rc) return rc;
    return ring_phase(work, W, count, B, dtype, ring, chunk_elems, ORC_PHASE_AG, op);
}
/* All-Reduce (sum) */
int orc_allreduce(void *const *work, int W, size_t count, int dtype,
                  const int *ring, size_t chunk_elems)
{
    return orc_allreduce_op(work, W, count, dtype, ORC_SUM, ring, chunk_elems);
}

/* Reduce-Scatter (sum): work[r] holds W*recvcount elements (rank r's full
   input; used as scratch, contents undefined on exit); out[r] receives
   recvcount elements = block r of the ring-order sum. */
int orc_reduce_scatter_op(void *const *work, void *const *out, int W, size_t recvcount,
                          int dtype, int op, const int *ring, size_t chunk_elems)
{
    if (!args_ok(W, dtype) || !op_ok(op)) return ORC_BAD_ARG;
    int rc = ring_phase(work, W, (size_t)W * recvcount, recvcount, dtype, ring,
                        chunk_elems, ORC_PHASE_RS, op);
    if (rc) return rc;
    size_t es = orc_esize(dtype);
    for (int r = 0; r < W; ++r)
        memcpy(out[r], (const unsigned char *)work[r] + (size_t)r * recvcount * es, recvcount * es);
    return ORC_OK;
}
int orc_reduce_scatter(void *const *work, void *const *out, int W, size_t recvcount,
                       int dtype, const int *ring, size_t chunk_elems)
{
    return orc_reduce_scatter_op(work, out, W, recvcount, dtype, ORC_SUM, ring, chunk_elems);
}

/* All-Gather: in[r] holds sendcount elements; out[r] (W*sendcount elements)
   ends with block q equal to in[q] for every q. */
int orc_all_gather(const void *const *in, void *const *out, int W, size_t sendcount,
                   int dtype, const int *ring, size_t chunk_elems)
{
    if (!args_ok(W, dtype)) return ORC_BAD_ARG;
    size_t es = orc_esize(dtype);
    for (int r = 0; r < W; ++r)   /* each rank starts with its own block in place */
        memcpy((unsigned char *)out[r] + (size_t)r * sendcount * es, in[r], sendcount * es);
    return ring_phase(out, W, (size_t)W * sendcount, sendcount, dtype, ring,
                      chunk_elems, ORC_PHASE_AG, ORC_SUM);
}

/* ------------------------------------------------------------------ */
/* the other collectives the paper evaluates (Appendix E.1 "Other       */
/* Collective Communication Operations"): Reduce, Broadcast, All-to-All */
/* ------------------------------------------------------------------ */

/* Reduce (sum) to `root` along the ring, as a chain of messages: the rank
   after the root sends its vector to its successor, every following rank adds
   its own vector to what arrived (incoming operand on the left, one hop per
   rank, rounded to the wire type) and passes the partial on; the chain ends at
   the root.  in[r]: count elements, untouched.  out: count elements, the
   root's result.  The fold order equals that of block `root` of the ring
   All-Reduce, applied to the whole vector. */
int orc_reduce_op(const void *const *in, void *out, int W, size_t count, int dtype, int op,
                  const int *ring, int root, size_t chunk_elems)
{
    int pos[64];
    if (!args_ok(W, dtype) || !op_ok(op) || root < 0 || root >= W) return ORC_BAD_ARG;
    if (!ring_ok(W, ring, pos)) return ORC_BAD_ARG;
    size_t es = orc_esize(dtype), C = chunk_elems ? chunk_elems : count, c0;
    unsigned char *msg = (unsigned char *)malloc(count * es + 1);
    unsigned char *mine = (unsigned char *)malloc(count * es + 1);
    if (!msg || !mine) { free(msg); free(mine); return ORC_NO_MEM; }
    /* first sender: the rank after the root */
    memcpy(msg, in[ring_at(ring, wrap(pos[root] + 1, W))], count * es);
    for (int k = 2; k <= W; ++k) {
        int r = ring_at(ring, wrap(pos[root] + k, W));      /* receives msg, adds its own */
        memcpy(mine, in[r], count * es);
        for (c0 = 0; c0 < count; c0 += C) {
            size_t n = (count - c0 < C) ? count - c0 : C;
            if (op == ORC_SUM) hop_run(mine + c0 * es, msg + c0 * es, n, dtype);
            else               hop_run_op(mine + c0 * es, msg + c0 * es, n, dtype, op);
        }
        memcpy(msg, mine, count * es);                      /* the partial travels on */
    }
    memcpy(out, msg, count * es);                           /* W == 1: the root's own vector */
    free(msg); free(mine);
    return ORC_OK;
}
int orc_reduce(const void *const *in, void *out, int W, size_t count, int dtype,
               const int *ring, int root, size_t chunk_elems)
{
    return orc_reduce_op(in, out, W, count, dtype, ORC_SUM, ring, root, chunk_elems);
}

/* Broadcast from `root` along the ring: out[r] (count elements) becomes a copy
   of `in` for every rank, each rank copying what its predecessor holds. */
int orc_broadcast(const void *in, void *const *out, int W, size_t count, int dtype,
                  const int *ring, int root)
{
    int pos[64];
    if (!args_ok(W, dtype) || root < 0 || root >= W) return ORC_BAD_ARG;
    if (!ring_ok(W, ring, pos)) return ORC_BAD_ARG;
    size_t es = orc_esize(dtype);
    memcpy(out[root], in, count * es);
    for (int k = 1; k < W; ++k) {
        int r = ring_at(ring, wrap(pos[root] + k, W));
        int p = ring_at(ring, wrap(pos[root] + k - 1, W));
        memcpy(out[r], out[p], count * es);
    }
    return ORC_OK;
}

/* All-to-All: in[r] and out[r] hold W blocks of n elements; block q of out[r]
   is block r of in[q].  (The plain definition; no ring is involved.) */
int orc_alltoall(const void *const *in, void *const *out, int W, size_t n, int dtype)
{
    if (!args_ok(W, dtype)) return ORC_BAD_ARG;
    size_t es = orc_esize(dtype);
    for (int r = 0; r < W; ++r)
        for (int q = 0; q < W; ++q)
            memcpy((unsigned char *)out[r] + (size_t)q * n * es,
                   (const unsigned char *)in[q] + (size_t)r * n * es, n * es);
    return ORC_OK;
}

/* ------------------------------------------------------------------ */
/* reordered-class variant: binary32 accumulation, one final rounding   */
/* ------------------------------------------------------------------ */
/* The paper accepts collectives that differ in reduction order within
   floating-point tolerance (Appendix E.2 "LLM Training Convergence").  This
   variant keeps the ring's order of operands for block c (next(c), ..., c)
   but carries the running sum in binary32 and rounds to the wire type once,
   at the end.  For fp32 and int32 it equals the ring result.  It is a
   different result from the per-hop ring for bf16 / fp16, within 2 ulp of the
   correctly rounded exact sum in the cases the tests bound. */
static void sum_fp32acc_run(const void *const *in, const int *order, int W, size_t off, size_t n,
                            int dtype, void *out)
{
    ptrdiff_t i, nn = (ptrdiff_t)n;
    if (dtype == ORC_FP32) {
        float *o = (float *)out;
        #pragma omp parallel for schedule(static) if (nn > 32768)
        for (i = 0; i < nn; ++i) {
            float acc = ((const float *)in[order[0]])[off + i];
            for (int k = 1; k < W; ++k) acc = acc + ((const float *)in[order[k]])[off + i];
            o[i] = acc;
        }
    } else if (dtype == ORC_INT32) {
        int32_t *o = (int32_t *)out;
        #pragma omp parallel for schedule(static) if (nn > 32768)
        for (i = 0; i < nn; ++i) {
            uint32_t acc = (uint32_t)((const int32_t *)in[order[0]])[off + i];
            for (int k = 1; k < W; ++k) acc += (uint32_t)((const int32_t *)in[order[k]])[off + i];
            o[i] = (int32_t)acc;
        }
    } else {
        uint16_t *o = (uint16_t *)out;
        #pragma omp parallel for schedule(static) if (nn > 32768)
        for (i = 0; i < nn; ++i) {
            uint16_t x = ((const uint16_t *)in[order[0]])[off + i];
            float acc = dtype == ORC_BF16 ? orc_bf16_to_f32(x) : orc_f16_to_f32(x);
            for (int k = 1; k < W; ++k) {
                x = ((const uint16_t *)in[order[k]])[off + i];
                acc = acc + (dtype == ORC_BF16 ? orc_bf16_to_f32(x) : orc_f16_to_f32(x));
            }
            o[i] = dtype == ORC_BF16 ? orc_f32_to_bf16(acc) : orc_f32_to_f16(acc);
        }
    }
}

/* All-Reduce with binary32 accumulation: in[r] count elements (untouched),
   out[r] count elements, identical for every rank. */
int orc_allreduce_fp32acc(const void *const *in, void *const *out, int W, size_t count, int dtype,
                          const int *ring)
{
    int pos[64], order[64];
    if (!args_ok(W, dtype) || dtype > ORC_INT32 || !ring_ok(W, ring, pos)) return ORC_BAD_ARG;
    size_t es = orc_esize(dtype), B = (count + (size_t)W - 1) / (size_t)W;
    for (int c = 0; c < W; ++c) {
        size_t lo, hi;
        block_range(count, B, c, &lo, &hi);
        for (int k = 0; k < W; ++k) order[k] = ring_at(ring, wrap(pos[c] + 1 + k, W));
        sum_fp32acc_run(in, order, W, lo, hi - lo, dtype, (unsigned char *)out[0] + lo * es);
    }
    for (int r = 1; r < W; ++r) memcpy(out[r], out[0], count * es);
    return ORC_OK;
}

/* Reduce-Scatter with binary32 accumulation: in[r] W*n elements, out[r] n elements (block r). */
int orc_reduce_scatter_fp32acc(const void *const *in, void *const *out, int W, size_t n, int dtype,
                               const int *ring)
{
    int pos[64], order[64];
    if (!args_ok(W, dtype) || dtype > ORC_INT32 || !ring_ok(W, ring, pos)) return ORC_BAD_ARG;
    for (int c = 0; c < W; ++c) {
        for (int k = 0; k < W; ++k) order[k] = ring_at(ring, wrap(pos[c] + 1 + k, W));
        sum_fp32acc_run(in, order, W, (size_t)c * n, n, dtype, out[c]);
    }
    return ORC_OK;
}

/* Reduce to root with binary32 accumulation: in[r] count elements, out count elements. */
int orc_reduce_fp32acc(const void *const *in, void *out, int W, size_t count, int dtype,
                       const int *ring, int root)
{
    int pos[64], order[64];
    if (!args_ok(W, dtype) || dtype > ORC_INT32 || root < 0 || root >= W || !ring_ok(W, ring, pos)) return ORC_BAD_ARG;
    for (int k = 0; k < W; ++k) order[k] = ring_at(ring, wrap(pos[root] + 1 + k, W));
    sum_fp32acc_run(in, order, W, 0, count, dtype, out);
    return ORC_OK;
}

/* ------------------------------------------------------------------ */
/* reordered-class variants in general: operator, order, rounding       */
/* ------------------------------------------------------------------ */
/* Combines the W values v[0..W-1] (already in the order they enter) into one.
   order RING: ((v0 op v1) op v2) ... op v[W-1].
   order TREE: level by level, neighbours first; an odd last value moves up.
   rounding EACH: every intermediate result travels in the wire type;
   rounding ONCE: intermediates stay in binary32.  The caller rounds the
   returned value to the wire type (a no-op after EACH). */
static float combine_f32(float *v, int W, int dtype, int op, int order, int rounding)
{
    if (order == ORC_ORDER_RING) {
        float acc = v[0];
        for (int k = 1; k < W; ++k) {
            acc = f32_apply(op, acc, v[k]);
            if (rounding == ORC_ROUND_EACH) acc = through_wire(acc, dtype);
        }
        return acc;
    }
    int n = W;
    while (n > 1) {
        int m = 0;
        for (int k = 0; k + 1 < n; k += 2) {
            float t = f32_apply(op, v[k], v[k + 1]);
            if (rounding == ORC_ROUND_EACH) t = through_wire(t, dtype);
            v[m++] = t;
        }
        if (n & 1) v[m++] = v[n - 1];
        n = m;
    }
    return v[0];
}
static int32_t combine_i32(int32_t *v, int W, int op, int order)
{
    if (order == ORC_ORDER_RING) {
        int32_t acc = v[0];
        for (int k = 1; k < W; ++k) acc = i32_apply(op, acc, v[k]);
        return acc;
    }
    int n = W;
    while (n > 1) {
        int m = 0;
        for (int k = 0; k + 1 < n; k += 2) v[m++] = i32_apply(op, v[k], v[k + 1]);
        if (n & 1) v[m++] = v[n - 1];
        n = m;
    }
    return v[0];
}
/* the same shapes for the wire types that are their own accumulation type: no rounding step */
#define ORC_COMBINE(NAME, T, APPLY)                                              \
static T NAME(T *v, int W, int op, int order)                                    \
{                                                                                \
    if (order == ORC_ORDER_RING) {                                               \
        T acc = v[0];                                                            \
        for (int k = 1; k < W; ++k) acc = APPLY(op, acc, v[k]);                  \
        return acc;                                                              \
    }                                                                            \
    int n = W;                                                                   \
    while (n > 1) {                                                              \
        int m = 0;                                                               \
        for (int k = 0; k + 1 < n; k += 2) v[m++] = APPLY(op, v[k], v[k + 1]);   \
        if (n & 1) v[m++] = v[n - 1];                                            \
        n = m;                                                                   \
    }                                                                            \
    return v[0];                                                                 \
}
ORC_COMBINE(combine_f64, double, f64_apply)
ORC_COMBINE(combine_i64, int64_t, i64_apply)
ORC_COMBINE(combine_u8, uint8_t, u8_apply)
#undef ORC_COMBINE

/* out[i] = combination of in[who[k]][off + i], k = 0..W-1, for i in [0, n) */
static void combine_run(const void *const *in, const int *who, int W, size_t off, size_t n, int dtype,
                        int op, int order, int rounding, void *out)
{
    ptrdiff_t i, nn = (ptrdiff_t)n;
    #pragma omp parallel for schedule(static) if (nn > 32768)
    for (i = 0; i < nn; ++i) {
        if (dtype == ORC_INT32) {
            int32_t v[64];
            for (int k = 0; k < W; ++k) v[k] = ((const int32_t *)in[who[k]])[off + (size_t)i];
            ((int32_t *)out)[i] = combine_i32(v, W, op, order);
        } else if (dtype == ORC_FP64) {
            double v[64];
            for (int k = 0; k < W; ++k) v[k] = ((const double *)in[who[k]])[off + (size_t)i];
            ((double *)out)[i] = combine_f64(v, W, op, order);
        } else if (dtype == ORC_INT64) {
            int64_t v[64];
            for (int k = 0; k < W; ++k) v[k] = ((const int64_t *)in[who[k]])[off + (size_t)i];
            ((int64_t *)out)[i] = combine_i64(v, W, op, order);
        } else if (dtype == ORC_UINT8) {
            uint8_t v[64];
            for (int k = 0; k < W; ++k) v[k] = ((const uint8_t *)in[who[k]])[off + (size_t)i];
            ((uint8_t *)out)[i] = combine_u8(v, W, op, order);
        } else {
            float v[64];
            for (int k = 0; k < W; ++k) v[k] = wire_to_f32(in[who[k]], off + (size_t)i, dtype);
            f32_to_wire(out, (size_t)i, dtype, combine_f32(v, W, dtype, op, order, rounding));
        }
    }
}
/* the order in which the ranks' values enter block c (or the root's vector) */
static void entry_order(int W, const int *ring, const int *pos, int c, int order, int *who)
{
    for (int k = 0; k < W; ++k)
        who[k] = order == ORC_ORDER_RING ? ring_at(ring, wrap(pos[c] + 1 + k, W)) : ring_at(ring, k);
}
static int var_ok(int op, int order, int rounding)
{
    return op_ok(op) && (order == ORC_ORDER_RING || order == ORC_ORDER_TREE)
        && (rounding == ORC_ROUND_EACH || rounding == ORC_ROUND_ONCE);
}

/* All-Reduce variant: in[r] count elements (untouched), out[r] count elements,
   identical for every rank.  (RING, EACH) is the ring's own result. */
int orc_allreduce_var(const void *const *in, void *const *out, int W, size_t count, int dtype,
                      int op, const int *ring, int order, int rounding)
{
    int pos[64], who[64];
    if (!args_ok(W, dtype) || !var_ok(op, order, rounding) || !ring_ok(W, ring, pos)) return ORC_BAD_ARG;
    size_t es = orc_esize(dtype), B = (count + (size_t)W - 1) / (size_t)W;
    for (int c = 0; c < W; ++c) {
        size_t lo, hi;
        block_range(count, B, c, &lo, &hi);
        entry_order(W, ring, pos, c, order, who);
        combine_run(in, who, W, lo, hi - lo, dtype, op, order, rounding, (unsigned char *)out[0] + lo * es);
    }
    for (int r = 1; r < W; ++r) memcpy(out[r], out[0], count * es);
    return ORC_OK;
}
/* Reduce-Scatter variant: in[r] W*n elements, out[r] n elements (block r). */
int orc_reduce_scatter_var(const void *const *in, void *const *out, int W, size_t n, int dtype,
                           int op, const int *ring, int order, int rounding)
{
    int pos[64], who[64];
    if (!args_ok(W, dtype) || !var_ok(op, order, rounding) || !ring_ok(W, ring, pos)) return ORC_BAD_ARG;
    for (int c = 0; c < W; ++c) {
        entry_order(W, ring, pos, c, order, who);
        combine_run(in, who, W, (size_t)c * n, n, dtype, op, order, rounding, out[c]);
    }
    return ORC_OK;
}
/* Reduce-to-root variant: in[r] count elements, out count elements. */
int orc_reduce_var(const void *const *in, void *out, int W, size_t count, int dtype,
                   int op, const int *ring, int root, int order, int rounding)
{
    int pos[64], who[64];
    if (!args_ok(W, dtype) || !var_ok(op, order, rounding) || root < 0 || root >= W
        || !ring_ok(W, ring, pos)) return ORC_BAD_ARG;
    entry_order(W, ring, pos, root, order, who);
    combine_run(in, who, W, 0, count, dtype, op, order, rounding, out);
    return ORC_OK;
}

/* bulk conversions, for the conversion pins */
void orc_f32_to_bf16_n(const float *x, uint16_t *y, size_t n) { for (size_t i = 0; i < n; ++i) y[i] = orc_f32_to_bf16(x[i]); }
void orc_f32_to_f16_n (const float *x, uint16_t *y, size_t n) { for (size_t i = 0; i < n; ++i) y[i] = orc_f32_to_f16(x[i]); }
void orc_bf16_to_f32_n(const uint16_t *x, float *y, size_t n) { for (size_t i = 0; i < n; ++i) y[i] = orc_bf16_to_f32(x[i]); }
void orc_f16_to_f32_n (const uint16_t *x, float *y, size_t n) { for (size_t i = 0; i < n; ++i) y[i] = orc_f16_to_f32(x[i]); }
/* y[i] = hop(a[i], b[i]) for the hop pins */
void orc_hop_n(const void *a, const void *b, void *y, size_t n, int dtype)
{
    memcpy(y, b, n * orc_esize(dtype));
    hop_run(y, a, n, dtype);
}

/* y[i] = hop with operator `op` of (a[i], b[i]) */
void orc_hop_op_n(const void *a, const void *b, void *y, size_t n, int dtype, int op)
{
    memcpy(y, b, n * orc_esize(dtype));
    hop_run_op(y, a, n, dtype, op);
}

/* thread control for the timing harness: 0 = leave the OpenMP default */
int orc_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
    return omp_get_max_threads();
#else
    (void)n; return 1;
#endif
}

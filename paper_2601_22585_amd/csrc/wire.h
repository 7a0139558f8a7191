// Device-side helpers shared by the gfx950 reduce-copy kernels: 128-bit memory
// access, the wire types' hop arithmetic, and the tile decomposition.
//
// Arithmetic of one hop (reductions run on the GPU, Appendix E.3):
//   partial = round_T(op(f32(incoming), f32(local))), round to nearest even
// (fp64: one binary64 operation; integers wrap modulo 2^bits),
// op = sum by default; product, maximum and minimum are the other operators of
// the call shape (Section 4.4).  Maximum / minimum follow IEEE 754-2019 clause
// 9.6: a NaN operand gives NaN, -0 orders below +0.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "reduce_copy.h"

namespace hcl {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

enum { DT_FP32 = 0, DT_BF16 = 1, DT_FP16 = 2, DT_INT32 = 3, DT_FP64 = 4, DT_INT64 = 5, DT_UINT8 = 6 };

// ---------------------------------------------------------------------------
// memory access helpers
// ---------------------------------------------------------------------------
// 128-bit accesses that promise no alignment beyond one byte: the instruction is the same
// global_load_dwordx4 / global_store_dwordx4, and the hardware serves any address
typedef u32x4 u32x4_any __attribute__((aligned(1)));
template <bool NT>
__device__ __forceinline__ u32x4 ld16(const char* p) {
  const u32x4_any* q = reinterpret_cast<const u32x4_any*>(p);
  if (NT) return __builtin_nontemporal_load(q);
  return *q;
}
// Store kinds.  ST_PLAIN: an ordinary store; the line stays dirty in the XCD's L2 until it is
// evicted or the end-of-kernel write-back flushes it.  ST_STREAM: non-temporal, for output that
// nothing reads soon.  ST_THROUGH: written through the L2 at once (the sc1 bit, the form the
// compiler itself emits for an agent-scope atomic store; it has no 128-bit builtin, hence the
// instruction is spelled out): nothing is left for the write-back at the end of the kernel, and the
// line sits in the memory-side last-level cache when the next launch reads it.  Measured on MI355X
// for the partial sums one ring step hands to the next: +4 to +5 % of HBM peak over ST_PLAIN at
// every size from 32 MiB to 1 GiB per rank, +8 over ST_STREAM.
enum { ST_PLAIN = 0, ST_THROUGH = 1, ST_STREAM = 2 };
template <int KIND>
__device__ __forceinline__ void st16(char* p, u32x4 v) {
  u32x4_any* q = reinterpret_cast<u32x4_any*>(p);
  if (KIND == ST_STREAM) {
    __builtin_nontemporal_store(v, q);
  } else if (KIND == ST_THROUGH) {
    // p is device (or pinned host) memory, so its flat address is its global address.  The
    // compiler does not see inside the statement, so the statement itself keeps the wait states
    // this ISA requires between a store of more than 64 bits and a vector-ALU write to the
    // registers that hold its data: two (with one, a next instruction that reused a data register
    // corrupted the stored value now and then); four are kept, the cost does not show.
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 3" : : "v"(q), "v"(v) : "memory");
  } else {
    *q = v;
  }
}

// ---------------------------------------------------------------------------
// wire types: one hop on a 32-bit word (one 4-byte or two 2-byte elements)
// and on a single element
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint32_t f2u(float f) { return __float_as_uint(f); }
__device__ __forceinline__ float u2f(uint32_t u) { return __uint_as_float(u); }

// binary32 pair -> packed bfloat16 pair with the gfx950 conversion instruction
// (v_cvt_pk_bf16_f32): round to nearest even, subnormal results kept, NaN stays
// NaN.  lo lands in bits 0..15, hi in bits 16..31.
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t bf16_pack_rne(float lo, float hi) {
  f32x2 s;
  s.x = lo;
  s.y = hi;
  const bf16x2 r = __builtin_convertvector(s, bf16x2);
  uint32_t u;
  __builtin_memcpy(&u, &r, 4);
  return u;
}

template <int DT> struct Wire;

// kWide: the type has a binary32-accumulation variant that differs from the
// per-hop one (two-byte floats); widen2 / narrow2 split a word into its two
// elements as binary32 and pack two binary32 values back with one rounding.
template <> struct Wire<DT_FP32> {
  typedef uint32_t elem_t;
  static constexpr bool kWide = false;
  __device__ static __forceinline__ uint32_t hop_word(uint32_t in, uint32_t loc) { return f2u(u2f(in) + u2f(loc)); }
  __device__ static __forceinline__ elem_t hop_elem(elem_t in, elem_t loc) { return hop_word(in, loc); }
  __device__ static __forceinline__ void widen2(uint32_t, float&, float&) {}
  __device__ static __forceinline__ uint32_t narrow2(float, float) { return 0; }
};
template <> struct Wire<DT_INT32> {
  typedef uint32_t elem_t;
  static constexpr bool kWide = false;
  __device__ static __forceinline__ uint32_t hop_word(uint32_t in, uint32_t loc) { return in + loc; }
  __device__ static __forceinline__ elem_t hop_elem(elem_t in, elem_t loc) { return in + loc; }
  __device__ static __forceinline__ void widen2(uint32_t, float&, float&) {}
  __device__ static __forceinline__ uint32_t narrow2(float, float) { return 0; }
};
template <> struct Wire<DT_BF16> {
  typedef uint16_t elem_t;
  static constexpr bool kWide = true;
  __device__ static __forceinline__ void widen2(uint32_t w, float& lo, float& hi) {
    lo = u2f(w << 16);
    hi = u2f(w & 0xFFFF0000u);
  }
  __device__ static __forceinline__ uint32_t narrow2(float lo, float hi) { return bf16_pack_rne(lo, hi); }
  __device__ static __forceinline__ uint32_t hop_word(uint32_t in, uint32_t loc) {
    const float lo = u2f(in << 16) + u2f(loc << 16);
    const float hi = u2f(in & 0xFFFF0000u) + u2f(loc & 0xFFFF0000u);
    return bf16_pack_rne(lo, hi);
  }
  __device__ static __forceinline__ elem_t hop_elem(elem_t in, elem_t loc) {
    const float s = u2f((uint32_t)in << 16) + u2f((uint32_t)loc << 16);
    return (elem_t)(bf16_pack_rne(s, 0.0f) & 0xFFFFu);
  }
};
template <> struct Wire<DT_FP16> {
  typedef uint16_t elem_t;
  static constexpr bool kWide = true;
  __device__ static __forceinline__ void widen2(uint32_t w, float& lo, float& hi) {
    lo = widen((uint16_t)(w & 0xFFFFu));
    hi = widen((uint16_t)(w >> 16));
  }
  __device__ static __forceinline__ uint32_t narrow2(float lo, float hi) {
    return (uint32_t)narrow(lo) | ((uint32_t)narrow(hi) << 16);
  }
  __device__ static __forceinline__ float widen(uint16_t h) {
    _Float16 x;
    __builtin_memcpy(&x, &h, 2);
    return (float)x;
  }
  // binary32 -> binary16 conversion instruction: round to nearest even in the
  // default rounding mode, subnormal results kept
  __device__ static __forceinline__ uint16_t narrow(float f) {
    const _Float16 x = (_Float16)f;
    uint16_t h;
    __builtin_memcpy(&h, &x, 2);
    return h;
  }
  __device__ static __forceinline__ elem_t hop_elem(elem_t in, elem_t loc) { return narrow(widen(in) + widen(loc)); }
  __device__ static __forceinline__ uint32_t hop_word(uint32_t in, uint32_t loc) {
    const uint32_t lo = hop_elem((uint16_t)(in & 0xFFFFu), (uint16_t)(loc & 0xFFFFu));
    const uint32_t hi = hop_elem((uint16_t)(in >> 16), (uint16_t)(loc >> 16));
    return lo | (hi << 16);
  }
};

// eight-byte types: a 128-bit vector holds two elements; hop_word is never used
__device__ __forceinline__ uint64_t d2u(double d) { return (uint64_t)__double_as_longlong(d); }
__device__ __forceinline__ double u2d(uint64_t u) { return __longlong_as_double((long long)u); }
template <> struct Wire<DT_FP64> {
  typedef uint64_t elem_t;
  static constexpr bool kWide = false;
  __device__ static __forceinline__ elem_t hop_elem(elem_t in, elem_t loc) { return d2u(u2d(in) + u2d(loc)); }
  __device__ static __forceinline__ uint32_t hop_word(uint32_t, uint32_t) { return 0; }
  __device__ static __forceinline__ void widen2(uint32_t, float&, float&) {}
  __device__ static __forceinline__ uint32_t narrow2(float, float) { return 0; }
};
template <> struct Wire<DT_INT64> {
  typedef uint64_t elem_t;
  static constexpr bool kWide = false;
  __device__ static __forceinline__ elem_t hop_elem(elem_t in, elem_t loc) { return in + loc; }
  __device__ static __forceinline__ uint32_t hop_word(uint32_t, uint32_t) { return 0; }
  __device__ static __forceinline__ void widen2(uint32_t, float&, float&) {}
  __device__ static __forceinline__ uint32_t narrow2(float, float) { return 0; }
};
// one-byte type: four elements per word, added without carries between bytes
template <> struct Wire<DT_UINT8> {
  typedef uint8_t elem_t;
  static constexpr bool kWide = false;
  __device__ static __forceinline__ elem_t hop_elem(elem_t in, elem_t loc) { return (elem_t)(in + loc); }
  __device__ static __forceinline__ uint32_t hop_word(uint32_t in, uint32_t loc) {
    return ((in & 0x7F7F7F7Fu) + (loc & 0x7F7F7F7Fu)) ^ ((in ^ loc) & 0x80808080u);
  }
  __device__ static __forceinline__ void widen2(uint32_t, float&, float&) {}
  __device__ static __forceinline__ uint32_t narrow2(float, float) { return 0; }
};

template <int DT>
__device__ __forceinline__ u32x4 hop_vec(u32x4 in, u32x4 loc) {
  u32x4 r;
  if (sizeof(typename Wire<DT>::elem_t) == 8) {
    const uint64_t lo = Wire<DT>::hop_elem((uint64_t)in.x | ((uint64_t)in.y << 32), (uint64_t)loc.x | ((uint64_t)loc.y << 32));
    const uint64_t hi = Wire<DT>::hop_elem((uint64_t)in.z | ((uint64_t)in.w << 32), (uint64_t)loc.z | ((uint64_t)loc.w << 32));
    r.x = (uint32_t)lo;
    r.y = (uint32_t)(lo >> 32);
    r.z = (uint32_t)hi;
    r.w = (uint32_t)(hi >> 32);
    return r;
  }
  r.x = Wire<DT>::hop_word(in.x, loc.x);
  r.y = Wire<DT>::hop_word(in.y, loc.y);
  r.z = Wire<DT>::hop_word(in.z, loc.z);
  r.w = Wire<DT>::hop_word(in.w, loc.w);
  return r;
}

// Sum of W vectors in order with binary32 accumulation and one final rounding
// (two-byte float types only).
template <int DT, int W>
__device__ __forceinline__ u32x4 sum_wide(const u32x4 (&v)[W]) {
  float acc[8];
  Wire<DT>::widen2(v[0].x, acc[0], acc[1]);
  Wire<DT>::widen2(v[0].y, acc[2], acc[3]);
  Wire<DT>::widen2(v[0].z, acc[4], acc[5]);
  Wire<DT>::widen2(v[0].w, acc[6], acc[7]);
#pragma unroll
  for (int k = 1; k < W; ++k) {
    float t[8];
    Wire<DT>::widen2(v[k].x, t[0], t[1]);
    Wire<DT>::widen2(v[k].y, t[2], t[3]);
    Wire<DT>::widen2(v[k].z, t[4], t[5]);
    Wire<DT>::widen2(v[k].w, t[6], t[7]);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = acc[j] + t[j];
  }
  u32x4 r;
  r.x = Wire<DT>::narrow2(acc[0], acc[1]);
  r.y = Wire<DT>::narrow2(acc[2], acc[3]);
  r.z = Wire<DT>::narrow2(acc[4], acc[5]);
  r.w = Wire<DT>::narrow2(acc[6], acc[7]);
  return r;
}
// the same for one element: element e of a word-pair is widened through widen2
template <int DT>
__device__ __forceinline__ float widen1(typename Wire<DT>::elem_t x) {
  float lo, hi;
  Wire<DT>::widen2((uint32_t)x, lo, hi);
  return lo;
}
template <int DT>
__device__ __forceinline__ typename Wire<DT>::elem_t narrow1(float f) {
  return (typename Wire<DT>::elem_t)(Wire<DT>::narrow2(f, 0.0f) & 0xFFFFu);
}

// ---------------------------------------------------------------------------
// operators other than the sum (op: 1 product, 2 maximum, 3 minimum; 0 sum)
// ---------------------------------------------------------------------------
enum { OP_SUM = 0, OP_PROD = 1, OP_MAX = 2, OP_MIN = 3 };

__device__ __forceinline__ float maximum_f32(float a, float b) {
  float m = a > b ? a : b;
  if (a == b) m = (f2u(a) >> 31) ? b : a;  // equal values differ at most in the sign of zero
  if (a != a || b != b) m = u2f(0x7FC00000u);
  return m;
}
__device__ __forceinline__ float minimum_f32(float a, float b) {
  float m = a < b ? a : b;
  if (a == b) m = (f2u(a) >> 31) ? a : b;
  if (a != a || b != b) m = u2f(0x7FC00000u);
  return m;
}
__device__ __forceinline__ float apply_f32(uint32_t op, float a, float b) {
  switch (op) {
    case OP_PROD: return a * b;
    case OP_MAX: return maximum_f32(a, b);
    case OP_MIN: return minimum_f32(a, b);
    default: return a + b;
  }
}
__device__ __forceinline__ uint32_t apply_i32(uint32_t op, uint32_t a, uint32_t b) {
  switch (op) {
    case OP_PROD: return a * b;
    case OP_MAX: return (int32_t)a > (int32_t)b ? a : b;
    case OP_MIN: return (int32_t)a < (int32_t)b ? a : b;
    default: return a + b;
  }
}

__device__ __forceinline__ double apply_f64(uint32_t op, double a, double b) {
  switch (op) {
    case OP_PROD: return a * b;
    case OP_MAX: {
      double m = a > b ? a : b;
      if (a == b) m = (d2u(a) >> 63) ? b : a;
      if (a != a || b != b) m = u2d(0x7FF8000000000000ull);
      return m;
    }
    case OP_MIN: {
      double m = a < b ? a : b;
      if (a == b) m = (d2u(a) >> 63) ? a : b;
      if (a != a || b != b) m = u2d(0x7FF8000000000000ull);
      return m;
    }
    default: return a + b;
  }
}
__device__ __forceinline__ uint64_t apply_i64(uint32_t op, uint64_t a, uint64_t b) {
  switch (op) {
    case OP_PROD: return a * b;
    case OP_MAX: return (int64_t)a > (int64_t)b ? a : b;
    case OP_MIN: return (int64_t)a < (int64_t)b ? a : b;
    default: return a + b;
  }
}
// four unsigned bytes at once
__device__ __forceinline__ uint32_t apply_u8x4(uint32_t op, uint32_t a, uint32_t b) {
  if (op == OP_SUM) return Wire<DT_UINT8>::hop_word(a, b);
  uint32_t r = 0;
#pragma unroll
  for (int s = 0; s < 32; s += 8) {
    const uint32_t x = (a >> s) & 0xFFu, y = (b >> s) & 0xFFu;
    const uint32_t v = op == OP_PROD ? (x * y) & 0xFFu : (op == OP_MAX ? (x > y ? x : y) : (x < y ? x : y));
    r |= v << s;
  }
  return r;
}
// one eight-byte element
template <int DT>
__device__ __forceinline__ uint64_t op_elem64(uint32_t op, uint64_t in, uint64_t loc) {
  return DT == DT_FP64 ? d2u(apply_f64(op, u2d(in), u2d(loc))) : apply_i64(op, in, loc);
}

// One hop with a run-time operator on a 32-bit word / on one element.
template <int DT>
__device__ __forceinline__ uint32_t op_word(uint32_t op, uint32_t in, uint32_t loc) {
  if (DT == DT_UINT8) return apply_u8x4(op, in, loc);
  if (DT == DT_INT32) return apply_i32(op, in, loc);
  if (DT == DT_FP32) return f2u(apply_f32(op, u2f(in), u2f(loc)));
  float a0, a1, b0, b1;
  Wire<DT>::widen2(in, a0, a1);
  Wire<DT>::widen2(loc, b0, b1);
  return Wire<DT>::narrow2(apply_f32(op, a0, b0), apply_f32(op, a1, b1));
}
template <int DT>
__device__ __forceinline__ typename Wire<DT>::elem_t op_elem(uint32_t op, typename Wire<DT>::elem_t in,
                                                             typename Wire<DT>::elem_t loc) {
  typedef typename Wire<DT>::elem_t elem_t;
  if (sizeof(elem_t) == 8) return (elem_t)op_elem64<DT>(op, (uint64_t)in, (uint64_t)loc);
  // narrower than a word: the element sits in the low bits, the rest of the word is dropped
  return (elem_t)op_word<DT>(op, (uint32_t)in, (uint32_t)loc);
}
template <int DT>
__device__ __forceinline__ u32x4 op_vec(uint32_t op, u32x4 in, u32x4 loc) {
  u32x4 r;
  if (sizeof(typename Wire<DT>::elem_t) == 8) {
    const uint64_t lo = op_elem64<DT>(op, (uint64_t)in.x | ((uint64_t)in.y << 32), (uint64_t)loc.x | ((uint64_t)loc.y << 32));
    const uint64_t hi = op_elem64<DT>(op, (uint64_t)in.z | ((uint64_t)in.w << 32), (uint64_t)loc.z | ((uint64_t)loc.w << 32));
    r.x = (uint32_t)lo;
    r.y = (uint32_t)(lo >> 32);
    r.z = (uint32_t)hi;
    r.w = (uint32_t)(hi >> 32);
    return r;
  }
  r.x = op_word<DT>(op, in.x, loc.x);
  r.y = op_word<DT>(op, in.y, loc.y);
  r.z = op_word<DT>(op, in.z, loc.z);
  r.w = op_word<DT>(op, in.w, loc.w);
  return r;
}

// ---------------------------------------------------------------------------
// tile -> (chunk, segment, position) decomposition shared by all kernels
// ---------------------------------------------------------------------------
struct TilePos {
  uint32_t d;   // segment (step kernels) or block (fused kernels)
  uint64_t j;   // chunk index
  uint64_t lo;  // first element inside the segment
};

// stagger: segment d takes the tiles of a chunk in rotated order, starting
// d * stagger tiles in, so that segments whose base addresses are congruent
// modulo a large power of two are not walked at the same offset at the same time
__device__ __forceinline__ TilePos locate(uint32_t t, uint32_t tiles_per_chunk, uint32_t nseg,
                                          uint64_t chunk, uint32_t tile, uint32_t stagger = 0) {
  TilePos p;
  uint32_t k = t % tiles_per_chunk;
  const uint32_t q = t / tiles_per_chunk;
  p.d = q % nseg;
  p.j = q / nseg;
  if (stagger) k = (k + p.d * stagger) % tiles_per_chunk;
  p.lo = p.j * chunk + (uint64_t)k * tile;
  return p;
}
// Head of a run of n elements of ES bytes that starts at `p`: the elements before the first
// 128-byte boundary.  The tile that starts the run does them one by one and the tile grid covers
// the rest, so that every 128-bit access of a wavefront is aligned and its 1 KiB covers whole cache
// lines wherever the block map or the caller puts the run -- for every stream that is congruent
// to `p` modulo 128 bytes, which equal block offsets in equally aligned buffers are.  (Blocks of
// ceil(count / W) elements start at odd offsets for most counts; walking them unaligned cost
// 14 % of bandwidth on MI355X.)
template <uint32_t ES>
__device__ __forceinline__ uint32_t head_elems(const void* p, uint64_t n) {
  const uint32_t h = (uint32_t)((0u - (uint32_t)(uintptr_t)p) & 127u) / ES;
  return n < h ? (uint32_t)n : h;
}

// Elements of this tile: up to the end of its chunk, clipped to the n elements
// of the segment; 0 = nothing to do.
__device__ __forceinline__ uint32_t tile_len(const TilePos& p, uint64_t n, uint64_t chunk, uint32_t tile) {
  uint64_t cend = (p.j + 1) * chunk;
  if (cend > n) cend = n;
  if (p.lo >= cend) return 0;
  const uint64_t left = cend - p.lo;
  return left < tile ? (uint32_t)left : tile;
}

}  // namespace hcl

// gfx950 reduce-copy kernels for the ring collectives.
//
// The work is streaming and element-wise (at most one fp32 add per 6-12 bytes
// moved), so the design targets HBM bandwidth, not the matrix cores: every
// lane moves 128-bit vectors, a wavefront's 64 lanes cover 1 KiB of contiguous
// memory per access, each thread issues all loads of a tile (UNROLL vectors
// per source) before the first use, and streamed outputs use non-temporal
// stores.  A launch is a persistent grid striding over tiles.
//
// Arithmetic of one hop (reductions run on the GPU, Appendix E.3):
//   partial = round_T(f32(incoming) + f32(local)), round to nearest even.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "reduce_copy.h"

namespace hcl {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

enum { DT_FP32 = 0, DT_BF16 = 1, DT_FP16 = 2, DT_INT32 = 3 };

// ---------------------------------------------------------------------------
// memory access helpers
// ---------------------------------------------------------------------------
template <bool NT>
__device__ __forceinline__ u32x4 ld16(const char* p) {
  const u32x4* q = reinterpret_cast<const u32x4*>(p);
  if (NT) return __builtin_nontemporal_load(q);
  return *q;
}
template <bool NT>
__device__ __forceinline__ void st16(char* p, u32x4 v) {
  u32x4* q = reinterpret_cast<u32x4*>(p);
  if (NT) __builtin_nontemporal_store(v, q);
  else *q = v;
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

template <int DT>
__device__ __forceinline__ u32x4 hop_vec(u32x4 in, u32x4 loc) {
  u32x4 r;
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
// Elements of this tile: up to the end of its chunk, clipped to the n elements
// of the segment; 0 = nothing to do.
__device__ __forceinline__ uint32_t tile_len(const TilePos& p, uint64_t n, uint64_t chunk, uint32_t tile) {
  uint64_t cend = (p.j + 1) * chunk;
  if (cend > n) cend = n;
  if (p.lo >= cend) return 0;
  const uint64_t left = cend - p.lo;
  return left < tile ? (uint32_t)left : tile;
}

// ---------------------------------------------------------------------------
// STEPWISE: one ring step of every rank.  128-bit path.
// ---------------------------------------------------------------------------
template <int DT, int NSRC, int NDST, int UNROLL, bool NT>
__global__ void __launch_bounds__(1024) reduce_copy_vec(const StepArgs a) {
  typedef typename Wire<DT>::elem_t elem_t;
  constexpr uint32_t ES = sizeof(elem_t);
  constexpr uint32_t VE = 16 / ES;
  const uint32_t tid = threadIdx.x, nthr = blockDim.x;
  const uint32_t tile = nthr * VE * UNROLL;

  for (uint32_t t = blockIdx.x; t < a.total_tiles; t += gridDim.x) {
    const TilePos p = locate(t, a.tiles_per_chunk, a.nseg, a.chunk, tile, a.stagger);
    const uint32_t len = tile_len(p, a.seg[p.d].n, a.chunk, tile);
    if (len == 0) continue;

    const uint64_t boff = p.lo * ES;
    const char* s0 = a.seg[p.d].src0 + boff;
    const char* s1 = NSRC == 2 ? a.seg[p.d].src1 + boff : nullptr;
    char* d0 = a.seg[p.d].dst0 + boff;
    char* d1 = NDST == 2 ? a.seg[p.d].dst1 + boff : nullptr;

    if (len == tile) {
      u32x4 v0[UNROLL], v1[UNROLL];
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) {
        const uint32_t off = (u * nthr + tid) * 16u;
        v0[u] = ld16<NT>(s0 + off);
        if (NSRC == 2) v1[u] = ld16<NT>(s1 + off);
      }
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) {
        const uint32_t off = (u * nthr + tid) * 16u;
        const u32x4 r = NSRC == 2 ? hop_vec<DT>(v0[u], v1[u]) : v0[u];
        st16<NT>(d0 + off, r);
        if (NDST == 2) st16<NT>(d1 + off, r);
      }
    } else {
      const uint32_t nvec = len / VE;
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) {
        const uint32_t vi = u * nthr + tid;
        if (vi < nvec) {
          const uint32_t off = vi * 16u;
          u32x4 r = ld16<NT>(s0 + off);
          if (NSRC == 2) r = hop_vec<DT>(r, ld16<NT>(s1 + off));
          st16<NT>(d0 + off, r);
          if (NDST == 2) st16<NT>(d1 + off, r);
        }
      }
      // fewer than VE elements may remain at the very end of a segment
      const uint32_t e = nvec * VE + tid;
      if (e < len) {
        elem_t r = reinterpret_cast<const elem_t*>(s0)[e];
        if (NSRC == 2) r = Wire<DT>::hop_elem(r, reinterpret_cast<const elem_t*>(s1)[e]);
        reinterpret_cast<elem_t*>(d0)[e] = r;
        if (NDST == 2) reinterpret_cast<elem_t*>(d1)[e] = r;
      }
    }
  }
}

// Element-wise path for addresses that are not 16-byte aligned.  Same tiles.
template <int DT, int NSRC, int NDST>
__global__ void __launch_bounds__(1024) reduce_copy_elem(const StepArgs a, const uint32_t tile) {
  typedef typename Wire<DT>::elem_t elem_t;
  const uint32_t tid = threadIdx.x, nthr = blockDim.x;
  for (uint32_t t = blockIdx.x; t < a.total_tiles; t += gridDim.x) {
    const TilePos p = locate(t, a.tiles_per_chunk, a.nseg, a.chunk, tile, a.stagger);
    const uint32_t len = tile_len(p, a.seg[p.d].n, a.chunk, tile);
    if (len == 0) continue;
    const elem_t* s0 = reinterpret_cast<const elem_t*>(a.seg[p.d].src0) + p.lo;
    const elem_t* s1 = NSRC == 2 ? reinterpret_cast<const elem_t*>(a.seg[p.d].src1) + p.lo : nullptr;
    elem_t* d0 = reinterpret_cast<elem_t*>(a.seg[p.d].dst0) + p.lo;
    elem_t* d1 = NDST == 2 ? reinterpret_cast<elem_t*>(a.seg[p.d].dst1) + p.lo : nullptr;
    for (uint32_t e = tid; e < len; e += nthr) {
      elem_t r = s0[e];
      if (NSRC == 2) r = Wire<DT>::hop_elem(r, s1[e]);
      d0[e] = r;
      if (NDST == 2) d1[e] = r;
    }
  }
}

// ---------------------------------------------------------------------------
// FUSED: the whole ring pass of an element inside one thread.
// Block c's sum starts at the rank after c in the ring and ends at c, rounding
// to the wire type after every addition -- the value the stepwise ring
// produces, with each rank's element read once.
// ---------------------------------------------------------------------------
__host__ __device__ constexpr int fused_unroll_c(int W) { return W <= 2 ? 4 : (W <= 4 ? 4 : (W <= 8 ? 2 : 1)); }

template <int DT, int W, bool NT, bool WIDE>
__global__ void __launch_bounds__(1024) ring_fused_vec(const FusedArgs a) {
  typedef typename Wire<DT>::elem_t elem_t;
  constexpr uint32_t ES = sizeof(elem_t);
  constexpr uint32_t VE = 16 / ES;
  constexpr int U = fused_unroll_c(W);
  const uint32_t tid = threadIdx.x, nthr = blockDim.x;
  const uint32_t tile = nthr * VE * U;
  const bool to_all = a.mode == 0;
  const bool whole = a.mode == 3;  // Reduce: one block, the whole vector, summed in the root's order

  for (uint32_t t = blockIdx.x; t < a.total_tiles; t += gridDim.x) {
    const TilePos p = locate(t, a.tiles_per_chunk, whole ? 1u : (uint32_t)W, a.chunk, tile);
    const uint32_t c = whole ? a.root : p.d;
    uint64_t blo = whole ? 0 : (uint64_t)c * a.B, bhi = blo + a.B;
    if (blo > a.count) blo = a.count;
    if (bhi > a.count) bhi = a.count;
    const uint32_t len = tile_len(p, bhi - blo, a.chunk, tile);
    if (len == 0) continue;

    const uint64_t voff = (blo + p.lo) * ES;  // offset inside a full vector
    const uint32_t pc = a.pos[c];
    const char* sp[W];
#pragma unroll
    for (int k = 0; k < W; ++k) sp[k] = a.src[a.order[(pc + 1 + k) % W]] + voff;

    const uint32_t nvec = len / VE;
    u32x4 v[U][W];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t vi = u * nthr + tid;
      if (vi < nvec) {
#pragma unroll
        for (int k = 0; k < W; ++k) v[u][k] = ld16<NT>(sp[k] + vi * 16u);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t vi = u * nthr + tid;
      if (vi < nvec) {
        u32x4 acc;
        if (WIDE) {
          acc = sum_wide<DT, W>(v[u]);
        } else {
          acc = v[u][0];
#pragma unroll
          for (int k = 1; k < W; ++k) acc = hop_vec<DT>(acc, v[u][k]);
        }
        if (to_all) {
#pragma unroll
          for (int r = 0; r < W; ++r) st16<NT>(a.dst[r] + voff + vi * 16u, acc);
        } else {
          st16<NT>(a.dst[c] + p.lo * ES + vi * 16u, acc);
        }
      }
    }
    const uint32_t e = nvec * VE + tid;
    if (e < len) {
      elem_t acc = reinterpret_cast<const elem_t*>(sp[0])[e];
      if (WIDE) {
        float f = widen1<DT>(acc);
#pragma unroll
        for (int k = 1; k < W; ++k) f = f + widen1<DT>(reinterpret_cast<const elem_t*>(sp[k])[e]);
        acc = narrow1<DT>(f);
      } else {
#pragma unroll
        for (int k = 1; k < W; ++k) acc = Wire<DT>::hop_elem(acc, reinterpret_cast<const elem_t*>(sp[k])[e]);
      }
      if (to_all) {
#pragma unroll
        for (int r = 0; r < W; ++r) reinterpret_cast<elem_t*>(a.dst[r] + voff)[e] = acc;
      } else {
        reinterpret_cast<elem_t*>(a.dst[c] + p.lo * ES)[e] = acc;
      }
    }
  }
}

// All-Gather in one launch: block c is read once from rank c and stored to all ranks.
template <int ES, bool NT>
__global__ void __launch_bounds__(1024) gather_fused_vec(const FusedArgs a) {
  constexpr uint32_t VE = 16 / ES;
  constexpr int U = 4;
  const uint32_t tid = threadIdx.x, nthr = blockDim.x;
  const uint32_t tile = nthr * VE * U;
  const uint32_t W = a.W;
  const bool whole = a.mode == 4;  // Broadcast: one block, the root's whole vector
  for (uint32_t t = blockIdx.x; t < a.total_tiles; t += gridDim.x) {
    const TilePos p = locate(t, a.tiles_per_chunk, whole ? 1u : W, a.chunk, tile);
    const uint32_t c = whole ? a.root : p.d;
    const uint32_t len = tile_len(p, a.B, a.chunk, tile);
    if (len == 0) continue;
    const char* s = a.src[c] + p.lo * ES;
    const uint64_t voff = ((whole ? 0 : (uint64_t)c * a.B) + p.lo) * ES;
    const uint32_t nvec = len / VE;
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t vi = u * nthr + tid;
      if (vi < nvec) v[u] = ld16<NT>(s + vi * 16u);
    }
    for (uint32_t r = 0; r < W; ++r) {
      char* d = a.dst[r] + voff;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t vi = u * nthr + tid;
        if (vi < nvec) st16<NT>(d + vi * 16u, v[u]);
      }
    }
    const uint32_t e = nvec * VE + tid;
    if (e < len) {
      if (ES == 2) {
        const uint16_t x = reinterpret_cast<const uint16_t*>(s)[e];
        for (uint32_t r = 0; r < W; ++r) reinterpret_cast<uint16_t*>(a.dst[r] + voff)[e] = x;
      } else {
        const uint32_t x = reinterpret_cast<const uint32_t*>(s)[e];
        for (uint32_t r = 0; r < W; ++r) reinterpret_cast<uint32_t*>(a.dst[r] + voff)[e] = x;
      }
    }
  }
}

// Element-wise fused path (any alignment, any W, all three modes).
template <int DT>
__global__ void __launch_bounds__(1024) ring_fused_elem(const FusedArgs a, const uint32_t tile, const bool wide) {
  typedef typename Wire<DT>::elem_t elem_t;
  const uint32_t tid = threadIdx.x, nthr = blockDim.x;
  const uint32_t W = a.W;
  const bool whole = a.mode >= 3;  // Reduce / Broadcast: one block, the whole vector, owned by the root
  const bool one_src = a.mode == 2 || a.mode == 4;
  const bool one_dst = a.mode == 1 || a.mode == 3;
  for (uint32_t t = blockIdx.x; t < a.total_tiles; t += gridDim.x) {
    const TilePos p = locate(t, a.tiles_per_chunk, whole ? 1u : W, a.chunk, tile);
    const uint32_t c = whole ? a.root : p.d;
    uint64_t blo = whole ? 0 : (uint64_t)c * a.B, bhi = blo + a.B;
    if (blo > a.count) blo = a.count;
    if (bhi > a.count) bhi = a.count;
    const uint32_t len = tile_len(p, bhi - blo, a.chunk, tile);
    if (len == 0) continue;
    const uint32_t pc = a.pos[c];
    for (uint32_t e = tid; e < len; e += nthr) {
      const uint64_t i = p.lo + e;  // inside block c
      elem_t acc;
      if (one_src) {
        acc = reinterpret_cast<const elem_t*>(a.src[c])[i];
      } else {
        acc = reinterpret_cast<const elem_t*>(a.src[a.order[(pc + 1) % W]])[blo + i];
        if (Wire<DT>::kWide && wide) {
          float f = widen1<DT>(acc);
          for (uint32_t k = 2; k <= W; ++k)
            f = f + widen1<DT>(reinterpret_cast<const elem_t*>(a.src[a.order[(pc + k) % W]])[blo + i]);
          acc = narrow1<DT>(f);
        } else {
          for (uint32_t k = 2; k <= W; ++k)
            acc = Wire<DT>::hop_elem(acc, reinterpret_cast<const elem_t*>(a.src[a.order[(pc + k) % W]])[blo + i]);
        }
      }
      if (one_dst) {
        reinterpret_cast<elem_t*>(a.dst[c])[i] = acc;
      } else {
        for (uint32_t r = 0; r < W; ++r) reinterpret_cast<elem_t*>(a.dst[r])[blo + i] = acc;
      }
    }
  }
}

// ---------------------------------------------------------------------------
// host-side dispatch
// ---------------------------------------------------------------------------
uint64_t tile_elems(int dtype, const Tuning& t) {
  const uint32_t es = (dtype == DT_BF16 || dtype == DT_FP16) ? 2 : 4;
  return (uint64_t)t.threads * (16 / es) * t.unroll;
}
int fused_unroll(int W) { return fused_unroll_c(W); }

template <int DT, int NSRC, int NDST>
static int launch_step_t(const StepArgs& a, const Tuning& t, hipStream_t s) {
  const dim3 g(t.blocks), b(t.threads);
  if (!t.vec) {
    reduce_copy_elem<DT, NSRC, NDST><<<g, b, 0, s>>>(a, (uint32_t)tile_elems(DT, t));
    return (int)hipGetLastError();
  }
#define HCL_CASE(U)                                                                      \
  case U:                                                                                \
    if (t.nontemporal) reduce_copy_vec<DT, NSRC, NDST, U, true><<<g, b, 0, s>>>(a);      \
    else reduce_copy_vec<DT, NSRC, NDST, U, false><<<g, b, 0, s>>>(a);                   \
    break;
  switch (t.unroll) {
    HCL_CASE(1) HCL_CASE(2) HCL_CASE(4) HCL_CASE(8)
    default: return (int)hipErrorInvalidValue;
  }
#undef HCL_CASE
  return (int)hipGetLastError();
}

template <int DT>
static int launch_step_d(const StepArgs& a, int nsrc, int ndst, const Tuning& t, hipStream_t s) {
  if (nsrc == 1 && ndst == 1) return launch_step_t<DT, 1, 1>(a, t, s);
  if (nsrc == 1 && ndst == 2) return launch_step_t<DT, 1, 2>(a, t, s);
  if (nsrc == 2 && ndst == 1) return launch_step_t<DT, 2, 1>(a, t, s);
  if (nsrc == 2 && ndst == 2) return launch_step_t<DT, 2, 2>(a, t, s);
  return (int)hipErrorInvalidValue;
}

int launch_step(const StepArgs& a, int dtype, int nsrc, int ndst, const Tuning& t, void* stream) {
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  // a copy moves bits: share the integer instantiations of the same element size
  if (nsrc == 1) dtype = (dtype == DT_BF16 || dtype == DT_FP16) ? DT_BF16 : DT_INT32;
  switch (dtype) {
    case DT_FP32: return launch_step_d<DT_FP32>(a, nsrc, ndst, t, s);
    case DT_BF16: return launch_step_d<DT_BF16>(a, nsrc, ndst, t, s);
    case DT_FP16: return launch_step_d<DT_FP16>(a, nsrc, ndst, t, s);
    case DT_INT32: return launch_step_d<DT_INT32>(a, nsrc, ndst, t, s);
  }
  return (int)hipErrorInvalidValue;
}

template <int DT>
static int launch_fused_d(const FusedArgs& a, const Tuning& t, hipStream_t s) {
  const dim3 g(t.blocks), b(t.threads);
  if (!t.vec) {
    const uint32_t es = sizeof(typename Wire<DT>::elem_t);
    const int U = (a.mode == 2 || a.mode == 4) ? 4 : fused_unroll_c((int)a.W);
    ring_fused_elem<DT><<<g, b, 0, s>>>(a, (uint32_t)(t.threads * (16 / es) * U), t.wide_acc);
    return (int)hipGetLastError();
  }
  if (a.mode == 2 || a.mode == 4) {
    constexpr int ES = sizeof(typename Wire<DT>::elem_t);
    if (t.nontemporal) gather_fused_vec<ES, true><<<g, b, 0, s>>>(a);
    else gather_fused_vec<ES, false><<<g, b, 0, s>>>(a);
    return (int)hipGetLastError();
  }
  constexpr bool kW = Wire<DT>::kWide;
  const bool wide = kW && t.wide_acc;
#define HCL_CASE(WW)                                                                      \
  case WW:                                                                                \
    if (wide) {                                                                           \
      if (t.nontemporal) ring_fused_vec<DT, WW, true, kW><<<g, b, 0, s>>>(a);             \
      else ring_fused_vec<DT, WW, false, kW><<<g, b, 0, s>>>(a);                          \
    } else {                                                                              \
      if (t.nontemporal) ring_fused_vec<DT, WW, true, false><<<g, b, 0, s>>>(a);          \
      else ring_fused_vec<DT, WW, false, false><<<g, b, 0, s>>>(a);                       \
    }                                                                                     \
    break;
  switch (a.W) {
    HCL_CASE(2) HCL_CASE(3) HCL_CASE(4) HCL_CASE(5) HCL_CASE(6) HCL_CASE(7) HCL_CASE(8) HCL_CASE(9)
    HCL_CASE(10) HCL_CASE(11) HCL_CASE(12) HCL_CASE(13) HCL_CASE(14) HCL_CASE(15) HCL_CASE(16)
    default: return (int)hipErrorInvalidValue;
  }
#undef HCL_CASE
  return (int)hipGetLastError();
}

int launch_fused(const FusedArgs& a, int dtype, const Tuning& t, void* stream) {
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  switch (dtype) {
    case DT_FP32: return launch_fused_d<DT_FP32>(a, t, s);
    case DT_BF16: return launch_fused_d<DT_BF16>(a, t, s);
    case DT_FP16: return launch_fused_d<DT_FP16>(a, t, s);
    case DT_INT32: return launch_fused_d<DT_INT32>(a, t, s);
  }
  return (int)hipErrorInvalidValue;
}

}  // namespace hcl

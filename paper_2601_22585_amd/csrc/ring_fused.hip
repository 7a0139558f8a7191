// gfx950 kernels for the FUSED schedule: the whole ring pass of an element
// stays inside one thread, every rank's value is read once.
//
// This file is compiled once per (HCL_FUSED_DT, HCL_FUSED_PART): the wire type
// (0 fp32, 1 bf16, 2 fp16, 3 int32, 4 fp64, 5 int64, 6 uint8) and the part -- 0: ring-order sums and the
// All-Gather / Broadcast kernel; 1: the general form
// (run-time operator, tree order, rounding once).  Each object file holds one
// explicit instantiation of launch_fused_sum<DT> or launch_fused_gen<DT>.
#include "wire.h"

#if !defined(HCL_FUSED_DT) || !defined(HCL_FUSED_PART)
#error "compile with -DHCL_FUSED_DT=<0..6> -DHCL_FUSED_PART=<0|1>"
#endif

namespace hcl {

#if HCL_FUSED_PART == 0
// ---------------------------------------------------------------------------
// FUSED: the whole ring pass of an element inside one thread.
// Block c's sum starts at the rank after c in the ring and ends at c, rounding
// to the wire type after every addition -- the value the stepwise ring
// produces, with each rank's element read once.
// ---------------------------------------------------------------------------
// NT: 0 ordinary loads and stores; 1 non-temporal loads, stores written through the L2; 2
// non-temporal loads and stores (as in the step kernels)
template <int DT, int W, int NT, bool WIDE>
__global__ void __launch_bounds__(1024) ring_fused_vec(const FusedArgs a) {
  constexpr bool NTL = NT != 0;
  constexpr int NTS = NT == 2 ? ST_STREAM : NT == 1 ? ST_THROUGH : ST_PLAIN;
  typedef typename Wire<DT>::elem_t elem_t;
  constexpr uint32_t ES = sizeof(elem_t);
  constexpr uint32_t VE = 16 / ES;
  constexpr int U = fused_unroll(W);
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
    // The block's head, up to the first 128-byte boundary, is done by the tile that starts the
    // block (part 0: a few unaligned vectors and single elements); the tile grid covers the rest
    // (part 1).  The boundary is that of the streams that carry most of the traffic: the W
    // destinations of an All-Reduce, the W sources of a reduction to one owner.
    const uint32_t pre = head_elems<ES>((to_all ? a.dst[0] : a.src[0]) + blo * ES, bhi - blo);
    for (int part = (p.lo == 0 && pre) ? 0 : 1; part < 2; ++part) {
      const uint64_t lo = part ? pre + p.lo : 0;  // first element inside the block
      const uint32_t len = part ? tile_len(p, bhi - blo - pre, a.chunk, tile) : pre;
      if (len == 0) continue;

      const uint64_t voff = (blo + lo) * ES;  // offset inside a full vector
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
          for (int k = 0; k < W; ++k) v[u][k] = ld16<NTL>(sp[k] + vi * 16u);
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
            for (int r = 0; r < W; ++r) st16<NTS>(a.dst[r] + voff + vi * 16u, acc);
          } else {
            st16<NTS>(a.dst[c] + lo * ES + vi * 16u, acc);
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
          reinterpret_cast<elem_t*>(a.dst[c] + lo * ES)[e] = acc;
        }
      }
    }
  }
}

// All-Gather in one launch: block c is read once from rank c and stored to all ranks.
template <int ES, int NT, int U>
__global__ void __launch_bounds__(1024) gather_fused_vec(const FusedArgs a) {
  constexpr bool NTL = NT != 0;
  constexpr int NTS = NT == 2 ? ST_STREAM : NT == 1 ? ST_THROUGH : ST_PLAIN;
  constexpr uint32_t VE = 16 / ES;
  const uint32_t tid = threadIdx.x, nthr = blockDim.x;
  const uint32_t tile = nthr * VE * U;
  const uint32_t W = a.W;
  const bool whole = a.mode == 4;  // Broadcast: one block, the root's whole vector
  for (uint32_t t = blockIdx.x; t < a.total_tiles; t += gridDim.x) {
    const TilePos p = locate(t, a.tiles_per_chunk, whole ? 1u : W, a.chunk, tile);
    const uint32_t c = whole ? a.root : p.d;
    // head of the block (up to the first 128-byte boundary of the W destination streams): part 0,
    // by the tile that starts the block; the tile grid covers the rest: part 1
    const uint64_t boff = whole ? 0 : (uint64_t)c * a.B;
    const uint32_t pre = head_elems<ES>(a.dst[0] + boff * ES, a.B);
    for (int part = (p.lo == 0 && pre) ? 0 : 1; part < 2; ++part) {
      const uint64_t lo = part ? pre + p.lo : 0;
      const uint32_t len = part ? tile_len(p, a.B - pre, a.chunk, tile) : pre;
      if (len == 0) continue;
      const char* s = a.src[c] + lo * ES;
      const uint64_t voff = (boff + lo) * ES;
      const uint32_t nvec = len / VE;
      u32x4 v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t vi = u * nthr + tid;
        if (vi < nvec) v[u] = ld16<NTL>(s + vi * 16u);
      }
      for (uint32_t r = 0; r < W; ++r) {
        char* d = a.dst[r] + voff;
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const uint32_t vi = u * nthr + tid;
          if (vi < nvec) st16<NTS>(d + vi * 16u, v[u]);
        }
      }
      const uint32_t e = nvec * VE + tid;
      if (e < len) {
        // up to VE - 1 elements: the tail of a 16-byte vector (ES = 8 never gets here)
        if (ES == 1) {
          const uint8_t x = reinterpret_cast<const uint8_t*>(s)[e];
          for (uint32_t r = 0; r < W; ++r) reinterpret_cast<uint8_t*>(a.dst[r] + voff)[e] = x;
        } else if (ES == 2) {
          const uint16_t x = reinterpret_cast<const uint16_t*>(s)[e];
          for (uint32_t r = 0; r < W; ++r) reinterpret_cast<uint16_t*>(a.dst[r] + voff)[e] = x;
        } else if (ES == 4) {
          const uint32_t x = reinterpret_cast<const uint32_t*>(s)[e];
          for (uint32_t r = 0; r < W; ++r) reinterpret_cast<uint32_t*>(a.dst[r] + voff)[e] = x;
        } else {
          const uint64_t x = reinterpret_cast<const uint64_t*>(s)[e];
          for (uint32_t r = 0; r < W; ++r) reinterpret_cast<uint64_t*>(a.dst[r] + voff)[e] = x;
        }
      }
    }
  }
}

#else
// ---------------------------------------------------------------------------
// FUSED, general form: run-time operator (a.op), ring or tree order (a.tree),
// per-result rounding or binary32 intermediates with one rounding (a.wide).
// Ring order: block c's values enter in the order next(c), ..., c.  Tree order:
// ranks in ring order ring[0] .. ring[W-1] for every block, neighbours combined
// first, level by level; an odd last value moves up unchanged.
// ---------------------------------------------------------------------------
template <int DT, int W>
__device__ __forceinline__ uint32_t combine_word(const uint32_t (&w)[W], uint32_t op, bool tree, bool wide) {
  if (DT == DT_INT32 || DT == DT_UINT8) {
    uint32_t v[W];
#pragma unroll
    for (int k = 0; k < W; ++k) v[k] = w[k];
    if (!tree) {
#pragma unroll
      for (int k = 1; k < W; ++k) v[0] = op_word<DT>(op, v[0], v[k]);
    } else {
#pragma unroll
      for (int n = W; n > 1; n = (n + 1) / 2) {
#pragma unroll
        for (int k = 0; k + 1 < n; k += 2) v[k / 2] = op_word<DT>(op, v[k], v[k + 1]);
        if (n & 1) v[n / 2] = v[n - 1];
      }
    }
    return v[0];
  }
  constexpr bool kTwo = Wire<DT>::kWide;  // two elements per word
  float lo[W], hi[W];
#pragma unroll
  for (int k = 0; k < W; ++k) {
    if (kTwo) {
      Wire<DT>::widen2(w[k], lo[k], hi[k]);
    } else {
      lo[k] = u2f(w[k]);
      hi[k] = 0.0f;
    }
  }
  // one node: the operator, then (unless wide) a trip through the wire type
  auto node = [&](float& alo, float& ahi, float blo, float bhi) {
    alo = apply_f32(op, alo, blo);
    if (kTwo) {
      ahi = apply_f32(op, ahi, bhi);
      if (!wide) Wire<DT>::widen2(Wire<DT>::narrow2(alo, ahi), alo, ahi);
    }
  };
  if (!tree) {
#pragma unroll
    for (int k = 1; k < W; ++k) node(lo[0], hi[0], lo[k], hi[k]);
  } else {
#pragma unroll
    for (int n = W; n > 1; n = (n + 1) / 2) {
#pragma unroll
      for (int k = 0; k + 1 < n; k += 2) {
        float a = lo[k], b = hi[k];
        node(a, b, lo[k + 1], hi[k + 1]);
        lo[k / 2] = a;
        hi[k / 2] = b;
      }
      if (n & 1) {
        lo[n / 2] = lo[n - 1];
        hi[n / 2] = hi[n - 1];
      }
    }
  }
  return kTwo ? Wire<DT>::narrow2(lo[0], hi[0]) : f2u(lo[0]);
}

// the same for one eight-byte element (fp64, int64): nothing to widen or round
template <int DT, int W>
__device__ __forceinline__ uint64_t combine64(const uint64_t (&w)[W], uint32_t op, bool tree) {
  uint64_t v[W];
#pragma unroll
  for (int k = 0; k < W; ++k) v[k] = w[k];
  if (!tree) {
#pragma unroll
    for (int k = 1; k < W; ++k) v[0] = op_elem64<DT>(op, v[0], v[k]);
  } else {
#pragma unroll
    for (int n = W; n > 1; n = (n + 1) / 2) {
#pragma unroll
      for (int k = 0; k + 1 < n; k += 2) v[k / 2] = op_elem64<DT>(op, v[k], v[k + 1]);
      if (n & 1) v[n / 2] = v[n - 1];
    }
  }
  return v[0];
}

// a whole 128-bit vector per rank
template <int DT, int W>
__device__ __forceinline__ u32x4 combine_vec(const u32x4 (&v)[W], uint32_t op, bool tree, bool wide) {
  u32x4 acc;
  if (sizeof(typename Wire<DT>::elem_t) == 8) {
    uint64_t lo[W], hi[W];
#pragma unroll
    for (int k = 0; k < W; ++k) {
      lo[k] = (uint64_t)v[k].x | ((uint64_t)v[k].y << 32);
      hi[k] = (uint64_t)v[k].z | ((uint64_t)v[k].w << 32);
    }
    const uint64_t a = combine64<DT, W>(lo, op, tree), b = combine64<DT, W>(hi, op, tree);
    acc.x = (uint32_t)a;
    acc.y = (uint32_t)(a >> 32);
    acc.z = (uint32_t)b;
    acc.w = (uint32_t)(b >> 32);
    return acc;
  }
  uint32_t wx[W], wy[W], wz[W], ww[W];
#pragma unroll
  for (int k = 0; k < W; ++k) {
    wx[k] = v[k].x;
    wy[k] = v[k].y;
    wz[k] = v[k].z;
    ww[k] = v[k].w;
  }
  acc.x = combine_word<DT, W>(wx, op, tree, wide);
  acc.y = combine_word<DT, W>(wy, op, tree, wide);
  acc.z = combine_word<DT, W>(wz, op, tree, wide);
  acc.w = combine_word<DT, W>(ww, op, tree, wide);
  return acc;
}

template <int DT, int W, int NT>
__global__ void __launch_bounds__(kGenMaxThreads) ring_fused_gen(const FusedArgs a) {
  constexpr bool NTL = NT != 0;
  constexpr int NTS = NT == 2 ? ST_STREAM : NT == 1 ? ST_THROUGH : ST_PLAIN;
  typedef typename Wire<DT>::elem_t elem_t;
  constexpr uint32_t ES = sizeof(elem_t);
  constexpr uint32_t VE = 16 / ES;
  constexpr int U = kGenUnroll;
  const uint32_t tid = threadIdx.x, nthr = blockDim.x;
  const uint32_t tile = nthr * VE * U;
  const bool to_all = a.mode == 0;
  const bool whole = a.mode == 3;
  const uint32_t op = a.op;
  const bool tree = a.tree != 0, wide = a.wide != 0;

  for (uint32_t t = blockIdx.x; t < a.total_tiles; t += gridDim.x) {
    const TilePos p = locate(t, a.tiles_per_chunk, whole ? 1u : (uint32_t)W, a.chunk, tile);
    const uint32_t c = whole ? a.root : p.d;
    uint64_t blo = whole ? 0 : (uint64_t)c * a.B, bhi = blo + a.B;
    if (blo > a.count) blo = a.count;
    if (bhi > a.count) bhi = a.count;
    // head of the block up to the first 128-byte boundary: part 0, by the tile that starts the
    // block; the tile grid covers the rest: part 1 (as in the sum kernel)
    const uint32_t pre = head_elems<ES>((to_all ? a.dst[0] : a.src[0]) + blo * ES, bhi - blo);
    for (int part = (p.lo == 0 && pre) ? 0 : 1; part < 2; ++part) {
      const uint64_t lo = part ? pre + p.lo : 0;
      const uint32_t len = part ? tile_len(p, bhi - blo - pre, a.chunk, tile) : pre;
      if (len == 0) continue;

      const uint64_t voff = (blo + lo) * ES;
      const uint32_t first = tree ? 0u : a.pos[c] + 1u;  // ring position of the first value to enter
      const char* sp[W];
#pragma unroll
      for (int k = 0; k < W; ++k) sp[k] = a.src[a.order[(first + k) % W]] + voff;

      const uint32_t nvec = len / VE;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t vi = u * nthr + tid;
        if (vi < nvec) {
          u32x4 v[W];
#pragma unroll
          for (int k = 0; k < W; ++k) v[k] = ld16<NTL>(sp[k] + vi * 16u);
          const u32x4 acc = combine_vec<DT, W>(v, op, tree, wide);
          if (to_all) {
#pragma unroll
            for (int r = 0; r < W; ++r) st16<NTS>(a.dst[r] + voff + vi * 16u, acc);
          } else {
            st16<NTS>(a.dst[c] + lo * ES + vi * 16u, acc);
          }
        }
      }
      const uint32_t e = nvec * VE + tid;
      if (e < len) {
        // one element: put it into the low bits of a word (or a 64-bit value) and combine those
        elem_t acc;
        if (sizeof(elem_t) == 8) {
          uint64_t w1[W];
#pragma unroll
          for (int k = 0; k < W; ++k) w1[k] = (uint64_t)reinterpret_cast<const elem_t*>(sp[k])[e];
          acc = (elem_t)combine64<DT, W>(w1, op, tree);
        } else {
          uint32_t w1[W];
#pragma unroll
          for (int k = 0; k < W; ++k) w1[k] = (uint32_t)reinterpret_cast<const elem_t*>(sp[k])[e];
          acc = (elem_t)combine_word<DT, W>(w1, op, tree, wide);
        }
        if (to_all) {
#pragma unroll
          for (int r = 0; r < W; ++r) reinterpret_cast<elem_t*>(a.dst[r] + voff)[e] = acc;
        } else {
          reinterpret_cast<elem_t*>(a.dst[c] + lo * ES)[e] = acc;
        }
      }
    }
  }
}

#endif

// ---------------------------------------------------------------------------
// host-side dispatch
// ---------------------------------------------------------------------------
#if HCL_FUSED_PART == 0
template <int DT>
int launch_fused_sum(const FusedArgs& a, const Tuning& t, void* stream) {
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  const dim3 g(t.blocks), b(t.threads);
  if (a.mode == 2 || a.mode == 4) {
    constexpr int ES = sizeof(typename Wire<DT>::elem_t);
#define HCL_CASE(UU)                                                            \
  case UU:                                                                      \
    if (t.nt == 2) gather_fused_vec<ES, 2, UU><<<g, b, 0, s>>>(a);              \
    else if (t.nt == 1) gather_fused_vec<ES, 1, UU><<<g, b, 0, s>>>(a);         \
    else gather_fused_vec<ES, 0, UU><<<g, b, 0, s>>>(a);                        \
    break;
    switch (t.unroll) {
      HCL_CASE(1) HCL_CASE(2) HCL_CASE(4)
      default: return (int)hipErrorInvalidValue;
    }
#undef HCL_CASE
    return (int)hipGetLastError();
  }
  constexpr bool kW = Wire<DT>::kWide;
  const bool wide = kW && a.wide;
#define HCL_CASE(WW)                                                                      \
  case WW:                                                                                \
    if (wide) {                                                                           \
      if (t.nt == 2) ring_fused_vec<DT, WW, 2, kW><<<g, b, 0, s>>>(a);                    \
      else if (t.nt == 1) ring_fused_vec<DT, WW, 1, kW><<<g, b, 0, s>>>(a);               \
      else ring_fused_vec<DT, WW, 0, kW><<<g, b, 0, s>>>(a);                              \
    } else {                                                                              \
      if (t.nt == 2) ring_fused_vec<DT, WW, 2, false><<<g, b, 0, s>>>(a);                 \
      else if (t.nt == 1) ring_fused_vec<DT, WW, 1, false><<<g, b, 0, s>>>(a);            \
      else ring_fused_vec<DT, WW, 0, false><<<g, b, 0, s>>>(a);                           \
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
template int launch_fused_sum<HCL_FUSED_DT>(const FusedArgs&, const Tuning&, void*);
#else
template <int DT>
int launch_fused_gen(const FusedArgs& a, const Tuning& t, void* stream) {
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  const dim3 g(t.blocks), b(t.threads);
  if (t.threads > kGenMaxThreads) return (int)hipErrorInvalidValue;
#define HCL_CASE(WW)                                                              \
  case WW:                                                                        \
    if (t.nt == 2) ring_fused_gen<DT, WW, 2><<<g, b, 0, s>>>(a);                  \
    else if (t.nt == 1) ring_fused_gen<DT, WW, 1><<<g, b, 0, s>>>(a);             \
    else ring_fused_gen<DT, WW, 0><<<g, b, 0, s>>>(a);                            \
    break;
  switch (a.W) {
    HCL_CASE(2) HCL_CASE(3) HCL_CASE(4) HCL_CASE(5) HCL_CASE(6) HCL_CASE(7) HCL_CASE(8) HCL_CASE(9)
    HCL_CASE(10) HCL_CASE(11) HCL_CASE(12) HCL_CASE(13) HCL_CASE(14) HCL_CASE(15) HCL_CASE(16)
    default: return (int)hipErrorInvalidValue;
  }
#undef HCL_CASE
  return (int)hipGetLastError();
}
template int launch_fused_gen<HCL_FUSED_DT>(const FusedArgs&, const Tuning&, void*);
#endif

}  // namespace hcl

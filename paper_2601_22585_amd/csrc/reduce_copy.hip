// gfx950 reduce-copy kernels for the ring collectives: one ring step of every rank.
//
// The work is streaming and element-wise (at most one fp32 operation per 6-12
// bytes moved), so the design targets HBM bandwidth, not the matrix cores: every
// lane moves 128-bit vectors, a wavefront's 64 lanes cover 1 KiB of contiguous
// memory per access, each thread issues all loads of a tile (UNROLL vectors
// per source) before the first use; outputs the next launch reads are written
// through the L2, all others with non-temporal stores.  A launch covers one tile per workgroup, or strides over the tiles
// when the grid is capped.
#include "wire.h"
#include "ring_sched.h"

namespace hcl {

// ---------------------------------------------------------------------------
// STEPWISE: one ring step of every rank.  128-bit path.
// ---------------------------------------------------------------------------
// GEN: the operator is a.op at run time (product, maximum, minimum); otherwise the sum.
// NT: 0 ordinary loads and stores; 1 non-temporal loads, stores written through the L2 -- what a
// step writes is then in the 256 MiB last-level cache when the next step reads it as its incoming
// operand; 2 non-temporal loads and stores, for outputs that exceed that cache or that no later
// launch reads.
template <int DT, int NSRC, int NDST, int UNROLL, int NT, bool GEN>
__global__ void __launch_bounds__(1024) reduce_copy_vec(const StepArgs a) {
  constexpr bool NTL = NT >= 1;
  constexpr int NTS = NT == 2 ? ST_STREAM : NT == 1 ? ST_THROUGH : ST_PLAIN;
  typedef typename Wire<DT>::elem_t elem_t;
  constexpr uint32_t ES = sizeof(elem_t);
  constexpr uint32_t VE = 16 / ES;
  const uint32_t tid = threadIdx.x, nthr = blockDim.x;
  const uint32_t tile = nthr * VE * UNROLL;

  for (uint32_t t0 = blockIdx.x; t0 < a.total_tiles; t0 += gridDim.x) {
    // consecutive steps walk the tiles in opposite directions: what the step before wrote last
    // is what the last-level cache still holds, so it is read first
    const uint32_t t = a.reverse ? a.total_tiles - 1u - t0 : t0;
    const TilePos p = locate(t, a.tiles_per_chunk, a.nseg, a.chunk, tile, a.stagger);
    // the segment's head, up to the first 128-byte boundary of its destination: element by
    // element, by the tile that starts the segment; the tile grid covers what follows it
    const uint32_t pre = head_elems<ES>(a.seg[p.d].dst0, a.seg[p.d].n);
    if (p.lo == 0 && pre) {
      const elem_t* h0 = reinterpret_cast<const elem_t*>(a.seg[p.d].src0);
      const elem_t* h1 = reinterpret_cast<const elem_t*>(a.seg[p.d].src1);
      for (uint32_t e = tid; e < pre; e += nthr) {
        elem_t r = h0[e];
        if (NSRC == 2) r = GEN ? op_elem<DT>(a.op, r, h1[e]) : Wire<DT>::hop_elem(r, h1[e]);
        reinterpret_cast<elem_t*>(a.seg[p.d].dst0)[e] = r;
        if (NDST == 2) reinterpret_cast<elem_t*>(a.seg[p.d].dst1)[e] = r;
      }
    }
    const uint32_t len = tile_len(p, a.seg[p.d].n - pre, a.chunk, tile);
    if (len == 0) continue;

    const uint64_t boff = (pre + p.lo) * ES;
    const char* s0 = a.seg[p.d].src0 + boff;
    const char* s1 = NSRC == 2 ? a.seg[p.d].src1 + boff : nullptr;
    char* d0 = a.seg[p.d].dst0 + boff;
    char* d1 = NDST == 2 ? a.seg[p.d].dst1 + boff : nullptr;

    if (len == tile) {
      u32x4 v0[UNROLL], v1[UNROLL];
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) {
        const uint32_t off = (u * nthr + tid) * 16u;
        v0[u] = ld16<NTL>(s0 + off);
        if (NSRC == 2) v1[u] = ld16<NTL>(s1 + off);
      }
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) {
        const uint32_t off = (u * nthr + tid) * 16u;
        const u32x4 r = NSRC == 2 ? (GEN ? op_vec<DT>(a.op, v0[u], v1[u]) : hop_vec<DT>(v0[u], v1[u])) : v0[u];
        st16<NTS>(d0 + off, r);
        if (NDST == 2) st16<NTS>(d1 + off, r);
      }
    } else {
      const uint32_t nvec = len / VE;
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) {
        const uint32_t vi = u * nthr + tid;
        if (vi < nvec) {
          const uint32_t off = vi * 16u;
          u32x4 r = ld16<NTL>(s0 + off);
          if (NSRC == 2) r = GEN ? op_vec<DT>(a.op, r, ld16<NTL>(s1 + off)) : hop_vec<DT>(r, ld16<NTL>(s1 + off));
          st16<NTS>(d0 + off, r);
          if (NDST == 2) st16<NTS>(d1 + off, r);
        }
      }
      // fewer than VE elements may remain at the very end of a segment
      const uint32_t e = nvec * VE + tid;
      if (e < len) {
        elem_t r = reinterpret_cast<const elem_t*>(s0)[e];
        if (NSRC == 2) {
          const elem_t x = reinterpret_cast<const elem_t*>(s1)[e];
          r = GEN ? op_elem<DT>(a.op, r, x) : Wire<DT>::hop_elem(r, x);
        }
        reinterpret_cast<elem_t*>(d0)[e] = r;
        if (NDST == 2) reinterpret_cast<elem_t*>(d1)[e] = r;
      }
    }
  }
}

// ---------------------------------------------------------------------------
// host-side dispatch
// ---------------------------------------------------------------------------
uint64_t tile_elems(int dtype, const Tuning& t) {
  const uint32_t es = (uint32_t)elem_size(dtype);
  return (uint64_t)t.threads * (16 / es) * t.unroll;
}

// GEN: the kernel reads the operator from the step's arguments (anything but the sum)
template <int DT, int NSRC, int NDST, bool GEN>
static int launch_step_vec(const StepArgs& a, const Tuning& t, hipStream_t s) {
  const dim3 g(t.blocks), b(t.threads);
#define HCL_CASE(U)                                                                          \
  case U:                                                                                    \
    if (t.nt == 2) reduce_copy_vec<DT, NSRC, NDST, U, 2, GEN><<<g, b, 0, s>>>(a);            \
    else if (t.nt == 1) reduce_copy_vec<DT, NSRC, NDST, U, 1, GEN><<<g, b, 0, s>>>(a);       \
    else reduce_copy_vec<DT, NSRC, NDST, U, 0, GEN><<<g, b, 0, s>>>(a);                      \
    break;
  switch (t.unroll) {
    HCL_CASE(1) HCL_CASE(2) HCL_CASE(4) HCL_CASE(8)
    default: return (int)hipErrorInvalidValue;
  }
#undef HCL_CASE
  return (int)hipGetLastError();
}

template <int DT, int NSRC, int NDST>
static int launch_step_t(const StepArgs& a, const Tuning& t, hipStream_t s) {
  if constexpr (NSRC == 2) {
    if (a.op != OP_SUM) return launch_step_vec<DT, NSRC, NDST, true>(a, t, s);
  }
  return launch_step_vec<DT, NSRC, NDST, false>(a, t, s);
}

// A copy moves bits: only one wire type per element size carries the NSRC = 1 kernels.
template <int DT>
constexpr bool kCopyType = DT == DT_UINT8 || DT == DT_BF16 || DT == DT_INT32 || DT == DT_INT64;

template <int DT>
static int launch_step_d(const StepArgs& a, int nsrc, int ndst, const Tuning& t, hipStream_t s) {
  if constexpr (kCopyType<DT>) {
    if (nsrc == 1 && ndst == 1) return launch_step_t<DT, 1, 1>(a, t, s);
    if (nsrc == 1 && ndst == 2) return launch_step_t<DT, 1, 2>(a, t, s);
  }
  if (nsrc == 2 && ndst == 1) return launch_step_t<DT, 2, 1>(a, t, s);
  if (nsrc == 2 && ndst == 2) return launch_step_t<DT, 2, 2>(a, t, s);
  return (int)hipErrorInvalidValue;
}

int launch_step(const StepArgs& a, int dtype, int nsrc, int ndst, const Tuning& t, void* stream) {
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  // a copy moves bits: route it to the wire type that carries the copy kernels of this element size
  if (nsrc == 1) {
    switch (elem_size(dtype)) {
      case 1: dtype = DT_UINT8; break;
      case 2: dtype = DT_BF16; break;
      case 8: dtype = DT_INT64; break;
      default: dtype = DT_INT32; break;
    }
  }
  switch (dtype) {
    case DT_FP32: return launch_step_d<DT_FP32>(a, nsrc, ndst, t, s);
    case DT_BF16: return launch_step_d<DT_BF16>(a, nsrc, ndst, t, s);
    case DT_FP16: return launch_step_d<DT_FP16>(a, nsrc, ndst, t, s);
    case DT_INT32: return launch_step_d<DT_INT32>(a, nsrc, ndst, t, s);
    case DT_FP64: return launch_step_d<DT_FP64>(a, nsrc, ndst, t, s);
    case DT_INT64: return launch_step_d<DT_INT64>(a, nsrc, ndst, t, s);
    case DT_UINT8: return launch_step_d<DT_UINT8>(a, nsrc, ndst, t, s);
  }
  return (int)hipErrorInvalidValue;
}

// FUSED: the kernels of each wire type live in object files of their own
int launch_fused(const FusedArgs& a, int dtype, const Tuning& t, void* stream) {
  const bool copy = a.mode == 2 || a.mode == 4;
  const bool gen = !copy && (a.op != OP_SUM || a.tree);
  switch (dtype) {
    case DT_FP32: return gen ? launch_fused_gen<DT_FP32>(a, t, stream) : launch_fused_sum<DT_FP32>(a, t, stream);
    case DT_BF16: return gen ? launch_fused_gen<DT_BF16>(a, t, stream) : launch_fused_sum<DT_BF16>(a, t, stream);
    case DT_FP16: return gen ? launch_fused_gen<DT_FP16>(a, t, stream) : launch_fused_sum<DT_FP16>(a, t, stream);
    case DT_INT32: return gen ? launch_fused_gen<DT_INT32>(a, t, stream) : launch_fused_sum<DT_INT32>(a, t, stream);
    case DT_FP64: return gen ? launch_fused_gen<DT_FP64>(a, t, stream) : launch_fused_sum<DT_FP64>(a, t, stream);
    case DT_INT64: return gen ? launch_fused_gen<DT_INT64>(a, t, stream) : launch_fused_sum<DT_INT64>(a, t, stream);
    case DT_UINT8: return gen ? launch_fused_gen<DT_UINT8>(a, t, stream) : launch_fused_sum<DT_UINT8>(a, t, stream);
  }
  return (int)hipErrorInvalidValue;
}

}  // namespace hcl

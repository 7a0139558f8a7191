// Launch interface of the gfx950 reduce-copy kernels (host side sees only PODs).
#pragma once
#include <cstddef>
#include <cstdint>

namespace hcl {

constexpr int kMaxSegs = 32;
constexpr int kMaxFusedRanks = 16;
// blocks from this size on are copied with four vectors per thread by the one-source kernel
constexpr uint64_t kGatherBigBlock = 1ull << 30;

// One rank's work in one ring step: dst0[i] (and dst1[i]) = hop(src0[i], src1[i])
// for NSRC = 2, or = src0[i] for NSRC = 1, i in [0, n).
struct Seg {
  const char* src0;  // incoming operand (predecessor's buffer or this rank's inbox)
  const char* src1;  // local operand (NSRC = 2 only)
  char* dst0;        // this rank's buffer
  char* dst1;        // forwarded copy (NDST = 2 only)
  uint64_t n;        // elements
};

// All ranks' segments of one step.  Tiles are ordered chunk-major: tile index
// t -> (chunk j, segment d, tile k inside the chunk), j slowest.
struct StepArgs {
  Seg seg[kMaxSegs];
  uint32_t nseg;
  uint32_t tiles_per_chunk;
  uint32_t total_tiles;
  uint32_t stagger;  // segment d starts its walk through a chunk d * stagger tiles in (mod tiles_per_chunk)
  uint64_t chunk;    // elements per chunk (> 0)
  uint32_t op;       // NSRC = 2: 0 sum, 1 product, 2 maximum, 3 minimum
  uint32_t reverse;  // 1: the tiles are walked from the last to the first
};

// Whole-collective launch: every element's ring pass stays in one thread.
struct FusedArgs {
  const char* src[16];  // per rank, start of its full vector (AR, RS, Reduce) or of its shard (AG)
  char* dst[16];        // per rank, start of its full vector (AR, AG, Broadcast) or of its shard (RS)
  uint8_t order[16];    // ring order
  uint8_t pos[16];      // ring position of each rank
  uint64_t count;       // elements in the full vector
  uint64_t B;           // elements per block
  uint64_t chunk;       // elements per chunk (> 0)
  uint32_t tiles_per_chunk;
  uint32_t total_tiles;
  uint32_t W;
  uint32_t mode;        // 0 All-Reduce, 1 Reduce-Scatter, 2 All-Gather, 3 Reduce, 4 Broadcast
  uint32_t root;        // Reduce / Broadcast: the whole vector is one block that belongs to this rank
  uint8_t op;           // 0 sum, 1 product, 2 maximum, 3 minimum
  uint8_t tree;         // 0: ring order, block c's values enter as next(c) .. c; 1: tree over ring order
  uint8_t wide;         // 1: binary32 intermediates, one rounding at the end (two-byte float types)
  uint8_t pad_;
};

struct Tuning {
  int threads;      // per workgroup, multiple of 64
  int blocks;       // workgroups
  int unroll;       // 1, 2, 4, 8
  int nt;           // cache policy: 0 ordinary loads and stores; 1 non-temporal (streaming) loads, stores
                    // written through the L2; 2 non-temporal loads and stores
};

// Elements one tile covers for this dtype / tuning.
uint64_t tile_elems(int dtype, const Tuning& t);
// 128-bit vectors per thread and rank the fused kernels keep in flight for a given W.  One
// vector (1 KiB per wavefront and rank) measured best on MI355X for every W: against two or
// four it gained 8-14 % at W = 2, 3, a few per cent up to W = 8, and two vectors at W = 16
// ran into the register budget of 1024-thread workgroups.
constexpr int fused_unroll(int /*W*/) { return 1; }
// vectors per thread of the one-source, W-destination kernel (All-Gather, Broadcast) for a
// block of `block_bytes`.  Measured on MI355X: one vector is 3-14 % faster than two or four up
// to 512 MiB blocks, four vectors are 10 % faster at 2 GiB blocks.
constexpr int gather_unroll(uint64_t block_bytes) { return block_bytes >= kGatherBigBlock ? 4 : 1; }
// the general-form kernel (run-time operator, tree order) always keeps one
constexpr int kGenUnroll = 1;

// The general-form fused kernel keeps every rank's vector and its widened
// elements in registers: it is built for workgroups of at most this many threads.
constexpr int kGenMaxThreads = 256;

// Both return a hipError_t value (0 = success) from the launch.
int launch_step(const StepArgs& a, int dtype, int nsrc, int ndst, const Tuning& t, void* stream);
int launch_fused(const FusedArgs& a, int dtype, const Tuning& t, void* stream);

// Per wire type (0 fp32, 1 bf16, 2 fp16, 3 int32, 4 fp64, 5 int64, 6 uint8), one object file each:
// ring-order sums and copies / the general form.
template <int DT> int launch_fused_sum(const FusedArgs& a, const Tuning& t, void* stream);
template <int DT> int launch_fused_gen(const FusedArgs& a, const Tuning& t, void* stream);

}  // namespace hcl

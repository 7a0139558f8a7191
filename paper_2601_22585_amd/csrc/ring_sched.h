// Ring chunk scheduler: host-only integer logic (no HIP types).
//
// The paper takes the vendor libraries' host side -- how a message is cut up
// and which piece moves when -- as a black box (Section 4.2); this is that
// logic for the textbook ring, written out: which block every rank sends and
// receives at every step, where a block sits in the vector, and how a block is
// cut into chunks.
#pragma once
#include <cstddef>
#include <cstdint>

namespace hcl {

constexpr int kMaxRanks = 16;

struct Ring {
  int W = 0;
  int order[kMaxRanks];  // order[k] = rank at ring position k
  int pos[kMaxRanks];    // pos[r]   = ring position of rank r

  // false if `ring` is not a permutation of 0..W-1 (nullptr = identity)
  bool init(int W_, const int* ring);
  int next(int r) const { return order[(pos[r] + 1) % W]; }
  int prev(int r) const { return order[(pos[r] + W - 1) % W]; }
  int at(int k) const { return order[((k % W) + W) % W]; }

  // Reduce-Scatter step s: rank r passes on block at(pos-s-1) and receives,
  // then reduces into its own data, block at(pos-s-2).  After step W-2 the
  // received block is r itself: rank r owns the finished block r.
  int rs_send(int r, int s) const { return at(pos[r] - s - 1); }
  int rs_recv(int r, int s) const { return at(pos[r] - s - 2); }
  // All-Gather step s: rank r passes on block at(pos-s) (its own finished
  // block at s = 0) and receives block at(pos-s-1).
  int ag_send(int r, int s) const { return at(pos[r] - s); }
  int ag_recv(int r, int s) const { return at(pos[r] - s - 1); }
};

// Block c of a `count`-element vector cut into pieces of B elements:
// [min(c*B, count), min((c+1)*B, count)).
struct BlockMap {
  uint64_t count = 0, B = 0;
  uint64_t lo(int c) const { uint64_t a = (uint64_t)c * B; return a < count ? a : count; }
  uint64_t hi(int c) const { uint64_t a = (uint64_t)(c + 1) * B; return a < count ? a : count; }
  uint64_t len(int c) const { return hi(c) - lo(c); }
};

inline uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }
// bytes per element of a wire type: fp32 0, bf16 1, fp16 2, int32 3, fp64 4, int64 5, uint8 6
inline size_t elem_size(int dtype) {
  switch (dtype) {
    case 1: case 2: return 2u;
    case 4: case 5: return 8u;
    case 6: return 1u;
    default: return 4u;
  }
}

}  // namespace hcl

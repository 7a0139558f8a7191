// C ABI of libhcl: validation, the ring chunk scheduler and the per-step
// launch plans.  Every step of a collective is a kernel launch on the caller's
// stream; nothing is computed on the host.
#include <hip/hip_runtime_api.h>

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "hcl.h"
#include "internal.h"
#include "reduce_copy.h"
#include "ring_sched.h"

using namespace hcl;

// ---------------------------------------------------------------------------
// errors
// ---------------------------------------------------------------------------
static thread_local char g_err[512] = "";

hcl_status_t hcl::fail(hcl_status_t st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return st;
}

extern "C" const char* hcl_status_string(hcl_status_t s) {
  switch (s) {
    case HCL_OK: return "HCL_OK";
    case HCL_ERR_INVALID_ARG: return "HCL_ERR_INVALID_ARG";
    case HCL_ERR_UNSUPPORTED: return "HCL_ERR_UNSUPPORTED";
    case HCL_ERR_ALIAS: return "HCL_ERR_ALIAS";
    case HCL_ERR_WORKSPACE: return "HCL_ERR_WORKSPACE";
    case HCL_ERR_HIP: return "HCL_ERR_HIP";
  }
  return "HCL_ERR_UNKNOWN";
}
extern "C" const char* hcl_last_error(void) { return g_err; }
extern "C" int hcl_version(void) { return HCL_VERSION; }

// ---------------------------------------------------------------------------
// scheduler (host only)
// ---------------------------------------------------------------------------
bool Ring::init(int W_, const int* ring) {
  if (W_ < 1 || W_ > kMaxRanks) return false;
  W = W_;
  for (int r = 0; r < W; ++r) pos[r] = -1;
  for (int k = 0; k < W; ++k) {
    const int r = ring ? ring[k] : k;
    if (r < 0 || r >= W || pos[r] != -1) return false;
    order[k] = r;
    pos[r] = k;
  }
  return true;
}

extern "C" hcl_status_t hcl_ring_step(int W, const int* ring, int phase, int step, int rank,
                                      int* send_block, int* recv_block) {
  Ring rg;
  if (!rg.init(W, ring)) return fail(HCL_ERR_INVALID_ARG, "W must be in [1,%d] and ring a permutation of 0..W-1", kMaxRanks);
  if (rank < 0 || rank >= W) return fail(HCL_ERR_INVALID_ARG, "rank %d out of range", rank);
  if (step < 0 || step > W - 2) return fail(HCL_ERR_INVALID_ARG, "step %d out of range [0,%d]", step, W - 2);
  if (!send_block || !recv_block) return fail(HCL_ERR_INVALID_ARG, "null output pointer");
  if (phase == HCL_PHASE_RS) {
    *send_block = rg.rs_send(rank, step);
    *recv_block = rg.rs_recv(rank, step);
  } else if (phase == HCL_PHASE_AG) {
    *send_block = rg.ag_send(rank, step);
    *recv_block = rg.ag_recv(rank, step);
  } else {
    return fail(HCL_ERR_INVALID_ARG, "phase must be 0 (reduce-scatter) or 1 (all-gather)");
  }
  return HCL_OK;
}

static bool dtype_ok(int d) { return d >= HCL_FP32 && d <= HCL_UINT8; }

extern "C" hcl_status_t hcl_schedule_items(int W, const int* ring, size_t count, hcl_dtype_t dtype,
                                           size_t chunk_bytes, int phase, int step,
                                           hcl_work_item_t* items, size_t max_items, size_t* n_items) {
  Ring rg;
  if (!rg.init(W, ring)) return fail(HCL_ERR_INVALID_ARG, "W must be in [1,%d] and ring a permutation of 0..W-1", kMaxRanks);
  if (!dtype_ok(dtype)) return fail(HCL_ERR_UNSUPPORTED, "unknown dtype %d", (int)dtype);
  if (phase != HCL_PHASE_RS && phase != HCL_PHASE_AG) return fail(HCL_ERR_INVALID_ARG, "bad phase");
  if (!n_items || (max_items && !items)) return fail(HCL_ERR_INVALID_ARG, "null output pointer");
  const size_t es = elem_size(dtype);
  if (chunk_bytes % es) return fail(HCL_ERR_INVALID_ARG, "chunk_bytes must be a multiple of the element size");
  *n_items = 0;
  if (W == 1 || count == 0) return HCL_OK;
  if (step < 0 || step > W - 2) return fail(HCL_ERR_INVALID_ARG, "step %d out of range [0,%d]", step, W - 2);
  BlockMap bm{count, ceil_div(count, (uint64_t)W)};
  const uint64_t C = chunk_bytes ? chunk_bytes / es : bm.B;
  const uint64_t nchunks = ceil_div(bm.B, C);
  size_t n = 0;
  for (uint64_t j = 0; j < nchunks; ++j) {
    for (int k = 0; k < W; ++k) {
      const int r = rg.order[k];
      const int rb = phase == HCL_PHASE_RS ? rg.rs_recv(r, step) : rg.ag_recv(r, step);
      const int sb = phase == HCL_PHASE_RS ? rg.rs_send(r, step) : rg.ag_send(r, step);
      const uint64_t len = bm.len(rb);
      if (j * C >= len) continue;
      if (n < max_items) {
        hcl_work_item_t& it = items[n];
        it.phase = phase;
        it.step = step;
        it.rank = r;
        it.from_rank = rg.prev(r);
        it.block = rb;
        it.send_block = sb;
        it.chunk = j;
        it.elem_offset = j * C;
        it.elem_count = (len - j * C < C) ? len - j * C : C;
        it.vec_offset = bm.lo(rb) + j * C;
      }
      ++n;
    }
  }
  *n_items = n;
  return HCL_OK;
}

// ---------------------------------------------------------------------------
// device info and measurement helpers
// ---------------------------------------------------------------------------
extern "C" int hcl_device_cu_count(void) {
  static thread_local int cached_dev = -1, cached_cus = -1;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return -1; }
  if (dev != cached_dev) {
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) {
      (void)hipGetLastError();
      return -1;
    }
    cached_dev = dev;
    cached_cus = cus;
  }
  return cached_cus;
}

extern "C" hcl_status_t hcl_events_create(int n, void** out) {
  if (n < 0 || (n && !out)) return fail(HCL_ERR_INVALID_ARG, "bad event array");
  for (int i = 0; i < n; ++i) {
    hipEvent_t e;
    hipError_t rc = hipEventCreate(&e);
    if (rc != hipSuccess) {
      for (int k = 0; k < i; ++k) (void)hipEventDestroy((hipEvent_t)out[k]);
      return fail(HCL_ERR_HIP, "hipEventCreate: %s", hipGetErrorString(rc));
    }
    out[i] = (void*)e;
  }
  return HCL_OK;
}
extern "C" hcl_status_t hcl_events_destroy(int n, void* const* ev) {
  if (n < 0 || (n && !ev)) return fail(HCL_ERR_INVALID_ARG, "bad event array");
  for (int i = 0; i < n; ++i)
    if (ev[i]) (void)hipEventDestroy((hipEvent_t)ev[i]);
  return HCL_OK;
}
extern "C" hcl_status_t hcl_event_record(void* ev, void* stream) {
  if (!ev) return fail(HCL_ERR_INVALID_ARG, "null event");
  hipError_t rc = hipEventRecord((hipEvent_t)ev, (hipStream_t)stream);
  if (rc != hipSuccess) return fail(HCL_ERR_HIP, "hipEventRecord: %s", hipGetErrorString(rc));
  return HCL_OK;
}
extern "C" hcl_status_t hcl_event_elapsed_ms(void* a, void* b, float* ms) {
  if (!a || !b || !ms) return fail(HCL_ERR_INVALID_ARG, "null argument");
  hipError_t rc = hipEventElapsedTime(ms, (hipEvent_t)a, (hipEvent_t)b);
  if (rc != hipSuccess) return fail(HCL_ERR_HIP, "hipEventElapsedTime: %s", hipGetErrorString(rc));
  return HCL_OK;
}

// ---------------------------------------------------------------------------
// call context
// ---------------------------------------------------------------------------
namespace {

struct Range {
  const char* p;
  uint64_t bytes;
  bool overlaps(const Range& o) const {
    if (!bytes || !o.bytes) return false;
    return p < o.p + o.bytes && o.p < p + bytes;
  }
};

uint64_t round_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

int env_int(const char* name, int dflt) {
  const char* v = getenv(name);
  return (v && *v) ? atoi(v) : dflt;
}

// a reducing step whose segments add up to more than this runs one wavefront x 1 vector per workgroup
constexpr uint64_t kSmallTileFrom = 512ull << 20;
// capacity of the memory-side last-level cache (MI355X: 256 MiB)
constexpr uint64_t kLastLevelCache = 256ull << 20;
// how much of one block the one-source fused kernel walks before it moves to the next, for blocks of
// kGatherBigBlock bytes and more
constexpr uint64_t kGatherBigChunk = 64ull << 20;

// The chunk a launch orders its tiles by: about `chunk` elements, but such that n elements make a
// whole number of equal chunks of whole tiles.  A block of 8 chunks and one element would otherwise
// get a ninth row of tiles with one element of work in it (a tenth of the workgroups of every
// launch empty: 4 % of bandwidth on MI355X), and a chunk that is no multiple of the tile would end
// in a partial tile.
uint64_t even_chunk(uint64_t n, uint64_t chunk, uint64_t tile) {
  if (n == 0 || chunk == 0) return chunk;
  uint64_t k = (n + chunk / 2) / chunk;
  if (k == 0) k = 1;
  uint64_t even = round_up(ceil_div(n, k), tile);
  if (even > (tile << 20)) even = round_up(ceil_div(n, k + 1), tile);
  return even;
}

struct Ctx {
  Ring ring;
  int W = 0;
  int dtype = 0;
  uint64_t es = 4;
  uint64_t chunk_elems = 0;  // 0 = one chunk per block
  int sched = 0, xport = 0;
  int op = 0;         // hcl_op_t of the reducing collectives
  bool tree = false;  // FUSED: tree order instead of ring order
  bool wide = false;  // FUSED: binary32 intermediates, one rounding
  bool fuse_rs_ag = false;
  Tuning tune{};
  bool auto_threads = true, auto_unroll = true;  // launch shape left to the library
  bool auto_nt = true;                           // cache policy left to the library
  int max_blocks = 0;
  const hcl_opts_t* opts = nullptr;
  void* stream = nullptr;
  int launches = 0;
  bool phase_events = false;  // events at phase boundaries instead of around every launch
  int phases = 0;
  void* stream2 = nullptr;    // second dependency chain (opts->aux_stream), STEPWISE only
  bool forked = false;        // stream2 currently waits on / runs ahead of `stream`
  int steps_issued = 0;       // step launches so far: odd ones walk their tiles backwards
  uint64_t slab_lo = 0, slab_hi = ~0ull;  // launches cover these elements of every segment only (see for_each_slab)
  uint64_t slab_budget = kLastLevelCache;  // bytes one step may write per slab; ~0 = no slabs
  bool chains_planned = false;
  uint64_t split_elems = 0;   // elements of a segment before this offset: caller's stream; from it on: stream2

  hcl_status_t init(int W_, hcl_dtype_t dt, size_t chunk_bytes, const hcl_opts_t* o, void* st, int op_ = HCL_SUM) {
    opts = o;
    stream = st;
    if (op_ < HCL_SUM || op_ > HCL_MIN) return fail(HCL_ERR_UNSUPPORTED, "unknown reduction operator %d", op_);
    op = op_;
    if (W_ < 1 || W_ > kMaxRanks) return fail(HCL_ERR_INVALID_ARG, "W = %d outside [1,%d]", W_, kMaxRanks);
    if (!ring.init(W_, o ? o->ring : nullptr)) return fail(HCL_ERR_INVALID_ARG, "ring is not a permutation of 0..W-1");
    W = W_;
    if (!dtype_ok(dt)) return fail(HCL_ERR_UNSUPPORTED, "unknown dtype %d", (int)dt);
    dtype = dt;
    es = elem_size(dt);
    if (chunk_bytes % es) return fail(HCL_ERR_INVALID_ARG, "chunk_bytes %zu is not a multiple of the element size %d", chunk_bytes, (int)es);
    chunk_elems = chunk_bytes / es;
    sched = o ? o->sched : 0;
    xport = o ? o->xport : 0;
    if (sched != HCL_SCHED_STEPWISE && sched != HCL_SCHED_FUSED) return fail(HCL_ERR_UNSUPPORTED, "unknown schedule %d", sched);
    if (xport != HCL_XPORT_DIRECT && xport != HCL_XPORT_HOST_STAGED) return fail(HCL_ERR_UNSUPPORTED, "unknown transport %d", xport);
    if (sched == HCL_SCHED_FUSED && xport == HCL_XPORT_HOST_STAGED)
      return fail(HCL_ERR_UNSUPPORTED, "the fused schedule has no staged transport: no block travels between ranks");
    fuse_rs_ag = o && o->fuse_rs_ag;
    const int acc = o ? o->accumulate : 0;
    if (acc != HCL_ACC_PER_HOP && acc != HCL_ACC_FP32) return fail(HCL_ERR_UNSUPPORTED, "unknown accumulate mode %d", acc);
    if (acc == HCL_ACC_FP32 && sched != HCL_SCHED_FUSED)
      return fail(HCL_ERR_UNSUPPORTED, "binary32 accumulation exists for the fused schedule only: in a stepwise ring the partial travels in the wire type");
    wide = acc == HCL_ACC_FP32;
    const int order = o ? o->order : 0;
    if (order != HCL_ORDER_RING && order != HCL_ORDER_TREE) return fail(HCL_ERR_UNSUPPORTED, "unknown order %d", order);
    if (order == HCL_ORDER_TREE && sched != HCL_SCHED_FUSED)
      return fail(HCL_ERR_UNSUPPORTED, "tree order exists for the fused schedule only: a stepwise ring adds in ring order");
    tree = order == HCL_ORDER_TREE;
    if (o && o->n_events < 0) return fail(HCL_ERR_INVALID_ARG, "n_events < 0");
    if (o && o->n_events > 0 && !o->events) return fail(HCL_ERR_INVALID_ARG, "n_events > 0 with null events");
    phase_events = o && o->events_per_phase;
    if (o && o->slab_bytes) slab_budget = o->slab_bytes == (size_t)-1 ? ~0ull : (uint64_t)o->slab_bytes;
    if (xport == HCL_XPORT_HOST_STAGED) slab_budget = ~0ull;  // bound by the host link, and the inbox slots hold whole blocks
    if (o && o->aux_stream) {
      if (sched != HCL_SCHED_STEPWISE) return fail(HCL_ERR_UNSUPPORTED, "aux_stream: the fused schedule is one launch, there is no chain to split");
      if (o->aux_stream == st) return fail(HCL_ERR_INVALID_ARG, "aux_stream must differ from the stream of the call");
      if (!o->aux_events || !o->aux_events[0] || !o->aux_events[1]) return fail(HCL_ERR_INVALID_ARG, "aux_stream needs two events in aux_events");
      stream2 = o->aux_stream;
    }

    int threads = o && o->threads ? o->threads : env_int("HCL_THREADS", 0);
    int unroll = o && o->unroll ? o->unroll : env_int("HCL_UNROLL", 0);
    int blocks = o && o->blocks ? o->blocks : env_int("HCL_BLOCKS", 0);
    int nt = o && o->nontemporal ? o->nontemporal : env_int("HCL_NONTEMPORAL", 0);
    // 0 = not chosen by the caller: the launch picks the default of the kernel it runs
    auto_threads = threads == 0;
    auto_unroll = unroll == 0;
    if (auto_threads) threads = sched == HCL_SCHED_FUSED ? 64 : 128;
    if (auto_unroll) unroll = 2;
    if (threads < 64 || threads > 1024 || threads % 64) return fail(HCL_ERR_INVALID_ARG, "threads = %d must be a multiple of 64 in [64,1024]", threads);
    if (unroll != 1 && unroll != 2 && unroll != 4 && unroll != 8) return fail(HCL_ERR_INVALID_ARG, "unroll = %d must be 1, 2, 4 or 8", unroll);
    if (blocks < 0) return fail(HCL_ERR_INVALID_ARG, "blocks < 0");
    if (nt < -1 || nt > 2) return fail(HCL_ERR_INVALID_ARG, "nontemporal must be -1, 0, 1 or 2");
    tune.threads = threads;
    tune.unroll = unroll;
    auto_nt = nt == 0;
    tune.nt = nt < 0 ? 0 : (nt == 2 ? 1 : 2);  // -1 off; 1 loads and stores; 2 loads, stores written through; 0: by size, see launch()
    max_blocks = blocks;  // 0 = decide at launch from the CU count
    return HCL_OK;
  }

  // Segments (ranks) of a step usually sit at addresses that are congruent
  // modulo a large power of two (equal block offsets in equally aligned
  // buffers).  Walking them at the same offset at the same time cost 3-6 % of
  // bandwidth on MI355X; starting segment d a few tiles further in removes
  // that.  17 tiles measured best among 0..1025 (anything from 5 to 129 was within 0.3 %).
  static uint32_t stagger_for(uint64_t tiles_per_chunk) {
    const int forced = env_int("HCL_STAGGER", -1);  // for sweeps
    if (forced >= 0) return (uint32_t)forced;
    if (tiles_per_chunk > 17) return 17;
    return tiles_per_chunk > 1 ? 1 : 0;
  }

  // Slabs.  Chunk j of a step needs only chunk j of the step before, so the ring can run to
  // completion -- every Reduce-Scatter step, then every All-Gather step -- on one slab of every
  // block before it touches the next slab, which is also how the vendor libraries walk a large
  // buffer.  A slab is as many whole chunks as keep one step's output (all blocks together)
  // within the last-level cache: then every step's incoming operand is still there when the next
  // launch reads it, at any message size.  body(first) issues the steps of one slab.
  template <class F>
  hcl_status_t for_each_slab(uint64_t block_elems, uint64_t blocks_per_step, F body) {
    uint64_t slab = block_elems;
    if (slab_budget != ~0ull) {
      const uint64_t granule = chunk_elems ? chunk_elems : (uint64_t)(1u << 16);
      const uint64_t fit = slab_budget / (blocks_per_step * es);
      slab = fit / granule * granule;
      if (slab == 0) slab = granule;
      if (slab > block_elems) slab = block_elems;
    }
    hcl_status_t st = HCL_OK;
    for (uint64_t lo = 0; lo < block_elems && !st;) {
      // a remainder of less than 1/32 of a slab joins the last slab: a ring of its own over a few
      // elements would cost 2 (W - 1) launches for nothing (blocks of 8 chunks and 64 elements: 4 %)
      uint64_t hi = lo + slab;
      if (hi >= block_elems || block_elems - hi <= slab / 32) hi = block_elems;
      slab_lo = lo;
      slab_hi = hi;
      st = body(lo == 0);
      lo = hi;
    }
    slab_lo = 0;
    slab_hi = ~0ull;
    return st;
  }

  // Default: one tile per workgroup, which measured faster on MI355X than a
  // persistent grid; opts->blocks caps the grid and the kernels then stride.
  // The runtime refuses a launch of 2^32 threads or more, so a larger one
  // strides as well.
  int grid_for(uint32_t total_tiles, int threads) const {
    uint32_t cap = 0xFFFFFFFFu / (uint32_t)(threads > 0 ? threads : 1);
    if (cap > 0x7FFFFFFFu) cap = 0x7FFFFFFFu;
    if (max_blocks && (uint32_t)max_blocks < cap) cap = (uint32_t)max_blocks;
    return (int)(total_tiles < cap ? total_tiles : cap);
  }

  // start of a phase (Reduce-Scatter steps, All-Gather steps, or the single fused launch)
  hcl_status_t phase() {
    if (!phase_events) return HCL_OK;
    return record(phases++);
  }
  hcl_status_t mark(int idx) { return phase_events ? HCL_OK : record(idx); }
  hcl_status_t record(int idx) {
    if (opts && opts->events && idx < opts->n_events) {
      hipError_t rc = hipEventRecord((hipEvent_t)opts->events[idx], (hipStream_t)stream);
      if (rc != hipSuccess) return fail(HCL_ERR_HIP, "hipEventRecord: %s", hipGetErrorString(rc));
    }
    return HCL_OK;
  }

  // Second dependency chain.  The chunks of a step are independent of each other and chunk j
  // of one step needs only chunk j of the step before, so the two halves of the chunk range
  // can run as two chains of launches on two streams: while one chain is between two kernels
  // (the next one is only dispatched when the last wave of the one before has retired) the
  // other chain's kernel has the memory system to itself.
  hcl_status_t fork() {
    if (forked) return HCL_OK;
    hipError_t rc = hipEventRecord((hipEvent_t)opts->aux_events[0], (hipStream_t)stream);
    if (rc == hipSuccess) rc = hipStreamWaitEvent((hipStream_t)stream2, (hipEvent_t)opts->aux_events[0], 0);
    if (rc != hipSuccess) return fail(HCL_ERR_HIP, "fork onto the second stream: %s", hipGetErrorString(rc));
    forked = true;
    return HCL_OK;
  }
  hcl_status_t join() {
    if (!forked) return HCL_OK;
    forked = false;
    hipError_t rc = hipEventRecord((hipEvent_t)opts->aux_events[1], (hipStream_t)stream2);
    if (rc == hipSuccess) rc = hipStreamWaitEvent((hipStream_t)stream, (hipEvent_t)opts->aux_events[1], 0);
    if (rc != hipSuccess) return fail(HCL_ERR_HIP, "join of the second stream: %s", hipGetErrorString(rc));
    return HCL_OK;
  }
  ~Ctx() { (void)join(); }  // an error return between fork and finish() must not leave the streams apart

  // Completes the tile grid of a step and launches it.  Empty steps are skipped.
  // reread: a later launch of the same call reads what this one writes
  hcl_status_t launch(StepArgs& a, int nsrc, int ndst, bool reread) {
    if (a.nseg == 0) return HCL_OK;
    if (a.nseg > (uint32_t)kMaxSegs) return fail(HCL_ERR_INVALID_ARG, "internal: a step with more than %d segments", kMaxSegs);
    uint64_t maxn = 0;
    for (uint32_t i = 0; i < a.nseg; ++i)
      if (a.seg[i].n > maxn) maxn = a.seg[i].n;
    // Which chain an element belongs to must not change during a call: elements before
    // `split_elems` (a whole number of the caller's chunks, about half of the longest block;
    // fixed by the first launch of the call, which always holds a full-length block) go to the
    // caller's stream, the rest to the second one.
    if (!chains_planned) {
      chains_planned = true;
      if (stream2 && chunk_elems && chunk_elems < maxn) split_elems = ceil_div(maxn, chunk_elems) / 2 * chunk_elems;
    }
    a.op = nsrc == 2 ? (uint32_t)op : 0u;
    // Consecutive steps walk their tiles in opposite directions: the end of what one step wrote is
    // what the last-level cache still holds when the next step starts (+1.5 % at 256 MiB per rank,
    // where one step's output is as large as that cache; neutral elsewhere).
    a.reverse = (uint32_t)(steps_issued++ & 1) & (uint32_t)(env_int("HCL_ZIGZAG", 1) != 0);  // the variable: for sweeps
    Tuning t = tune;
    uint64_t step_bytes = 0;  // what this step writes within the slab in progress
    for (uint32_t i = 0; i < a.nseg; ++i) {
      const uint64_t top = a.seg[i].n < slab_hi ? a.seg[i].n : slab_hi;
      if (top > slab_lo) step_bytes += (top - slab_lo) * es;
    }
    // Cache policy.  Loads are non-temporal.  What a step writes is the incoming operand of the
    // next step: while one step's output (all ranks together) fits the 256 MiB last-level cache,
    // it is written through the L2 and the next launch finds it in that cache (on MI355X +7 to +8 %
    // of HBM peak over non-temporal stores at 64 MiB to 1 GiB per rank, +4 to +5 over ordinary
    // stores, whose dirty lines wait in the L2 for the end of the kernel); beyond, and for results
    // no later launch reads, non-temporal stores.  Pinned host memory is always written with
    // non-temporal stores.
    // (a slab may exceed the budget by 1/32, see for_each_slab)
    if (auto_nt) t.nt = (reread && xport == HCL_XPORT_DIRECT && step_bytes <= kLastLevelCache + kLastLevelCache / 32) ? 1 : 2;
    // Launch shape, from sweeps on MI355X: 128 threads x 2 vectors per source for steps that write
    // through (reducing or copying); one wavefront x 1 vector for copies with non-temporal stores
    // (84 % against 70 % of HBM peak) and for reducing steps that write more than 512 MiB, where it
    // measured 2-5 % faster (W = 16 at 1 GiB per rank, 2 GiB blocks as one slab) and far less
    // sensitive to where the buffers lie in memory.
    if (auto_threads && auto_unroll && ((nsrc == 1 && t.nt != 1) || step_bytes > kSmallTileFrom)) {
      t.threads = 64;
      t.unroll = 1;
    }
    // the slab in progress, and within it the two chains' shares
    const uint64_t lo = slab_lo, hi = maxn < slab_hi ? maxn : slab_hi;
    if (lo >= hi) return HCL_OK;
    if (split_elems == 0 || hi <= split_elems) return launch_range(a, nsrc, ndst, t, lo, hi, stream);
    hcl_status_t st = fork();
    if (st) return st;
    if (lo < split_elems && (st = launch_range(a, nsrc, ndst, t, lo, split_elems, stream))) return st;
    return launch_range(a, nsrc, ndst, t, lo > split_elems ? lo : split_elems, hi, stream2);
  }

  // Elements [lo, hi) of every segment of `a`, on stream `on`: as many launches as the tile
  // index of a launch (31 bits) makes necessary, normally one.
  hcl_status_t launch_range(const StepArgs& a, int nsrc, int ndst, const Tuning& t, uint64_t lo, uint64_t hi, void* on) {
    StepArgs b = a;
    b.nseg = 0;
    uint64_t maxn = 0;
    for (uint32_t i = 0; i < a.nseg; ++i) {
      if (a.seg[i].n <= lo) continue;
      Seg s = a.seg[i];
      s.src0 += lo * es;
      if (s.src1) s.src1 += lo * es;
      s.dst0 += lo * es;
      if (s.dst1) s.dst1 += lo * es;
      s.n = (s.n < hi ? s.n : hi) - lo;
      if (s.n > maxn) maxn = s.n;
      b.seg[b.nseg++] = s;
    }
    if (b.nseg == 0) return HCL_OK;
    const uint64_t tile = tile_elems(dtype, t);
    uint64_t chunk = (chunk_elems && chunk_elems < maxn) ? chunk_elems : maxn;
    // a chunk only orders the work: a longer one is walked in pieces of 2^20 tiles, so that any
    // number of chunks can be split over launches of at most 2^31 - 1 tiles each
    if (chunk > (tile << 20)) chunk = tile << 20;
    chunk = even_chunk(maxn, chunk, tile);
    const uint64_t nchunks = ceil_div(maxn, chunk);
    const uint64_t tpc = ceil_div(chunk, tile);
    const uint64_t per_launch = 0x7FFFFFFFull / ((uint64_t)b.nseg * tpc);  // chunks one launch can index: >= 63
    b.chunk = chunk;
    b.tiles_per_chunk = (uint32_t)tpc;
    b.stagger = stagger_for(tpc);
    for (uint64_t c0 = 0; c0 < nchunks; c0 += per_launch) {
      const uint64_t c1 = c0 + per_launch < nchunks ? c0 + per_launch : nchunks;
      hcl_status_t st = launch_chunks(b, nsrc, ndst, t, c0, c1, c0 == 0 && c1 == nchunks, on);
      if (st) return st;
    }
    return HCL_OK;
  }

  // One launch over the chunks [c0, c1) of every segment of `a`.
  hcl_status_t launch_chunks(const StepArgs& a, int nsrc, int ndst, Tuning t, uint64_t c0, uint64_t c1, bool whole,
                             void* on) {
    StepArgs b = a;
    if (!whole) {
      const uint64_t lo = c0 * a.chunk, span = (c1 - c0) * a.chunk;
      b.nseg = 0;
      for (uint32_t i = 0; i < a.nseg; ++i) {
        if (a.seg[i].n <= lo) continue;
        Seg s = a.seg[i];
        s.src0 += lo * es;
        if (s.src1) s.src1 += lo * es;
        s.dst0 += lo * es;
        if (s.dst1) s.dst1 += lo * es;
        s.n = s.n - lo < span ? s.n - lo : span;
        b.seg[b.nseg++] = s;
      }
      if (b.nseg == 0) return HCL_OK;
    }
    b.total_tiles = (uint32_t)((c1 - c0) * b.nseg * b.tiles_per_chunk);
    t.blocks = grid_for(b.total_tiles, t.threads);
    hcl_status_t st = mark(launches);
    if (st) return st;
    int rc = launch_step(b, dtype, nsrc, ndst, t, on);
    if (rc) return fail(HCL_ERR_HIP, "kernel launch failed: %s", hipGetErrorString((hipError_t)rc));
    ++launches;
    return HCL_OK;
  }

  hcl_status_t launch(FusedArgs& a) {
    if (a.count == 0) return HCL_OK;
    const bool one_block = a.mode >= 3;  // Reduce / Broadcast
    const bool copy_mode = a.mode == 2 || a.mode == 4;
    uint64_t chunk = (chunk_elems && chunk_elems < a.B) ? chunk_elems : a.B;
    // The chunk only orders the tiles.  The one-source kernel on blocks of 1 GiB and more measured
    // 3 % faster on MI355X when it walks 64 MiB of a block before it moves to the next block.
    if (copy_mode && a.B * es >= kGatherBigBlock && chunk * es < kGatherBigChunk) chunk = kGatherBigChunk / es;
    Tuning t = tune;
    // the general-form kernel (operator other than the sum, or tree order) is
    // built for small workgroups and one vector per thread and rank
    const bool general = !copy_mode && (op != HCL_SUM || tree);
    if (copy_mode) {
      // the caller's choice if it is one the kernel is built for, else by block size
      const int asked = opts && opts->unroll ? opts->unroll : env_int("HCL_UNROLL", 0);
      t.unroll = (asked == 1 || asked == 2 || asked == 4) ? asked : gather_unroll(a.B * es);
    } else {
      t.unroll = general ? kGenUnroll : fused_unroll(W);
    }
    if (general && t.threads > kGenMaxThreads) t.threads = kGenMaxThreads;
    // Cache policy of the one-launch kernels, from sweeps on MI355X.  Loads are non-temporal.  The
    // one-source kernel writes through the L2 (+1.5 to +5 % of HBM peak from 64 MiB to 4 GiB per
    // rank) except in its four-vector shape for blocks of 1 GiB and more, where non-temporal
    // stores are 9 points ahead.  The reductions write through while everything they write fits
    // the last-level cache (All-Reduce over 8 ranks: +8 points at 16 MiB per rank, +13 at 32 MiB;
    // over 16 ranks +11 at 16 MiB) and with non-temporal stores beyond (written through: -7 to +4
    // at twice the cache, depending on where the buffers lie; -4 to +0.6 further up).
    if (auto_nt) {
      if (copy_mode) {
        t.nt = t.unroll == 4 ? 2 : 1;
      } else {
        const uint64_t written = (a.mode == 0 ? (uint64_t)W : 1) * a.count * es;
        t.nt = written <= kLastLevelCache ? 1 : 2;
      }
    }
    const uint64_t tile = tile_elems(dtype, t);
    chunk = even_chunk(a.B, chunk, tile);
    const uint64_t nchunks = ceil_div(a.B, chunk);
    const uint64_t tpc = ceil_div(chunk, tile);
    const uint64_t total = nchunks * (uint64_t)(one_block ? 1 : W) * tpc;
    if (total > 0x7FFFFFFFull) return fail(HCL_ERR_INVALID_ARG, "collective needs %llu tiles, more than one launch can index", (unsigned long long)total);
    a.chunk = chunk;
    a.tiles_per_chunk = (uint32_t)tpc;
    a.total_tiles = (uint32_t)total;
    a.op = copy_mode ? 0 : (uint8_t)op;
    a.tree = !copy_mode && tree;
    a.wide = !copy_mode && wide;
    t.blocks = grid_for(a.total_tiles, t.threads);
    hcl_status_t st = mark(launches);
    if (st) return st;
    int rc = launch_fused(a, dtype, t, stream);
    if (rc) return fail(HCL_ERR_HIP, "kernel launch failed: %s", hipGetErrorString((hipError_t)rc));
    ++launches;
    return HCL_OK;
  }

  hcl_status_t finish() {
    hcl_status_t st = join();
    if (st) return st;
    if (launches) st = phase_events ? record(phases) : record(launches);
    if (opts && opts->n_launches) *opts->n_launches = launches;
    return st;
  }
};

void add_seg(StepArgs& a, const void* s0, const void* s1, void* d0, void* d1, uint64_t n) {
  if (n == 0) return;
  if (a.nseg >= (uint32_t)kMaxSegs) {  // cannot happen for W <= 16; Ctx::launch refuses such a step
    a.nseg = kMaxSegs + 1;
    return;
  }
  Seg& s = a.seg[a.nseg++];
  s.src0 = (const char*)s0;
  s.src1 = (const char*)s1;
  s.dst0 = (char*)d0;
  s.dst1 = (char*)d1;
  s.n = n;
}

const char* off(const void* p, uint64_t elems, uint64_t es) { return (const char*)p + elems * es; }
char* off(void* p, uint64_t elems, uint64_t es) { return (char*)p + elems * es; }

hcl_status_t check_ptrs(const void* const* send, void* const* recv, int W, uint64_t es) {
  if (!send || !recv) return fail(HCL_ERR_INVALID_ARG, "null send / recv array");
  for (int r = 0; r < W; ++r) {
    if (!send[r] || !recv[r]) return fail(HCL_ERR_INVALID_ARG, "null buffer for rank %d", r);
    if (((uintptr_t)send[r] | (uintptr_t)recv[r]) % es) return fail(HCL_ERR_INVALID_ARG, "buffer of rank %d is not aligned to the element size", r);
  }
  return HCL_OK;
}

// recv buffers must not overlap each other, nor any send buffer unless the pair
// (r, r) is the exact in-place aliasing `inplace_send_of_recv`.
hcl_status_t check_alias(const void* const* send, void* const* recv, int W, uint64_t send_bytes,
                         uint64_t recv_bytes, const Range* extra, int n_extra, bool inplace,
                         bool send_written) {
  for (int r = 0; r < W; ++r) {
    Range rr{(const char*)recv[r], recv_bytes};
    for (int q = 0; q < W; ++q) {
      if (q != r && rr.overlaps(Range{(const char*)recv[q], recv_bytes}))
        return fail(HCL_ERR_ALIAS, "recv buffers of ranks %d and %d overlap", r, q);
      if (!(inplace && q == r) && rr.overlaps(Range{(const char*)send[q], send_bytes}))
        return fail(HCL_ERR_ALIAS, "recv buffer of rank %d overlaps send buffer of rank %d", r, q);
      if (send_written && q != r && Range{(const char*)send[r], send_bytes}.overlaps(Range{(const char*)send[q], send_bytes}))
        return fail(HCL_ERR_ALIAS, "send buffers of ranks %d and %d overlap but are written in place", r, q);
    }
    for (int k = 0; k < n_extra; ++k) {
      if (rr.overlaps(extra[k]) || Range{(const char*)send[r], send_bytes}.overlaps(extra[k]))
        return fail(HCL_ERR_ALIAS, "workspace / staging memory overlaps a buffer of rank %d", r);
    }
  }
  return HCL_OK;
}

// Inboxes in pinned host memory: two slots of one block per rank.
struct Inbox {
  char* base = nullptr;
  uint64_t slot_bytes = 0;
  char* slot(int rank, int parity) const { return base + ((uint64_t)rank * 2 + (parity & 1)) * slot_bytes; }
};

// Slots of the workspace and of the pinned inboxes: one block rounded up to 256 bytes, plus
// 4 KiB.  With slots exactly one power-of-two block apart, the incoming slot, the local block and
// the outgoing slot of a step sit at addresses congruent modulo the block size; on some machines
// (it depends on where the allocation lands physically) that cost the 2 GiB-block Reduce-Scatter
// 4-7 % of bandwidth, and the 4 KiB took it away; where it cost nothing, the pad changed nothing.
constexpr uint64_t kSlotPad = 4096;  // also leaves room for the partial to start up to 127 bytes into its slot
uint64_t slot_bytes_for(uint64_t block_elems, uint64_t es) { return round_up(block_elems * es, 256) + kSlotPad; }

hcl_status_t get_inbox(const Ctx& c, uint64_t block_elems, Inbox& ib) {
  if (c.xport != HCL_XPORT_HOST_STAGED) return HCL_OK;
  ib.slot_bytes = slot_bytes_for(block_elems, c.es);
  const uint64_t need = ib.slot_bytes * 2 * c.W;
  if (!c.opts || !c.opts->host_stage) return fail(HCL_ERR_WORKSPACE, "host-staged transport needs opts->host_stage (%llu bytes)", (unsigned long long)need);
  if (c.opts->host_stage_bytes < need) return fail(HCL_ERR_WORKSPACE, "host_stage has %zu bytes, %llu needed", c.opts->host_stage_bytes, (unsigned long long)need);
  if ((uintptr_t)c.opts->host_stage % 16) return fail(HCL_ERR_INVALID_ARG, "host_stage must be 16-byte aligned");
  ib.base = (char*)c.opts->host_stage;
  return HCL_OK;
}

bool size_overflows(uint64_t count, uint64_t mult, uint64_t es) {
  if (count == 0) return false;
  const uint64_t lim = (uint64_t)1 << 62;
  return count > lim / es / (mult ? mult : 1);
}

}  // namespace

// ---------------------------------------------------------------------------
// HCL_DEBUG=1: the call and the work items of its schedule, on stderr
// ---------------------------------------------------------------------------
static bool debug_on() {
  const char* v = getenv("HCL_DEBUG");
  return v && *v && *v != '0';
}

// `vec_count`: elements of the full vector the block map cuts (All-Reduce: count; Reduce-Scatter /
// All-Gather: W * count).  rs / ag: which phases the call runs; ag_first: its first All-Gather step.
static void debug_call(const char* name, const Ctx& c, uint64_t vec_count, size_t chunk_bytes, bool rs, bool ag,
                       int ag_first) {
  static const char* const dt[] = {"fp32", "bf16", "fp16", "int32", "fp64", "int64", "uint8"};
  static const char* const ops[] = {"sum", "prod", "max", "min"};
  char ring[8 * kMaxRanks] = "";
  int ring_i[kMaxRanks];
  for (int k = 0, at = 0; k < c.W; ++k) {
    ring_i[k] = c.ring.order[k];
    at += snprintf(ring + at, sizeof ring - at, k ? " %d" : "%d", ring_i[k]);
  }
  fprintf(stderr, "hcl: %s W=%d elements=%llu dtype=%s op=%s chunk_bytes=%zu sched=%s xport=%s%s%s ring=[%s]\n", name, c.W,
          (unsigned long long)vec_count, dt[c.dtype], ops[c.op], chunk_bytes, c.sched == HCL_SCHED_FUSED ? "fused" : "stepwise",
          c.xport == HCL_XPORT_HOST_STAGED ? "host_staged" : "direct", c.fuse_rs_ag ? " fuse_rs_ag" : "",
          c.stream2 ? " two_chains" : "", ring);
  if (c.W < 2 || c.sched != HCL_SCHED_STEPWISE) return;
  const size_t cap = (size_t)env_int("HCL_DEBUG_ITEMS", 64);  // items printed per step
  hcl_work_item_t* items = (hcl_work_item_t*)malloc((cap ? cap : 1) * sizeof(hcl_work_item_t));
  if (!items) return;
  for (int phase = 0; phase < 2; ++phase) {
    if (!(phase == HCL_PHASE_RS ? rs : ag)) continue;
    for (int s = phase == HCL_PHASE_AG ? ag_first : 0; s <= c.W - 2; ++s) {
      size_t n = 0;
      if (hcl_schedule_items(c.W, ring_i, vec_count, (hcl_dtype_t)c.dtype, chunk_bytes, phase, s, items, cap, &n) != HCL_OK) break;
      fprintf(stderr, "hcl:  %s step %d: %zu work items\n", phase == HCL_PHASE_RS ? "reduce-scatter" : "all-gather", s, n);
      for (size_t i = 0; i < n && i < cap; ++i) {
        const hcl_work_item_t& it = items[i];
        fprintf(stderr, "hcl:   rank %d <- rank %d: block %d chunk %llu, elements [%llu, %llu) of the vector%s; passes on block %d\n",
                it.rank, it.from_rank, it.block, (unsigned long long)it.chunk, (unsigned long long)it.vec_offset,
                (unsigned long long)(it.vec_offset + it.elem_count), phase == HCL_PHASE_RS ? ", reduced" : ", copied", it.send_block);
      }
      if (n > cap) fprintf(stderr, "hcl:   ... and %zu more\n", n - cap);
    }
  }
  free(items);
}

// ---------------------------------------------------------------------------
// workspace queries
// ---------------------------------------------------------------------------
extern "C" size_t hcl_workspace_bytes(int kind, int W, size_t count, hcl_dtype_t dtype, size_t chunk_bytes,
                                      const hcl_opts_t* opts) {
  (void)chunk_bytes;
  if (W < 1 || W > kMaxRanks || !dtype_ok(dtype)) return 0;
  const int sched = opts ? opts->sched : 0, xport = opts ? opts->xport : 0;
  if (sched != HCL_SCHED_STEPWISE || xport != HCL_XPORT_DIRECT || W <= 2) return 0;
  if (size_overflows(count, 2 * (uint64_t)W, elem_size(dtype))) return 0;
  if (kind == HCL_KIND_REDUCE) return (size_t)slot_bytes_for(count, elem_size(dtype));
  if (kind != HCL_KIND_REDUCE_SCATTER) return 0;
  return (size_t)(slot_bytes_for(count, elem_size(dtype)) * W);
}

extern "C" size_t hcl_host_stage_bytes(int kind, int W, size_t count, hcl_dtype_t dtype, size_t chunk_bytes,
                                       const hcl_opts_t* opts) {
  (void)chunk_bytes;
  if (W < 1 || W > kMaxRanks || !dtype_ok(dtype)) return 0;
  if (!opts || opts->xport != HCL_XPORT_HOST_STAGED) return 0;
  uint64_t B = count;
  if (kind == HCL_KIND_ALLREDUCE) B = ceil_div(count, (uint64_t)W);
  if (size_overflows(B, 2 * (uint64_t)W, elem_size(dtype))) return 0;
  return (size_t)(slot_bytes_for(B, elem_size(dtype)) * 2 * W);
}

// ---------------------------------------------------------------------------
// the three collectives
// ---------------------------------------------------------------------------

// Reduce-Scatter steps 0..W-2 over the block map `bm`.
//   own[r]   : where rank r's own data of a block is read from
//   part[r]  : full-vector buffer where rank r keeps its partial sums (DIRECT)
//   first[r] : full-vector buffer the successor reads rank r's block from at step 0
//   fin[r]   : where rank r's finished block r goes (already offset to the block)
//   push[r]  : non-null: the finished block r is also stored there (next rank's buffer, offset)
//   final_reread : the finished blocks are read again by the same call (the All-Gather phase of an All-Reduce)
//   ws       : non-null (with ws_slot bytes per slot): the travelling partial sum of block b lives in
//              workspace slot b from the step that first forms it to the last but one -- every step
//              reads it there, combines the rank's own block and writes it back to the same
//              addresses (the block is handled by exactly one rank per step), which keeps a step at
//              two read streams plus a write into lines just read, as in place; part[] is unused
static hcl_status_t run_rs(Ctx& c, const BlockMap& bm, const void* const* own, char* const* part,
                           const void* const* first, char* const* fin, char* const* push,
                           char* ws, uint64_t ws_slot, const Inbox& ib, bool forward_last, bool final_reread) {
  const int W = c.W;
  const uint64_t es = c.es;
  const bool staged = c.xport == HCL_XPORT_HOST_STAGED;
  hcl_status_t st;
  if (staged) {
    // every rank puts the block it sends first into its successor's inbox
    StepArgs a{};
    for (int k = 0; k < W; ++k) {
      const int r = c.ring.order[k], sb = c.ring.rs_send(r, 0);
      add_seg(a, off(first[r], bm.lo(sb), es), nullptr, ib.slot(c.ring.next(r), 0), nullptr, bm.len(sb));
    }
    if ((st = c.launch(a, 1, 1, true))) return st;
  }
  for (int s = 0; s <= W - 2; ++s) {
    const bool last = s == W - 2;
    StepArgs a{};
    int ndst = 1;
    for (int k = 0; k < W; ++k) {
      const int r = c.ring.order[k], p = c.ring.prev(r), b = c.ring.rs_recv(r, s);
      const uint64_t lo = bm.lo(b), n = bm.len(b);
      const char* local = off(own[r], lo, es);
      if (staged) {
        const char* in = ib.slot(r, s);
        char* fwd = ib.slot(c.ring.next(r), s + 1);
        if (!last) {
          add_seg(a, in, local, fwd, nullptr, n);  // the partial only travels on
        } else if (forward_last) {
          add_seg(a, in, local, fin[r], fwd, n);
          ndst = 2;
        } else {
          add_seg(a, in, local, fin[r], nullptr, n);
        }
      } else {
        // inside its slot the partial starts at the block's own offset modulo 128 bytes, so that
        // it is congruent with the local operands (the kernels align on 128-byte lines)
        char* slot = ws ? ws + (uint64_t)b * ws_slot + ((uintptr_t)off(own[c.ring.order[0]], lo, es) & 127) : nullptr;
        const char* in;
        if (s == 0) in = off(first[p], lo, es);
        else if (ws) in = slot;
        else in = off(part[p], lo, es);
        char* out;
        if (last) out = fin[r];
        else if (ws) out = slot;
        else out = off(part[r], lo, es);
        if (last && push) {
          add_seg(a, in, local, out, push[r], n);
          ndst = 2;
        } else {
          add_seg(a, in, local, out, nullptr, n);
        }
      }
    }
    if ((st = c.launch(a, 2, ndst, !last || final_reread))) return st;
  }
  return HCL_OK;
}

// All-Gather steps first_step..W-2 over `bm`; buf[r] is rank r's full vector.
// src0[r] non-null: at step 0 the successor of r reads r's block from there
// instead of buf[r] (out-of-place All-Gather).  parity0: inbox slot parity the
// block of step 0 arrives in.
static hcl_status_t run_ag(Ctx& c, const BlockMap& bm, char* const* buf, const void* const* src0,
                           int first_step, const Inbox& ib, int parity0) {
  const int W = c.W;
  const uint64_t es = c.es;
  const bool staged = c.xport == HCL_XPORT_HOST_STAGED;
  hcl_status_t st;
  for (int s = first_step; s <= W - 2; ++s) {
    const bool last = s == W - 2;
    StepArgs a{};
    int ndst = 1;
    for (int k = 0; k < W; ++k) {
      const int r = c.ring.order[k], p = c.ring.prev(r), g = c.ring.ag_recv(r, s);
      const uint64_t lo = bm.lo(g), n = bm.len(g);
      char* out = off(buf[r], lo, es);
      if (staged) {
        const char* in = ib.slot(r, parity0 + s);
        if (!last) {
          add_seg(a, in, nullptr, out, ib.slot(c.ring.next(r), parity0 + s + 1), n);
          ndst = 2;
        } else {
          add_seg(a, in, nullptr, out, nullptr, n);
        }
      } else {
        const char* in = (s == 0 && src0) ? (const char*)src0[p] : off(buf[p], lo, es);
        add_seg(a, in, nullptr, out, nullptr, n);
      }
    }
    if ((st = c.launch(a, 1, ndst, !last))) return st;
  }
  return HCL_OK;
}

static void fill_fused(const Ctx& c, FusedArgs& f, const void* const* send, void* const* recv,
                       uint64_t count, uint64_t B, int mode, int root = 0) {
  memset(&f, 0, sizeof f);
  f.root = (uint32_t)root;
  for (int r = 0; r < c.W; ++r) {
    f.src[r] = send ? (const char*)send[r] : nullptr;
    f.dst[r] = recv ? (char*)recv[r] : nullptr;
    f.order[r] = (uint8_t)c.ring.order[r];
    f.pos[r] = (uint8_t)c.ring.pos[r];
  }
  f.count = count;
  f.B = B;
  f.W = (uint32_t)c.W;
  f.mode = (uint32_t)mode;
}

// plain copies send[r] -> recv[r] of n elements each, one launch
static hcl_status_t copy_all(Ctx& c, const void* const* send, void* const* recv, uint64_t n) {
  StepArgs a{};
  for (int r = 0; r < c.W; ++r)
    if (send[r] != recv[r]) add_seg(a, send[r], nullptr, recv[r], nullptr, n);
  return c.launch(a, 1, 1, false);
}

extern "C" hcl_status_t hcl_allreduce_sim(const void* const* send, void* const* recv, int W, size_t count,
                                          hcl_dtype_t dtype, hcl_op_t op, size_t chunk_bytes,
                                          const hcl_opts_t* opts, void* stream) {
  Ctx c;
  hcl_status_t st = c.init(W, dtype, chunk_bytes, opts, stream, op);
  if (st) return st;
  if (size_overflows(count, 1, c.es)) return fail(HCL_ERR_INVALID_ARG, "count overflows");
  if (count == 0) return c.finish();
  if ((st = check_ptrs(send, recv, W, c.es))) return st;
  int same = 0;
  for (int r = 0; r < W; ++r) same += send[r] == recv[r];
  if (same != 0 && same != W) return fail(HCL_ERR_ALIAS, "in-place All-Reduce needs recv[r] == send[r] for every rank");
  const bool inplace = same == W;
  const uint64_t bytes = count * c.es;
  const BlockMap bm{count, ceil_div(count, (uint64_t)W)};
  Inbox ib;
  if ((st = get_inbox(c, bm.B, ib))) return st;
  Range extra[1] = {{ib.base, ib.slot_bytes * 2 * W}};
  if ((st = check_alias(send, recv, W, bytes, bytes, extra, ib.base ? 1 : 0, inplace, false))) return st;

  if (debug_on()) debug_call("all-reduce", c, count, chunk_bytes, true, true, (c.fuse_rs_ag && c.xport == HCL_XPORT_DIRECT) ? 1 : 0);
  if (W == 1) {
    if ((st = c.phase())) return st;
    if ((st = copy_all(c, send, recv, count))) return st;
    return c.finish();
  }
  if (c.sched == HCL_SCHED_FUSED) {
    FusedArgs f;
    fill_fused(c, f, send, recv, count, bm.B, 0);
    if ((st = c.phase())) return st;
    if ((st = c.launch(f))) return st;
    return c.finish();
  }
  char* part[kMaxRanks];
  char* fin[kMaxRanks];
  char* push[kMaxRanks];
  const bool staged = c.xport == HCL_XPORT_HOST_STAGED;
  const bool fuse = c.fuse_rs_ag && !staged;
  for (int r = 0; r < W; ++r) {
    part[r] = (char*)recv[r];
    fin[r] = off(recv[r], bm.lo(r), c.es);
    push[r] = off(recv[c.ring.next(r)], bm.lo(r), c.es);
  }
  st = c.for_each_slab(bm.B, (uint64_t)W, [&](bool first) -> hcl_status_t {
    hcl_status_t s2;
    if (first && (s2 = c.phase())) return s2;
    if ((s2 = run_rs(c, bm, send, part, send, fin, fuse ? push : nullptr, nullptr, 0, ib, /*forward_last=*/true, /*final_reread=*/true))) return s2;
    if (first && (s2 = c.phase())) return s2;
    return run_ag(c, bm, part, nullptr, fuse ? 1 : 0, ib, W - 1);
  });
  if (st) return st;
  return c.finish();
}

extern "C" hcl_status_t hcl_reduce_scatter_sim(const void* const* send, void* const* recv, int W, size_t recvcount,
                                               hcl_dtype_t dtype, hcl_op_t op, size_t chunk_bytes,
                                               const hcl_opts_t* opts, void* stream) {
  Ctx c;
  hcl_status_t st = c.init(W, dtype, chunk_bytes, opts, stream, op);
  if (st) return st;
  if (size_overflows(recvcount, (uint64_t)W, c.es)) return fail(HCL_ERR_INVALID_ARG, "count overflows");
  if (recvcount == 0) return c.finish();
  if ((st = check_ptrs(send, recv, W, c.es))) return st;
  const uint64_t n = recvcount, es = c.es;
  int same = 0;
  for (int r = 0; r < W; ++r) same += (const char*)recv[r] == off(send[r], (uint64_t)r * n, es);
  if (same != 0 && same != W) return fail(HCL_ERR_ALIAS, "in-place Reduce-Scatter needs recv[r] == send[r] + r * recvcount for every rank");
  const bool inplace = same == W;
  const BlockMap bm{n * W, n};
  Inbox ib;
  if ((st = get_inbox(c, n, ib))) return st;
  const bool stepwise_direct = c.sched == HCL_SCHED_STEPWISE && c.xport == HCL_XPORT_DIRECT;
  char* ws = nullptr;
  uint64_t ws_slot = 0, ws_need = 0;
  if (!inplace && stepwise_direct && W > 2) {
    ws_slot = slot_bytes_for(n, es);
    ws_need = ws_slot * W;
    if (!opts || !opts->workspace) return fail(HCL_ERR_WORKSPACE, "out-of-place stepwise Reduce-Scatter needs opts->workspace (%llu bytes)", (unsigned long long)ws_need);
    if (opts->workspace_bytes < ws_need) return fail(HCL_ERR_WORKSPACE, "workspace has %zu bytes, %llu needed", opts->workspace_bytes, (unsigned long long)ws_need);
    if ((uintptr_t)opts->workspace % 16) return fail(HCL_ERR_INVALID_ARG, "workspace must be 16-byte aligned");
    ws = (char*)opts->workspace;
  }
  Range extra[2] = {{ib.base, ib.slot_bytes * 2 * W}, {ws, ws_need}};
  // a staged in-place ring never writes partials into send[], a direct one does
  if ((st = check_alias(send, recv, W, n * W * es, n * es, extra, 2, inplace, inplace && stepwise_direct))) return st;

  if (debug_on()) debug_call("reduce-scatter", c, n * W, chunk_bytes, true, false, 0);
  if (W == 1) {
    if ((st = c.phase())) return st;
    if ((st = copy_all(c, send, recv, n))) return st;
    return c.finish();
  }
  if (c.sched == HCL_SCHED_FUSED) {
    FusedArgs f;
    fill_fused(c, f, send, recv, n * W, n, 1);
    if ((st = c.phase())) return st;
    if ((st = c.launch(f))) return st;
    return c.finish();
  }
  char* part[kMaxRanks];
  char* fin[kMaxRanks];
  for (int r = 0; r < W; ++r) {
    part[r] = inplace ? (char*)const_cast<void*>(send[r]) : nullptr;  // unused when ws or staged
    fin[r] = (char*)recv[r];
  }
  if ((st = c.phase())) return st;
  st = c.for_each_slab(n, (uint64_t)W, [&](bool) -> hcl_status_t {
    return run_rs(c, bm, send, part, send, fin, nullptr, ws, ws_slot, ib, /*forward_last=*/false, /*final_reread=*/false);
  });
  if (st) return st;
  return c.finish();
}

extern "C" hcl_status_t hcl_all_gather_sim(const void* const* send, void* const* recv, int W, size_t sendcount,
                                           hcl_dtype_t dtype, size_t chunk_bytes,
                                           const hcl_opts_t* opts, void* stream) {
  Ctx c;
  hcl_status_t st = c.init(W, dtype, chunk_bytes, opts, stream);
  if (st) return st;
  if (size_overflows(sendcount, (uint64_t)W, c.es)) return fail(HCL_ERR_INVALID_ARG, "count overflows");
  if (sendcount == 0) return c.finish();
  if ((st = check_ptrs(send, recv, W, c.es))) return st;
  const uint64_t n = sendcount, es = c.es;
  int same = 0;
  for (int r = 0; r < W; ++r) same += (const char*)send[r] == off((const void*)recv[r], (uint64_t)r * n, es);
  if (same != 0 && same != W) return fail(HCL_ERR_ALIAS, "in-place All-Gather needs send[r] == recv[r] + r * sendcount for every rank");
  const bool inplace = same == W;
  const BlockMap bm{n * W, n};
  Inbox ib;
  if ((st = get_inbox(c, n, ib))) return st;
  Range extra[1] = {{ib.base, ib.slot_bytes * 2 * W}};
  if ((st = check_alias(send, recv, W, n * es, n * W * es, extra, 1, inplace, false))) return st;

  if (debug_on()) debug_call("all-gather", c, n * W, chunk_bytes, false, true, 0);
  if (c.sched == HCL_SCHED_FUSED) {
    FusedArgs f;
    fill_fused(c, f, send, recv, n * W, n, 2);
    if ((st = c.phase())) return st;
    if ((st = c.launch(f))) return st;
    return c.finish();
  }
  char* buf[kMaxRanks];
  for (int r = 0; r < W; ++r) buf[r] = (char*)recv[r];
  const bool staged = c.xport == HCL_XPORT_HOST_STAGED;
  if ((st = c.phase())) return st;
  st = c.for_each_slab(n, (uint64_t)W, [&](bool) -> hcl_status_t {
    hcl_status_t s2;
    if (staged && W > 1) {
      // every rank puts its own block into its successor's inbox (and, out of
      // place, into its own result)
      StepArgs a{};
      for (int k = 0; k < W; ++k) {
        const int r = c.ring.order[k];
        add_seg(a, send[r], nullptr, ib.slot(c.ring.next(r), 0), inplace ? nullptr : off(recv[r], bm.lo(r), es), n);
      }
      if ((s2 = c.launch(a, 1, inplace ? 1 : 2, true))) return s2;
    } else if (!inplace) {
      // own block into own result
      StepArgs a{};
      for (int r = 0; r < W; ++r) add_seg(a, send[r], nullptr, off(recv[r], bm.lo(r), es), nullptr, n);
      if ((s2 = c.launch(a, 1, 1, false))) return s2;
    }
    if (W > 1) return run_ag(c, bm, buf, (inplace || staged) ? nullptr : send, 0, ib, 0);
    return HCL_OK;
  });
  if (st) return st;
  return c.finish();
}


// ---------------------------------------------------------------------------
// Reduce, Broadcast, All-to-All: the other collectives the paper evaluates
// (Appendix E.1 "Other Collective Communication Operations"), on the same kernels
// ---------------------------------------------------------------------------
static hcl_status_t only_direct(const Ctx& c, const char* what) {
  if (c.xport != HCL_XPORT_DIRECT) return fail(HCL_ERR_UNSUPPORTED, "%s has no staged transport", what);
  return HCL_OK;
}

extern "C" hcl_status_t hcl_reduce_sim(const void* const* send, void* const* recv, int W, size_t count,
                                       hcl_dtype_t dtype, hcl_op_t op, int root, size_t chunk_bytes,
                                       const hcl_opts_t* opts, void* stream) {
  Ctx c;
  hcl_status_t st = c.init(W, dtype, chunk_bytes, opts, stream, op);
  if (st) return st;
  if ((st = only_direct(c, "Reduce"))) return st;
  if (root < 0 || root >= W) return fail(HCL_ERR_INVALID_ARG, "root %d out of range", root);
  if (size_overflows(count, 1, c.es)) return fail(HCL_ERR_INVALID_ARG, "count overflows");
  if (count == 0) return c.finish();
  if (!send || !recv || !recv[root]) return fail(HCL_ERR_INVALID_ARG, "null send array or null recv[root]");
  for (int r = 0; r < W; ++r) {
    if (!send[r]) return fail(HCL_ERR_INVALID_ARG, "null send buffer for rank %d", r);
    if ((uintptr_t)send[r] % c.es) return fail(HCL_ERR_INVALID_ARG, "send buffer of rank %d is not aligned to the element size", r);
  }
  if ((uintptr_t)recv[root] % c.es) return fail(HCL_ERR_INVALID_ARG, "recv[root] is not aligned to the element size");
  const uint64_t es = c.es, bytes = count * es;
  char* ws = nullptr;
  uint64_t slot = 0, need = 0;
  if (c.sched == HCL_SCHED_STEPWISE && W > 2) {
    slot = slot_bytes_for(count, es);
    need = slot;
    if (!opts || !opts->workspace) return fail(HCL_ERR_WORKSPACE, "stepwise Reduce needs opts->workspace (%llu bytes)", (unsigned long long)need);
    if (opts->workspace_bytes < need) return fail(HCL_ERR_WORKSPACE, "workspace has %zu bytes, %llu needed", opts->workspace_bytes, (unsigned long long)need);
    if ((uintptr_t)opts->workspace % 16) return fail(HCL_ERR_INVALID_ARG, "workspace must be 16-byte aligned");
    ws = (char*)opts->workspace;
  }
  const Range out{(const char*)recv[root], bytes}, wsr{ws, need};
  for (int r = 0; r < W; ++r) {
    const Range in{(const char*)send[r], bytes};
    if (!(r == root && send[r] == recv[root]) && out.overlaps(in)) return fail(HCL_ERR_ALIAS, "recv[root] overlaps the send buffer of rank %d", r);
    if (wsr.overlaps(in)) return fail(HCL_ERR_ALIAS, "workspace overlaps the send buffer of rank %d", r);
  }
  if (wsr.overlaps(out)) return fail(HCL_ERR_ALIAS, "workspace overlaps recv[root]");

  if ((st = c.phase())) return st;
  if (W == 1) {
    StepArgs a{};
    if (send[0] != recv[0]) add_seg(a, send[0], nullptr, recv[0], nullptr, count);
    if ((st = c.launch(a, 1, 1, false))) return st;
    return c.finish();
  }
  if (c.sched == HCL_SCHED_FUSED) {
    FusedArgs f;
    fill_fused(c, f, send, recv, count, count, 3, root);
    for (int r = 0; r < W; ++r)
      if (r != root) f.dst[r] = nullptr;
    if ((st = c.launch(f))) return st;
    return c.finish();
  }
  // hop k (1 .. W-1): the k-th rank after the first sender adds its vector to what arrived
  const int p0 = c.ring.pos[root];
  st = c.for_each_slab(count, 1, [&](bool) -> hcl_status_t {
    for (int k = 1; k <= W - 1; ++k) {
      const int r = c.ring.at(p0 + 1 + k), p = c.ring.at(p0 + k);
      // the travelling partial sum stays in the one workspace slot: read, combined, written back
      // (at the senders' offset modulo 128 bytes, so that it is congruent with them)
      char* slot_p = ws + ((uintptr_t)send[c.ring.order[0]] & 127);
      const char* in = k == 1 ? (const char*)send[p] : slot_p;
      char* out_p = k == W - 1 ? (char*)recv[root] : slot_p;
      StepArgs a{};
      add_seg(a, in, send[r], out_p, nullptr, count);
      hcl_status_t s2 = c.launch(a, 2, 1, k < W - 1);
      if (s2) return s2;
    }
    return HCL_OK;
  });
  if (st) return st;
  return c.finish();
}

extern "C" hcl_status_t hcl_broadcast_sim(const void* const* send, void* const* recv, int W, size_t count,
                                          hcl_dtype_t dtype, int root, size_t chunk_bytes,
                                          const hcl_opts_t* opts, void* stream) {
  Ctx c;
  hcl_status_t st = c.init(W, dtype, chunk_bytes, opts, stream);
  if (st) return st;
  if ((st = only_direct(c, "Broadcast"))) return st;
  if (root < 0 || root >= W) return fail(HCL_ERR_INVALID_ARG, "root %d out of range", root);
  if (size_overflows(count, 1, c.es)) return fail(HCL_ERR_INVALID_ARG, "count overflows");
  if (count == 0) return c.finish();
  if (!send || !recv || !send[root]) return fail(HCL_ERR_INVALID_ARG, "null recv array or null send[root]");
  if ((uintptr_t)send[root] % c.es) return fail(HCL_ERR_INVALID_ARG, "send[root] is not aligned to the element size");
  const uint64_t bytes = count * c.es;
  const Range in{(const char*)send[root], bytes};
  for (int r = 0; r < W; ++r) {
    if (!recv[r]) return fail(HCL_ERR_INVALID_ARG, "null recv buffer for rank %d", r);
    if ((uintptr_t)recv[r] % c.es) return fail(HCL_ERR_INVALID_ARG, "recv buffer of rank %d is not aligned to the element size", r);
    const Range o{(const char*)recv[r], bytes};
    if (!(r == root && recv[r] == send[root]) && o.overlaps(in)) return fail(HCL_ERR_ALIAS, "recv buffer of rank %d overlaps send[root]", r);
    for (int q = 0; q < r; ++q)
      if (o.overlaps(Range{(const char*)recv[q], bytes})) return fail(HCL_ERR_ALIAS, "recv buffers of ranks %d and %d overlap", q, r);
  }
  if ((st = c.phase())) return st;
  if (c.sched == HCL_SCHED_FUSED) {
    FusedArgs f;
    fill_fused(c, f, nullptr, recv, count, count, 4, root);
    f.src[root] = (const char*)send[root];
    if ((st = c.launch(f))) return st;
    return c.finish();
  }
  // hop k: the k-th rank after the root copies what its predecessor holds; the
  // first launch also puts the root's vector into its own result when out of place
  const int p0 = c.ring.pos[root];
  st = c.for_each_slab(count, 1, [&](bool) -> hcl_status_t {
    bool own_done = send[root] == recv[root];
    for (int k = 1; k <= W - 1 || !own_done; ++k) {
      StepArgs a{};
      if (!own_done) {
        add_seg(a, send[root], nullptr, recv[root], nullptr, count);
        own_done = true;
      }
      if (k <= W - 1) {
        const int r = c.ring.at(p0 + k), p = c.ring.at(p0 + k - 1);
        add_seg(a, k == 1 ? send[root] : (const void*)recv[p], nullptr, recv[r], nullptr, count);
      }
      hcl_status_t s2 = c.launch(a, 1, 1, k < W - 1);
      if (s2) return s2;
    }
    return HCL_OK;
  });
  if (st) return st;
  return c.finish();
}

extern "C" hcl_status_t hcl_alltoall_sim(const void* const* send, void* const* recv, int W, size_t count,
                                         hcl_dtype_t dtype, size_t chunk_bytes,
                                         const hcl_opts_t* opts, void* stream) {
  Ctx c;
  hcl_status_t st = c.init(W, dtype, chunk_bytes, opts, stream);
  if (st) return st;
  if ((st = only_direct(c, "All-to-All"))) return st;
  if (size_overflows(count, (uint64_t)W, c.es)) return fail(HCL_ERR_INVALID_ARG, "count overflows");
  if (count == 0) return c.finish();
  if ((st = check_ptrs(send, recv, W, c.es))) return st;
  const uint64_t n = count, es = c.es, bytes = n * W * es;
  if ((st = check_alias(send, recv, W, bytes, bytes, nullptr, 0, /*inplace=*/false, false))) return st;
  if ((st = c.phase())) return st;
  // exchange k: every rank receives the block addressed to it from the rank k places
  // before it in the ring (k = 0: its own block).  STEPWISE: one launch per exchange;
  // FUSED: as many exchanges per launch as the launch's segment table holds.
  const int per_launch = c.sched == HCL_SCHED_FUSED ? kMaxSegs / W : 1;
  for (int k0 = 0; k0 < W; k0 += per_launch) {
    StepArgs a{};
    for (int k = k0; k < k0 + per_launch && k < W; ++k) {
      for (int i = 0; i < W; ++i) {
        const int r = c.ring.order[i], q = c.ring.at(i - k);
        add_seg(a, off(send[q], (uint64_t)r * n, es), nullptr, off(recv[r], (uint64_t)q * n, es), nullptr, n);
      }
    }
    if ((st = c.launch(a, 1, 1, false))) return st;
  }
  return c.finish();
}

// TEST INFRASTRUCTURE: the host side of the library (hcl_api.cpp) built with g++
// against recording stand-ins for the HIP runtime and the kernel launchers
// (hip_stub.cpp), meant to run under AddressSanitizer and UBSan.
//
// The recorded launch plans are executed on SYMBOLIC memory: every element of a
// rank buffer is a (which vector element, which ranks entered, in which order)
// value, a reducing segment appends the local operand's ranks to the incoming
// ones, a copying segment moves the value.  That checks, without a GPU and for
// any pointer values, that
//   - every address a launch touches lies inside a buffer the caller passed,
//   - no launch reads what another segment of the same launch writes,
//   - with two streams, nothing is touched by both chains between fork and join,
//   - the finished buffers hold exactly the ring's result: block c reduced in the
//     order next(c), ..., c, every block gathered to every rank,
//   - launches never index more than 2^31 - 1 tiles and their grids are
//     consistent with the tile decomposition the kernels use.
//
// usage: host_check            run every check, print "host_check: ok"
//        host_check dump       one small All-Reduce with HCL_DEBUG=1 (stderr shows the work items)
#include <algorithm>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <random>
#include <string>
#include <vector>

#include "hcl.h"
#include "reduce_copy.h"
#include "ring_sched.h"
#include "shim.h"

using hcl::ceil_div;

static int g_fail = 0;
static std::string g_case;
static void bad(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  fprintf(stderr, "host_check FAILED [%s]: ", g_case.c_str());
  vfprintf(stderr, fmt, ap);
  fprintf(stderr, "\n");
  va_end(ap);
  if (++g_fail > 20) exit(1);
}

// ---------------------------------------------------------------------------
// symbolic memory
// ---------------------------------------------------------------------------
struct Sym {
  int64_t idx = -1;   // which element of the collective's vector; -1 = never written
  uint8_t len = 0;    // ranks that entered, in order
  uint8_t seq[16] = {};
  int8_t w_stream = -1;  // 0 caller's stream, 1 second stream
  int w_epoch = -1, r_epoch[2] = {-1, -1};
};
struct Buf {
  std::string name;
  uintptr_t base;
  uint64_t es, n;
  std::vector<Sym> e;
};
struct Mem {
  std::vector<Buf> bufs;
  uintptr_t next = 0x100000000000ull;  // made-up addresses, never dereferenced
  int add(const std::string& name, uint64_t n, uint64_t es, uint64_t misalign_elems = 0) {
    Buf b{name, next + misalign_elems * es, es, n, std::vector<Sym>(n)};
    next += ((n + misalign_elems) * es + 4096 + 0xFFFF) & ~0xFFFFull;
    bufs.push_back(b);
    return (int)bufs.size() - 1;
  }
  Sym* at(const char* p, uint64_t es) {
    const uintptr_t a = (uintptr_t)p;
    for (Buf& b : bufs)
      if (a >= b.base && a + es <= b.base + b.n * b.es) {
        if ((a - b.base) % es) { bad("address inside %s not on an element boundary", b.name.c_str()); return nullptr; }
        return &b.e[(a - b.base) / es];
      }
    return nullptr;
  }
  void* ptr(int b, uint64_t elem = 0) { return (void*)(bufs[b].base + elem * bufs[b].es); }
};

// epochs: a new one starts at every hipStreamWaitEvent (the fork and the join of a call)
static int epoch_of(size_t launch_index) {
  int e = 0;
  for (const shim::StreamOp& op : shim::stream_ops())
    if (op.kind == shim::StreamOp::WAIT && op.before_launch <= launch_index) ++e;
  return e;
}

static Sym read(Mem& m, const char* p, uint64_t es, int stream, int epoch, const char* what) {
  Sym* s = m.at(p, es);
  if (!s) { bad("%s: read outside every buffer of the call", what); return Sym(); }
  if (s->idx < 0) bad("%s: read of an element nothing has written", what);
  if (s->w_stream >= 0 && s->w_stream != stream && s->w_epoch == epoch) bad("%s: reads what the other stream wrote since the last synchronisation", what);
  s->r_epoch[stream] = epoch;
  return *s;
}
static void write(Mem& m, char* p, uint64_t es, Sym v, int stream, int epoch, const char* what) {
  Sym* s = m.at(p, es);
  if (!s) { bad("%s: write outside every buffer of the call", what); return; }
  if (s->w_stream >= 0 && s->w_stream != stream && s->w_epoch == epoch) bad("%s: both streams write one element without synchronisation", what);
  if (s->r_epoch[1 - stream] == epoch) bad("%s: overwrites what the other stream read since the last synchronisation", what);
  v.w_stream = (int8_t)stream;
  v.w_epoch = epoch;
  v.r_epoch[0] = s->r_epoch[0];
  v.r_epoch[1] = s->r_epoch[1];
  *s = v;
}

static Sym hop(const Sym& in, const Sym& loc, const char* what) {
  Sym r = in;
  if (in.idx != loc.idx) bad("%s: operands are different vector elements (%lld, %lld)", what, (long long)in.idx, (long long)loc.idx);
  for (int k = 0; k < loc.len; ++k) {
    if (r.len >= 16) { bad("%s: more than 16 operands", what); break; }
    r.seq[r.len++] = loc.seq[k];
  }
  return r;
}

// Executes the launches recorded since the last reset; main = the caller's stream.
static void execute(Mem& m, void* main_stream, uint64_t es) {
  const std::vector<shim::Launch>& L = shim::launches();
  for (size_t li = 0; li < L.size(); ++li) {
    const shim::Launch& l = L[li];
    const int stream = l.stream == main_stream ? 0 : 1;
    const int epoch = epoch_of(li);
    char what[96];
    snprintf(what, sizeof what, "launch %zu", li);
    const uint64_t tile = hcl::tile_elems(l.dtype, l.tune);
    if (l.tune.blocks < 1) bad("%s: empty grid", what);
    if (!l.fused) {
      const hcl::StepArgs& a = l.step;
      if (a.nseg < 1 || a.nseg > (uint32_t)hcl::kMaxSegs) { bad("%s: %u segments", what, a.nseg); continue; }
      uint64_t maxn = 0;
      for (uint32_t d = 0; d < a.nseg; ++d) maxn = std::max(maxn, a.seg[d].n);
      if (a.chunk == 0 || a.tiles_per_chunk != ceil_div(a.chunk, tile)) bad("%s: tiles_per_chunk %u does not fit chunk %llu / tile %llu", what, a.tiles_per_chunk, (unsigned long long)a.chunk, (unsigned long long)tile);
      const uint64_t want_tiles = ceil_div(maxn, a.chunk) * a.nseg * a.tiles_per_chunk;
      if (want_tiles > 0x7FFFFFFFull || a.total_tiles != want_tiles) bad("%s: total_tiles %u, the segments need %llu", what, a.total_tiles, (unsigned long long)want_tiles);
      if ((uint32_t)l.tune.blocks > a.total_tiles) bad("%s: grid larger than the tile count", what);
      // reads first (all segments of a launch run at once), then the writes
      struct W1 { char* p; Sym v; uint32_t d; uint64_t i; };
      std::vector<W1> writes;
      std::map<uintptr_t, std::pair<uint32_t, uint64_t>> written;  // address -> (segment, element)
      for (uint32_t d = 0; d < a.nseg; ++d) {
        const hcl::Seg& s = a.seg[d];
        if (s.n == 0) bad("%s: empty segment", what);
        for (uint64_t i = 0; i < s.n; ++i) {
          Sym v = read(m, s.src0 + i * es, es, stream, epoch, what);
          if (l.nsrc == 2) v = hop(v, read(m, s.src1 + i * es, es, stream, epoch, what), what);
          writes.push_back({s.dst0 + i * es, v, d, i});
          if (l.ndst == 2) writes.push_back({s.dst1 + i * es, v, d, i});
        }
      }
      for (const W1& w : writes) {
        auto ins = written.insert({(uintptr_t)w.p, {w.d, w.i}});
        if (!ins.second) bad("%s: two segments write one address", what);
      }
      for (uint32_t d = 0; d < a.nseg; ++d) {
        const hcl::Seg& s = a.seg[d];
        for (uint64_t i = 0; i < s.n; ++i)
          for (int k = 0; k < l.nsrc; ++k) {
            auto it = written.find((uintptr_t)((k ? s.src1 : s.src0) + i * es));
            if (it != written.end() && !(it->second.first == d && it->second.second == i))
              bad("%s: segment %u reads an address that another thread of the launch writes", what, d);
          }
      }
      for (const W1& w : writes) write(m, w.p, es, w.v, stream, epoch, what);
    } else {
      const hcl::FusedArgs& f = l.fusedargs;
      const bool whole = f.mode >= 3, copy = f.mode == 2 || f.mode == 4;
      const uint32_t nblk = whole ? 1 : f.W;
      const uint64_t want_tiles = ceil_div(f.B, f.chunk) * nblk * f.tiles_per_chunk;
      if (f.chunk == 0 || f.tiles_per_chunk != ceil_div(f.chunk, tile) || f.total_tiles != want_tiles) bad("%s: fused tile grid inconsistent", what);
      for (uint32_t c = 0; c < nblk; ++c) {
        const uint32_t blk = whole ? f.root : c;
        uint64_t blo = whole ? 0 : (uint64_t)blk * f.B, bhi = blo + f.B;
        blo = std::min(blo, f.count);
        bhi = std::min(bhi, f.count);
        for (uint64_t i = blo; i < bhi; ++i) {
          Sym v;
          if (copy) {
            v = read(m, f.src[blk] + (f.mode == 2 ? i - blo : i) * es, es, stream, epoch, what);
          } else {
            const uint32_t first = f.tree ? 0u : f.pos[blk] + 1u;
            v = read(m, f.src[f.order[first % f.W]] + i * es, es, stream, epoch, what);
            for (uint32_t k = 1; k < f.W; ++k) v = hop(v, read(m, f.src[f.order[(first + k) % f.W]] + i * es, es, stream, epoch, what), what);
          }
          if (f.mode == 0 || copy) {
            for (uint32_t r = 0; r < f.W; ++r) write(m, f.dst[r] + i * es, es, v, stream, epoch, what);
          } else {
            write(m, f.dst[blk] + (f.mode == 1 ? i - blo : i) * es, es, v, stream, epoch, what);
          }
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// one symbolic run of each collective
// ---------------------------------------------------------------------------
struct Case {
  int W;
  uint64_t n;  // count argument of the entry point
  int dtype;
  uint64_t chunk_elems;
  bool inplace, fused, staged, fuse_rs_ag, two_chains;
  std::vector<int> ring;
  int threads, unroll, blocks;
  uint64_t misalign;
  size_t slab_bytes;  // 0 default, (size_t)-1 none, else what one step may write per slab
};

static void fill_input(Mem& m, int b, int rank, int64_t idx0) {
  for (uint64_t i = 0; i < m.bufs[b].n; ++i) {
    Sym& s = m.bufs[b].e[i];
    s.idx = idx0 + (int64_t)i;
    s.len = 1;
    s.seq[0] = (uint8_t)rank;
  }
}
static void expect(Mem& m, int b, uint64_t i, int64_t idx, const std::vector<int>& seq, const char* what) {
  const Sym& s = m.bufs[b].e[i];
  bool ok = s.idx == idx && s.len == seq.size();
  for (size_t k = 0; ok && k < seq.size(); ++k) ok = s.seq[k] == seq[k];
  if (!ok) bad("%s: %s[%llu] holds element %lld with %d operands (first rank %d), expected element %lld with %zu operands starting at rank %d",
               what, m.bufs[b].name.c_str(), (unsigned long long)i, (long long)s.idx, s.len, s.len ? s.seq[0] : -1, (long long)idx, seq.size(), seq[0]);
}
static std::vector<int> ring_order_of_block(const std::vector<int>& ring, int W, int c) {
  std::vector<int> pos(W);
  for (int k = 0; k < W; ++k) pos[ring[k]] = k;
  std::vector<int> seq;
  for (int k = 1; k <= W; ++k) seq.push_back(ring[(pos[c] + k) % W]);
  return seq;
}

static void* const MAIN = (void*)0x77770000ull;
static void* const AUX = (void*)0x88880000ull;

static hcl_opts_t make_opts(const Case& c, Mem& m, int kind, void* const* events) {
  hcl_opts_t o;
  memset(&o, 0, sizeof o);
  o.ring = c.ring.data();
  o.sched = c.fused ? HCL_SCHED_FUSED : HCL_SCHED_STEPWISE;
  o.xport = c.staged ? HCL_XPORT_HOST_STAGED : HCL_XPORT_DIRECT;
  o.threads = c.threads;
  o.unroll = c.unroll;
  o.blocks = c.blocks;
  o.fuse_rs_ag = c.fuse_rs_ag;
  o.slab_bytes = c.slab_bytes;
  if (c.two_chains) {
    o.aux_stream = AUX;
    o.aux_events = events;
  }
  const size_t es = hcl::elem_size(c.dtype);
  const size_t wsb = hcl_workspace_bytes(kind, c.W, c.n, (hcl_dtype_t)c.dtype, c.chunk_elems * es, &o);
  if (wsb) {
    o.workspace = m.ptr(m.add("workspace", wsb / es, es));
    o.workspace_bytes = wsb;
  }
  const size_t hsb = hcl_host_stage_bytes(kind, c.W, c.n, (hcl_dtype_t)c.dtype, c.chunk_elems * es, &o);
  if (hsb) {
    o.host_stage = m.ptr(m.add("host_stage", hsb / es, es));
    o.host_stage_bytes = hsb;
  }
  return o;
}

static void check_stream_ops(const Case& c, size_t nlaunch) {
  // with two chains in use: exactly one fork (record on the caller's stream, wait on the second)
  // before the first launch on the second stream and one join (the reverse) after the last launch
  const auto& ops = shim::stream_ops();
  bool used_aux = false;
  size_t first_aux = 0;
  for (size_t i = 0; i < shim::launches().size(); ++i)
    if (shim::launches()[i].stream == AUX) {
      if (!used_aux) first_aux = i;
      used_aux = true;
    } else if (shim::launches()[i].stream != MAIN) {
      bad("a launch on an unknown stream");
    }
  if (!used_aux) {
    if (!ops.empty()) bad("stream operations without a second chain");
    return;
  }
  if (!c.two_chains) bad("second stream used without being asked for");
  if (ops.size() != 4) { bad("%zu stream operations, expected fork + join", ops.size()); return; }
  const bool fork_ok = ops[0].kind == shim::StreamOp::RECORD && ops[0].stream == MAIN && ops[1].kind == shim::StreamOp::WAIT &&
                       ops[1].stream == AUX && ops[0].event == ops[1].event && ops[1].before_launch <= first_aux;
  const bool join_ok = ops[2].kind == shim::StreamOp::RECORD && ops[2].stream == AUX && ops[3].kind == shim::StreamOp::WAIT &&
                       ops[3].stream == MAIN && ops[2].event == ops[3].event && ops[2].before_launch == nlaunch;
  if (!fork_ok) bad("fork is not record(main) -> wait(second) before the second chain's first launch");
  if (!join_ok) bad("join is not record(second) -> wait(main) after the last launch");
}

static std::string describe(const char* kind, const Case& c) {
  char b[256];
  snprintf(b, sizeof b, "%s W=%d n=%llu dtype=%d chunk=%llu inplace=%d fused=%d staged=%d fuse=%d chains=%d shape=%dx%d blocks=%d mis=%llu slab=%lld",
           kind, c.W, (unsigned long long)c.n, c.dtype, (unsigned long long)c.chunk_elems, c.inplace, c.fused, c.staged,
           c.fuse_rs_ag, c.two_chains ? 2 : 1, c.threads, c.unroll, c.blocks, (unsigned long long)c.misalign, (long long)c.slab_bytes);
  return b;
}

static void run_allreduce(const Case& c) {
  g_case = describe("allreduce", c);
  Mem m;
  const uint64_t es = hcl::elem_size(c.dtype);
  std::vector<int> sb(c.W), rb(c.W);
  const void* send[16];
  void* recv[16];
  for (int r = 0; r < c.W; ++r) {
    sb[r] = m.add("send" + std::to_string(r), c.n, es, c.misalign);
    fill_input(m, sb[r], r, 0);
    rb[r] = c.inplace ? sb[r] : m.add("recv" + std::to_string(r), c.n, es, c.misalign);
    send[r] = m.ptr(sb[r]);
    recv[r] = m.ptr(rb[r]);
  }
  void* ev[2] = {(void*)0x1, (void*)0x2};
  hcl_opts_t o = make_opts(c, m, HCL_KIND_ALLREDUCE, ev);
  int nl = -1;
  o.n_launches = &nl;
  shim::reset();
  hcl_status_t st = hcl_allreduce_sim(send, recv, c.W, c.n, (hcl_dtype_t)c.dtype, HCL_SUM, c.chunk_elems * es, &o, MAIN);
  if (st != HCL_OK) { bad("status %s: %s", hcl_status_string(st), hcl_last_error()); return; }
  if (nl != (int)shim::launches().size()) bad("n_launches %d, %zu launches recorded", nl, shim::launches().size());
  check_stream_ops(c, shim::launches().size());
  execute(m, MAIN, es);
  const uint64_t B = ceil_div(c.n, (uint64_t)c.W);
  for (int r = 0; r < c.W; ++r)
    for (uint64_t i = 0; i < c.n; ++i) expect(m, rb[r], i, (int64_t)i, ring_order_of_block(c.ring, c.W, (int)(i / B)), "all-reduce result");
  if (!c.inplace)
    for (int r = 0; r < c.W; ++r)
      for (uint64_t i = 0; i < c.n; ++i) expect(m, sb[r], i, (int64_t)i, {r}, "send[] must stay untouched");
}

static void run_rs_then_ag(const Case& c) {
  Mem m;
  const uint64_t es = hcl::elem_size(c.dtype), n = c.n;
  std::vector<int> sb(c.W), rb(c.W);
  const void* send[16];
  void* recv[16];
  g_case = describe("reduce-scatter", c);
  for (int r = 0; r < c.W; ++r) {
    sb[r] = m.add("send" + std::to_string(r), n * c.W, es, c.misalign);
    fill_input(m, sb[r], r, 0);
    send[r] = m.ptr(sb[r]);
    if (!c.inplace) {
      rb[r] = m.add("recv" + std::to_string(r), n, es, c.misalign);
      recv[r] = m.ptr(rb[r]);
    } else {
      recv[r] = m.ptr(sb[r], (uint64_t)r * n);
    }
  }
  void* ev[2] = {(void*)0x1, (void*)0x2};
  hcl_opts_t o = make_opts(c, m, HCL_KIND_REDUCE_SCATTER, ev);
  shim::reset();
  hcl_status_t st = hcl_reduce_scatter_sim(send, recv, c.W, n, (hcl_dtype_t)c.dtype, HCL_SUM, c.chunk_elems * es, &o, MAIN);
  if (st != HCL_OK) { bad("status %s: %s", hcl_status_string(st), hcl_last_error()); return; }
  check_stream_ops(c, shim::launches().size());
  execute(m, MAIN, es);
  for (int r = 0; r < c.W; ++r)
    for (uint64_t i = 0; i < n; ++i) {
      const std::vector<int> seq = ring_order_of_block(c.ring, c.W, r);
      if (c.inplace) expect(m, sb[r], (uint64_t)r * n + i, (int64_t)((uint64_t)r * n + i), seq, "reduce-scatter result (in place)");
      else expect(m, rb[r], i, (int64_t)((uint64_t)r * n + i), seq, "reduce-scatter result");
    }

  // All-Gather of fresh shards
  g_case = describe("all-gather", c);
  Mem g;
  std::vector<int> full(c.W), shard(c.W);
  for (int r = 0; r < c.W; ++r) {
    full[r] = g.add("recv" + std::to_string(r), n * c.W, es, c.misalign);
    recv[r] = g.ptr(full[r]);
    if (c.inplace) {
      for (uint64_t i = 0; i < n; ++i) {
        Sym& s = g.bufs[full[r]].e[(uint64_t)r * n + i];
        s.idx = (int64_t)((uint64_t)r * n + i);
        s.len = 1;
        s.seq[0] = (uint8_t)r;
      }
      send[r] = g.ptr(full[r], (uint64_t)r * n);
    } else {
      shard[r] = g.add("send" + std::to_string(r), n, es, c.misalign);
      fill_input(g, shard[r], r, (int64_t)((uint64_t)r * n));
      send[r] = g.ptr(shard[r]);
    }
  }
  Case cg = c;
  hcl_opts_t og = make_opts(cg, g, HCL_KIND_ALL_GATHER, ev);
  shim::reset();
  st = hcl_all_gather_sim(send, recv, c.W, n, (hcl_dtype_t)c.dtype, c.chunk_elems * es, &og, MAIN);
  if (st != HCL_OK) { bad("status %s: %s", hcl_status_string(st), hcl_last_error()); return; }
  check_stream_ops(c, shim::launches().size());
  execute(g, MAIN, es);
  for (int r = 0; r < c.W; ++r)
    for (int q = 0; q < c.W; ++q)
      for (uint64_t i = 0; i < n; ++i) expect(g, full[r], (uint64_t)q * n + i, (int64_t)((uint64_t)q * n + i), {q}, "all-gather result");
}

static void run_reduce_broadcast_alltoall(const Case& c, int root) {
  const uint64_t es = hcl::elem_size(c.dtype), n = c.n;
  void* ev[2] = {(void*)0x1, (void*)0x2};
  {
    g_case = describe("reduce", c);
    Mem m;
    std::vector<int> sb(c.W);
    const void* send[16];
    void* recv[16] = {};
    for (int r = 0; r < c.W; ++r) {
      sb[r] = m.add("send" + std::to_string(r), n, es, c.misalign);
      fill_input(m, sb[r], r, 0);
      send[r] = m.ptr(sb[r]);
    }
    const int out = c.inplace ? sb[root] : m.add("recv_root", n, es, c.misalign);
    recv[root] = m.ptr(out);
    hcl_opts_t o = make_opts(c, m, HCL_KIND_REDUCE, ev);
    shim::reset();
    hcl_status_t st = hcl_reduce_sim(send, recv, c.W, n, (hcl_dtype_t)c.dtype, HCL_SUM, root, c.chunk_elems * es, &o, MAIN);
    if (st != HCL_OK) { bad("status %s: %s", hcl_status_string(st), hcl_last_error()); return; }
    check_stream_ops(c, shim::launches().size());
    execute(m, MAIN, es);
    for (uint64_t i = 0; i < n; ++i) expect(m, out, i, (int64_t)i, ring_order_of_block(c.ring, c.W, root), "reduce result");
  }
  {
    g_case = describe("broadcast", c);
    Mem m;
    std::vector<int> rb(c.W);
    const void* send[16] = {};
    void* recv[16];
    for (int r = 0; r < c.W; ++r) {
      rb[r] = m.add("recv" + std::to_string(r), n, es, c.misalign);
      recv[r] = m.ptr(rb[r]);
    }
    int src = rb[root];
    if (!c.inplace) src = m.add("send_root", n, es, c.misalign);
    fill_input(m, src, root, 0);
    send[root] = m.ptr(src);
    hcl_opts_t o = make_opts(c, m, HCL_KIND_BROADCAST, ev);
    shim::reset();
    hcl_status_t st = hcl_broadcast_sim(send, recv, c.W, n, (hcl_dtype_t)c.dtype, root, c.chunk_elems * es, &o, MAIN);
    if (st != HCL_OK) { bad("status %s: %s", hcl_status_string(st), hcl_last_error()); return; }
    check_stream_ops(c, shim::launches().size());
    execute(m, MAIN, es);
    for (int r = 0; r < c.W; ++r)
      for (uint64_t i = 0; i < n; ++i) expect(m, rb[r], i, (int64_t)i, {root}, "broadcast result");
  }
  {
    g_case = describe("all-to-all", c);
    Mem m;
    std::vector<int> sb(c.W), rb(c.W);
    const void* send[16];
    void* recv[16];
    for (int r = 0; r < c.W; ++r) {
      sb[r] = m.add("send" + std::to_string(r), n * c.W, es, c.misalign);
      fill_input(m, sb[r], r, (int64_t)((uint64_t)r * n * c.W));
      rb[r] = m.add("recv" + std::to_string(r), n * c.W, es, c.misalign);
      send[r] = m.ptr(sb[r]);
      recv[r] = m.ptr(rb[r]);
    }
    hcl_opts_t o = make_opts(c, m, HCL_KIND_ALLTOALL, ev);
    shim::reset();
    hcl_status_t st = hcl_alltoall_sim(send, recv, c.W, n, (hcl_dtype_t)c.dtype, c.chunk_elems * es, &o, MAIN);
    if (st != HCL_OK) { bad("status %s: %s", hcl_status_string(st), hcl_last_error()); return; }
    check_stream_ops(c, shim::launches().size());
    execute(m, MAIN, es);
    for (int r = 0; r < c.W; ++r)
      for (int q = 0; q < c.W; ++q)
        for (uint64_t i = 0; i < n; ++i)
          expect(m, rb[r], (uint64_t)q * n + i, (int64_t)(((uint64_t)q * c.W + r) * n + i), {q}, "all-to-all result");
  }
}

// ---------------------------------------------------------------------------
// scheduler tables and work items
// ---------------------------------------------------------------------------
static void check_scheduler(std::mt19937& rng) {
  g_case = "scheduler";
  for (int W = 1; W <= 16; ++W) {
    std::vector<int> ring(W);
    for (int k = 0; k < W; ++k) ring[k] = k;
    std::shuffle(ring.begin(), ring.end(), rng);
    std::vector<int> pos(W);
    for (int k = 0; k < W; ++k) pos[ring[k]] = k;
    for (int r = 0; r < W; ++r)
      for (int s = 0; s <= W - 2; ++s) {
        int sb = -1, rb = -1;
        if (hcl_ring_step(W, ring.data(), HCL_PHASE_RS, s, r, &sb, &rb) != HCL_OK) bad("ring_step failed");
        // what a rank receives is what its predecessor sends in the same step
        int psb = -1, prb = -1;
        hcl_ring_step(W, ring.data(), HCL_PHASE_RS, s, ring[(pos[r] + W - 1) % W], &psb, &prb);
        if (psb != rb) bad("W=%d rank %d step %d: receives block %d, predecessor sends %d", W, r, s, rb, psb);
        if (s == W - 2 && rb != r) bad("W=%d: rank %d does not end the reduce-scatter with its own block", W, r);
        hcl_ring_step(W, ring.data(), HCL_PHASE_AG, s, r, &sb, &rb);
        if (s == 0 && sb != r) bad("W=%d: rank %d does not start the all-gather with its own block", W, r);
      }
    int bad_rank = -1, x, y;
    if (hcl_ring_step(W, ring.data(), HCL_PHASE_RS, 0, W, &x, &y) == HCL_OK && W > 0) bad_rank = 0;
    if (bad_rank == 0) bad("rank out of range accepted");
    // work items: every element of every block exactly once per step, also when the caller's array is short
    for (uint64_t count : {(uint64_t)1, (uint64_t)W, (uint64_t)(W * 37 + 5), (uint64_t)1000}) {
      for (uint64_t chunk_elems : {(uint64_t)0, (uint64_t)1, (uint64_t)7, (uint64_t)64}) {
        for (int phase = 0; phase < 2 && W > 1; ++phase) {
          size_t n = 0;
          if (hcl_schedule_items(W, ring.data(), count, HCL_FP32, chunk_elems * 4, phase, 0, nullptr, 0, &n) != HCL_OK) bad("schedule_items count query failed");
          std::vector<hcl_work_item_t> items(n ? n : 1);
          size_t n2 = 0;
          hcl_schedule_items(W, ring.data(), count, HCL_FP32, chunk_elems * 4, phase, 0, items.data(), n, &n2);
          if (n2 != n) bad("schedule_items count changed between calls");
          std::vector<int> seen(count, 0);
          for (size_t i = 0; i < n; ++i)
            for (uint64_t e = 0; e < items[i].elem_count; ++e) seen[items[i].vec_offset + e]++;
          for (uint64_t e = 0; e < count; ++e)
            if (seen[e] != 1) { bad("W=%d count=%llu chunk=%llu phase %d: element %llu covered %d times", W, (unsigned long long)count, (unsigned long long)chunk_elems, phase, (unsigned long long)e, seen[e]); break; }
          if (n > 1) {  // a short array must not be overrun (the sanitizer watches the heap block)
            std::vector<hcl_work_item_t> few(n - 1);
            hcl_schedule_items(W, ring.data(), count, HCL_FP32, chunk_elems * 4, phase, 0, few.data(), n - 1, &n2);
            if (n2 != n) bad("schedule_items must report the total even when the array is short");
          }
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// sizes no symbolic memory can hold: bounds, tile counts, coverage by intervals
// ---------------------------------------------------------------------------
static void check_large(uint64_t n, int dtype, uint64_t chunk_bytes, int threads, int unroll, bool two_chains, size_t min_launches_per_step) {
  const int W = 8;
  const uint64_t es = hcl::elem_size(dtype);
  char d[160];
  snprintf(d, sizeof d, "large reduce-scatter n=%llu dtype=%d chunk_bytes=%llu shape=%dx%d chains=%d", (unsigned long long)n, dtype,
           (unsigned long long)chunk_bytes, threads, unroll, two_chains ? 2 : 1);
  g_case = d;
  const uintptr_t base = 0x200000000000ull, stride = 0x80000000000ull;  // 8 TiB apart
  const void* send[16];
  void* recv[16];
  for (int r = 0; r < W; ++r) {
    send[r] = (void*)(base + (uintptr_t)r * stride);
    recv[r] = (void*)(base + (uintptr_t)(W + r) * stride);
  }
  hcl_opts_t o;
  memset(&o, 0, sizeof o);
  o.threads = threads;
  o.unroll = unroll;
  o.slab_bytes = (size_t)-1;  // every step one pass: consecutive launches that cover W blocks form a step
  void* ev[2] = {(void*)0x1, (void*)0x2};
  if (two_chains) {
    o.aux_stream = AUX;
    o.aux_events = ev;
  }
  o.workspace_bytes = hcl_workspace_bytes(HCL_KIND_REDUCE_SCATTER, W, n, (hcl_dtype_t)dtype, chunk_bytes, &o);
  o.workspace = (void*)(base + (uintptr_t)(2 * W) * stride);
  shim::reset();
  hcl_status_t st = hcl_reduce_scatter_sim(send, recv, W, n, (hcl_dtype_t)dtype, HCL_SUM, chunk_bytes, &o, MAIN);
  if (st != HCL_OK) { bad("status %s: %s", hcl_status_string(st), hcl_last_error()); return; }
  const auto& L = shim::launches();
  // consecutive launches with the same first source block form one step; the destination
  // intervals of a step must tile W blocks of n elements exactly once
  std::vector<std::pair<uintptr_t, uintptr_t>> iv;
  size_t in_step = 0, steps = 0;
  uint64_t covered = 0;
  auto close_step = [&]() {
    std::sort(iv.begin(), iv.end());
    for (size_t i = 1; i < iv.size(); ++i)
      if (iv[i].first < iv[i - 1].second) bad("destination intervals of one step overlap");
    if (covered != (uint64_t)W * n) bad("a step writes %llu elements, expected %llu", (unsigned long long)covered, (unsigned long long)W * n);
    if (in_step < min_launches_per_step) bad("a step ran in %zu launches, expected at least %zu", in_step, min_launches_per_step);
    iv.clear();
    covered = 0;
    in_step = 0;
    ++steps;
  };
  for (size_t li = 0; li < L.size(); ++li) {
    const hcl::StepArgs& a = L[li].step;
    const uint64_t tile = hcl::tile_elems(dtype, L[li].tune);
    uint64_t maxn = 0;
    for (uint32_t s = 0; s < a.nseg; ++s) maxn = std::max(maxn, a.seg[s].n);
    const uint64_t want = ceil_div(maxn, a.chunk) * a.nseg * a.tiles_per_chunk;
    if (want > 0x7FFFFFFFull || a.total_tiles != want || a.tiles_per_chunk != ceil_div(a.chunk, tile)) bad("launch %zu: tile grid inconsistent or beyond 2^31 - 1 (%llu)", li, (unsigned long long)want);
    // the runtime refuses a launch of 2^32 threads or more: larger tile counts must stride
    const uint64_t grid = (uint64_t)L[li].tune.blocks, thr = (uint64_t)L[li].tune.threads;
    if (grid < 1 || grid > a.total_tiles || grid * thr > 0xFFFFFFFFull) bad("launch %zu: grid %llu x %llu threads", li, (unsigned long long)grid, (unsigned long long)thr);
    for (uint32_t s = 0; s < a.nseg; ++s) {
      const uintptr_t lo = (uintptr_t)a.seg[s].dst0, hi = lo + a.seg[s].n * es;
      iv.push_back({lo, hi});
      covered += a.seg[s].n;
      // every pointer inside the rank buffers or the workspace
      for (const char* p : {a.seg[s].src0, a.seg[s].src1, (const char*)a.seg[s].dst0}) {
        const uintptr_t q = (uintptr_t)p, off = (q - base) % stride, which = (q - base) / stride;
        const uint64_t limit = which < (uintptr_t)W ? (uint64_t)W * n * es : which < (uintptr_t)(2 * W) ? n * es : o.workspace_bytes;
        if (q < base || which > (uintptr_t)(2 * W) || off + a.seg[s].n * es > limit) bad("launch %zu: a segment leaves its buffer", li);
      }
    }
    ++in_step;
    if (covered >= (uint64_t)W * n) close_step();
  }
  if (steps != (size_t)W - 1 || covered) bad("%zu complete steps, expected %d", steps, W - 1);
}

// The default slab budget on the ZeRO-style shape: 2 GiB blocks in 64 slabs of 32 MiB, every
// launch writing at most 256 MiB, all launches together every element once per step.
static void check_large_slabs() {
  g_case = "large reduce-scatter, default slabs";
  const int W = 8;
  const uint64_t n = (uint64_t)1 << 30, es = 2;
  const uintptr_t base = 0x200000000000ull, stride = 0x4000000000ull;
  const void* send[16];
  void* recv[16];
  for (int r = 0; r < W; ++r) {
    send[r] = (void*)(base + (uintptr_t)r * stride);
    recv[r] = (void*)(base + (uintptr_t)(W + r) * stride);
  }
  hcl_opts_t o;
  memset(&o, 0, sizeof o);
  o.workspace_bytes = hcl_workspace_bytes(HCL_KIND_REDUCE_SCATTER, W, n, HCL_BF16, 4 << 20, &o);
  o.workspace = (void*)(base + (uintptr_t)(2 * W) * stride);
  shim::reset();
  hcl_status_t st = hcl_reduce_scatter_sim(send, recv, W, n, HCL_BF16, HCL_SUM, 4 << 20, &o, MAIN);
  if (st != HCL_OK) { bad("status %s: %s", hcl_status_string(st), hcl_last_error()); return; }
  const auto& L = shim::launches();
  if (L.size() != 64u * (W - 1)) bad("%zu launches, expected 64 slabs x %d steps", L.size(), W - 1);
  uint64_t total = 0;
  for (size_t li = 0; li < L.size(); ++li) {
    uint64_t wrote = 0;
    for (uint32_t s2 = 0; s2 < L[li].step.nseg; ++s2) wrote += L[li].step.seg[s2].n;
    if (wrote * es > (256ull << 20)) bad("launch %zu writes %llu bytes, more than the slab budget", li, (unsigned long long)(wrote * es));
    total += wrote;
    // launch li belongs to slab li / (W - 1): its segments start that many slabs into their blocks
    const uint64_t slab = (uint64_t)(li / (W - 1)) * (32ull << 20);
    const uintptr_t d = (uintptr_t)L[li].step.seg[0].dst0;
    const uint64_t off = (d - base) % stride;
    const bool last = li % (W - 1) == (size_t)(W - 2);
    if (last ? off != slab : (off % ((2ull << 30) + 4096)) != slab) bad("launch %zu does not start at its slab", li);
  }
  if (total != (uint64_t)(W - 1) * W * n) bad("the launches write %llu elements in all, expected %llu", (unsigned long long)total, (unsigned long long)((W - 1) * W * n));
}

static void check_validation() {
  g_case = "validation";
  const void* send[16];
  void* recv[16];
  for (int r = 0; r < 16; ++r) {
    send[r] = (void*)(0x10000000ull + r * 0x100000ull);
    recv[r] = (void*)(0x20000000ull + r * 0x100000ull);
  }
  hcl_opts_t o;
  memset(&o, 0, sizeof o);
  shim::reset();
  if (hcl_allreduce_sim(send, recv, 0, 16, HCL_FP32, HCL_SUM, 0, &o, MAIN) != HCL_ERR_INVALID_ARG) bad("W = 0 accepted");
  if (hcl_allreduce_sim(send, recv, 17, 16, HCL_FP32, HCL_SUM, 0, &o, MAIN) != HCL_ERR_INVALID_ARG) bad("W = 17 accepted");
  if (hcl_allreduce_sim(send, recv, 4, 16, HCL_FP32, HCL_SUM, 6, &o, MAIN) != HCL_ERR_INVALID_ARG) bad("ragged chunk accepted");
  if (hcl_allreduce_sim(send, recv, 4, 16, (hcl_dtype_t)9, HCL_SUM, 0, &o, MAIN) != HCL_ERR_UNSUPPORTED) bad("dtype 9 accepted");
  if (hcl_reduce_scatter_sim(send, recv, 4, 16, HCL_FP32, HCL_SUM, 0, &o, MAIN) != HCL_ERR_WORKSPACE) bad("missing workspace accepted");
  o.workspace = (void*)0x30000001ull;
  o.workspace_bytes = 1 << 20;
  if (hcl_reduce_scatter_sim(send, recv, 4, 16, HCL_FP32, HCL_SUM, 0, &o, MAIN) != HCL_ERR_INVALID_ARG) bad("misaligned workspace accepted");
  o.workspace = nullptr;
  o.xport = HCL_XPORT_HOST_STAGED;
  if (hcl_allreduce_sim(send, recv, 4, 16, HCL_FP32, HCL_SUM, 0, &o, MAIN) != HCL_ERR_WORKSPACE) bad("missing host stage accepted");
  o.xport = 0;
  recv[1] = (char*)recv[0] + 8;
  if (hcl_allreduce_sim(send, recv, 4, 16, HCL_FP32, HCL_SUM, 0, &o, MAIN) != HCL_ERR_ALIAS) bad("overlapping recv buffers accepted");
  if (!shim::launches().empty()) bad("a refused call launched something");
  if (hcl_allreduce_sim(send, recv, 4, 0, HCL_FP32, HCL_SUM, 0, &o, MAIN) != HCL_OK || !shim::launches().empty()) bad("count 0 must be a no-op");
}

int main(int argc, char** argv) {
  if (argc > 1 && !strcmp(argv[1], "dump")) {
    setenv("HCL_DEBUG", "1", 1);
    Case c{4, 10, HCL_FP32, 2, false, false, false, false, false, {2, 0, 3, 1}, 0, 0, 0, 0, 0};
    run_allreduce(c);
    return g_fail ? 1 : 0;
  }
  unsetenv("HCL_DEBUG");
  std::mt19937 rng(20260);
  check_scheduler(rng);
  check_validation();
  // symbolic runs: every collective, schedule, transport and launch shape on small counts
  int cases = 0;
  for (int W : {1, 2, 3, 4, 5, 8, 13, 16}) {
    for (int rep = 0; rep < 6; ++rep) {
      Case c;
      c.W = W;
      c.dtype = (int[]){HCL_FP32, HCL_BF16, HCL_UINT8, HCL_FP64}[rng() % 4];
      c.n = (uint64_t[]){1, 3, 17, 100, 257, 600}[rng() % 6];
      c.chunk_elems = (uint64_t[]){0, 0, 1, 5, 16, 64}[rng() % 6];
      c.inplace = rng() % 3 == 0;
      c.fused = rng() % 3 == 0;
      c.staged = !c.fused && rng() % 4 == 0;
      c.fuse_rs_ag = rng() % 3 == 0;
      c.two_chains = !c.fused && rng() % 2 == 0;
      c.ring.resize(W);
      for (int k = 0; k < W; ++k) c.ring[k] = k;
      if (rng() % 2) std::shuffle(c.ring.begin(), c.ring.end(), rng);
      c.threads = (int[]){0, 0, 64, 256}[rng() % 4];
      c.unroll = (int[]){0, 0, 1, 4}[rng() % 4];
      c.blocks = (int[]){0, 0, 3}[rng() % 3];
      c.misalign = rng() % 4 == 0 ? 1 : 0;
      c.slab_bytes = (size_t[]){0, 0, (size_t)-1, 64, 200, 1024}[rng() % 6];  // small budgets: several slabs per block
      run_allreduce(c);
      run_rs_then_ag(c);
      Case d = c;
      d.staged = false;  // Reduce, Broadcast and All-to-All have the direct transport only
      run_reduce_broadcast_alltoall(d, (int)(rng() % W));
      cases += 6;
    }
  }
  // sizes beyond 32-bit byte offsets and beyond 2^31 - 1 tiles per step
  check_large((uint64_t)1 << 30, HCL_BF16, 4 << 20, 0, 0, false, 1);       // 2 GiB blocks, 16 GiB vectors
  check_large((uint64_t)1 << 30, HCL_BF16, 4 << 20, 0, 0, true, 2);
  check_large((uint64_t)1 << 39, HCL_UINT8, 1, 64, 1, false, 3);            // 512 GiB blocks in 1 KiB tiles: 2^32 tiles a step
  check_large((uint64_t)1 << 39, HCL_UINT8, 1, 64, 1, true, 4);
  check_large(((uint64_t)1 << 30) + 12345, HCL_FP64, 0, 64, 1, false, 1);   // one chunk of 8 GiB per block
  check_large_slabs();
  if (g_fail) {
    fprintf(stderr, "host_check: %d failure(s)\n", g_fail);
    return 1;
  }
  printf("host_check: ok (%d symbolic collective runs)\n", cases);
  return 0;
}

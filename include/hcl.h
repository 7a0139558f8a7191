/*
 * hcl.h -- C ABI of libhcl: ring Reduce-Scatter / All-Gather / All-Reduce over
 * W simulated ranks whose buffers all live in one GPU's memory (or, for the
 * staged transport, partly in pinned host memory).
 *
 * The paper's library presents the vendor collective libraries' call shape to
 * the framework -- send buffer, receive buffer, count, datatype, reduction
 * operator, stream (Section 4.4 "Zero Code Modification") -- and leaves the
 * partitioning of a message and the device kernels to the vendor library
 * (Section 4.1 "Key Approach", Section 4.2).  This library is that inside for
 * one GPU: the communicator is replaced by explicit arrays of W per-rank
 * pointers, and "sending to the next rank" is a read of that rank's buffer.
 *
 * Common conventions
 *   - send[] / recv[] / ring are HOST arrays of length W, read during the call
 *     and not retained.  The pointers they hold are DEVICE pointers (memory
 *     the GPU can access at full speed); opts->host_stage is PINNED HOST
 *     memory mapped into the GPU's address space (hipHostMalloc).
 *   - Every buffer is owned by the caller.  The library allocates and frees no
 *     device or pinned memory; scratch comes in through hcl_opts_t.
 *   - Ring: ring[] is a permutation of 0..W-1 (NULL = identity); rank ring[k]
 *     sends to rank ring[(k+1) mod W].
 *   - Result bits.  Integer sums wrap modulo 2^bits.  For fp32 / bf16 / fp16 every
 *     hop computes round_T(f32(incoming) + f32(local)) with round to nearest
 *     even, subnormals kept, overflow to infinity, NaN propagated (any NaN
 *     pattern).  Block c's sum starts with the rank after c in the ring and
 *     ends at rank c.  Every schedule, transport, chunk size and launch shape
 *     produces the same bits.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream) and the call returns without synchronising; the
 *     calls only launch kernels, so they may be captured into a HIP graph.
 *   - Errors: validation is synchronous and happens before anything is
 *     enqueued; on any status other than HCL_OK nothing was launched (except
 *     HCL_ERR_HIP, where a launch itself failed part-way).  hcl_last_error()
 *     gives a thread-local message.  No exceptions, no abort.
 *   - W in [1, 16].  count == 0 is HCL_OK and a no-op.  chunk_bytes == 0 means
 *     one chunk per block; otherwise it must be a positive multiple of the
 *     element size.  A chunk only orders the work inside a block.
 *   - Rank buffers must be aligned to the element size; nothing more is
 *     required of them (opts->workspace and opts->host_stage must be 16-byte
 *     aligned).  Every path moves 128-bit vectors at whatever address the data
 *     has; buffers that are not 16-byte aligned (or not congruent modulo 128
 *     bytes with each other) make accesses straddle cache lines and measured
 *     10-25 % slower on MI355X than 256-byte aligned ones.
 *   - Layout advice: give every rank buffer an allocation of its own (or pack
 *     them back to back) with at least 256-byte alignment.  The kernels walk the
 *     ranks' streams at staggered offsets, so equally aligned buffers do not
 *     collide in DRAM; offsetting the buffers against each other by odd amounts
 *     (64 KiB + 256 B, say) measured 3-7 % slower on MI355X.
 *   - Launch-shape fields of hcl_opts_t that are 0 may be overridden by the
 *     environment variables HCL_THREADS, HCL_UNROLL, HCL_BLOCKS,
 *     HCL_NONTEMPORAL, HCL_STAGGER and HCL_ZIGZAG (0 = every step walks its
 *     tiles forwards) (for sweeps); values in the struct win.
 *   - HCL_DEBUG=1 in the environment makes every collective call print its
 *     arguments and the work items of its schedule (hcl_schedule_items) to
 *     stderr before it enqueues anything.
 *   - Calls are re-entrant; the only global state is cached device properties
 *     and the thread-local error string.
 */
#ifndef HCL_H_
#define HCL_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HCL_MAX_RANKS 16
#define HCL_VERSION 104
/* size of the library-owned scratch array behind hcl_reduce_scatter_sim_static */
#define HCL_STATIC_SCRATCH_BYTES (32u << 20)

typedef enum {
  HCL_OK = 0,
  HCL_ERR_INVALID_ARG = 1, /* null pointer, W out of range, bad ring, misaligned pointer or chunk */
  HCL_ERR_UNSUPPORTED = 2, /* unknown operator / dtype, or a schedule / transport / order combination
                              that does not exist */
  HCL_ERR_ALIAS = 3,       /* buffers overlap in a way the schedule cannot honour */
  HCL_ERR_WORKSPACE = 4,   /* opts->workspace or opts->host_stage missing or too small */
  HCL_ERR_HIP = 5          /* a HIP runtime call failed */
} hcl_status_t;

/* Wire types.  fp32 / bf16 / fp16 hops compute in binary32 and round to the wire
 * type; fp64 hops are one binary64 operation; the integer types wrap modulo
 * 2^bits (int32, int64: signed comparisons; uint8: unsigned -- also the type for
 * moving raw bytes of any format through All-Gather, Broadcast and All-to-All). */
typedef enum {
  HCL_FP32 = 0, HCL_BF16 = 1, HCL_FP16 = 2, HCL_INT32 = 3, HCL_FP64 = 4, HCL_INT64 = 5, HCL_UINT8 = 6
} hcl_dtype_t;
/* Reduction operator of one hop: partial = round_T(op(f32(incoming), f32(local))).
 * SUM and PROD round to nearest even (the product of two bf16 / fp16 values is
 * exact in binary32, so PROD is the correctly rounded product); MAX and MIN
 * return one of the operands and follow IEEE 754-2019 `maximum` / `minimum`: a
 * NaN operand gives NaN, -0 orders below +0.  int32: SUM and PROD wrap modulo
 * 2^32, MAX and MIN compare as signed integers. */
typedef enum { HCL_SUM = 0, HCL_PROD = 1, HCL_MAX = 2, HCL_MIN = 3 } hcl_op_t;

/* STEPWISE: the ring as each rank executes it, one launch per ring step doing
 *   every rank's reduce-copy (or copy) of that step.
 * FUSED: one launch per collective; each thread keeps its elements' whole ring
 *   pass in registers, reading every rank's value once, in ring order, with
 *   the same per-hop rounding. */
typedef enum { HCL_SCHED_STEPWISE = 0, HCL_SCHED_FUSED = 1 } hcl_sched_t;

/* DIRECT: a rank reads the incoming block straight out of its predecessor's
 *   buffer (peer-to-peer mode, Section 2.1 "Intra-node communication").
 * HOST_STAGED: every block travelling between ranks is written to the
 *   receiver's inbox in pinned host memory and read back from there by the
 *   receiver (host-staged path, Section 2.1 "Inter-node communication and
 *   RDMA"; Appendix F.1), local operands and results stay in device memory. */
typedef enum { HCL_XPORT_DIRECT = 0, HCL_XPORT_HOST_STAGED = 1 } hcl_xport_t;

/* PER_HOP: the ring's arithmetic, every addition rounded to the wire type.
 * FP32 (FUSED sums only): the same order of operands, but the running sum
 *   stays in binary32 and is rounded to the wire type once.  For bf16 / fp16
 *   this is a DIFFERENT result from the ring's -- the reordered class the
 *   paper tolerates between backends (Appendix E.2) -- within 2 ulp of the
 *   correctly rounded exact sum; for fp32 and int32 it is the ring's result. */
typedef enum { HCL_ACC_PER_HOP = 0, HCL_ACC_FP32 = 1 } hcl_acc_t;

/* RING: block c's values enter its reduction in the order next(c), ..., c -- the
 *   order the stepwise ring produces.
 * TREE (FUSED reductions only): the ranks' values are taken in ring order
 *   ring[0], ..., ring[W-1], the same for every block, and combined level by
 *   level, neighbours first ((v0 op v1), (v2 op v3), ...; an odd last value moves
 *   up unchanged).  A reordered-class result (Appendix E.2): different bits from
 *   the ring's for the float types' SUM and PROD, identical for MAX, MIN and int32.
 *   With PER_HOP every node is rounded to the wire type, with HCL_ACC_FP32 the
 *   tree is evaluated in binary32 and rounded once. */
typedef enum { HCL_ORDER_RING = 0, HCL_ORDER_TREE = 1 } hcl_order_t;

typedef enum {
  HCL_KIND_ALLREDUCE = 0, HCL_KIND_REDUCE_SCATTER = 1, HCL_KIND_ALL_GATHER = 2,
  HCL_KIND_REDUCE = 3, HCL_KIND_BROADCAST = 4, HCL_KIND_ALLTOALL = 5
} hcl_kind_t;
typedef enum { HCL_PHASE_RS = 0, HCL_PHASE_AG = 1 } hcl_phase_t;

/* Optional settings; a NULL hcl_opts_t* or a zero-filled struct means defaults. */
typedef struct hcl_opts {
  const int *ring;         /* host array, permutation of 0..W-1; NULL = identity            */
  int sched;               /* hcl_sched_t                                                   */
  int xport;               /* hcl_xport_t                                                   */
  void *workspace;         /* device scratch; see hcl_workspace_bytes                       */
  size_t workspace_bytes;
  void *host_stage;        /* pinned host inboxes; see hcl_host_stage_bytes                 */
  size_t host_stage_bytes;
  int threads;             /* threads per workgroup: 0 = default (reducing steps 128, copying steps
                              and the FUSED schedule 64), else 64..1024, multiple of 64; FUSED
                              reductions with an operator other than SUM or with tree order use at
                              most 256                                                         */
  int blocks;              /* workgroups per launch: 0 = default (one tile per workgroup); smaller
                              values give a persistent grid striding over the tiles            */
  int unroll;              /* 128-bit vectors in flight per thread and source: 0 = default (reducing
                              steps 2, copying steps 1 -- when threads is 0 too; FUSED All-Gather /
                              Broadcast 1, or 4 for blocks of 1 GiB
                              and more), else 1, 2, 4 or 8 (8: step kernels only).  The FUSED
                              reductions always keep one vector per thread and rank           */
  int nontemporal;         /* cache policy of the memory accesses.  0 = default: non-temporal
                              (streaming) loads; a STEPWISE step whose output a later launch of
                              the call reads, and which fits the 256 MiB last-level cache, writes
                              it through the L2 so that the next launch finds it in that cache;
                              the FUSED kernels write through while what they write fits that
                              cache (the one-source kernel: unless it runs its shape for blocks
                              of 1 GiB and more); all other stores are non-temporal.
                              1 = loads and stores non-temporal, 2 = loads non-temporal and
                              stores written through, -1 = ordinary loads and stores          */
  int fuse_rs_ag;          /* STEPWISE All-Reduce only: 1 = the last Reduce-Scatter step also
                              writes the finished block into the next rank's buffer and the
                              first All-Gather step is dropped (same bits, one read fewer)   */
  void *const *events;     /* measurement hook: host array of n_events hipEvent_t; event k is
                              recorded on the stream before launch k, and one more after the
                              last launch; launches beyond n_events-1 are not bracketed; all
                              events are recorded on `stream`, also for launches that go to
                              aux_stream                                                     */
  int n_events;
  int events_per_phase;    /* 0: as above.  1: events only at phase boundaries -- event 0 before the
                              first Reduce-Scatter launch (or the only phase of the call), event 1
                              before the first All-Gather launch of an All-Reduce, the next one
                              after the last launch: the cheap way to time a phase's launches
                              (with several slabs, see slab_bytes, the two phases of an All-Reduce
                              interleave and only the first and the last event are meaningful)  */
  int *n_launches;         /* if non-NULL, receives the number of kernel launches enqueued  */
  int accumulate;          /* hcl_acc_t; anything but PER_HOP needs sched == FUSED           */
  int order;               /* hcl_order_t; TREE needs sched == FUSED                          */
  size_t slab_bytes;       /* STEPWISE, DIRECT: the ring runs to completion (all Reduce-Scatter steps, then
                              all All-Gather steps) on one slab of every block before the next slab
                              starts; a slab is as many whole chunks as keep what one step writes, all
                              blocks together, within this many bytes (a remainder of less than 1/32 of a
                              slab joins the last one).  0 = default: 256 MiB, the
                              last-level cache, so that a step's incoming operand is still cached
                              when the next launch reads it, at any message size; (size_t)-1 = no
                              slabs, every step one pass over the whole blocks.  Same bits           */
  void *aux_stream;        /* STEPWISE only, optional: a second hipStream_t.  The chunks of every step
                              are split in two halves; the second half's launches go to this stream,
                              as a dependency chain of their own (chunk j of a step needs only chunk
                              j of the step before), forked from `stream` before its first launch and
                              joined back before the call returns -- one chain's kernel runs while the
                              other chain is between two kernels.  Same bits.  Both streams must have
                              the same (default) priority; legal under stream capture of `stream`    */
  void *const *aux_events; /* with aux_stream: host array of two hipEvent_t (hcl_events_create makes
                              them) used for the fork and the join; the library creates no events    */
} hcl_opts_t;

/* One unit of the ring schedule, as hcl_schedule_items reports it. */
typedef struct hcl_work_item {
  int phase;               /* hcl_phase_t                                            */
  int step;                /* 0 .. W-2                                               */
  int rank;                /* the rank doing the work                                */
  int from_rank;           /* its predecessor in the ring, whose block arrives       */
  int block;               /* block index received (and, in RS, reduced)             */
  int send_block;          /* block this rank passes on in the same step             */
  uint64_t chunk;          /* chunk index inside the block                           */
  uint64_t elem_offset;    /* first element, counted from the start of the block     */
  uint64_t elem_count;     /* elements in this chunk                                 */
  uint64_t vec_offset;     /* first element, counted from the start of the full vector */
} hcl_work_item_t;

/*
 * All-Reduce.  send[r] and recv[r] hold `count` elements; afterwards every
 * recv[r] holds the ring-order reduction (operator `op`) over all ranks
 * (bit-identical across ranks).  The vector is cut into W blocks of ceil(count / W) elements; the
 * collective is W-1 Reduce-Scatter steps then W-1 All-Gather steps (Section 1;
 * Appendix B.1 "Communication patterns in DL"; Appendix D.4).
 * In place: recv[r] == send[r] for every r (all ranks or none).  Otherwise
 * no recv buffer may overlap any other buffer, and send[] is left untouched.
 * Needs no workspace.  HOST_STAGED needs opts->host_stage.
 */
hcl_status_t hcl_allreduce_sim(const void *const *send, void *const *recv, int W, size_t count,
                               hcl_dtype_t dtype, hcl_op_t op, size_t chunk_bytes,
                               const hcl_opts_t *opts, void *stream);

/*
 * Reduce-Scatter: the gradient half of ZeRO-2/3 (Appendix D.4, Table
 * "Communication patterns across DeepSpeed ZeRO stages").  send[r] holds
 * W * recvcount elements, recv[r] receives recvcount elements = block r of the
 * ring-order reduction (operator `op`).
 * In place: recv[r] == send[r] + r * recvcount (elements) for every r; the
 * other blocks of send[r] are then used for partial sums and left undefined.
 * Out of place with the STEPWISE schedule and W > 2, partial sums live in
 * opts->workspace (hcl_workspace_bytes); send[] is left untouched.
 */
hcl_status_t hcl_reduce_scatter_sim(const void *const *send, void *const *recv, int W, size_t recvcount,
                                    hcl_dtype_t dtype, hcl_op_t op, size_t chunk_bytes,
                                    const hcl_opts_t *opts, void *stream);

/*
 * Reduce-Scatter for callers that cannot allocate device memory or bring a
 * workspace along: code running under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, semantics and result bits
 * as hcl_reduce_scatter_sim, except that opts->workspace is ignored: where that
 * entry point needs a workspace (out of place, STEPWISE, DIRECT, W > 2) the
 * partial sums live in an array of HCL_STATIC_SCRATCH_BYTES (32 MiB) that is
 * part of the library's code object -- every GPU the process uses holds one copy
 * until the process ends.  The call allocates and frees nothing.  A call whose
 * partial sums need more than that (hcl_workspace_bytes(HCL_KIND_REDUCE_SCATTER,
 * ...) > HCL_STATIC_SCRATCH_BYTES, i.e. blocks beyond about 32 MiB / W) returns
 * HCL_ERR_WORKSPACE and launches nothing.  Nothing in the array has to be
 * cleared between calls (each partial is written before it is read), but all
 * calls on one GPU share it: two such calls may not overlap in time on the same
 * GPU (different streams, or graphs replayed concurrently) -- they would race.
 */
hcl_status_t hcl_reduce_scatter_sim_static(const void *const *send, void *const *recv, int W,
                                           size_t recvcount, hcl_dtype_t dtype, hcl_op_t op,
                                           size_t chunk_bytes, const hcl_opts_t *opts, void *stream);
/* HCL_STATIC_SCRATCH_BYTES as the built library has it. */
size_t hcl_static_scratch_bytes(void);

/*
 * All-Gather: the parameter half of ZeRO-3 (same passages).  send[r] holds
 * sendcount elements, recv[r] receives W * sendcount elements, block q equal
 * to send[q].  In place: send[r] == recv[r] + r * sendcount for every r.
 */
hcl_status_t hcl_all_gather_sim(const void *const *send, void *const *recv, int W, size_t sendcount,
                                hcl_dtype_t dtype, size_t chunk_bytes,
                                const hcl_opts_t *opts, void *stream);

/*
 * Reduce to `root` along the ring -- one of the further collectives the
 * paper evaluates (Appendix E.1 "Other Collective Communication Operations").
 * send[r] holds `count` elements for every rank; only recv[root] is written
 * (the other recv entries are ignored and may be NULL).  The rank after the
 * root sends its vector on, every following rank combines its own with one hop, the
 * chain ends at the root: the reduction runs in the order next(root), ..., root, i.e.
 * as block `root` of the All-Reduce does.  In place: recv[root] == send[root].
 * STEPWISE (W - 1 launches) with W > 2 keeps the travelling partial in
 * opts->workspace (hcl_workspace_bytes with HCL_KIND_REDUCE: one slot of the
 * vector); FUSED is one launch and needs none.  DIRECT transport only.
 */
hcl_status_t hcl_reduce_sim(const void *const *send, void *const *recv, int W, size_t count,
                            hcl_dtype_t dtype, hcl_op_t op, int root, size_t chunk_bytes,
                            const hcl_opts_t *opts, void *stream);

/*
 * Broadcast from `root` along the ring (same passage).  Only send[root] is read
 * (`count` elements; other send entries are ignored and may be NULL); every
 * recv[r] receives a copy, each rank copying what its predecessor holds
 * (STEPWISE, W - 1 launches) or all at once from the root (FUSED, one launch).
 * In place: recv[root] == send[root].  DIRECT transport only.
 */
hcl_status_t hcl_broadcast_sim(const void *const *send, void *const *recv, int W, size_t count,
                               hcl_dtype_t dtype, int root, size_t chunk_bytes,
                               const hcl_opts_t *opts, void *stream);

/*
 * All-to-All (same passage; the expert-parallel exchange of Appendix B.1).
 * send[r] and recv[r] hold W blocks of `count` elements; block q of recv[r]
 * becomes block r of send[q].  No in-place form: any overlap is HCL_ERR_ALIAS.
 * STEPWISE: W launches, launch k moving the blocks every rank receives from the
 * rank k places before it in the ring; FUSED: the same copies packed into as few
 * launches as the per-launch segment table (32 entries) allows.  DIRECT only.
 */
hcl_status_t hcl_alltoall_sim(const void *const *send, void *const *recv, int W, size_t count,
                              hcl_dtype_t dtype, size_t chunk_bytes,
                              const hcl_opts_t *opts, void *stream);

/* Device scratch a call of this kind and shape needs in opts->workspace: where the
 * travelling partial sums live when they can live in neither send[] nor recv[]
 * (the library's counterpart of the vendor library's internal buffers, Section
 * 4.2).  `count` is the count argument of that kind's entry point.
 *   - STEPWISE, DIRECT Reduce-Scatter with W > 2: W slots, one per block, in
 *     which the block's travelling partial sum is read, combined and written
 *     back step after step; the figure is the out-of-place one (the in-place
 *     form keeps its partial sums in send[] and ignores the workspace; this
 *     query cannot know which form the call will be).
 *   - STEPWISE Reduce with W > 2: 1 slot.
 *   - everything else: 0.
 * A slot is one block (Reduce: the vector) rounded up to 256 bytes, plus 4 KiB.
 * opts->workspace must be 16-byte aligned.  Returns 0 on invalid arguments too. */
size_t hcl_workspace_bytes(int kind, int W, size_t count, hcl_dtype_t dtype, size_t chunk_bytes,
                           const hcl_opts_t *opts);

/* Pinned host memory the HOST_STAGED transport needs in opts->host_stage (the
 * staging buffers of the host-staged path, Section 2.1 "Inter-node communication
 * and RDMA"; Appendix F.1): two inbox slots per rank, each one block rounded up to
 * 256 bytes, plus 4 KiB.  0 for the DIRECT transport.  opts->host_stage must be
 * 16-byte aligned. */
size_t hcl_host_stage_bytes(int kind, int W, size_t count, hcl_dtype_t dtype, size_t chunk_bytes,
                            const hcl_opts_t *opts);

/* Ring chunk scheduler, host only: the message partitioning that the paper's
 * library leaves to the vendor library's host side (Section 4.2), written out
 * for the textbook ring.  Which block `rank` sends and which it receives at
 * (phase, step): Reduce-Scatter step s sends
 * ring[(pos - s - 1) mod W] and receives (and reduces) ring[(pos - s - 2) mod W];
 * All-Gather step s sends ring[(pos - s) mod W] and receives
 * ring[(pos - s - 1) mod W], pos being the rank's index in ring[]. */
hcl_status_t hcl_ring_step(int W, const int *ring, int phase, int step, int rank,
                           int *send_block, int *recv_block);

/* The same partitioning (Section 4.2) down to chunks: enumerates the work items
 * of one ring step (every rank, every chunk, chunk-major, then ring position).
 * This is a description of the schedule for inspection, tests and the HCL_DEBUG
 * dump; no kernel consumes the list -- a launch carries one segment per rank and
 * its workgroups derive (chunk, rank, offset) from their tile index.  For a vector of W blocks of
 * `block_elems` elements where the last block may be shorter: `count` is the
 * full vector length (All-Reduce: count; RS / AG: W * per-rank count).
 * Writes at most max_items items and always reports the total in *n_items.
 * Host only. */
hcl_status_t hcl_schedule_items(int W, const int *ring, size_t count, hcl_dtype_t dtype,
                                size_t chunk_bytes, int phase, int step,
                                hcl_work_item_t *items, size_t max_items, size_t *n_items);

/* Measurement helpers: thin wrappers over hipEventCreate / hipEventDestroy /
 * hipEventElapsedTime so that a caller without HIP headers can time launches
 * on the stream they run on (see hcl_opts_t.events). */
hcl_status_t hcl_events_create(int n, void **events_out);
hcl_status_t hcl_events_destroy(int n, void *const *events);
hcl_status_t hcl_event_record(void *event, void *stream);
hcl_status_t hcl_event_elapsed_ms(void *start, void *stop, float *ms);

/* Number of compute units of the current device (cached), or -1. */
int hcl_device_cu_count(void);

const char *hcl_status_string(hcl_status_t s);
const char *hcl_last_error(void);
int hcl_version(void);

#ifdef __cplusplus
}
#endif
#endif /* HCL_H_ */

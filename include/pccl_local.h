/*
 * pccl_local.h -- C ABI of libpccl_local.so: the on-GPU work one rank does inside the
 * two-level (hierarchical) reduce-scatter, all-gather and all-reduce of PCCL
 * ("The Big Send-off: Scalable and Performant Collectives for Deep Learning").
 *
 * The library covers the paper's two device-local kernels:
 *   - the GPU vector-reduction kernel that sums received buffers into the owned shard
 *     (Section III-B; Section IV-B, PCCL_ring / PCCL_rec), generalised to many sources;
 *   - the device-local shuffle (a chunk transpose) between the two-level layout and
 *     rank order (Section IV-A, step 3 of the hierarchical all-gather, and its inverse
 *     for the reduce-scatter).
 * Transport (MPI / RCCL messages) is not part of it: every buffer a rank would have
 * received is simply a region of this GPU's memory.
 *
 * Vocabulary (Section IV-A): N = nodes, M = gpus_per_node, P = N*M ranks,
 * rank r = n*M + g for node n and local id g.  A message of m bytes per rank is P chunks;
 * "rank order" is [node][gpu][chunk], "hierarchical order" is [gpu][node][chunk].
 *
 * Common rules for every entry point
 *   Pointers   All data pointers are DEVICE pointers (hipMalloc'ed memory of the current
 *              device) unless a parameter is explicitly called "host".  Arrays of pointers
 *              (d_srcs, d_inter, d_slots) and descriptor tables (d_buckets) are themselves
 *              device-resident.
 *   Ownership  The caller owns every buffer, scratch included.  The library allocates
 *              nothing, frees nothing and keeps no pointer after the call returns.  (One
 *              entry point, pccl_reduce_scatter_local_static, keeps its scratch in a static
 *              device array of the library instead of taking it from the caller.)
 *   Stream     Work is only enqueued on `stream` (a hipStream_t; NULL = the default
 *              stream).  No call synchronises the device; results are valid once the
 *              caller has synchronised the stream.
 *   Errors     A status code is returned; nothing throws or aborts.  All argument checks
 *              run on the host before the first HIP call, so a rejected call has no side
 *              effect.  A failed launch is reported as PCCL_ERR_HIP.
 *   Checked    Raw pointers cannot be checked for free, and a kernel given a host pointer
 *              or a range longer than its allocation takes a GPU memory fault.  With the
 *              environment variable PCCL_CHECK_POINTERS=1 (read when the library is loaded,
 *              see pccl_diag_reload_env) every call, once its arguments
 *              have passed the checks above, asks the HIP runtime whether each range the
 *              host can see lies inside ONE allocation that kernels can address (device,
 *              managed or pinned host memory) and returns PCCL_ERR_ADDRESS instead of
 *              launching when one does not; the device-resident pointer arrays and
 *              descriptor tables are checked as ranges only.  PCCL_CHECK_POINTERS=2 also
 *              copies those arrays back on `stream`, WAITS for the stream, checks every
 *              pointer in them and compares a descriptor table with its host mirror
 *              (PCCL_ERR_INVALID when they differ); on a stream that is being captured
 *              into a graph it behaves as level 1.  About
 *              a microsecond per range; off when unset or 0.  Memory handed out by a
 *              caching sub-allocator is checked against the block it was carved from.
 *   Empty      count == 0 / chunk_bytes == 0 / chunk_count == 0 / nbuckets == 0 succeed
 *              and launch nothing.
 *   Alignment  Any element-aligned pointer is accepted.  Pointers, strides and chunk sizes
 *              that are multiples of 16 bytes take the 128-bit path; others take a slower
 *              element-wise path with identical results.  Multiples of 128 bytes (a cache
 *              line) are fastest: a shuffle whose chunk size is only a multiple of 16 loses
 *              about 5 % to source reads that straddle lines (10 % with odd multiples of 2
 *              bytes, 18 % with odd byte counts), a two-level reduce-scatter
 *              share 5-10 %, and one whose chunks hold an odd number of 16-bit elements
 *              about 20 % (every other chunk then starts in the middle of a 32-bit word).
 *   Sizes      Counts and byte sizes are size_t; buffers beyond 4 GiB are fine.  The largest
 *              launches: a reduction of up to 2^31 * 65535 / 256 vector tiles (far beyond
 *              device memory), a permutation with chunks below 64 GiB; beyond that
 *              PCCL_ERR_INVALID is returned.
 *   Aliasing   Outputs must not overlap inputs.  Where both ranges are visible to the
 *              host (strided forms) an overlap is rejected with PCCL_ERR_OVERLAP; for
 *              pointer-array forms it is undefined behaviour.
 *   Arithmetic Every sum is accumulated in IEEE binary32 with round-to-nearest-even adds,
 *              no FMA, no reassociation, subnormals kept; the accumulator starts from the
 *              first source.  bf16 / fp16 -> fp32 widening is exact; fp32 -> bf16 / fp16
 *              rounds to nearest even, overflows to infinity and keeps subnormals (a NaN
 *              stays a quiet NaN of the same sign; its payload is unspecified).  Results
 *              are therefore bit-reproducible.
 */
#ifndef PCCL_LOCAL_H
#define PCCL_LOCAL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  PCCL_OK = 0,
  PCCL_ERR_NULL = 1,        /* a required pointer is NULL */
  PCCL_ERR_INVALID = 2,     /* a count, stride, index or size is out of range or overflows */
  PCCL_ERR_UNSUPPORTED = 3, /* unknown dtype, dtype pair or op */
  PCCL_ERR_OVERLAP = 4,     /* an output range overlaps an input range */
  PCCL_ERR_HIP = 5,         /* the HIP runtime refused a launch */
  PCCL_ERR_ADDRESS = 6,     /* checked mode: a range is not inside one reachable allocation */
  PCCL_ERR_SCRATCH = 7      /* the call needs more than the library's static workspace holds */
} pccl_status_t;

/* fp32, bf16 and fp16 (IEEE binary16) elements.  Where an entry point takes an input and an
 * output dtype, the pair is a type with itself or fp32 on one side (bf16 with fp16 is
 * PCCL_ERR_UNSUPPORTED). */
typedef enum { PCCL_F32 = 0, PCCL_BF16 = 1, PCCL_F16 = 2 } pccl_dtype_t;
/* PCCL_SUM: the paper's collectives are sums.  PCCL_AVG (data-parallel training averages
 * gradients, Section II-A): the finished binary32 sum is divided by the number of
 * contributing ranks -- nsrc, or nodes*gpus_per_node -- with one IEEE binary32 division
 * before the output rounding; node partials stay plain sums.  The rank count must not
 * exceed 2^24.  The step-wise entry points (pccl_accumulate and the ring / halving replays)
 * take PCCL_SUM only. */
typedef enum { PCCL_SUM = 0, PCCL_AVG = 1 } pccl_op_t;
typedef void* pccl_stream_t;             /* a hipStream_t */

/* One bucket of a batched two-level reduce-scatter share (see
 * pccl_reduce_scatter_local_batched).  All pointers are device pointers. */
typedef struct {
  void* shard;               /* out: [chunk_count] elements of io_dt                    */
  void* partial;             /* out: [nodes][chunk_count] elements of io_dt             */
  const void* intra_base;    /* in : piece g' at intra_base + g'*intra_stride_bytes,    */
  size_t intra_stride_bytes; /*      each piece [nodes][chunk_count] elements of io_dt  */
  size_t chunk_count;        /* elements per rank-chunk                                 */
} pccl_bucket_t;

/* Flat local reduce -- the GPU vector-reduction kernel of Sections III-B / IV-B applied to
 * nsrc received buffers at once:
 *     dst[e] = ((x_0[e] + x_1[e]) + x_2[e]) + ... + x_{nsrc-1}[e],   e in [0, count)
 * with x_s = (const char*)src_base + s*src_stride_bytes holding `count` elements of in_dt,
 * dst holding `count` elements of out_dt.  nsrc == 1 is a (converting) copy.
 * src_stride_bytes must be >= count*sizeof(in_dt) when nsrc > 1 and a multiple of the
 * element size.  Errors: NULL dst/src_base; nsrc < 1; size overflow; dst overlapping the
 * source span. */
pccl_status_t pccl_local_reduce(void* dst, const void* src_base, size_t src_stride_bytes,
                                int nsrc, size_t count, pccl_dtype_t in_dt,
                                pccl_dtype_t out_dt, pccl_op_t op, pccl_stream_t stream);

/* The same flat sum with the sources given by a device array of nsrc device pointers
 * (d_srcs[s] -> `count` elements of in_dt), summed in array order. */
pccl_status_t pccl_local_reduce_ptrs(void* dst, const void* const* d_srcs, int nsrc,
                                     size_t count, pccl_dtype_t in_dt, pccl_dtype_t out_dt,
                                     pccl_op_t op, pccl_stream_t stream);

/* Two-level sum over a node-major device pointer array, d_srcs[n*gpus_per_node + g] = the
 * chunk contributed by rank (n, g) -- the whole local reduction of one shard of a two-level
 * reduce-scatter / all-reduce (Section IV-A: intra-node phase, then inter-node phase):
 *     t_n    = x[n][0] + x[n][1] + ... + x[n][M-1]        (left to right)
 *     p_n    = t_n rounded through in_dt (identity for fp32 messages)
 *     dst[e] = (p_0 + p_1) + ... + p_{N-1}                  (left to right), stored as out_dt
 * Built for many small chunks (2048 ranks x 64 KB): the per-node sums run in parallel and
 * are staged in LDS, the node order is kept. */
pccl_status_t pccl_local_reduce_ptrs_two_level(void* dst, const void* const* d_srcs, int nodes,
                                               int gpus_per_node, size_t count,
                                               pccl_dtype_t in_dt, pccl_dtype_t out_dt,
                                               pccl_op_t op, pccl_stream_t stream);

/* Pre-shuffle of a reduce-scatter message (inverse of the all-gather shuffle of Section
 * IV-A): rank order [node][gpu][chunk] -> hierarchical order [gpu][node][chunk],
 *     dst chunk (g*N + n) = src chunk (n*M + g),  chunk_bytes bytes each.
 * dst and src hold N*M*chunk_bytes bytes and must not overlap.  Pure byte movement. */
pccl_status_t pccl_hier_pack(void* dst, const void* src, int nodes, int gpus_per_node,
                             size_t chunk_bytes, pccl_stream_t stream);

/* Step 3 of the hierarchical all-gather (Section IV-A, the device-local shuffle):
 * hierarchical order [gpu][node][chunk] -> rank order [node][gpu][chunk],
 *     dst chunk (n*M + g) = src chunk (g*N + n). */
pccl_status_t pccl_hier_unpack(void* dst, const void* src, int nodes, int gpus_per_node,
                               size_t chunk_bytes, pccl_stream_t stream);

/* One GPU's share of a two-level reduce-scatter (Section IV-A: the mirror image of the
 * two-level all-gather, intra-node phase first; reductions on the GPU, Section IV-B).
 *   Phase 1: partial[n][e] = round_io( sum over g' = 0..M-1, in order, of piece_g'[n][e] )
 *            piece_g' = intra_base + g'*intra_stride_bytes, [nodes][chunk_count] of io_dt:
 *            what node-mate g' sent, i.e. its chunks bound for this local id on every node.
 *   Phase 2: shard[e] = round_io( sum over n' = 0..N-1, in order, of inter_n'[e] )
 *            inter_n' = what node n' sent for this node.
 *            d_inter == NULL: inter_n' = partial[n'] (one GPU standing in for all nodes);
 *            else d_inter is a device array of `nodes` device pointers to chunk_count
 *            elements each; slot my_node is ignored and partial[my_node] is used.
 * partial is caller-provided scratch/output: [nodes][chunk_count] of io_dt (it is the
 * buffer that would go on the wire between the phases).  With d_inter given and 1, 2, 4, 8 or
 * 16 GPUs per node, ONE kernel is enqueued: phase 2 needs only the own node's row of the
 * partial, so the blocks that compute that row go straight on to add the received chunks
 * (every row of partial is still written; same bits).  Otherwise, and beyond 16 nodes when
 * the message is too short to cover that longer tail (under about 10 MiB per 16 nodes), two.
 * shard == NULL runs phase 1 only (one kernel; d_inter and my_node are then unused apart from
 * their checks): for callers that finish with pccl_phase2_reassemble_local.
 * Errors: NULLs; nodes/gpus < 1; my_node outside [0, nodes); stride < nodes*chunk bytes;
 * shard or partial overlapping the intra span or each other. */
pccl_status_t pccl_reduce_scatter_local(void* shard, void* partial, const void* intra_base,
                                        size_t intra_stride_bytes, const void* const* d_inter,
                                        int nodes, int gpus_per_node, int my_node,
                                        size_t chunk_count, pccl_dtype_t io_dt, pccl_op_t op,
                                        pccl_stream_t stream);

/* pccl_reduce_scatter_local for callers that cannot allocate device memory -- code running
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc -- and so have
 * no `partial` buffer to hand over: the phase-1 result is kept in a workspace inside the
 * library, a static device array of PCCL_STATIC_SCRATCH_BYTES bytes (one copy on every GPU the
 * library runs on, held until the process ends).  Everything else -- arguments, the
 * kernels, the order of the sums, the bits of `shard` -- is as in pccl_reduce_scatter_local.
 * The call allocates and frees nothing and runs no checked-mode queries, whatever
 * PCCL_CHECK_POINTERS says; its first use on a device asks the runtime for the workspace's
 * address there (no stream work) and keeps it.
 * Limit: nodes*chunk_count*sizeof(io_dt) <= PCCL_STATIC_SCRATCH_BYTES, else PCCL_ERR_SCRATCH
 * (checked on the host before any HIP call, like every other argument error).
 * Every call on a GPU uses that GPU's one workspace and overwrites what the last call left
 * (nothing in it needs clearing: phase 1 writes every element phase 2 reads): two calls whose
 * kernels may run at the same time on one GPU -- different streams, or graph branches -- RACE;
 * keep them in stream order.  The partial cannot be read back by the caller. */
#define PCCL_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
pccl_status_t pccl_reduce_scatter_local_static(void* shard, const void* intra_base,
                                               size_t intra_stride_bytes, const void* const* d_inter,
                                               int nodes, int gpus_per_node, int my_node,
                                               size_t chunk_count, pccl_dtype_t io_dt, pccl_op_t op,
                                               pccl_stream_t stream);

/* The same share without the pre-shuffle: phase 1 reads the node-mates' messages in RANK
 * order, so no pccl_hier_pack pass (one read and one write of the whole message on every
 * GPU, which the paper's timings include as "intra-GPU transposes", Section III-A) is needed.
 * Message g' (what node-mate g' holds: [nodes][gpus_per_node][chunk_count] of io_dt) is
 *     d_msgs == NULL: (const char*)msgs_base + g'*msg_stride_bytes
 *     else          : d_msgs[g']   (device array of gpus_per_node device pointers)
 * and piece_g'[n][e] = message_g'[(n*gpus_per_node + my_gpu)*chunk_count + e]: the chunks
 * bound for local id my_gpu on every node, read through the node stride.  Everything else
 * (partial, shard, d_inter, my_node, order of the sums) is as in pccl_reduce_scatter_local,
 * and the results are bit-identical to packing every message first (shard == NULL: phase 1
 * only, as there).  One kernel when d_inter is given and the messages are strided (d_msgs ==
 * NULL), under the conditions stated there; else one per phase.
 * Errors: as there; my_gpu outside [0, gpus_per_node); nodes > 65535. */
pccl_status_t pccl_reduce_scatter_local_unpacked(void* shard, void* partial, const void* msgs_base,
                                                 size_t msg_stride_bytes,
                                                 const void* const* d_msgs,
                                                 const void* const* d_inter, int nodes,
                                                 int gpus_per_node, int my_node, int my_gpu,
                                                 size_t chunk_count, pccl_dtype_t io_dt,
                                                 pccl_op_t op, pccl_stream_t stream);

/* The all-gather shuffle with the gathered chunks either contiguous in hierarchical order
 * (d_slots == NULL, `src` used; identical to pccl_hier_unpack) or each in its own buffer
 * (d_slots = device array of P device pointers indexed by hierarchical slot g*N + n, `src`
 * ignored):  dst chunk (n*M + g) = slot (g*N + n). */
pccl_status_t pccl_allgather_reassemble(void* dst, const void* src, const void* const* d_slots,
                                        int nodes, int gpus_per_node, size_t chunk_bytes,
                                        pccl_stream_t stream);

/* The tail of one rank's two-level all-reduce in ONE launch (Section IV-A: all-reduce = the
 * two-level reduce-scatter, then the two-level all-gather, whose step 3 is the device-local
 * shuffle; Section III-A: the timings include the intra-GPU transposes): the inter-node phase
 * of the reduce-scatter share and the all-gather shuffle together, the rank's own shard being
 * stored straight at its rank-order place instead of in a buffer that a later pass copies.
 *   dst chunk (my_node*M + my_gpu)[e] = round_io( sum over n' = 0..N-1, in order, of inter_n'[e] )
 *            with inter_n' as in phase 2 of pccl_reduce_scatter_local: partial[n'] when
 *            d_inter == NULL, else d_inter[n'] (slot my_node ignored, partial[my_node] used);
 *            partial is [nodes][chunk_count] of io_dt, the phase-1 result (read only);
 *            op = PCCL_AVG divides this chunk's sum by N*M (the gathered chunks arrive finished).
 *   dst chunk (n*M + g) = slot (g*N + n)  for every other rank (n, g), chunk_count elements
 *            each, the slots contiguous in hierarchical order at `src` (d_slots == NULL) or
 *            each in its own buffer (d_slots: device array of P device pointers, `src` unused).
 *            The rank's own slot, g = my_gpu and n = my_node, is never read.
 * dst holds N*M*chunk_count elements.  The bits of dst are those of
 * pccl_reduce_scatter_local's phase 2 followed by pccl_allgather_reassemble with the shard in the
 * rank's own slot.  Errors: NULL dst / partial / both of src and d_slots; nodes/gpus < 1;
 * my_node or my_gpu out of range; size overflow; dst overlapping partial or src; more than
 * 65535 gpus_per_node or nodes. */
pccl_status_t pccl_phase2_reassemble_local(void* dst, const void* partial, const void* const* d_inter,
                                           const void* src, const void* const* d_slots, int nodes,
                                           int gpus_per_node, int my_node, int my_gpu, size_t chunk_count,
                                           pccl_dtype_t io_dt, pccl_op_t op, pccl_stream_t stream);

/* nbuckets independent two-level reduce-scatter shares (pccl_reduce_scatter_local with
 * d_inter == NULL) in one launch per phase -- the shape of the many reduce-scatters a
 * ZeRO-3 / FSDP step issues (Section II-A, message-size figure).
 * d_buckets: device array of nbuckets descriptors read by the kernels.
 * h_buckets: HOST copy of the same descriptors, used only for argument checks and to size
 * the launch; must be identical to d_buckets.  nodes, gpus_per_node and io_dt are common
 * to the batch.  nbuckets <= PCCL_MAX_BUCKETS.  A bucket with chunk_count == 0 is skipped. */
#define PCCL_MAX_BUCKETS 512
pccl_status_t pccl_reduce_scatter_local_batched(const pccl_bucket_t* d_buckets,
                                                const pccl_bucket_t* h_buckets, int nbuckets,
                                                int nodes, int gpus_per_node,
                                                pccl_dtype_t io_dt, pccl_op_t op,
                                                pccl_stream_t stream);

/* The batched share straight from rank-order messages (the batched form of
 * pccl_reduce_scatter_local_unpacked with d_msgs == NULL and d_inter == NULL): in every bucket
 * intra_base is the first of gpus_per_node rank-order MESSAGES of
 * nodes*gpus_per_node*chunk_count elements, intra_stride_bytes apart, and phase 1 reads chunk
 * (n, my_gpu) of each.  No pre-shuffle of any bucket is needed; results are bit-identical to
 * pccl_hier_pack_batched followed by pccl_reduce_scatter_local_batched.
 * Errors: as there, with the stride checked against a message; my_gpu outside
 * [0, gpus_per_node). */
pccl_status_t pccl_reduce_scatter_local_unpacked_batched(const pccl_bucket_t* d_buckets,
                                                         const pccl_bucket_t* h_buckets,
                                                         int nbuckets, int nodes, int gpus_per_node,
                                                         int my_gpu, pccl_dtype_t io_dt, pccl_op_t op,
                                                         pccl_stream_t stream);

/* One bucket of a batched shuffle: dst and src each hold nodes*gpus_per_node chunks of
 * chunk_bytes bytes and must not overlap.  Device pointers. */
typedef struct {
  void* dst;
  const void* src;
  size_t chunk_bytes;
} pccl_permute_bucket_t;

/* nbuckets independent shuffles in ONE launch -- the all-gathers (parameters) and the
 * reduce-scatter pre-shuffles (gradients) a ZeRO-3 / FSDP step issues by the dozen (Section
 * II-A).  pccl_allgather_reassemble_batched applies pccl_hier_unpack to every bucket
 * (hierarchical order -> rank order), pccl_hier_pack_batched applies pccl_hier_pack (rank
 * order -> hierarchical order).  d_buckets: device array read by the kernel; h_buckets: HOST
 * copy of the same descriptors for the argument checks and the launch size.  nodes and
 * gpus_per_node are common to the batch; a bucket with chunk_bytes == 0 is skipped;
 * nbuckets <= PCCL_MAX_BUCKETS; at most 2^32 - 1 KiB-tiles per call.
 * Errors: NULLs; nodes/gpus < 1; size overflow; a bucket whose dst overlaps its src. */
pccl_status_t pccl_allgather_reassemble_batched(const pccl_permute_bucket_t* d_buckets,
                                                const pccl_permute_bucket_t* h_buckets,
                                                int nbuckets, int nodes, int gpus_per_node,
                                                pccl_stream_t stream);
pccl_status_t pccl_hier_pack_batched(const pccl_permute_bucket_t* d_buckets,
                                     const pccl_permute_bucket_t* h_buckets, int nbuckets,
                                     int nodes, int gpus_per_node, pccl_stream_t stream);

/* The vector-reduction kernel in the paper's literal form (Section III-B: a reduce-scatter
 * from point-to-point messages plus a GPU vector reduction; Section IV-B: PCCL_ring and
 * PCCL_rec schedule their local reduction on the GPU): the buffer a step has just received
 * is added into the local data, in place,
 *     acc[e] = round_io( acc[e] + recv[e] ),   e in [0, count)
 * both buffers holding `count` elements of io_dt; the sum is stored in io_dt because it is
 * what the next message carries.  Errors: NULLs; size overflow; acc overlapping recv. */
pccl_status_t pccl_accumulate(void* acc, const void* recv, size_t count, pccl_dtype_t io_dt,
                              pccl_op_t op, pccl_stream_t stream);

/* npairs independent steps acc_k += recv_k (pccl_accumulate) of different sizes in ONE launch:
 * what a rank runs when several collectives -- the reduce-scatters of many gradient buckets,
 * Section II-A -- reach the same ring or halving step together.  d_pairs: device array read by
 * the kernel; h_pairs: HOST copy of the same descriptors for the argument checks and the launch
 * size.  A pair with count == 0 is skipped; npairs <= PCCL_MAX_BUCKETS.
 * Errors: NULLs; size overflow; an acc range overlapping its own recv, or any range of an
 * earlier pair other than recv with recv (two pairs may read the same received buffer). */
typedef struct {
  void* acc;        /* in/out: count elements of io_dt */
  const void* recv; /* in    : count elements of io_dt */
  size_t count;
} pccl_accumulate_pair_t;
pccl_status_t pccl_accumulate_batched(const pccl_accumulate_pair_t* d_pairs, const pccl_accumulate_pair_t* h_pairs,
                                      int npairs, pccl_dtype_t io_dt, pccl_op_t op, pccl_stream_t stream);

/* One rank's reduction work in a ring reduce-scatter over `nranks` ranks (Section II-B ring;
 * Section IV-B PCCL_ring): every rank sends to rank+1 and receives from rank-1, and rank r
 * ends up owning chunk r.  msg is this rank's message, [nranks][chunk_count] of io_dt,
 * updated in place.  At step s = 0 .. nranks-2 the chunk received from rank-1,
 *     recv_s = (const char*)recv_base + s*recv_stride_bytes   (chunk_count elements),
 * is added into chunk (rank - 2 - s) mod nranks of msg; that chunk is what step s+1 would
 * forward, and after the last step chunk `rank` of msg is the owned shard.  The steps update
 * nranks-1 DIFFERENT chunks, so ONE kernel is enqueued for all of them (every received chunk
 * must be there when it starts); a caller that starts each step as its message arrives calls
 * pccl_accumulate per step instead, with the same bits.
 * Errors: NULLs; nranks < 1; rank outside [0, nranks); recv_stride_bytes < chunk bytes when
 * more than one chunk is received; msg overlapping the recv span. */
pccl_status_t pccl_ring_reduce_scatter_local(void* msg, const void* recv_base,
                                             size_t recv_stride_bytes, int nranks, int rank,
                                             size_t chunk_count, pccl_dtype_t io_dt,
                                             pccl_op_t op, pccl_stream_t stream);

/* One rank's reduction work in a recursive-halving reduce-scatter over nranks = 2^k ranks
 * (Section II-B; Section IV-B PCCL_rec).  At step t = 0 .. k-1 the partner is
 * rank xor (nranks >> (t+1)); the rank keeps the half of its active chunk range that
 * contains `rank` and adds the received copy of that half into it.  msg is
 * [nranks][chunk_count] of io_dt, updated in place; recv holds the received halves back to
 * back: step t's half ([nranks >> (t+1)][chunk_count]) starts at element
 * chunk_count * (nranks - (nranks >> t)), (nranks-1)*chunk_count elements in all.  After the
 * last step chunk `rank` of msg is the owned shard.  The kept ranges are nested, so ONE kernel
 * is enqueued: every chunk of the first kept half is read once, takes the additions of the
 * steps it is part of in registers -- each sum rounded through io_dt exactly as the stored
 * result of a step is -- and is written once (every received half must be there at the start;
 * per step, call pccl_accumulate on the kept range: same bits).
 * Errors: NULLs; nranks not a power of two; rank outside [0, nranks); msg overlapping recv. */
pccl_status_t pccl_halving_reduce_scatter_local(void* msg, const void* recv, int nranks, int rank,
                                                size_t chunk_count, pccl_dtype_t io_dt,
                                                pccl_op_t op, pccl_stream_t stream);

/* ---- closed-form cost model (host arithmetic only, no GPU work) -----------------------------
 * The paper's two cost equations (Section II-B): for p processes and an m-byte buffer, with
 * alpha the start-up latency per message and beta the inverse point-to-point bandwidth,
 *     ring:                         T = alpha*(p-1)   + beta*((p-1)/p)*m        (Eq. 1)
 *     recursive doubling / halving: T = alpha*log2(p) + beta*((p-1)/p)*m        (Eq. 2)
 * They stand in for the learned dispatcher of Section IV-C, whose training set is machine
 * measurements: with one (alpha, beta) pair fitted per algorithm the cheaper algorithm is a
 * closed form.  (With a single shared pair Eq. 2 never loses; the cross-over the paper
 * measures between PCCL_ring and PCCL_rec needs each algorithm's own effective beta.)
 * Both return seconds; NaN for p < 1 or a negative / non-finite argument; pccl_model_rec
 * returns +infinity when p is not a power of two. */
typedef enum { PCCL_ALGO_RING = 0, PCCL_ALGO_REC = 1 } pccl_algo_t;
typedef struct {
  double alpha_ring_s, beta_ring_s_per_byte; /* fitted to the ring implementation      */
  double alpha_rec_s, beta_rec_s_per_byte;   /* fitted to the recursive implementation */
} pccl_link_model_t;
double pccl_model_ring(int p, double m_bytes, double alpha_s, double beta_s_per_byte);
double pccl_model_rec(int p, double m_bytes, double alpha_s, double beta_s_per_byte);
/* *algo = the cheaper algorithm under `model` (the ring on a tie or when p is not a power of
 * two); the two modelled times are stored through t_ring_s / t_rec_s when not NULL (HOST
 * pointers).  Errors: NULL model or algo; arguments the two functions above reject. */
pccl_status_t pccl_choose_algorithm(int p, double m_bytes, const pccl_link_model_t* model,
                                    pccl_algo_t* algo, double* t_ring_s, double* t_rec_s);
/* Modelled time of one two-level collective on an m-byte buffer (Section IV-A): the
 * inter-node algorithm over `nodes` processes on m/gpus_per_node bytes, the intra-node ring
 * over gpus_per_node processes on m bytes, and the device-local kernels as
 * local_bytes / hbm_bytes_per_s (local_bytes = the algorithmic bytes of the transposes and
 * reductions this library runs for the collective).  NaN on invalid arguments. */
double pccl_model_two_level(int nodes, int gpus_per_node, double m_bytes, pccl_algo_t inter_algo,
                            double alpha_inter_s, double beta_inter_s_per_byte,
                            double alpha_intra_s, double beta_intra_s_per_byte,
                            double local_bytes, double hbm_bytes_per_s);

/* The test behind PCCL_CHECK_POINTERS, callable on its own (it launches nothing): PCCL_OK when
 * [ptr, ptr + bytes) lies inside one allocation that kernels of the current device can address
 * or bytes == 0, PCCL_ERR_NULL for NULL with bytes > 0, else PCCL_ERR_ADDRESS. */
pccl_status_t pccl_check_device_range(const void* ptr, size_t bytes);

/* Diagnostics.  The library reads a handful of PCCL_* environment variables (checked mode
 * above; switches that pin a kernel or a block shape for tests and profiler A/B runs) ONCE,
 * when it is loaded; no call looks at the environment afterwards.  This reads them again.
 * Not safe against calls running at the same time on other threads. */
void pccl_diag_reload_env(void);

/* Identity of the sources the library was built from (a hash the build script passes in;
 * "unknown" for a build made without it).  Static string, never NULL. */
const char* pccl_build_id(void);

/* Static, human-readable name of a status code (never NULL). */
const char* pccl_status_string(pccl_status_t status);

#ifdef __cplusplus
}
#endif
#endif /* PCCL_LOCAL_H */

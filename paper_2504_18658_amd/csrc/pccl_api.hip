// C ABI of libpccl_local.so: argument checks on the host, then kernel launches on the
// caller's stream.  Every check runs before the first HIP call, so a rejected call has no
// side effect and the error paths can be exercised on a machine without a GPU.  With
// PCCL_CHECK_POINTERS set, a call that passed those checks then asks the runtime whether every
// range lies inside memory a kernel can reach, and launches only if so.
#include <atomic>

#include "../../include/pccl_local.h"
#include "address_check.h"
#include "kernels.h"
#include "knobs.h"

// Workspace of pccl_reduce_scatter_local_static: the phase-1 result of a share whose caller
// cannot provide (allocate) one.  One copy per GPU the library runs on, held until the process
// ends.  Host code never uses the array's name as an address: the device address is asked for
// once per device and kept.
static __device__ __align__(256) unsigned char scratch[PCCL_STATIC_SCRATCH_BYTES];

static constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device (nullptr when the runtime refuses).
static void* static_scratch() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    return nullptr;
  }
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
      (void)hipGetLastError();
      return nullptr;
    }
    g_scratch_ptr[dev].store(p, std::memory_order_release);  // every thread finds the same address
  }
  return p;
}

namespace {

using pccl::PermuteProblem;
using pccl::ReduceProblem;

inline bool dtype_ok(pccl_dtype_t d) { return d == PCCL_F32 || d == PCCL_BF16 || d == PCCL_F16; }
inline size_t esize(pccl_dtype_t d) { return d == PCCL_F32 ? 4 : 2; }

inline bool mul_ok(size_t a, size_t b, size_t* out) { return !__builtin_mul_overflow(a, b, out); }
inline bool add_ok(size_t a, size_t b, size_t* out) { return !__builtin_add_overflow(a, b, out); }

inline bool elem_aligned(const void* p, size_t es) {
  return (reinterpret_cast<uintptr_t>(p) & (es - 1)) == 0;
}

// [a, a+la) and [b, b+lb) share a byte
inline bool overlaps(const void* a, size_t la, const void* b, size_t lb) {
  if (la == 0 || lb == 0) return false;
  const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
  return x < y + lb && y < x + la;
}

inline pccl_status_t from_hip(hipError_t e) { return e == hipSuccess ? PCCL_OK : PCCL_ERR_HIP; }

// Opt-in address checks of one call: the first failure is kept.
struct AddressChecks {
  int level;
  hipStream_t st;
  pccl_status_t status;
  explicit AddressChecks(pccl_stream_t stream)
      : level(pccl::address_check_level()), st(reinterpret_cast<hipStream_t>(stream)), status(PCCL_OK) {
    if (level > 1) {  // level 2 copies tables back and waits: not possible while the stream is being captured
      hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
      if (hipStreamIsCapturing(st, &capturing) != hipSuccess) (void)hipGetLastError();
      if (capturing != hipStreamCaptureStatusNone) level = 1;
    }
  }
  bool on() const { return level > 0; }
  void range(const void* p, size_t bytes) {
    if (level > 0 && status == PCCL_OK) status = pccl::check_range(p, bytes);
  }
  void pointers(const void* const* d_table, size_t n, size_t offset, size_t bytes_each, long long skip = -1) {
    if (level > 0 && status == PCCL_OK)
      status = pccl::check_pointer_table(d_table, n, offset, bytes_each, skip, level, st);
  }
  void descriptors(const void* d_table, const void* h_table, size_t bytes) {
    if (level > 0 && status == PCCL_OK)
      status = pccl::check_descriptor_table(d_table, h_table, bytes, level, st);
  }
};

ReduceProblem blank_problem() {
  ReduceProblem p;
  p.dst = nullptr;
  p.partial = nullptr;
  p.base = nullptr;
  p.ptrs = nullptr;
  p.override_ptr = nullptr;
  p.stride_n = 0;
  p.stride_g = 0;
  p.count = 0;
  p.src_offset = 0;
  p.row_stride_src = 0;
  p.row_stride_dst = 0;
  p.nodes = 1;
  p.gpus = 1;
  p.override_index = -1;
  p.round_partial = 0;
  p.rows = 1;
  p.row_pad = 0;
  p.keep_cached = 0;
  p.divisor = 0.0f;
  return p;
}

// dtype pairs: a type with itself, or fp32 on one side (never bf16 mixed with fp16)
pccl_status_t check_common(pccl_dtype_t in_dt, pccl_dtype_t out_dt, pccl_op_t op) {
  if (!dtype_ok(in_dt) || !dtype_ok(out_dt)) return PCCL_ERR_UNSUPPORTED;
  if (in_dt != out_dt && in_dt != PCCL_F32 && out_dt != PCCL_F32) return PCCL_ERR_UNSUPPORTED;
  if (op != PCCL_SUM && op != PCCL_AVG) return PCCL_ERR_UNSUPPORTED;
  return PCCL_OK;
}

// op = average divides the finished sum by the number of contributing ranks; the count must
// be exact in binary32
inline bool divisor_ok(pccl_op_t op, size_t ranks) { return op != PCCL_AVG || ranks <= (1u << 24); }
inline float divisor_for(pccl_op_t op, size_t ranks) { return op == PCCL_AVG ? (float)ranks : 0.0f; }

pccl_status_t permute_common(void* dst, const void* src, const void* const* slots, int rows,
                             int cols, size_t chunk_bytes, pccl_stream_t stream) {
  if (dst == nullptr || (src == nullptr && slots == nullptr)) return PCCL_ERR_NULL;
  if (rows < 1 || cols < 1) return PCCL_ERR_INVALID;
  size_t chunks, total;
  if (!mul_ok((size_t)rows, (size_t)cols, &chunks) || chunks > 0x7FFFFFFFull)
    return PCCL_ERR_INVALID;
  if (!mul_ok(chunks, chunk_bytes, &total)) return PCCL_ERR_INVALID;
  if (slots == nullptr && overlaps(dst, total, src, total)) return PCCL_ERR_OVERLAP;
  if (chunk_bytes == 0) return PCCL_OK;
  AddressChecks ck(stream);
  if (ck.on()) {
    ck.range(dst, total);
    if (slots == nullptr)
      ck.range(src, total);
    else
      ck.pointers(slots, chunks, 0, chunk_bytes);
    if (ck.status != PCCL_OK) return ck.status;
  }
  PermuteProblem p;
  p.dst = reinterpret_cast<char*>(dst);
  p.src = reinterpret_cast<const char*>(src);
  p.slots = slots;
  p.chunk_bytes = chunk_bytes;
  p.rows = rows;
  p.cols = cols;
  const hipError_t e = pccl::launch_permute(p, reinterpret_cast<hipStream_t>(stream));
  return e == hipErrorInvalidValue ? PCCL_ERR_INVALID : from_hip(e);
}

// A flat sum (p.nodes == 1, p.gpus sources).  Beyond 16 sources the streaming kernel walks
// them batch after batch with too few loads in flight for short sources; the LDS-staged flat
// kernel then keeps every load of an element slice in flight at once.
hipError_t launch_flat(const ReduceProblem& p, int in_dt, int out_dt, hipStream_t st) {
  ReduceProblem q = p;
  q.nodes = p.gpus;
  q.gpus = 1;
  q.stride_n = p.stride_g;
  q.stride_g = 0;
  if (p.rows == 1 && p.partial == nullptr) {
    const int forced = pccl::knobs().flat_kernel;  // 1 streaming, 2 two-level LDS, 3 flat LDS: pinned for tests
    const bool lds = forced == 0 && pccl::prefer_flat_lds(q, in_dt);
    if (forced == 2 || (lds && pccl::prefer_two_level_for_flat(q, in_dt)))
      return pccl::launch_reduce_two_level_lds(q, in_dt, out_dt, st);
    if (forced == 3 || lds) return pccl::launch_reduce_flat_lds(q, in_dt, out_dt, st);
  }
  return pccl::launch_reduce(p, in_dt, out_dt, st);
}

// phase 2 (inter-node) of a two-level reduce-scatter share: shard[e] = sum over n' of
// inter_n'[e], an N-source flat sum over the partial's rows or over received chunks
pccl_status_t phase2(void* shard, void* partial, const void* const* d_inter, int nodes, int my_node,
                     size_t chunk_count, size_t chunk_bytes, int dt, float divisor, hipStream_t st) {
  ReduceProblem p2 = blank_problem();
  p2.dst = shard;
  p2.count = chunk_count;
  p2.gpus = nodes;
  p2.divisor = divisor;
  if (d_inter == nullptr) {
    p2.base = reinterpret_cast<const char*>(partial);
    p2.stride_g = chunk_bytes;
  } else {
    p2.ptrs = d_inter;
    p2.override_index = my_node;
    p2.override_ptr = reinterpret_cast<const char*>(partial) + (size_t)my_node * chunk_bytes;
  }
  const hipError_t e = launch_flat(p2, dt, dt, st);
  return e == hipErrorInvalidValue ? PCCL_ERR_INVALID : from_hip(e);
}

pccl_status_t permute_batched_common(const pccl_permute_bucket_t* d_buckets,
                                     const pccl_permute_bucket_t* h_buckets, int nbuckets, int rows,
                                     int cols, pccl_stream_t stream) {
  if (nbuckets < 0 || nbuckets > PCCL_MAX_BUCKETS) return PCCL_ERR_INVALID;
  if (nbuckets > 0 && (d_buckets == nullptr || h_buckets == nullptr)) return PCCL_ERR_NULL;
  if (rows < 1 || cols < 1) return PCCL_ERR_INVALID;
  size_t chunks;
  if (!mul_ok((size_t)rows, (size_t)cols, &chunks) || chunks > 0x7FFFFFFFull) return PCCL_ERR_INVALID;
  bool any = false;
  for (int b = 0; b < nbuckets; ++b) {
    const pccl_permute_bucket_t& k = h_buckets[b];
    if (k.chunk_bytes == 0) continue;  // an empty bucket is skipped whatever its pointers are
    if (k.dst == nullptr || k.src == nullptr) return PCCL_ERR_NULL;
    size_t total;
    if (!mul_ok(chunks, k.chunk_bytes, &total)) return PCCL_ERR_INVALID;
    if (overlaps(k.dst, total, k.src, total)) return PCCL_ERR_OVERLAP;
    any = true;
  }
  if (!any) return PCCL_OK;
  AddressChecks ck(stream);
  if (ck.on()) {
    ck.descriptors(d_buckets, h_buckets, (size_t)nbuckets * sizeof(pccl_permute_bucket_t));
    for (int b = 0; b < nbuckets; ++b) {
      ck.range(h_buckets[b].dst, chunks * h_buckets[b].chunk_bytes);
      ck.range(h_buckets[b].src, chunks * h_buckets[b].chunk_bytes);
    }
    if (ck.status != PCCL_OK) return ck.status;
  }
  const hipError_t e = pccl::launch_permute_batched(d_buckets, h_buckets, nbuckets, rows, cols,
                                                    reinterpret_cast<hipStream_t>(stream));
  return e == hipErrorInvalidValue ? PCCL_ERR_INVALID : from_hip(e);
}

// Sizes of one two-level reduce-scatter share, and the checks that do not involve the partial.
struct ShareSizes {
  size_t es, piece_count, piece_bytes, chunk_bytes, span;
};

// (a NULL shard is the caller's business: phase 1 only, where the entry point allows it)
pccl_status_t check_share(const void* shard, const void* intra_base, size_t intra_stride_bytes, int nodes,
                          int gpus_per_node, int my_node, size_t chunk_count, pccl_dtype_t io_dt, pccl_op_t op,
                          ShareSizes* z) {
  if (intra_base == nullptr) return PCCL_ERR_NULL;
  if (pccl_status_t s = check_common(io_dt, io_dt, op)) return s;
  if (nodes < 1 || gpus_per_node < 1 || my_node < 0 || my_node >= nodes) return PCCL_ERR_INVALID;
  if (!divisor_ok(op, (size_t)nodes * (size_t)gpus_per_node)) return PCCL_ERR_INVALID;
  z->es = esize(io_dt);
  if (!mul_ok((size_t)nodes, chunk_count, &z->piece_count) || !mul_ok(z->piece_count, z->es, &z->piece_bytes))
    return PCCL_ERR_INVALID;
  z->chunk_bytes = chunk_count * z->es;
  if (!elem_aligned(shard, z->es) || !elem_aligned(intra_base, z->es)) return PCCL_ERR_INVALID;
  if (gpus_per_node > 1 && (intra_stride_bytes < z->piece_bytes || intra_stride_bytes % z->es != 0))
    return PCCL_ERR_INVALID;
  if (!mul_ok((size_t)(gpus_per_node - 1), gpus_per_node > 1 ? intra_stride_bytes : 0, &z->span) ||
      !add_ok(z->span, z->piece_bytes, &z->span))
    return PCCL_ERR_INVALID;
  if (shard != nullptr && overlaps(shard, z->chunk_bytes, intra_base, z->span)) return PCCL_ERR_OVERLAP;
  return PCCL_OK;
}

// Both phases of a checked share, the phase-1 result going through `partial`.
pccl_status_t launch_share(void* shard, void* partial, const void* intra_base, size_t intra_stride_bytes,
                           const void* const* d_inter, int nodes, int gpus_per_node, int my_node,
                           size_t chunk_count, pccl_dtype_t io_dt, pccl_op_t op, const ShareSizes& z,
                           hipStream_t st) {
  const int dt = io_dt;
  const float divisor = divisor_for(op, (size_t)nodes * (size_t)gpus_per_node);
  // With the other nodes' chunks at hand phase 2 only needs the own node's row of the partial:
  // one launch does both phases (step by step on request, for A/B runs, and for shapes without that form).
  if (d_inter != nullptr && shard != nullptr && pccl::knobs().share_launches != 2) {
    pccl::ShareProblem sp;
    sp.shard = shard;
    sp.partial = partial;
    sp.intra_base = reinterpret_cast<const char*>(intra_base);
    sp.own_src = sp.intra_base + (size_t)my_node * z.chunk_bytes;
    sp.d_inter = d_inter;
    sp.intra_stride = gpus_per_node > 1 ? intra_stride_bytes : 0;
    sp.chunk_count = chunk_count;
    sp.nodes = nodes;
    sp.gpus = gpus_per_node;
    sp.my_node = my_node;
    sp.divisor = divisor;
    const hipError_t e = pccl::launch_share_fused(sp, dt, pccl::knobs().share_launches == 1, st);
    if (e != hipErrorNotSupported) return e == hipErrorInvalidValue ? PCCL_ERR_INVALID : from_hip(e);
  }
  // phase 1 (intra-node): partial[n][e] = sum over g' of piece_g'[n][e], an M-source flat
  // sum over the nodes*chunk_count elements of a piece
  ReduceProblem p1 = blank_problem();
  p1.dst = partial;
  p1.base = reinterpret_cast<const char*>(intra_base);
  p1.stride_g = gpus_per_node > 1 ? intra_stride_bytes : 0;
  p1.count = z.piece_count;
  p1.gpus = gpus_per_node;
  const hipError_t e = launch_flat(p1, dt, dt, st);
  if (e != hipSuccess) return e == hipErrorInvalidValue ? PCCL_ERR_INVALID : PCCL_ERR_HIP;
  if (shard == nullptr) return PCCL_OK;  // phase 1 only
  return phase2(shard, partial, d_inter, nodes, my_node, chunk_count, z.chunk_bytes, dt, divisor, st);
}

}  // namespace

extern "C" {

pccl_status_t pccl_local_reduce(void* dst, const void* src_base, size_t src_stride_bytes,
                                int nsrc, size_t count, pccl_dtype_t in_dt,
                                pccl_dtype_t out_dt, pccl_op_t op, pccl_stream_t stream) {
  if (dst == nullptr || src_base == nullptr) return PCCL_ERR_NULL;
  if (pccl_status_t s = check_common(in_dt, out_dt, op)) return s;
  if (nsrc < 1 || !divisor_ok(op, (size_t)nsrc)) return PCCL_ERR_INVALID;
  const size_t ei = esize(in_dt), eo = esize(out_dt);
  size_t in_bytes, out_bytes, span;
  if (!mul_ok(count, ei, &in_bytes) || !mul_ok(count, eo, &out_bytes)) return PCCL_ERR_INVALID;
  if (!elem_aligned(dst, eo) || !elem_aligned(src_base, ei)) return PCCL_ERR_INVALID;
  if (nsrc > 1 && (src_stride_bytes < in_bytes || src_stride_bytes % ei != 0))
    return PCCL_ERR_INVALID;
  if (!mul_ok((size_t)(nsrc - 1), nsrc > 1 ? src_stride_bytes : 0, &span) ||
      !add_ok(span, in_bytes, &span))
    return PCCL_ERR_INVALID;
  if (overlaps(dst, out_bytes, src_base, span)) return PCCL_ERR_OVERLAP;
  if (count == 0) return PCCL_OK;
  AddressChecks ck(stream);
  if (ck.on()) {
    ck.range(dst, out_bytes);
    ck.range(src_base, span);
    if (ck.status != PCCL_OK) return ck.status;
  }
  ReduceProblem p = blank_problem();
  p.dst = dst;
  p.base = reinterpret_cast<const char*>(src_base);
  p.stride_g = nsrc > 1 ? src_stride_bytes : 0;
  p.count = count;
  p.gpus = nsrc;
  p.divisor = divisor_for(op, (size_t)nsrc);
  const hipError_t e = launch_flat(p, in_dt, out_dt, reinterpret_cast<hipStream_t>(stream));
  return e == hipErrorInvalidValue ? PCCL_ERR_INVALID : from_hip(e);
}

pccl_status_t pccl_local_reduce_ptrs(void* dst, const void* const* d_srcs, int nsrc,
                                     size_t count, pccl_dtype_t in_dt, pccl_dtype_t out_dt,
                                     pccl_op_t op, pccl_stream_t stream) {
  if (dst == nullptr || d_srcs == nullptr) return PCCL_ERR_NULL;
  if (pccl_status_t s = check_common(in_dt, out_dt, op)) return s;
  if (nsrc < 1 || !divisor_ok(op, (size_t)nsrc)) return PCCL_ERR_INVALID;
  size_t bytes;
  if (!mul_ok(count, esize(in_dt), &bytes) || !mul_ok(count, esize(out_dt), &bytes))
    return PCCL_ERR_INVALID;
  if (!elem_aligned(dst, esize(out_dt))) return PCCL_ERR_INVALID;
  if (count == 0) return PCCL_OK;
  AddressChecks ck(stream);
  if (ck.on()) {
    ck.range(dst, count * esize(out_dt));
    ck.pointers(d_srcs, (size_t)nsrc, 0, count * esize(in_dt));
    if (ck.status != PCCL_OK) return ck.status;
  }
  ReduceProblem p = blank_problem();
  p.dst = dst;
  p.ptrs = d_srcs;
  p.count = count;
  p.gpus = nsrc;
  p.divisor = divisor_for(op, (size_t)nsrc);
  const int ib = in_dt, ob = out_dt;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const hipError_t e = launch_flat(p, ib, ob, st);
  return e == hipErrorInvalidValue ? PCCL_ERR_INVALID : from_hip(e);
}

pccl_status_t pccl_local_reduce_ptrs_two_level(void* dst, const void* const* d_srcs, int nodes,
                                               int gpus_per_node, size_t count,
                                               pccl_dtype_t in_dt, pccl_dtype_t out_dt,
                                               pccl_op_t op, pccl_stream_t stream) {
  if (dst == nullptr || d_srcs == nullptr) return PCCL_ERR_NULL;
  if (pccl_status_t s = check_common(in_dt, out_dt, op)) return s;
  if (nodes < 1 || gpus_per_node < 1) return PCCL_ERR_INVALID;
  size_t ranks, bytes;
  if (!mul_ok((size_t)nodes, (size_t)gpus_per_node, &ranks) || ranks > 0x7FFFFFFFull ||
      !divisor_ok(op, ranks))
    return PCCL_ERR_INVALID;
  if (!mul_ok(count, esize(in_dt), &bytes) || !mul_ok(count, esize(out_dt), &bytes))
    return PCCL_ERR_INVALID;
  if (!elem_aligned(dst, esize(out_dt))) return PCCL_ERR_INVALID;
  if (count == 0) return PCCL_OK;
  AddressChecks ck(stream);
  if (ck.on()) {
    ck.range(dst, count * esize(out_dt));
    ck.pointers(d_srcs, ranks, 0, count * esize(in_dt));
    if (ck.status != PCCL_OK) return ck.status;
  }
  ReduceProblem p = blank_problem();
  p.dst = dst;
  p.ptrs = d_srcs;
  p.count = count;
  p.nodes = nodes;
  p.gpus = gpus_per_node;
  p.round_partial = 1;
  p.divisor = divisor_for(op, ranks);
  const int ib = in_dt, ob = out_dt;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const int forced = pccl::knobs().two_level_kernel;  // 1 streaming, 2 LDS-staged: pinned for tests
  const bool lds = forced == 2 || (forced == 0 && pccl::prefer_lds_two_level(p, ib));
  const hipError_t e = lds ? pccl::launch_reduce_two_level_lds(p, ib, ob, st)
                           : pccl::launch_reduce(p, ib, ob, st);
  return e == hipErrorInvalidValue ? PCCL_ERR_INVALID : from_hip(e);
}

pccl_status_t pccl_hier_pack(void* dst, const void* src, int nodes, int gpus_per_node,
                             size_t chunk_bytes, pccl_stream_t stream) {
  if (src == nullptr) return PCCL_ERR_NULL;
  // src is [node][gpu]: rows = nodes, cols = gpus; dst chunk (g*N + n) = src chunk (n*M + g)
  return permute_common(dst, src, nullptr, nodes, gpus_per_node, chunk_bytes, stream);
}

pccl_status_t pccl_hier_unpack(void* dst, const void* src, int nodes, int gpus_per_node,
                               size_t chunk_bytes, pccl_stream_t stream) {
  if (src == nullptr) return PCCL_ERR_NULL;
  // src is [gpu][node]: rows = gpus, cols = nodes; dst chunk (n*M + g) = src chunk (g*N + n)
  return permute_common(dst, src, nullptr, gpus_per_node, nodes, chunk_bytes, stream);
}

pccl_status_t pccl_allgather_reassemble(void* dst, const void* src, const void* const* d_slots,
                                        int nodes, int gpus_per_node, size_t chunk_bytes,
                                        pccl_stream_t stream) {
  return permute_common(dst, d_slots != nullptr ? nullptr : src, d_slots, gpus_per_node, nodes,
                        chunk_bytes, stream);
}

pccl_status_t pccl_allgather_reassemble_batched(const pccl_permute_bucket_t* d_buckets,
                                                const pccl_permute_bucket_t* h_buckets,
                                                int nbuckets, int nodes, int gpus_per_node,
                                                pccl_stream_t stream) {
  // every src is [gpu][node]: rows = gpus, cols = nodes
  return permute_batched_common(d_buckets, h_buckets, nbuckets, gpus_per_node, nodes, stream);
}

pccl_status_t pccl_hier_pack_batched(const pccl_permute_bucket_t* d_buckets,
                                     const pccl_permute_bucket_t* h_buckets, int nbuckets,
                                     int nodes, int gpus_per_node, pccl_stream_t stream) {
  // every src is [node][gpu]: rows = nodes, cols = gpus
  return permute_batched_common(d_buckets, h_buckets, nbuckets, nodes, gpus_per_node, stream);
}

pccl_status_t pccl_reduce_scatter_local(void* shard, void* partial, const void* intra_base,
                                        size_t intra_stride_bytes, const void* const* d_inter,
                                        int nodes, int gpus_per_node, int my_node,
                                        size_t chunk_count, pccl_dtype_t io_dt, pccl_op_t op,
                                        pccl_stream_t stream) {
  if (partial == nullptr) return PCCL_ERR_NULL;
  ShareSizes z;
  if (pccl_status_t s = check_share(shard, intra_base, intra_stride_bytes, nodes, gpus_per_node, my_node,
                                    chunk_count, io_dt, op, &z))
    return s;
  if (!elem_aligned(partial, z.es)) return PCCL_ERR_INVALID;
  if (overlaps(partial, z.piece_bytes, intra_base, z.span) ||
      (shard != nullptr && overlaps(shard, z.chunk_bytes, partial, z.piece_bytes)))
    return PCCL_ERR_OVERLAP;
  if (chunk_count == 0) return PCCL_OK;
  AddressChecks ck(stream);
  if (ck.on()) {
    if (shard != nullptr) ck.range(shard, z.chunk_bytes);
    ck.range(partial, z.piece_bytes);
    ck.range(intra_base, z.span);
    if (d_inter != nullptr) ck.pointers(d_inter, (size_t)nodes, 0, z.chunk_bytes, my_node);
    if (ck.status != PCCL_OK) return ck.status;
  }
  return launch_share(shard, partial, intra_base, intra_stride_bytes, d_inter, nodes, gpus_per_node, my_node,
                      chunk_count, io_dt, op, z, reinterpret_cast<hipStream_t>(stream));
}

pccl_status_t pccl_reduce_scatter_local_static(void* shard, const void* intra_base,
                                               size_t intra_stride_bytes, const void* const* d_inter,
                                               int nodes, int gpus_per_node, int my_node,
                                               size_t chunk_count, pccl_dtype_t io_dt, pccl_op_t op,
                                               pccl_stream_t stream) {
  if (shard == nullptr) return PCCL_ERR_NULL;  // the partial cannot be read back: there is no phase-1-only form
  ShareSizes z;
  if (pccl_status_t s = check_share(shard, intra_base, intra_stride_bytes, nodes, gpus_per_node, my_node,
                                    chunk_count, io_dt, op, &z))
    return s;
  if (z.piece_bytes > PCCL_STATIC_SCRATCH_BYTES) return PCCL_ERR_SCRATCH;
  if (chunk_count == 0) return PCCL_OK;
  void* partial = static_scratch();
  if (partial == nullptr) return PCCL_ERR_HIP;
  return launch_share(shard, partial, intra_base, intra_stride_bytes, d_inter, nodes, gpus_per_node, my_node,
                      chunk_count, io_dt, op, z, reinterpret_cast<hipStream_t>(stream));
}

pccl_status_t pccl_reduce_scatter_local_unpacked(void* shard, void* partial, const void* msgs_base,
                                                 size_t msg_stride_bytes,
                                                 const void* const* d_msgs,
                                                 const void* const* d_inter, int nodes,
                                                 int gpus_per_node, int my_node, int my_gpu,
                                                 size_t chunk_count, pccl_dtype_t io_dt,
                                                 pccl_op_t op, pccl_stream_t stream) {
  if (partial == nullptr || (msgs_base == nullptr && d_msgs == nullptr)) return PCCL_ERR_NULL;
  if (pccl_status_t s = check_common(io_dt, io_dt, op)) return s;
  if (nodes < 1 || gpus_per_node < 1 || my_node < 0 || my_node >= nodes || my_gpu < 0 ||
      my_gpu >= gpus_per_node || nodes > 65535 ||
      !divisor_ok(op, (size_t)nodes * (size_t)gpus_per_node))
    return PCCL_ERR_INVALID;
  const size_t es = esize(io_dt);
  size_t chunk_bytes, node_bytes, msg_bytes, piece_bytes, span;
  if (!mul_ok(chunk_count, es, &chunk_bytes) ||
      !mul_ok(chunk_bytes, (size_t)gpus_per_node, &node_bytes) ||
      !mul_ok(node_bytes, (size_t)nodes, &msg_bytes) ||
      !mul_ok(chunk_bytes, (size_t)nodes, &piece_bytes))
    return PCCL_ERR_INVALID;
  if (!elem_aligned(shard, es) || !elem_aligned(partial, es)) return PCCL_ERR_INVALID;
  if (shard != nullptr && overlaps(shard, chunk_bytes, partial, piece_bytes)) return PCCL_ERR_OVERLAP;
  if (d_msgs == nullptr) {
    if (!elem_aligned(msgs_base, es)) return PCCL_ERR_INVALID;
    if (gpus_per_node > 1 && (msg_stride_bytes < msg_bytes || msg_stride_bytes % es != 0))
      return PCCL_ERR_INVALID;
    if (!mul_ok((size_t)(gpus_per_node - 1), gpus_per_node > 1 ? msg_stride_bytes : 0, &span) ||
        !add_ok(span, msg_bytes, &span))
      return PCCL_ERR_INVALID;
    if (overlaps(partial, piece_bytes, msgs_base, span) ||
        (shard != nullptr && overlaps(shard, chunk_bytes, msgs_base, span)))
      return PCCL_ERR_OVERLAP;
  }
  if (chunk_count == 0) return PCCL_OK;
  AddressChecks ck(stream);
  if (ck.on()) {
    if (shard != nullptr) ck.range(shard, chunk_bytes);
    ck.range(partial, piece_bytes);
    if (d_msgs == nullptr)
      ck.range(msgs_base, span);
    else
      ck.pointers(d_msgs, (size_t)gpus_per_node, 0, msg_bytes);
    if (d_inter != nullptr) ck.pointers(d_inter, (size_t)nodes, 0, chunk_bytes, my_node);
    if (ck.status != PCCL_OK) return ck.status;
  }
  const int dt = io_dt;
  const float divisor = divisor_for(op, (size_t)nodes * (size_t)gpus_per_node);
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);

  // phase 1 straight from the rank-order messages: row n of the partial sums chunk
  // (n, my_gpu) of every node-mate's message, i.e. rows that are M chunks apart
  ReduceProblem p1 = blank_problem();
  p1.dst = partial;
  p1.count = chunk_count;
  p1.gpus = gpus_per_node;
  p1.rows = nodes;
  p1.row_stride_src = node_bytes;
  p1.row_stride_dst = chunk_bytes;
  if (d_msgs == nullptr) {
    p1.base = reinterpret_cast<const char*>(msgs_base) + (size_t)my_gpu * chunk_bytes;
    p1.stride_g = gpus_per_node > 1 ? msg_stride_bytes : 0;
    // every row of the first message starts on a cache line when the message and the chunk do
    p1.row_pad = (reinterpret_cast<uintptr_t>(msgs_base) % 128 != 0 || chunk_bytes % 128 != 0) ? 1 : 0;
  } else {
    p1.ptrs = d_msgs;
    p1.src_offset = (size_t)my_gpu * chunk_bytes;
    p1.row_pad = 1;  // the messages' addresses are on the device
  }
  // With the other nodes' chunks at hand and strided messages, one launch does both phases: the
  // blocks of row my_node go on to add the received chunks (as in pccl_reduce_scatter_local).
  if (d_inter != nullptr && shard != nullptr && d_msgs == nullptr && pccl::knobs().share_launches != 2) {
    pccl::ShareProblem sp;
    sp.shard = shard;
    sp.partial = partial;
    sp.intra_base = p1.base;
    sp.own_src = p1.base + (size_t)my_node * node_bytes;
    sp.d_inter = d_inter;
    sp.intra_stride = p1.stride_g;
    sp.chunk_count = chunk_count;
    sp.nodes = nodes;
    sp.gpus = gpus_per_node;
    sp.my_node = my_node;
    sp.divisor = divisor;
    const hipError_t f = pccl::launch_share_rows_fused(sp, p1, dt, pccl::knobs().share_launches == 1, st);
    if (f != hipErrorNotSupported) return f == hipErrorInvalidValue ? PCCL_ERR_INVALID : from_hip(f);
  }
  const hipError_t e = pccl::launch_reduce(p1, dt, dt, st);
  if (e != hipSuccess) return e == hipErrorInvalidValue ? PCCL_ERR_INVALID : PCCL_ERR_HIP;
  if (shard == nullptr) return PCCL_OK;  // phase 1 only
  return phase2(shard, partial, d_inter, nodes, my_node, chunk_count, chunk_bytes, dt, divisor, st);
}

pccl_status_t pccl_phase2_reassemble_local(void* dst, const void* partial, const void* const* d_inter,
                                           const void* src, const void* const* d_slots, int nodes,
                                           int gpus_per_node, int my_node, int my_gpu, size_t chunk_count,
                                           pccl_dtype_t io_dt, pccl_op_t op, pccl_stream_t stream) {
  if (dst == nullptr || partial == nullptr || (src == nullptr && d_slots == nullptr)) return PCCL_ERR_NULL;
  if (pccl_status_t s = check_common(io_dt, io_dt, op)) return s;
  if (nodes < 1 || gpus_per_node < 1 || my_node < 0 || my_node >= nodes || my_gpu < 0 || my_gpu >= gpus_per_node)
    return PCCL_ERR_INVALID;
  size_t ranks, chunk_bytes, piece_bytes, total;
  if (!mul_ok((size_t)nodes, (size_t)gpus_per_node, &ranks) || ranks > 0x7FFFFFFFull || !divisor_ok(op, ranks))
    return PCCL_ERR_INVALID;
  const size_t es = esize(io_dt);
  if (!mul_ok(chunk_count, es, &chunk_bytes) || !mul_ok(chunk_bytes, (size_t)nodes, &piece_bytes) ||
      !mul_ok(chunk_bytes, ranks, &total))
    return PCCL_ERR_INVALID;
  if (!elem_aligned(dst, es) || !elem_aligned(partial, es)) return PCCL_ERR_INVALID;
  if (overlaps(dst, total, partial, piece_bytes)) return PCCL_ERR_OVERLAP;
  if (d_slots == nullptr && overlaps(dst, total, src, total)) return PCCL_ERR_OVERLAP;
  if (chunk_count == 0) return PCCL_OK;
  AddressChecks ck(stream);
  if (ck.on()) {
    ck.range(dst, total);
    ck.range(partial, piece_bytes);
    if (d_inter != nullptr) ck.pointers(d_inter, (size_t)nodes, 0, chunk_bytes, my_node);
    if (d_slots == nullptr)
      ck.range(src, total);
    else
      ck.pointers(d_slots, ranks, 0, chunk_bytes, (long long)my_gpu * nodes + my_node);
    if (ck.status != PCCL_OK) return ck.status;
  }
  // inter-node phase: a flat sum of `nodes` chunks into the rank's own chunk of the result
  ReduceProblem p2 = blank_problem();
  p2.dst = reinterpret_cast<char*>(dst) + ((size_t)my_node * gpus_per_node + my_gpu) * chunk_bytes;
  p2.count = chunk_count;
  p2.gpus = nodes;
  p2.divisor = divisor_for(op, ranks);
  if (d_inter == nullptr) {
    p2.base = reinterpret_cast<const char*>(partial);
    p2.stride_g = chunk_bytes;
  } else {
    p2.ptrs = d_inter;
    p2.override_index = my_node;
    p2.override_ptr = reinterpret_cast<const char*>(partial) + (size_t)my_node * chunk_bytes;
  }
  // shuffle: source chunk (g, n) = hierarchical slot g*N + n -> rank-order chunk n*M + g
  PermuteProblem q;
  q.dst = reinterpret_cast<char*>(dst);
  q.src = d_slots != nullptr ? nullptr : reinterpret_cast<const char*>(src);
  q.slots = d_slots;
  q.chunk_bytes = chunk_bytes;
  q.rows = gpus_per_node;
  q.cols = nodes;
  const hipError_t e = pccl::launch_phase2_reassemble(p2, q, my_gpu, my_node, io_dt,
                                                      reinterpret_cast<hipStream_t>(stream));
  return e == hipErrorInvalidValue ? PCCL_ERR_INVALID : from_hip(e);
}

// Both batched shares.  my_gpu < 0: intra_base holds gpus_per_node pre-shuffled pieces of
// nodes*chunk_count elements; my_gpu >= 0: it holds gpus_per_node rank-order messages of
// nodes*gpus_per_node*chunk_count elements.
static pccl_status_t rs_batched_common(const pccl_bucket_t* d_buckets, const pccl_bucket_t* h_buckets,
                                       int nbuckets, int nodes, int gpus_per_node, int my_gpu,
                                       pccl_dtype_t io_dt, pccl_op_t op, pccl_stream_t stream) {
  if (nbuckets < 0 || nbuckets > PCCL_MAX_BUCKETS) return PCCL_ERR_INVALID;
  if (nbuckets > 0 && (d_buckets == nullptr || h_buckets == nullptr)) return PCCL_ERR_NULL;
  if (pccl_status_t s = check_common(io_dt, io_dt, op)) return s;
  if (nodes < 1 || gpus_per_node < 1 || my_gpu >= gpus_per_node) return PCCL_ERR_INVALID;
  if (!divisor_ok(op, (size_t)nodes * (size_t)gpus_per_node)) return PCCL_ERR_INVALID;
  const size_t es = esize(io_dt);
  const size_t per_source_chunks = my_gpu < 0 ? 1 : (size_t)gpus_per_node;  // chunks per node in a source
  bool any = false;
  for (int b = 0; b < nbuckets; ++b) {
    const pccl_bucket_t& k = h_buckets[b];
    if (k.chunk_count == 0) continue;  // an empty bucket is skipped whatever its pointers are
    if (k.shard == nullptr || k.partial == nullptr || k.intra_base == nullptr)
      return PCCL_ERR_NULL;
    size_t piece_count, piece_bytes, source_bytes, span;
    if (!mul_ok((size_t)nodes, k.chunk_count, &piece_count) ||
        !mul_ok(piece_count, es, &piece_bytes) || !mul_ok(piece_bytes, per_source_chunks, &source_bytes))
      return PCCL_ERR_INVALID;
    if (!elem_aligned(k.shard, es) || !elem_aligned(k.partial, es) ||
        !elem_aligned(k.intra_base, es))
      return PCCL_ERR_INVALID;
    if (gpus_per_node > 1 && (k.intra_stride_bytes < source_bytes || k.intra_stride_bytes % es != 0))
      return PCCL_ERR_INVALID;
    if (!mul_ok((size_t)(gpus_per_node - 1), gpus_per_node > 1 ? k.intra_stride_bytes : 0,
                &span) ||
        !add_ok(span, source_bytes, &span))
      return PCCL_ERR_INVALID;
    const size_t chunk_bytes = k.chunk_count * es;
    if (overlaps(k.partial, piece_bytes, k.intra_base, span) ||
        overlaps(k.shard, chunk_bytes, k.intra_base, span) ||
        overlaps(k.shard, chunk_bytes, k.partial, piece_bytes))
      return PCCL_ERR_OVERLAP;
    any = true;
  }
  if (!any) return PCCL_OK;
  AddressChecks ck(stream);
  if (ck.on()) {
    ck.descriptors(d_buckets, h_buckets, (size_t)nbuckets * sizeof(pccl_bucket_t));
    for (int b = 0; b < nbuckets; ++b) {
      const pccl_bucket_t& k = h_buckets[b];
      if (k.chunk_count == 0) continue;
      const size_t piece_bytes = (size_t)nodes * k.chunk_count * es;
      ck.range(k.shard, k.chunk_count * es);
      ck.range(k.partial, piece_bytes);
      ck.range(k.intra_base, (size_t)(gpus_per_node - 1) * (gpus_per_node > 1 ? k.intra_stride_bytes : 0) +
                                 piece_bytes * per_source_chunks);
    }
    if (ck.status != PCCL_OK) return ck.status;
  }
  const hipError_t e =
      pccl::launch_rs_batched(d_buckets, h_buckets, nbuckets, nodes, gpus_per_node, io_dt,
                              divisor_for(op, (size_t)nodes * (size_t)gpus_per_node),
                              reinterpret_cast<hipStream_t>(stream), my_gpu);
  return e == hipErrorInvalidValue ? PCCL_ERR_INVALID : from_hip(e);
}

pccl_status_t pccl_reduce_scatter_local_batched(const pccl_bucket_t* d_buckets,
                                                const pccl_bucket_t* h_buckets, int nbuckets,
                                                int nodes, int gpus_per_node,
                                                pccl_dtype_t io_dt, pccl_op_t op,
                                                pccl_stream_t stream) {
  return rs_batched_common(d_buckets, h_buckets, nbuckets, nodes, gpus_per_node, -1, io_dt, op, stream);
}

pccl_status_t pccl_reduce_scatter_local_unpacked_batched(const pccl_bucket_t* d_buckets,
                                                         const pccl_bucket_t* h_buckets, int nbuckets,
                                                         int nodes, int gpus_per_node, int my_gpu,
                                                         pccl_dtype_t io_dt, pccl_op_t op,
                                                         pccl_stream_t stream) {
  if (my_gpu < 0) return PCCL_ERR_INVALID;
  return rs_batched_common(d_buckets, h_buckets, nbuckets, nodes, gpus_per_node, my_gpu, io_dt, op, stream);
}

pccl_status_t pccl_accumulate(void* acc, const void* recv, size_t count, pccl_dtype_t io_dt,
                              pccl_op_t op, pccl_stream_t stream) {
  if (acc == nullptr || recv == nullptr) return PCCL_ERR_NULL;
  if (pccl_status_t s = check_common(io_dt, io_dt, op)) return s;
  if (op != PCCL_SUM) return PCCL_ERR_UNSUPPORTED;  // a step adds; scaling belongs to the last store
  const size_t es = esize(io_dt);
  size_t bytes;
  if (!mul_ok(count, es, &bytes)) return PCCL_ERR_INVALID;
  if (!elem_aligned(acc, es) || !elem_aligned(recv, es)) return PCCL_ERR_INVALID;
  if (overlaps(acc, bytes, recv, bytes)) return PCCL_ERR_OVERLAP;
  AddressChecks ck(stream);
  if (ck.on()) {
    ck.range(acc, bytes);
    ck.range(recv, bytes);
    if (ck.status != PCCL_OK) return ck.status;
  }
  const hipError_t e = pccl::launch_accumulate(acc, recv, count, io_dt,
                                               reinterpret_cast<hipStream_t>(stream));
  return e == hipErrorInvalidValue ? PCCL_ERR_INVALID : from_hip(e);
}

pccl_status_t pccl_accumulate_batched(const pccl_accumulate_pair_t* d_pairs, const pccl_accumulate_pair_t* h_pairs,
                                      int npairs, pccl_dtype_t io_dt, pccl_op_t op, pccl_stream_t stream) {
  if (npairs < 0 || npairs > PCCL_MAX_BUCKETS) return PCCL_ERR_INVALID;
  if (npairs > 0 && (d_pairs == nullptr || h_pairs == nullptr)) return PCCL_ERR_NULL;
  if (pccl_status_t s = check_common(io_dt, io_dt, op)) return s;
  if (op != PCCL_SUM) return PCCL_ERR_UNSUPPORTED;
  const size_t es = esize(io_dt);
  bool any = false;
  for (int b = 0; b < npairs; ++b) {
    const pccl_accumulate_pair_t& k = h_pairs[b];
    if (k.count == 0) continue;  // an empty pair is skipped whatever its pointers are
    if (k.acc == nullptr || k.recv == nullptr) return PCCL_ERR_NULL;
    size_t bytes;
    if (!mul_ok(k.count, es, &bytes)) return PCCL_ERR_INVALID;
    if (!elem_aligned(k.acc, es) || !elem_aligned(k.recv, es)) return PCCL_ERR_INVALID;
    if (overlaps(k.acc, bytes, k.recv, bytes)) return PCCL_ERR_OVERLAP;
    for (int a = 0; a < b; ++a) {  // two pairs that update the same elements would race
      const pccl_accumulate_pair_t& j = h_pairs[a];
      if (j.count != 0 && (overlaps(k.acc, bytes, j.acc, j.count * es) || overlaps(k.acc, bytes, j.recv, j.count * es) ||
                           overlaps(k.recv, bytes, j.acc, j.count * es)))
        return PCCL_ERR_OVERLAP;
    }
    any = true;
  }
  if (!any) return PCCL_OK;
  AddressChecks ck(stream);
  if (ck.on()) {
    ck.descriptors(d_pairs, h_pairs, (size_t)npairs * sizeof(pccl_accumulate_pair_t));
    for (int b = 0; b < npairs; ++b) {
      ck.range(h_pairs[b].acc, h_pairs[b].count * es);
      ck.range(h_pairs[b].recv, h_pairs[b].count * es);
    }
    if (ck.status != PCCL_OK) return ck.status;
  }
  const hipError_t e = pccl::launch_accumulate_batched(d_pairs, h_pairs, npairs, io_dt,
                                                       reinterpret_cast<hipStream_t>(stream));
  return e == hipErrorInvalidValue ? PCCL_ERR_INVALID : from_hip(e);
}

pccl_status_t pccl_ring_reduce_scatter_local(void* msg, const void* recv_base,
                                             size_t recv_stride_bytes, int nranks, int rank,
                                             size_t chunk_count, pccl_dtype_t io_dt,
                                             pccl_op_t op, pccl_stream_t stream) {
  if (msg == nullptr || recv_base == nullptr) return PCCL_ERR_NULL;
  if (pccl_status_t s = check_common(io_dt, io_dt, op)) return s;
  if (op != PCCL_SUM) return PCCL_ERR_UNSUPPORTED;
  if (nranks < 1 || rank < 0 || rank >= nranks) return PCCL_ERR_INVALID;
  const size_t es = esize(io_dt);
  size_t chunk_bytes, msg_bytes, span;
  if (!mul_ok(chunk_count, es, &chunk_bytes) || !mul_ok(chunk_bytes, (size_t)nranks, &msg_bytes))
    return PCCL_ERR_INVALID;
  if (!elem_aligned(msg, es) || !elem_aligned(recv_base, es)) return PCCL_ERR_INVALID;
  const int steps = nranks - 1;
  if (steps > 1 && (recv_stride_bytes < chunk_bytes || recv_stride_bytes % es != 0))
    return PCCL_ERR_INVALID;
  if (!mul_ok((size_t)(steps > 1 ? steps - 1 : 0), steps > 1 ? recv_stride_bytes : 0, &span) ||
      !add_ok(span, chunk_bytes, &span))
    return PCCL_ERR_INVALID;
  if (steps > 0 && overlaps(msg, msg_bytes, recv_base, span)) return PCCL_ERR_OVERLAP;
  if (chunk_count == 0) return PCCL_OK;
  AddressChecks ck(stream);
  if (ck.on()) {
    ck.range(msg, msg_bytes);
    if (steps > 0) ck.range(recv_base, span);
    if (ck.status != PCCL_OK) return ck.status;
  }
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  // The steps touch distinct chunks, so one launch takes them all; step by step only on request
  // (A/B runs) or beyond the launch's 65535 rows.
  if (steps > 0 && steps <= 65535 && !pccl::knobs().step_launches) {
    const hipError_t e = pccl::launch_ring_steps(msg, recv_base, steps > 1 ? recv_stride_bytes : 0, chunk_count,
                                                 nranks, rank, io_dt, st);
    return e == hipErrorInvalidValue ? PCCL_ERR_INVALID : from_hip(e);
  }
  for (int s = 0; s < steps; ++s) {
    // rank r forwards chunk r-1 first; what arrives at step s is chunk r-2-s, further reduced
    const int c = ((rank - 2 - s) % nranks + nranks) % nranks;
    const hipError_t e = pccl::launch_accumulate(
        reinterpret_cast<char*>(msg) + (size_t)c * chunk_bytes,
        reinterpret_cast<const char*>(recv_base) + (size_t)s * recv_stride_bytes, chunk_count,
        io_dt, st);
    if (e != hipSuccess) return e == hipErrorInvalidValue ? PCCL_ERR_INVALID : PCCL_ERR_HIP;
  }
  return PCCL_OK;
}

pccl_status_t pccl_halving_reduce_scatter_local(void* msg, const void* recv, int nranks, int rank,
                                                size_t chunk_count, pccl_dtype_t io_dt,
                                                pccl_op_t op, pccl_stream_t stream) {
  if (msg == nullptr || recv == nullptr) return PCCL_ERR_NULL;
  if (pccl_status_t s = check_common(io_dt, io_dt, op)) return s;
  if (op != PCCL_SUM) return PCCL_ERR_UNSUPPORTED;
  if (nranks < 1 || (nranks & (nranks - 1)) != 0 || rank < 0 || rank >= nranks)
    return PCCL_ERR_INVALID;
  const size_t es = esize(io_dt);
  size_t chunk_bytes, msg_bytes;
  if (!mul_ok(chunk_count, es, &chunk_bytes) || !mul_ok(chunk_bytes, (size_t)nranks, &msg_bytes))
    return PCCL_ERR_INVALID;
  if (!elem_aligned(msg, es) || !elem_aligned(recv, es)) return PCCL_ERR_INVALID;
  if (nranks > 1 && overlaps(msg, msg_bytes, recv, msg_bytes - chunk_bytes)) return PCCL_ERR_OVERLAP;
  if (chunk_count == 0) return PCCL_OK;
  AddressChecks ck(stream);
  if (ck.on()) {
    ck.range(msg, msg_bytes);
    ck.range(recv, msg_bytes - chunk_bytes);
    if (ck.status != PCCL_OK) return ck.status;
  }
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  // The kept ranges are nested: one launch reads every chunk of the first kept half once, applies
  // the steps it takes part in in registers and writes it once.  Step by step only on request.
  if (nranks > 1 && (nranks >> 1) <= 65535 && !pccl::knobs().step_launches) {
    const hipError_t e = pccl::launch_halving_steps(msg, recv, chunk_count, nranks, rank, io_dt, st);
    return e == hipErrorInvalidValue ? PCCL_ERR_INVALID : from_hip(e);
  }
  size_t lo = 0, len = (size_t)nranks, recv_off = 0;  // active chunk range, received chunks so far
  for (int dist = nranks >> 1; dist >= 1; dist >>= 1) {
    len >>= 1;
    if (rank & dist) lo += len;  // keep the half that contains this rank
    const hipError_t e = pccl::launch_accumulate(
        reinterpret_cast<char*>(msg) + lo * chunk_bytes,
        reinterpret_cast<const char*>(recv) + recv_off * chunk_bytes, len * chunk_count,
        io_dt, st);
    if (e != hipSuccess) return e == hipErrorInvalidValue ? PCCL_ERR_INVALID : PCCL_ERR_HIP;
    recv_off += len;
  }
  return PCCL_OK;
}

pccl_status_t pccl_check_device_range(const void* ptr, size_t bytes) {
  return pccl::check_range(ptr, bytes);
}

const char* pccl_status_string(pccl_status_t status) {
  switch (status) {
    case PCCL_OK: return "PCCL_OK";
    case PCCL_ERR_NULL: return "PCCL_ERR_NULL: a required pointer is NULL";
    case PCCL_ERR_INVALID: return "PCCL_ERR_INVALID: a count, stride, index or size is out of range";
    case PCCL_ERR_UNSUPPORTED: return "PCCL_ERR_UNSUPPORTED: unknown dtype, dtype pair or reduction op";
    case PCCL_ERR_OVERLAP: return "PCCL_ERR_OVERLAP: an output range overlaps an input range";
    case PCCL_ERR_HIP: return "PCCL_ERR_HIP: the HIP runtime refused a kernel launch";
    case PCCL_ERR_ADDRESS:
      return "PCCL_ERR_ADDRESS: a range is not inside one allocation kernels can reach (checked mode)";
    case PCCL_ERR_SCRATCH:
      return "PCCL_ERR_SCRATCH: the call needs more than the library's static workspace holds";
  }
  return "PCCL: unknown status";
}

}  // extern "C"

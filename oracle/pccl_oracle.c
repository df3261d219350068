/*
 * CPU oracle for the on-GPU local work of PCCL's hierarchical collectives
 * ("The Big Send-off: Scalable and Performant Collectives for Deep Learning").
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow,
 * one-element-at-a-time statement of what each operation computes, used only
 * by the test-suite, the smoke check and the CPU-baseline leg of the
 * benchmark.  It shares no code, header, table or helper with the HIP
 * library and must never be called from the product path.
 *
 * What the paper fixes (Section IV-A, "Hierarchical Collective Algorithms"):
 *   - N nodes x M GPUs per node; inter-node groups join GPUs with the same
 *     local id, intra-node groups join the GPUs of one node.
 *   - all-gather  = inter-node all-gather, intra-node all-gather, then a
 *     device-local shuffle ("transpose kernel") into rank order.
 *   - reduce-scatter = the mirror image: intra-node phase first, inter-node
 *     phase second, with the vector reduction done on the GPU (Section IV-B).
 *   - all-reduce  = two-level reduce-scatter followed by two-level all-gather.
 * What the paper leaves open and this file fixes:
 *   - rank r = n*M + g  (block placement of ranks on nodes);
 *   - summation order: within a node in ascending local id, then across
 *     nodes in ascending node id; the accumulator starts from the first
 *     source (not from 0.0); every add is one IEEE binary32 add;
 *   - the per-node partial is stored in the message dtype (rounded to bf16
 *     with round-to-nearest-even when the message is bf16);
 *   - NaN payloads after bf16 rounding are "parity unpinned": a NaN stays a
 *     quiet NaN with its sign, nothing more is promised;
 *   - the step-wise inter-node algorithms of Section IV-B (ring, recursive
 *     halving) add each received buffer into the local one and forward the
 *     result, so every step's result is stored in the message dtype; ring
 *     direction is rank -> rank+1 with rank r ending up owner of chunk r, and
 *     recursive halving starts at partner distance p/2 (power-of-two p only).
 *     The schedules themselves (which chunk at which step) live in the Python
 *     wrapper and the whole-world simulation next to this file.
 *   - fp16 (IEEE binary16) is accepted next to bf16 as a 16-bit message dtype,
 *     with the same rules (exact widening, round-to-nearest-even narrowing,
 *     overflow to infinity, subnormal halves kept);
 *   - op = average (data-parallel training averages gradients, Section II-A):
 *     the finished binary32 sum is divided by the number of contributing
 *     ranks -- one IEEE binary32 division -- before the output rounding; node
 *     partials stay plain sums.
 *
 * Loops run over elements (optionally split over OpenMP threads, which does
 * not change any per-element order of operations).  Build with
 *   gcc -O2 -std=c11 -fPIC -shared -fopenmp -ffp-contract=off
 * and never with -ffast-math.
 */
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#define ORACLE_F32 0
#define ORACLE_BF16 1
#define ORACLE_F16 2

#define ORACLE_OK 0
#define ORACLE_BAD_ARG 1

/* ---- bf16 <-> f32 ------------------------------------------------------ */

/* bf16 is the upper half of a binary32: widening is exact. */
static float bf16_bits_to_f32(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return f;
}

/* Round a binary32 to the nearest bf16, ties to the even 7-bit mantissa.
 * Written as the textbook rule on (kept half, dropped half): round up when
 * the dropped half is above one half ulp, or exactly one half ulp and the
 * kept half is odd.  A carry out of the mantissa moves into the exponent,
 * so the largest finite values round to infinity, as IEEE prescribes. */
static uint16_t f32_to_bf16_bits(float f) {
  uint32_t u;
  memcpy(&u, &f, sizeof u);
  uint32_t kept = u >> 16;
  uint32_t dropped = u & 0xFFFFu;
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) {
    /* NaN: keep sign, force the quiet bit so the result is still a NaN. */
    return (uint16_t)(kept | 0x0040u);
  }
  if (dropped > 0x8000u || (dropped == 0x8000u && (kept & 1u))) kept += 1u;
  return (uint16_t)kept;
}

uint16_t pccl_oracle_f32_to_bf16(uint32_t f32_bits) {
  float f;
  memcpy(&f, &f32_bits, sizeof f);
  return f32_to_bf16_bits(f);
}

void pccl_oracle_f32_to_bf16_array(uint16_t* out, const uint32_t* f32_bits, size_t n) {
  for (size_t i = 0; i < n; ++i) out[i] = pccl_oracle_f32_to_bf16(f32_bits[i]);
}

/* ---- fp16 (IEEE binary16) <-> f32 --------------------------------------- */

/* binary16: 1 sign, 5 exponent (bias 15), 10 mantissa bits.  Widening is exact. */
static float f16_bits_to_f32(uint16_t h) {
  uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
  uint32_t eh = (h >> 10) & 0x1Fu;
  uint32_t mh = h & 0x3FFu;
  uint32_t u;
  if (eh == 0x1Fu) {
    u = sign | 0x7F800000u | (mh << 13); /* inf, or NaN with its payload moved up */
  } else if (eh != 0) {
    u = sign | ((eh + 112u) << 23) | (mh << 13); /* rebias 15 -> 127 */
  } else if (mh == 0) {
    u = sign; /* +-0 */
  } else {
    /* subnormal: mh * 2^-24; normalise by hand */
    uint32_t e = 113u; /* exponent field of 2^-14 */
    while (!(mh & 0x400u)) {
      mh <<= 1;
      e -= 1u;
    }
    u = sign | (e << 23) | ((mh & 0x3FFu) << 13);
  }
  float f;
  memcpy(&f, &u, sizeof f);
  return f;
}

/* Round a binary32 to the nearest binary16, ties to the even mantissa.  The value is
 * written as sig * 2^k with a 24-bit integer significand; the half keeps the top bits,
 * the rule on (kept, dropped) is the same textbook rule as for bf16.  Results too small
 * for a normal half become subnormal halves (multiples of 2^-24) or zero; a carry out of
 * the mantissa moves into the exponent, so values from 65520 up round to infinity. */
static uint16_t f32_to_f16_bits(float f) {
  uint32_t u;
  memcpy(&u, &f, sizeof u);
  uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
  uint32_t e = (u >> 23) & 0xFFu;
  uint32_t m = u & 0x7FFFFFu;
  if (e == 0xFFu) {
    if (m == 0) return (uint16_t)(sign | 0x7C00u);            /* infinity */
    return (uint16_t)(sign | 0x7E00u | (m >> 13));            /* NaN: quiet bit forced */
  }
  int eh = (int)e - 127 + 15; /* exponent field the half would have */
  if (eh >= 0x1F) return (uint16_t)(sign | 0x7C00u);          /* beyond the half range */
  uint32_t kept, dropped, half_ulp;
  if (eh >= 1) {
    kept = ((uint32_t)eh << 10) | (m >> 13);
    dropped = m & 0x1FFFu;
    half_ulp = 0x1000u;
  } else {
    if (e == 0) return sign;                                   /* fp32 subnormals are far below 2^-25 */
    uint32_t sig = m | 0x800000u;                              /* 1.m as a 24-bit integer */
    int r = 14 - eh;                                           /* |x| = (sig / 2^r) * 2^-24: r bits are dropped */
    if (r > 24) return sign;                                   /* below half of the smallest subnormal */
    kept = sig >> r;
    dropped = sig & ((1u << r) - 1u);
    half_ulp = 1u << (r - 1);
  }
  if (dropped > half_ulp || (dropped == half_ulp && (kept & 1u))) kept += 1u;
  return (uint16_t)(sign | kept);
}

uint16_t pccl_oracle_f32_to_f16(uint32_t f32_bits) {
  float f;
  memcpy(&f, &f32_bits, sizeof f);
  return f32_to_f16_bits(f);
}

void pccl_oracle_f32_to_f16_array(uint16_t* out, const uint32_t* f32_bits, size_t n) {
  for (size_t i = 0; i < n; ++i) out[i] = pccl_oracle_f32_to_f16(f32_bits[i]);
}

void pccl_oracle_f16_to_f32_array(uint32_t* out, const uint16_t* f16_bits, size_t n) {
  for (size_t i = 0; i < n; ++i) {
    float f = f16_bits_to_f32(f16_bits[i]);
    memcpy(&out[i], &f, sizeof f);
  }
}

static float load_as_f32(const void* buf, size_t e, int dt) {
  if (dt == ORACLE_BF16) return bf16_bits_to_f32(((const uint16_t*)buf)[e]);
  if (dt == ORACLE_F16) return f16_bits_to_f32(((const uint16_t*)buf)[e]);
  return ((const float*)buf)[e];
}

static void store_from_f32(void* buf, size_t e, int dt, float v) {
  if (dt == ORACLE_BF16)
    ((uint16_t*)buf)[e] = f32_to_bf16_bits(v);
  else if (dt == ORACLE_F16)
    ((uint16_t*)buf)[e] = f32_to_f16_bits(v);
  else
    ((float*)buf)[e] = v;
}

/* Value of v after a trip through storage of type dt. */
static float round_through(float v, int dt) {
  if (dt == ORACLE_BF16) return bf16_bits_to_f32(f32_to_bf16_bits(v));
  if (dt == ORACLE_F16) return f16_bits_to_f32(f32_to_f16_bits(v));
  return v;
}

static int dtype_ok(int dt) { return dt == ORACLE_F32 || dt == ORACLE_BF16 || dt == ORACLE_F16; }

/* op = average (data-parallel training averages gradients, Section II-A): the finished
 * binary32 sum is divided by the number of contributing ranks, one IEEE binary32
 * division, before it is rounded to the output dtype.  divisor == 0 means plain sum. */
static float finish(float acc, int divisor) {
  if (divisor > 0) return acc / (float)divisor;
  return acc;
}

/* ---- reductions -------------------------------------------------------- */

/* Flat local reduce (the GPU vector-reduction kernel of Sections III-B and
 * IV-B applied to nsrc received buffers):
 *   out[e] = ((x_0[e] + x_1[e]) + x_2[e]) + ... + x_{nsrc-1}[e]
 * accumulated in binary32, sources in the order given. */
int pccl_oracle_flat_reduce(void* out, const void* const* srcs, int nsrc, size_t count,
                            int in_dt, int out_dt, int divisor, int nthreads) {
  if (!out || !srcs || nsrc < 1 || !dtype_ok(in_dt) || !dtype_ok(out_dt) || divisor < 0)
    return ORACLE_BAD_ARG;
  if (nthreads < 1) nthreads = 1;
#pragma omp parallel for num_threads(nthreads) schedule(static)
  for (size_t e = 0; e < count; ++e) {
    float acc = load_as_f32(srcs[0], e, in_dt);
    for (int s = 1; s < nsrc; ++s) acc = acc + load_as_f32(srcs[s], e, in_dt);
    store_from_f32(out, e, out_dt, finish(acc, divisor));
  }
  return ORACLE_OK;
}

/* Two-level sum of nodes*gpus sources, srcs[n*gpus + g] = contribution of
 * rank (n, g) to this shard (Section IV-A: intra-node phase, then inter-node
 * phase):
 *   t_n  = x[n][0] + x[n][1] + ... + x[n][gpus-1]      (left to right)
 *   p_n  = t_n rounded through the message dtype in_dt
 *   out  = (p_0 + p_1) + ... + p_{nodes-1}              (left to right)
 * If partials != NULL it receives p_n as [nodes][count] of in_dt. */
int pccl_oracle_two_level_reduce(void* out, void* partials, const void* const* srcs, int nodes,
                                 int gpus, size_t count, int in_dt, int out_dt, int divisor,
                                 int nthreads) {
  if (!out || !srcs || nodes < 1 || gpus < 1 || !dtype_ok(in_dt) || !dtype_ok(out_dt) ||
      divisor < 0)
    return ORACLE_BAD_ARG;
  if (nthreads < 1) nthreads = 1;
#pragma omp parallel for num_threads(nthreads) schedule(static)
  for (size_t e = 0; e < count; ++e) {
    float acc = 0.0f;
    for (int n = 0; n < nodes; ++n) {
      float t = load_as_f32(srcs[(size_t)n * gpus + 0], e, in_dt);
      for (int g = 1; g < gpus; ++g) t = t + load_as_f32(srcs[(size_t)n * gpus + g], e, in_dt);
      float p = round_through(t, in_dt);
      if (partials) store_from_f32(partials, (size_t)n * count + e, in_dt, p);
      acc = (n == 0) ? p : acc + p;
    }
    store_from_f32(out, e, out_dt, finish(acc, divisor));
  }
  return ORACLE_OK;
}

/* Phase 1 of one GPU's share of a two-level reduce-scatter (intra-node):
 * piece g (g = 0..gpus-1) is what node-mate g sent: [nodes][chunk] elements
 * holding the chunks bound for this GPU's local id on every node.
 *   partial[n][e] = round_io( piece_0[n][e] + piece_1[n][e] + ... ) */
int pccl_oracle_rs_phase1(void* partial, const void* const* pieces, int nodes, int gpus,
                          size_t chunk, int io_dt, int nthreads) {
  if (!partial || !pieces || nodes < 1 || gpus < 1 || !dtype_ok(io_dt)) return ORACLE_BAD_ARG;
  if (nthreads < 1) nthreads = 1;
  size_t total = (size_t)nodes * chunk;
#pragma omp parallel for num_threads(nthreads) schedule(static)
  for (size_t i = 0; i < total; ++i) {
    float t = load_as_f32(pieces[0], i, io_dt);
    for (int g = 1; g < gpus; ++g) t = t + load_as_f32(pieces[g], i, io_dt);
    store_from_f32(partial, i, io_dt, t);
  }
  return ORACLE_OK;
}

/* Phase 2 (inter-node): inter[n] is the chunk received from node n (this
 * node's own partial included, at its own index).
 *   shard[e] = round_out( inter_0[e] + inter_1[e] + ... + inter_{nodes-1}[e] )
 * (divided by `divisor`, the total rank count, first when the op is average) */
int pccl_oracle_rs_phase2(void* shard, const void* const* inter, int nodes, size_t chunk,
                          int io_dt, int out_dt, int divisor, int nthreads) {
  return pccl_oracle_flat_reduce(shard, inter, nodes, chunk, io_dt, out_dt, divisor, nthreads);
}

/* The paper's GPU vector-reduction kernel in its literal form (Section III-B: a
 * reduce-scatter made of point-to-point messages plus a GPU vector reduction; Section
 * IV-B: the local reduction of PCCL_ring and PCCL_rec runs on the GPU): the buffer that
 * has just been received is added into the local data, in place, and the result is what
 * the next message carries, so it is stored in the message dtype:
 *   acc[e] = round_io( acc[e] + recv[e] ) */
int pccl_oracle_accumulate(void* acc, const void* recv, size_t count, int io_dt, int nthreads) {
  if (!acc || !recv || !dtype_ok(io_dt)) return ORACLE_BAD_ARG;
  if (nthreads < 1) nthreads = 1;
#pragma omp parallel for num_threads(nthreads) schedule(static)
  for (size_t e = 0; e < count; ++e) {
    float a = load_as_f32(acc, e, io_dt);
    float r = load_as_f32(recv, e, io_dt);
    store_from_f32(acc, e, io_dt, a + r);
  }
  return ORACLE_OK;
}

/* ---- permutations ------------------------------------------------------ */

/* Pre-shuffle of a reduce-scatter message: rank order [node][gpu][chunk] to
 * hierarchical order [gpu][node][chunk], so that the nodes chunks bound for
 * local id g form one contiguous piece.  Pure byte movement. */
int pccl_oracle_hier_pack(void* dst, const void* src, int nodes, int gpus, size_t chunk_bytes) {
  if (!dst || !src || nodes < 1 || gpus < 1) return ORACLE_BAD_ARG;
  const unsigned char* s = (const unsigned char*)src;
  unsigned char* d = (unsigned char*)dst;
  for (int n = 0; n < nodes; ++n)
    for (int g = 0; g < gpus; ++g)
      for (size_t b = 0; b < chunk_bytes; ++b)
        d[((size_t)g * nodes + n) * chunk_bytes + b] = s[((size_t)n * gpus + g) * chunk_bytes + b];
  return ORACLE_OK;
}

/* Step 3 of the hierarchical all-gather (Section IV-A): after the inter-node
 * and intra-node gathers the buffer holds the chunk of rank (n, g) in slot
 * g*nodes + n; the shuffle moves it to slot n*gpus + g (rank order). */
int pccl_oracle_hier_unpack(void* dst, const void* src, int nodes, int gpus, size_t chunk_bytes) {
  if (!dst || !src || nodes < 1 || gpus < 1) return ORACLE_BAD_ARG;
  const unsigned char* s = (const unsigned char*)src;
  unsigned char* d = (unsigned char*)dst;
  for (int g = 0; g < gpus; ++g)
    for (int n = 0; n < nodes; ++n)
      for (size_t b = 0; b < chunk_bytes; ++b)
        d[((size_t)n * gpus + g) * chunk_bytes + b] = s[((size_t)g * nodes + n) * chunk_bytes + b];
  return ORACLE_OK;
}

/* The same shuffle with every hierarchical slot given by its own pointer:
 * slots[g*nodes + n] -> dst chunk n*gpus + g. */
int pccl_oracle_allgather_reassemble(void* dst, const void* const* slots, int nodes, int gpus,
                                     size_t chunk_bytes) {
  if (!dst || !slots || nodes < 1 || gpus < 1) return ORACLE_BAD_ARG;
  unsigned char* d = (unsigned char*)dst;
  for (int g = 0; g < gpus; ++g)
    for (int n = 0; n < nodes; ++n) {
      const unsigned char* s = (const unsigned char*)slots[(size_t)g * nodes + n];
      for (size_t b = 0; b < chunk_bytes; ++b) d[((size_t)n * gpus + g) * chunk_bytes + b] = s[b];
    }
  return ORACLE_OK;
}

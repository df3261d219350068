/* Drives the C oracle over ragged shapes under AddressSanitizer and UBSan (built and run by
 * tests/test_oracle_sanitizers.py on the CPU): every buffer is allocated at its exact size,
 * so any out-of-bounds index in the oracle's loops aborts the program. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int pccl_oracle_flat_reduce(void*, const void* const*, int, size_t, int, int, int, int);
int pccl_oracle_two_level_reduce(void*, void*, const void* const*, int, int, size_t, int, int, int, int);
int pccl_oracle_rs_phase1(void*, const void* const*, int, int, size_t, int, int);
int pccl_oracle_rs_phase2(void*, const void* const*, int, size_t, int, int, int, int);
int pccl_oracle_accumulate(void*, const void*, size_t, int, int);
int pccl_oracle_hier_pack(void*, const void*, int, int, size_t);
int pccl_oracle_hier_unpack(void*, const void*, int, int, size_t);
int pccl_oracle_allgather_reassemble(void*, const void* const*, int, int, size_t);
void pccl_oracle_f32_to_bf16_array(uint16_t*, const uint32_t*, size_t);
void pccl_oracle_f32_to_f16_array(uint16_t*, const uint32_t*, size_t);
void pccl_oracle_f16_to_f32_array(uint32_t*, const uint16_t*, size_t);

static uint32_t rng = 12345u;
static uint32_t next(void) { rng = rng * 1664525u + 1013904223u; return rng; }

static void* filled(size_t bytes) {
  unsigned char* p = malloc(bytes ? bytes : 1);
  for (size_t i = 0; i < bytes; ++i) p[i] = (unsigned char)(next() >> 24);
  return p;
}

#define CHECK(x) do { if ((x) != 0) { fprintf(stderr, "oracle call failed: %s\n", #x); return 1; } } while (0)

int main(void) {
  const int esz[3] = {4, 2, 2};
  for (int dt = 0; dt < 3; ++dt) {
    for (int nodes = 1; nodes <= 5; nodes += 2) {
      for (int gpus = 1; gpus <= 4; ++gpus) {
        for (size_t count = 0; count <= 37; count += 9) {
          const int ns = nodes * gpus;
          const void** srcs = malloc(sizeof(void*) * (size_t)ns);
          for (int s = 0; s < ns; ++s) srcs[s] = filled(count * (size_t)esz[dt]);
          void* out = filled(count * (size_t)esz[dt]);
          void* out32 = filled(count * 4);
          void* partials = filled((size_t)nodes * count * (size_t)esz[dt]);
          CHECK(pccl_oracle_flat_reduce(out, srcs, ns, count, dt, dt, 0, 2));
          CHECK(pccl_oracle_flat_reduce(out32, srcs, ns, count, dt, 0, ns, 1));
          CHECK(pccl_oracle_two_level_reduce(out, partials, srcs, nodes, gpus, count, dt, dt, ns, 2));
          CHECK(pccl_oracle_two_level_reduce(out, NULL, srcs, nodes, gpus, count, dt, dt, 0, 1));
          CHECK(pccl_oracle_rs_phase2(out, srcs, ns, count, dt, dt, ns, 1));
          CHECK(pccl_oracle_accumulate(out, srcs[0], count, dt, 2));
          /* phase 1: gpus pieces of nodes*count elements */
          const void** pieces = malloc(sizeof(void*) * (size_t)gpus);
          for (int g = 0; g < gpus; ++g) pieces[g] = filled((size_t)nodes * count * (size_t)esz[dt]);
          CHECK(pccl_oracle_rs_phase1(partials, pieces, nodes, gpus, count, dt, 1));
          /* permutations on count-byte chunks */
          void* a = filled((size_t)ns * count);
          void* b = filled((size_t)ns * count);
          void* c = filled((size_t)ns * count);
          CHECK(pccl_oracle_hier_pack(b, a, nodes, gpus, count));
          CHECK(pccl_oracle_hier_unpack(c, b, nodes, gpus, count));
          if (memcmp(a, c, (size_t)ns * count) != 0) { fprintf(stderr, "round trip differs\n"); return 1; }
          const void** slots = malloc(sizeof(void*) * (size_t)ns);
          for (int s = 0; s < ns; ++s) slots[s] = (const unsigned char*)b + (size_t)s * count;
          CHECK(pccl_oracle_allgather_reassemble(c, slots, nodes, gpus, count));
          if (memcmp(a, c, (size_t)ns * count) != 0) { fprintf(stderr, "reassemble differs\n"); return 1; }
          for (int s = 0; s < ns; ++s) free((void*)srcs[s]);
          for (int g = 0; g < gpus; ++g) free((void*)pieces[g]);
          free(srcs); free(pieces); free(slots); free(out); free(out32); free(partials); free(a); free(b); free(c);
        }
      }
    }
  }
  /* conversions over every exponent, both signs, mantissa corners */
  const size_t n = 2 * 256 * 8;
  uint32_t* bits = malloc(n * 4);
  size_t k = 0;
  const uint32_t mant[8] = {0u, 1u, 0x0FFFu, 0x1000u, 0x1001u, 0x7FFFu, 0x8000u, 0x7FFFFFu};
  for (uint32_t s = 0; s < 2; ++s)
    for (uint32_t e = 0; e < 256; ++e)
      for (int m = 0; m < 8; ++m) bits[k++] = (s << 31) | (e << 23) | mant[m];
  uint16_t* h = malloc(n * 2);
  uint32_t* back = malloc(n * 4);
  pccl_oracle_f32_to_bf16_array(h, bits, n);
  pccl_oracle_f32_to_f16_array(h, bits, n);
  pccl_oracle_f16_to_f32_array(back, h, n);
  free(bits); free(h); free(back);
  puts("oracle sanitizer run OK");
  return 0;
}

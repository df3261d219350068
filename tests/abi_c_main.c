/* A plain C99 caller of the library's header: compiled with -pedantic-errors by
 * tests/test_header_c.py, linked against the built library, and run WITHOUT a GPU.  It only
 * reaches host code: status strings, the cost model (Section II-B, Eq. 1 and Eq. 2) and
 * argument checks that reject a call before any HIP call is made. */
#include <math.h>
#include <stdio.h>
#include <string.h>

#include "pccl_local.h"

static int fails = 0;
#define EXPECT(cond)                                                  \
  do {                                                                \
    if (!(cond)) {                                                    \
      printf("FAILED line %d: %s\n", __LINE__, #cond);                \
      ++fails;                                                        \
    }                                                                 \
  } while (0)

int main(void) {
  pccl_link_model_t model;
  pccl_algo_t algo = PCCL_ALGO_RING;
  double t_ring = 0.0, t_rec = 0.0;
  char fake[64];
  pccl_bucket_t bucket;
  pccl_permute_bucket_t pbucket;

  EXPECT(strcmp(pccl_status_string(PCCL_OK), pccl_status_string(PCCL_ERR_INVALID)) != 0);
  EXPECT(pccl_status_string((pccl_status_t)1234) != NULL);

  /* Eq. 1 with p = 4, m = 8: 3 alpha + (3/4) 8 beta; Eq. 2: 2 alpha + (3/4) 8 beta */
  EXPECT(pccl_model_ring(4, 8.0, 1.0, 0.5) == 3.0 + 3.0);
  EXPECT(pccl_model_rec(4, 8.0, 1.0, 0.5) == 2.0 + 3.0);
  EXPECT(isinf(pccl_model_rec(6, 8.0, 1.0, 0.5)));
  EXPECT(isnan(pccl_model_ring(0, 8.0, 1.0, 0.5)));

  model.alpha_ring_s = 1.0;
  model.beta_ring_s_per_byte = 0.5;
  model.alpha_rec_s = 1.0;
  model.beta_rec_s_per_byte = 0.5;
  EXPECT(pccl_choose_algorithm(4, 8.0, &model, &algo, &t_ring, &t_rec) == PCCL_OK);
  EXPECT(algo == PCCL_ALGO_REC && t_ring == 6.0 && t_rec == 5.0);
  EXPECT(pccl_choose_algorithm(4, 8.0, NULL, &algo, NULL, NULL) == PCCL_ERR_NULL);

  /* rejected on the host, before any HIP call: the addresses are never used */
  EXPECT(pccl_local_reduce(NULL, fake, 16, 2, 4, PCCL_F32, PCCL_F32, PCCL_SUM, NULL) == PCCL_ERR_NULL);
  EXPECT(pccl_local_reduce(fake, fake + 32, 16, 0, 4, PCCL_F32, PCCL_F32, PCCL_SUM, NULL) == PCCL_ERR_INVALID);
  EXPECT(pccl_local_reduce(fake, fake + 32, 16, 2, 4, PCCL_BF16, PCCL_F16, PCCL_SUM, NULL) == PCCL_ERR_UNSUPPORTED);
  EXPECT(pccl_local_reduce(fake, fake + 32, 16, 2, 4, PCCL_F32, PCCL_F32, (pccl_op_t)7, NULL) == PCCL_ERR_UNSUPPORTED);
  EXPECT(pccl_local_reduce(fake, fake + 8, 16, 2, 4, PCCL_F32, PCCL_F32, PCCL_SUM, NULL) == PCCL_ERR_OVERLAP);
  EXPECT(pccl_hier_pack(fake, fake + 32, 0, 2, 8, NULL) == PCCL_ERR_INVALID);
  EXPECT(pccl_hier_unpack(fake, fake + 8, 2, 2, 8, NULL) == PCCL_ERR_OVERLAP);
  EXPECT(pccl_accumulate(NULL, fake, 4, PCCL_BF16, PCCL_SUM, NULL) == PCCL_ERR_NULL);
  /* empty problems succeed and launch nothing */
  EXPECT(pccl_local_reduce(fake, fake + 32, 16, 2, 0, PCCL_F32, PCCL_F32, PCCL_SUM, NULL) == PCCL_OK);
  EXPECT(pccl_hier_pack(fake, fake + 32, 2, 2, 0, NULL) == PCCL_OK);
  EXPECT(pccl_reduce_scatter_local_batched(&bucket, &bucket, 0, 2, 2, PCCL_BF16, PCCL_SUM, NULL) == PCCL_OK);
  EXPECT(pccl_hier_pack_batched(&pbucket, &pbucket, 0, 2, 2, NULL) == PCCL_OK);
  EXPECT(PCCL_MAX_BUCKETS >= 40);

  if (fails == 0) printf("abi_c_main: ok\n");
  return fails == 0 ? 0 : 1;
}

// Closed-form choice between the ring and the recursive (doubling / halving) inter-node
// algorithm from the paper's two cost equations (Section II-B, Eqs. 1 and 2), in place of the
// learned dispatcher of Section IV-C, whose training data are machine measurements.  Host
// arithmetic only; nothing here touches the GPU.
#include <cmath>
#include <limits>

#include "../../include/pccl_local.h"

namespace {
inline bool args_ok(int p, double m, double alpha, double beta) {
  return p >= 1 && m >= 0.0 && alpha >= 0.0 && beta >= 0.0 && std::isfinite(m) && std::isfinite(alpha) &&
         std::isfinite(beta);
}
const double kNaN = std::numeric_limits<double>::quiet_NaN();
const double kInf = std::numeric_limits<double>::infinity();
}  // namespace

extern "C" {

double pccl_model_ring(int p, double m_bytes, double alpha_s, double beta_s_per_byte) {
  if (!args_ok(p, m_bytes, alpha_s, beta_s_per_byte)) return kNaN;
  const double steps = (double)(p - 1);
  return alpha_s * steps + beta_s_per_byte * (steps / (double)p) * m_bytes;
}

double pccl_model_rec(int p, double m_bytes, double alpha_s, double beta_s_per_byte) {
  if (!args_ok(p, m_bytes, alpha_s, beta_s_per_byte)) return kNaN;
  if ((p & (p - 1)) != 0) return kInf;  // recursive doubling / halving pairs ranks by bit flips
  int steps = 0;
  while ((1 << steps) < p) ++steps;     // log2 of a power of two, exact
  return alpha_s * (double)steps + beta_s_per_byte * ((double)(p - 1) / (double)p) * m_bytes;
}

pccl_status_t pccl_choose_algorithm(int p, double m_bytes, const pccl_link_model_t* model,
                                    pccl_algo_t* algo, double* t_ring_s, double* t_rec_s) {
  if (model == nullptr || algo == nullptr) return PCCL_ERR_NULL;
  const double a = pccl_model_ring(p, m_bytes, model->alpha_ring_s, model->beta_ring_s_per_byte);
  const double b = pccl_model_rec(p, m_bytes, model->alpha_rec_s, model->beta_rec_s_per_byte);
  if (std::isnan(a) || std::isnan(b)) return PCCL_ERR_INVALID;
  *algo = b < a ? PCCL_ALGO_REC : PCCL_ALGO_RING;
  if (t_ring_s != nullptr) *t_ring_s = a;
  if (t_rec_s != nullptr) *t_rec_s = b;
  return PCCL_OK;
}

double pccl_model_two_level(int nodes, int gpus_per_node, double m_bytes, pccl_algo_t inter_algo,
                            double alpha_inter_s, double beta_inter_s_per_byte,
                            double alpha_intra_s, double beta_intra_s_per_byte,
                            double local_bytes, double hbm_bytes_per_s) {
  if (nodes < 1 || gpus_per_node < 1 || !(local_bytes >= 0.0) || !(hbm_bytes_per_s > 0.0)) return kNaN;
  if (inter_algo != PCCL_ALGO_RING && inter_algo != PCCL_ALGO_REC) return kNaN;
  const double per_group = m_bytes / (double)gpus_per_node;
  const double inter = inter_algo == PCCL_ALGO_RING
                           ? pccl_model_ring(nodes, per_group, alpha_inter_s, beta_inter_s_per_byte)
                           : pccl_model_rec(nodes, per_group, alpha_inter_s, beta_inter_s_per_byte);
  const double intra = pccl_model_ring(gpus_per_node, m_bytes, alpha_intra_s, beta_intra_s_per_byte);
  return inter + intra + local_bytes / hbm_bytes_per_s;
}

}  // extern "C"

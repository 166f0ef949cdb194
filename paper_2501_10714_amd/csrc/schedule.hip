// Pipeline-degree selection of FSMoE Sec. 4 (host code, no GPU work): the linear performance models of
// Sec. 4.1, the seven conditions Q1..Q7 and four cases of Sec. 4.2, and Algorithm 1
// (FindOptimalPipelineDegree) over integer degrees.
#include <cmath>
#include <limits>

#include "common.h"

namespace moe {
namespace {

struct ChunkTimes {
  double a2a, ag, rs, exp;
};

// Sec. 4.1, Eq. (1): time of one of r chunks
ChunkTimes chunk_times(const moe_pipeline_model_t& m, double r) {
  ChunkTimes t;
  t.a2a = m.alpha_a2a + m.n_a2a / r * m.beta_a2a;
  t.ag = m.alpha_ag + m.n_ag / r * m.beta_ag;
  t.rs = m.alpha_rs + m.n_rs / r * m.beta_rs;
  t.exp = m.alpha_exp + m.n_exp / r * m.beta_exp;
  return t;
}

// Sec. 4.2: which case degree r falls into (the four conditions partition all truth assignments of Q1..Q7)
// and the time of the MoE layer in that case.
double pipeline_time(const moe_pipeline_model_t& m, double r, int* which) {
  const ChunkTimes t = chunk_times(m, r);
  const bool q1 = t.a2a > t.ag;
  const bool q2 = r * t.exp > 2.0 * (r - 1.0) * t.a2a;
  const bool q3 = r * t.exp > (r - 1.0) * (t.ag + t.rs);
  const bool q4 = m.t_gar > t.ag + t.rs;
  const bool q5 = m.t_gar > r * t.exp - 2.0 * (r - 1.0) * t.a2a + t.ag + t.rs;
  const bool q6 = m.t_gar > r * t.ag + r * t.rs - 2.0 * (r - 1.0) * t.a2a;
  const bool q7 = m.t_gar > t.ag + t.rs + r * t.exp - 2.0 * (r - 1.0) * t.a2a;
  int c;
  if (q1) c = q2 ? (q5 ? 1 : 2) : (q4 ? 1 : 3);
  else c = q3 ? (q7 ? 1 : 2) : (q6 ? 1 : 4);
  if (which != nullptr) *which = c;
  switch (c) {
    case 1: return 2.0 * r * t.a2a + m.t_gar;                    // inter-node communication dominates
    case 2: return 2.0 * t.a2a + t.ag + t.rs + r * t.exp;        // expert computation dominates
    case 3: return 2.0 * r * t.a2a + t.ag + t.rs;                // AlltoAll dominates
    default: return 2.0 * t.a2a + r * t.ag + r * t.rs;           // intra-node communication dominates
  }
}

bool model_ok(const moe_pipeline_model_t* m) {
  if (m == nullptr) return false;
  const double v[] = {m->alpha_a2a, m->beta_a2a, m->n_a2a, m->alpha_ag, m->beta_ag, m->n_ag, m->alpha_rs,
                      m->beta_rs,   m->n_rs,     m->alpha_exp, m->beta_exp, m->n_exp, m->t_gar};
  for (double x : v)
    if (!(x >= 0.0) || std::isinf(x)) return false;
  return true;
}

}  // namespace
}  // namespace moe

extern "C" {

double moe_pipeline_time(const moe_pipeline_model_t* model, double r, int32_t* which_case) {
  if (!moe::model_ok(model) || !(r >= 1.0)) return std::numeric_limits<double>::quiet_NaN();
  int c = 0;
  const double t = moe::pipeline_time(*model, r, &c);
  if (which_case != nullptr) *which_case = c;
  return t;
}

moe_status_t moe_find_pipeline_degree(const moe_pipeline_model_t* model, int32_t r_max, int32_t* r, double* t_moe,
                                      int32_t* which_case) {
  if (!moe::model_ok(model)) {
    moe::set_error("moe_find_pipeline_degree: model is NULL or has a negative or non-finite coefficient");
    return MOE_ERR_INVALID_ARG;
  }
  if (r_max < 1 || r == nullptr) {
    moe::set_error("moe_find_pipeline_degree: r_max=%d must be >= 1 and r must not be NULL", r_max);
    return MOE_ERR_INVALID_ARG;
  }
  // Algorithm 1: solve(f_i) = the smallest value of case i's closed form over the degrees that satisfy case
  // i's condition (here by enumeration of 1..r_max, which is exact, in place of the paper's SLSQP on a real
  // r); then the best of the four.  Ties go to the smaller degree, then to the lower case number.
  double best_t[5];
  int best_r[5];
  for (int c = 1; c <= 4; ++c) { best_t[c] = std::numeric_limits<double>::infinity(); best_r[c] = 0; }
  for (int d = 1; d <= r_max; ++d) {
    int c = 0;
    const double t = moe::pipeline_time(*model, (double)d, &c);
    if (t < best_t[c]) { best_t[c] = t; best_r[c] = d; }
  }
  int bc = 0;
  for (int c = 1; c <= 4; ++c)
    if (best_r[c] != 0 && (bc == 0 || best_t[c] < best_t[bc] || (best_t[c] == best_t[bc] && best_r[c] < best_r[bc]))) bc = c;
  *r = best_r[bc];
  if (t_moe != nullptr) *t_moe = best_t[bc];
  if (which_case != nullptr) *which_case = bc;
  return MOE_OK;
}

}  // extern "C"

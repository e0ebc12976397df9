// Host-side bit-width decision: Score Engine statistics -> global EMAs -> score -> Map
// (Algorithm 1, the periodic "if" body; Eq. 2, 3, 4, 7, 8 and Section 3.4 of the paper).
// Two passes over the layers, O(L) time, O(1) state.
#include <cmath>
#include <limits>
#include <vector>

#include "stq.h"

namespace {

// Map: a step function of the score.  A score equal to a threshold takes the higher width.
uint8_t map_width(double score, const stq_decide_cfg* cfg) {
  uint32_t above = 0;
  for (uint32_t i = 0; i < cfg->n_thr; ++i) above += (cfg->thr[i] <= score) ? 1u : 0u;
  return cfg->bits[above];
}

}  // namespace

extern "C" int stq_decide_due(uint32_t step, uint32_t update_every) {
  return ((update_every != 0 && step % update_every == 0) || step < 5) ? 1 : 0;
}

extern "C" int stq_decide(stq_decide_state* ema, const stq_layer_stats* stats, uint32_t n,
                          const stq_decide_cfg* cfg, uint32_t step, stq_bits* plan_out,
                          double* score_out) {
  if (!ema || !stats || !cfg || !plan_out || n == 0) return STQ_EINVAL;
  if (cfg->n_thr > 0 && !cfg->thr) return STQ_EINVAL;
  if (!cfg->bits || !(cfg->tau > 0.0) || !(cfg->alpha >= 0.0 && cfg->alpha <= 1.0)) return STQ_EINVAL;
  for (uint32_t l = 0; l < n; ++l) if (stats[l].count == 0) return STQ_EINVAL;

  // pass 1: per-layer factors and their means over the layers
  std::vector<double> fac(3 * static_cast<size_t>(n));
  double sum_n = 0.0, sum_r = 0.0, sum_v = 0.0;
  for (uint32_t l = 0; l < n; ++l) {
    const double cnt = static_cast<double>(stats[l].count);
    const double mean_sq = stats[l].g_sq_sum / cnt;          // v_l   (Eq. 8)
    const double mean_abs = stats[l].g_abs_sum / cnt;
    const double rms = std::sqrt(mean_sq);                   // n_l   (Eq. 2)
    double var;
    if (cfg->flags & STQ_DECIDE_R_ALG1) {
      const double mean = stats[l].g_sum / cnt;
      var = mean_sq - mean * mean;                           // sigma(g)^2, Algorithm 1's form
    } else {
      var = mean_sq - mean_abs * mean_abs;                   // sigma(|g|)^2, Eq. 3
    }
    if (var < 0.0) var = 0.0;
    const double cv = std::sqrt(var) / (mean_abs + cfg->eps);  // r_l
    fac[3 * l] = rms; fac[3 * l + 1] = cv; fac[3 * l + 2] = mean_sq;
    sum_n += rms; sum_r += cv; sum_v += mean_sq;
  }
  const double a = cfg->alpha, inv_n = 1.0 / static_cast<double>(n);
  ema->n_ema = a * (sum_n * inv_n) + (1.0 - a) * ema->n_ema;  // Eq. 4
  ema->r_ema = a * (sum_r * inv_n) + (1.0 - a) * ema->r_ema;
  ema->v_ema = a * (sum_v * inv_n) + (1.0 - a) * ema->v_ema;

  // temporal annealing factor, Eq. 7
  const double s_t = 1.0 + 1.0 / std::cosh(static_cast<double>(step) / cfg->tau);
  const double log_s = std::log2(s_t);

  // pass 2: score and Map
  for (uint32_t l = 0; l < n; ++l) {
    double score = cfg->phi;
    if (!(cfg->flags & STQ_DECIDE_NO_DUAL))
      score += std::log2(fac[3 * l + 1] / (ema->r_ema + cfg->eps)) + std::log2(fac[3 * l] / (ema->n_ema + cfg->eps));
    if (!(cfg->flags & STQ_DECIDE_NO_TEMPORAL)) score += log_s;
    if (!(cfg->flags & STQ_DECIDE_NO_SPATIAL)) score += std::log2(fac[3 * l + 2] / (ema->v_ema + cfg->eps));
    if (score_out) score_out[l] = score;
    plan_out[l].m_bits = map_width(score, cfg);
    plan_out[l].v_bits = map_width(score + cfg->v_offset, cfg);
  }
  return STQ_OK;
}

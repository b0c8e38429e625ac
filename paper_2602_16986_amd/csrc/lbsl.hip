// Load-Balanced Stochastic Length (paper Section 4.1 and Alg. 1 of the appendix) for one process that plays every rank:
// the length sampler that keeps the per-rank attention load sum n^gamma level across a data-parallel job.  Host code
// only; it deals in sequence lengths and never touches a GPU.  The step between ranks that the paper does with an
// all-reduce of one number is a mean over the simulated ranks here.
//
// Stochastic Length (SL) as the paper uses it: with sampling length l_SL, a sequence of n <= l_SL items is left alone, a
// longer one stays whole with probability (l_SL / n)^2 and is cut to l_SL items otherwise.  What the listing leaves to
// its reference, as taken here: SLWeight(n) is that probability; StandardSL_Loads is the expected load of the batch under
// SL; a sequence outside the untruncated set is cut to l_SL if it is longer.  A sequence shorter than l_SL weighs
// n^gamma whether "sampled" or not, so the all-sampled batch is priced at sum min(n, l_SL)^gamma and admitting u costs
// n^gamma - min(n, l_SL)^gamma: the listing's b l_SL^gamma and n^gamma - l_SL^gamma whenever no sequence is shorter than
// l_SL, and a budget that still lets a rank reach the target when many are.
// The weighted permutation without replacement uses exponential clocks on uniforms the caller supplies: key
// -ln(U_u) / p_u, ascending, ties by index.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <limits>
#include <utility>
#include <vector>

#include "../../include/hstu_attn.h"

namespace {

double weight_of(int32_t n, int32_t sl_len) {
  if (n <= sl_len) return 1.0;
  const double q = (double)sl_len / (double)n;
  return q * q;
}
double load_of(int32_t n, double gamma) { return n > 0 ? std::pow((double)n, gamma) : 0.0; }
double expected_load_of(int32_t n, int32_t sl_len, double gamma) {
  const double w = weight_of(n, sl_len);
  return w * load_of(n, gamma) + (1.0 - w) * load_of(std::min(n, sl_len), gamma);
}
bool valid(const hstu_lbsl_config* c) {
  return c->world_size >= 1 && c->warmup_steps >= 1 && c->recal_interval >= 1 && c->sl_len >= 1 && c->gamma > 0.0 && std::isfinite(c->gamma);
}

}  // namespace

extern "C" {

double hstu_lbsl_weight(int32_t n, int32_t sl_len) { return weight_of(n, sl_len); }
double hstu_lbsl_expected_load(int32_t n, int32_t sl_len, double gamma) { return expected_load_of(n, sl_len, gamma); }

int hstu_lbsl_init(const hstu_lbsl_config* cfg, hstu_lbsl_state* st) {
  if (!cfg || !st || !st->rank_load) return HSTU_ERR_NULL;
  if (!valid(cfg)) return HSTU_ERR_SHAPE;
  st->step = 0;
  st->target = 0.0;
  for (int r = 0; r < cfg->world_size; ++r) st->rank_load[r] = 0.0;
  return HSTU_OK;
}

int hstu_lbsl_step(const hstu_lbsl_config* cfg, hstu_lbsl_state* st, const int32_t* rank_offsets, const int32_t* lengths,
                   const double* uniforms, int32_t* new_lengths, uint8_t* unsampled, double* realised_load) {
  if (!cfg || !st || !st->rank_load || !rank_offsets) return HSTU_ERR_NULL;
  if (!valid(cfg)) return HSTU_ERR_SHAPE;
  const int R = cfg->world_size;
  if (rank_offsets[0] != 0) return HSTU_ERR_SHAPE;
  for (int r = 0; r < R; ++r)
    if (rank_offsets[r + 1] < rank_offsets[r]) return HSTU_ERR_SHAPE;
  const int64_t total = rank_offsets[R];
  if (total > 0 && (!lengths || !uniforms || !new_lengths || !unsampled)) return HSTU_ERR_NULL;
  for (int64_t i = 0; i < total; ++i)
    if (lengths[i] < 0 || !(uniforms[i] > 0.0 && uniforms[i] <= 1.0)) return HSTU_ERR_SHAPE;

  const int64_t t = st->step + 1;
  const int32_t sl = cfg->sl_len;
  const double gamma = cfg->gamma;
  std::vector<std::pair<double, int32_t>> keys;
  std::vector<double> sampled;
  for (int r = 0; r < R; ++r) {
    const int32_t lo = rank_offsets[r], b = rank_offsets[r + 1] - lo;
    const int32_t* len = lengths + lo;
    const double* u = uniforms + lo;
    int32_t* out = new_lengths + lo;
    uint8_t* keep = unsampled + lo;
    double acc = 0.0;                                              // this step's load under plain SL, in expectation
    for (int32_t i = 0; i < b; ++i) acc += expected_load_of(len[i], sl, gamma);
    st->rank_load[r] += acc;
    if (t <= cfg->warmup_steps) {                                  // warm-up: plain SL
      for (int32_t i = 0; i < b; ++i) keep[i] = u[i] < weight_of(len[i], sl) ? 1 : 0;
    } else {
      keys.resize(b);
      sampled.resize(b);
      double floor_load = 0.0;
      for (int32_t i = 0; i < b; ++i) {
        const double w = weight_of(len[i], sl);
        keys[i] = {w > 0.0 ? -std::log(u[i]) / w : std::numeric_limits<double>::infinity(), i};
        sampled[i] = load_of(std::min(len[i], sl), gamma);
        floor_load += sampled[i];
        keep[i] = 0;
      }
      std::sort(keys.begin(), keys.end());                         // weighted order without replacement
      const double budget = st->target - floor_load;
      double s = 0.0;
      for (int32_t k = 0; k < b; ++k) {                            // greedy fill
        const int32_t i = keys[k].second;
        const double extra = load_of(len[i], gamma) - sampled[i];
        if (s + extra <= budget) { keep[i] = 1; s += extra; }
      }
    }
    double real = 0.0;
    for (int32_t i = 0; i < b; ++i) {
      out[i] = keep[i] ? len[i] : std::min(len[i], sl);
      real += load_of(out[i], gamma);
    }
    if (realised_load) realised_load[r] = real;
  }
  st->step = t;
  const bool end_of_warmup = t == cfg->warmup_steps;
  // (recalibration starts after the warm-up: a reset inside it would leave the warm-up mean short of steps)
  if (end_of_warmup || (t > cfg->warmup_steps && t % cfg->recal_interval == 0)) {
    double sum = 0.0;
    for (int r = 0; r < R; ++r) sum += st->rank_load[r];
    st->target = sum / ((double)R * (double)(end_of_warmup ? cfg->warmup_steps : cfg->recal_interval));
    for (int r = 0; r < R; ++r) st->rank_load[r] = 0.0;
  }
  return HSTU_OK;
}

int hstu_lbsl_fit_gamma(int32_t n, const double* lengths, const double* times, double* gamma) {
  if (!lengths || !times || !gamma) return HSTU_ERR_NULL;
  if (n < 2) return HSTU_ERR_SHAPE;
  double mx = 0.0, my = 0.0;
  for (int i = 0; i < n; ++i) {
    if (!(lengths[i] > 0.0) || !(times[i] > 0.0)) return HSTU_ERR_SHAPE;
    mx += std::log(lengths[i]);
    my += std::log(times[i]);
  }
  mx /= n; my /= n;
  double sxy = 0.0, sxx = 0.0;
  for (int i = 0; i < n; ++i) {
    const double dx = std::log(lengths[i]) - mx;
    sxy += dx * (std::log(times[i]) - my);
    sxx += dx * dx;
  }
  if (!(sxx > 0.0)) return HSTU_ERR_SHAPE;
  *gamma = sxy / sxx;
  return HSTU_OK;
}

}  // extern "C"

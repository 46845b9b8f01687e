// Host-side pieces of the configuration search that need no data: the cost F(alpha) of a layer-wise
// configuration (Section 3.2, "Prioritizing Sparser Subnets"; F is the network's FLOPs) and the two-step
// sampling of configurations (Section 3.2, "Sampling Strategy"; Appendix, two-step sampling algorithm).  No
// GPU work: the supernet's training loop calls them once per step between the sparse layers' launches.
#include "nm_sparse.h"

namespace {

inline bool level_ok(int32_t N, int32_t M) { return (M == 4 || M == 8 || M == 16) && N >= 1 && N <= M; }

// F(alpha): a linear layer at N:M performs N/M of its dense multiply-accumulates, the rest is unchanged
inline double cost_of(const double* layer_macs, const int32_t* N, const int32_t* M, int32_t L, double fixed_cost) {
  double total = fixed_cost;
  for (int32_t l = 0; l < L; ++l) total += layer_macs[l] * (double)N[l] / (double)M[l];
  return total;
}

}  // namespace

extern "C" {

double nm_config_cost(const double* layer_macs, const int32_t* N, const int32_t* M, int32_t L, double fixed_cost) {
  if (!layer_macs || !N || !M || L <= 0) return -1.0;
  for (int32_t l = 0; l < L; ++l)
    if (!level_ok(N[l], M[l]) || !(layer_macs[l] >= 0.0)) return -1.0;
  return cost_of(layer_macs, N, M, L, fixed_cost);
}

int32_t nm_sample_config(const double* layer_macs, int32_t L, double fixed_cost, const int32_t* choice_N,
                         const int32_t* choice_M, int32_t S, const double* probs, const double* edges,
                         int32_t n_edges, const double* uniforms, int64_t n_uniforms, int32_t* choice,
                         int32_t* interval, int64_t* used) {
  if (!layer_macs || !choice_N || !choice_M || !probs || !edges || !uniforms || !choice || !interval || !used)
    return NM_ERR_NULL;
  if (L <= 0 || S <= 0 || n_edges < 2 || n_uniforms < 1) return NM_ERR_SHAPE;
  for (int32_t s = 0; s < S; ++s)
    if (!level_ok(choice_N[s], choice_M[s])) return NM_ERR_LEVEL;
  for (int32_t i = 0; i + 1 < n_edges; ++i)
    if (!(edges[i] < edges[i + 1])) return NM_ERR_SHAPE;
  // step 1: an interval, uniformly
  const int32_t n_int = n_edges - 1;
  int32_t it = (int32_t)(uniforms[0] * (double)n_int);
  if (it > n_int - 1) it = n_int - 1;
  if (it < 0) it = 0;
  const double lo = edges[it], hi = edges[it + 1];
  // step 2: configurations from the layers' choice probabilities until one falls into the interval
  int64_t at = 1;
  while (at + L <= n_uniforms) {
    double cost = fixed_cost;
    for (int32_t l = 0; l < L; ++l) {
      const double u = uniforms[at + l];
      const double* p = probs + (int64_t)l * S;
      double acc = 0.0;
      int32_t pick = S - 1;
      for (int32_t s = 0; s < S; ++s) {
        acc += p[s];
        if (u < acc) { pick = s; break; }
      }
      choice[l] = pick;
      cost += layer_macs[l] * (double)choice_N[pick] / (double)choice_M[pick];
    }
    at += L;
    if ((lo <= cost && cost < hi) || (it == n_int - 1 && cost == hi)) {
      *interval = it;
      *used = at;
      return NM_OK;
    }
  }
  *used = at;
  return NM_ERR_EXHAUSTED;
}

}  // extern "C"

// Placement planning on the host (no GPU): multilevel description, location renumbering,
// communication-topology construction (paper Sec. 4.1, Algorithm 1) and the closed-form
// optimum of the stream model (Sec. 3.3 / 3.4).  Produces the expert_dest_rank map that
// moe_set_placement consumes.
#include <cstdint>

#include "moe.h"

namespace {

bool valid_levels(int32_t L, const int32_t* SF, const int32_t* S_ED, int64_t* G_out) {
  if (L < 1 || L > MOE_PLAN_MAX_LEVELS || SF == nullptr) return false;
  int64_t G = 1;
  for (int l = 0; l < L; ++l) {
    if (SF[l] < 1) return false;
    if (S_ED != nullptr && (S_ED[l] < 1 || S_ED[l] > SF[l] || SF[l] % S_ED[l] != 0)) return false;
    G *= SF[l];
    if (G > (1 << 20)) return false;
  }
  *G_out = G;
  return true;
}

// x_i = floor(m / prod_{j>i} SF[j]) mod SF[i]: mixed-radix digits, most significant first
void locate(int64_t m, int32_t L, const int32_t* SF, int32_t* loc) {
  for (int l = L - 1; l >= 0; --l) {
    loc[l] = (int32_t)(m % SF[l]);
    m /= SF[l];
  }
}

// rule MOE_PLAN_RULE_ALL_OTHER: every other coordinate must agree; MOE_PLAN_RULE_PRINTED: only
// the deeper ones, as Algorithm 1 is printed
int comm_type(const int32_t* lm, const int32_t* ln, int32_t level, int32_t L, const int32_t* S_ED,
              int32_t rule = MOE_PLAN_RULE_ALL_OTHER) {
  for (int l = rule == MOE_PLAN_RULE_PRINTED ? level + 1 : 0; l < L; ++l)
    if (l != level && lm[l] != ln[l]) return MOE_COMM_NONE;
  const int32_t s = S_ED[level];
  const int32_t dm = lm[level] / s, om = lm[level] % s;
  const int32_t dn = ln[level] / s, on = ln[level] % s;
  if (dm == dn && om != on) return MOE_COMM_AG;
  if (dm != dn && om == on) return MOE_COMM_A2A;
  return MOE_COMM_NONE;
}

double model_latency(double p, double D, double P_E, double B, double lat_pe, int32_t G) {
  const double lat_ag = P_E * (G - 1) * (1.0 - p) / B;
  const double lat_a2a = D * (G - 1) * p / (G * B);
  return lat_pe + lat_ag + 2.0 * lat_a2a - (lat_pe < lat_ag ? lat_pe : lat_ag);
}

}  // namespace

extern "C" {

int moe_plan_location(int32_t rank, int32_t L, const int32_t* SF, int32_t* loc) {
  int64_t G;
  if (!valid_levels(L, SF, nullptr, &G) || loc == nullptr || rank < 0 || rank >= G)
    return MOE_EINVAL;
  locate(rank, L, SF, loc);
  return MOE_OK;
}

int moe_plan_comm_type_rule(int32_t m, int32_t n, int32_t level, int32_t L, const int32_t* SF,
                            const int32_t* S_ED, int32_t rule, int32_t* type_out) {
  int64_t G;
  if (S_ED == nullptr || !valid_levels(L, SF, S_ED, &G) || type_out == nullptr) return MOE_EINVAL;
  if (m < 0 || m >= G || n < 0 || n >= G || level < 0 || level >= L) return MOE_EINVAL;
  if (rule != MOE_PLAN_RULE_ALL_OTHER && rule != MOE_PLAN_RULE_PRINTED) return MOE_EINVAL;
  int32_t lm[MOE_PLAN_MAX_LEVELS], ln[MOE_PLAN_MAX_LEVELS];
  locate(m, L, SF, lm);
  locate(n, L, SF, ln);
  *type_out = comm_type(lm, ln, level, L, S_ED, rule);
  return MOE_OK;
}

int moe_plan_comm_type(int32_t m, int32_t n, int32_t level, int32_t L, const int32_t* SF,
                       const int32_t* S_ED, int32_t* type_out) {
  return moe_plan_comm_type_rule(m, n, level, L, SF, S_ED, MOE_PLAN_RULE_ALL_OTHER, type_out);
}

int moe_plan_comm_frequency(int32_t L, const int32_t* SF, const int32_t* S_ED, int64_t* n_ag,
                            int64_t* n_a2a) {
  return moe_plan_comm_frequency_rule(L, SF, S_ED, MOE_PLAN_RULE_ALL_OTHER, n_ag, n_a2a);
}

int moe_plan_comm_frequency_rule(int32_t L, const int32_t* SF, const int32_t* S_ED, int32_t rule,
                                 int64_t* n_ag, int64_t* n_a2a) {
  int64_t G;
  if (S_ED == nullptr || !valid_levels(L, SF, S_ED, &G) || n_ag == nullptr || n_a2a == nullptr)
    return MOE_EINVAL;
  if (rule != MOE_PLAN_RULE_ALL_OTHER && rule != MOE_PLAN_RULE_PRINTED) return MOE_EINVAL;
  if (G > 4096) return MOE_EUNSUPPORTED;  // all ordered pairs are enumerated
  int64_t ag = 0, a2a = 0;
  int32_t lm[MOE_PLAN_MAX_LEVELS], ln[MOE_PLAN_MAX_LEVELS];
  for (int64_t m = 0; m < G; ++m) {
    locate(m, L, SF, lm);
    for (int64_t n = 0; n < G; ++n) {
      if (n == m) continue;
      locate(n, L, SF, ln);
      for (int l = 0; l < L; ++l) {
        const int t = comm_type(lm, ln, l, L, S_ED, rule);
        ag += t == MOE_COMM_AG;
        a2a += t == MOE_COMM_A2A;
      }
    }
  }
  *n_ag = ag;
  *n_a2a = a2a;
  return MOE_OK;
}

int moe_plan_expert_dest_rank(int32_t local_rank, int32_t E, int32_t L, const int32_t* SF,
                              const int32_t* S_ED, int32_t* dest) {
  int64_t G;
  if (S_ED == nullptr || !valid_levels(L, SF, S_ED, &G) || dest == nullptr) return MOE_EINVAL;
  if (local_rank < 0 || local_rank >= G || E < G || E % G != 0) return MOE_EINVAL;
  const int32_t per = (int32_t)(E / G);
  int32_t lm[MOE_PLAN_MAX_LEVELS], ln[MOE_PLAN_MAX_LEVELS];
  locate(local_rank, L, SF, lm);
  for (int32_t e = 0; e < E; ++e) {
    locate(e / per, L, SF, ln);
    int64_t r = 0;
    for (int l = 0; l < L; ++l) {
      const int32_t s = S_ED[l];
      // inside the home's domain the expert was all-gathered: the coordinate stays; else
      // the worker of the home's domain that has the local worker's offset (all-to-all)
      const int32_t x = (lm[l] / s == ln[l] / s) ? lm[l] : (ln[l] / s) * s + lm[l] % s;
      r = r * SF[l] + x;
    }
    dest[e] = (int32_t)r;
  }
  return MOE_OK;
}

int moe_plan_model(double D, double P_E, double B, double lat_pe, int32_t G, double* p_star,
                   int32_t* case_id, int32_t* best_S) {
  if (!(D > 0) || !(P_E > 0) || !(B > 0) || !(lat_pe >= 0) || G < 2) return MOE_EINVAL;
  if (p_star == nullptr || case_id == nullptr || best_S == nullptr) return MOE_EINVAL;
  const bool mix = 2.0 * D - (double)G * P_E < 0;
  *case_id = mix ? MOE_PLAN_CASE_MIX : MOE_PLAN_CASE_AG_ONLY;
  double p = 0.0;
  if (mix) {
    p = 1.0 - B * lat_pe / (P_E * (G - 1));
    p = p < 0.0 ? 0.0 : (p > 1.0 ? 1.0 : p);
  }
  *p_star = p;
  int32_t bs = 1;
  double bl = -1.0;
  for (int32_t S = 1; S <= G; ++S) {
    if (G % S) continue;
    const double lat = model_latency((double)(G - S) / (G - 1), D, P_E, B, lat_pe, G);
    if (bl < 0 || lat < bl - 1e-15 * (bl < 0 ? -bl : bl)) {
      bs = S;
      bl = lat;
    }
  }
  *best_S = bs;
  return MOE_OK;
}

}  // extern "C"

// Worker-allocation tool (include/moe_alloc.h): host code only.
#include "../../include/moe_alloc.h"

#include <algorithm>
#include <cmath>
#include <vector>

namespace {
inline bool bad_model(const moe_alloc_model_t* m) {
  return !m || !(m->C_a > 0) || !(m->C_f > 0) || !(m->V > 0) || !(m->P > 0) || !(m->B > 0);
}
inline double stage(double C, double P, int gpus, double V, int nics, double B) {
  const double comp = C / (P * gpus), comm = V / (nics * B);
  return comp > comm ? comp : comm;
}
inline int clip(long v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : (int)v); }
}  // namespace

extern "C" {

int moe_alloc_costs(double b, double S, double H, double g, double k, double D_e, int n_mat, int bytes_per_elem,
                    double* C_a, double* C_f, double* V, double* I_attn, double* I_ffn) {
  if (!(b > 0) || !(S > 0) || !(H > 0) || !(g > 0) || !(k > 0) || !(D_e > 0) || n_mat < 1 || bytes_per_elem < 1)
    return MOE_ALLOC_EINVAL;
  const double ca = b * (S * H * H * (2.0 + 2.0 / g) + 4.0 * S * S * H);
  const double cf = b * (2.0 * n_mat * k * S * H * D_e);
  const double v = b * (bytes_per_elem * k * S * H);
  if (C_a) *C_a = ca;
  if (C_f) *C_f = cf;
  if (V) *V = v;
  if (I_attn) *I_attn = ca / v;
  if (I_ffn) *I_ffn = cf / v;
  return MOE_ALLOC_OK;
}

int moe_alloc_eval(const moe_alloc_model_t* m, int W, int M_tot, int M, int M_a, double* T_a, double* T_f,
                   double* U_a, double* U_f) {
  if (bad_model(m) || W < 2 || M_tot < 2 || M < 1 || M >= W || M_a < 1 || M_a >= M_tot) return MOE_ALLOC_EINVAL;
  const int N = W - M, M_f = M_tot - M_a;
  const double ta = stage(m->C_a, m->P, M, m->V, M_a, m->B);
  const double tf = stage(m->C_f, m->P, N, m->V, M_f, m->B);
  if (T_a) *T_a = ta;
  if (T_f) *T_f = tf;
  if (U_a) *U_a = m->C_a / (m->P * M * ta);
  if (U_f) *U_f = m->C_f / (m->P * N * tf);
  return MOE_ALLOC_OK;
}

int moe_alloc_seed(const moe_alloc_model_t* m, int W, int M_tot, double eps, int* M0, int* Ma0, double* T_star,
                   int* n_candidates) {
  if (bad_model(m) || W < 2 || M_tot < 2 || !(eps >= 0) || !M0 || !Ma0) return MOE_ALLOC_EINVAL;
  // The grid is small ((W-1)(M_tot-1) points), so it is tabulated once: bottleneck time and score per split,
  // split index i = (M-1)*(M_tot-1) + (M_a-1), i.e. GPU split outer, NIC split inner, both ascending.
  const int cols = M_tot - 1;
  const size_t n = (size_t)(W - 1) * cols;
  std::vector<double> bottleneck(n), score(n);
  for (size_t i = 0; i < n; ++i) {
    double ta, tf, ua, uf;
    moe_alloc_eval(m, W, M_tot, 1 + (int)(i / cols), 1 + (int)(i % cols), &ta, &tf, &ua, &uf);
    bottleneck[i] = std::max(ta, tf);
    score[i] = ua + uf;
  }
  // Candidate set under the tolerance: walking the table in index order, `first` marks where the set last
  // restarted (a split that undercuts the reference time by more than eps becomes the new reference and
  // empties the set); every later split within eps of the reference belongs to the set.  With eps = 0 this
  // is exactly the set of minimisers of the bottleneck time.
  size_t first = 0;
  double ref_T = INFINITY;
  for (size_t i = 0; i < n; ++i)
    if (bottleneck[i] < ref_T - eps) { ref_T = bottleneck[i]; first = i; }
  // Seed = the member with the highest score, the earliest one on equal scores.
  size_t pick = first;
  int members = 0;
  for (size_t i = first; i < n; ++i) {
    if (bottleneck[i] > ref_T + eps) continue;
    ++members;
    if (score[i] > score[pick]) pick = i;
  }
  *M0 = 1 + (int)(pick / cols);
  *Ma0 = 1 + (int)(pick % cols);
  if (T_star) *T_star = ref_T;
  if (n_candidates) *n_candidates = members;
  return MOE_ALLOC_OK;
}

int moe_alloc_refine(int W, int M_tot, int M0, int Ma0, int K, const int* dM, const int* dMa,
                     moe_alloc_profile_fn profile, void* user, int* M_best, int* Ma_best, double* T_best) {
  if (W < 2 || M_tot < 2 || M0 < 1 || M0 >= W || Ma0 < 1 || Ma0 >= M_tot || K < 0 || !profile || !M_best || !Ma_best ||
      (K > 0 && (!dM || !dMa)))
    return MOE_ALLOC_EINVAL;
  int m = M0, ma = Ma0;
  double t = profile(m, ma, user);
  for (int i = 0; i < K; ++i) {
    const int cm = clip((long)m + dM[i], 1, W - 1), cma = clip((long)ma + dMa[i], 1, M_tot - 1);
    const double ct = profile(cm, cma, user);
    if (ct < t) { t = ct; m = cm; ma = cma; }
  }
  *M_best = m; *Ma_best = ma;
  if (T_best) *T_best = t;
  return MOE_ALLOC_OK;
}

int moe_alloc_group_layers(int L, int p, int g, int* layers, int cap, int* n) {
  if (L < 1 || p < 1 || g < 0 || g >= p || !n || cap < 0 || (cap > 0 && !layers)) return MOE_ALLOC_EINVAL;
  const int count = g < L ? (L - g + p - 1) / p : 0;
  if (count > cap) return MOE_ALLOC_EINVAL;
  for (int j = 0; j < count; ++j) layers[j] = g + j * p;
  *n = count;
  return MOE_ALLOC_OK;
}

int moe_alloc_bubbles(int PP, int L, int v, double T_a, double T_f, double T_a2a, double T_p2p, double T_m2n,
                      double* base, double* af) {
  if (PP < 1 || L < 1 || v < 1 || T_a < 0 || T_f < 0 || T_a2a < 0 || T_p2p < 0 || T_m2n < 0) return MOE_ALLOC_EINVAL;
  if (base) *base = (PP - 1) * (L * (T_a + T_f + 2.0 * T_a2a) + T_p2p) / v;
  if (af) *af = (PP - 1) * ((T_a > T_f ? T_a : T_f) + T_m2n) / (2.0 * v);
  return MOE_ALLOC_OK;
}

}  // extern "C"

/*
 * moe_alloc.h -- C ABI of the worker-allocation tool (host code only, no GPU work).
 *
 * The paper's adaptive worker allocation (design section "Adaptive worker allocation"): W GPUs and
 * M_tot NICs are split between an attention group (M GPUs, M_a NICs) and an FFN group (N = W - M
 * GPUs, M_f = M_tot - M_a NICs).  With per-iteration FLOPs C_a, C_f, inter-group volume V (bytes),
 * per-GPU compute density P (FLOP/s) and per-NIC bandwidth B (bytes/s) the stage latencies are
 *     T_a = max(C_a / (P M), V / (M_a B)),   T_f = max(C_f / (P N), V / (M_f B))      (stage-latency equations)
 * and the pipeline runs at max(T_a, T_f).  All pointers are HOST pointers; nothing is allocated
 * or retained; every function returns MOE_ALLOC_OK or MOE_ALLOC_EINVAL (bad argument, nothing written).
 */
#ifndef MOE_ALLOC_H
#define MOE_ALLOC_H

#ifdef __cplusplus
extern "C" {
#endif

enum { MOE_ALLOC_OK = 0, MOE_ALLOC_EINVAL = 1 };

typedef struct {
  double C_a, C_f; /* per-iteration FLOPs of the attention / FFN group */
  double V;        /* inter-group communication volume, bytes */
  double P;        /* GPU compute density, FLOP/s */
  double B;        /* bandwidth of one NIC, bytes/s */
} moe_alloc_model_t;

/*
 * moe_alloc_costs -- the FLOP and byte model of the roofline paragraph:
 *   C_a = b (S H^2 (2 + 2/g) + 4 S^2 H)    group-query attention with group size g
 *   C_f = b (2 n_mat k S H D_e)            n_mat = 2: the paper's up/down GroupGEMMs (4 k S H D_e);
 *                                          n_mat = 3: SwiGLU experts as built in this library
 *   V   = b (bytes_per_elem k S H)         bf16: 2 S k H bytes
 *   I_attn = C_a / V, I_ffn = C_f / V      (n_mat = 2, bf16: (H(2+2/g)+4S)/(2k) and 2 D_e)
 * Any output pointer may be NULL.
 */
int moe_alloc_costs(double b, double S, double H, double g, double k, double D_e, int n_mat,
                    int bytes_per_elem, double* C_a, double* C_f, double* V, double* I_attn, double* I_ffn);

/* Stage latencies and the two groups' attained fractions of their compute roofs
 * U_a = C_a / (P M T_a), U_f = C_f / (P N T_f) for one split.  1 <= M < W, 1 <= M_a < M_tot. */
int moe_alloc_eval(const moe_alloc_model_t* model, int W, int M_tot, int M, int M_a, double* T_a,
                   double* T_f, double* U_a, double* U_f);

/*
 * moe_alloc_seed -- the roofline seed of the allocation algorithm (its first two phases), found by
 * tabulating every split instead of calling a MILP solver: GPU split M = 1..W-1 (outer) and NIC split
 * M_a = 1..M_tot-1 (inner), ascending.
 *   Bottleneck time of a split: max(T_a, T_f).  The candidate set holds the splits whose bottleneck time
 *   is within eps of the reference time T*; T* moves down (and the set empties) each time a split in
 *   table order undercuts it by more than eps, so with eps = 0 the set is exactly the minimisers and T*
 *   the minimum over the table; with eps > 0 membership follows the table order, as the algorithm states it.
 *   Tie-break inside the set: the paper maximises I_attn + I_ffn there.  The model constants C/V do not
 *   depend on the split, so this library reads the score as the two groups' attained fractions of their
 *   compute roofs, U_a + U_f (moe_alloc_eval): how far the NIC split lifts each group to its roof.  The
 *   earliest split in table order wins on equal scores.
 * Outputs: *M0, *Ma0 the seed, *T_star the reference time, *n_candidates the size of the set.
 */
int moe_alloc_seed(const moe_alloc_model_t* model, int W, int M_tot, double eps, int* M0, int* Ma0,
                   double* T_star, int* n_candidates);

/*
 * moe_alloc_refine -- phase 3, profile-guided local search from a seed: for trial t = 0..K-1 the
 * candidate is (clip(M* + dM[t], 1, W-1), clip(M_a* + dMa[t], 1, M_tot-1)); it replaces the
 * incumbent when profile(candidate) < T*.  The perturbations dM, dMa (each in [-r, r]) are the
 * caller's random draws; profile(M, M_a, user) returns a measured (or modelled) step time.
 */
typedef double (*moe_alloc_profile_fn)(int M, int M_a, void* user);
int moe_alloc_refine(int W, int M_tot, int M0, int Ma0, int K, const int* dM, const int* dMa,
                     moe_alloc_profile_fn profile, void* user, int* M_best, int* Ma_best, double* T_best);

/*
 * moe_alloc_group_layers -- disaggregated placement: group g of a component holds the layers
 * { g + j p : j = 0, 1, ... } below L (every p-th occurrence).  Writes them to layers[0..*n) if
 * cap suffices (else EINVAL) and the count to *n.
 */
int moe_alloc_group_layers(int L, int p, int g, int* layers, int cap, int* n);

/* Warm-up bubbles of the baseline pipeline and of AF-Pipe (the two bubble equations):
 *   base = (PP-1) [L (T_a + T_f + 2 T_a2a) + T_p2p] / v      af = (PP-1) [max(T_a, T_f) + T_m2n] / (2 v) */
int moe_alloc_bubbles(int PP, int L, int v, double T_a, double T_f, double T_a2a, double T_p2p, double T_m2n,
                      double* base, double* af);

#ifdef __cplusplus
}
#endif
#endif /* MOE_ALLOC_H */

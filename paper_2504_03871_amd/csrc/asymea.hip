// Host-only part of the library: the planner of the asymmetric expert assignment (Section 4.2 of the
// paper, Algorithm 1 "gather and squeeze" and its memory-bound variant) and the mapping from a layer's
// offload count to the slice ranges the device entry points take.  No device code, no HIP calls.
#include <climits>
#include <cmath>
#include <cstdint>

#include "../../include/moe.h"

#pragma clang fp contract(off)   // plain IEEE double steps, each rounded once

namespace {

// n_1: experts one attention GPU acquires per chunk; n_2: experts one expert GPU offloads per chunk
// (Algorithm 1, first two lines).  False unless one of M, N divides the other (the paper's assumption).
bool chunk_sizes(int M, int N, int* n_1, int* n_2) {
  if (M <= 0 || N <= 0 || (M % N != 0 && N % M != 0)) return false;
  *n_1 = N / M > 1 ? N / M : 1;
  *n_2 = (int)((long long)*n_1 * M / N);
  return true;
}

}  // namespace

extern "C" {

int moe_asymea_plan(int32_t n, int32_t L, int32_t M, int32_t N, double T_A_attn, double T_E_attn,
                    double T_E_exp, int32_t n_min, int32_t n_max, int32_t* o) {
  if (o == nullptr) return MOE_ERR_NULL;
  int n_1, n_2;
  if (n <= 0 || L <= 0 || !chunk_sizes(M, N, &n_1, &n_2)) return MOE_ERR_BAD_SHAPE;
  if (!std::isfinite(T_A_attn) || !std::isfinite(T_E_attn) || !std::isfinite(T_E_exp)) return MOE_ERR_BAD_SHAPE;
  const double T_gather = T_E_exp - T_A_attn;
  const double T_squeeze = (T_E_exp * N / n) * n_1 + (T_E_attn * N / n) * n_2;
  if (!(T_squeeze > 0.0)) return MOE_ERR_BAD_SHAPE;
  const bool bounded = n_min > 0 || n_max >= 0;
  if (n_min < 0) n_min = 0;
  if (bounded) {
    if (n_max < 0) n_max = (int32_t)((long long)n * L > INT_MAX ? INT_MAX : (long long)n * L);
    if (n_max < n_min) return MOE_ERR_BAD_SHAPE;
  }
  if (T_gather <= 0.0) {   // the expert GPUs are not the slower side: no bubble to gather
    if (bounded && n_min > 0) return MOE_ERR_BAD_SHAPE;
    for (int l = 0; l < L; ++l) o[l] = 0;
    return MOE_OK;
  }
  double step = T_gather;
  if (bounded) {
    const double lt = (double)L * T_gather;
    double alpha = (double)(n_max / n_2) * T_squeeze / lt;
    if (alpha > 1.0) alpha = 1.0;
    double beta = (double)((n_min + n_2 - 1) / n_2) * T_squeeze / lt;
    if (beta < 1.0) beta = 1.0;
    step = alpha * beta * T_gather;
  }
  double t_bubble = 0.0;
  for (int l = 0; l < L; ++l) {
    o[l] = 0;
    t_bubble = t_bubble + step;
    if (t_bubble >= T_squeeze) {
      const double chunks = std::floor(t_bubble / T_squeeze);
      if (chunks * n_2 > (double)INT_MAX) return MOE_ERR_BAD_SHAPE;
      t_bubble = t_bubble - chunks * T_squeeze;
      o[l] = (int32_t)chunks * n_2;
    }
  }
  return MOE_OK;
}

int moe_asymea_shares(int32_t n, int32_t M, int32_t N, int32_t o_l, int32_t role, int32_t rank,
                      int32_t* slice_lo, int32_t* slice_hi) {
  if (slice_lo == nullptr || slice_hi == nullptr) return MOE_ERR_NULL;
  int n_1, n_2;
  if (n <= 0 || !chunk_sizes(M, N, &n_1, &n_2) || n % N != 0) return MOE_ERR_BAD_SHAPE;
  const int per = n / N;
  if (o_l < 0 || o_l > per || o_l % n_2 != 0) return MOE_ERR_BAD_SHAPE;
  if ((role != 0 && role != 1) || rank < 0 || rank >= (role == 0 ? N : M)) return MOE_ERR_BAD_SHAPE;
  const int run = (int)((long long)o_l * N / M);   // experts one attention GPU acquires
  for (int e = 0; e < n; ++e) {
    const int g = e / per, local = e % per;
    const bool moved = local >= per - o_l;
    bool mine;
    if (role == 0) {
      mine = !moved && g == rank;
    } else {
      const int pos = g * o_l + (local - (per - o_l));   // position among the offloaded experts, by ascending id
      mine = moved && pos / run == rank;
    }
    slice_lo[e] = 0;
    slice_hi[e] = mine ? INT32_MAX : 0;
  }
  return MOE_OK;
}

}  // extern "C"

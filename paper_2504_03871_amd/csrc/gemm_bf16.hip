// Launchers of the MFMA grouped GEMM for 16-bit storage, bf16 or fp16 (kernel in gemm_bf16_kernel.h).
#include "gemm_bf16_kernel.h"

namespace moe {

// Block tile 256 x 256 (SwiGLU forward: 256 x 128 for each of its two weight matrices), 2 x 4 waves: two
// waves per SIMD, so one wave's LDS and global traffic hides under the other's MFMAs.  Global loads write LDS
// directly, two 64-wide K stages for all three operand layouts.
constexpr int T_BM = 256, T_BN = 256, T_BN_DUAL = 128, T_WGM = 2, T_WGN = 4;
int gemm_bf16_tile_rows() { return T_BM; }

// adds the SPLIT_K partial sums of every split row tile and writes the 16-bit rows of C [rows][N]
template <typename ST>
static int launch_split_reduce(const GemmArgs& g, hipStream_t s) {
  const dim3 grid((SPLIT_ROWS * (g.N / 4) + 255) / 256, g.E);
  split_reduce_kernel<ST><<<grid, 256, 0, s>>>(g);
  return launch_status();
}

template <typename ST, int MODE, int EPI, bool DUAL, bool CHAIN>
static int launch_one(const GemmArgs& g, int max_tiles, hipStream_t s) {
  constexpr int BN = DUAL ? T_BN_DUAL : T_BN;
  constexpr bool TAB = (EPI == EPI_GELU_BWD || EPI == EPI_GELU_FWD) && Half16<ST>::GELU_TABLE;
  constexpr int lds = gemm_bf16_lds_bytes<T_BM, BN, DUAL, T_WGM, T_WGN, TAB>();
  auto kern = gemm_bf16_kernel<ST, MODE, EPI, DUAL, CHAIN, T_BM, BN, T_WGM, T_WGN>;
  // more than 64 KB of dynamic LDS needs the attribute on the current device; set on every launch (a cheap
  // host-side call) rather than remembered, so the library keeps no per-process or per-device state
  {
    hipError_t err = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (err != hipSuccess) return set_hip_error(err);
  }
  const int ntn = (g.N + BN - 1) / BN;
  long long tiles;
  if (MODE == MODE_TN) tiles = (long long)((ntn * ((g.M + T_BM - 1) / T_BM) + NUM_XCD - 1) / NUM_XCD * NUM_XCD) * g.E;
  else tiles = (long long)ntn * max_tiles;
  const bool split = MODE != MODE_TN && EPI == EPI_STORE && !CHAIN && g.split_ws != nullptr;
  if (split) tiles += (long long)g.E * ntn * (SPLIT_K - 1);   // every split row tile: SPLIT_K blocks per column tile instead of one
  kern<<<dim3(gemm_bf16_grid(tiles)), T_WGM * T_WGN * 64, lds, s>>>(g);
  int rc = launch_status();
  if (rc != MOE_OK || !split) return rc;
  return launch_split_reduce<ST>(g, s);
}

// A row-tile GEMM (NT) and a weight-gradient GEMM (TN) in one launch; the first one's blocks come first.
template <typename ST, int EPI1, bool CHAIN1>
static int launch_pair(const GemmArgs& g1, int max_tiles, const GemmArgs& g2, hipStream_t s) {
  constexpr int lds1 = gemm_bf16_lds_bytes<T_BM, T_BN, false, T_WGM, T_WGN, EPI1 == EPI_GELU_BWD && Half16<ST>::GELU_TABLE>();
  constexpr int lds2 = gemm_bf16_lds_bytes<T_BM, T_BN, false, T_WGM, T_WGN>();
  constexpr int lds = lds1 > lds2 ? lds1 : lds2;
  auto kern = gemm_bf16_pair_kernel<ST, MODE_NT, EPI1, CHAIN1, MODE_TN, EPI_DW, T_BM, T_BN, T_WGM, T_WGN>;
  // more than 64 KB of dynamic LDS needs the attribute on the current device; set on every launch (a cheap
  // host-side call) rather than remembered, so the library keeps no per-process or per-device state
  {
    hipError_t err = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (err != hipSuccess) return set_hip_error(err);
  }
  // the first GEMM's block count is a multiple of the XCD count, so that a tile number still tells the
  // XCD its block runs on for the second one (numbers past the last tile return at once)
  // (a plain-store first GEMM may split its smallest row tiles along K: SPLIT_K blocks per column tile, see gemm.h)
  const int ntn1 = (g1.N + T_BN - 1) / T_BN;
  const bool split = EPI1 == EPI_STORE && !CHAIN1 && g1.split_ws != nullptr;
  const long long t1 = (long long)ntn1 * max_tiles + (split ? (long long)g1.E * ntn1 * (SPLIT_K - 1) : 0);
  const long long n1 = (t1 + NUM_XCD - 1) / NUM_XCD * NUM_XCD;
  const long long p2 = (long long)((g2.N + T_BN - 1) / T_BN) * ((g2.M + T_BM - 1) / T_BM);
  const long long n2 = (p2 + NUM_XCD - 1) / NUM_XCD * NUM_XCD * g2.E;
  if (n1 + n2 > 0x7fffffffll) return MOE_ERR_BAD_SHAPE;
  kern<<<dim3(gemm_bf16_grid(n1 + n2)), T_WGM * T_WGN * 64, lds, s>>>(g1, g2, (int)n1);
  const int rc = launch_status();
  if (rc != MOE_OK || !split) return rc;
  return launch_split_reduce<ST>(g1, s);
}

template <typename ST>
static int pair_for(int epi1, bool chain1, const GemmArgs& g1, int max_tiles, const GemmArgs& g2, hipStream_t s) {
  if (epi1 == EPI_GELU_BWD) return launch_pair<ST, EPI_GELU_BWD, false>(g1, max_tiles, g2, s);
  if (epi1 == EPI_SWIGLU_BWD) return launch_pair<ST, EPI_SWIGLU_BWD, false>(g1, max_tiles, g2, s);
  if (epi1 == EPI_STORE && !chain1) return launch_pair<ST, EPI_STORE, false>(g1, max_tiles, g2, s);
  if (epi1 == EPI_STORE && chain1) return launch_pair<ST, EPI_STORE, true>(g1, max_tiles, g2, s);
  return MOE_ERR_BAD_DTYPE;
}

template <typename ST>
static int one_for(int mode, int epi, bool dual, bool chain, const GemmArgs& g, int max_tiles, hipStream_t s) {
  if (mode == MODE_NN && epi == EPI_GELU_FWD) return launch_one<ST, MODE_NN, EPI_GELU_FWD, false, false>(g, max_tiles, s);
  if (mode == MODE_NN && epi == EPI_SWIGLU_FWD && dual) return launch_one<ST, MODE_NN, EPI_SWIGLU_FWD, true, false>(g, max_tiles, s);
  if (mode == MODE_NN && epi == EPI_STORE) return launch_one<ST, MODE_NN, EPI_STORE, false, false>(g, max_tiles, s);
  if (mode == MODE_NT && epi == EPI_GELU_BWD) return launch_one<ST, MODE_NT, EPI_GELU_BWD, false, false>(g, max_tiles, s);
  if (mode == MODE_NT && epi == EPI_SWIGLU_BWD) return launch_one<ST, MODE_NT, EPI_SWIGLU_BWD, false, false>(g, max_tiles, s);
  if (mode == MODE_NT && epi == EPI_STORE && !chain) return launch_one<ST, MODE_NT, EPI_STORE, false, false>(g, max_tiles, s);
  if (mode == MODE_NT && epi == EPI_STORE && chain) return launch_one<ST, MODE_NT, EPI_STORE, false, true>(g, max_tiles, s);
  if (mode == MODE_TN && epi == EPI_DW) return launch_one<ST, MODE_TN, EPI_DW, false, false>(g, max_tiles, s);
  return MOE_ERR_BAD_DTYPE;
}

int launch_gemm_half_pair(int dtype, int epi1, bool chain1, const GemmArgs& g1, int max_tiles, const GemmArgs& g2, hipStream_t s) {
  return dtype == MOE_DTYPE_F16 ? pair_for<f16>(epi1, chain1, g1, max_tiles, g2, s) : pair_for<bf16>(epi1, chain1, g1, max_tiles, g2, s);
}

int launch_gemm_half(int dtype, int mode, int epi, bool dual, bool chain, const GemmArgs& g, int max_tiles, hipStream_t s) {
  return dtype == MOE_DTYPE_F16 ? one_for<f16>(mode, epi, dual, chain, g, max_tiles, s) : one_for<bf16>(mode, epi, dual, chain, g, max_tiles, s);
}

}  // namespace moe

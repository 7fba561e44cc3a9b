// Grouped (per-expert, ragged) GEMM plumbing shared by the fp32 and the bf16 MFMA kernels.
//
// The expert FFN of the paper is "mainly GEMMs" (Section 2.1) and its cost must follow the number
// of token rows an expert receives, not the number of experts (Section 4.2, the remark on
// T_E^Exp).  So every GEMM here walks a device-resident list of row tiles built from
// offsets / kept / shares: no padding of experts to a common size and no host read-back of counts.
#pragma once
#include "common.h"

namespace moe {

// One tile of consecutive permuted rows belonging to one expert.
struct RowTile {
  int32_t e;      // expert
  int32_t row0;   // first row (absolute index into the permuted buffers)
  int32_t nrows;  // valid rows in this tile (1..tile height)
  int32_t pad;
};

// Tables over the bf16 numbers for the bf16 GELU epilogues.  The pre-activation is stored as a bf16
// number, so the forward applies GELU to exactly that number (as a separate activation kernel on the
// stored tensor would) and the backward takes the derivative at it; both are looked up instead of
// computed: Phi(v) for the forward (h = a Phi(v)), gelu'(v) for the backward.  Entry [sign][m],
// m = (bits & 0x7fff) - (GELU_TAB_EXP0 << 7) clamped to [0, GELU_TAB_NMAG): magnitudes from 2^-16 up to
// (not including) 8; smaller ones read the first entry (Phi and gelu' are 0.5 there to within 1.3e-5),
// larger ones the last (gelu' is 1 or 0 there to within 1e-13; the last Phi entries are set to exactly 1 and 0).
enum GeluTable { GELU_TAB_NONE = 0, GELU_TAB_PHI = 1, GELU_TAB_GRAD = 2 };
// Split-K for the smallest row tiles.  A partly filled row tile of at most SPLIT_ROWS rows has almost no
// MFMA work, but a block still walks all K stages for it at the pace of memory latency, and such tiles
// run last, on a mostly idle chip.  For the plain-store GEMMs each of them is therefore cut into
// SPLIT_K blocks along K that write fp32 partial sums [tile][k part][SPLIT_ROWS][N] into the workspace;
// split_reduce adds the parts in fixed order and writes the bf16 rows.  Used when K is long enough
// to matter and the experts are few (the partial sums take E * SPLIT_K * SPLIT_ROWS * N * 4 bytes).
constexpr int SPLIT_ROWS = 64;
constexpr int SPLIT_K = 8;
constexpr int SPLIT_MAX_E = 32;
constexpr int SPLIT_MIN_K = 2048;
// (each K part must be whole 64-wide stages of the row-tile GEMMs)
inline bool split_k_applies(int E, int K) { return E <= SPLIT_MAX_E && K >= SPLIT_MIN_K && K % (SPLIT_K * 64) == 0; }
inline size_t split_ws_bytes(int E, int N) { return (size_t)E * SPLIT_K * SPLIT_ROWS * N * 4; }

constexpr int GELU_TAB_EXP0 = 111;                 // biased exponent of 2^-16
constexpr int GELU_TAB_NMAG = (130 - 111) * 128;   // 2432 magnitudes per sign
constexpr int GELU_TAB_FLOATS = 6144;              // 2 * 2432 entries, padded to 24 KB (whole 1 KB wave loads)

// Tile map in the workspace: header[0] = number of tiles, header[1] = number of tiles at the head of the
// list that are walked XCD by XCD (the full tiles; with many experts of few tiles each the list is
// expert-major and this is all of it), header[2] = number of tiles of at most SPLIT_ROWS rows at the
// end of the list that may be split along K (0 for an expert-major list); then the
// tiles; then order[E] = the experts by descending share length (heaviest first); then one table as above.
struct TileMap {
  int32_t* header;
  RowTile* tiles;
  int32_t* order;
  float* gelu_tab;
};
inline size_t tile_map_bytes(int max_tiles, int E) {
  return 16 + (size_t)max_tiles * sizeof(RowTile) + (((size_t)E * 4 + 15) & ~(size_t)15) + (size_t)GELU_TAB_FLOATS * 4;
}
inline TileMap tile_map_at(void* ws_region, int max_tiles, int E) {
  TileMap m;
  char* base = reinterpret_cast<char*>(ws_region);
  m.header = reinterpret_cast<int32_t*>(base);
  m.tiles = reinterpret_cast<RowTile*>(base + 16);
  m.order = reinterpret_cast<int32_t*>(base + 16 + (size_t)max_tiles * sizeof(RowTile));
  m.gelu_tab = reinterpret_cast<float*>(base + 16 + (size_t)max_tiles * sizeof(RowTile) + (((size_t)E * 4 + 15) & ~(size_t)15));
  return m;
}
inline int max_row_tiles(int A, int E, int tile_rows) { return (A + tile_rows - 1) / tile_rows + E; }

enum GemmMode {
  MODE_NN = 0,  // C[rows, N] = A[rows, K] * B_e[K, N]          (forward GEMMs)
  MODE_NT = 1,  // C[rows, N] = A[rows, K] * B_e[N, K]^T        (dH, dX)
  MODE_TN = 2   // C_e[M, N] (+)= A[rows_e, M]^T * B[rows_e, N]  (weight gradients)
};

enum Epilogue {
  EPI_STORE = 0,       // C = acc
  EPI_GELU_FWD = 1,    // C = acc (pre-activation), C2 = gelu(acc)
  EPI_SWIGLU_FWD = 2,  // dual accumulators g,u: C = g, C2 = u, C3 = silu(g)*u
  EPI_GELU_BWD = 3,    // C = acc * gelu'(S1)
  EPI_SWIGLU_BWD = 4,  // C = dG = acc * S2 * silu'(S1), C2 = dU = acc * silu(S1)   (S1 = G, S2 = U)
  EPI_DW = 5           // fp32 C_e = acc (+ C_e)
};

struct GemmArgs {
  const void* A;
  const void* A2;   // second activation operand (SwiGLU dX: dU)
  const void* B;
  const void* B2;   // second weight operand (SwiGLU: W1b)
  void* C;
  void* C2;
  void* C3;
  const void* S1;
  const void* S2;
  const RowTile* tiles;
  const int32_t* ntiles;
  const int32_t* order;     // experts by descending share length (weight-gradient GEMMs start the heaviest first)
  const float* gelu_tab;    // bf16 GELU epilogues: Phi (forward) or gelu' (backward) over the bf16 numbers
  float* split_ws;          // fp32 partial sums of the split row tiles, or NULL: no split-K (see SPLIT_K)
  const int32_t* offsets;
  const int32_t* kept;
  const int32_t* lo;
  const int32_t* hi;
  int M, N, K;   // NN/NT: N and K fixed (M unused); TN: M and N fixed (K is the expert's row count)
  int E;
  int accumulate;
};

// table: which GELU table to fill as well (bf16 GELU layers: GELU_TAB_PHI before the forward GEMMs,
// GELU_TAB_GRAD before the backward ones)
int launch_tile_map(const int32_t* offsets, const int32_t* kept, const int32_t* lo, const int32_t* hi, int E,
                    int tile_rows, TileMap map, int table, hipStream_t s);

// fp32 storage, fp32 FMA (any shape that passes check_cfg)
int launch_gemm_f32(int mode, int epi, bool dual, bool chain, const GemmArgs& g, int max_tiles, hipStream_t s);
// 16-bit storage (dtype = MOE_DTYPE_BF16 or MOE_DTYPE_F16), MFMA with fp32 accumulation
int launch_gemm_half(int dtype, int mode, int epi, bool dual, bool chain, const GemmArgs& g, int max_tiles, hipStream_t s);
// one launch for an NT GEMM (epilogue epi1, chained or not) followed by a TN weight-gradient GEMM
int launch_gemm_half_pair(int dtype, int epi1, bool chain1, const GemmArgs& g1, int max_tiles, const GemmArgs& g2, hipStream_t s);
int gemm_bf16_tile_rows();

#ifdef __HIPCC__
// Element-wise epilogues, shared by both kernels.  `row` is the absolute permuted row, `col` the
// output column, `ldc` the row pitch of the output(s).
template <typename T, int EPI>
__device__ __forceinline__ void epilogue(const GemmArgs& g, size_t idx, float acc, float acc2) {
  if constexpr (EPI == EPI_STORE) {
    reinterpret_cast<T*>(g.C)[idx] = from_f32<T>(acc);
  } else if constexpr (EPI == EPI_GELU_FWD) {
    reinterpret_cast<T*>(g.C)[idx] = from_f32<T>(acc);
    reinterpret_cast<T*>(g.C2)[idx] = from_f32<T>(gelu_f(acc));
  } else if constexpr (EPI == EPI_SWIGLU_FWD) {
    reinterpret_cast<T*>(g.C)[idx] = from_f32<T>(acc);
    reinterpret_cast<T*>(g.C2)[idx] = from_f32<T>(acc2);
    reinterpret_cast<T*>(g.C3)[idx] = from_f32<T>(acc * sigmoid_f(acc) * acc2);
  } else if constexpr (EPI == EPI_GELU_BWD) {
    const float a = to_f32(reinterpret_cast<const T*>(g.S1)[idx]);
    reinterpret_cast<T*>(g.C)[idx] = from_f32<T>(acc * gelu_grad_f(a));
  } else if constexpr (EPI == EPI_SWIGLU_BWD) {
    const float gg = to_f32(reinterpret_cast<const T*>(g.S1)[idx]);
    const float uu = to_f32(reinterpret_cast<const T*>(g.S2)[idx]);
    const float sg = sigmoid_f(gg);
    reinterpret_cast<T*>(g.C)[idx] = from_f32<T>(acc * uu * sg * (1.f + gg * (1.f - sg)));
    reinterpret_cast<T*>(g.C2)[idx] = from_f32<T>(acc * gg * sg);
  } else {
    float* c = reinterpret_cast<float*>(g.C);
    c[idx] = g.accumulate ? c[idx] + acc : acc;
  }
}
#endif

}  // namespace moe

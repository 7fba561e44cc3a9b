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

// ---- block -> tile numbering of the MFMA grouped GEMMs (host and device: a host-side test enumerates it) ----
#ifdef __HIPCC__
#define MOE_HD __host__ __device__
#else
#define MOE_HD
#endif
constexpr int NUM_XCD = 8;

// Row-tile GEMMs.  Tiles are numbered (row tile, column tile) with the full row tiles first.  The full region
// is walked in groups of GROUP row tiles, column by column, and cut into one contiguous range per XCD
// (workgroups go to the eight XCDs round-robin), so tiles that run together on an XCD share operand panels in
// its L2.  The partly filled row tiles follow in dispatch order: they are the last blocks to start and fill
// the chip's final round.
MOE_HD inline bool block_to_tile(int b, int n_rt, int n_full_rt, int ntn, int& rt, int& nt) {
  constexpr int GROUP = 4;
  const int n_full = n_full_rt * ntn, n_all = n_rt * ntn;
  if (b >= n_all) return false;
  if (b >= n_full) {                          // partial row tiles, largest first, in dispatch order
    rt = n_full_rt + (b - n_full) / ntn;
    nt = (b - n_full) % ntn;
    return true;
  }
  const int per = n_full / NUM_XCD;           // full tiles per XCD; the few left over keep their own index
  const int logical = (b < per * NUM_XCD) ? (b % NUM_XCD) * per + b / NUM_XCD : b;
  const int per_group = GROUP * ntn;
  const int grp = logical / per_group, in = logical % per_group;
  const int first = grp * GROUP, gsz = (GROUP < n_full_rt - first) ? GROUP : n_full_rt - first;
  rt = first + in % gsz;
  nt = in / gsz;
  return true;
}

// Block vb of a row-tile GEMM launch over n_rt row tiles (the first n_full_rt of them walked XCD by XCD), of
// which the last n_sp are split along K: those are not part of the regular numbering; their blocks follow it,
// SPLIT_K per (row tile, column tile), each with a K part of its own.  False: no tile (surplus block).
struct RowBlock { int rt, nt, split_tile, ksplit; };
MOE_HD inline bool row_tile_block(int vb, int n_rt, int n_full_rt, int n_sp, int ntn, RowBlock& r) {
  const int n_reg = n_rt - n_sp;
  r.split_tile = -1;
  r.ksplit = 0;
  if (vb < n_reg * ntn) return block_to_tile(vb, n_reg, n_full_rt, ntn, r.rt, r.nt);
  const int q = vb - n_reg * ntn;
  if (q >= n_sp * ntn * SPLIT_K) return false;
  r.ksplit = q % SPLIT_K;
  r.nt = (q / SPLIT_K) % ntn;
  r.split_tile = q / (SPLIT_K * ntn);
  r.rt = n_reg + r.split_tile;
  return true;
}

// Block vb of a weight-gradient launch: tile (expert slot in descending-size order, m tile, n tile).  Every
// expert's ntm x ntn tiles are split evenly over the XCDs (block b runs on XCD b % 8), so a skewed load is
// even across XCDs.  An XCD's share of an expert is a contiguous range of the expert's tiles in patch order
// (four m tiles at a time, column by column), so the 32 tiles it runs together form a 4 x 8 patch that needs
// 12 operand panels per K stage from its L2 instead of up to 18 with the tiles dealt one by one.
MOE_HD inline bool dw_block(int vb, int ntm, int ntn, int& slot, int& mt, int& nt) {
  constexpr int GROUP = 4;
  const int P = ntm * ntn, P8 = (P + NUM_XCD - 1) / NUM_XCD * NUM_XCD;
  const int q = vb % P8, x = q % NUM_XCD, i = q / NUM_XCD;      // XCD, and the block's turn on it for this expert
  const int base = P / NUM_XCD, extra = P % NUM_XCD;            // XCD x takes base (+1 for the first `extra`) tiles
  if (i >= base + (x < extra ? 1 : 0)) return false;
  const int p = x * base + (x < extra ? x : extra) + i;         // position in patch order
  slot = vb / P8;
  const int per_group = GROUP * ntn, grp = p / per_group, in = p % per_group;
  const int first = grp * GROUP, gsz = (GROUP < ntm - first) ? GROUP : ntm - first;
  mt = first + in % gsz;
  nt = in / gsz;
  return true;
}

enum GemmMode {
  MODE_NN = 0,  // C[rows, N] = A[rows, K] * B_e[K, N]          (forward GEMMs)
  MODE_NT = 1,  // C[rows, N] = A[rows, K] * B_e[N, K]^T        (dH, dX)
  MODE_TN = 2   // C_e[M, N] (+)= A[rows_e, M]^T * B[rows_e, N]  (weight gradients)
};

enum Epilogue {
  EPI_STORE = 0,       // C = acc
  EPI_GELU_FWD = 1,    // C = acc (pre-activation; skipped when C is NULL), C2 = gelu(acc)
  EPI_SWIGLU_FWD = 2,  // dual accumulators g,u: C = g, C2 = u (both skipped when C is NULL), C3 = silu(g)*u
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
  } else if constexpr (EPI == EPI_GELU_FWD) {   // C == NULL: the caller keeps only the hidden activation
    if (g.C != nullptr) reinterpret_cast<T*>(g.C)[idx] = from_f32<T>(acc);
    reinterpret_cast<T*>(g.C2)[idx] = from_f32<T>(gelu_f(acc));
  } else if constexpr (EPI == EPI_SWIGLU_FWD) {
    if (g.C != nullptr) {
      reinterpret_cast<T*>(g.C)[idx] = from_f32<T>(acc);
      reinterpret_cast<T*>(g.C2)[idx] = from_f32<T>(acc2);
    }
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

// Row-tile map builder and the fp32 grouped GEMM (fp32 storage, fp32 FMA accumulation).
//
// The fp32 path exists for the small full-precision configuration, whose tolerance (1e-5) rules out
// reduced-precision matrix instructions; it is a plain LDS-tiled kernel, not a tuned one.
#include "gemm.h"

namespace moe {

// Tile order: every full tile (tile_rows valid rows) first, in expert order, then the experts' last,
// partly filled tiles by descending row count.  Blocks are dispatched in tile order, so the short
// tiles fill the chip's last round instead of each costing a full round.
// header[0] = number of tiles, header[1] = tiles walked XCD by XCD, header[2] = trailing tiles that may be split along K (gemm.h).
constexpr int TM_THREADS = 4 * MOE_MAX_E;   // four threads per expert
__global__ __launch_bounds__(TM_THREADS) void tile_map_kernel(const int32_t* __restrict__ offsets, const int32_t* __restrict__ kept,
                                                              const int32_t* __restrict__ lo, const int32_t* __restrict__ hi,
                                                              int E, int tile_rows, int32_t* __restrict__ header,
                                                              RowTile* __restrict__ tiles, int32_t* __restrict__ order,
                                                              float* __restrict__ gelu_tab, int table) {
  // sort keys: (value << 32) | (MOE_MAX_E - 1 - id), so that "ahead of me" (larger value, ties by lower id) is
  // one 64-bit comparison; entries from E on hold value 0 and ids above every real one: never ahead
  __shared__ __align__(16) unsigned long long s_klen[MOE_MAX_E], s_krem[MOE_MAX_E];
  __shared__ int s_full[MOE_MAX_E], s_rem[MOE_MAX_E], s_start[MOE_MAX_E], s_base[MOE_MAX_E];
  __shared__ int s_nfull, s_major;
  if (blockIdx.x > 0) {   // blocks past the first fill the table: Phi(v) or gelu'(v) for the bf16 numbers (layout: gemm.h)
    for (int i = (blockIdx.x - 1) * blockDim.x + threadIdx.x; i < GELU_TAB_FLOATS; i += (gridDim.x - 1) * blockDim.x) {
      float v = 0.f;
      if (i < 2 * GELU_TAB_NMAG) {
        const uint32_t bits = (uint32_t)((i % GELU_TAB_NMAG) + (GELU_TAB_EXP0 << 7)) | (i >= GELU_TAB_NMAG ? 0x8000u : 0u);
        const float a = __uint_as_float(bits << 16);
        v = table == GELU_TAB_PHI ? 0.5f * erfcf(-a * 0.70710678118654752440f) : gelu_grad_f(a);
        // the last magnitude also stands for everything larger: Phi is exactly 1 or 0 there, so that
        // h = a Phi stays a or 0 however large a is
        if (table == GELU_TAB_PHI && i % GELU_TAB_NMAG == GELU_TAB_NMAG - 1) v = i >= GELU_TAB_NMAG ? 0.f : 1.f;
      }
      gelu_tab[i] = v;
    }
    return;
  }
  const int tid = threadIdx.x;
  if (tid < MOE_MAX_E) {
    int l = 0, h = 0, base = 0;
    if (tid < E) {
      share_of(lo, hi, kept[tid], tid, l, h);
      base = offsets[tid] + l;
    }
    const int rem = (h - l) % tile_rows;
    s_full[tid] = (h - l) / tile_rows;
    s_rem[tid] = rem;
    s_base[tid] = base;
    s_klen[tid] = ((unsigned long long)(h - l) << 32) | (unsigned)(MOE_MAX_E - 1 - tid);
    s_krem[tid] = ((unsigned long long)rem << 32) | (unsigned)(MOE_MAX_E - 1 - tid);
  }
  __syncthreads();
  // Expert e = tid / 4; its four threads each compare it with a quarter of the experts and add up.
  const int e = tid >> 2, part = tid & 3;
  const int per = 2 * ((E + 7) / 8);     // entries per quarter, even (16-byte LDS reads)
  auto rank_desc = [&](const unsigned long long* key) {   // number of entries ahead of key[e]
    const unsigned long long mine = key[e];
    int rank = 0;
#pragma unroll 4
    for (int o = part * per; o < min((part + 1) * per, MOE_MAX_E); o += 2) {
      const ulonglong2 v = *reinterpret_cast<const ulonglong2*>(key + o);
      rank += (v.x > mine) + (v.y > mine);
    }
    rank += __shfl_xor(rank, 1, WAVE);
    rank += __shfl_xor(rank, 2, WAVE);
    return rank;
  };
  const int rank_len = rank_desc(s_klen), rank_rem = rank_desc(s_krem);
  if (part == 0 && e < E) order[rank_len] = e;   // experts by descending share length, ties by id
  if (tid < WAVE) {   // the first wave scans the experts, four per lane (MOE_MAX_E = 4 x 64)
    int full[4], some[4], sum_full = 0, sum_part = 0, sum_small = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      full[i] = s_full[tid * 4 + i];
      const int rem = s_rem[tid * 4 + i];
      some[i] = rem > 0;
      sum_full += full[i];
      sum_part += some[i];
      sum_small += (rem > 0 && rem <= SPLIT_ROWS);
    }
    const int run = wave_sum_i(sum_full), parts = wave_sum_i(sum_part), small = wave_sum_i(sum_small);
    // Many experts of few row tiles each: an expert's weight panels are used by two or three tiles only,
    // so these must run together (same XCD, same time) or the panels are fetched once per tile.  The
    // list is then expert-major (each expert's full tiles, then its partly filled one) and the whole of
    // it is walked as the full region is.
    const bool major = E > SPLIT_MAX_E && run < 3 * E;
    const int mine = major ? sum_full + sum_part : sum_full;
    int pos = wave_scan_i(mine) - mine;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      s_start[tid * 4 + i] = pos;
      pos += full[i] + (major ? some[i] : 0);
    }
    if (tid == 0) {
      s_nfull = run;
      s_major = major;
      header[0] = run + parts;
      header[1] = major ? run + parts : run;
      header[2] = major ? 0 : small;   // the last entries: the partly filled tiles are sorted by descending size
    }
  }
  __syncthreads();
  if (e < E) {
    const int base = s_base[e], nfull = s_full[e], rem = s_rem[e];
    if (s_major) {
      // Expert-major list: an expert's rows are cut into its ceil(len / tile_rows) tiles evenly (in steps of 64
      // rows, two MFMA row bands) instead of full tiles plus a remainder.  A remainder of a few rows costs a
      // block the whole weight panel for next to no arithmetic; two tiles of 140 rows cost less than one of
      // 256 and one of 24, and every output row is computed the same way wherever its tile starts.
      const int len = nfull * tile_rows + rem, ntile = nfull + (rem > 0);
      int per = tile_rows;
      if (ntile > 1) {
        per = min(tile_rows, ((len + ntile - 1) / ntile + 63) & ~63);
        if ((ntile - 1) * per >= len) per = tile_rows;   // many tiles: the rounding would leave the last one empty
      }
      for (int i = part; i < ntile; i += 4) {   // the expert's four threads share its tiles
        RowTile t;
        t.e = e;
        t.row0 = base + i * per;
        t.nrows = min(per, len - i * per);
        t.pad = 0;
        tiles[s_start[e] + i] = t;
      }
    } else {
      for (int i = part; i < nfull; i += 4) {
        RowTile t;
        t.e = e;
        t.row0 = base + i * tile_rows;
        t.nrows = tile_rows;
        t.pad = 0;
        tiles[s_start[e] + i] = t;
      }
      if (part == 0 && rem > 0) {   // position among the partial tiles: more rows first, ties by expert id
        RowTile t;
        t.e = e;
        t.row0 = base + nfull * tile_rows;
        t.nrows = rem;
        t.pad = 0;
        tiles[s_nfull + rank_rem] = t;
      }
    }
  }
}

int launch_tile_map(const int32_t* offsets, const int32_t* kept, const int32_t* lo, const int32_t* hi, int E,
                    int tile_rows, TileMap map, int table, hipStream_t s) {
  const int grid = table == GELU_TAB_NONE ? 1 : 1 + (GELU_TAB_FLOATS + TM_THREADS - 1) / TM_THREADS;   // one thread per table entry
  tile_map_kernel<<<grid, TM_THREADS, 0, s>>>(offsets, kept, lo, hi, E, tile_rows, map.header, map.tiles, map.order,
                                    map.gelu_tab, table);
  return launch_status();
}

constexpr int SB = 64;   // tile edge
constexpr int SK = 32;   // k step
constexpr int EPT = SB * SK / 256;   // operand elements a thread moves per k step

// NN/NT: grid = (ceil(N/SB), max row tiles).  TN: grid = (ceil(N/SB), ceil(M/SB), E).
template <int MODE, int EPI, bool DUAL, bool CHAIN>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmArgs g) {
  __shared__ float As[SK][SB + 4];
  __shared__ float Bs[SK][SB + 4];
  __shared__ float Bs2[DUAL ? SK : 1][SB + 4];
  const int tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
  const int n0 = blockIdx.x * SB;
  int e, row0, mvalid, klen, m0 = 0;
  if constexpr (MODE == MODE_TN) {
    e = blockIdx.z;
    m0 = blockIdx.y * SB;
    int l, h;
    share_of(g.lo, g.hi, g.kept[e], e, l, h);
    row0 = g.offsets[e] + l;
    klen = h - l;
    mvalid = min(SB, g.M - m0);
    if (klen == 0 && g.accumulate) return;
  } else {
    if ((int)blockIdx.y >= g.ntiles[0]) return;
    const RowTile t = g.tiles[blockIdx.y];
    e = t.e;
    row0 = t.row0;
    mvalid = t.nrows;
    klen = g.K;
  }
  const int nvalid = min(SB, g.N - n0);
  float acc[4][4] = {}, acc2[DUAL ? 4 : 1][4] = {};
  // The global loads of K step k0 + SK are issued before the arithmetic of step k0 (registers va/vb), so
  // their latency hides behind it; a chained GEMM runs its two operand pairs back to back.
  const int nsteps = (klen + SK - 1) / SK, total = nsteps * (CHAIN ? 2 : 1);
  float va[EPT], vb[EPT], vb2[DUAL ? EPT : 1];
  auto fetch = [&](int step) {
    const int pass = step / max(nsteps, 1), k0 = (step - pass * nsteps) * SK;
    const float* A = reinterpret_cast<const float*>(pass == 0 ? g.A : g.A2);
    const float* B = reinterpret_cast<const float*>(pass == 0 ? g.B : g.B2);
    const float* B2 = reinterpret_cast<const float*>(g.B2);
#pragma unroll
    for (int i = 0; i < EPT; ++i) {
      const int id = tid + 256 * i;
      {  // A element (m, kk)
        int m, kk;
        if constexpr (MODE == MODE_TN) { m = id % SB; kk = id / SB; } else { m = id / SK; kk = id % SK; }
        float v = 0.f;
        if (m < mvalid && k0 + kk < klen) {
          if constexpr (MODE == MODE_TN) v = A[(size_t)(row0 + k0 + kk) * g.M + m0 + m];
          else v = A[(size_t)(row0 + m) * g.K + k0 + kk];
        }
        va[i] = v;
      }
      {  // B element (kk, n)
        int n, kk;
        if constexpr (MODE == MODE_NT) { n = id / SK; kk = id % SK; } else { n = id % SB; kk = id / SB; }
        float v = 0.f, v2 = 0.f;
        if (n < nvalid && k0 + kk < klen) {
          size_t off;
          if constexpr (MODE == MODE_TN) off = (size_t)(row0 + k0 + kk) * g.N + n0 + n;
          else if constexpr (MODE == MODE_NN) off = ((size_t)e * g.K + k0 + kk) * g.N + n0 + n;
          else off = ((size_t)e * g.N + n0 + n) * g.K + k0 + kk;
          v = B[off];
          if constexpr (DUAL) v2 = B2[off];
        }
        vb[i] = v;
        if constexpr (DUAL) vb2[i] = v2;
      }
    }
  };
  if (total > 0) fetch(0);
  for (int step = 0; step < total; ++step) {
#pragma unroll
    for (int i = 0; i < EPT; ++i) {
      const int id = tid + 256 * i;
      if constexpr (MODE == MODE_TN) As[id / SB][id % SB] = va[i]; else As[id % SK][id / SK] = va[i];
      if constexpr (MODE == MODE_NT) Bs[id % SK][id / SK] = vb[i]; else Bs[id / SB][id % SB] = vb[i];
      if constexpr (DUAL) { if constexpr (MODE == MODE_NT) Bs2[id % SK][id / SK] = vb2[i]; else Bs2[id / SB][id % SB] = vb2[i]; }
    }
    __syncthreads();
    if (step + 1 < total) fetch(step + 1);
#pragma unroll
    for (int kk = 0; kk < SK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
      if constexpr (DUAL) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc2[i][j] = fmaf(a[i], Bs2[kk][tx * 4 + j], acc2[i][j]);
      }
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = ty * 4 + i, n = tx * 4 + j;
      if (m < mvalid && n < nvalid) {
        size_t idx;
        if constexpr (MODE == MODE_TN) idx = ((size_t)e * g.M + m0 + m) * g.N + n0 + n;
        else idx = (size_t)(row0 + m) * g.N + n0 + n;
        epilogue<float, EPI>(g, idx, acc[i][j], DUAL ? acc2[DUAL ? i : 0][j] : 0.f);
      }
    }
}

template <int MODE, int EPI, bool DUAL, bool CHAIN>
static int launch_one(const GemmArgs& g, int max_tiles, hipStream_t s) {
  dim3 grid;
  if (MODE == MODE_TN) grid = dim3((g.N + SB - 1) / SB, (g.M + SB - 1) / SB, g.E);
  else grid = dim3((g.N + SB - 1) / SB, max_tiles, 1);
  gemm_f32_kernel<MODE, EPI, DUAL, CHAIN><<<grid, 256, 0, s>>>(g);
  return launch_status();
}

int launch_gemm_f32(int mode, int epi, bool dual, bool chain, const GemmArgs& g, int max_tiles, hipStream_t s) {
  if (mode == MODE_NN && epi == EPI_GELU_FWD) return launch_one<MODE_NN, EPI_GELU_FWD, false, false>(g, max_tiles, s);
  if (mode == MODE_NN && epi == EPI_SWIGLU_FWD && dual) return launch_one<MODE_NN, EPI_SWIGLU_FWD, true, false>(g, max_tiles, s);
  if (mode == MODE_NN && epi == EPI_STORE) return launch_one<MODE_NN, EPI_STORE, false, false>(g, max_tiles, s);
  if (mode == MODE_NT && epi == EPI_GELU_BWD) return launch_one<MODE_NT, EPI_GELU_BWD, false, false>(g, max_tiles, s);
  if (mode == MODE_NT && epi == EPI_SWIGLU_BWD) return launch_one<MODE_NT, EPI_SWIGLU_BWD, false, false>(g, max_tiles, s);
  if (mode == MODE_NT && epi == EPI_STORE && !chain) return launch_one<MODE_NT, EPI_STORE, false, false>(g, max_tiles, s);
  if (mode == MODE_NT && epi == EPI_STORE && chain) return launch_one<MODE_NT, EPI_STORE, false, true>(g, max_tiles, s);
  if (mode == MODE_TN && epi == EPI_DW) return launch_one<MODE_TN, EPI_DW, false, false>(g, max_tiles, s);
  return MOE_ERR_BAD_DTYPE;
}

}  // namespace moe

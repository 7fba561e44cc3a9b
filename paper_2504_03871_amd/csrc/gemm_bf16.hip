// bf16 grouped GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation).
//
// Block = 256 threads = 2x2 waves; wave tile = (WTM*32) x (WTN*32); K step per stage = 64.
// Tiles are staged global -> registers -> LDS (double buffered), operands are read from LDS either
// with 16-byte reads (operand stored with K contiguous) or with the transposing 8-byte LDS read of
// gfx950 (operand stored with K strided, i.e. exactly as it lies in memory), so no operand is ever
// transposed in global memory.
//
// MFMA 32x32x16 register layout (checked on the hardware): lane l supplies row/column l%32 and the
// eight K values (l/32)*8..+7; accumulator register v of lane l is row (v/4)*8 + (l/32)*4 + v%4,
// column l%32.
#include "gemm.h"

namespace moe {

typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BK = 64;   // K elements per stage (128 bytes of a K-contiguous row)

// ---- LDS layouts -------------------------------------------------------------------------------
// K-contiguous tile: [rows][64] bf16, 128 bytes per row, 16-byte chunks XOR-swizzled by (row/2)%8 so
// that 16 lanes reading the same chunk of 16 consecutive rows touch 16 distinct 16-byte bank groups.
__device__ __forceinline__ int kc_off(int row, int chunk) { return row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4); }
// K-strided tile: [64][W] bf16 (W*2 bytes per K row), 64-byte granules XOR-swizzled by k%4 so that
// the four K rows one transposing read touches fall into different bank groups.
template <int W>
__device__ __forceinline__ int ks_off(int krow, int col_byte) {
  return krow * (W * 2) + ((((col_byte >> 6) ^ (krow & 3)) << 6) | (col_byte & 63));
}

__device__ __forceinline__ bf16x8 lds_read_kc(const char* tile, int row, int chunk) {
  return *reinterpret_cast<const bf16x8*>(tile + kc_off(row, chunk));
}
// Eight K values (k0 .. k0+7 of this lane's K group) for column `col` from a K-strided tile.
// The transposing read works on blocks of 16 lanes: lane s of a block reads 8 bytes at
// (k row s/4, columns 4*(s%4)..+3) and receives the four K rows for column s.
template <int W>
__device__ __forceinline__ bf16x8 lds_read_ks(const char* tile, int kstep, int col_base, int lane) {
  const int b = lane >> 4, s = lane & 15;
  const int krow = kstep * 16 + (b >> 1) * 8 + (s >> 2);
  const int colb = (col_base + (b & 1) * 16 + (s & 3) * 4) * 2;
  typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(tile + ks_off<W>(krow, colb)));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(tile + ks_off<W>(krow + 4, colb)));
  union { struct { s16x4 a, b; } p; bf16x8 v; } u;
  u.p.a = lo;
  u.p.b = hi;
  return u.v;
}

template <int MODE, int EPI, bool DUAL, bool CHAIN, int WTM, int WTN>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmArgs g) {
  constexpr int BM = 2 * WTM * 32, BN = 2 * WTN * 32;
  constexpr bool A_KC = (MODE != MODE_TN);   // A stored with K contiguous
  constexpr bool B_KC = (MODE == MODE_NT);
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
  constexpr int STAGE = A_BYTES + B_BYTES * (DUAL ? 2 : 1);
  constexpr int A_CH = BM * BK / 8 / 256, B_CH = BN * BK / 8 / 256;   // 16-byte chunks per thread
  extern __shared__ __attribute__((aligned(16))) char smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  int e, row0, mvalid, klen, m0 = 0, n0;
  if constexpr (MODE == MODE_TN) {
    const int ntn = (g.N + BN - 1) / BN, ntm = (g.M + BM - 1) / BM;
    int b = blockIdx.x;
    n0 = (b % ntn) * BN;
    b /= ntn;
    m0 = (b % ntm) * BM;
    e = b / ntm;
    int l, h;
    share_of(g.lo, g.hi, g.kept[e], e, l, h);
    row0 = g.offsets[e] + l;
    klen = h - l;
    mvalid = min(BM, g.M - m0);
    if (klen == 0 && g.accumulate) return;
  } else {
    const int ntn = (g.N + BN - 1) / BN;
    const int rt = blockIdx.x / ntn;
    if (rt >= g.ntiles[0]) return;
    n0 = (blockIdx.x % ntn) * BN;
    const RowTile t = g.tiles[rt];
    e = t.e;
    row0 = t.row0;
    mvalid = t.nrows;
    klen = g.K;
  }
  const int nvalid = min(BN, g.N - n0);

  f32x16 acc[WTM][WTN], acc2[DUAL ? WTM : 1][DUAL ? WTN : 1];
#pragma unroll
  for (int i = 0; i < WTM; ++i)
#pragma unroll
    for (int j = 0; j < WTN; ++j) {
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
      if constexpr (DUAL) {
#pragma unroll
        for (int v = 0; v < 16; ++v) acc2[i][j][v] = 0.f;
      }
    }

  for (int pass = 0; pass < (CHAIN ? 2 : 1); ++pass) {
    const bf16* A = reinterpret_cast<const bf16*>(pass == 0 ? g.A : g.A2);
    const bf16* B = reinterpret_cast<const bf16*>(pass == 0 ? g.B : g.B2);
    const bf16* B2 = reinterpret_cast<const bf16*>(g.B2);
    uint4 ra[A_CH], rb[B_CH], rb2[DUAL ? B_CH : 1];

    auto load_global = [&](int k0) {
#pragma unroll
      for (int i = 0; i < A_CH; ++i) {
        const int id = tid + 256 * i;
        if constexpr (A_KC) {
          const int r = id >> 3, c = id & 7;
          const int rr = min(r, mvalid - 1);   // rows past the tile's end repeat its last row (never stored)
          ra[i] = *reinterpret_cast<const uint4*>(A + (size_t)(row0 + rr) * g.K + k0 + c * 8);
        } else {
          const int kr = id / (BM / 8), c = id % (BM / 8);
          ra[i] = make_uint4(0, 0, 0, 0);
          if (k0 + kr < klen && c * 8 < mvalid)
            ra[i] = *reinterpret_cast<const uint4*>(A + (size_t)(row0 + k0 + kr) * g.M + m0 + c * 8);
        }
      }
#pragma unroll
      for (int i = 0; i < B_CH; ++i) {
        const int id = tid + 256 * i;
        rb[i] = make_uint4(0, 0, 0, 0);
        if constexpr (DUAL) rb2[i] = make_uint4(0, 0, 0, 0);
        if constexpr (B_KC) {
          const int r = id >> 3, c = id & 7;
          if (r < nvalid) rb[i] = *reinterpret_cast<const uint4*>(B + ((size_t)e * g.N + n0 + r) * g.K + k0 + c * 8);
        } else {
          const int kr = id / (BN / 8), c = id % (BN / 8);
          if (c * 8 < nvalid) {
            if constexpr (MODE == MODE_TN) {
              if (k0 + kr < klen) rb[i] = *reinterpret_cast<const uint4*>(B + (size_t)(row0 + k0 + kr) * g.N + n0 + c * 8);
            } else {
              const size_t off = ((size_t)e * g.K + k0 + kr) * g.N + n0 + c * 8;
              rb[i] = *reinterpret_cast<const uint4*>(B + off);
              if constexpr (DUAL) rb2[i] = *reinterpret_cast<const uint4*>(B2 + off);
            }
          }
        }
      }
    };
    auto store_lds = [&](int buf) {
      char* sa = smem + buf * STAGE;
      char* sb = sa + A_BYTES;
#pragma unroll
      for (int i = 0; i < A_CH; ++i) {
        const int id = tid + 256 * i;
        if constexpr (A_KC) *reinterpret_cast<uint4*>(sa + kc_off(id >> 3, id & 7)) = ra[i];
        else *reinterpret_cast<uint4*>(sa + ks_off<BM>(id / (BM / 8), (id % (BM / 8)) * 16)) = ra[i];
      }
#pragma unroll
      for (int i = 0; i < B_CH; ++i) {
        const int id = tid + 256 * i;
        int off;
        if constexpr (B_KC) off = kc_off(id >> 3, id & 7);
        else off = ks_off<BN>(id / (BN / 8), (id % (BN / 8)) * 16);
        *reinterpret_cast<uint4*>(sb + off) = rb[i];
        if constexpr (DUAL) *reinterpret_cast<uint4*>(sb + B_BYTES + off) = rb2[i];
      }
    };
    auto compute = [&](int buf) {
      const char* sa = smem + buf * STAGE;
      const char* sb = sa + A_BYTES;
#pragma unroll
      for (int ks = 0; ks < BK / 16; ++ks) {
        bf16x8 af[WTM], bfr[WTN], bfr2[DUAL ? WTN : 1];
#pragma unroll
        for (int i = 0; i < WTM; ++i) {
          const int base = (wm * WTM + i) * 32;
          if constexpr (A_KC) af[i] = lds_read_kc(sa, base + (lane & 31), ks * 2 + (lane >> 5));
          else af[i] = lds_read_ks<BM>(sa, ks, base, lane);
        }
#pragma unroll
        for (int j = 0; j < WTN; ++j) {
          const int base = (wn * WTN + j) * 32;
          if constexpr (B_KC) bfr[j] = lds_read_kc(sb, base + (lane & 31), ks * 2 + (lane >> 5));
          else bfr[j] = lds_read_ks<BN>(sb, ks, base, lane);
          if constexpr (DUAL) bfr2[j] = lds_read_ks<BN>(sb + B_BYTES, ks, base, lane);
        }
#pragma unroll
        for (int i = 0; i < WTM; ++i)
#pragma unroll
          for (int j = 0; j < WTN; ++j) {
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
            if constexpr (DUAL) acc2[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr2[j], acc2[i][j], 0, 0, 0);
          }
      }
    };

    const int KT = (klen + BK - 1) / BK;
    if (KT > 0) {
      load_global(0);
      __syncthreads();   // every wave is done reading the previous pass's buffers
      store_lds(0);
      __syncthreads();
      for (int kt = 0; kt < KT; ++kt) {
        if (kt + 1 < KT) load_global((kt + 1) * BK);
        compute(kt & 1);
        if (kt + 1 < KT) store_lds((kt + 1) & 1);
        __syncthreads();
      }
    }
  }

  // epilogue: accumulator register v of lane l is (row (v/4)*8 + (l/32)*4 + v%4, column l%32) of its 32x32 tile
#pragma unroll
  for (int i = 0; i < WTM; ++i)
#pragma unroll
    for (int j = 0; j < WTN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = (wm * WTM + i) * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
        const int n = (wn * WTN + j) * 32 + (lane & 31);
        if (m < mvalid && n < nvalid) {
          size_t idx;
          if constexpr (MODE == MODE_TN) idx = ((size_t)e * g.M + m0 + m) * g.N + n0 + n;
          else idx = (size_t)(row0 + m) * g.N + n0 + n;
          epilogue<bf16, EPI>(g, idx, acc[i][j][v], DUAL ? acc2[DUAL ? i : 0][DUAL ? j : 0][v] : 0.f);
        }
      }
}

constexpr int V1_WTM = 2, V1_WTN = 2;   // 128 x 128 block tile
int gemm_bf16_tile_rows() { return 2 * V1_WTM * 32; }

template <int MODE, int EPI, bool DUAL, bool CHAIN>
static int launch_one(const GemmArgs& g, int max_tiles, hipStream_t s) {
  constexpr int WTM = V1_WTM, WTN = V1_WTN;
  constexpr int BM = 2 * WTM * 32, BN = 2 * WTN * 32;
  constexpr int lds = 2 * (BM * BK * 2 + BN * BK * 2 * (DUAL ? 2 : 1));
  auto kern = gemm_bf16_kernel<MODE, EPI, DUAL, CHAIN, WTM, WTN>;
  static bool attr_done = false;   // benign race: the attribute call is idempotent
  if (!attr_done) {
    hipError_t err = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (err != hipSuccess) return set_hip_error(err);
    attr_done = true;
  }
  const int ntn = (g.N + BN - 1) / BN;
  long long blocks;
  if (MODE == MODE_TN) blocks = (long long)ntn * ((g.M + BM - 1) / BM) * g.E;
  else blocks = (long long)ntn * max_tiles;
  kern<<<dim3((unsigned)blocks), 256, lds, s>>>(g);
  return launch_status();
}

int launch_gemm_bf16(int mode, int epi, bool dual, bool chain, const GemmArgs& g, int max_tiles, hipStream_t s) {
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

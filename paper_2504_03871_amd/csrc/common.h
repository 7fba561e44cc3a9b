// Shared host/device helpers of the MoE library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/moe.h"

namespace moe {

constexpr int WAVE = 64;

// ---------------------------------------------------------------- host side
int set_hip_error(hipError_t e);          // records e for moe_last_hip_error(), returns MOE_ERR_HIP
int check_cfg(const moe_cfg* c);          // MOE_OK or an argument error
inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }
inline int launch_status() {
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? MOE_OK : set_hip_error(e);
}
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline size_t elt_size(const moe_cfg* c) { return c->dtype == MOE_DTYPE_F32 ? 4 : 2; }
inline bool is_half(const moe_cfg* c) { return c->dtype != MOE_DTYPE_F32; }   // 16-bit storage: the MFMA kernels
// The grouped GEMMs reach an operand through one buffer descriptor and a 32-bit byte offset per lane.  The
// longest walks are an expert's whole share in the weight-gradient GEMM (rows x max(d, f) elements; one expert
// may hold every assignment) and one expert's weight matrix (d x f elements; fp32 gradients are 4 bytes wide).
inline bool offsets_fit_32_bits(long long T, long long k, long long d, long long f, int elt_bytes) {
  const long long lim = 1ll << 32;
  return T * k * (d > f ? d : f) * elt_bytes < lim && d * f * 4 < lim;
}

// Workspace layout (bytes from the start of `ws`), one region per user; see api.hip.
struct WsLayout {
  size_t dispatch_blk_cnt;  // int32 [nblk + 1][E]: per-block counts (or their prefixes) and a row of totals
  size_t tile_map;          // int32 header + int4 entries (grouped GEMM row tiles)
  size_t route_partials;    // fp32 [token slice][E][d]: partial sums of the gate weight gradient
  size_t route_wrt;         // fp32 [E][d]: transposed router weight
  size_t ffn_split;         // fp32 partial sums of split-K row tiles (gemm.h), when split_k_applies
  size_t ffn_bwd_dact;      // storage type [planes][T*k][f]: dA (GELU) or dG | dU (SwiGLU)
  size_t total;
};
WsLayout ws_layout(const moe_cfg* c);
size_t route_wfrag_bytes(int d, int E);   // gate weight in MFMA operand layout (route.hip)

constexpr int DISPATCH_CHUNK = 1024;   // assignments ranked by one block

// Geometry of the dense gate-weight-gradient kernel: a thread owns one 16-byte column group, cg_pow2
// threads span a token row (a power of two, at most 256; wider rows take several column blocks), a block
// of 256 threads works on 256 / cg_pow2 token slices at once, each `tps` tokens long, and every slice
// writes its own row of partial sums.  More than 16 experts are split into groups of 16 that run as blocks of
// their own.  tps grows with the problem and with the number of groups so that the grid stays near two
// blocks per compute unit and the partial sums (a row of E x d floats per slice) stay small.
struct RouteBwdGeom { int cg_pow2, slices_per_block, tps, col_blocks, row_blocks, partial_rows; };
inline RouteBwdGeom route_bwd_geom(int T, int d, int elt_bytes, int E) {
  RouteBwdGeom gm;
  const int cg = d / (16 / elt_bytes);
  gm.cg_pow2 = 4;   // at most 64 slices per block
  while (gm.cg_pow2 < cg && gm.cg_pow2 < 256) gm.cg_pow2 <<= 1;
  gm.slices_per_block = 256 / gm.cg_pow2;
  gm.col_blocks = (cg + gm.cg_pow2 - 1) / gm.cg_pow2;
  const int groups = (E + 15) / 16;
  long long tps = ((long long)T * gm.col_blocks * groups) / (512ll * gm.slices_per_block);
  const int cap = 1024 / gm.slices_per_block;   // the block stages slices * tps * E <= 1024 * 16 floats in LDS
  gm.tps = (int)(tps < 16 ? 16 : (tps > 256 ? 256 : tps));
  if (gm.tps > cap) gm.tps = cap;
  gm.row_blocks = (T + gm.tps * gm.slices_per_block - 1) / (gm.tps * gm.slices_per_block);
  gm.partial_rows = gm.row_blocks * gm.slices_per_block;
  return gm;
}
// Gate weight gradient on the matrix cores (bf16 or fp16 inputs, more than 16 experts): a block owns 128 columns of
// x, up to 128 experts and a slice of tokens, a multiple of 32 long, chosen so that the grid is about two
// blocks per compute unit; every slice writes one row of E x d partial sums.
constexpr int ROUTE_BWD_MFMA_COLS = 128, ROUTE_BWD_MFMA_KSTEP = 32, ROUTE_BWD_MFMA_EXPERTS = 128;
struct RouteBwdMfmaGeom { int col_blocks, expert_blocks, slice_tokens, rows; };
inline bool route_bwd_uses_mfma(int storage_is_16bit, int E) { return storage_is_16bit && E > 16; }
inline RouteBwdMfmaGeom route_bwd_mfma_geom(int T, int d, int E) {
  RouteBwdMfmaGeom gm;
  gm.col_blocks = (d + ROUTE_BWD_MFMA_COLS - 1) / ROUTE_BWD_MFMA_COLS;
  gm.expert_blocks = (E + ROUTE_BWD_MFMA_EXPERTS - 1) / ROUTE_BWD_MFMA_EXPERTS;
  int slices = 512 / (gm.col_blocks * gm.expert_blocks);
  if (slices < 1) slices = 1;
  int len = (T + slices - 1) / slices;
  len = (len + ROUTE_BWD_MFMA_KSTEP - 1) / ROUTE_BWD_MFMA_KSTEP * ROUTE_BWD_MFMA_KSTEP;
  if (len < 4 * ROUTE_BWD_MFMA_KSTEP) len = 4 * ROUTE_BWD_MFMA_KSTEP;
  gm.slice_tokens = len;
  gm.rows = (T + len - 1) / len;
  if (gm.rows < 1) gm.rows = 1;
  return gm;
}
constexpr int TILE_ROWS_MIN = 64;      // smallest row-tile height any grouped GEMM uses (sizes the tile map)

// ---------------------------------------------------------------- device side
#ifdef __HIPCC__
typedef __bf16 bf16;
typedef _Float16 f16;

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  bf16 h = (bf16)f;  // v_cvt_pk_bf16_f32: round to nearest even
  return (uint32_t)(*reinterpret_cast<unsigned short*>(&h));
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}
__device__ __forceinline__ float f16_bits_to_f32(uint32_t b) {
  const unsigned short h = (unsigned short)b;
  return (float)(*reinterpret_cast<const f16*>(&h));
}
__device__ __forceinline__ uint32_t f32_to_f16_bits(float f) {
  const f16 h = (f16)f;   // round to nearest even
  return (uint32_t)(*reinterpret_cast<const unsigned short*>(&h));
}
__device__ __forceinline__ uint32_t pack_f16x2(float lo, float hi) {
  return f32_to_f16_bits(lo) | (f32_to_f16_bits(hi) << 16);
}

// 16-byte vector of activations: 4 fp32 or 8 bf16.  load_nt / store_nt mark streaming traffic (data touched
// once by the kernel) as non-temporal, which is what lets a plain copy reach the machine's HBM ceiling.
typedef unsigned nt_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load16_nt(const void* p) {
  const nt_u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const nt_u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store16_nt(void* p, const uint4& r) {
  __builtin_nontemporal_store(nt_u32x4{r.x, r.y, r.z, r.w}, reinterpret_cast<nt_u32x4*>(p));
}
template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int N = 4;
  float4 raw;
  __device__ __forceinline__ void load(const float* p) { raw = *reinterpret_cast<const float4*>(p); }
  __device__ __forceinline__ void store(float* p) const { *reinterpret_cast<float4*>(p) = raw; }
  __device__ __forceinline__ void load_nt(const float* p) { const uint4 u = load16_nt(p); raw = make_float4(__uint_as_float(u.x), __uint_as_float(u.y), __uint_as_float(u.z), __uint_as_float(u.w)); }
  __device__ __forceinline__ void store_nt(float* p) const { store16_nt(p, make_uint4(__float_as_uint(raw.x), __float_as_uint(raw.y), __float_as_uint(raw.z), __float_as_uint(raw.w))); }
  __device__ __forceinline__ void unpack(float* f) const { f[0] = raw.x; f[1] = raw.y; f[2] = raw.z; f[3] = raw.w; }
  __device__ __forceinline__ void pack(const float* f) { raw = make_float4(f[0], f[1], f[2], f[3]); }
};
template <> struct Vec16<bf16> {
  static constexpr int N = 8;
  uint4 raw;
  __device__ __forceinline__ void load(const bf16* p) { raw = *reinterpret_cast<const uint4*>(p); }
  __device__ __forceinline__ void store(bf16* p) const { *reinterpret_cast<uint4*>(p) = raw; }
  __device__ __forceinline__ void load_nt(const bf16* p) { raw = load16_nt(p); }
  __device__ __forceinline__ void store_nt(bf16* p) const { store16_nt(p, raw); }
  __device__ __forceinline__ void unpack(float* f) const {
    const uint32_t u[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) { f[2 * i] = __uint_as_float(u[i] << 16); f[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u); }
  }
  __device__ __forceinline__ void pack(const float* f) {
    raw = make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
  }
};

template <> struct Vec16<f16> {
  static constexpr int N = 8;
  uint4 raw;
  __device__ __forceinline__ void load(const f16* p) { raw = *reinterpret_cast<const uint4*>(p); }
  __device__ __forceinline__ void store(f16* p) const { *reinterpret_cast<uint4*>(p) = raw; }
  __device__ __forceinline__ void load_nt(const f16* p) { raw = load16_nt(p); }
  __device__ __forceinline__ void store_nt(f16* p) const { store16_nt(p, raw); }
  __device__ __forceinline__ void unpack(float* f) const {
    const uint32_t u[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) { f[2 * i] = f16_bits_to_f32(u[i] & 0xffffu); f[2 * i + 1] = f16_bits_to_f32(u[i] >> 16); }
  }
  __device__ __forceinline__ void pack(const float* f) {
    raw = make_uint4(pack_f16x2(f[0], f[1]), pack_f16x2(f[2], f[3]), pack_f16x2(f[4], f[5]), pack_f16x2(f[6], f[7]));
  }
};

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(f16 v) { return (float)v; }
__device__ __forceinline__ float to_f32(bf16 v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return (bf16)v; }
template <> __device__ __forceinline__ f16 from_f32<f16>(float v) { return (f16)v; }

// This GPU's share [l, h) of expert e's kept list: clamped to [0, kept], inverted = empty.
__device__ __forceinline__ void share_of(const int32_t* __restrict__ lo, const int32_t* __restrict__ hi,
                                         int m, int e, int& l, int& h) {
  l = 0;
  h = m;
  if (lo != nullptr) {
    l = min(max(lo[e], 0), m);
    h = min(max(hi[e], 0), m);
    if (h < l) h = l;
  }
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int s = 32; s > 0; s >>= 1) v += __shfl_xor(v, s, WAVE);
  return v;
}

__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
  for (int s = 32; s > 0; s >>= 1) v += __shfl_xor(v, s, WAVE);
  return v;
}
// inclusive prefix sum over the lanes of a wave
__device__ __forceinline__ int wave_scan_i(int v) {
  const int lane = threadIdx.x & (WAVE - 1);
#pragma unroll
  for (int d = 1; d < WAVE; d <<= 1) {
    const int up = __shfl_up(v, d, WAVE);
    if (lane >= d) v += up;
  }
  return v;
}

// exact-erf GELU pieces, SiLU pieces (fp32)
__device__ __forceinline__ float gelu_f(float a) { return 0.5f * a * erfcf(-a * 0.70710678118654752440f); }
__device__ __forceinline__ float gelu_grad_f(float a) {
  return 0.5f * erfcf(-a * 0.70710678118654752440f) + a * 0.39894228040143267794f * __expf(-0.5f * a * a);
}
__device__ __forceinline__ float sigmoid_f(float g) { return 1.0f / (1.0f + __expf(-g)); }
// Phi(v) and the normal density at v for the fp16 GELU epilogues, which have no table: erfc by the rational
// approximation 7.1.26 of Abramowitz and Stegun (t = 1 / (1 + p x), erfc(x) = t (a1 + ... + a5 t^4) exp(-x^2),
// absolute error 1.5e-7), one exponential and one reciprocal instead of a library erfc.  Over every finite fp16
// number Phi is within 2.8e-7 and gelu' within 3e-7 of the exact values, against an fp16 resolution of 4.9e-4.
__device__ __forceinline__ void gelu_pieces_fast(float v, float& phi, float& pdf) {
  const float x = fabsf(v) * 0.70710678118654752440f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, x, 1.0f));
  const float poly = t * fmaf(t, fmaf(t, fmaf(t, fmaf(t, 1.061405429f, -1.453152027f), 1.421413741f), -0.284496736f), 0.254829592f);
  const float ex = __builtin_amdgcn_exp2f(-(x * x) * 1.44269504088896340736f);   // exp(-v^2 / 2)
  const float half = 0.5f * poly * ex;
  phi = v >= 0.f ? 1.0f - half : half;
  pdf = 0.39894228040143267794f * ex;
}
__device__ __forceinline__ float phi_fast(float v) {
  float phi, pdf;
  gelu_pieces_fast(v, phi, pdf);
  return phi;
}
__device__ __forceinline__ float gelu_grad_fast(float v) {
  float phi, pdf;
  gelu_pieces_fast(v, phi, pdf);
  return fmaf(v, pdf, phi);
}
#endif  // __HIPCC__

}  // namespace moe

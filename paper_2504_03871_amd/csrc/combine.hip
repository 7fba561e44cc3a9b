// Combine (weighted un-permute) and its backward.
//
// Section 2.1 of the paper: the outputs of a token's top-k experts are weighted by the gate scores
// and summed.  Written in gather form (one wave per token walks its k slots in slot order), so the
// fp32 sum has a fixed order and no atomics are needed.  Section 5: the gradient of the block output
// feeds both the expert outputs (dy = w * dOut) and the scores (dw = <dOut, y>).
#include "common.h"

namespace moe {

constexpr int CB_THREADS = 256;

// Row of slot a if it is kept and inside this GPU's share, else -1.
__device__ __forceinline__ int live_row(int a, const int32_t* __restrict__ topk_idx, const int32_t* __restrict__ row_of,
                                        const int32_t* __restrict__ offsets, const int32_t* __restrict__ kept,
                                        const int32_t* __restrict__ lo, const int32_t* __restrict__ hi) {
  const int row = row_of[a];
  if (row < 0) return -1;
  if (lo == nullptr) return row;
  const int e = topk_idx[a];
  int l, h;
  share_of(lo, hi, kept[e], e, l, h);
  const int pos = row - offsets[e];
  return (pos >= l && pos < h) ? row : -1;
}

// KMAX: compile-time bound on k (2, 4 or 8); CU: column chunks of 16 bytes per lane kept in flight
// (k * CU loads are issued before anything is used).  y_perm is read once: non-temporal loads.
template <typename T, int KMAX, int CU>
__global__ __launch_bounds__(CB_THREADS) void combine_kernel(
    const T* __restrict__ y_perm, const float* __restrict__ topk_w, const int32_t* __restrict__ topk_idx,
    const int32_t* __restrict__ row_of, const int32_t* __restrict__ offsets, const int32_t* __restrict__ kept,
    const int32_t* __restrict__ lo, const int32_t* __restrict__ hi, T* __restrict__ out, int Tn, int d, int k,
    int accumulate) {
  constexpr int VN = Vec16<T>::N;
  const int lane = threadIdx.x & (WAVE - 1);
  const int t = (blockIdx.x * CB_THREADS + threadIdx.x) / WAVE;
  if (t >= Tn) return;
  int rows[KMAX];
  float wj[KMAX];
#pragma unroll
  for (int j = 0; j < KMAX; ++j) {
    rows[j] = -1;
    wj[j] = 0.f;
    if (j < k) {
      rows[j] = live_row(t * k + j, topk_idx, row_of, offsets, kept, lo, hi);
      wj[j] = (topk_w != nullptr) ? topk_w[(size_t)t * k + j] : 1.f;
    }
  }
  for (int c0 = lane * VN; c0 < d; c0 += WAVE * VN * CU) {
    Vec16<T> v[KMAX][CU];
#pragma unroll
    for (int j = 0; j < KMAX; ++j)
      if (rows[j] >= 0) {
#pragma unroll
        for (int u = 0; u < CU; ++u)
          if (c0 + u * WAVE * VN < d) v[j][u].load_nt(y_perm + (size_t)rows[j] * d + c0 + u * WAVE * VN);
      }
#pragma unroll
    for (int u = 0; u < CU; ++u) {
      const int c = c0 + u * WAVE * VN;
      if (c >= d) break;
      float acc[VN];
      if (accumulate) {
        Vec16<T> o;
        o.load(out + (size_t)t * d + c);
        o.unpack(acc);
      } else {
#pragma unroll
        for (int i = 0; i < VN; ++i) acc[i] = 0.f;
      }
#pragma unroll
      for (int j = 0; j < KMAX; ++j)     // fixed slot order: the sum is deterministic
        if (rows[j] >= 0) {
          float f[VN];
          v[j][u].unpack(f);
#pragma unroll
          for (int i = 0; i < VN; ++i) acc[i] = fmaf(wj[j], f[i], acc[i]);
        }
      Vec16<T> o;
      o.pack(acc);
      o.store(out + (size_t)t * d + c);
    }
  }
}

template <typename T, int KMAX, int CU>
__global__ __launch_bounds__(CB_THREADS) void combine_bwd_kernel(
    const T* __restrict__ d_out, const T* __restrict__ y_perm, const float* __restrict__ topk_w,
    const int32_t* __restrict__ topk_idx, const int32_t* __restrict__ row_of, const int32_t* __restrict__ offsets,
    const int32_t* __restrict__ kept, const int32_t* __restrict__ lo, const int32_t* __restrict__ hi,
    T* __restrict__ dy_perm, float* __restrict__ d_topk_w, int Tn, int d, int k) {
  constexpr int VN = Vec16<T>::N;
  const int lane = threadIdx.x & (WAVE - 1);
  const int t = (blockIdx.x * CB_THREADS + threadIdx.x) / WAVE;
  if (t >= Tn) return;
  int rows[KMAX];
  float wj[KMAX], dot[KMAX];
#pragma unroll
  for (int j = 0; j < KMAX; ++j) {
    rows[j] = -1;
    wj[j] = 0.f;
    dot[j] = 0.f;
    if (j < k) {
      rows[j] = live_row(t * k + j, topk_idx, row_of, offsets, kept, lo, hi);
      wj[j] = topk_w[(size_t)t * k + j];
    }
  }
  for (int c0 = lane * VN; c0 < d; c0 += WAVE * VN * CU) {
    Vec16<T> g[CU], v[KMAX][CU];
#pragma unroll
    for (int u = 0; u < CU; ++u)
      if (c0 + u * WAVE * VN < d) g[u].load_nt(d_out + (size_t)t * d + c0 + u * WAVE * VN);
#pragma unroll
    for (int j = 0; j < KMAX; ++j)
      if (rows[j] >= 0) {
#pragma unroll
        for (int u = 0; u < CU; ++u)
          if (c0 + u * WAVE * VN < d) v[j][u].load_nt(y_perm + (size_t)rows[j] * d + c0 + u * WAVE * VN);
      }
#pragma unroll
    for (int u = 0; u < CU; ++u) {
      const int c = c0 + u * WAVE * VN;
      if (c >= d) break;
      float gf[VN];
      g[u].unpack(gf);
#pragma unroll
      for (int j = 0; j < KMAX; ++j)
        if (rows[j] >= 0) {
          float f[VN], o[VN];
          v[j][u].unpack(f);
#pragma unroll
          for (int i = 0; i < VN; ++i) { dot[j] = fmaf(gf[i], f[i], dot[j]); o[i] = wj[j] * gf[i]; }
          Vec16<T> ov;
          ov.pack(o);
          ov.store_nt(dy_perm + (size_t)rows[j] * d + c);
        }
    }
  }
#pragma unroll
  for (int j = 0; j < KMAX; ++j)
    if (j < k) {
      const float s = wave_sum(dot[j]);
      if (lane == 0) d_topk_w[(size_t)t * k + j] = (rows[j] >= 0) ? s : 0.f;
    }
}

// Column units in flight per lane: enough to cover a whole row where the row is long (k <= 2: eight units = 8 KB of
// 16-bit elements; more experts per token: four), half that for short rows, where the extra units would only be
// predicated off.
template <typename TY, int KM, int CU>
static void launch_combine_one(const moe_cfg* c, const void* y_perm, const float* w, const int32_t* idx, const int32_t* row_of,
                               const int32_t* offsets, const int32_t* kept, const int32_t* lo, const int32_t* hi, void* out,
                               int accumulate, hipStream_t s) {
  const int grid = (c->T + CB_THREADS / WAVE - 1) / (CB_THREADS / WAVE);
  combine_kernel<TY, KM, CU><<<grid, CB_THREADS, 0, s>>>((const TY*)y_perm, w, idx, row_of, offsets, kept, lo, hi, (TY*)out,
                                                         c->T, c->d_model, c->k, accumulate);
}
template <typename TY, int KM, int CU>
static void launch_combine_bwd_one(const moe_cfg* c, const void* d_out, const void* y_perm, const float* w, const int32_t* idx,
                                   const int32_t* row_of, const int32_t* offsets, const int32_t* kept, const int32_t* lo,
                                   const int32_t* hi, void* dy_perm, float* dw, hipStream_t s) {
  const int grid = (c->T + CB_THREADS / WAVE - 1) / (CB_THREADS / WAVE);
  combine_bwd_kernel<TY, KM, CU><<<grid, CB_THREADS, 0, s>>>((const TY*)d_out, (const TY*)y_perm, w, idx, row_of, offsets, kept,
                                                             lo, hi, (TY*)dy_perm, dw, c->T, c->d_model, c->k);
}
// true when a row spans more than `units` column units of a wave (16 bytes per lane each)
template <typename TY>
static bool long_row(const moe_cfg* c, int units) { return c->d_model > units * WAVE * Vec16<TY>::N; }

template <typename TY>
static void launch_combine_typed(const moe_cfg* c, const void* y_perm, const float* w, const int32_t* idx, const int32_t* row_of,
                                 const int32_t* offsets, const int32_t* kept, const int32_t* lo, const int32_t* hi, void* out,
                                 int accumulate, hipStream_t s) {
#define MOE_ARGS c, y_perm, w, idx, row_of, offsets, kept, lo, hi, out, accumulate, s
  if (c->k <= 2) { if (long_row<TY>(c, 4)) launch_combine_one<TY, 2, 8>(MOE_ARGS); else launch_combine_one<TY, 2, 4>(MOE_ARGS); }
  else if (c->k <= 4) { if (long_row<TY>(c, 2)) launch_combine_one<TY, 4, 4>(MOE_ARGS); else launch_combine_one<TY, 4, 2>(MOE_ARGS); }
  else { if (long_row<TY>(c, 2)) launch_combine_one<TY, 8, 4>(MOE_ARGS); else launch_combine_one<TY, 8, 2>(MOE_ARGS); }
#undef MOE_ARGS
}
template <typename TY>
static void launch_combine_bwd_typed(const moe_cfg* c, const void* d_out, const void* y_perm, const float* w, const int32_t* idx,
                                     const int32_t* row_of, const int32_t* offsets, const int32_t* kept, const int32_t* lo,
                                     const int32_t* hi, void* dy_perm, float* dw, hipStream_t s) {
#define MOE_ARGS c, d_out, y_perm, w, idx, row_of, offsets, kept, lo, hi, dy_perm, dw, s
  if (c->k <= 2) { if (long_row<TY>(c, 4)) launch_combine_bwd_one<TY, 2, 8>(MOE_ARGS); else launch_combine_bwd_one<TY, 2, 4>(MOE_ARGS); }
  else if (c->k <= 4) { if (long_row<TY>(c, 2)) launch_combine_bwd_one<TY, 4, 4>(MOE_ARGS); else launch_combine_bwd_one<TY, 4, 2>(MOE_ARGS); }
  else { if (long_row<TY>(c, 2)) launch_combine_bwd_one<TY, 8, 4>(MOE_ARGS); else launch_combine_bwd_one<TY, 8, 2>(MOE_ARGS); }
#undef MOE_ARGS
}

int launch_combine(const moe_cfg* c, const void* y_perm, const float* w, const int32_t* idx, const int32_t* row_of,
                   const int32_t* offsets, const int32_t* kept, const int32_t* lo, const int32_t* hi, void* out,
                   int accumulate, hipStream_t s) {
  if (c->dtype == MOE_DTYPE_BF16) launch_combine_typed<bf16>(c, y_perm, w, idx, row_of, offsets, kept, lo, hi, out, accumulate, s);
  else if (c->dtype == MOE_DTYPE_F16) launch_combine_typed<f16>(c, y_perm, w, idx, row_of, offsets, kept, lo, hi, out, accumulate, s);
  else launch_combine_typed<float>(c, y_perm, w, idx, row_of, offsets, kept, lo, hi, out, accumulate, s);
  return launch_status();
}

int launch_combine_bwd(const moe_cfg* c, const void* d_out, const void* y_perm, const float* w, const int32_t* idx,
                       const int32_t* row_of, const int32_t* offsets, const int32_t* kept, const int32_t* lo,
                       const int32_t* hi, void* dy_perm, float* dw, hipStream_t s) {
  if (c->dtype == MOE_DTYPE_BF16) launch_combine_bwd_typed<bf16>(c, d_out, y_perm, w, idx, row_of, offsets, kept, lo, hi, dy_perm, dw, s);
  else if (c->dtype == MOE_DTYPE_F16) launch_combine_bwd_typed<f16>(c, d_out, y_perm, w, idx, row_of, offsets, kept, lo, hi, dy_perm, dw, s);
  else launch_combine_bwd_typed<float>(c, d_out, y_perm, w, idx, row_of, offsets, kept, lo, hi, dy_perm, dw, s);
  return launch_status();
}

}  // namespace moe

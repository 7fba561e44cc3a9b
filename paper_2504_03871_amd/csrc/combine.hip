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

template <typename T>
__global__ __launch_bounds__(CB_THREADS) void combine_kernel(
    const T* __restrict__ y_perm, const float* __restrict__ topk_w, const int32_t* __restrict__ topk_idx,
    const int32_t* __restrict__ row_of, const int32_t* __restrict__ offsets, const int32_t* __restrict__ kept,
    const int32_t* __restrict__ lo, const int32_t* __restrict__ hi, T* __restrict__ out, int Tn, int d, int k,
    int accumulate) {
  constexpr int VN = Vec16<T>::N;
  const int lane = threadIdx.x & (WAVE - 1);
  const int t = (blockIdx.x * CB_THREADS + threadIdx.x) / WAVE;
  if (t >= Tn) return;
  int rows[MOE_MAX_K];
  float wj[MOE_MAX_K];
#pragma unroll
  for (int j = 0; j < MOE_MAX_K; ++j) {
    rows[j] = -1;
    wj[j] = 0.f;
    if (j < k) {
      rows[j] = live_row(t * k + j, topk_idx, row_of, offsets, kept, lo, hi);
      wj[j] = (topk_w != nullptr) ? topk_w[(size_t)t * k + j] : 1.f;
    }
  }
  for (int c = lane * VN; c < d; c += WAVE * VN) {
    Vec16<T> v[MOE_MAX_K];
#pragma unroll
    for (int j = 0; j < MOE_MAX_K; ++j)
      if (rows[j] >= 0) v[j].load(y_perm + (size_t)rows[j] * d + c);
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
    for (int j = 0; j < MOE_MAX_K; ++j)
      if (rows[j] >= 0) {
        float f[VN];
        v[j].unpack(f);
#pragma unroll
        for (int i = 0; i < VN; ++i) acc[i] = fmaf(wj[j], f[i], acc[i]);
      }
    Vec16<T> o;
    o.pack(acc);
    o.store(out + (size_t)t * d + c);
  }
}

template <typename T>
__global__ __launch_bounds__(CB_THREADS) void combine_bwd_kernel(
    const T* __restrict__ d_out, const T* __restrict__ y_perm, const float* __restrict__ topk_w,
    const int32_t* __restrict__ topk_idx, const int32_t* __restrict__ row_of, const int32_t* __restrict__ offsets,
    const int32_t* __restrict__ kept, const int32_t* __restrict__ lo, const int32_t* __restrict__ hi,
    T* __restrict__ dy_perm, float* __restrict__ d_topk_w, int Tn, int d, int k) {
  constexpr int VN = Vec16<T>::N;
  const int lane = threadIdx.x & (WAVE - 1);
  const int t = (blockIdx.x * CB_THREADS + threadIdx.x) / WAVE;
  if (t >= Tn) return;
  int rows[MOE_MAX_K];
  float wj[MOE_MAX_K], dot[MOE_MAX_K];
#pragma unroll
  for (int j = 0; j < MOE_MAX_K; ++j) {
    rows[j] = -1;
    wj[j] = 0.f;
    dot[j] = 0.f;
    if (j < k) {
      rows[j] = live_row(t * k + j, topk_idx, row_of, offsets, kept, lo, hi);
      wj[j] = topk_w[(size_t)t * k + j];
    }
  }
  for (int c = lane * VN; c < d; c += WAVE * VN) {
    Vec16<T> g, v[MOE_MAX_K];
    g.load(d_out + (size_t)t * d + c);
#pragma unroll
    for (int j = 0; j < MOE_MAX_K; ++j)
      if (rows[j] >= 0) v[j].load(y_perm + (size_t)rows[j] * d + c);
    float gf[VN];
    g.unpack(gf);
#pragma unroll
    for (int j = 0; j < MOE_MAX_K; ++j)
      if (rows[j] >= 0) {
        float f[VN], o[VN];
        v[j].unpack(f);
#pragma unroll
        for (int i = 0; i < VN; ++i) { dot[j] = fmaf(gf[i], f[i], dot[j]); o[i] = wj[j] * gf[i]; }
        Vec16<T> ov;
        ov.pack(o);
        ov.store(dy_perm + (size_t)rows[j] * d + c);
      }
  }
#pragma unroll
  for (int j = 0; j < MOE_MAX_K; ++j)
    if (j < k) {
      const float s = wave_sum(dot[j]);
      if (lane == 0) d_topk_w[(size_t)t * k + j] = (rows[j] >= 0) ? s : 0.f;
    }
}

int launch_combine(const moe_cfg* c, const void* y_perm, const float* w, const int32_t* idx, const int32_t* row_of,
                   const int32_t* offsets, const int32_t* kept, const int32_t* lo, const int32_t* hi, void* out,
                   int accumulate, hipStream_t s) {
  const int grid = (c->T + CB_THREADS / WAVE - 1) / (CB_THREADS / WAVE);
  if (c->dtype == MOE_DTYPE_BF16)
    combine_kernel<bf16><<<grid, CB_THREADS, 0, s>>>((const bf16*)y_perm, w, idx, row_of, offsets, kept, lo, hi, (bf16*)out, c->T, c->d_model, c->k, accumulate);
  else
    combine_kernel<float><<<grid, CB_THREADS, 0, s>>>((const float*)y_perm, w, idx, row_of, offsets, kept, lo, hi, (float*)out, c->T, c->d_model, c->k, accumulate);
  return launch_status();
}

int launch_combine_bwd(const moe_cfg* c, const void* d_out, const void* y_perm, const float* w, const int32_t* idx,
                       const int32_t* row_of, const int32_t* offsets, const int32_t* kept, const int32_t* lo,
                       const int32_t* hi, void* dy_perm, float* dw, hipStream_t s) {
  const int grid = (c->T + CB_THREADS / WAVE - 1) / (CB_THREADS / WAVE);
  if (c->dtype == MOE_DTYPE_BF16)
    combine_bwd_kernel<bf16><<<grid, CB_THREADS, 0, s>>>((const bf16*)d_out, (const bf16*)y_perm, w, idx, row_of, offsets, kept, lo, hi, (bf16*)dy_perm, dw, c->T, c->d_model, c->k);
  else
    combine_bwd_kernel<float><<<grid, CB_THREADS, 0, s>>>((const float*)d_out, (const float*)y_perm, w, idx, row_of, offsets, kept, lo, hi, (float*)dy_perm, dw, c->T, c->d_model, c->k);
  return launch_status();
}

}  // namespace moe

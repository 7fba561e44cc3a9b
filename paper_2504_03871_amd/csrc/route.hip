// Gate forward and backward (Section 2.1 and the gate paragraph of Section 5 of the paper).
//
// Forward: logits = x Wr (+ bias) with fp32 accumulation, then a wavefront-reduction top-k on the
// stored fp32 logits and the softmax over the selected ones.
// Backward: softmax-over-selected backward, dWr = x^T dlogits, dx += dlogits Wr^T.
#include "common.h"

namespace moe {

constexpr int RT_TPW = 4;                 // tokens a wave accumulates at once
constexpr int RT_WAVES = 4;               // waves per block
constexpr int RT_TPB = RT_TPW * RT_WAVES; // tokens per block
constexpr int RT_EB = 8;                  // experts per accumulation pass

// One step of the transposing wave reduction: halves the number of live values per lane and
// doubles the number of lanes each value has been summed over.
template <int N>
__device__ __forceinline__ void fold(float (&v)[RT_TPW * RT_EB], int lane, int bit) {
  const bool upper = (lane & bit) != 0;
#pragma unroll
  for (int i = 0; i < N; ++i) {
    const float keep = upper ? v[N + i] : v[i];
    const float give = upper ? v[i] : v[N + i];
    v[i] = keep + __shfl_xor(give, bit, WAVE);
  }
}

template <typename T>
__global__ __launch_bounds__(RT_WAVES* WAVE) void route_kernel(
    const T* __restrict__ x, const float* __restrict__ Wr, const float* __restrict__ bias,
    const float* __restrict__ logits_in, float* __restrict__ logits_out,
    int32_t* __restrict__ topk_idx, float* __restrict__ topk_w, int Tn, int d, int E, int k) {
  __shared__ float s_logit[RT_TPB * MOE_MAX_E];
  const int lane = threadIdx.x & (WAVE - 1);
  const int wave = threadIdx.x / WAVE;
  const int tok0 = blockIdx.x * RT_TPB;

  if (logits_in != nullptr) {
    const int n = min(RT_TPB, Tn - tok0) * E;
    for (int i = threadIdx.x; i < n; i += blockDim.x) s_logit[i] = logits_in[(size_t)tok0 * E + i];
  } else {
    constexpr int VN = Vec16<T>::N;
    const int wt0 = tok0 + wave * RT_TPW;   // first token of this wave
    for (int e0 = 0; e0 < E; e0 += RT_EB) {
      float acc[RT_TPW * RT_EB];
#pragma unroll
      for (int i = 0; i < RT_TPW * RT_EB; ++i) acc[i] = 0.f;
      for (int c = lane * VN; c < d; c += WAVE * VN) {
        float xv[RT_TPW][VN];
#pragma unroll
        for (int t = 0; t < RT_TPW; ++t) {
          const int tok = min(wt0 + t, Tn - 1);   // clamp: rows past the end are computed, not stored
          Vec16<T> v;
          v.load(x + (size_t)tok * d + c);
          v.unpack(xv[t]);
        }
#pragma unroll
        for (int i = 0; i < VN; ++i) {
          float wv[RT_EB];
#pragma unroll
          for (int e = 0; e < RT_EB; ++e) wv[e] = (e0 + e < E) ? Wr[(size_t)(c + i) * E + e0 + e] : 0.f;
#pragma unroll
          for (int t = 0; t < RT_TPW; ++t)
#pragma unroll
            for (int e = 0; e < RT_EB; ++e) acc[t * RT_EB + e] = fmaf(xv[t][i], wv[e], acc[t * RT_EB + e]);
        }
      }
      // 32 values over 64 lanes: after the folds lane l holds value l>>1, summed over the wave
      fold<16>(acc, lane, 32);
      fold<8>(acc, lane, 16);
      fold<4>(acc, lane, 8);
      fold<2>(acc, lane, 4);
      fold<1>(acc, lane, 2);
      const float total = acc[0] + __shfl_xor(acc[0], 1, WAVE);
      const int vi = lane >> 1, t = vi / RT_EB, e = e0 + vi % RT_EB;
      if ((lane & 1) == 0 && e < E)
        s_logit[(wave * RT_TPW + t) * E + e] = total + (bias != nullptr ? bias[e] : 0.f);
    }
  }
  __syncthreads();
  if (logits_out != nullptr) {
    const int n = min(RT_TPB, Tn - tok0) * E;
    for (int i = threadIdx.x; i < n; i += blockDim.x) logits_out[(size_t)tok0 * E + i] = s_logit[i];
  }

  // top-k: lane owns experts lane, lane+64, ...; k rounds of a wave-wide lexicographic arg-max
  for (int t = 0; t < RT_TPW; ++t) {
    const int tl = wave * RT_TPW + t, tok = tok0 + tl;
    if (tok >= Tn) break;   // uniform per wave
    float v[MOE_MAX_E / WAVE];
#pragma unroll
    for (int s = 0; s < MOE_MAX_E / WAVE; ++s) {
      const int e = lane + s * WAVE;
      v[s] = e < E ? s_logit[tl * E + e] : 0.f;
    }
    unsigned taken = 0;
    float sel[MOE_MAX_K];
    int sid[MOE_MAX_K];
#pragma unroll
    for (int j = 0; j < MOE_MAX_K; ++j) {
      if (j < k) {
        float bv = -INFINITY;
        int bi = 0x7fffffff;
#pragma unroll
        for (int s = 0; s < MOE_MAX_E / WAVE; ++s) {
          const int e = lane + s * WAVE;
          if (e < E && !((taken >> s) & 1u) && (bi == 0x7fffffff || v[s] > bv)) { bv = v[s]; bi = e; }
        }
#pragma unroll
        for (int sft = 32; sft > 0; sft >>= 1) {
          const float ov = __shfl_xor(bv, sft, WAVE);
          const int oi = __shfl_xor(bi, sft, WAVE);
          // a real candidate beats "none"; larger value wins; equal values: lower id wins
          const bool better = (oi != 0x7fffffff) && (bi == 0x7fffffff || ov > bv || (ov == bv && oi < bi));
          if (better) { bv = ov; bi = oi; }
        }
        sel[j] = bv;
        sid[j] = bi;
        if ((bi & (WAVE - 1)) == lane) taken |= 1u << (bi / WAVE);
      }
    }
    float z[MOE_MAX_K], zs = 0.f;
#pragma unroll
    for (int j = 0; j < MOE_MAX_K; ++j)
      if (j < k) { z[j] = expf(sel[j] - sel[0]); zs += z[j]; }
#pragma unroll
    for (int j = 0; j < MOE_MAX_K; ++j)
      if (j < k && lane == j) {
        topk_idx[(size_t)tok * k + j] = sid[j];
        topk_w[(size_t)tok * k + j] = z[j] / zs;
      }
  }
}

// ---------------------------------------------------------------- backward
// Block = one token chunk x one column block.  Thread owns VEC adjacent columns i of x / dx / Wr.
// LDS: s_wr[e][col] = Wr[col][e] (for dx) and s_acc[e][col] (dWr partial of this token chunk).
template <typename T, int VEC>
__global__ void route_bwd_kernel(const T* __restrict__ x, const float* __restrict__ Wr,
                                 const int32_t* __restrict__ topk_idx, const float* __restrict__ topk_w,
                                 const float* __restrict__ d_topk_w, float* __restrict__ d_logits,
                                 float* __restrict__ partials, T* __restrict__ dx, int Tn, int d, int E, int k,
                                 int cols) {
  extern __shared__ float smem[];
  float* s_wr = smem;                       // [E][cols]
  float* s_acc = smem + (size_t)E * cols;   // [E][cols]
  float* s_ds = s_acc + (size_t)E * cols;   // [ROUTE_BWD_TOKENS][k] dsel
  int* s_e = reinterpret_cast<int*>(s_ds + ROUTE_BWD_TOKENS * MOE_MAX_K);  // [ROUTE_BWD_TOKENS][k]
  const int c0 = blockIdx.x * cols;
  const int t0 = blockIdx.y * ROUTE_BWD_TOKENS;
  const int nt = min(ROUTE_BWD_TOKENS, Tn - t0);
  const int ncol = min(cols, d - c0);

  for (int i = threadIdx.x; i < E * cols; i += blockDim.x) {
    const int e = i / cols, c = i % cols;
    s_wr[i] = (c < ncol) ? Wr[(size_t)(c0 + c) * E + e] : 0.f;
    s_acc[i] = 0.f;
  }
  for (int i = threadIdx.x; i < nt; i += blockDim.x) {
    const size_t a0 = (size_t)(t0 + i) * k;
    float g = 0.f;
    for (int j = 0; j < k; ++j) g += topk_w[a0 + j] * d_topk_w[a0 + j];
    for (int j = 0; j < k; ++j) {
      s_ds[i * MOE_MAX_K + j] = topk_w[a0 + j] * (d_topk_w[a0 + j] - g);
      s_e[i * MOE_MAX_K + j] = topk_idx[a0 + j];
    }
  }
  __syncthreads();
  if (blockIdx.x == 0 && d_logits != nullptr) {
    for (int i = threadIdx.x; i < nt * E; i += blockDim.x) {
      const int t = i / E, e = i % E;
      float v = 0.f;
      for (int j = 0; j < k; ++j) v = (s_e[t * MOE_MAX_K + j] == e) ? s_ds[t * MOE_MAX_K + j] : v;
      d_logits[(size_t)t0 * E + i] = v;
    }
  }
  const int c = threadIdx.x * VEC;
  if (c < ncol) {
    for (int t = 0; t < nt; ++t) {
      const size_t off = (size_t)(t0 + t) * d + c0 + c;
      float xv[VEC], gv[VEC];
#pragma unroll
      for (int v = 0; v < VEC; ++v) { xv[v] = to_f32(x[off + v]); gv[v] = 0.f; }
      for (int j = 0; j < k; ++j) {
        const int e = s_e[t * MOE_MAX_K + j];
        const float ds = s_ds[t * MOE_MAX_K + j];
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
          gv[v] = fmaf(ds, s_wr[e * cols + c + v], gv[v]);
          s_acc[e * cols + c + v] = fmaf(ds, xv[v], s_acc[e * cols + c + v]);
        }
      }
      if (dx != nullptr) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) dx[off + v] = from_f32<T>(to_f32(dx[off + v]) + gv[v]);
      }
    }
    // partials[chunk][col][e]
    for (int e = 0; e < E; ++e)
#pragma unroll
      for (int v = 0; v < VEC; ++v)
        partials[((size_t)blockIdx.y * d + c0 + c + v) * E + e] = s_acc[e * cols + c + v];
  }
}

__global__ void route_bwd_reduce_kernel(const float* __restrict__ partials, float* __restrict__ dWr, int n, int chunks) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float s = 0.f;
  for (int c = 0; c < chunks; ++c) s += partials[(size_t)c * n + i];   // fixed order: deterministic
  dWr[i] = s;
}

// ---------------------------------------------------------------- launchers
int launch_route(const moe_cfg* c, const void* x, const float* Wr, const float* bias, const float* logits_in,
                 float* logits_out, int32_t* idx, float* w, hipStream_t s) {
  const int grid = (c->T + RT_TPB - 1) / RT_TPB;
  if (c->dtype == MOE_DTYPE_BF16)
    route_kernel<bf16><<<grid, RT_WAVES * WAVE, 0, s>>>((const bf16*)x, Wr, bias, logits_in, logits_out, idx, w, c->T, c->d_model, c->E, c->k);
  else
    route_kernel<float><<<grid, RT_WAVES * WAVE, 0, s>>>((const float*)x, Wr, bias, logits_in, logits_out, idx, w, c->T, c->d_model, c->E, c->k);
  return launch_status();
}

int route_bwd_cols(int E) {
  // 2*E*cols fp32 of LDS, at most 128 KiB; a power of two between 64 and 512
  int cols = 512;
  while (cols > 64 && (size_t)2 * E * cols * 4 > 128 * 1024) cols >>= 1;
  return cols;
}

int launch_route_bwd(const moe_cfg* c, const void* x, const float* Wr, const int32_t* idx, const float* w,
                     const float* dw, float* d_logits, float* dWr, void* dx, float* partials, hipStream_t s) {
  const int cols = route_bwd_cols(c->E);
  const int chunks = (c->T + ROUTE_BWD_TOKENS - 1) / ROUTE_BWD_TOKENS;
  const dim3 grid((c->d_model + cols - 1) / cols, chunks);
  const size_t lds = (size_t)2 * c->E * cols * 4 + ROUTE_BWD_TOKENS * MOE_MAX_K * 8;
  constexpr int VEC = 2;
  const int threads = cols / VEC;
  if (c->dtype == MOE_DTYPE_BF16) {
    auto kern = route_bwd_kernel<bf16, VEC>;
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return set_hip_error(e);
    kern<<<grid, threads, lds, s>>>((const bf16*)x, Wr, idx, w, dw, d_logits, partials, (bf16*)dx, c->T, c->d_model, c->E, c->k, cols);
  } else {
    auto kern = route_bwd_kernel<float, VEC>;
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return set_hip_error(e);
    kern<<<grid, threads, lds, s>>>((const float*)x, Wr, idx, w, dw, d_logits, partials, (float*)dx, c->T, c->d_model, c->E, c->k, cols);
  }
  int rc = launch_status();
  if (rc != MOE_OK) return rc;
  const int n = c->d_model * c->E;
  route_bwd_reduce_kernel<<<(n + 255) / 256, 256, 0, s>>>(partials, dWr, n, chunks);
  return launch_status();
}

}  // namespace moe

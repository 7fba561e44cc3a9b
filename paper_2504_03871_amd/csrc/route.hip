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
// Three small kernels.
//  1. WrT[e][i] = Wr[i][e], so that the input-gradient kernel reads contiguous weights.
//  2. One wave per token: dsel_j = w_j (dw_j - sum_i w_i dw_i); writes the token's d_logits row and
//     adds sum_j dsel_j WrT[e_j][:] to dx[t][:].
//  3. dWr = x^T d_logits in its sparse form (k non-zeros per token): a block owns a tile of columns
//     and a chunk of tokens, every wave keeps a private [E][columns] accumulator in LDS for a quarter
//     of the chunk, the waves are summed in a fixed order and the per-chunk partials are reduced by a
//     last kernel in chunk order, so the result is bit-reproducible.
__global__ void wr_transpose_kernel(const float* __restrict__ Wr, float* __restrict__ WrT, int d, int E) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < d * E) WrT[(size_t)(i % E) * d + i / E] = Wr[i];
}

template <typename T>
__global__ __launch_bounds__(256) void route_bwd_dx_kernel(
    const float* __restrict__ WrT, const int32_t* __restrict__ topk_idx, const float* __restrict__ topk_w,
    const float* __restrict__ d_topk_w, float* __restrict__ d_logits, T* __restrict__ dx, int Tn, int d, int E, int k) {
  constexpr int VN = Vec16<T>::N;
  const int lane = threadIdx.x & (WAVE - 1);
  const int t = (blockIdx.x * blockDim.x + threadIdx.x) / WAVE;
  if (t >= Tn) return;
  float ds[MOE_MAX_K];
  int ej[MOE_MAX_K];
  float gsum = 0.f;
#pragma unroll
  for (int j = 0; j < MOE_MAX_K; ++j)
    if (j < k) gsum = fmaf(topk_w[(size_t)t * k + j], d_topk_w[(size_t)t * k + j], gsum);
#pragma unroll
  for (int j = 0; j < MOE_MAX_K; ++j) {
    ds[j] = 0.f;
    ej[j] = 0;
    if (j < k) {
      ds[j] = topk_w[(size_t)t * k + j] * (d_topk_w[(size_t)t * k + j] - gsum);
      ej[j] = topk_idx[(size_t)t * k + j];
    }
  }
  for (int e = lane; e < E; e += WAVE) {
    float v = 0.f;
#pragma unroll
    for (int j = 0; j < MOE_MAX_K; ++j) v = (j < k && ej[j] == e) ? ds[j] : v;
    d_logits[(size_t)t * E + e] = v;
  }
  if (dx == nullptr) return;
  for (int c = lane * VN; c < d; c += WAVE * VN) {
    Vec16<T> v;
    v.load(dx + (size_t)t * d + c);
    float acc[VN];
    v.unpack(acc);
#pragma unroll
    for (int j = 0; j < MOE_MAX_K; ++j)
      if (j < k) {
        const float* wr = WrT + (size_t)ej[j] * d + c;
#pragma unroll
        for (int i = 0; i < VN; i += 4) {
          const float4 w4 = *reinterpret_cast<const float4*>(wr + i);
          acc[i] = fmaf(ds[j], w4.x, acc[i]);
          acc[i + 1] = fmaf(ds[j], w4.y, acc[i + 1]);
          acc[i + 2] = fmaf(ds[j], w4.z, acc[i + 2]);
          acc[i + 3] = fmaf(ds[j], w4.w, acc[i + 3]);
        }
      }
    v.pack(acc);
    v.store(dx + (size_t)t * d + c);
  }
}

constexpr int RB_MAX_WAVES = 4;  // waves per block of the dWr kernel (fewer when E is large: LDS)
constexpr int RB_BATCH = 8;      // tokens whose x values a thread keeps in flight

// Block = nw waves; thread owns VEC adjacent columns; wave w handles tokens w, w+nw, ... of the chunk.
template <typename T, int VEC>
__global__ __launch_bounds__(RB_MAX_WAVES* WAVE) void route_bwd_dwr_kernel(
    const T* __restrict__ x, const int32_t* __restrict__ topk_idx, const float* __restrict__ d_logits,
    float* __restrict__ partials, int Tn, int d, int E, int k) {
  extern __shared__ float smem[];
  constexpr int COLS = WAVE * VEC;
  const int lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x / WAVE, nw = blockDim.x / WAVE;
  float* acc = smem + (size_t)wave * E * COLS;   // [E][COLS], private to the wave
  const int c0 = blockIdx.x * COLS + lane * VEC;
  const int t0 = blockIdx.y * ROUTE_BWD_TOKENS;
  const int nt = min(ROUTE_BWD_TOKENS, Tn - t0);
  for (int i = lane; i < E * COLS; i += WAVE) acc[i] = 0.f;
  const bool live = c0 < d;   // d is a multiple of VEC
  for (int tb = wave; tb < nt; tb += nw * RB_BATCH) {
    float xv[RB_BATCH][VEC];
#pragma unroll
    for (int u = 0; u < RB_BATCH; ++u) {
      const int t = tb + u * nw;
#pragma unroll
      for (int v = 0; v < VEC; ++v) xv[u][v] = (live && t < nt) ? to_f32(x[(size_t)(t0 + t) * d + c0 + v]) : 0.f;
    }
#pragma unroll
    for (int u = 0; u < RB_BATCH; ++u) {
      const int t = tb + u * nw;
      if (t < nt) {
        for (int j = 0; j < k; ++j) {
          const int e = topk_idx[(size_t)(t0 + t) * k + j];        // wave-uniform
          const float ds = d_logits[(size_t)(t0 + t) * E + e];
#pragma unroll
          for (int v = 0; v < VEC; ++v) acc[e * COLS + lane * VEC + v] = fmaf(ds, xv[u][v], acc[e * COLS + lane * VEC + v]);
        }
      }
    }
  }
  __syncthreads();
  // sum the waves in wave order and write partials[chunk][col][e]
  for (int i = threadIdx.x; i < E * COLS; i += blockDim.x) {
    const int e = i / COLS, c = i % COLS;
    float s = 0.f;
    for (int w = 0; w < nw; ++w) s += smem[(size_t)w * E * COLS + i];
    const int col = blockIdx.x * COLS + c;
    if (col < d) partials[((size_t)blockIdx.y * d + col) * E + e] = s;
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

template <typename T, int VEC>
static int launch_dwr(const moe_cfg* c, const void* x, const int32_t* idx, const float* d_logits, float* partials,
                      int chunks, hipStream_t s) {
  int nw = RB_MAX_WAVES;
  while (nw > 1 && (size_t)nw * c->E * WAVE * VEC * 4 > 128 * 1024) nw >>= 1;
  const size_t lds = (size_t)nw * c->E * WAVE * VEC * 4;
  auto kern = route_bwd_dwr_kernel<T, VEC>;
  hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return set_hip_error(e);
  const dim3 grid((c->d_model + WAVE * VEC - 1) / (WAVE * VEC), chunks);
  kern<<<grid, nw * WAVE, lds, s>>>((const T*)x, idx, d_logits, partials, c->T, c->d_model, c->E, c->k);
  return launch_status();
}

int launch_route_bwd(const moe_cfg* c, const void* x, const float* Wr, const int32_t* idx, const float* w,
                     const float* dw, float* d_logits, float* dWr, void* dx, float* partials, float* WrT,
                     hipStream_t s) {
  const int n = c->d_model * c->E;
  const int chunks = (c->T + ROUTE_BWD_TOKENS - 1) / ROUTE_BWD_TOKENS;
  const bool bf = c->dtype == MOE_DTYPE_BF16;
  int rc;
  if (dx != nullptr) {
    wr_transpose_kernel<<<(n + 255) / 256, 256, 0, s>>>(Wr, WrT, c->d_model, c->E);
    if ((rc = launch_status()) != MOE_OK) return rc;
  }
  const int grid = (c->T + 3) / 4;
  if (bf) route_bwd_dx_kernel<bf16><<<grid, 256, 0, s>>>(WrT, idx, w, dw, d_logits, (bf16*)dx, c->T, c->d_model, c->E, c->k);
  else route_bwd_dx_kernel<float><<<grid, 256, 0, s>>>(WrT, idx, w, dw, d_logits, (float*)dx, c->T, c->d_model, c->E, c->k);
  if ((rc = launch_status()) != MOE_OK) return rc;
  // columns per thread: as many as 128 KiB of LDS allow for 4 waves x E experts (d is a multiple of 4)
  const int vec = (c->E <= 32) ? 4 : (c->E <= 64 ? 2 : 1);
  if (vec == 4) rc = bf ? launch_dwr<bf16, 4>(c, x, idx, d_logits, partials, chunks, s) : launch_dwr<float, 4>(c, x, idx, d_logits, partials, chunks, s);
  else if (vec == 2) rc = bf ? launch_dwr<bf16, 2>(c, x, idx, d_logits, partials, chunks, s) : launch_dwr<float, 2>(c, x, idx, d_logits, partials, chunks, s);
  else rc = bf ? launch_dwr<bf16, 1>(c, x, idx, d_logits, partials, chunks, s) : launch_dwr<float, 1>(c, x, idx, d_logits, partials, chunks, s);
  if (rc != MOE_OK) return rc;
  route_bwd_reduce_kernel<<<(n + 255) / 256, 256, 0, s>>>(partials, dWr, n, chunks);
  return launch_status();
}

}  // namespace moe

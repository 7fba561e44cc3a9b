// Gate forward and backward (Section 2.1 and the gate paragraph of Section 5 of the paper).
//
// Forward: logits = x Wr (+ bias) with fp32 accumulation, then a wavefront-reduction top-k on the
// stored fp32 logits and the softmax over the selected ones.
// Backward: softmax-over-selected backward, dWr = x^T dlogits, dx += dlogits Wr^T.
#include "common.h"
#include <type_traits>

namespace moe {

// Forward kernel for fp32 inputs and for routing from given logits.  A block of 256 threads owns TOK tokens.  Thread (token, k part, expert group) keeps
// the dot products of its token with four experts over its share of every d chunk, so x Wr needs no
// cross-lane reduction beyond adding the k parts (adjacent lanes) at the end.  x chunks [TOK][DC] and
// Wr chunks [DC][E4] are staged through LDS (coalesced global loads, prefetched into registers one
// chunk ahead); the four weights of a step come from one 16-byte LDS read shared by all tokens.
// Top-k: the G = KS*EGP lanes of a token scan the logits in LDS (expert g, g+G, ...) and run k rounds
// of a lexicographic arg-max (larger value first, then lower expert id) with xor shuffles.
constexpr int RT_THREADS = 256;
constexpr int RT_XPAD = 8;   // elements of padding per staged x row (keeps 16-byte alignment, spreads banks)

struct RouteGeom {
  int egp_log2;   // lanes per (token, k part): pow2 >= ceil(E/4)
  int ks_log2;    // k parts per token
  int tok;        // tokens per block = 256 / (KS * EGP)
  int dc;         // d elements per chunk
  int e4;         // padded expert count = 4 * EGP
};
static RouteGeom route_geom(int E) {
  RouteGeom g;
  const int eg = (E + 3) / 4;
  g.egp_log2 = 0;
  while ((1 << g.egp_log2) < eg) ++g.egp_log2;
  g.ks_log2 = 0;
  while ((1 << (g.ks_log2 + g.egp_log2)) < 8) ++g.ks_log2;
  g.tok = RT_THREADS >> (g.ks_log2 + g.egp_log2);
  g.e4 = 4 << g.egp_log2;
  g.dc = 64;
  while (g.dc * g.e4 > 2048) g.dc >>= 1;
  // few experts: longer chunks (fewer block barriers per token) while the Wr chunk stays within 8 KB
  // and the x chunk within four 16-byte vectors per thread even for fp32 (TOK * DC * 4 / 16 <= 1024)
  while (g.dc < 128 && g.dc * 2 * g.e4 <= 2048 && g.tok * g.dc * 2 <= 4096) g.dc <<= 1;
  return g;
}

// Top-k and weights of token `tok` from its E logits in LDS (row tl of s_logit), run by the G lanes g =
// 0..G-1 of the token (G <= 64 and a power of two: the lanes sit in one wave).  Lane g scans the experts
// g, g+G, ...; k rounds of a lexicographic arg-max (larger value first, then lower expert id) with xor
// shuffles; weights = softmax over the selected logits.  Every lane of the wave must call this.
// `ld` = row pitch of s_logit in floats.
__device__ __forceinline__ void route_select(const float* s_logit, int ld, int tl, int g, int G, bool live, int tok, int E,
                                             int k, int32_t* __restrict__ topk_idx, float* __restrict__ topk_w) {
  unsigned taken = 0;
  float sel[MOE_MAX_K];
  int sid[MOE_MAX_K];
#pragma unroll
  for (int j = 0; j < MOE_MAX_K; ++j) {
    if (j < k) {
      float bv = -INFINITY;
      int bi = 0x7fffffff;
      if (live) {
        int slot = 0;
        for (int e = g; e < E; e += G, ++slot) {
          const float v = s_logit[tl * ld + e];
          if (!((taken >> slot) & 1u) && (bi == 0x7fffffff || v > bv)) { bv = v; bi = e; }
        }
      }
      for (int sft = G >> 1; sft > 0; sft >>= 1) {
        const float ov = __shfl_xor(bv, sft, WAVE);
        const int oi = __shfl_xor(bi, sft, WAVE);
        // a real candidate beats "none"; larger value wins; equal values: lower id wins
        const bool better = (oi != 0x7fffffff) && (bi == 0x7fffffff || ov > bv || (ov == bv && oi < bi));
        if (better) { bv = ov; bi = oi; }
      }
      sel[j] = bv;
      sid[j] = bi;
      if (bi != 0x7fffffff && (bi & (G - 1)) == g) taken |= 1u << (bi / G);
    }
  }
  if (live) {
    float z[MOE_MAX_K], zs = 0.f;
#pragma unroll
    for (int j = 0; j < MOE_MAX_K; ++j)
      if (j < k) { z[j] = expf(sel[j] - sel[0]); zs += z[j]; }
#pragma unroll
    for (int j = 0; j < MOE_MAX_K; ++j)
      if (j < k && g == (j & (G - 1))) {
        topk_idx[(size_t)tok * k + j] = sid[j];
        topk_w[(size_t)tok * k + j] = z[j] / zs;
      }
  }
}

template <typename T>
__global__ __launch_bounds__(RT_THREADS) void route_kernel(
    const T* __restrict__ x, const float* __restrict__ Wr, const float* __restrict__ bias,
    const float* __restrict__ logits_in, float* __restrict__ logits_out,
    int32_t* __restrict__ topk_idx, float* __restrict__ topk_w, int Tn, int d, int E, int k, RouteGeom gm) {
  constexpr int VN = Vec16<T>::N;
  extern __shared__ __attribute__((aligned(16))) char rsm[];
  const int EGP = 1 << gm.egp_log2, KS = 1 << gm.ks_log2, G = EGP * KS, TOK = gm.tok, DC = gm.dc, E4 = gm.e4;
  const int xpitch = DC + RT_XPAD;
  T* xs = reinterpret_cast<T*>(rsm);                                                   // [TOK][xpitch]
  float* wsm = reinterpret_cast<float*>(rsm + (size_t)TOK * xpitch * sizeof(T));       // [DC][E4]
  float* s_logit = wsm + (size_t)DC * E4;                                              // [TOK][E]
  const int tid = threadIdx.x;
  const int eg = tid & (EGP - 1), ks = (tid >> gm.egp_log2) & (KS - 1), tl = tid >> (gm.egp_log2 + gm.ks_log2);
  const int tok0 = blockIdx.x * TOK;
  const int ntok = min(TOK, Tn - tok0);

  if (logits_in != nullptr) {
    for (int i = tid; i < ntok * E; i += RT_THREADS) s_logit[i] = logits_in[(size_t)tok0 * E + i];
  } else {
    const int xv_per_row = DC / VN, n_xv = TOK * xv_per_row;   // 16-byte vectors of one x chunk
    const int n_wv = DC * E4 / 4;                              // float4 of one Wr chunk
    Vec16<T> xr[4];
    float4 wr[2];
    auto fetch = [&](int c0) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int q = tid + u * RT_THREADS;
        if (q < n_xv) {
          const int r = q / xv_per_row, c = c0 + (q % xv_per_row) * VN;
          if (r < ntok && c < d) xr[u].load(x + (size_t)(tok0 + r) * d + c);
          else { float z[VN] = {}; xr[u].pack(z); }
        }
      }
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int q = tid + u * RT_THREADS;
        if (q < n_wv) {
          const int i = c0 + (q * 4) / E4, e = (q * 4) % E4;
          float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
          if (i < d) {
            const float* src = Wr + (size_t)i * E + e;
            if ((E & 3) == 0) { if (e < E) v = *reinterpret_cast<const float4*>(src); }
            else {
              if (e < E) v.x = src[0];
              if (e + 1 < E) v.y = src[1];
              if (e + 2 < E) v.z = src[2];
              if (e + 3 < E) v.w = src[3];
            }
          }
          wr[u] = v;
        }
      }
    };
    auto stash = [&]() {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int q = tid + u * RT_THREADS;
        if (q < n_xv) xr[u].store(xs + (size_t)(q / xv_per_row) * xpitch + (q % xv_per_row) * VN);
      }
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int q = tid + u * RT_THREADS;
        if (q < n_wv) *reinterpret_cast<float4*>(wsm + (size_t)q * 4) = wr[u];
      }
    };
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    const int part = DC / KS;   // elements of a chunk this thread multiplies
    fetch(0);
    for (int c0 = 0; c0 < d; c0 += DC) {
      __syncthreads();   // the previous chunk has been consumed
      stash();
      __syncthreads();
      if (c0 + DC < d) fetch(c0 + DC);
      const T* xrow = xs + (size_t)tl * xpitch + ks * part;
      const float* wcol = wsm + (size_t)(ks * part) * E4 + eg * 4;
      for (int ii = 0; ii < part; ii += VN) {
        Vec16<T> xv;
        xv.load(xrow + ii);
        float xf[VN];
        xv.unpack(xf);
#pragma unroll
        for (int u = 0; u < VN; ++u) {
          const float4 w4 = *reinterpret_cast<const float4*>(wcol + (size_t)(ii + u) * E4);
          acc[0] = fmaf(xf[u], w4.x, acc[0]);
          acc[1] = fmaf(xf[u], w4.y, acc[1]);
          acc[2] = fmaf(xf[u], w4.z, acc[2]);
          acc[3] = fmaf(xf[u], w4.w, acc[3]);
        }
      }
    }
    // add the k parts (lanes EGP apart), fixed order
    for (int s = EGP; s < G; s <<= 1) {
#pragma unroll
      for (int q = 0; q < 4; ++q) acc[q] += __shfl_xor(acc[q], s, WAVE);
    }
    if (ks == 0 && tl < ntok) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int e = eg * 4 + q;
        if (e < E) s_logit[tl * E + e] = acc[q] + (bias != nullptr ? bias[e] : 0.f);
      }
    }
  }
  __syncthreads();
  if (logits_out != nullptr)
    for (int i = tid; i < ntok * E; i += RT_THREADS) logits_out[(size_t)tok0 * E + i] = s_logit[i];

  route_select(s_logit, E, tl, tid & (G - 1), G, tl < ntok, tok0 + tl, E, k, topk_idx, topk_w);
}

// ---------------------------------------------------------------- forward on the matrix cores (bf16 or fp16 x)
// logits = x Wr as a [T x d] x [d x E] product on v_mfma_f32_16x16x32_bf16.  x is bf16 already (fp16: the exact
// sum of two bf16 terms, XTerms below); the fp32
// gate weight is split into two bf16 terms, w = hi + lo with hi = bf16(w), lo = bf16(w - hi), and both
// products are accumulated in fp32, which keeps the weight to about 16 mantissa bits (relative error
// 2^-17 per product, far below the bf16 resolution of x itself).
//
// A block of NW waves owns TT tiles of 16 tokens (64 tokens with eight waves, 32 with four); the waves split K in
// blocks of 128 (wave w: blocks w, w+NW, ...), each multiplies its share for all experts (NET tiles of 16) with
// the 16 x 16 x 32 MFMA, and the partial tiles are added in wave order through LDS (deterministic).  Operands
// come straight from memory, no LDS staging:
//  * A: lane (row r = l%16 of a token tile, quarter c = l/16) reads the 64 contiguous bytes
//    x[t0+r][kb*128 + c*32 .. +31], so the four lanes of a row cover two whole 128-byte lines, and uses 8 of
//    those 32 elements in each of four MFMA steps;
//  * B: wr_frag_kernel writes the two bf16 terms once per call in exactly the register layout of those
//    steps: unit ((((nt*nkb + kb)*4 + s)*2 + term)*64 + lane) holds, for lane (expert e = l%16 of tile nt,
//    quarter c), the eight values Wr[kb*128 + c*32 + s*8 + i][nt*16 + e], i = 0..7 (zero past d or E); a wave
//    reads a unit as one contiguous kilobyte, once for all its token tiles.
// The K order inside a step differs from memory order, which a dot product does not mind as long as
// both operands agree.  MFMA register layout: see gemm_bf16_kernel.h.  (An earlier version on 32 x 32 x 16
// tiles with 32 tokens per block read twice as many weight bytes from L2 as x bytes from memory.)
typedef bf16 rt_bf16x8 __attribute__((ext_vector_type(8)));
typedef float rt_f32x4 __attribute__((ext_vector_type(4)));

__global__ void wr_frag_kernel(const float* __restrict__ Wr, rt_bf16x8* __restrict__ wfrag, int d, int E, int nkb, int net) {
  const int u = blockIdx.x * blockDim.x + threadIdx.x;
  if (u >= net * nkb * 4 * 2 * 64) return;
  const int lane = u & 63, term = (u >> 6) & 1, s = (u >> 7) & 3, kb = (u >> 9) % nkb, nt = (u >> 9) / nkb;
  const int e = nt * 16 + (lane & 15), k0 = kb * 128 + (lane >> 4) * 32 + s * 8;
  rt_bf16x8 v;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float w = (e < E && k0 + i < d) ? Wr[(size_t)(k0 + i) * E + e] : 0.f;
    const bf16 hi = (bf16)w;
    v[i] = term == 0 ? hi : (bf16)(w - (float)hi);
  }
  wfrag[u] = v;
}

// Sixteen bytes of x as bf16 MFMA operands.  bf16 storage: as they are.  fp16 storage: every value (11
// significant bits) is the exact sum of two bf16 numbers, its first 8 significant bits and the rest (at most 3
// bits; bf16's exponent range covers fp16's subnormals), so the product with the two-term weight takes four
// MFMAs instead of two and no fp16 range question (subnormal low-order terms) comes up.
template <typename T> struct XTerms;
template <> struct XTerms<bf16> {
  static constexpr int N = 1;
  static __device__ __forceinline__ void split(const uint4& raw, rt_bf16x8* out) { out[0] = __builtin_bit_cast(rt_bf16x8, raw); }
};
template <> struct XTerms<f16> {
  static constexpr int N = 2;
  static __device__ __forceinline__ void split(const uint4& raw, rt_bf16x8* out) {
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
    uint4 h, l;
    uint32_t* hp = &h.x;
    uint32_t* lp = &l.x;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float f0 = f16_bits_to_f32(w[i] & 0xffffu), f1 = f16_bits_to_f32(w[i] >> 16);
      const uint32_t h0 = __float_as_uint(f0) & 0xffff0000u, h1 = __float_as_uint(f1) & 0xffff0000u;
      // exact; an infinity (or NaN) stays in the first term alone instead of making inf - inf
      const float r0 = (h0 & 0x7f800000u) == 0x7f800000u ? 0.f : f0 - __uint_as_float(h0);
      const float r1 = (h1 & 0x7f800000u) == 0x7f800000u ? 0.f : f1 - __uint_as_float(h1);
      hp[i] = (h0 >> 16) | h1;
      lp[i] = (__float_as_uint(r0) >> 16) | (__float_as_uint(r1) & 0xffff0000u);
    }
    out[0] = __builtin_bit_cast(rt_bf16x8, h);
    out[1] = __builtin_bit_cast(rt_bf16x8, l);
  }
};

template <typename T, int NET, int TT, int NW>
__global__ __launch_bounds__(NW * 64) void route_mfma_kernel(
    const T* __restrict__ x, const rt_bf16x8* __restrict__ wfrag, const float* __restrict__ bias,
    float* __restrict__ logits_out, int32_t* __restrict__ topk_idx, float* __restrict__ topk_w, int Tn, int d, int E, int k) {
  extern __shared__ float part[];   // [NW waves][TOK tokens][LD]; the sum ends up in part[0]
  constexpr int TOK = TT * 16, LD = NET * 16;
  static_assert(TOK == NW * 8, "the selection runs eight lanes per token over the whole block");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int tok0 = blockIdx.x * TOK, nkb = (d + 127) / 128;
  const int r = lane & 15, c = lane >> 4;
  constexpr int XT = XTerms<T>::N;
  const T* xrow[TT];
#pragma unroll
  for (int tt = 0; tt < TT; ++tt) xrow[tt] = x + (size_t)min(tok0 + tt * 16 + r, Tn - 1) * d + c * 32;   // rows past the batch repeat the last token
  rt_f32x4 acc[TT][NET];
#pragma unroll
  for (int tt = 0; tt < TT; ++tt)
#pragma unroll
    for (int nt = 0; nt < NET; ++nt) acc[tt][nt] = rt_f32x4{0.f, 0.f, 0.f, 0.f};
  auto load_a = [&](uint4 (*dst)[4], int kb) {   // raw 16-byte pieces; split into operands once they have arrived
    const bool inb = kb * 128 + c * 32 < d;   // d is a multiple of 64: a lane's 32 elements lie inside the row or past it
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
      for (int s = 0; s < 4; ++s)
        dst[tt][s] = inb ? *reinterpret_cast<const uint4*>(xrow[tt] + (size_t)kb * 128 + s * 8) : uint4{0u, 0u, 0u, 0u};
  };
  auto split_a = [&](rt_bf16x8 (*dst)[4][XT], uint4 (*raw)[4]) {
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
      for (int s = 0; s < 4; ++s) XTerms<T>::split(raw[tt][s], dst[tt][s]);
  };
  auto load_b = [&](rt_bf16x8* dst, int kb, int nt) {
    const rt_bf16x8* wf = wfrag + ((size_t)(nt * nkb + kb) * 8) * 64 + lane;
#pragma unroll
    for (int q = 0; q < 8; ++q) dst[q] = wf[q * 64];
  };
  auto mfmas = [&](rt_bf16x8 (*a)[4][XT], const rt_bf16x8* b, int nt) {
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
      for (int xt = 0; xt < XT; ++xt)
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
          acc[tt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[tt][s][xt], b[s * 2], acc[tt][nt], 0, 0, 0);
          acc[tt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[tt][s][xt], b[s * 2 + 1], acc[tt][nt], 0, 0, 0);
        }
  };
  if constexpr (NET >= 4) {
    // Many expert tiles: a block streams the whole gate weight (1-2 MB) through its four waves, and a wave
    // that waits for each 8 KB unit before asking for the next one spends its time in L2 round trips.  The
    // units run through a ring of PF register buffers, PF - 1 of them in flight ahead of the one the
    // MFMAs use, across the K blocks; the token rows of the next K block are loaded one block ahead.
    constexpr int PF = 4;
    static_assert(NET % PF == 0, "unit nt of any K block sits in buffer nt % PF");
    uint4 raw[TT][4];
    rt_bf16x8 a[TT][4][XT], b[PF][8];
    const int n_it = wave < nkb ? (nkb - wave + NW - 1) / NW : 0;   // K blocks wave, wave + NW, ... of this wave
    auto kb_of = [&](int it) { return wave + NW * it; };
    if (n_it > 0) {
      load_a(raw, kb_of(0));
#pragma unroll
      for (int p = 0; p < PF - 1; ++p) load_b(b[p], kb_of(0), p);
      split_a(a, raw);
    }
    for (int it = 0; it < n_it; ++it) {
      const int kb = kb_of(it);
      const bool more = it + 1 < n_it;
      const int kbn = more ? kb_of(it + 1) : kb;
      if (more) load_a(raw, kbn);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int nt = 0; nt < NET; ++nt) {
        constexpr int AHEAD = PF - 1;
        if (nt + AHEAD < NET) load_b(b[(nt + AHEAD) % PF], kb, nt + AHEAD);
        else if (more) load_b(b[(nt + AHEAD) % PF], kbn, nt + AHEAD - NET);
        __builtin_amdgcn_sched_barrier(0);   // the loads stay here, ahead of the MFMAs: left alone, the scheduler sinks each to its use
        mfmas(a, b[nt % PF], nt);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (more) split_a(a, raw);
    }
  } else {
    // one or two expert tiles: a 16-byte piece of x is split into its operands right before its MFMAs (fp16:
    // keeps the registers of the second term out of the loop's budget; with two tiles it is split twice)
    for (int kb = wave; kb < nkb; kb += NW) {
      uint4 raw[TT][4];
      load_a(raw, kb);
#pragma unroll
      for (int nt = 0; nt < NET; ++nt) {
        rt_bf16x8 b[8];
        load_b(b, kb, nt);
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
          for (int tt = 0; tt < TT; ++tt) {
            rt_bf16x8 t[XT];
            XTerms<T>::split(raw[tt][s], t);
#pragma unroll
            for (int xt = 0; xt < XT; ++xt) {
              acc[tt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(t[xt], b[s * 2], acc[tt][nt], 0, 0, 0);
              acc[tt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(t[xt], b[s * 2 + 1], acc[tt][nt], 0, 0, 0);
            }
          }
      }
    }
  }
  // partial tiles to LDS: accumulator register v of lane l is token (l/16)*4 + v, expert l%16 of its tile
  float* mine = part + (size_t)wave * TOK * LD;
#pragma unroll
  for (int tt = 0; tt < TT; ++tt)
#pragma unroll
    for (int nt = 0; nt < NET; ++nt)
#pragma unroll
      for (int v = 0; v < 4; ++v) mine[(tt * 16 + c * 4 + v) * LD + nt * 16 + r] = acc[tt][nt][v];
  __syncthreads();
  for (int i = tid; i < TOK * LD; i += NW * 64) {
    const int e = i % LD;
    float sum = part[i];
#pragma unroll
    for (int w = 1; w < NW; ++w) sum += part[w * TOK * LD + i];   // wave order: deterministic
    part[i] = sum + ((bias != nullptr && e < E) ? bias[e] : 0.f);
  }
  __syncthreads();
  const int ntok = min(TOK, Tn - tok0);
  for (int i = tid; i < ntok * E; i += NW * 64) logits_out[(size_t)tok0 * E + i] = part[(i / E) * LD + i % E];
  const int tl = tid >> 3;   // eight lanes per token
  route_select(part, LD, tl, tid & 7, 8, tl < ntok, tok0 + tl, E, k, topk_idx, topk_w);
}

// ---------------------------------------------------------------- backward
// Four small kernels.
//  1. WrT[e][i] = Wr[i][e], so that the input-gradient kernel reads contiguous weights.
//  2. One wave per token: dsel_j = w_j (dw_j - sum_i w_i dw_i); writes the token's d_logits row and
//     adds sum_j dsel_j WrT[e_j][:] to dx[t][:].
//  3. dWr = x^T d_logits, dense: token slices accumulate [16 experts] x [columns] blocks in registers, one row
//     of partial sums per slice, and a last kernel adds the rows in a fixed order, so the result is
//     bit-reproducible.
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
      if (ej[j] < 0 || ej[j] >= E) { ej[j] = -1; ds[j] = 0.f; }   // an id outside [0, E) contributes nothing
    }
  }
  for (int e = lane; e < E; e += WAVE) {
    float v = 0.f;
#pragma unroll
    for (int j = 0; j < MOE_MAX_K; ++j) v = (j < k && ej[j] == e) ? ds[j] : v;
    d_logits[(size_t)t * E + e] = v;
  }
  if (dx == nullptr) return;
  constexpr int U = 4;   // 16-byte pieces of the dx row per lane in flight (dx is touched once here: streaming access)
  for (int c0 = lane * VN; c0 < d; c0 += WAVE * VN * U) {
    Vec16<T> v[U];
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (c0 + u * WAVE * VN < d) v[u].load_nt(dx + (size_t)t * d + c0 + u * WAVE * VN);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int c = c0 + u * WAVE * VN;
      if (c >= d) break;
      float acc[VN];
      v[u].unpack(acc);
#pragma unroll
      for (int j = 0; j < MOE_MAX_K; ++j)
        if (j < k) {
          const float* wr = WrT + (size_t)max(ej[j], 0) * d + c;
#pragma unroll
          for (int i = 0; i < VN; i += 4) {
            const float4 w4 = *reinterpret_cast<const float4*>(wr + i);
            acc[i] = fmaf(ds[j], w4.x, acc[i]);
            acc[i + 1] = fmaf(ds[j], w4.y, acc[i + 1]);
            acc[i + 2] = fmaf(ds[j], w4.z, acc[i + 2]);
            acc[i + 3] = fmaf(ds[j], w4.w, acc[i + 3]);
          }
        }
      v[u].pack(acc);
      v[u].store_nt(dx + (size_t)t * d + c);
    }
  }
}

// Gate weight gradient dWr = x^T d_logits.  Experts in groups of EB <= 16 along gridDim.z: every thread keeps an [EB] x
// (16-byte column group) block of the weight gradient in registers and adds d_logits[t][:] (x) x[t][cols] token after token,
// zeros of the unselected experts included; no LDS read-modify-write, no branches, one 16-byte load of
// x per token.  The slice's d_logits rows are staged in LDS once, padded with zeros to EB per row, and
// read back as 16-byte broadcasts.  Geometry: RouteBwdGeom.
template <typename T, int EB>
__global__ __launch_bounds__(256) void route_bwd_dwr_dense_kernel(
    const T* __restrict__ x, const float* __restrict__ d_logits, float* __restrict__ partials, int Tn, int d, int E,
    RouteBwdGeom gm) {
  extern __shared__ float4 s_dl4[];   // [slices_per_block][tps][EB] floats
  float* s_dl = reinterpret_cast<float*>(s_dl4);
  constexpr int VN = Vec16<T>::N, U = 8;   // tokens whose x pieces a thread keeps in flight
  const int c = threadIdx.x & (gm.cg_pow2 - 1), slice = threadIdx.x / gm.cg_pow2;
  const int col = (blockIdx.x * gm.cg_pow2 + c) * VN;
  const int row = blockIdx.y * gm.slices_per_block + slice;   // row of partial sums = token slice
  const int e0 = blockIdx.z * EB;                               // this block's group of experts (more than EB experts: x is read once per group)
  const int t0 = row * gm.tps;
  const int nt = max(0, min(gm.tps, Tn - t0));
  {   // the block's slices are adjacent tokens: one pass over them, zero past the last token and past E
    const int tb = blockIdx.y * gm.slices_per_block * gm.tps, n = gm.slices_per_block * gm.tps * EB;
    for (int i = threadIdx.x; i < n; i += 256) {
      const int t = tb + i / EB, e = i % EB;
      s_dl[i] = (t < Tn && e0 + e < E) ? d_logits[(size_t)t * E + e0 + e] : 0.f;
    }
  }
  __syncthreads();
  if (col >= d) return;
  const float4* dl = s_dl4 + (size_t)slice * gm.tps * (EB / 4);
  float acc[EB][VN];
#pragma unroll
  for (int e = 0; e < EB; ++e)
#pragma unroll
    for (int v = 0; v < VN; ++v) acc[e][v] = 0.f;
  for (int tb = 0; tb < nt; tb += U) {
    Vec16<T> xv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) xv[u].load_nt(x + (size_t)(t0 + min(tb + u, nt - 1)) * d + col);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float xf[VN];
      xv[u].unpack(xf);
      const float live = (tb + u < nt) ? 1.f : 0.f;   // the clamped reload of the last token counts once
#pragma unroll
      for (int q = 0; q < EB / 4; ++q) {
        const float4 g4 = dl[min(tb + u, nt - 1) * (EB / 4) + q];
        const float g[4] = {g4.x * live, g4.y * live, g4.z * live, g4.w * live};
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int v = 0; v < VN; ++v) acc[q * 4 + j][v] = fmaf(g[j], xf[v], acc[q * 4 + j][v]);
      }
    }
  }
  float* out = partials + (size_t)row * E * d + col;   // [row][e][col]: 16-byte stores, adjacent lanes adjacent
#pragma unroll
  for (int e = 0; e < EB; ++e)
    if (e0 + e < E) {
#pragma unroll
      for (int v = 0; v < VN; v += 4)
        *reinterpret_cast<float4*>(out + (size_t)(e0 + e) * d + v) = make_float4(acc[e][v], acc[e][v + 1], acc[e][v + 2], acc[e][v + 3]);
    }
}

// Gate weight gradient on the matrix cores (bf16 x, more than 16 experts, where the kernel above is bound by its
// fp32 multiply-adds: E of them per token and column for k non-zeros).  dWr^T[e][c] = sum_t d_logits[t][e] x[t][c]
// is an MFMA with experts as M, columns as N and tokens as K.  Both operands have K (tokens) as the slow index in
// memory, so the tiles of a K step of 32 tokens lie in LDS as [token][column] and [token][expert] and the
// fragments come from transposing LDS reads.  d_logits is fp32 and enters as two bf16 terms (hi + lo, about 16
// mantissa bits), like the gate weight in the forward kernel.  LDS rows are 256 bytes or longer; their 64-byte
// granules are XOR-swizzled with token % 4 and the 32-byte halves with (token / 8) % 2, which spreads the four
// token rows of one transposing read, and two reads eight rows apart, over the banks.
// A block: 128 columns, a slice of tokens, up to 128 experts (NET tiles of 16; more experts: gridDim.z blocks,
// which keeps the accumulators at 64 registers and several blocks on a compute unit); a wave: 32 of the
// columns.  Global loads of the next K step are in flight while the MFMAs of this one run.
typedef short rt_s16x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ int rt_ks_mask(int krow) { return ((krow & 3) << 6) | (((krow >> 3) & 1) << 5); }
// the eight K values of a lane (column l % 16 of a 16-column tile, K rows 8 (l / 16) .. + 7): two transposing
// reads of four K rows each; lane s of a 16-lane block passes the address of (K row s / 4, columns 4 (s % 4) .. + 3)
__device__ __forceinline__ rt_bf16x8 rt_read_tr(const char* p, int row_bytes) {
  typedef __attribute__((address_space(3))) rt_s16x4 lds_v;
  union { struct { rt_s16x4 a, b; } q; rt_bf16x8 v; } u;
  u.q.a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v*)(p));
  u.q.b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v*)(p + 4 * row_bytes));
  return u.v;
}
template <typename T, int NET>
__global__ __launch_bounds__(256) void route_bwd_dwr_mfma_kernel(
    const T* __restrict__ x, const float* __restrict__ d_logits, float* __restrict__ partials, int Tn, int d, int E,
    int slice_tokens) {
  constexpr int CB = ROUTE_BWD_MFMA_COLS, KS = ROUTE_BWD_MFMA_KSTEP, EP = NET * 16;
  constexpr int XB = CB * 2;                      // bytes per token row of the x tile
  constexpr int PB = (EP < 128 ? 128 : EP) * 2;   // bytes per token row of a d_logits plane
  constexpr int NP = KS * EP / 2 / 256;           // pairs of adjacent experts per thread and K step
  static_assert(CB == 128 && KS == 32 && NP >= 1, "256 threads: 16 column groups x 16 token rows, twice");
  constexpr int XT = XTerms<T>::N;                // x tiles: one (bf16) or two (the bf16 terms of fp16 values)
  extern __shared__ __align__(16) char dwr_smem[];
  char* xs = dwr_smem;
  char* ph = dwr_smem + XT * KS * XB;
  char* pl = ph + KS * PB;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c0 = blockIdx.x * CB, t_begin = blockIdx.y * slice_tokens, t_end = min(Tn, t_begin + slice_tokens);
  const int e_base = blockIdx.z * EP;
  const int nsteps = (t_end - t_begin + KS - 1) / KS;

  uint4 xr[2];
  float dr[NP][2];
  auto fetch = [&](int step) {   // global -> registers; tokens past the slice or the batch: x of the last token, d_logits 0
    const int t0 = t_begin + step * KS;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int t = min(t0 + (tid >> 4) + h * 16, Tn - 1), col = c0 + (tid & 15) * 8;
      xr[h] = col < d ? *reinterpret_cast<const uint4*>(x + (size_t)t * d + col) : uint4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int j = 0; j < NP; ++j) {
      const int i = tid + 256 * j, t = t0 + i / (EP / 2), e = e_base + (i % (EP / 2)) * 2;
      const float* row = d_logits + (size_t)min(t, Tn - 1) * E;
      dr[j][0] = (t < t_end && e < E) ? row[e] : 0.f;
      dr[j][1] = (t < t_end && e + 1 < E) ? row[e + 1] : 0.f;
    }
  };
  auto stash = [&]() {           // registers -> LDS, d_logits split into its two bf16 terms
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int r = (tid >> 4) + h * 16;
      rt_bf16x8 terms[XT];
      XTerms<T>::split(xr[h], terms);
#pragma unroll
      for (int xt = 0; xt < XT; ++xt)
        *reinterpret_cast<rt_bf16x8*>(xs + xt * KS * XB + r * XB + (((tid & 15) * 16) ^ rt_ks_mask(r))) = terms[xt];
    }
#pragma unroll
    for (int j = 0; j < NP; ++j) {
      const int i = tid + 256 * j, r = i / (EP / 2), e = (i % (EP / 2)) * 2;
      const uint32_t h0 = f32_to_bf16_bits(dr[j][0]), h1 = f32_to_bf16_bits(dr[j][1]);
      const uint32_t l0 = f32_to_bf16_bits(dr[j][0] - bf16_bits_to_f32(h0)), l1 = f32_to_bf16_bits(dr[j][1] - bf16_bits_to_f32(h1));
      const int off = r * PB + ((e * 2) ^ rt_ks_mask(r));
      *reinterpret_cast<uint32_t*>(ph + off) = h0 | (h1 << 16);
      *reinterpret_cast<uint32_t*>(pl + off) = l0 | (l1 << 16);
    }
  };

  rt_f32x4 acc[NET][2];
#pragma unroll
  for (int nt = 0; nt < NET; ++nt)
#pragma unroll
    for (int ct = 0; ct < 2; ++ct) acc[nt][ct] = rt_f32x4{0.f, 0.f, 0.f, 0.f};
  const int s16 = lane & 15, kgrp = lane >> 4;
  const int krow = kgrp * 8 + (s16 >> 2), mask = rt_ks_mask(krow), sub = 8 * (s16 & 3);   // this lane's piece of a transposing read
  fetch(0);
  for (int step = 0; step < nsteps; ++step) {
    stash();
    __syncthreads();
    if (step + 1 < nsteps) fetch(step + 1);
    rt_bf16x8 bx[XT][2];
#pragma unroll
    for (int xt = 0; xt < XT; ++xt)
#pragma unroll
      for (int ct = 0; ct < 2; ++ct)
        bx[xt][ct] = rt_read_tr(xs + xt * KS * XB + krow * XB + (((wave * 32 + ct * 16) * 2) ^ mask) + sub, XB);
#pragma unroll
    for (int nt = 0; nt < NET; ++nt) {
      const int off = krow * PB + ((nt * 32) ^ mask) + sub;
      const rt_bf16x8 hi = rt_read_tr(ph + off, PB), lo = rt_read_tr(pl + off, PB);
#pragma unroll
      for (int xt = 0; xt < XT; ++xt) {
#pragma unroll
        for (int ct = 0; ct < 2; ++ct) acc[nt][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hi, bx[xt][ct], acc[nt][ct], 0, 0, 0);
#pragma unroll
        for (int ct = 0; ct < 2; ++ct) acc[nt][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(lo, bx[xt][ct], acc[nt][ct], 0, 0, 0);
      }
    }
    __syncthreads();   // every wave is done with the tiles before the next K step overwrites them
  }
  // accumulator register v of lane l: expert 4 (l / 16) + v of the tile, column l % 16
  float* out = partials + (size_t)blockIdx.y * E * d;
#pragma unroll
  for (int nt = 0; nt < NET; ++nt)
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int e = e_base + nt * 16 + kgrp * 4 + v, col = c0 + wave * 32 + ct * 16 + s16;
        if (e < E && col < d) out[(size_t)e * d + col] = acc[nt][ct][v];
      }
}
template <typename T, int NET>
static int launch_dwr_mfma(const moe_cfg* c, const void* x, const float* d_logits, float* partials, hipStream_t s) {
  const RouteBwdMfmaGeom gm = route_bwd_mfma_geom(c->T, c->d_model, c->E);
  constexpr int EP = NET * 16, PB = (EP < 128 ? 128 : EP) * 2;
  static_assert(EP <= ROUTE_BWD_MFMA_EXPERTS, "a block along gridDim.z covers ROUTE_BWD_MFMA_EXPERTS experts");
  const size_t lds = (size_t)ROUTE_BWD_MFMA_KSTEP * (XTerms<T>::N * ROUTE_BWD_MFMA_COLS * 2 + 2 * PB);
  route_bwd_dwr_mfma_kernel<T, NET><<<dim3(gm.col_blocks, gm.rows, gm.expert_blocks), 256, lds, s>>>((const T*)x, d_logits, partials, c->T,
                                                                              c->d_model, c->E, gm.slice_tokens);
  return launch_status();
}

// dWr = sum over the rows of partial sums, in a fixed order (deterministic).  A block owns 64 adjacent
// elements of a row of partial sums; its four waves take the rows r = w, w+4, ... (each a coalesced
// 256-byte read), and the four wave sums are added in wave order.  The rows are laid out [E][d], dWr itself [d][E].
__global__ __launch_bounds__(256) void route_bwd_reduce_kernel(const float* __restrict__ partials, float* __restrict__ dWr,
                                                               int d, int E, int rows, int accumulate) {
  __shared__ float s_part[4][64];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, n = d * E;
  const int i = blockIdx.x * 64 + lane;
  float s = 0.f;
  if (i < n) {
#pragma unroll 8
    for (int r = w; r < rows; r += 4) s += partials[(size_t)r * n + i];
  }
  s_part[w][lane] = s;
  __syncthreads();
  if (w == 0 && i < n) {
    const float t = ((s_part[0][lane] + s_part[1][lane]) + s_part[2][lane]) + s_part[3][lane];
    float* o = dWr + (size_t)(i % d) * E + i / d;
    *o = accumulate ? *o + t : t;
  }
}

// ---------------------------------------------------------------- launchers
static int route_expert_tiles(int E) { return E <= 16 ? 1 : (E <= 32 ? 2 : (E <= 64 ? 4 : (E <= 128 ? 8 : 16))); }
size_t route_wfrag_bytes(int d, int E) {
  return (size_t)route_expert_tiles(E) * ((d + 127) / 128) * 8 * 64 * 16;
}

template <typename T, int NET, int TT, int NW>
static int launch_route_mfma(const moe_cfg* c, const void* x, const float* Wr, const float* bias, float* logits_out,
                             int32_t* idx, float* w, void* wfrag, hipStream_t s) {
  constexpr int TOK = TT * 16;
  const int nkb = (c->d_model + 127) / 128, units = NET * nkb * 8 * 64;
  wr_frag_kernel<<<(units + 255) / 256, 256, 0, s>>>(Wr, (rt_bf16x8*)wfrag, c->d_model, c->E, nkb, NET);
  int rc = launch_status();
  if (rc != MOE_OK) return rc;
  const size_t lds = (size_t)NW * TOK * NET * 16 * 4;
  auto kern = route_mfma_kernel<T, NET, TT, NW>;
  if (lds > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return set_hip_error(e);
  }
  kern<<<(c->T + TOK - 1) / TOK, NW * 64, lds, s>>>((const T*)x, (const rt_bf16x8*)wfrag, bias, logits_out, idx, w,
                                                 c->T, c->d_model, c->E, c->k);
  return launch_status();
}

// wfrag: workspace for the gate weight in MFMA operand layout (route_wfrag_bytes), used for bf16 x
template <typename T>
static int route_mfma_typed(const moe_cfg* c, const void* x, const float* Wr, const float* bias, float* logits_out,
                            int32_t* idx, float* w, void* wfrag, hipStream_t s) {
  // long rows and few expert tiles: eight waves and 64 tokens per block; else four waves and 32 tokens
  const bool wide = c->d_model >= 2048;
  switch (route_expert_tiles(c->E)) {
    case 1: return wide ? launch_route_mfma<T, 1, 4, 8>(c, x, Wr, bias, logits_out, idx, w, wfrag, s)
                        : launch_route_mfma<T, 1, 2, 4>(c, x, Wr, bias, logits_out, idx, w, wfrag, s);
    case 2: return wide ? launch_route_mfma<T, 2, 4, 8>(c, x, Wr, bias, logits_out, idx, w, wfrag, s)
                        : launch_route_mfma<T, 2, 2, 4>(c, x, Wr, bias, logits_out, idx, w, wfrag, s);
    case 4: return launch_route_mfma<T, 4, 2, 4>(c, x, Wr, bias, logits_out, idx, w, wfrag, s);
    case 8: return launch_route_mfma<T, 8, 2, 4>(c, x, Wr, bias, logits_out, idx, w, wfrag, s);
    default: return launch_route_mfma<T, 16, 2, 4>(c, x, Wr, bias, logits_out, idx, w, wfrag, s);
  }
}

int launch_route(const moe_cfg* c, const void* x, const float* Wr, const float* bias, const float* logits_in,
                 float* logits_out, int32_t* idx, float* w, void* wfrag, hipStream_t s) {
  if ((c->dtype == MOE_DTYPE_BF16 || c->dtype == MOE_DTYPE_F16) && logits_in == nullptr)
    return c->dtype == MOE_DTYPE_BF16 ? route_mfma_typed<bf16>(c, x, Wr, bias, logits_out, idx, w, wfrag, s)
                                      : route_mfma_typed<f16>(c, x, Wr, bias, logits_out, idx, w, wfrag, s);
  const RouteGeom gm = route_geom(c->E);
  const int grid = (c->T + gm.tok - 1) / gm.tok;
  const size_t es = elt_size(c);
  const size_t lds = (size_t)gm.tok * (gm.dc + RT_XPAD) * es + (size_t)gm.dc * gm.e4 * 4 + (size_t)gm.tok * c->E * 4;
  if (c->dtype == MOE_DTYPE_BF16)
    route_kernel<bf16><<<grid, RT_THREADS, lds, s>>>((const bf16*)x, Wr, bias, logits_in, logits_out, idx, w, c->T, c->d_model, c->E, c->k, gm);
  else if (c->dtype == MOE_DTYPE_F16)
    route_kernel<f16><<<grid, RT_THREADS, lds, s>>>((const f16*)x, Wr, bias, logits_in, logits_out, idx, w, c->T, c->d_model, c->E, c->k, gm);
  else
    route_kernel<float><<<grid, RT_THREADS, lds, s>>>((const float*)x, Wr, bias, logits_in, logits_out, idx, w, c->T, c->d_model, c->E, c->k, gm);
  return launch_status();
}

template <typename T>
static int route_bwd_typed(const moe_cfg* c, const void* x, const float* Wr, const int32_t* idx, const float* w,
                           const float* dw, float* d_logits, float* dWr, void* dx, int accumulate, float* partials,
                           float* WrT, hipStream_t s) {
  const int n = c->d_model * c->E;
  int rc;
  if (dx != nullptr) {
    wr_transpose_kernel<<<(n + 255) / 256, 256, 0, s>>>(Wr, WrT, c->d_model, c->E);
    if ((rc = launch_status()) != MOE_OK) return rc;
  }
  const int grid = (c->T + 3) / 4;
  route_bwd_dx_kernel<T><<<grid, 256, 0, s>>>(WrT, idx, w, dw, d_logits, (T*)dx, c->T, c->d_model, c->E, c->k);
  if ((rc = launch_status()) != MOE_OK) return rc;
  if (dWr == nullptr) return MOE_OK;
  if constexpr (!std::is_same<T, float>::value) {
    if (route_bwd_uses_mfma(1, c->E)) {
      switch (route_expert_tiles(c->E)) {
        case 2: rc = launch_dwr_mfma<T, 2>(c, x, d_logits, partials, s); break;
        case 4: rc = launch_dwr_mfma<T, 4>(c, x, d_logits, partials, s); break;
        default: rc = launch_dwr_mfma<T, 8>(c, x, d_logits, partials, s); break;   // 128 experts per block
      }
      if (rc != MOE_OK) return rc;
      route_bwd_reduce_kernel<<<(n + 63) / 64, 256, 0, s>>>(partials, dWr, c->d_model, c->E,
                                                          route_bwd_mfma_geom(c->T, c->d_model, c->E).rows, accumulate);
      return launch_status();
    }
  }
  const RouteBwdGeom gm = route_bwd_geom(c->T, c->d_model, (int)sizeof(T), c->E);
  const int eb = c->E <= 4 ? 4 : (c->E <= 8 ? 8 : 16);
  const dim3 dgrid(gm.col_blocks, gm.row_blocks, (c->E + eb - 1) / eb);
  const size_t lds = (size_t)gm.slices_per_block * gm.tps * eb * 4;
#define MOE_DWR_DENSE(EB) \
  route_bwd_dwr_dense_kernel<T, EB><<<dgrid, 256, lds, s>>>((const T*)x, d_logits, partials, c->T, c->d_model, c->E, gm)
  if (eb == 4) MOE_DWR_DENSE(4); else if (eb == 8) MOE_DWR_DENSE(8); else MOE_DWR_DENSE(16);
#undef MOE_DWR_DENSE
  if ((rc = launch_status()) != MOE_OK) return rc;
  route_bwd_reduce_kernel<<<(n + 63) / 64, 256, 0, s>>>(partials, dWr, c->d_model, c->E, gm.partial_rows, accumulate);
  return launch_status();
}

int launch_route_bwd(const moe_cfg* c, const void* x, const float* Wr, const int32_t* idx, const float* w,
                     const float* dw, float* d_logits, float* dWr, void* dx, int accumulate, float* partials,
                     float* WrT, hipStream_t s) {
  if (c->dtype == MOE_DTYPE_BF16) return route_bwd_typed<bf16>(c, x, Wr, idx, w, dw, d_logits, dWr, dx, accumulate, partials, WrT, s);
  if (c->dtype == MOE_DTYPE_F16) return route_bwd_typed<f16>(c, x, Wr, idx, w, dw, d_logits, dWr, dx, accumulate, partials, WrT, s);
  return route_bwd_typed<float>(c, x, Wr, idx, w, dw, d_logits, dWr, dx, accumulate, partials, WrT, s);
}

}  // namespace moe

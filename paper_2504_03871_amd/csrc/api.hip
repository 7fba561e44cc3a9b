// C ABI of the MoE library: argument validation, workspace layout, kernel sequencing.
#include "common.h"
#include "gemm.h"
#include "prof.h"
#include <algorithm>

namespace moe {

static thread_local int g_last_hip_error = 0;
int set_hip_error(hipError_t e) {
  g_last_hip_error = (int)e;
  return MOE_ERR_HIP;
}

int check_cfg(const moe_cfg* c) {
  if (c == nullptr) return MOE_ERR_NULL;
  if (c->dtype != MOE_DTYPE_F32 && c->dtype != MOE_DTYPE_BF16 && c->dtype != MOE_DTYPE_F16) return MOE_ERR_BAD_DTYPE;
  if (c->act != MOE_ACT_GELU && c->act != MOE_ACT_SWIGLU) return MOE_ERR_BAD_DTYPE;
  if (c->T < 0 || c->d_model <= 0 || c->d_ff <= 0) return MOE_ERR_BAD_SHAPE;
  if (c->E < 1 || c->E > MOE_MAX_E) return MOE_ERR_BAD_SHAPE;
  if (c->k < 1 || c->k > MOE_MAX_K || c->k > c->E) return MOE_ERR_BAD_SHAPE;
  const int mult = is_half(c) ? 64 : 4;
  if (c->d_model % mult != 0 || c->d_ff % mult != 0) return MOE_ERR_BAD_SHAPE;
  if ((long long)c->T * c->k > (1ll << 30)) return MOE_ERR_BAD_SHAPE;
  if (!offsets_fit_32_bits(c->T, c->k, c->d_model, c->d_ff, (int)elt_size(c))) return MOE_ERR_BAD_SHAPE;
  return MOE_OK;
}

WsLayout ws_layout(const moe_cfg* c) {
  WsLayout w{};
  const size_t A = (size_t)c->T * c->k;
  size_t off = 0;
  w.dispatch_blk_cnt = off;
  off += align_up(((A + DISPATCH_CHUNK - 1) / DISPATCH_CHUNK + 1) * (size_t)c->E * 4, 256);   // + a row of totals
  w.tile_map = off;
  off += align_up(tile_map_bytes(max_row_tiles((int)A, c->E, TILE_ROWS_MIN), c->E), 256);
  w.route_partials = off;
  const size_t partial_rows = route_bwd_uses_mfma(c->dtype != MOE_DTYPE_F32, c->E)
                                  ? (size_t)route_bwd_mfma_geom(c->T, c->d_model, c->E).rows
                                  : (size_t)route_bwd_geom(c->T, c->d_model, (int)elt_size(c), c->E).partial_rows;
  off += align_up(partial_rows * c->d_model * c->E * 4, 256);
  w.route_wrt = off;   // shared with the forward's gate weight in MFMA operand layout (never live together)
  off += align_up(std::max((size_t)c->d_model * c->E * 4, route_wfrag_bytes(c->d_model, c->E)), 256);
  w.ffn_split = off;
  if (is_half(c) && split_k_applies(c->E, c->d_ff))
    off += align_up(split_ws_bytes(c->E, std::max(c->d_model, 1)), 256);
  w.ffn_bwd_dact = off;
  off += align_up((c->act == MOE_ACT_SWIGLU ? 2 : 1) * A * c->d_ff * elt_size(c), 256);
  w.total = off;
  return w;
}

// defined in the kernel files
int launch_route(const moe_cfg*, const void*, const float*, const float*, const float*, float*, int32_t*, float*, void*,
                 hipStream_t);
int launch_route_bwd(const moe_cfg*, const void*, const float*, const int32_t*, const float*, const float*, float*,
                     float*, void*, int, float*, float*, hipStream_t);
int launch_dispatch(const moe_cfg*, const void*, const int32_t*, const int32_t*, const int32_t*, int32_t*, int32_t*,
                    int32_t*, int32_t*, int32_t*, void*, int32_t*, hipStream_t);
int dispatch_static_scratch(int32_t** out);
int launch_combine(const moe_cfg*, const void*, const float*, const int32_t*, const int32_t*, const int32_t*,
                   const int32_t*, const int32_t*, const int32_t*, void*, int, hipStream_t);
int launch_combine_bwd(const moe_cfg*, const void*, const void*, const float*, const int32_t*, const int32_t*,
                       const int32_t*, const int32_t*, const int32_t*, const int32_t*, void*, float*, hipStream_t);

__global__ void fill_zero_kernel(float* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0.f;
}

// Streaming copy / fill for the benchmark: 16-byte vectors, four per thread in flight, grid-stride.
typedef unsigned bs_u32x4 __attribute__((ext_vector_type(4)));
template <bool FILL>
__global__ __launch_bounds__(256) void bench_stream_kernel(bs_u32x4* __restrict__ dst, const bs_u32x4* __restrict__ src, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256 * 4;
  for (size_t i = (size_t)blockIdx.x * 256 * 4 + threadIdx.x; i < n16; i += stride) {
    bs_u32x4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      v[u] = bs_u32x4{0u, 0u, 0u, 0u};
      if (!FILL && i + u * 256 < n16) v[u] = __builtin_nontemporal_load(src + i + u * 256);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (i + u * 256 < n16) __builtin_nontemporal_store(v[u], dst + i + u * 256);
  }
}

// One lane samples the shader-clock counter and the 100 MHz real-time counter n times, sleeping in between
// (a bounded loop: the kernel always ends).  Two consecutive samples give the shader clock over that interval.
__global__ void clock_probe_kernel(unsigned long long* __restrict__ out, int n, int sleeps) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  for (int i = 0; i < n; ++i) {
    out[2 * i] = __builtin_amdgcn_s_memtime();
    out[2 * i + 1] = __builtin_amdgcn_s_memrealtime();
    for (int s = 0; s < sleeps; ++s) __builtin_amdgcn_s_sleep(127);
  }
}

// Nothing but MFMAs on register operands: 32 accumulations per round, each on an accumulator of its own
// (16 x 16 x 32: 32 accumulators of 4 registers; 32 x 32 x 16: 8 accumulators of 16 registers, four rounds of them).
typedef __bf16 ml_bf16x8 __attribute__((ext_vector_type(8)));
typedef float ml_f32x4 __attribute__((ext_vector_type(4)));
typedef float ml_f32x16 __attribute__((ext_vector_type(16)));
template <int KIND>
__global__ __launch_bounds__(512, 1) void mfma_loop_kernel(const ml_bf16x8* __restrict__ in, float* __restrict__ out, int iters) {
  ml_bf16x8 a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a[i] = in[(threadIdx.x * 8 + i) % 4096];
    b[i] = in[(threadIdx.x * 8 + 4 + i) % 4096];
  }
  float s = 0.f;
  if constexpr (KIND == 0) {
    ml_f32x4 acc[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) acc[i] = ml_f32x4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 32; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i % 4], b[(i / 4) % 4], acc[i], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 32; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
  } else {
    ml_f32x16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    for (int it = 0; it < 2 * iters; ++it) {   // 16 instructions of twice the FLOP = the FLOP of a round above
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i % 4], b[(i / 4) % 4], acc[i], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) s += acc[i][v];
  }
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

static int check_ws(const moe_cfg* c, const void* ws, size_t ws_bytes) {
  return (ws != nullptr && ws_bytes < ws_layout(c).total) ? MOE_ERR_WORKSPACE : MOE_OK;
}

static int check_slices(const int32_t* lo, const int32_t* hi) {
  return ((lo == nullptr) != (hi == nullptr)) ? MOE_ERR_BAD_SLICE : MOE_OK;
}

static int launch_gemm(const moe_cfg* c, int mode, int epi, bool dual, bool chain, const GemmArgs& g, int max_tiles,
                       hipStream_t s) {
  return is_half(c) ? launch_gemm_half(c->dtype, mode, epi, dual, chain, g, max_tiles, s)
                    : launch_gemm_f32(mode, epi, dual, chain, g, max_tiles, s);
}
static int tile_rows_for(const moe_cfg* c) { return is_half(c) ? gemm_bf16_tile_rows() : 64; }

}  // namespace moe

using namespace moe;

#define REQUIRE(p) do { if ((p) == nullptr) return MOE_ERR_NULL; } while (0)
#define ALIGNED(p) do { if (misaligned(p)) return MOE_ERR_ALIGN; } while (0)
#define CHECK(expr) do { int rc_ = (expr); if (rc_ != MOE_OK) return rc_; } while (0)

extern "C" {

const char* moe_error_string(int code) {
  switch (code) {
    case MOE_OK: return "ok";
    case MOE_ERR_NULL: return "a required pointer is NULL";
    case MOE_ERR_BAD_SHAPE: return "unsupported shape (T, d_model, d_ff, E or k)";
    case MOE_ERR_BAD_DTYPE: return "unknown dtype or activation";
    case MOE_ERR_BAD_SLICE: return "slice_lo and slice_hi must both be given or both be NULL";
    case MOE_ERR_ALIGN: return "device pointer not 16-byte aligned";
    case MOE_ERR_HIP: return "HIP launch failed (see moe_last_hip_error)";
    case MOE_ERR_WORKSPACE: return "workspace smaller than moe_workspace_bytes(cfg), or problem too large for the static scratch";
    default: return "unknown error code";
  }
}

int moe_last_hip_error(void) { return g_last_hip_error; }

int moe_bench_stream(void* dst, const void* src, size_t bytes, int32_t mode, void* stream) {
  REQUIRE(dst);
  if (mode != 0 && mode != 1) return MOE_ERR_BAD_DTYPE;
  if (mode == 0) REQUIRE(src);
  ALIGNED(dst); ALIGNED(src);
  if (bytes % 16 != 0) return MOE_ERR_BAD_SHAPE;
  if (bytes == 0) return MOE_OK;
  const size_t n16 = bytes / 16;
  const size_t want = (n16 + 1023) / 1024;
  const unsigned grid = (unsigned)(want < 256 * 16 ? want : 256 * 16);
  if (mode == 0) bench_stream_kernel<false><<<grid, 256, 0, (hipStream_t)stream>>>((bs_u32x4*)dst, (const bs_u32x4*)src, n16);
  else bench_stream_kernel<true><<<grid, 256, 0, (hipStream_t)stream>>>((bs_u32x4*)dst, nullptr, n16);
  return launch_status();
}

int moe_bench_clock_probe(uint64_t* samples, int32_t n, int32_t sleeps, void* stream) {
  REQUIRE(samples);
  ALIGNED(samples);
  if (n < 1 || n > (1 << 20) || sleeps < 0 || sleeps > 1000) return MOE_ERR_BAD_SHAPE;
  clock_probe_kernel<<<1, 64, 0, (hipStream_t)stream>>>(reinterpret_cast<unsigned long long*>(samples), n, sleeps);
  return launch_status();
}

int moe_bench_mfma_loop(int32_t kind, int32_t iters, const void* operand, float* sink, void* stream) {
  REQUIRE(operand);
  REQUIRE(sink);
  ALIGNED(operand);
  ALIGNED(sink);
  if (kind < 0 || kind > 1 || iters < 1 || iters > 1000000) return MOE_ERR_BAD_SHAPE;
  if (kind == 0)
    mfma_loop_kernel<0><<<1024, 512, 0, (hipStream_t)stream>>>(reinterpret_cast<const ml_bf16x8*>(operand), sink, iters);
  else
    mfma_loop_kernel<1><<<1024, 512, 0, (hipStream_t)stream>>>(reinterpret_cast<const ml_bf16x8*>(operand), sink, iters);
  return launch_status();
}

int moe_gemm_block_tile(int32_t kind, int64_t block, int32_t n_rt, int32_t n_full_rt, int32_t n_split, int32_t ntm,
                        int32_t ntn, int32_t* out) {
  REQUIRE(out);
  if (block < 0 || block > 0x7fffffffll || ntn < 1 || n_rt < 0 || n_full_rt < 0 || n_full_rt > n_rt || n_split < 0 ||
      n_split > n_rt - n_full_rt)
    return MOE_ERR_BAD_SHAPE;
  for (int i = 0; i < 6; ++i) out[i] = -1;
  if (kind == 0) {
    RowBlock r;
    out[0] = row_tile_block((int)block, n_rt, n_full_rt, n_split, ntn, r) ? 1 : 0;
    if (out[0]) { out[1] = r.rt; out[3] = r.nt; out[4] = r.split_tile; out[5] = r.ksplit; }
    return MOE_OK;
  }
  if (kind == 1) {
    if (ntm < 1) return MOE_ERR_BAD_SHAPE;
    int slot, mt, nt;
    out[0] = dw_block((int)block, ntm, ntn, slot, mt, nt) ? 1 : 0;
    if (out[0]) { out[1] = slot; out[2] = mt; out[3] = nt; }
    return MOE_OK;
  }
  return MOE_ERR_BAD_DTYPE;
}

int moe_workspace_bytes(const moe_cfg* cfg, size_t* bytes) {
  CHECK(check_cfg(cfg));
  REQUIRE(bytes);
  *bytes = ws_layout(cfg).total;
  return MOE_OK;
}

int moe_saved_bytes(const moe_cfg* cfg, size_t* bytes) {
  CHECK(check_cfg(cfg));
  REQUIRE(bytes);
  *bytes = (size_t)(cfg->act == MOE_ACT_SWIGLU ? 3 : 2) * cfg->T * cfg->k * cfg->d_ff * elt_size(cfg);
  return MOE_OK;
}

int moe_route(const moe_cfg* cfg, const void* x, const float* Wr, const float* bias, const float* logits_in,
              float* logits_out, int32_t* topk_idx, float* topk_w, void* ws, size_t ws_bytes, void* stream) {
  CHECK(check_cfg(cfg));
  if (logits_in == nullptr) { REQUIRE(x); REQUIRE(Wr); REQUIRE(logits_out); }
  if (logits_in == nullptr && cfg->dtype != MOE_DTYPE_F32) REQUIRE(ws);   // the matrix-core gate (16-bit storage)
  REQUIRE(topk_idx);
  REQUIRE(topk_w);
  ALIGNED(x); ALIGNED(Wr); ALIGNED(bias); ALIGNED(logits_in); ALIGNED(logits_out); ALIGNED(topk_idx); ALIGNED(topk_w);
  ALIGNED(ws);
  CHECK(check_ws(cfg, ws, ws_bytes));
  if (cfg->T == 0) return MOE_OK;
  void* wfrag = ws != nullptr ? static_cast<char*>(ws) + ws_layout(cfg).route_wrt : nullptr;
  ProfScope ps(cfg, MOE_PROF_ROUTE, (hipStream_t)stream);
  return launch_route(cfg, x, Wr, bias, logits_in, logits_out, topk_idx, topk_w, wfrag, (hipStream_t)stream);
}

int moe_dispatch(const moe_cfg* cfg, const void* x, const int32_t* topk_idx, const int32_t* slice_lo,
                 const int32_t* slice_hi, int32_t* counts, int32_t* kept, int32_t* offsets, int32_t* row_of,
                 int32_t* src_of, void* x_perm, void* ws, size_t ws_bytes, void* stream) {
  CHECK(check_cfg(cfg));
  CHECK(check_slices(slice_lo, slice_hi));
  REQUIRE(topk_idx); REQUIRE(counts); REQUIRE(kept); REQUIRE(offsets); REQUIRE(row_of); REQUIRE(src_of); REQUIRE(ws);
  if (x_perm != nullptr) REQUIRE(x);
  ALIGNED(x); ALIGNED(topk_idx); ALIGNED(slice_lo); ALIGNED(slice_hi); ALIGNED(counts); ALIGNED(kept);
  ALIGNED(offsets); ALIGNED(row_of); ALIGNED(src_of); ALIGNED(x_perm); ALIGNED(ws);
  CHECK(check_ws(cfg, ws, ws_bytes));
  const WsLayout w = ws_layout(cfg);
  int32_t* blk_cnt = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + w.dispatch_blk_cnt);
  // T == 0 still has to produce zero counts and offsets: the kernels handle an empty assignment list
  return launch_dispatch(cfg, x, topk_idx, slice_lo, slice_hi, counts, kept, offsets, row_of, src_of, x_perm, blk_cnt,
                         (hipStream_t)stream);
}

int moe_dispatch_static(const moe_cfg* cfg, const void* x, const int32_t* topk_idx, const int32_t* slice_lo,
                        const int32_t* slice_hi, int32_t* counts, int32_t* kept, int32_t* offsets, int32_t* row_of,
                        int32_t* src_of, void* x_perm, void* stream) {
  CHECK(check_cfg(cfg));
  CHECK(check_slices(slice_lo, slice_hi));
  REQUIRE(topk_idx); REQUIRE(counts); REQUIRE(kept); REQUIRE(offsets); REQUIRE(row_of); REQUIRE(src_of);
  if (x_perm != nullptr) REQUIRE(x);
  ALIGNED(x); ALIGNED(topk_idx); ALIGNED(slice_lo); ALIGNED(slice_hi); ALIGNED(counts); ALIGNED(kept);
  ALIGNED(offsets); ALIGNED(row_of); ALIGNED(src_of); ALIGNED(x_perm);
  // the same per-block histogram region as the workspace version, held to the size of the static array
  const size_t A = (size_t)cfg->T * cfg->k;
  const size_t need = ((A + DISPATCH_CHUNK - 1) / DISPATCH_CHUNK + 1) * (size_t)cfg->E * 4;
  if (need > MOE_DISPATCH_STATIC_BYTES) return MOE_ERR_WORKSPACE;
  int32_t* blk_cnt = nullptr;
  CHECK(dispatch_static_scratch(&blk_cnt));
  return launch_dispatch(cfg, x, topk_idx, slice_lo, slice_hi, counts, kept, offsets, row_of, src_of, x_perm, blk_cnt,
                         (hipStream_t)stream);
}

namespace {
// GEMM1 with its activation epilogue into `saved` (or, saved == NULL, its hidden activation alone into
// `hidden`), then (y_perm != NULL) GEMM2.
int ffn_fwd_impl(const moe_cfg* cfg, const void* x_perm, const void* W1, const void* W1b, const void* W2,
                 const int32_t* offsets, const int32_t* kept, const int32_t* slice_lo, const int32_t* slice_hi,
                 void* saved, void* hidden, void* y_perm, void* ws, hipStream_t s) {
  const bool swiglu = cfg->act == MOE_ACT_SWIGLU;
  const WsLayout w = ws_layout(cfg);
  const int A = cfg->T * cfg->k, d = cfg->d_model, f = cfg->d_ff;
  const int tr = tile_rows_for(cfg), max_tiles = max_row_tiles(A, cfg->E, tr);
  TileMap map = tile_map_at(static_cast<char*>(ws) + w.tile_map, max_row_tiles(A, cfg->E, TILE_ROWS_MIN), cfg->E);
  CHECK(launch_tile_map(offsets, kept, slice_lo, slice_hi, cfg->E, tr, map,
                        !swiglu && cfg->dtype == MOE_DTYPE_BF16 ? GELU_TAB_PHI : GELU_TAB_NONE, s));
  const size_t plane = (size_t)A * f * elt_size(cfg);
  char* sv = static_cast<char*>(saved);
  GemmArgs g = {};
  g.tiles = map.tiles; g.ntiles = map.header; g.order = map.order; g.gelu_tab = map.gelu_tab;
  g.offsets = offsets; g.kept = kept; g.lo = slice_lo; g.hi = slice_hi; g.E = cfg->E;
  // hidden = act(x_perm W1)
  g.A = x_perm; g.B = W1; g.B2 = W1b; g.N = f; g.K = d;
  g.C = sv; g.C2 = sv + plane; g.C3 = sv + 2 * plane;
  char* hid = swiglu ? sv + 2 * plane : sv + plane;
  if (saved == nullptr) {   // keep nothing but the hidden activation
    hid = static_cast<char*>(hidden);
    g.C = nullptr; g.C2 = swiglu ? nullptr : hid; g.C3 = swiglu ? hid : nullptr;
  }
  {
    ProfScope ps(cfg, MOE_PROF_GEMM1_FWD, s);
    CHECK(launch_gemm(cfg, MODE_NN, swiglu ? EPI_SWIGLU_FWD : EPI_GELU_FWD, swiglu, false, g, max_tiles, s));
  }
  if (y_perm == nullptr) return MOE_OK;
  // y = hidden W2
  g.A = hid; g.B = W2; g.B2 = nullptr; g.N = d; g.K = f;
  g.C = y_perm; g.C2 = g.C3 = nullptr;
  if (is_half(cfg) && split_k_applies(cfg->E, f))   // smallest row tiles: split-K (gemm.h)
    g.split_ws = reinterpret_cast<float*>(static_cast<char*>(ws) + w.ffn_split);
  ProfScope ps(cfg, MOE_PROF_GEMM2_FWD, s);
  return launch_gemm(cfg, MODE_NN, EPI_STORE, false, false, g, max_tiles, s);
}
}  // namespace

int moe_expert_ffn_fwd(const moe_cfg* cfg, const void* x_perm, const void* W1, const void* W1b, const void* W2,
                       const int32_t* offsets, const int32_t* kept, const int32_t* slice_lo, const int32_t* slice_hi,
                       void* saved, void* y_perm, void* ws, size_t ws_bytes, void* stream) {
  CHECK(check_cfg(cfg));
  CHECK(check_slices(slice_lo, slice_hi));
  REQUIRE(x_perm); REQUIRE(W1); REQUIRE(W2); REQUIRE(offsets); REQUIRE(kept); REQUIRE(saved); REQUIRE(y_perm); REQUIRE(ws);
  const bool swiglu = cfg->act == MOE_ACT_SWIGLU;
  if (swiglu) REQUIRE(W1b);
  if (!swiglu && W1b != nullptr) return MOE_ERR_BAD_DTYPE;
  ALIGNED(x_perm); ALIGNED(W1); ALIGNED(W1b); ALIGNED(W2); ALIGNED(offsets); ALIGNED(kept); ALIGNED(slice_lo);
  ALIGNED(slice_hi); ALIGNED(saved); ALIGNED(y_perm); ALIGNED(ws);
  CHECK(check_ws(cfg, ws, ws_bytes));
  if (cfg->T == 0) return MOE_OK;
  return ffn_fwd_impl(cfg, x_perm, W1, W1b, W2, offsets, kept, slice_lo, slice_hi, saved, nullptr, y_perm, ws,
                      (hipStream_t)stream);
}

int moe_expert_ffn_fwd_light(const moe_cfg* cfg, const void* x_perm, const void* W1, const void* W1b, const void* W2,
                             const int32_t* offsets, const int32_t* kept, const int32_t* slice_lo,
                             const int32_t* slice_hi, void* hidden, void* y_perm, void* ws, size_t ws_bytes,
                             void* stream) {
  CHECK(check_cfg(cfg));
  CHECK(check_slices(slice_lo, slice_hi));
  REQUIRE(x_perm); REQUIRE(W1); REQUIRE(W2); REQUIRE(offsets); REQUIRE(kept); REQUIRE(hidden); REQUIRE(y_perm); REQUIRE(ws);
  const bool swiglu = cfg->act == MOE_ACT_SWIGLU;
  if (swiglu) REQUIRE(W1b);
  if (!swiglu && W1b != nullptr) return MOE_ERR_BAD_DTYPE;
  ALIGNED(x_perm); ALIGNED(W1); ALIGNED(W1b); ALIGNED(W2); ALIGNED(offsets); ALIGNED(kept); ALIGNED(slice_lo);
  ALIGNED(slice_hi); ALIGNED(hidden); ALIGNED(y_perm); ALIGNED(ws);
  CHECK(check_ws(cfg, ws, ws_bytes));
  if (cfg->T == 0) return MOE_OK;
  return ffn_fwd_impl(cfg, x_perm, W1, W1b, W2, offsets, kept, slice_lo, slice_hi, nullptr, hidden, y_perm, ws,
                      (hipStream_t)stream);
}

int moe_expert_ffn_recompute(const moe_cfg* cfg, const void* x_perm, const void* W1, const void* W1b,
                             const int32_t* offsets, const int32_t* kept, const int32_t* slice_lo,
                             const int32_t* slice_hi, void* saved, void* ws, size_t ws_bytes, void* stream) {
  CHECK(check_cfg(cfg));
  CHECK(check_slices(slice_lo, slice_hi));
  REQUIRE(x_perm); REQUIRE(W1); REQUIRE(offsets); REQUIRE(kept); REQUIRE(saved); REQUIRE(ws);
  const bool swiglu = cfg->act == MOE_ACT_SWIGLU;
  if (swiglu) REQUIRE(W1b);
  if (!swiglu && W1b != nullptr) return MOE_ERR_BAD_DTYPE;
  ALIGNED(x_perm); ALIGNED(W1); ALIGNED(W1b); ALIGNED(offsets); ALIGNED(kept); ALIGNED(slice_lo); ALIGNED(slice_hi);
  ALIGNED(saved); ALIGNED(ws);
  CHECK(check_ws(cfg, ws, ws_bytes));
  if (cfg->T == 0) return MOE_OK;
  return ffn_fwd_impl(cfg, x_perm, W1, W1b, nullptr, offsets, kept, slice_lo, slice_hi, saved, nullptr, nullptr, ws,
                      (hipStream_t)stream);
}

int moe_combine(const moe_cfg* cfg, const void* y_perm, const float* topk_w, const int32_t* topk_idx,
                const int32_t* row_of, const int32_t* offsets, const int32_t* kept, const int32_t* slice_lo,
                const int32_t* slice_hi, void* out, int32_t accumulate, void* stream) {
  CHECK(check_cfg(cfg));
  CHECK(check_slices(slice_lo, slice_hi));
  REQUIRE(y_perm); REQUIRE(topk_idx); REQUIRE(row_of); REQUIRE(offsets); REQUIRE(kept); REQUIRE(out);
  ALIGNED(y_perm); ALIGNED(topk_w); ALIGNED(topk_idx); ALIGNED(row_of); ALIGNED(offsets); ALIGNED(kept);
  ALIGNED(slice_lo); ALIGNED(slice_hi); ALIGNED(out);
  if (cfg->T == 0) return MOE_OK;
  ProfScope ps(cfg, MOE_PROF_COMBINE, (hipStream_t)stream);
  return launch_combine(cfg, y_perm, topk_w, topk_idx, row_of, offsets, kept, slice_lo, slice_hi, out, accumulate,
                        (hipStream_t)stream);
}

int moe_combine_bwd(const moe_cfg* cfg, const void* d_out, const void* y_perm, const float* topk_w,
                    const int32_t* topk_idx, const int32_t* row_of, const int32_t* offsets, const int32_t* kept,
                    const int32_t* slice_lo, const int32_t* slice_hi, void* dy_perm, float* d_topk_w, void* stream) {
  CHECK(check_cfg(cfg));
  CHECK(check_slices(slice_lo, slice_hi));
  REQUIRE(d_out); REQUIRE(y_perm); REQUIRE(topk_w); REQUIRE(topk_idx); REQUIRE(row_of); REQUIRE(offsets);
  REQUIRE(kept); REQUIRE(dy_perm); REQUIRE(d_topk_w);
  ALIGNED(d_out); ALIGNED(y_perm); ALIGNED(topk_w); ALIGNED(topk_idx); ALIGNED(row_of); ALIGNED(offsets);
  ALIGNED(kept); ALIGNED(slice_lo); ALIGNED(slice_hi); ALIGNED(dy_perm); ALIGNED(d_topk_w);
  if (cfg->T == 0) return MOE_OK;
  ProfScope ps(cfg, MOE_PROF_COMBINE_BWD, (hipStream_t)stream);
  return launch_combine_bwd(cfg, d_out, y_perm, topk_w, topk_idx, row_of, offsets, kept, slice_lo, slice_hi, dy_perm,
                            d_topk_w, (hipStream_t)stream);
}

int moe_expert_ffn_bwd(const moe_cfg* cfg, const void* dy_perm, const void* x_perm, const void* saved, const void* W1,
                       const void* W1b, const void* W2, const int32_t* offsets, const int32_t* kept,
                       const int32_t* slice_lo, const int32_t* slice_hi, void* dx_perm, float* dW1, float* dW1b,
                       float* dW2, int32_t accumulate, void* ws, size_t ws_bytes, void* stream) {
  CHECK(check_cfg(cfg));
  CHECK(check_slices(slice_lo, slice_hi));
  REQUIRE(dy_perm); REQUIRE(x_perm); REQUIRE(saved); REQUIRE(W1); REQUIRE(W2); REQUIRE(offsets); REQUIRE(kept);
  REQUIRE(dx_perm); REQUIRE(dW1); REQUIRE(dW2); REQUIRE(ws);
  const bool swiglu = cfg->act == MOE_ACT_SWIGLU;
  if (swiglu) { REQUIRE(W1b); REQUIRE(dW1b); }
  if (!swiglu && (W1b != nullptr || dW1b != nullptr)) return MOE_ERR_BAD_DTYPE;
  ALIGNED(dy_perm); ALIGNED(x_perm); ALIGNED(saved); ALIGNED(W1); ALIGNED(W1b); ALIGNED(W2); ALIGNED(offsets);
  ALIGNED(kept); ALIGNED(slice_lo); ALIGNED(slice_hi); ALIGNED(dx_perm); ALIGNED(dW1); ALIGNED(dW1b); ALIGNED(dW2);
  ALIGNED(ws);
  CHECK(check_ws(cfg, ws, ws_bytes));
  if (cfg->T == 0) return MOE_OK;
  hipStream_t s = (hipStream_t)stream;
  const WsLayout w = ws_layout(cfg);
  const int A = cfg->T * cfg->k, d = cfg->d_model, f = cfg->d_ff;
  const int tr = tile_rows_for(cfg), max_tiles = max_row_tiles(A, cfg->E, tr);
  TileMap map = tile_map_at(static_cast<char*>(ws) + w.tile_map, max_row_tiles(A, cfg->E, TILE_ROWS_MIN), cfg->E);
  CHECK(launch_tile_map(offsets, kept, slice_lo, slice_hi, cfg->E, tr, map,
                        !swiglu && cfg->dtype == MOE_DTYPE_BF16 ? GELU_TAB_GRAD : GELU_TAB_NONE, s));
  const size_t plane = (size_t)A * f * elt_size(cfg);
  const char* sv = static_cast<const char*>(saved);
  char* dact = static_cast<char*>(ws) + w.ffn_bwd_dact;
  const void* hidden = swiglu ? sv + 2 * plane : sv + plane;
  GemmArgs g = {};
  g.tiles = map.tiles; g.ntiles = map.header; g.order = map.order; g.gelu_tab = map.gelu_tab;
  g.offsets = offsets; g.kept = kept; g.lo = slice_lo; g.hi = slice_hi; g.E = cfg->E;
  g.accumulate = accumulate;
  // Four GEMMs: dH = dy W2^T fused with the activation derivative -> dA (GELU) or dG, dU (SwiGLU);
  // dW2[e] = H^T dy;  dW1[e] = x_perm^T dA (SwiGLU: dW1 from dG, dW1b from dU);
  // dx_perm = dA W1^T (SwiGLU: dG W1^T + dU W1b^T).
  GemmArgs gh = g, gw2 = g, gw1 = g, gx = g;
  gh.A = dy_perm; gh.B = W2; gh.N = f; gh.K = d; gh.C = dact; gh.C2 = dact + plane; gh.S1 = sv; gh.S2 = sv + plane;
  gw2.A = hidden; gw2.B = dy_perm; gw2.M = f; gw2.N = d;  gw2.C = dW2;
  gw1.A = x_perm; gw1.B = dact; gw1.M = d; gw1.N = f; gw1.C = dW1;
  gx.A = dact; gx.A2 = dact + plane; gx.B = W1; gx.B2 = W1b; gx.N = d; gx.K = f; gx.C = dx_perm;
  const int epi_h = swiglu ? EPI_SWIGLU_BWD : EPI_GELU_BWD;
  // bf16: a row-tile GEMM with few rounds of tiles shares its launch with the weight-gradient GEMM that
  // follows it (dH with dW2, dx with dW1), whose tiles then start on the compute units that its last,
  // partly filled round leaves idle.  With many rounds that idle share is small and separate launches
  // keep the cache to one GEMM at a time.  (Timing brackets: a shared launch counts under the row-tile GEMM.)
  const bool bf = is_half(cfg);
  const long long few = 8ll * 256;   // tiles: about eight rounds on this chip
  const bool pair_h = bf && (long long)((f + tr - 1) / tr) * max_tiles <= few;
  const bool pair_x = bf && (long long)((d + tr - 1) / tr) * max_tiles <= few;
  {
    ProfScope ps(cfg, MOE_PROF_DH_BWD, s);
    if (pair_h) CHECK(launch_gemm_half_pair(cfg->dtype, epi_h, false, gh, max_tiles, gw2, s));
    else CHECK(launch_gemm(cfg, MODE_NT, epi_h, false, false, gh, max_tiles, s));
  }
  if (!pair_h) {
    ProfScope ps(cfg, MOE_PROF_DW2_BWD, s);
    CHECK(launch_gemm(cfg, MODE_TN, EPI_DW, false, false, gw2, 0, s));
  }
  if (!pair_x || swiglu) {
    ProfScope ps(cfg, MOE_PROF_DW1_BWD, s);
    if (!pair_x) CHECK(launch_gemm(cfg, MODE_TN, EPI_DW, false, false, gw1, 0, s));
    if (swiglu) {
      GemmArgs gw1b = gw1;
      gw1b.B = dact + plane; gw1b.C = dW1b;
      CHECK(launch_gemm(cfg, MODE_TN, EPI_DW, false, false, gw1b, 0, s));
    }
  }
  ProfScope ps(cfg, MOE_PROF_DX_BWD, s);
  if (bf && !swiglu && split_k_applies(cfg->E, f))   // the smallest row tiles of the GELU dx use split-K (gemm.h)
    gx.split_ws = reinterpret_cast<float*>(static_cast<char*>(ws) + w.ffn_split);
  if (pair_x) return launch_gemm_half_pair(cfg->dtype, EPI_STORE, swiglu, gx, max_tiles, gw1, s);
  return launch_gemm(cfg, MODE_NT, EPI_STORE, false, swiglu, gx, max_tiles, s);
}

int moe_route_bwd(const moe_cfg* cfg, const void* x, const float* Wr, const int32_t* topk_idx, const float* topk_w,
                  const float* d_topk_w, float* d_logits, float* dWr, void* dx, int32_t accumulate, void* ws,
                  size_t ws_bytes, void* stream) {
  CHECK(check_cfg(cfg));
  REQUIRE(x); REQUIRE(Wr); REQUIRE(topk_idx); REQUIRE(topk_w); REQUIRE(d_topk_w); REQUIRE(d_logits);
  REQUIRE(ws);
  ALIGNED(x); ALIGNED(Wr); ALIGNED(topk_idx); ALIGNED(topk_w); ALIGNED(d_topk_w); ALIGNED(d_logits); ALIGNED(dWr);
  ALIGNED(dx); ALIGNED(ws);
  CHECK(check_ws(cfg, ws, ws_bytes));
  hipStream_t s = (hipStream_t)stream;
  if (cfg->T == 0) {
    if (accumulate || dWr == nullptr) return MOE_OK;
    const int n = cfg->d_model * cfg->E;
    fill_zero_kernel<<<(n + 255) / 256, 256, 0, s>>>(dWr, n);   // a kernel, not a memset: safe under graph capture
    return launch_status();
  }
  const WsLayout w = ws_layout(cfg);
  float* partials = reinterpret_cast<float*>(static_cast<char*>(ws) + w.route_partials);
  float* wrt = reinterpret_cast<float*>(static_cast<char*>(ws) + w.route_wrt);
  return launch_route_bwd(cfg, x, Wr, topk_idx, topk_w, d_topk_w, d_logits, dWr, dx, accumulate != 0, partials, wrt, s);
}

}  // extern "C"

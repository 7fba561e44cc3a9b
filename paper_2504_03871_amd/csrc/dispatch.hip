// Dispatch: stable group-by-expert of the T*k assignments and the row gather.
//
// The paper's dispatch all-to-all sends each token embedding to the GPU that holds the target
// expert (Section 2.1); on one GPU this is a permutation.  Order inside an expert is ascending
// token index, so the result is unique and the capacity cut ("first C of the list") is the
// stable rank itself.  Everything here is integer work and deterministic: per-block histograms,
// a scan over blocks, and an in-block stable rank built from wave ballots.
#include "common.h"
#include "prof.h"
#include <mutex>

namespace moe {

constexpr int DP_THREADS = 256;
constexpr int DP_WAVES = DP_THREADS / WAVE;
constexpr int DP_ROUNDS = DISPATCH_CHUNK / DP_THREADS;   // 4
constexpr int DP_SUB = DP_ROUNDS * DP_WAVES;             // 16 sub-chunks of 64 assignments, ascending
static_assert(MOE_MAX_E == 4 * WAVE, "the rank kernel scans the experts four per lane of one wave");

__global__ __launch_bounds__(DP_THREADS) void dispatch_hist_kernel(const int32_t* __restrict__ topk_idx, int A, int E,
                                                                  int32_t* __restrict__ blk_cnt) {
  __shared__ int s_cnt[MOE_MAX_E];
  for (int e = threadIdx.x; e < E; e += DP_THREADS) s_cnt[e] = 0;
  __syncthreads();
  const int base = blockIdx.x * DISPATCH_CHUNK;
#pragma unroll
  for (int r = 0; r < DP_ROUNDS; ++r) {
    const int a = base + r * DP_THREADS + threadIdx.x;
    if (a < A) {
      const int e = topk_idx[a];
      if (e >= 0 && e < E) atomicAdd(&s_cnt[e], 1);   // an id outside [0, E) is a dropped assignment
    }
  }
  __syncthreads();
  for (int e = threadIdx.x; e < E; e += DP_THREADS) blk_cnt[(size_t)blockIdx.x * E + e] = s_cnt[e];
}

// Many blocks (more than DP_INLINE_SCAN): the per-block counts are turned into exclusive prefixes over the
// blocks once, in place, one thread per expert, and row nblk receives the totals; the rank kernel then reads
// two rows instead of scanning all of them (which would make the work quadratic in the number of blocks).
constexpr int DP_INLINE_SCAN = 64;
__global__ __launch_bounds__(DP_THREADS) void dispatch_scan_kernel(int32_t* __restrict__ blk_cnt, int E, int nblk) {
  const int e = blockIdx.x * DP_THREADS + threadIdx.x;
  if (e >= E) return;
  int run = 0;
  for (int b = 0; b < nblk; ++b) {
    const int c = blk_cnt[(size_t)b * E + e];
    blk_cnt[(size_t)b * E + e] = run;
    run += c;
  }
  blk_cnt[(size_t)nblk * E + e] = run;
}

// SCANNED: blk_cnt holds exclusive prefixes and a row of totals (dispatch_scan_kernel) instead of counts.
template <bool SCANNED>
__global__ __launch_bounds__(DP_THREADS) void dispatch_rank_kernel(
    const int32_t* __restrict__ topk_idx, const int32_t* __restrict__ blk_cnt, int A, int E, int capacity, int nblk,
    int32_t* __restrict__ counts, int32_t* __restrict__ kept, int32_t* __restrict__ offsets,
    int32_t* __restrict__ row_of, int32_t* __restrict__ src_of) {
  __shared__ int s_before[MOE_MAX_E];            // assignments of expert e in earlier blocks
  __shared__ int s_kept[MOE_MAX_E];
  __shared__ int s_off[MOE_MAX_E + 1];
  __shared__ int s_sub[DP_SUB][MOE_MAX_E];       // per sub-chunk counts, then exclusive offsets
  const int tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid / WAVE;

  // this block's assignments: loaded first, so that their latency runs beside the scan over blocks
  const int base = blockIdx.x * DISPATCH_CHUNK;
  int my_e[DP_ROUNDS], my_rank[DP_ROUNDS];
#pragma unroll
  for (int r = 0; r < DP_ROUNDS; ++r) {
    const int a = base + r * DP_THREADS + tid;
    int e = (a < A) ? topk_idx[a] : -1;
    if (e < 0 || e >= E) e = -1;        // past the end, or an id outside [0, E): dropped, never an index
    my_e[r] = e;
  }

  // scan over blocks: s_before = assignments of e in earlier blocks, s_kept = all of them for now
  for (int e = tid; e < MOE_MAX_E; e += DP_THREADS) { s_before[e] = 0; s_kept[e] = 0; }
  for (int sc = 0; sc < DP_SUB; ++sc)
    for (int e = tid; e < E; e += DP_THREADS) s_sub[sc][e] = 0;
  __syncthreads();
  if constexpr (SCANNED) {
    for (int e = tid; e < E; e += DP_THREADS)
      if (nblk > 0) { s_before[e] = blk_cnt[(size_t)blockIdx.x * E + e]; s_kept[e] = blk_cnt[(size_t)nblk * E + e]; }
  } else {
    // few blocks: every block adds up all nblk x E counts itself: all threads load, eight counts each in
    // flight; a thread walks the flat index i = b * E + e in steps of the block size, keeps sums in
    // registers while its expert stays the same (always, when E divides the block size) and adds them to
    // LDS when it changes (integer sums: the order of the additions does not matter)
    const int n = nblk * E;
    const int db = DP_THREADS / E, de = DP_THREADS % E;
    int b = tid / E, e = tid % E;
    int cur = e, tot = 0, bef = 0;
    for (int i0 = tid; i0 < n; i0 += DP_THREADS * 8) {
      int c[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int i = i0 + u * DP_THREADS;
        c[u] = i < n ? blk_cnt[i] : 0;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (e != cur) {
          if (tot != 0) atomicAdd(&s_kept[cur], tot);
          if (bef != 0) atomicAdd(&s_before[cur], bef);
          cur = e; tot = 0; bef = 0;
        }
        tot += c[u];
        bef += (b < (int)blockIdx.x) ? c[u] : 0;
        b += db;
        e += de;
        if (e >= E) { e -= E; ++b; }
      }
    }
    if (tot != 0) atomicAdd(&s_kept[cur], tot);
    if (bef != 0) atomicAdd(&s_before[cur], bef);
  }
  __syncthreads();
  // kept counts and their exclusive scan over the experts: the first wave, four experts per lane
  if (wave == 0) {
    int m[4], sum = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = lane * 4 + i;
      const int total = s_kept[e];
      m[i] = (capacity > 0) ? min(total, capacity) : total;
      if (blockIdx.x == 0 && e < E) { counts[e] = total; kept[e] = m[i]; }
      sum += m[i];
    }
    const int incl = wave_scan_i(sum);
    int run = incl - sum;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = lane * 4 + i;
      s_kept[e] = m[i];
      s_off[e] = run;
      run += m[i];
    }
    if (lane == WAVE - 1) s_off[MOE_MAX_E] = run;
  }
  __syncthreads();
  // experts past E hold zero counts, so s_off[E] == s_off[MOE_MAX_E] == all kept rows
  if (blockIdx.x == 0)
    for (int e = tid; e <= E; e += DP_THREADS) offsets[e] = s_off[e];

#pragma unroll
  for (int r = 0; r < DP_ROUNDS; ++r) {
    const int e = my_e[r];
    const bool valid = e >= 0;
    // rank among the lanes of this wave with the same expert, and the number of such lanes
    int rank = 0;
    if (E <= 16) {   // few experts: one pass of ballots per distinct expert present
      unsigned long long todo = __ballot(valid);
      while (todo) {
        const int leader = __ffsll((long long)todo) - 1;
        const int e0 = __shfl(e, leader, WAVE);
        const unsigned long long same = __ballot(valid && e == e0);
        if (valid && e == e0) {
          rank = __popcll(same & ((1ull << lane) - 1ull));
          if (rank == 0) s_sub[r * DP_WAVES + wave][e0] = __popcll(same);   // one writer per (sub-chunk, expert)
        }
        todo &= ~same;
      }
    } else {         // many experts, up to 64 distinct ones in the wave: compare with every lane in turn
      int cnt = 0;
#pragma unroll
      for (int l = 0; l < WAVE; ++l) {
        const bool same = __builtin_amdgcn_readlane(e, l) == e;
        cnt += same;
        rank += same && l < lane;
      }
      if (valid && rank == 0) s_sub[r * DP_WAVES + wave][e] = cnt;
    }
    my_rank[r] = rank;
  }
  __syncthreads();
  for (int e = tid; e < E; e += DP_THREADS) {
    int run = s_before[e];
    for (int sc = 0; sc < DP_SUB; ++sc) { const int c = s_sub[sc][e]; s_sub[sc][e] = run; run += c; }
  }
  __syncthreads();
  const int R = s_off[E];
#pragma unroll
  for (int r = 0; r < DP_ROUNDS; ++r) {
    const int a = base + r * DP_THREADS + tid;
    if (a >= A) continue;
    const int e = my_e[r];
    int row = -1;
    if (e >= 0) {
      const int rank = s_sub[r * DP_WAVES + wave][e] + my_rank[r];
      if (rank < s_kept[e]) { row = s_off[e] + rank; src_of[row] = a; }
    }
    row_of[a] = row;
    if (a >= R) src_of[a] = -1;   // rows past the end of the kept lists
  }
}

// x_perm[row_of[t*k+j]] = x[t] for the slots that are kept and inside this GPU's shares.  Token-major: a wave
// owns a token, reads its row once (16 bytes per lane, GU column chunks in flight) and writes it to the rows
// of its live slots, so the read traffic is the T*d elements the algorithm needs however large k is.  Every
// in-share row belongs to exactly one slot, so all of them are written and no other row is touched.
// The stores are non-temporal (x_perm is far larger than the caches and is read next by another kernel).
constexpr int GU = 8;   // 16-byte column pieces per lane in flight: a row of 4096 16-bit elements in one pass
template <typename T, int KMAX>
__global__ __launch_bounds__(256) void dispatch_gather_kernel(
    const T* __restrict__ x, const int32_t* __restrict__ topk_idx, const int32_t* __restrict__ row_of,
    const int32_t* __restrict__ offsets, const int32_t* __restrict__ kept, const int32_t* __restrict__ lo,
    const int32_t* __restrict__ hi, T* __restrict__ x_perm, int Tn, int d, int k) {
  constexpr int VN = Vec16<T>::N;
  const int lane = threadIdx.x & (WAVE - 1);
  const int t = (blockIdx.x * blockDim.x + threadIdx.x) / WAVE;
  if (t >= Tn) return;
  int rows[KMAX];
  bool any = false;
#pragma unroll
  for (int j = 0; j < KMAX; ++j) {
    rows[j] = -1;
    if (j < k) {
      const int a = t * k + j, row = row_of[a];
      if (row >= 0) {
        bool mine = true;
        if (lo != nullptr) {   // with no shares given every kept row is ours: skip the expert lookup
          const int e = topk_idx[a];
          int l, h;
          share_of(lo, hi, kept[e], e, l, h);
          const int pos = row - offsets[e];
          mine = pos >= l && pos < h;
        }
        if (mine) { rows[j] = row; any = true; }
      }
    }
  }
  if (!any) return;
  const T* src = x + (size_t)t * d;
  for (int c0 = lane * VN; c0 < d; c0 += WAVE * VN * GU) {
    Vec16<T> v[GU];
#pragma unroll
    for (int u = 0; u < GU; ++u)
      if (c0 + u * WAVE * VN < d) v[u].load_nt(src + c0 + u * WAVE * VN);
#pragma unroll
    for (int j = 0; j < KMAX; ++j)
      if (rows[j] >= 0) {
#pragma unroll
        for (int u = 0; u < GU; ++u)
          if (c0 + u * WAVE * VN < d) v[u].store_nt(x_perm + (size_t)rows[j] * d + c0 + u * WAVE * VN);
      }
  }
}

// ---------------------------------------------------------------- dispatch without a caller workspace
// The per-block histograms of moe_dispatch_static live in this file-scope device array instead of the
// caller's workspace.  Every GPU the library runs on holds its own copy until the process ends.  In host
// code the array's name is only a handle: its device address is asked for once per device
// (hipGetSymbolAddress, with that device current) and kept; kernels and everything else get that pointer.
static __device__ __align__(256) int32_t scratch[MOE_DISPATCH_STATIC_BYTES / 4];

constexpr int MAX_DEVICES = 64;
static int32_t* g_scratch_ptr[MAX_DEVICES] = {};
static std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (MOE_ERR_HIP on failure).
int dispatch_static_scratch(int32_t** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return set_hip_error(e);
  if (dev < 0 || dev >= MAX_DEVICES) return MOE_ERR_BAD_SHAPE;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return set_hip_error(e);
    if (p == nullptr) return set_hip_error(hipErrorInvalidSymbol);
    g_scratch_ptr[dev] = static_cast<int32_t*>(p);
  }
  *out = g_scratch_ptr[dev];
  return MOE_OK;
}

int launch_dispatch(const moe_cfg* c, const void* x, const int32_t* idx, const int32_t* lo, const int32_t* hi,
                    int32_t* counts, int32_t* kept, int32_t* offsets, int32_t* row_of, int32_t* src_of, void* x_perm,
                    int32_t* blk_cnt, hipStream_t s) {
  const int A = c->T * c->k;
  const int nblk = (A + DISPATCH_CHUNK - 1) / DISPATCH_CHUNK;
  int rc = MOE_OK;
  if (nblk > 0) {
    dispatch_hist_kernel<<<nblk, DP_THREADS, 0, s>>>(idx, A, c->E, blk_cnt);
    rc = launch_status();
    if (rc != MOE_OK) return rc;
  }
  // with no assignments one block still writes the (all-zero) counts, kept and offsets
  if (nblk > DP_INLINE_SCAN) {
    dispatch_scan_kernel<<<(c->E + DP_THREADS - 1) / DP_THREADS, DP_THREADS, 0, s>>>(blk_cnt, c->E, nblk);
    rc = launch_status();
    if (rc != MOE_OK) return rc;
    dispatch_rank_kernel<true><<<nblk, DP_THREADS, 0, s>>>(idx, blk_cnt, A, c->E, c->capacity, nblk, counts, kept, offsets, row_of, src_of);
  } else {
    dispatch_rank_kernel<false><<<nblk > 0 ? nblk : 1, DP_THREADS, 0, s>>>(idx, blk_cnt, A, c->E, c->capacity, nblk, counts, kept, offsets, row_of, src_of);
  }
  rc = launch_status();
  if (rc != MOE_OK || x_perm == nullptr || A == 0) return rc;
  ProfScope ps(c, MOE_PROF_GATHER, s);
  const int grid = (c->T + 256 / WAVE - 1) / (256 / WAVE);
#define MOE_GATHER(TY, KM) \
  dispatch_gather_kernel<TY, KM><<<grid, 256, 0, s>>>((const TY*)x, idx, row_of, offsets, kept, lo, hi, (TY*)x_perm, c->T, c->d_model, c->k)
  if (c->dtype == MOE_DTYPE_BF16) { if (c->k <= 2) MOE_GATHER(bf16, 2); else if (c->k <= 4) MOE_GATHER(bf16, 4); else MOE_GATHER(bf16, 8); }
  else if (c->dtype == MOE_DTYPE_F16) { if (c->k <= 2) MOE_GATHER(f16, 2); else if (c->k <= 4) MOE_GATHER(f16, 4); else MOE_GATHER(f16, 8); }
  else { if (c->k <= 2) MOE_GATHER(float, 2); else if (c->k <= 4) MOE_GATHER(float, 4); else MOE_GATHER(float, 8); }
#undef MOE_GATHER
  return launch_status();
}

}  // namespace moe

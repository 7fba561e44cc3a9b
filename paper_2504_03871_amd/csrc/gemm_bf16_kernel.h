// Grouped GEMM kernel for the gfx950 matrix cores with 16-bit storage: bf16 (v_mfma_f32_16x16x32_bf16) or
// fp16 (v_mfma_f32_16x16x32_f16), fp32 accumulate.  The storage type ST is a template parameter of the one
// kernel; it selects the MFMA instruction, the conversions of the epilogues, and whether the GELU epilogues
// look their function up (bf16: a table over all bf16 numbers fits in LDS) or evaluate it (fp16).
//
// Why the 16 x 16 x 32 instruction and not 32 x 32 x 16 (same FLOP per cycle): the chip lowers its clock under
// matrix-core load, and by how much depends on the instruction.  A loop of nothing but MFMAs (the library's
// moe_bench_mfma_loop), matrix cores busy 99 % of the cycles in both cases, runs 1.14 times faster with
// 16 x 16 x 32 (about 2.0-2.1 PFLOP/s against 1.7-1.9): 32 x 32 x 16 moves twice the accumulator registers per
// FLOP.  In this kernel the change was worth 4-6 % on x W and dy W^T and 1-2 % on x^T dy, and the shader clock
// sampled during a whole layer step rose from 1.66 to 1.80 GHz.
//
// Work decomposition: block tile BM x BN, WGM x WGN waves; a wave owns BN/WGN adjacent columns and the
// 32-row bands b = wm, wm + WGM, ... of the tile, each band two 16-row MFMA tiles; K advances BKT elements
// per stage, 32 per MFMA ("K step").  Interleaving the bands spreads a partly filled row tile over every
// wave row.
//
// Pipeline: two LDS stages of 64 K values, filled by buffer loads that write LDS directly (no staging
// registers, no LDS store instructions).  An iteration multiplies one stage in two K steps; the first reads
// the fragments of the second, then every wave waits for its own loads of the next stage and joins the
// iteration's one block barrier; the second K step reads the first fragments of the next stage and issues
// the loads of the stage after that into the buffer just released.  64-wide because a 32-wide stage fetches
// an operand with contiguous K as 64-byte pieces of 128-byte lines, which fills the address FIFO of the
// memory pipe (counters: full thirteen times as often); the operands with strided K gain a little from the
// halved number of barriers (weight gradients +2 % against a ring of four 32-wide stages).
// The direct loads are raw instructions: if the compiler knew that they write LDS it would wait for
// every outstanding load before each LDS read it cannot prove disjoint.  The pipeline orders loads and
// reads itself (explicit vmcnt waits, block barriers); the LDS reads stay compiler-tracked.
//
// Operands: one whose K index is contiguous in memory is kept as [rows][BKT] in LDS and read with
// 16-byte LDS reads; one whose K index is strided is kept exactly as it lies in memory, [BKT][cols],
// and read with the transposing 8-byte LDS read of gfx950, so nothing is ever transposed in global
// memory and the same kernel serves x W (NN), dy W^T (NT) and x^T dy (TN).
//
// Epilogue: accumulators go through a per-wave LDS slab to turn the MFMA register layout into rows,
// so that every output (and every saved tensor the backward epilogues read) moves as 8-byte (bf16) or
// 16-byte (fp32 weight gradients) pieces per lane that fill whole 128-byte lines.
//
// MFMA 16x16x32 register layout: lane l supplies row/column l%16 and the eight K values (l/16)*8..+7 of
// the step; accumulator register v of lane l is row (l/16)*4 + v, column l%16 of the 16x16 tile.
#pragma once
#include "gemm.h"

namespace moe {

typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// What depends on the 16-bit storage type: packing two fp32 values, unpacking, and the MFMA instruction.
template <typename ST> struct Half16;
template <> struct Half16<bf16> {
  static constexpr bool GELU_TABLE = true;
  static __device__ __forceinline__ uint32_t pack2(float lo, float hi) { return pack_bf16x2(lo, hi); }
  static __device__ __forceinline__ float lo(uint32_t u) { return __uint_as_float(u << 16); }
  static __device__ __forceinline__ float hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
  static __device__ __forceinline__ f32x4 mfma(const bf16x8& a, const bf16x8& b, const f32x4& c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
  }
};
template <> struct Half16<f16> {
  static constexpr bool GELU_TABLE = false;
  static __device__ __forceinline__ uint32_t pack2(float lo, float hi) { return pack_f16x2(lo, hi); }
  static __device__ __forceinline__ float lo(uint32_t u) { return f16_bits_to_f32(u & 0xffffu); }
  static __device__ __forceinline__ float hi(uint32_t u) { return f16_bits_to_f32(u >> 16); }
  static __device__ __forceinline__ f32x4 mfma(const bf16x8& a, const bf16x8& b, const f32x4& c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  }
};

constexpr int BKT = 64;   // K values per LDS stage: two MFMA K steps; an operand row with contiguous K is one 128-byte line
constexpr int NBUF = 2;   // LDS stages

// ---- LDS layouts -------------------------------------------------------------------------------
// K-contiguous tile: [rows][BKT] bf16.  The 16-byte chunks of a row are XOR-swizzled with the index
// of the 256-byte LDS line the row lies in, so 16 lanes reading the same chunk of 16 consecutive
// rows hit 16 distinct 16-byte bank groups (the LDS serves 64 banks x 4 bytes per clock).
__device__ __forceinline__ int kc_off(int row, int chunk) {
  constexpr int CPR = BKT / 8, RP = 256 / (BKT * 2);
  return row * (BKT * 2) + ((chunk ^ ((row / RP) & (CPR - 1))) << 4);
}
// K-strided tile: [BKT][W] bf16; the 64-byte granules of a K row are XOR-swizzled with k%4, so the four
// K rows that one 16-lane block of a transposing read touches fall into different bank groups, and the
// 32-byte halves of a granule with (k/8)%2, which separates two blocks that read the same columns eight K
// rows apart (counters: no bank conflicts).
template <int W>
__device__ __forceinline__ int ks_off(int krow, int col_byte) {
  return krow * (W * 2) + (col_byte ^ (((krow & 3) << 6) | (((krow >> 3) & 1) << 5)));
}

// Fragment reads.  The eight K values of one lane (column l%16, K chunk l/16 of the step) of a K-strided
// tile come from two transposing reads: the instruction works on blocks of 16 lanes, lane s of a block
// reads 8 bytes at (K row s/4, columns 4*(s%4)..+3) and receives the four K rows of column s; the second
// read lies four K rows further on.  `p` is the lane's address of the first read.
template <int W>
__device__ __forceinline__ bf16x8 lds_read_ks2(const char* p) {
  typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * W * 2));
  union { struct { s16x4 a, b; } q; bf16x8 v; } u;
  u.q.a = lo;
  u.q.b = hi;
  return u.v;
}

// ---- global -> LDS loads of one stage ------------------------------------------------------------
// Global loads are raw buffer loads: the descriptor's byte count is set to the part of the operand
// this tile may read, and the hardware returns zero for anything past it.  That gives the ragged
// edges (rows past an expert's share, K rows past the share in the weight-gradient GEMM, columns past
// the matrix) for free, with no predicates, no branches and one 32-bit offset register per load.
typedef __attribute__((address_space(3))) char lds_char;
__device__ __forceinline__ unsigned lds_addr(const char* p) { return (unsigned)(uintptr_t)(const lds_char*)p; }
typedef u32x4 rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, size_t bytes) {
  const unsigned long long a = (unsigned long long)base;
  const unsigned n = bytes > 0xffffffffull ? 0xffffffffu : (unsigned)bytes;
  // raw buffer: base address, stride 0, byte count, 32-bit untyped data format
  return rsrc_t{(unsigned)a, (unsigned)(a >> 32) & 0xffffu, n, 0x00020000u};
}

// 16 bytes per lane from a buffer straight into LDS: lane l of the wave lands at LDS byte address
// lds + 16*l (lds is wave-uniform; the instruction takes it from M0).  Completion is tracked by
// vmcnt like any other buffer load.  Written as a raw instruction on purpose: the compiler must not
// know that this load writes LDS, or it waits for every outstanding load before each LDS read it
// cannot prove disjoint (the transposing reads).  The pipeline orders loads and reads itself with
// explicit vmcnt waits and block barriers; the memory clobber keeps LDS reads from moving across.
__device__ __forceinline__ void load_to_lds16(rsrc_t rs, unsigned lds, unsigned voffset) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
               :: "s"(lds), "v"(voffset), "s"(rs) : "memory", "m0");
}

// One operand tile of one stage, cut into 16-byte chunks; thread tid moves chunks tid + NT*i.
// KC: [ROWS][BKT], chunk id -> (row id/CPR, chunk id%CPR).
// KS: [BKT][ROWS] (ROWS = tile width), chunk id -> (K row id/(ROWS/8), chunk id%(ROWS/8)).
template <bool KC, int ROWS, int NT>
struct Stage {
  static constexpr int CPR = KC ? BKT / 8 : ROWS / 8;
  static constexpr int CH = ROWS * BKT / 8 / NT;
  static_assert(CH >= 1, "tile too small for this many threads");
  // A direct load places lane l of a wave at byte 16*l of the instruction's LDS window, so chunk id
  // lands at byte 16*id of the tile; this is the operand byte offset (pitch in bytes) whose data
  // belongs there: the tile's swizzle, inverted.
  static __device__ __forceinline__ unsigned goff(int i, int tid, unsigned pitch) {
    const int id = tid + NT * i, r = id / CPR, pc = id % CPR;
    if constexpr (KC) {
      constexpr int RP = 256 / (BKT * 2);
      return (unsigned)r * pitch + (unsigned)(pc ^ ((r / RP) & (CPR - 1))) * 16u;
    } else {
      return (unsigned)r * pitch + (unsigned)(pc ^ (((r & 3) << 2) | (((r >> 3) & 1) << 1))) * 16u;
    }
  }
};

// ---- fast activation pieces for bf16 outputs ----------------------------------------------------
__device__ __forceinline__ float sigmoid_fast(float g) {
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(g * -1.44269504088896340736f));
}

// Row-layout epilogue on four consecutive columns starting at flat index idx (bf16 tensors).
// Entry of the LDS copy of a GELU table (layout: gemm.h) for the bf16 number with bit pattern `bits`.
__device__ __forceinline__ float gelu_tab_lookup(const float* tab, uint32_t bits) {
  const int m = min(max((int)(bits & 0x7fffu) - (GELU_TAB_EXP0 << 7), 0), GELU_TAB_NMAG - 1);
  return tab[m + (int)(bits >> 15) * GELU_TAB_NMAG];
}

template <typename ST, int EPI>
__device__ __forceinline__ void epilogue4(const GemmArgs& g, size_t idx, const f32x4& a, const f32x4& a2,
                                          const u32x2& sv1, const u32x2& sv2, const float* tab) {
  typedef Half16<ST> H;
  auto st = [](void* base, size_t i, float v0, float v1, float v2, float v3) {
    // outputs are written once and read by a later launch: streaming stores keep them from displacing operand
    // panels in the L2 (measured: dH -1.3 %, the GELU workloads -0.4 to -1.5 % per step; the SwiGLU forward with
    // its three stores per element is 1 % faster with plain ones)
    const u32x2 v = u32x2{H::pack2(v0, v1), H::pack2(v2, v3)};
    u32x2* p = reinterpret_cast<u32x2*>(reinterpret_cast<ST*>(base) + i);
    if constexpr (EPI == EPI_SWIGLU_FWD) *p = v; else __builtin_nontemporal_store(v, p);
  };
  auto ld = [](const u32x2& r, float* f) {   // four saved 16-bit values, loaded by the caller ahead of time
    f[0] = H::lo(r.x); f[1] = H::hi(r.x);
    f[2] = H::lo(r.y); f[3] = H::hi(r.y);
  };
  if constexpr (EPI == EPI_STORE) {
    st(g.C, idx, a[0], a[1], a[2], a[3]);
  } else if constexpr (EPI == EPI_GELU_FWD) {
    // h = a Phi(v), v = the pre-activation as stored: GELU of the saved tensor; Phi looked up (bf16) or evaluated (fp16)
    const uint32_t p0 = H::pack2(a[0], a[1]), p1 = H::pack2(a[2], a[3]);
    if (g.C != nullptr) __builtin_nontemporal_store(u32x2{p0, p1}, reinterpret_cast<u32x2*>(reinterpret_cast<ST*>(g.C) + idx));   // NULL: only H is kept
    if constexpr (H::GELU_TABLE) {
      st(g.C2, idx, a[0] * gelu_tab_lookup(tab, p0 & 0xffffu), a[1] * gelu_tab_lookup(tab, p0 >> 16),
         a[2] * gelu_tab_lookup(tab, p1 & 0xffffu), a[3] * gelu_tab_lookup(tab, p1 >> 16));
    } else {
      st(g.C2, idx, a[0] * phi_fast(H::lo(p0)), a[1] * phi_fast(H::hi(p0)), a[2] * phi_fast(H::lo(p1)), a[3] * phi_fast(H::hi(p1)));
    }
  } else if constexpr (EPI == EPI_SWIGLU_FWD) {
    if (g.C != nullptr) {   // NULL: only H is kept
      st(g.C, idx, a[0], a[1], a[2], a[3]);
      st(g.C2, idx, a2[0], a2[1], a2[2], a2[3]);
    }
    float h[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) h[i] = a[i] * sigmoid_fast(a[i]) * a2[i];
    st(g.C3, idx, h[0], h[1], h[2], h[3]);
  } else if constexpr (EPI == EPI_GELU_BWD) {
    // the derivative at the saved pre-activation: looked up (bf16) or evaluated (fp16)
    float o0, o1, o2, o3;
    if constexpr (H::GELU_TABLE) {
      o0 = a[0] * gelu_tab_lookup(tab, sv1.x & 0xffffu); o1 = a[1] * gelu_tab_lookup(tab, sv1.x >> 16);
      o2 = a[2] * gelu_tab_lookup(tab, sv1.y & 0xffffu); o3 = a[3] * gelu_tab_lookup(tab, sv1.y >> 16);
    } else {
      o0 = a[0] * gelu_grad_fast(H::lo(sv1.x)); o1 = a[1] * gelu_grad_fast(H::hi(sv1.x));
      o2 = a[2] * gelu_grad_fast(H::lo(sv1.y)); o3 = a[3] * gelu_grad_fast(H::hi(sv1.y));
    }
    st(g.C, idx, o0, o1, o2, o3);
  } else if constexpr (EPI == EPI_SWIGLU_BWD) {
    float gg[4], uu[4], dg[4], du[4];
    ld(sv1, gg);
    ld(sv2, uu);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float sg = sigmoid_fast(gg[i]);
      dg[i] = a[i] * uu[i] * sg * fmaf(gg[i], 1.f - sg, 1.f);
      du[i] = a[i] * gg[i] * sg;
    }
    st(g.C, idx, dg[0], dg[1], dg[2], dg[3]);
    st(g.C2, idx, du[0], du[1], du[2], du[3]);
  }
}

template <int BM, int BN, bool DUAL>
constexpr int gemm_bf16_stage_bytes() { return BM * BKT * 2 + BN * BKT * 2 * (DUAL ? 2 : 1); }
// TAB: a GELU table sits behind the ring (the GELU epilogues)
template <int BM, int BN, bool DUAL, int WGM, int WGN, bool TAB = false>
constexpr int gemm_bf16_lds_bytes() {
  constexpr int ring = NBUF * gemm_bf16_stage_bytes<BM, BN, DUAL>();
  constexpr int slab = WGM * WGN * 32 * (BN / WGN + 8) * 4;   // epilogue: one 32-row fp32 slab per wave
  return (ring > slab ? ring : slab) + (TAB ? GELU_TAB_FLOATS * 4 : 0);
}

// One output tile; vb = the tile's number in dispatch order.  Block-uniform control flow; returns at
// once for numbers past the last tile (the grid is sized for the worst case).
template <typename ST, int MODE, int EPI, bool DUAL, bool CHAIN, int BM, int BN, int WGM, int WGN>
__device__ __forceinline__ void gemm_bf16_tile(const GemmArgs& g, const int vb, char* smem) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int WTM = BM / WGM / 32, WTN = BN / WGN / 32;
  constexpr int KS = BKT / 32;               // MFMA K steps per stage
  constexpr int TM = 2 * WTM, TNN = 2 * WTN; // 16 x 16 MFMA tiles of a wave
  constexpr bool A_KC = (MODE != MODE_TN);   // A stored with K contiguous
  constexpr bool B_KC = (MODE == MODE_NT);
  constexpr int A_BYTES = BM * BKT * 2, B_BYTES = BN * BKT * 2;
  constexpr int STAGE = gemm_bf16_stage_bytes<BM, BN, DUAL>();
  static_assert(KS == 2 && NBUF == 2, "the pipeline below: two stages of two K steps");

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps wave-dependent values scalar
  const int wm = wave / WGN, wn = wave % WGN;

  int e, row0, mvalid, klen, m0 = 0, n0;
  int split_tile = -1, ksplit = 0, kbase = 0;   // >= 0: this block computes one K part of a split row tile
  {
    const int ntn = (g.N + BN - 1) / BN;
    int rt, nt;
    if constexpr (MODE == MODE_TN) {
      // Weight gradients: tile (expert, m tile, n tile) costs its expert's row count.  Every expert's
      // tiles are split evenly over the XCDs (block b runs on XCD b % 8), so a skewed load is even across
      // XCDs; experts start in order of descending row count.  An XCD's share of an expert is a contiguous
      // range of the expert's tiles in patch order (four m tiles at a time, column by column), so the 32
      // tiles it runs together form a 4 x 8 patch that needs 12 operand panels per K stage from its L2
      // instead of up to 18 with the tiles dealt one by one (that order made dW2 of the Mixtral-like shape
      // read 6.9 times its operands through the fabric).
      const int ntm = (g.M + BM - 1) / BM;
      int slot, mt;
      if (!dw_block(vb, ntm, ntn, slot, mt, nt)) return;
      e = g.order[slot];
      m0 = mt * BM;
      rt = 0;
      int l, h;
      share_of(g.lo, g.hi, g.kept[e], e, l, h);
      row0 = g.offsets[e] + l;
      klen = h - l;
      mvalid = min(BM, g.M - m0);
      if (klen == 0 && g.accumulate) return;
    } else {
      constexpr bool CAN_SPLIT = (EPI == EPI_STORE && !CHAIN);
      const int n_rt = g.ntiles[0];
      // split-K (gemm.h): the last n_sp row tiles are not part of the regular numbering; their blocks
      // follow it, SPLIT_K per (row tile, column tile), each with a K range of its own
      const int n_sp = (CAN_SPLIT && g.split_ws != nullptr) ? g.ntiles[2] : 0;
      RowBlock rb;
      if (!row_tile_block(vb, n_rt, g.ntiles[1], n_sp, ntn, rb)) return;
      rt = rb.rt;
      nt = rb.nt;
      klen = g.K;
      if (rb.split_tile >= 0) {
        split_tile = rb.split_tile;
        ksplit = rb.ksplit;
        klen = g.K / SPLIT_K;
        kbase = ksplit * klen;
      }
      const RowTile t = g.tiles[rt];
      e = t.e;
      row0 = t.row0;
      mvalid = t.nrows;
    }
    n0 = nt * BN;
  }
  const int nvalid = min(BN, g.N - n0);

  f32x4 acc[TM][TNN], acc2[DUAL ? TM : 1][DUAL ? TNN : 1];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TNN; ++j) {
      acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
      if constexpr (DUAL) acc2[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

  const int KT = (klen + BKT - 1) / BKT;
  // MFMA row bands of this wave that contain valid rows
  // (row band b of the tile belongs to wave row b % WGM, as its band b / WGM: a partly filled tile then
  // spreads its valid bands over all wave rows instead of loading the first ones only)
  const int ni = (MODE == MODE_TN) ? WTM : min(max(((mvalid + 31) / 32 - wm + WGM - 1) / WGM, 0), WTM);
  typedef Stage<A_KC, BM, NT> StA;
  typedef Stage<B_KC, BN, NT> StB;

  // fragment read offsets inside a stage.  Lane l of a 16 x 16 x 32 MFMA holds row (column) l % 16 and the
  // eight K values of chunk l / 16.  K-contiguous: one offset per K step (MFMA tiles are a constant 16 rows
  // apart); K-strided: one per MFMA tile (K steps are a constant apart).
  int a_fr[A_KC ? KS : TM], b_fr[B_KC ? KS : TNN];
  if constexpr (A_KC) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) a_fr[ks] = kc_off(wm * 32 + (lane & 15), ks * 4 + (lane >> 4));
  } else {
#pragma unroll
    for (int i = 0; i < TM; ++i)
      a_fr[i] = ks_off<BM>((lane >> 4) * 8 + ((lane & 15) >> 2),
                           (((i >> 1) * WGM + wm) * 32 + (i & 1) * 16 + (lane & 3) * 4) * 2);
  }
  if constexpr (B_KC) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      b_fr[ks] = A_BYTES + kc_off(wn * WTN * 32 + (lane & 15), ks * 4 + (lane >> 4));
  } else {
#pragma unroll
    for (int j = 0; j < TNN; ++j)
      b_fr[j] = A_BYTES + ks_off<BN>((lane >> 4) * 8 + ((lane & 15) >> 2),
                                     (wn * WTN * 32 + j * 16 + (lane & 3) * 4) * 2);
  }

  {
    // operand bases of this tile (a chained GEMM has two operand pairs and runs their K ranges back to
    // back through one pipeline), byte counts the tile may read, pitches and the advance per K stage
    const bf16* A0 = reinterpret_cast<const bf16*>(g.A);
    const bf16* A1 = reinterpret_cast<const bf16*>(CHAIN ? g.A2 : g.A);
    const bf16* B0 = reinterpret_cast<const bf16*>(g.B);
    const bf16* B1 = reinterpret_cast<const bf16*>(g.B2);   // SwiGLU: second weight matrix
    size_t aoff, boff, abytes, bbytes;
    unsigned pa, pb, astep, bstep;
    if constexpr (MODE == MODE_TN) {
      // A = [rows][M] from (row0, m0), B = [rows][N] from (row0, n0); rows past the share read as zero
      aoff = (size_t)row0 * g.M + m0;  abytes = ((size_t)klen * g.M - m0) * 2;
      boff = (size_t)row0 * g.N + n0;  bbytes = ((size_t)klen * g.N - n0) * 2;
      pa = g.M * 2; pb = g.N * 2; astep = BKT * pa; bstep = BKT * pb;
    } else if constexpr (MODE == MODE_NN) {
      // A = [rows][K] rows row0..row0+mvalid; B = W_e [K][N] from column n0; both from K index kbase on
      aoff = (size_t)row0 * g.K + kbase;  abytes = ((size_t)mvalid * g.K - kbase) * 2;
      boff = ((size_t)e * g.K + kbase) * g.N + n0;  bbytes = ((size_t)(g.K - kbase) * g.N - n0) * 2;
      pa = g.K * 2; pb = g.N * 2; astep = BKT * 2; bstep = BKT * pb;
    } else {
      // A as above; B = W_e [N][K] rows n0..N
      aoff = (size_t)row0 * g.K + kbase;  abytes = ((size_t)mvalid * g.K - kbase) * 2;
      boff = ((size_t)e * g.N + n0) * g.K + kbase;  bbytes = ((size_t)(g.N - n0) * g.K - kbase) * 2;
      pa = g.K * 2; pb = g.K * 2; astep = BKT * 2; bstep = BKT * 2;
    }
    const rsrc_t ra = make_rsrc(A0 + aoff, abytes), ra1 = make_rsrc(A1 + aoff, abytes);
    const rsrc_t rb = make_rsrc(B0 + boff, bbytes), rb1 = make_rsrc(B1 + boff, bbytes);
    const int KT1 = KT;                      // stages of one operand pair
    const int KTT = CHAIN ? 2 * KT1 : KT1;   // stages in all
    // Iteration kt issues the loads of stage kt+D, multiplies stage kt (reading the fragments of stage
    // kt+1 meanwhile), then waits until its own loads of stage kt+2 have landed (all but the newest D-2
    // stages) and joins the block barrier, after which stage kt+2 is visible to every wave and stage
    // kt's buffer may be overwritten.
    constexpr int L = StA::CH + StB::CH * (DUAL ? 2 : 1);   // loads per thread per stage
    constexpr int PEND = L;                                  // loads that may stay in flight at the prologue's barrier: stage 1
    static_assert(PEND < 64, "the wait counter has six bits");
    constexpr int WAIT_L = (PEND & 15) | ((PEND >> 4) << 14) | 0x70 | (15 << 8);   // s_waitcnt vmcnt(PEND) only
    constexpr int WAIT_0 = 0x70 | (15 << 8);                                       // s_waitcnt vmcnt(0) only
    constexpr int WAIT_LGKM0 = 0xC07F;                                             // s_waitcnt lgkmcnt(0) only
    unsigned a_vo[StA::CH], b_vo[StB::CH];
#pragma unroll
    for (int i = 0; i < StA::CH; ++i) a_vo[i] = StA::goff(i, tid, pa);
#pragma unroll
    for (int i = 0; i < StB::CH; ++i) b_vo[i] = StB::goff(i, tid, pb);
    const int wbase = wave * 1024;   // a wave's 64 lanes fill 1 KB of the tile per load
    const unsigned smem_base = lds_addr(smem);
    // A K step is the 32 K values of one MFMA: TM x TNN instructions per wave, cut into TM regions that the
    // scheduler may not move instructions across (sched_barrier).  Region i holds the MFMAs of row tile i;
    // behind them, the read of row tile i's A fragment for the NEXT K step, into the same registers (their
    // last use has just been issued, and the fragment is not needed for another TM - 1 regions), in the
    // first TNN regions one B fragment of the next step (into the other of two B register sets), and this
    // region's share of the global -> LDS loads.  LDS reads and, above all, the global loads then arrive as a
    // steady trickle: loads issued in one burst fill the address FIFO of the memory pipe, and a wave that
    // cannot issue a load cannot issue the MFMAs behind it either.
    constexpr int NR = TM;                           // regions per K step
    bf16x8 af[TM], bfr[2][TNN], bfr2[2][DUAL ? TNN : 1];
#define MOE_LOAD(kt_, buf_)                                                                                 \
  do {                                                                                                      \
    _Pragma("unroll") for (int q__ = 0; q__ < L; ++q__) MOE_LOAD1(kt_, buf_, q__);                          \
  } while (0)
// load q_ (0 .. L-1) of a stage: the A chunks, then the B chunks (DUAL: both weight matrices in turn)
#define MOE_LOAD1(kt_, buf_, q_)                                                                            \
  do {                                                                                                      \
    const int kq__ = (kt_);                                                                                 \
    const bool sec__ = CHAIN && kq__ >= KT1;                                                                \
    const unsigned kl__ = (unsigned)(sec__ ? kq__ - KT1 : kq__);                                            \
    const unsigned st__ = smem_base + (buf_) + wbase;                                                       \
    if ((q_) < StA::CH) {                                                                                   \
      load_to_lds16(sec__ ? ra1 : ra, st__ + NT * 16 * (q_), a_vo[(q_) < StA::CH ? (q_) : 0] + kl__ * astep); \
    } else {                                                                                                \
      const int c__ = ((q_) - StA::CH) / (DUAL ? 2 : 1) % StB::CH;                                          \
      if (!DUAL || ((q_) - StA::CH) % 2 == 0)                                                               \
        load_to_lds16(sec__ ? rb1 : rb, st__ + A_BYTES + NT * 16 * c__, b_vo[c__] + kl__ * bstep);          \
      else                                                                                                  \
        load_to_lds16(rb1, st__ + A_BYTES + B_BYTES + NT * 16 * c__, b_vo[c__] + kl__ * bstep);             \
    }                                                                                                       \
  } while (0)
// A fragment of row tile i_ / B fragment(s) of column tile j_ for K step ks_ of the stage at buf_
#define MOE_FRAG_A(i_, buf_, ks_)                                                                           \
  do {                                                                                                      \
    const char* st__ = smem + (buf_);                                                                       \
    if constexpr (A_KC)                                                                                     \
      af[i_] = *reinterpret_cast<const bf16x8*>(st__ + a_fr[ks_] + ((i_) >> 1) * WGM * 32 * BKT * 2 + ((i_) & 1) * 16 * BKT * 2); \
    else af[i_] = lds_read_ks2<BM>(st__ + a_fr[i_] + (ks_) * 32 * BM * 2);                                  \
  } while (0)
#define MOE_FRAG_B(set_, j_, buf_, ks_)                                                                     \
  do {                                                                                                      \
    const char* st__ = smem + (buf_);                                                                       \
    if constexpr (B_KC) bfr[set_][j_] = *reinterpret_cast<const bf16x8*>(st__ + b_fr[ks_] + (j_) * 16 * BKT * 2); \
    else bfr[set_][j_] = lds_read_ks2<BN>(st__ + b_fr[j_] + (ks_) * 32 * BN * 2);                           \
    if constexpr (DUAL) bfr2[set_][j_] = lds_read_ks2<BN>(st__ + B_BYTES + b_fr[j_] + (ks_) * 32 * BN * 2); \
  } while (0)
#define MOE_FRAGS(set_, buf_, ks_)                                                                          \
  do {                                                                                                      \
    _Pragma("unroll") for (int i__ = 0; i__ < TM; ++i__) MOE_FRAG_A(i__, buf_, ks_);                        \
    _Pragma("unroll") for (int j__ = 0; j__ < TNN; ++j__) MOE_FRAG_B(set_, j__, buf_, ks_);                 \
  } while (0)
// One K step on B register set set_; DO_NEXT_: read the fragments of K step rks_ of the stage at rbuf_;
// DO_LOAD_: issue the loads LQ0_ .. LQ0_+LQN_-1 of stage lkt_ into the buffer at lbuf_.
#define MOE_STEP(set_, DO_NEXT_, rbuf_, rks_, DO_LOAD_, lkt_, lbuf_, LQ0_, LQN_, NI_)                       \
  do {                                                                                                      \
    _Pragma("unroll") for (int r__ = 0; r__ < NR; ++r__) {                                                  \
      if ((r__ >> 1) < (NI_)) {                                                                             \
        _Pragma("unroll") for (int j__ = 0; j__ < TNN; ++j__) {                                             \
          acc[r__][j__] = Half16<ST>::mfma(af[r__], bfr[set_][j__], acc[r__][j__]);                         \
          if constexpr (DUAL) acc2[r__][j__] = Half16<ST>::mfma(af[r__], bfr2[set_][j__], acc2[r__][j__]);  \
        }                                                                                                   \
      }                                                                                                     \
      if (DO_NEXT_) {                                                                                       \
        MOE_FRAG_A(r__, rbuf_, rks_);                                                                       \
        if (r__ < TNN) MOE_FRAG_B((set_) ^ 1, r__ < TNN ? r__ : 0, rbuf_, rks_);                            \
      }                                                                                                     \
      if (DO_LOAD_) {                                                                                       \
        _Pragma("unroll") for (int q__ = 0; q__ < (LQN_); ++q__)                                            \
          if (q__ * NR / ((LQN_) > 0 ? (LQN_) : 1) == r__) MOE_LOAD1(lkt_, lbuf_, (LQ0_) + q__);            \
      }                                                                                                     \
      __builtin_amdgcn_sched_barrier(0);                                                                    \
    }                                                                                                       \
  } while (0)
#define MOE_BLOCK_BARRIER()                                                                                 \
  do {                                                                                                      \
    asm volatile("" ::: "memory");                                                                          \
    __builtin_amdgcn_s_barrier();                                                                           \
    asm volatile("" ::: "memory");                                                                          \
  } while (0)
    if constexpr ((EPI == EPI_GELU_BWD || EPI == EPI_GELU_FWD) && Half16<ST>::GELU_TABLE) {
      // the GELU table rides along with the first stage loads (older than they are, so the
      // first wait of the pipeline covers it): 1 KB per wave and instruction, behind the ring
      static_assert(GELU_TAB_FLOATS * 4 % (NT * 16) == 0, "whole block-wide loads");
      const rsrc_t rt = make_rsrc(g.gelu_tab, (size_t)GELU_TAB_FLOATS * 4);
#pragma unroll
      for (int i = 0; i < GELU_TAB_FLOATS * 4 / (NT * 16); ++i)
        load_to_lds16(rt, smem_base + NBUF * STAGE + i * NT * 16 + wbase, (unsigned)(i * NT + tid) * 16u);
    }
    {
      // Iteration S multiplies stage S (two K steps) out of buffer S % 2.  K step 0 reads the fragments of
      // K step 1; then every wave waits for its own loads of stage S+1 and for its fragment reads and joins
      // the one block barrier of the iteration, after which stage S+1 is visible to all and nobody reads
      // buffer S % 2 again; K step 1 reads the fragments of step 0 of stage S+1 and issues the loads of
      // stage S+2 into buffer S % 2 (they have about a stage's worth of MFMAs to land).
#define MOE_ITER(S_, DO_NEXT_, DO_LOAD_, NI_)                                                                \
  do {                                                                                                      \
    MOE_STEP(0, true, b0, 1, false, 0, 0, 0, 0, NI_);                                                       \
    if (DO_NEXT_) {                                                                                         \
      __builtin_amdgcn_s_waitcnt(0);   /* vmcnt(0) lgkmcnt(0): own loads of stage S+1, own reads of stage S */ \
      MOE_BLOCK_BARRIER();                                                                                  \
    }                                                                                                       \
    MOE_STEP(1, DO_NEXT_, b1, 0, DO_LOAD_, (S_) + 2, b0, 0, L, NI_);                                        \
    { const int t__ = b0; b0 = b1; b1 = t__; }                                                              \
  } while (0)
      if (KTT > 0) {
        int b0 = 0, b1 = STAGE;
        MOE_LOAD(0, 0);
        if (KTT > 1) {
          MOE_LOAD(1, STAGE);
          __builtin_amdgcn_s_waitcnt(WAIT_L);   // stage 0 (and the table) have landed, stage 1 may be in flight
        } else {
          __builtin_amdgcn_s_waitcnt(WAIT_0);
        }
        MOE_BLOCK_BARRIER();
#define MOE_MAINLOOP(NI_)                                                                        \
  do {                                                                                          \
    MOE_FRAGS(0, b0, 0);                                                                        \
    __builtin_amdgcn_s_waitcnt(WAIT_LGKM0);   /* nothing pending at the loop head: the waits inside the loop then count only its own reads */ \
    int S = 0;                                                                                  \
    _Pragma("unroll 1") for (; S + 2 < KTT; ++S) MOE_ITER(S, true, true, NI_);                   \
    _Pragma("unroll 1") for (; S < KTT; ++S) MOE_ITER(S, S + 1 < KTT, S + 2 < KTT, NI_);         \
  } while (0)
        if (ni == WTM) MOE_MAINLOOP(WTM);
        else MOE_MAINLOOP(ni);
#undef MOE_MAINLOOP
        // the epilogue's slabs reuse the ring: every wave must be done reading fragments first
        __builtin_amdgcn_s_waitcnt(0);
        MOE_BLOCK_BARRIER();
      }
#undef MOE_ITER
    }
#undef MOE_LOAD
#undef MOE_LOAD1
#undef MOE_FRAG_A
#undef MOE_FRAG_B
#undef MOE_FRAGS
#undef MOE_STEP
#undef MOE_BLOCK_BARRIER
  }

  {
    // per-wave slab [32][WTN*32 + 4] fp32 (the stages are free: the loop ended with a block barrier)
    constexpr int C = WTN * 32, P = C + 4, LPR = C / 4, RPP = 64 / LPR, PASSES = 32 / RPP;
    float* slab = reinterpret_cast<float*>(smem) + wave * (32 * P);
    const int rr = lane / LPR, c4 = lane % LPR;
    constexpr bool NEED_S1 = (EPI == EPI_GELU_BWD || EPI == EPI_SWIGLU_BWD), NEED_S2 = (EPI == EPI_SWIGLU_BWD);
    const float* tab_lds = reinterpret_cast<const float*>(smem + NBUF * STAGE);
    // Saved tensors the backward epilogues read: the loads of a band are issued one band ahead (those of
    // the first band before anything else), so their latency hides behind the previous band's LDS round
    // trip and arithmetic (rows past the tile read the tile's first row and are dropped).
    u32x2 s1[NEED_S1 ? 2 : 1][NEED_S1 ? PASSES : 1], s2[NEED_S2 ? 2 : 1][NEED_S2 ? PASSES : 1];
    auto load_saved = [&](int band, u32x2* d1, u32x2* d2) {
#pragma unroll
      for (int p = 0; p < PASSES; ++p) {
        const int m = (band * WGM + wm) * 32 + p * RPP + rr, n = wn * C + c4 * 4;
        const bool ok = m < mvalid && n < nvalid;
        const size_t idx = (size_t)(row0 + (ok ? m : 0)) * g.N + n0 + (ok ? n : 0);
        d1[p] = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(reinterpret_cast<const bf16*>(g.S1) + idx));
        if constexpr (NEED_S2) d2[p] = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(reinterpret_cast<const bf16*>(g.S2) + idx));
      }
    };
    if constexpr (NEED_S1) load_saved(0, s1[0], s2[0]);
#pragma unroll
    for (int i = 0; i < WTM; ++i) {
      f32x4 va[PASSES], vb[DUAL ? PASSES : 1];
      if constexpr (NEED_S1) {
        if (i + 1 < WTM) load_saved(i + 1, s1[(i + 1) & 1], s2[NEED_S2 ? (i + 1) & 1 : 0]);
      }
#pragma unroll
      for (int half = 0; half < (DUAL ? 2 : 1); ++half) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int j = 0; j < TNN; ++j)
#pragma unroll
          for (int v = 0; v < 8; ++v) {   // lane l of a 16 x 16 tile: column l % 16, rows 4 (l / 16) .. + 3
            const int i2 = v >> 2, r = i2 * 16 + (lane >> 4) * 4 + (v & 3);
            slab[r * P + j * 16 + (lane & 15)] =
                (half == 0) ? acc[2 * i + i2][j][v & 3] : acc2[DUAL ? 2 * i + i2 : 0][DUAL ? j : 0][v & 3];
          }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
          const f32x4 t = *reinterpret_cast<const f32x4*>(slab + (p * RPP + rr) * P + c4 * 4);
          if (half == 0) va[p] = t; else vb[DUAL ? p : 0] = t;
        }
      }
#pragma unroll
      for (int p = 0; p < PASSES; ++p) {
        const int m = (i * WGM + wm) * 32 + p * RPP + rr;
        const int n = wn * C + c4 * 4;
        if (m < mvalid && n < nvalid) {
          if (MODE != MODE_TN && split_tile >= 0) {   // fp32 partial sum of this block's K part
            *reinterpret_cast<f32x4*>(g.split_ws + (((size_t)split_tile * SPLIT_K + ksplit) * SPLIT_ROWS + m) * g.N + n0 + n) = va[p];
          } else if constexpr (MODE == MODE_TN) {   // fp32 weight gradient of expert e, 16 bytes per lane
            f32x4* c = reinterpret_cast<f32x4*>(reinterpret_cast<float*>(g.C) + ((size_t)e * g.M + m0 + m) * g.N + n0 + n);
            if (g.accumulate) *c = *c + va[p]; else __builtin_nontemporal_store(va[p], c);
          } else {
            epilogue4<ST, EPI>(g, (size_t)(row0 + m) * g.N + n0 + n, va[p], vb[DUAL ? p : 0],
                           s1[NEED_S1 ? i & 1 : 0][NEED_S1 ? p : 0], s2[NEED_S2 ? i & 1 : 0][NEED_S2 ? p : 0], tab_lds);
          }
        }
      }
    }
  }
}

// Second half of split-K: C[row][n..n+3] = sum over the SPLIT_K parts, in part order, of the fp32 partial
// sums of split row tile blockIdx.y; a thread owns four adjacent columns of one row.
template <typename ST>
__global__ __launch_bounds__(256) void split_reduce_kernel(GemmArgs g) {
  const int n_sp = g.ntiles[2], st = blockIdx.y;
  if (st >= n_sp) return;
  const RowTile t = g.tiles[g.ntiles[0] - n_sp + st];
  const int per_row = g.N / 4, i = blockIdx.x * 256 + threadIdx.x;
  const int m = i / per_row, n = (i % per_row) * 4;
  if (m >= t.nrows) return;
  f32x4 sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int ks = 0; ks < SPLIT_K; ++ks)
    sum += *reinterpret_cast<const f32x4*>(g.split_ws + (((size_t)st * SPLIT_K + ks) * SPLIT_ROWS + m) * g.N + n);
  *reinterpret_cast<u32x2*>(reinterpret_cast<ST*>(g.C) + (size_t)(t.row0 + m) * g.N + n) =
      u32x2{Half16<ST>::pack2(sum[0], sum[1]), Half16<ST>::pack2(sum[2], sum[3])};
}

template <typename ST, int MODE, int EPI, bool DUAL, bool CHAIN, int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(WGM* WGN * 64, 1) void gemm_bf16_kernel(GemmArgs g) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  gemm_bf16_tile<ST, MODE, EPI, DUAL, CHAIN, BM, BN, WGM, WGN>(g, blockIdx.x, smem);
}

// Two independent GEMMs in one launch: blocks below `first_blocks` take a tile of the first, the others a
// tile of the second.  Blocks are dispatched in order, so the second GEMM's tiles start on the compute
// units that the first one's last, partly filled round leaves idle (no stream or event in between,
// and the two never compete for the cache from the start as two concurrent kernels would).
template <typename ST, int MODE1, int EPI1, bool CHAIN1, int MODE2, int EPI2, int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(WGM* WGN * 64, 1) void gemm_bf16_pair_kernel(GemmArgs g1, GemmArgs g2, int first_blocks) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  if ((int)blockIdx.x < first_blocks)
    gemm_bf16_tile<ST, MODE1, EPI1, false, CHAIN1, BM, BN, WGM, WGN>(g1, blockIdx.x, smem);
  else
    gemm_bf16_tile<ST, MODE2, EPI2, false, false, BM, BN, WGM, WGN>(g2, blockIdx.x - first_blocks, smem);
}

inline unsigned gemm_bf16_grid(long long tiles) { return (unsigned)(tiles > 0 ? tiles : 1); }

}  // namespace moe

// Score block, softmax and its two gradient contractions on the matrix cores (gfx950).
//
// For one chunk and one corrupted side the positives' operands Q (n_e x d) meet the chunk's
// shared negatives K (N x d): scores A = Q K^T (Sec. 2.1: every edge against the sampled
// negatives), log-sum-exp per edge (Eq. 1's log term), and with P = softmax rows
//     gQ = P K   (gradient w.r.t. the edge-side operand)        -- k_flash, online softmax
//     gK = P^T Q (gradient w.r.t. the negatives' rows)          -- k_flash_bwd, needs the final lse
// k_flash: a wave owns 16 stationary rows x of Q whose fragments stay in registers, and streams
// tiles of K through LDS:
//     T[y][x]   = sum_k K[y][k] Q[x][k]              v_mfma_f32_16x16x4_f32, lane <-> x
//     W[y][x]   = exp(T - reference[x])              in the accumulator registers
//     O^T[c][x] += sum_y K[y][c] W[y][x]             the accumulator layout of T is exactly the
//                                                    B-operand layout the second product needs
// so every per-x quantity (reference, running sum, rescale factor) is per lane and nothing is
// transposed.  The weights W are also written out once (4 B per pair) together with the reference
// they were formed with (one float per edge and 16 negatives): fp32 matrix throughput is ~20 flop
// per HBM byte on this chip while recomputing a score costs 2d flops, so k_flash_bwd reads them
// back, scales them by exp(reference - lse) and runs only the second product, with the roles of Q
// and K swapped.  Evaluation (PASS 3) only counts negatives scoring above
// the positive.  TransE uses |q - n|^2 = |q|^2 + |n|^2 - 2 q.n for the scores (pairs for which that expansion
// cancels are recomputed from the differences) and W = P / distance.
#include <type_traits>

#include "mar_common.h"
#include "mar_flash.h"

// A operands of the second product O^T[c][x] += sum_y Y[y][c] W[y][x] for one streamed row y.
// The 16 lanes m of a lane group supply the 16 output rows i of a matrix block; which output
// COLUMN c a row i stands for is free, so blocks are grouped so that one lane's operands for
// several blocks are consecutive floats of the row: a group of 4 blocks covers 64 columns with
// block j taking c = base + 4 i + j (one 16-byte LDS read feeds 4 matrix instructions), a group
// of 2 blocks 32 columns with c = base + 2 i + j, a single block c = base + i.
template <int NC>
__device__ __forceinline__ void load_orow(const float* __restrict__ yr, int m, float (&ya)[NC]) {
  constexpr int NG4 = NC / 4, NG2 = (NC % 4) / 2, NG1 = NC % 2;
#pragma unroll
  for (int q = 0; q < NG4; ++q) {
    const float4 v = *reinterpret_cast<const float4*>(yr + 64 * q + 4 * m);
    ya[4 * q + 0] = v.x; ya[4 * q + 1] = v.y; ya[4 * q + 2] = v.z; ya[4 * q + 3] = v.w;
  }
  if (NG2) {
    const float2 v = *reinterpret_cast<const float2*>(yr + 64 * NG4 + 2 * m);
    ya[4 * NG4 + 0] = v.x; ya[4 * NG4 + 1] = v.y;
  }
  if (NG1) ya[NC - 1] = yr[64 * NG4 + 32 * NG2 + m];
}

// Writes the accumulators of one stationary row back in row order, undoing the column grouping of
// load_orow: lane (g, .) register t of block cb holds output row i = 4g + t.  `sub` (TransE) is
// subtracted as xs[c] * ws.
template <int NC, bool SUB>
__device__ __forceinline__ void store_orow(float* __restrict__ orow, const float* __restrict__ xs, float ws, int dk, int g,
                                           const v4f (&o)[NC]) {
  constexpr int NG4 = NC / 4, NG2 = (NC % 4) / 2, NG1 = NC % 2;
#pragma unroll
  for (int q = 0; q < NG4; ++q) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int col = 64 * q + 16 * g + 4 * t;
      if (col < dk) {
        float4 v = make_float4(o[4 * q][t], o[4 * q + 1][t], o[4 * q + 2][t], o[4 * q + 3][t]);
        if (SUB) {
          const float4 x = *reinterpret_cast<const float4*>(xs + col);
          v.x -= x.x * ws; v.y -= x.y * ws; v.z -= x.z * ws; v.w -= x.w * ws;
        }
        *reinterpret_cast<float4*>(orow + col) = v;
      }
    }
  }
  if (NG2) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int col = 64 * NG4 + 8 * g + 2 * t;
      if (col < dk) {
        float2 v = make_float2(o[4 * NG4][t], o[4 * NG4 + 1][t]);
        if (SUB) {
          const float2 x = *reinterpret_cast<const float2*>(xs + col);
          v.x -= x.x * ws; v.y -= x.y * ws;
        }
        *reinterpret_cast<float2*>(orow + col) = v;
      }
    }
  }
  if (NG1) {
    const int col = 64 * NG4 + 32 * NG2 + 4 * g;
    if (col < dk) {
      float4 v = make_float4(o[NC - 1][0], o[NC - 1][1], o[NC - 1][2], o[NC - 1][3]);
      if (SUB) {
        const float4 x = *reinterpret_cast<const float4*>(xs + col);
        v.x -= x.x * ws; v.y -= x.y * ws; v.z -= x.z * ws; v.w -= x.w * ws;
      }
      *reinterpret_cast<float4*>(orow + col) = v;
    }
  }
}

template <int NK>
struct FlashGeom {
  static constexpr int KW = 4 * NK;                                  // tile width in floats
  static constexpr int PITCH = (KW % 8 == 4) ? KW : KW + 4;          // LDS row pitch: 4 mod 8
  static constexpr int N16 = NK / 4;                                  // k groups of 16 (b128 reads)
  static constexpr int NT = NK % 4;                                   // remaining k groups of 4
};

// Which float4 of a TY x NK tile (NK float4s per row) a thread moves in its u-th staging step.  Narrow rows:
// a thread owns one column group (thread % NKP, NKP = NK rounded up to a power of two; the threads beyond NK
// load a copy of the last group and store nothing) and steps through the rows with a fixed stride, so the
// only per-thread state is a row, a column and an LDS offset, and every step's LDS offset is a constant apart.
// Wide rows have no lanes to waste: slot = thread + 256 u over the row-major tile, recomputed where used.
template <int NK, int TY>
struct StageMap {
  static constexpr bool PO2 = NK <= 64;
  static constexpr int NKP = NK <= 16 ? 16 : (NK <= 32 ? 32 : 64);
  static constexpr int RPS = 256 / NKP;                                // rows per step
  static constexpr int NU = PO2 ? (TY + RPS - 1) / RPS : (TY * NK + 255) / 256;
  static_assert(!PO2 || TY % RPS == 0, "tile rows must be a multiple of the rows per staging step");
};

// PASS: 1 scores + online softmax + gQ (training), 3 rank counts (evaluation).  L2: TransE scores.
// XB: 16-row x-blocks per wave (a workgroup's stripe has 64*XB stationary rows); every LDS
// fragment of Y then feeds XB matrix instructions.
// LDS reads run one phase ahead of the matrix instructions that consume them: the first
// fragments of the next block's score product are fetched before the current block's
// second product is issued, and each row of the second product is fetched while the
// previous row is being multiplied.

// LDS of k_flash: one tile of the streamed matrix (DMA: two, unpadded) and, behind them, the streamed rows' squared
// norms (TransE), one set per tile buffer.
template <int NK, int TY, int DMA>
struct FwdGeom {
  static constexpr int PITCH = DMA ? FlashGeom<NK>::KW : FlashGeom<NK>::PITCH;
  static constexpr int TILE = TY * PITCH + 32;                          // floats per tile buffer
  static constexpr int NBUF = DMA ? 2 : 1;
  static constexpr size_t LDS_BYTES = (size_t)NBUF * (TILE + TY) * 4;
};

// DMA (compile time): the row width is exactly 4 NK floats, so a tile is one contiguous block of memory and is
// copied into LDS by buffer loads that write LDS directly (16 bytes per lane, 1 KB per wave instruction, zeros
// beyond the chunk's rows), two tiles ahead of their use in two alternating buffers: no staging registers, no
// LDS stores, one barrier per tile.  Otherwise tiles pass through registers into one padded LDS buffer.
template <int NK, int NC, int VT, int TY, int XB, int PASS, int L2, int DMA>
__global__ void __launch_bounds__(256) MAR_WAVES_PER_SIMD((NK * XB <= 64 ? 2 : 1))
k_flash(FlashArgs a) {
  typedef FlashGeom<NK> GM;
  typedef FwdGeom<NK, TY, DMA> FG;
  constexpr int PITCH = FG::PITCH;
  constexpr int N16 = GM::N16, NT = GM::NT;
  constexpr int PD = N16 <= 8 ? N16 : 4;                  // float4 fragments of the score product kept in flight
  constexpr int NU = DMA ? 1 : StageMap<NK, TY>::NU;      // float4 units staged per thread
  constexpr int SR = 64 * XB;                             // stationary rows per workgroup
  extern __shared__ __attribute__((aligned(16))) float smem[];
  const float* tile = (const float*)__builtin_assume_aligned(smem, 16);   // the tile being read
  float* const auy_all = smem + FG::NBUF * FG::TILE;      // [NBUF][TY] per streamed row: squared norm (TransE)
  const float* auy = auy_all;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = lane >> 4, m = lane & 15;

  // workgroup -> (chunk-side, stripe, part); consecutive workgroup ids rotate over the 8 XCDs, so
  // all workgroups of one chunk-side are given ids with the same residue and share one L2.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  int part, cs, stripe, tps = a.tps;
  if (slot < a.whole_slots) {
    part = slot % a.sy;
    const int slot2 = slot / a.sy;
    cs = (slot2 / a.nstripes) * 8 + xcd;
    stripe = slot2 % a.nstripes;
  } else {                                                // a part of a split stripe: these go round all XCDs
    const int r = (slot - a.whole_slots) * 8 + xcd;
    const int unit = r / a.rem_k;
    part = r % a.rem_k;
    cs = a.rem_cs0 + unit / a.nstripes;
    stripe = unit % a.nstripes;
    tps = a.rem_tps;
  }
  if (cs >= 2 * a.nchunks) return;
  const int side = cs & 1, c = cs >> 1;
  const int ne = min(a.S, a.n - c * a.S);                 // edges in this chunk
  const int n_x = ne;                                     // stationary: the chunk's edges
  const int n_y = a.N;                                    // streamed: the chunk's negatives
  if (stripe * SR >= n_x) return;
  const size_t q_base = (size_t)side * a.B + (size_t)c * a.S;       // first Q row of the chunk
  const size_t k_base = (size_t)side * a.C * a.N + (size_t)c * a.N; // first K row of the chunk
  const size_t x_base = q_base;
  const size_t y_base = k_base;
  const int dk = a.dk;

  // ---- stationary fragments: xf[4s+i] = X[x][16s + 4g + i], tail xf[4*N16+j] = X[x][16*N16 + 4j + g]
  int x[XB]; bool xv[XB]; const float* xrow[XB];
  float xf[XB][NK], xnorm[XB], posx[XB];
#pragma unroll
  for (int b = 0; b < XB; ++b) {
    x[b] = stripe * SR + (wave * XB + b) * 16 + m;
    xv[b] = x[b] < n_x;
    xrow[b] = a.X + (x_base + (xv[b] ? x[b] : 0)) * dk;
#pragma unroll
    for (int s = 0; s < N16; ++s) {
      const int col = 16 * s + 4 * g;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (xv[b] && col < dk) v = *reinterpret_cast<const float4*>(xrow[b] + col);
      xf[b][4 * s + 0] = v.x; xf[b][4 * s + 1] = v.y; xf[b][4 * s + 2] = v.z; xf[b][4 * s + 3] = v.w;
    }
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int col = 16 * N16 + 4 * j + g;
      xf[b][4 * N16 + j] = (xv[b] && col < dk) ? xrow[b][col] : 0.f;
    }
    xnorm[b] = 0.f; posx[b] = 0.f;
    if (L2) xnorm[b] = xv[b] ? a.xx[x_base + x[b]] : 0.f;
    if (PASS == 3) posx[b] = xv[b] ? a.pos[(size_t)c * a.S + x[b]] : 0.f;
  }

  // Output columns [0, 16*NC) of the second product go through 16x16 matrix blocks; with VT the last
  // 4 columns [16*NC, 16*NC + 4) go through the 4x4 outer-product instruction instead (per lane over its
  // own 4 streamed rows, summed over the 4 lane groups at the end): a 16-wide block for 4 columns would
  // waste 3/4 of its matrix instructions, and the vector ALU cannot run beside the fp32 matrix pipe.
  v4f oacc[XB][NC];
  v4f otail[XB];                                          // last 4 output columns (VT), per lane over its own streamed rows
  float mrun[XB], lrun[XB], wsum[XB];
  float ref_blk[XB];                                      // lane group g: reference of block g of the current tile
  int cnt[XB];
#pragma unroll
  for (int b = 0; b < XB; ++b) {
#pragma unroll
    for (int cb = 0; cb < NC; ++cb) oacc[b][cb] = (v4f){0.f, 0.f, 0.f, 0.f};
    otail[b] = (v4f){0.f, 0.f, 0.f, 0.f};
    mrun[b] = -3.0e38f; lrun[b] = 0.f; wsum[b] = 0.f; cnt[b] = 0; ref_blk[b] = 0.f;
  }

  // ---- streamed tiles, register-staged prefetch of the next tile
  const int ntiles_all = (n_y + TY - 1) / TY;
  const int t_begin = part * tps;
  const int ntiles = min(ntiles_all, t_begin + tps);       // this part streams tiles [t_begin, ntiles); may be empty
  // Per-thread staging slots: which row / float4 of a tile this thread moves (see StageMap).
  typedef StageMap<NK, TY> SM;
  v4f stage[NU];                                           // plain vectors: a struct copy from global memory would pin the array in memory
  float st_auy = 0.f;
  const int s_cu = threadIdx.x % SM::NKP, s_r0 = threadIdx.x / SM::NKP;   // narrow rows: this thread's column group and first row
  const int s_col = min(4 * s_cu, dk - 4);
  const int s_lds = s_r0 * (PITCH / 4) + s_cu;               // LDS offsets in float4 units: 16-byte stores
  // slot u of this thread: byte offset of its float4 inside a tile of the streamed matrix, and its LDS offset
  // in float4 units (-1: nothing to store)
  auto slot_of = [&](int u, int& gofs, int& lofs) {
    if (SM::PO2) {
      gofs = ((s_r0 + SM::RPS * u) * dk + s_col) * 4;
      lofs = s_cu < NK ? s_lds + u * SM::RPS * (PITCH / 4) : -1;
    } else {
      const int unit = threadIdx.x + 256 * u;
      const int r = unit / NK, cu = unit % NK;
      gofs = unit < TY * NK ? (r * dk + min(4 * cu, dk - 4)) * 4 : MAR_BUF_NOWHERE;
      lofs = unit < TY * NK ? r * (PITCH / 4) + cu : -1;
    }
  };
  // Every staging load is issued unconditionally: a row beyond the chunk reads as zeros (its scores are masked
  // to -inf, so it weighs nothing).  A column group beyond dk holds a copy of the row's last four columns; it
  // meets zero fragments of the stationary rows in the score product and produces output columns that are
  // never stored.
  const BufRsrc ysrc = buf_rsrc(a.Y + y_base * dk, (uint32_t)n_y * dk * 4);
  const BufRsrc yysrc = buf_rsrc(L2 ? a.yy + y_base : a.Y, L2 ? (uint32_t)n_y * 4 : 0u);
  int s_gofs[SM::PO2 ? 1 : NU];                            // wide rows: one offset per slot, kept in registers
  if (SM::PO2) s_gofs[0] = (s_r0 * dk + s_col) * 4;
  else {
#pragma unroll
    for (int u = 0; u < NU; ++u) { int lofs; slot_of(u, s_gofs[u], lofs); }
  }
  auto load_tile = [&](int t) {
    const int tofs = t * TY * dk * 4;                      // scalar: byte offset of the tile
#pragma unroll
    for (int u = 0; u < NU; ++u) {
      if (SM::PO2) stage[u] = buf_load4(ysrc, s_gofs[0], tofs + u * SM::RPS * dk * 4);
      else stage[u] = buf_load4(ysrc, s_gofs[u], tofs);
    }
    if (L2) st_auy = buf_load1(yysrc, (int)(threadIdx.x % TY) * 4, t * TY * 4);
  };
  // DMA path: wave w copies the tile's 1 KB pieces w, w + 4, ... ; a register load issued behind them is the
  // fence: memory operations complete in order, so once its value is there the pieces are in LDS.
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  const v4i ywords = buf_words(a.Y + y_base * dk, (uint32_t)n_y * dk * 4);
  float fence = 0.f;
  int token = 0;
  constexpr int NCH = TY * NK / 64;                        // 1 KB pieces per tile
  constexpr int NCW = (NCH + 3) / 4;                       // pieces per wave
  static_assert(!DMA || (TY * NK) % 64 == 0, "a tile is a whole number of 1 KB pieces");
  // piece q of this wave (0 <= q < NCW) of tile t into buffer `buf`; after its last piece the wave issues the fence load
  auto dma_piece = [&](int t, int buf, int q) {
    const int tofs = t * TY * dk * 4;
    const int c = 4 * q + wave_s;
    if (c < NCH) buf_load4_to_lds(ywords, lds_address(smem) + (buf * FG::TILE + c * 256) * 4, lane * 16, tofs + c * 1024, token);
    if (q == NCW - 1) {
      // the fence load's offset passes through the copies, so it is issued behind them
      if (L2) st_auy = buf_load1(yysrc, (int)(threadIdx.x % TY) * 4 + token, t * TY * 4);
      else fence = buf_load1(ysrc, token, tofs);
    }
  };
  auto dma_tile = [&](int t, int buf) {
#pragma unroll
    for (int q = 0; q < NCW; ++q) dma_piece(t, buf, q);
  };
  // the fence value is consumed (for TransE: stored) before the barrier that publishes tile t in buffer `buf`
  auto dma_land = [&](int buf) {
    if (L2) auy_all[buf * TY + threadIdx.x % TY] = st_auy;
    else asm volatile("" : : "v"(fence));
  };
  if (t_begin < ntiles) { if (DMA) dma_tile(t_begin, 0); else load_tile(t_begin); }

  // fragments of the score product: q16[s] = Y[yb*16 + m][16s + 4g .. +3], q1[j] the tail columns
  float4 q16[PD];
  float q1[NT > 0 ? NT : 1];
  auto load_head = [&](int yb) {
    const float* yrow = &tile[(yb * 16 + m) * PITCH + 4 * g];
#pragma unroll
    for (int s = 0; s < PD; ++s) q16[s] = *reinterpret_cast<const float4*>(yrow + 16 * s);
#pragma unroll
    for (int j = 0; j < NT; ++j) q1[j] = tile[(yb * 16 + m) * PITCH + 16 * N16 + 4 * j + g];
  };

  // Moves the prefetched tile from the staging registers into LDS.  Called at the end of a tile's
  // iteration (and once before the loop), between two barriers.
  auto stage_tile = [&]() {
#pragma unroll
    for (int u = 0; u < NU; ++u) {
      int gofs, lofs;
      slot_of(u, gofs, lofs);
      if (lofs >= 0) reinterpret_cast<v4f*>(smem)[lofs] = stage[u];
    }
    if (L2) auy_all[threadIdx.x % TY] = st_auy;            // threads that share a row write the same value
  };
  if (t_begin < ntiles) {
    if (DMA) dma_land(0); else stage_tile();
    __syncthreads();
  }

  // One tile.  HAS_NEXT (compile time): another tile follows, it is prefetched and this tile is full; the
  // last tile of the part is a second copy of the code without prefetch, with row masks if it is partial.
  // Keeping the prefetch unconditional inside a copy matters: a load under a branch makes the compiler
  // wait for every outstanding memory operation (the score stores' round trip included) where the branches
  // join.
  auto do_tile = [&](const int t, auto has_next_c) __attribute__((always_inline)) {
    constexpr bool HAS_NEXT = decltype(has_next_c)::value;
    const int buf = DMA ? (t - t_begin) & 1 : 0;
    if (DMA) {
      tile = (const float*)__builtin_assume_aligned(smem + buf * FG::TILE, 16);
      auy = auy_all + buf * TY;
    }
    constexpr int CPB = (NCW + TY / 16 - 1) / (TY / 16);   // DMA: pieces per wave issued inside one block,
    constexpr int DSTEP = N16 / CPB > 0 ? N16 / CPB : 1;   // one every DSTEP steps of its score product
    static_assert(!DMA || CPB <= N16, "more pieces per block than steps to put them in");
    if (HAS_NEXT && !DMA) load_tile(t + 1);
    const int y0 = t * TY;
    const int nblk = HAS_NEXT ? TY / 16 : min(TY / 16, (n_y - y0 + 15) / 16);
    load_head(0);
    // One 16-row block of the tile.  For a full tile the blocks are unrolled so that the compiler can count
    // the score stores issued after the next tile's prefetch loads and wait for the loads alone (loads and
    // stores share one in-order counter; waiting for "everything" would stall on the stores' round trip).
    auto process_block = [&](const int yb, const bool more, const bool masked) {
      const int yl = yb * 16 + 4 * g;                      // first of this lane's 4 streamed rows
      const float* yrow = &tile[(yb * 16 + m) * PITCH + 4 * g];
      const float* ycol = &tile[yl * PITCH];
      // row 0 of the second product's A operand, fetched under the score product
      float ya[NC > 0 ? NC : 1];
      if (PASS != 3) load_orow<NC>(ycol, m, ya);
      // -- T[y][x]: lane (g, m), register r holds y = yb*16 + 4g + r, x = m
      v4f tacc[XB];
#pragma unroll
      for (int b = 0; b < XB; ++b) tacc[b] = (v4f){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < N16; ++s) {
        const float4 yv = q16[s % PD];
        if (s + PD < N16) q16[s % PD] = *reinterpret_cast<const float4*>(yrow + 16 * (s + PD));
#pragma unroll
        for (int b = 0; b < XB; ++b) tacc[b] = mfma16(yv.x, xf[b][4 * s + 0], tacc[b]);
#pragma unroll
        for (int b = 0; b < XB; ++b) tacc[b] = mfma16(yv.y, xf[b][4 * s + 1], tacc[b]);
#pragma unroll
        for (int b = 0; b < XB; ++b) tacc[b] = mfma16(yv.z, xf[b][4 * s + 2], tacc[b]);
#pragma unroll
        for (int b = 0; b < XB; ++b) tacc[b] = mfma16(yv.w, xf[b][4 * s + 3], tacc[b]);
        // the next tile's pieces are issued a few at a time between the matrix instructions: a burst of them would
        // hold the wave at the memory pipeline's queue
        if (DMA && HAS_NEXT && s % DSTEP == 0 && s / DSTEP < CPB) {
          const int q = yb * CPB + s / DSTEP;
          if (q < NCW) dma_piece(t + 1, buf ^ 1, q);
        }
        if (N16 > PD) __builtin_amdgcn_sched_barrier(0);    // keeps the read PD fragments ahead of its use
      }
#pragma unroll
      for (int j = 0; j < NT; ++j) {
#pragma unroll
        for (int b = 0; b < XB; ++b) tacc[b] = mfma16(q1[j], xf[b][4 * N16 + j], tacc[b]);
      }
      // -- scores and weights
      float w[XB][4];
      float yy4[4] = {0.f, 0.f, 0.f, 0.f};
      if (L2) {
#pragma unroll
        for (int r = 0; r < 4; ++r) yy4[r] = auy[yl + r];
      }
#pragma unroll
      for (int b = 0; b < XB; ++b) {
        float sc[4], dist[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) sc[r] = tacc[b][r];
        if (L2) {
          // |q - n|^2 = |q|^2 + |n|^2 - 2 q.n cancels when n is close to q: its rounding error is of the size of
          // 2^-22 (|q|^2 + |n|^2).  Pairs whose expanded value falls below 2^-8 of that sum (the expansion is
          // then left with fewer than ~14 good bits) are recomputed from the differences q_k - n_k themselves:
          // the four lanes that hold the fragments of stationary row m each sum their own columns of the
          // streamed row, one flagged pair of the column at a time (rare: the loop is skipped by the whole wave
          // when nothing is flagged).
          float d2[4];
          unsigned flags = 0u;
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const float sum2 = xnorm[b] + yy4[r];
            d2[r] = fmaxf(sum2 - 2.f * tacc[b][r], 0.f);
            if (d2[r] < 0.00390625f * sum2) flags |= 1u << r;
          }
          if (__any(flags != 0u)) {
            unsigned F = flags << (4 * g);                 // bit 4 g' + r: streamed row yb*16 + 4 g' + r against stationary row m
            F |= __shfl_xor(F, 16);
            F |= __shfl_xor(F, 32);
            while (__any(F != 0u)) {
              const int idx = F ? __ffs(F) - 1 : 0;
              const float* yfix = &tile[(yb * 16 + idx) * PITCH];
              float part = 0.f;
              if (F) {
#pragma unroll
                for (int s2 = 0; s2 < N16; ++s2) {
                  if (16 * s2 + 4 * g < dk) {
                    const float4 yv = *reinterpret_cast<const float4*>(yfix + 16 * s2 + 4 * g);
                    const float e0 = xf[b][4 * s2 + 0] - yv.x, e1 = xf[b][4 * s2 + 1] - yv.y;
                    const float e2 = xf[b][4 * s2 + 2] - yv.z, e3 = xf[b][4 * s2 + 3] - yv.w;
                    part += (e0 * e0 + e1 * e1) + (e2 * e2 + e3 * e3);
                  }
                }
#pragma unroll
                for (int j = 0; j < NT; ++j) {
                  if (16 * N16 + 4 * j + g < dk) { const float e0 = xf[b][4 * N16 + j] - yfix[16 * N16 + 4 * j + g]; part += e0 * e0; }
                }
              }
              part += __shfl_xor(part, 16);
              part += __shfl_xor(part, 32);
              if (F && (idx >> 2) == g) {
#pragma unroll
                for (int r = 0; r < 4; ++r) if ((idx & 3) == r) d2[r] = part;
              }
              F &= F - 1u;
            }
          }
#pragma unroll
          for (int r = 0; r < 4; ++r) { dist[r] = sqrtf(d2[r]); sc[r] = -dist[r]; }
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          if (masked && y0 + yl + r >= n_y) sc[r] = -__builtin_inff();
        }
        if (PASS == 3) {
#pragma unroll
          for (int r = 0; r < 4; ++r) cnt[b] += sc[r] > posx[b] ? 1 : 0;
        } else if (PASS == 1) {
          // Online softmax with a lazily updated reference: the common reference mrun of row x only
          // moves when some score exceeds it by more than 16 (always true for the first block), so
          // the cross-lane maximum and the rescale of the accumulators are off the common path;
          // exp(score - mrun) <= e^16 cannot overflow.
          const float mloc = fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3]));
          if (__any(mloc > mrun[b] + 16.f)) {
            float mall = fmaxf(mloc, __shfl_xor(mloc, 16));
            mall = fmaxf(mall, __shfl_xor(mall, 32));
            const float mnew = fmaxf(mrun[b], mall);
            const float alpha = __expf(mrun[b] - mnew);
            lrun[b] *= alpha;
#pragma unroll
            for (int cb = 0; cb < NC; ++cb) oacc[b][cb] *= alpha;
            if (VT) otail[b] *= alpha;
            if (L2) wsum[b] *= alpha;
            mrun[b] = mnew;
          }
#pragma unroll
          for (int r = 0; r < 4; ++r) w[b][r] = __expf(sc[r] - mrun[b]);
          lrun[b] += (w[b][0] + w[b][1]) + (w[b][2] + w[b][3]);
        }
        if (PASS != 3 && L2) {
#pragma unroll
          for (int r = 0; r < 4; ++r) w[b][r] = dist[r] > 0.f ? w[b][r] / dist[r] : 0.f;
          wsum[b] += (w[b][0] + w[b][1]) + (w[b][2] + w[b][3]);
        }
        if (PASS == 1) {
          // keep the weights for the negatives' gradient pass: row = edge, 4 consecutive negatives (0 for the
          // columns beyond the chunk's negatives).  The buffer is padded to whole stripes and tiles, so the
          // store needs no bounds test (a conditional store would hide from the compiler how many stores follow
          // the prefetch loads).  Lane group g keeps the reference of block g of the tile for the store at the
          // tile's end.
          *reinterpret_cast<float4*>(a.T + ((size_t)cs * a.trows + x[b]) * a.tpitch + y0 + yl) = make_float4(w[b][0], w[b][1], w[b][2], w[b][3]);
          if (yb == g % (TY / 16)) ref_blk[b] = mrun[b];
        }
      }
      // first fragments of the next block's score product, fetched under the second product (the fence keeps
      // the compiler from sinking the reads down to their uses, where their latency would be exposed)
      if (more) load_head(yb + 1);
      __builtin_amdgcn_sched_barrier(0);
      if (PASS != 3) {
        // -- O^T[c][x] += sum_y Y[y][c] W[y][x]: A = Y fragment (row c), B = W (lane x)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          float cur[NC];
#pragma unroll
          for (int cb = 0; cb < NC; ++cb) cur[cb] = ya[cb];
          if (r < 3) load_orow<NC>(ycol + (r + 1) * PITCH, m, ya);
#pragma unroll
          for (int cb = 0; cb < NC; ++cb) {
#pragma unroll
            for (int b = 0; b < XB; ++b) oacc[b][cb] = mfma16(cur[cb], w[b][r], oacc[b][cb]);
          }
          if (VT) {
            const float yt = tile[(yl + r) * PITCH + 16 * NC + (m & 3)];
#pragma unroll
            for (int b = 0; b < XB; ++b) otail[b] = mfma4(yt, w[b][r], otail[b]);
          }
        }
      }
    };
    if (HAS_NEXT && NK <= 32) {                            // narrow rows: blocks unrolled (wide rows lack the registers)
#pragma unroll
      for (int yb = 0; yb < TY / 16; ++yb) process_block(yb, yb + 1 < TY / 16, false);
    } else {
      const bool full = y0 + TY <= n_y;                    // full tile: no row masks
#pragma unroll 1
      for (int yb = 0; yb < nblk; ++yb) process_block(yb, yb + 1 < nblk, !full);
    }
    if (PASS == 1) {
      // references of this tile's blocks: lane (g, m) writes block g's (with fewer than 4 blocks per tile the
      // surplus lane groups write a second copy of the same value)
      static_assert(TY / 16 <= 4, "one lane group per block of a tile");
#pragma unroll
      for (int b = 0; b < XB; ++b)
        a.R[((size_t)cs * (a.tpitch / 16) + (size_t)(t * (TY / 16) + g % (TY / 16))) * a.trows + x[b]] = ref_blk[b];
    }
    if (HAS_NEXT) {
      if (DMA) {
        dma_land(buf ^ 1);
        __syncthreads();                                   // tile t + 1 is in LDS; every wave is done with tile t
      } else {
        __syncthreads();                                   // every wave is done with this tile
        stage_tile();
        __syncthreads();
      }
    }
  };
  for (int t = t_begin; t + 1 < ntiles; ++t) do_tile(t, std::true_type());
  if (t_begin < ntiles) do_tile(ntiles - 1, std::false_type());

  // ---- epilogue: the part's statistics and unnormalised gradient rows (row x of the chunk-side at index x)
  float* ml_out = a.ml + ((size_t)part * 2 * a.B + x_base) * 2;
  float* o_out = a.out + ((size_t)part * 2 * a.B + x_base) * dk;
  if (slot >= a.whole_slots && part > 0) {                // parts 1.. of a split stripe
    const size_t xr = (size_t)(part - 1) * a.rem_rows + (size_t)(cs - a.rem_cs0) * a.trows;
    ml_out = a.mlx + xr * 2;
    o_out = a.outx + xr * dk;
  } else if (slot >= a.whole_slots) {                     // part 0 of a split stripe: the regular place
    ml_out = a.ml + x_base * 2;
    o_out = a.out + x_base * dk;
  }
#pragma unroll
  for (int b = 0; b < XB; ++b) {
    if (PASS == 3) {
      int cn = cnt[b];
      cn += __shfl_xor(cn, 16);
      cn += __shfl_xor(cn, 32);
      if (g == 0 && xv[b]) (side == MAR_SIDE_DST ? a.rank_dst : a.rank_src)[(size_t)c * a.S + x[b]] = 1 + cn;
      continue;
    }
    if (PASS == 1) {
      float ltot = lrun[b] + __shfl_xor(lrun[b], 16);
      ltot += __shfl_xor(ltot, 32);
      if (g == 0 && xv[b]) *reinterpret_cast<float2*>(ml_out + (size_t)x[b] * 2) = make_float2(mrun[b], ltot);
    }
    float ws = wsum[b];
    if (L2) {
      ws += __shfl_xor(ws, 16);
      ws += __shfl_xor(ws, 32);
    }
    float4 ot = make_float4(otail[b][0], otail[b][1], otail[b][2], otail[b][3]);
    if (VT) {
      ot.x += __shfl_xor(ot.x, 16); ot.y += __shfl_xor(ot.y, 16); ot.z += __shfl_xor(ot.z, 16); ot.w += __shfl_xor(ot.w, 16);
      ot.x += __shfl_xor(ot.x, 32); ot.y += __shfl_xor(ot.y, 32); ot.z += __shfl_xor(ot.z, 32); ot.w += __shfl_xor(ot.w, 32);
    }
    if (!xv[b]) continue;
    float* orow = o_out + (size_t)x[b] * dk;
    store_orow<NC, L2 != 0>(orow, xrow[b], ws, dk, g, oacc[b]);
    if (VT && g == 0 && 16 * NC < dk) {
      float4 o = ot;
      if (L2) {
        const float4 xs = *reinterpret_cast<const float4*>(xrow[b] + 16 * NC);
        o.x -= xs.x * ws; o.y -= xs.y * ws; o.z -= xs.z * ws; o.w -= xs.w * ws;
      }
      *reinterpret_cast<float4*>(orow + 16 * NC) = o;
    }
  }
}

// Gradient w.r.t. the negatives' rows from the stored weights: gK[j] = sum_e T[e][j] exp(R[e][j / 16] - lse[e]) Q[e]
// (TransE: T holds the weights divided by the distance; minus n_j times their sum).  A workgroup owns 64*XB
// negatives (16*XB per wave; XB = 1 measured best: more, smaller workgroups fill the chip more evenly than
// two blocks per wave save in LDS reads) and streams the chunk's edges in tiles of TY: the Q rows go through
// LDS, the weights straight from memory into registers -- lane (g, m) takes T[e = 4g + r][j = m]
// of its 16-negative block, which is the B-operand layout of O^T[c][j] += sum_e Q[e][c] W[e][j] --
// one tile ahead: as soon as a block's scores are consumed the same registers are refilled with
// the next tile's.  Only the second product runs on the matrix cores.
#ifndef MAR_BWD_WAVES
#define MAR_BWD_WAVES 3
#endif
template <int NK, int NC, int VT, int TY, int XB, int L2>
__global__ void __launch_bounds__(256) MAR_WAVES_PER_SIMD((NK * XB <= 32 ? MAR_BWD_WAVES : 2))
k_flash_bwd(FlashArgs a) {
  typedef FlashGeom<NK> GM;
  constexpr int PITCH = GM::PITCH;
  constexpr int SR = 64 * XB;                             // negatives per workgroup
  constexpr int NB = TY / 16;                             // 16-row blocks per tile
  constexpr int NU = StageMap<NK, TY>::NU;                // float4 units of the Q tile staged per thread
  __shared__ __attribute__((aligned(16))) float tile[TY * PITCH + 32];
  static_assert(XB == 1 && 4 * TY <= 256, "one scale factor per thread: (wave's 16-negative block, streamed edge)");
  __shared__ __attribute__((aligned(16))) float aux[4][TY];   // per wave: exp(reference - lse) of the streamed edges

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = lane >> 4, m = lane & 15;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int part = slot % a.sy, slot2 = slot / a.sy;
#ifdef MAR_BWD_FORWARD_ORDER
  const int cs = (slot2 / a.nstripes) * 8 + xcd;
#else
  // Chunk-sides are taken in the reverse of pass 1's order: the weights pass 1 wrote last are still in the
  // memory-side cache when this pass starts, and it reads them first.
  const int cs = 2 * a.nchunks - 1 - ((slot2 / a.nstripes) * 8 + xcd);
#endif
  const int stripe = slot2 % a.nstripes;
  if (cs < 0 || cs >= 2 * a.nchunks) return;
  const int side = cs & 1, c = cs >> 1;
  const int n_y = min(a.S, a.n - c * a.S);                // edges in this chunk (streamed)
  const int n_x = a.N;                                    // negatives (stationary)
  if (stripe * SR >= n_x) return;
  const size_t y_base = (size_t)side * a.B + (size_t)c * a.S;        // first Q row of the chunk
  const size_t x_base = (size_t)side * a.C * a.N + (size_t)c * a.N;  // first K row of the chunk
  const int dk = a.dk;

  v4f oacc[XB][NC];
  v4f otail[XB];                                          // last 4 output columns (see k_flash)
  float wsum[XB];
#pragma unroll
  for (int b = 0; b < XB; ++b) {
#pragma unroll
    for (int cb = 0; cb < NC; ++cb) oacc[b][cb] = (v4f){0.f, 0.f, 0.f, 0.f};
    otail[b] = (v4f){0.f, 0.f, 0.f, 0.f};
    wsum[b] = 0.f;
  }

  const int ntiles_all = (n_y + TY - 1) / TY;
  const int t_begin = part * a.tps;
  const int ntiles = min(ntiles_all, t_begin + a.tps);

  // staging slots of the Q tile (see StageMap).  As in k_flash every load is unconditional: a row beyond the
  // chunk reads as zeros and carries lse = +inf, so it weighs nothing.
  typedef StageMap<NK, TY> SM;
  v4f stage[NU];                                           // plain vectors: a struct copy from global memory would pin the array in memory
  float2 st_ml;                                           // softmax statistics (part 0) of this thread's streamed row
  float st_ref;                                           // reference of (this thread's wave slot, streamed row)
  const int a_row = threadIdx.x % TY, a_wave = (threadIdx.x / TY) % 4;   // the scale factor this thread prepares
  const int s_cu = threadIdx.x % SM::NKP, s_r0 = threadIdx.x / SM::NKP;   // narrow rows: this thread's column group and first row
  const int s_col = min(4 * s_cu, dk - 4);
  const int s_lds = s_r0 * (PITCH / 4) + s_cu;               // LDS offsets in float4 units: 16-byte stores
  auto slot_of = [&](int u, int& gofs, int& lofs) {         // see k_flash
    if (SM::PO2) {
      gofs = ((s_r0 + SM::RPS * u) * dk + s_col) * 4;
      lofs = s_cu < NK ? s_lds + u * SM::RPS * (PITCH / 4) : -1;
    } else {
      const int unit = threadIdx.x + 256 * u;
      const int r = unit / NK, cu = unit % NK;
      gofs = unit < TY * NK ? (r * dk + min(4 * cu, dk - 4)) * 4 : MAR_BUF_NOWHERE;
      lofs = unit < TY * NK ? r * (PITCH / 4) + cu : -1;
    }
  };
  // weights of the current tile: tr[yb][b][r] = T[e = y0 + 16 yb + 4g + r][j = stripe*SR + (wave*XB + b)*16 + m].
  // The buffer is padded to whole tiles and stripes, and pass 1 has written every row of a 64-row stripe that
  // holds at least one edge (finite values); rows beyond the chunk get the scale factor 0 and weigh nothing.
  float tr[NB][XB][4];
  const BufRsrc tsrc = buf_rsrc(a.T + (size_t)cs * a.trows * a.tpitch, (uint32_t)a.trows * a.tpitch * 4);
  const int t_vofs = (4 * g * a.tpitch + stripe * SR + wave * XB * 16 + m) * 4;
  auto load_scores = [&](int t, int yb) {
    const int row0 = t * TY + yb * 16;                     // scalar
#pragma unroll
    for (int r = 0; r < 4; ++r) {
#pragma unroll
      for (int b = 0; b < XB; ++b) tr[yb][b][r] = buf_load1(tsrc, t_vofs, ((row0 + r) * a.tpitch + 16 * b) * 4);
    }
  };
  const size_t ml_stride = (size_t)2 * a.B;               // rows per part of pass 1's statistics
  // Q rows and statistics of the streamed edges: loads beyond the chunk's edges return zeros
  const BufRsrc ysrc = buf_rsrc(a.Y + y_base * dk, (uint32_t)n_y * dk * 4);
  const BufRsrc mlsrc = buf_rsrc(a.ml + y_base * 2, (uint32_t)n_y * 8);
  const BufRsrc rsrc = buf_rsrc(a.R + (size_t)cs * (a.tpitch / 16) * a.trows, (uint32_t)(a.tpitch / 16) * a.trows * 4);
  const int r_vofs = ((stripe * (SR / 16) + a_wave) * a.trows + a_row) * 4;
  int s_gofs[SM::PO2 ? 1 : NU];
  if (SM::PO2) s_gofs[0] = (s_r0 * dk + s_col) * 4;
  else {
#pragma unroll
    for (int u = 0; u < NU; ++u) { int lofs; slot_of(u, s_gofs[u], lofs); }
  }
  auto load_tile = [&](int t) {
    const int tofs = t * TY * dk * 4;                      // scalar: byte offset of the tile
#pragma unroll
    for (int u = 0; u < NU; ++u) {
      if (SM::PO2) stage[u] = buf_load4(ysrc, s_gofs[0], tofs + u * SM::RPS * dk * 4);
      else stage[u] = buf_load4(ysrc, s_gofs[u], tofs);
    }
    // statistics of streamed row threadIdx.x % TY (part 0 of pass 1); the log-sum-exp is formed from them only
    // when the tile is staged, so that nothing waits for this load here
    st_ml = buf_load2(mlsrc, a_row * 8, t * TY * 8);
    st_ref = buf_load1(rsrc, r_vofs, t * TY * 4);
  };
  auto stage_tile = [&](int t) {
#pragma unroll
    for (int u = 0; u < NU; ++u) {
      int gofs, lofs;
      slot_of(u, gofs, lofs);
      if (lofs >= 0) reinterpret_cast<v4f*>(tile)[lofs] = stage[u];
    }
    {                                                      // every thread prepares one (wave slot, row) factor; threads beyond
      const int yr = t * TY + a_row;                       // 4 TY write a second copy, and no wave takes a branch of its own
      float mm = st_ml.x, ll = st_ml.y;
      if (a.sy_ml > 1 && yr < n_y) {                       // pass 1 was split (small batches): merge the parts
        const float2* __restrict__ mlp = reinterpret_cast<const float2*>(a.ml) + y_base + yr;
        for (int p = 1; p < a.sy_ml; ++p) mm = fmaxf(mm, mlp[p * ml_stride].x);
        ll *= __expf(st_ml.x - mm);
        for (int p = 1; p < a.sy_ml; ++p) { const float2 v = mlp[p * ml_stride]; ll += v.y * __expf(v.x - mm); }
      }
      // stored weight = exp(score - reference): times exp(reference - lse) it is the softmax probability
      aux[a_wave][a_row] = yr < n_y ? __expf(st_ref - (mm + logf(ll))) : 0.f;
    }
  };
  if (t_begin < ntiles) {
    load_tile(t_begin);
#pragma unroll
    for (int yb = 0; yb < NB; ++yb) load_scores(t_begin, yb);
    stage_tile(t_begin);
    __syncthreads();
  }

  // One tile; HAS_NEXT (compile time): another tile follows and is prefetched -- its Q rows into the staging
  // registers at the start, its scores into the registers of each block as soon as the block has consumed
  // them -- with no branch around any load (see k_flash).  The last tile is a second copy without prefetch.
  auto do_tile = [&](const int t, auto has_next_c) __attribute__((always_inline)) {
    constexpr bool HAS_NEXT = decltype(has_next_c)::value;
    // the copy for the last tile forms its lane coordinates afresh (from a thread id the compiler cannot see
    // through) instead of keeping values alive across the main loop, which has no registers to spare
    int tid_l = threadIdx.x;
    if (!HAS_NEXT) asm volatile("" : "+v"(tid_l));
    const int g = (tid_l & 63) >> 4, m = tid_l & 15, wave_l = tid_l >> 6;
    if (HAS_NEXT) load_tile(t + 1);
    const int y0 = t * TY;
    const int nblk = HAS_NEXT ? NB : min(NB, (n_y - y0 + 15) / 16);
#pragma unroll
    for (int yb = 0; yb < NB; ++yb) {
      if (HAS_NEXT || yb < nblk) {                         // uniform over the workgroup
        const int yl = yb * 16 + 4 * g;
        const float* ycol = &tile[yl * PITCH];
        float ya[NC];
        load_orow<NC>(ycol, m, ya);
        float w[XB][4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float fs = aux[wave_l][yl + r];            // 0 for rows beyond the chunk
#pragma unroll
          for (int b = 0; b < XB; ++b) w[b][r] = tr[yb][b][r] * fs;
        }
        if (HAS_NEXT) load_scores(t + 1, yb);              // refill the registers just consumed
        if (L2) {
#pragma unroll
          for (int b = 0; b < XB; ++b) wsum[b] += (w[b][0] + w[b][1]) + (w[b][2] + w[b][3]);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          float cur[NC];
#pragma unroll
          for (int cb = 0; cb < NC; ++cb) cur[cb] = ya[cb];
          if (r < 3) load_orow<NC>(ycol + (r + 1) * PITCH, m, ya);
#pragma unroll
          for (int cb = 0; cb < NC; ++cb) {
#pragma unroll
            for (int b = 0; b < XB; ++b) oacc[b][cb] = mfma16(cur[cb], w[b][r], oacc[b][cb]);
          }
          if (VT) {
            const float yt = tile[(yl + r) * PITCH + 16 * NC + (m & 3)];
#pragma unroll
            for (int b = 0; b < XB; ++b) otail[b] = mfma4(yt, w[b][r], otail[b]);
          }
        }
        __builtin_amdgcn_sched_barrier(0);                 // blocks are scheduled one by one: hoisting the next block's
      }                                                    // LDS reads over this one costs more registers than there are
    }
    if (HAS_NEXT) {
      __syncthreads();                                     // every wave is done with this tile
      stage_tile(t + 1);
      __syncthreads();
    }
  };
  for (int t = t_begin; t + 1 < ntiles; ++t) do_tile(t, std::true_type());
  if (t_begin < ntiles) do_tile(ntiles - 1, std::false_type());

  // The epilogue derives its lane coordinates from a copy of the thread id that the compiler cannot see
  // through, so that they are formed here instead of being carried (spilled) across the tile loop.
  int tid_e = threadIdx.x;
  asm volatile("" : "+v"(tid_e));
  const int wave_e = tid_e >> 6, g_e = (tid_e & 63) >> 4, m_e = tid_e & 15;
#pragma unroll
  for (int b = 0; b < XB; ++b) {
    float ws = wsum[b];
    if (L2) {
      ws += __shfl_xor(ws, 16);
      ws += __shfl_xor(ws, 32);
    }
    float4 ot = make_float4(otail[b][0], otail[b][1], otail[b][2], otail[b][3]);
    if (VT) {
      ot.x += __shfl_xor(ot.x, 16); ot.y += __shfl_xor(ot.y, 16); ot.z += __shfl_xor(ot.z, 16); ot.w += __shfl_xor(ot.w, 16);
      ot.x += __shfl_xor(ot.x, 32); ot.y += __shfl_xor(ot.y, 32); ot.z += __shfl_xor(ot.z, 32); ot.w += __shfl_xor(ot.w, 32);
    }
    const int x = stripe * SR + (wave_e * XB + b) * 16 + m_e;
    if (x >= n_x) continue;
    const float* xrow = a.X + (x_base + x) * dk;
    // gradient row of part `part` of this negative's occurrence (occurrences: roles*n edge-side ones, then the
    // destination-replacing negatives, then the source-replacing ones)
    float* orow = a.out + (a.roles * (size_t)a.n + ((side == MAR_SIDE_DST ? 0 : (size_t)a.cn) + (size_t)c * a.N + x) * a.sy + part) * dk;
    store_orow<NC, L2 != 0>(orow, xrow, ws, dk, g_e, oacc[b]);
    if (VT && g_e == 0 && 16 * NC < dk) {
      float4 o = ot;
      if (L2) {
        const float4 xs = *reinterpret_cast<const float4*>(xrow + 16 * NC);
        o.x -= xs.x * ws; o.y -= xs.y * ws; o.z -= xs.z * ws; o.w -= xs.w * ws;
      }
      *reinterpret_cast<float4*>(orow + 16 * NC) = o;
    }
  }
}

// Merges the parts of the split stripes of pass 1 into the regular place, so that every later kernel sees one
// part: m = max_p m_p, l = sum_p l_p exp(m_p - m), O = sum_p O_p exp(m_p - m), parts in their order.  One group of
// 32 lanes per row; the group reads every part's statistics before its first lane overwrites part 0's.
__global__ void __launch_bounds__(256) k_flash_merge(FlashArgs a) {
  const int grp = threadIdx.x >> 5, l = threadIdx.x & 31;
  const long rrow = (long)blockIdx.x * 8 + grp;
  if (rrow >= a.rem_rows) return;
  const int cs = a.rem_cs0 + (int)(rrow / a.trows), x = (int)(rrow % a.trows);
  const int side = cs & 1, c = cs >> 1;
  if (x >= min(a.S, a.n - c * a.S)) return;
  const size_t row = (size_t)side * a.B + (size_t)c * a.S + x;
  float2 v[MAR_MAX_PARTS];
  v[0] = reinterpret_cast<const float2*>(a.ml)[row];
#pragma unroll
  for (int p = 1; p < MAR_MAX_PARTS; ++p)
    v[p] = p < a.rem_k ? reinterpret_cast<const float2*>(a.mlx)[(size_t)(p - 1) * a.rem_rows + rrow] : make_float2(-3.0e38f, 0.f);
  float mx = v[0].x;
#pragma unroll
  for (int p = 1; p < MAR_MAX_PARTS; ++p) mx = fmaxf(mx, v[p].x);
  float fac[MAR_MAX_PARTS], ls = 0.f;
#pragma unroll
  for (int p = 0; p < MAR_MAX_PARTS; ++p) { fac[p] = __expf(v[p].x - mx); ls += fac[p] * v[p].y; }
  float* o0 = a.out + row * a.dk;
  for (int k = 4 * l; k < a.dk; k += 128) {
    float4 o = *reinterpret_cast<const float4*>(o0 + k);
    o.x *= fac[0]; o.y *= fac[0]; o.z *= fac[0]; o.w *= fac[0];
    for (int p = 1; p < a.rem_k; ++p) {
      const float4 q = *reinterpret_cast<const float4*>(a.outx + ((size_t)(p - 1) * a.rem_rows + rrow) * a.dk + k);
      o.x += fac[p] * q.x; o.y += fac[p] * q.y; o.z += fac[p] * q.z; o.w += fac[p] * q.w;
    }
    *reinterpret_cast<float4*>(o0 + k) = o;
  }
  if (l == 0) reinterpret_cast<float2*>(a.ml)[row] = make_float2(mx, ls);
}

// ------------------------------------------------------------------- launchers -----
int mar_flash_supported(int dk) { return dk >= 4 && dk <= 400; }
// Streamed rows per tile of the instantiation that serves dk: pass 1 / 3, and pass 2 (whose widest
// instantiation takes 16-row tiles so that two workgroups fit in a CU's registers).
#ifndef MAR_BWD_WIDE_TY
#define MAR_BWD_WIDE_TY 32
#endif
int mar_flash_tile_rows(int dk, int pass) { return dk / 4 <= 32 ? 64 : (pass == 2 && dk / 4 > 64 ? MAR_BWD_WIDE_TY : 32); }

// Stationary rows per workgroup (64 per x-block of the instantiation that serves dk): pass 1 / 3 and pass 2.
#ifndef MAR_BWD_XB
#define MAR_BWD_XB 1
#endif
int mar_flash_stripe_rows(int dk, int pass) { return pass == 2 && dk / 4 <= 32 ? 64 * MAR_BWD_XB : 64; }

// NK, NC, VT, TY, XB: pass 1 / 3 instantiation; BNC, BVT, BXB, BTY: pass 2's.
template <int NK, int NC, int VT, int TY, int XB, int BNC, int BVT, int BXB, int BTY>
static hipError_t launch_sized(const FlashArgs& a, int pass, int l2, dim3 grid, hipStream_t st) {
  // rows of exactly 4 NK floats take the direct-to-LDS copy (widths whose unpadded pitch is a multiple of 64 floats
  // would put every row of a block in the same LDS banks and stay on the padded register path)
  constexpr bool CAN_DMA = (4 * NK) % 64 != 0;
  constexpr int DM = CAN_DMA ? 1 : 0;
  constexpr size_t lds_dma = FwdGeom<NK, TY, DM>::LDS_BYTES, lds_reg = FwdGeom<NK, TY, 0>::LDS_BYTES;
  const bool dma = CAN_DMA && a.dk == 4 * NK;
#define FL(P, L) do { \
    if (dma) hipLaunchKernelGGL((k_flash<NK, NC, VT, TY, XB, P, L, DM>), grid, dim3(256), lds_dma, st, a); \
    else hipLaunchKernelGGL((k_flash<NK, NC, VT, TY, XB, P, L, 0>), grid, dim3(256), lds_reg, st, a); } while (0)
  if (pass == 1) { if (l2) FL(1, 1); else FL(1, 0); }
  else if (pass == 2) {
    if (l2) hipLaunchKernelGGL((k_flash_bwd<NK, BNC, BVT, BTY, BXB, 1>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((k_flash_bwd<NK, BNC, BVT, BTY, BXB, 0>), grid, dim3(256), 0, st, a);
  }
  else { if (l2) FL(3, 1); else FL(3, 0); }
#undef FL
  return hipGetLastError();
}

// Kernels whose LDS exceeds the default limit of a launch must be told so once per process and device.
template <int NK, int NC, int VT, int TY, int XB>
static hipError_t prepare_sized() {
  constexpr size_t lds = FwdGeom<NK, TY, 1>::LDS_BYTES;
  if (lds <= 64 * 1024) return hipSuccess;
  hipError_t e = hipSuccess;
#define PREP(P, L) if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_flash<NK, NC, VT, TY, XB, P, L, 1>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)
  PREP(1, 0); PREP(1, 1); PREP(3, 0); PREP(3, 1);
#undef PREP
  return e;
}
hipError_t mar_flash_prepare() { return prepare_sized<100, 25, 0, 32, 1>(); }

hipError_t mar_launch_flash(const mar_ctx* c, const MarBatch& b, int pass, int32_t* rank_dst, int32_t* rank_src,
                            hipStream_t st) {
  const MarDims& d = c->dm;
  const MarLayout& L = c->L;
  FlashArgs a;
  a.X = pass == 2 ? L.Km : L.Q;  a.Y = pass == 2 ? L.Q : L.Km;   // stationary / streamed matrix
  a.xx = L.qq; a.yy = L.kk;
  a.ml = L.ml; a.pos = L.pos;
  a.T = L.T; a.R = L.R; a.tpitch = (d.N + 127) & ~127; a.trows = (d.S + 63) & ~63;
  a.out = pass == 1 ? L.gQ : L.G;
  a.rank_dst = rank_dst; a.rank_src = rank_src;
  a.n = b.n; a.B = d.B; a.C = d.C; a.N = d.N; a.S = d.S; a.cn = b.cn; a.nchunks = b.nchunks; a.dk = d.dk;
  const int max_nx = pass == 2 ? d.N : (b.n < d.S ? b.n : d.S);
  const bool split = d.split && pass != 3;                 // evaluation always runs in fp32
  const int sr = split ? mar_split_stripe_rows(d.dk, pass) : mar_flash_stripe_rows(d.dk, pass);
  a.yimg = pass == 1 ? L.Kimg : L.Qimg;
  a.yimg_tiles = ((pass == 1 ? d.N : d.S) + 31) / 32;
  a.ximg = pass == 1 ? L.Qimg : L.Kimg;
  a.ximg_tiles = ((pass == 1 ? d.S : d.N) + 31) / 32;
  a.nstripes = (max_nx + sr - 1) / sr;
  const int ncs = 2 * b.nchunks;
  a.sy = pass == 1 ? d.sy1 : (pass == 2 ? d.sy2 : 1);
  a.tps = pass == 1 ? d.tps1 : (pass == 2 ? d.tps2 : (1 << 30));
  a.sy_ml = d.sy1; a.roles = d.roles;
  dim3 grid((unsigned)(8 * ((ncs + 7) / 8) * a.nstripes * a.sy));
  a.whole_slots = 0x7fffffff; a.rem_cs0 = ncs; a.rem_k = 1; a.rem_tps = 0; a.rem_rows = 0; a.mlx = nullptr; a.outx = nullptr;
  if (pass == 1 && d.rem_k > 1 && b.n == d.B) {            // full batch: split the stripes beyond the last whole round
    a.whole_slots = d.rem_cs0 / 8 * a.nstripes;
    a.rem_cs0 = d.rem_cs0; a.rem_k = d.rem_k; a.rem_tps = d.rem_tps; a.rem_rows = d.rem_rows;
    a.mlx = L.mlx; a.outx = L.gQx;
    const int rem_wgs = (ncs - d.rem_cs0) * a.nstripes * d.rem_k;
    grid = dim3((unsigned)(8 * (a.whole_slots + (rem_wgs + 7) / 8)));
  }
  if (split && pass == 2 && d.rem2_k > 1 && b.n == d.B) {   // full batch: split the stripes beyond the last whole round
    a.whole_slots = d.rem2_cs0 / 8 * a.nstripes;
    a.rem_cs0 = d.rem2_cs0; a.rem_k = d.rem2_k; a.rem_tps = d.rem2_tps; a.rem_rows = d.rem2_rows;
    a.outx = L.Gx;
    const int rem_wgs = (ncs - d.rem2_cs0) * a.nstripes * d.rem2_k;
    grid = dim3((unsigned)(8 * (a.whole_slots + (rem_wgs + 7) / 8)));
  }
  if (split) return mar_split_launch(a, pass, grid, st);
  const int l2 = c->cfg.model == MAR_MODEL_TRANSE;
  const int nk = d.dk / 4;
#ifndef MAR_BWD_TAIL_MFMA
#define MAR_BWD_TAIL_MFMA 0
#endif
  constexpr int BV = MAR_BWD_TAIL_MFMA ? 0 : 1;         // pass 2: last 4 columns on the vector ALU, or one more matrix block
  if (nk <= 13) return launch_sized<13, 3, 1, 64, 1, 3 + (1 - BV), BV, MAR_BWD_XB, 64>(a, pass, l2, grid, st);
  if (nk <= 25) return launch_sized<25, 6, 1, 64, 1, 6 + (1 - BV), BV, MAR_BWD_XB, 64>(a, pass, l2, grid, st);
  if (nk <= 32) return launch_sized<32, 8, 0, 64, 1, 8, 0, MAR_BWD_XB, 64>(a, pass, l2, grid, st);
  if (nk <= 64) return launch_sized<64, 16, 0, 32, 1, 16, 0, 1, 32>(a, pass, l2, grid, st);
  return launch_sized<100, 25, 0, 32, 1, 25, 0, 1, MAR_BWD_WIDE_TY>(a, pass, l2, grid, st);
}

int mar_flash_wgs_per_cu(int dk, int pass) { return pass == 2 ? (dk / 4 <= 32 ? MAR_BWD_WAVES : 2) : (dk / 4 <= 64 ? 2 : 1); }

hipError_t mar_launch_flash_merge(const mar_ctx* c, const MarBatch& b, hipStream_t st) {
  const MarDims& d = c->dm;
  if (d.rem_k <= 1 || b.n != d.B) return hipSuccess;
  FlashArgs a = {};
  a.ml = c->L.ml; a.mlx = c->L.mlx; a.out = c->L.gQ; a.outx = c->L.gQx;
  a.n = b.n; a.B = d.B; a.S = d.S; a.dk = d.dk; a.trows = (d.S + 63) & ~63;
  a.rem_cs0 = d.rem_cs0; a.rem_k = d.rem_k; a.rem_rows = d.rem_rows;
  hipLaunchKernelGGL(k_flash_merge, dim3((unsigned)((d.rem_rows + 7) / 8)), dim3(256), 0, st, a);
  return hipGetLastError();
}

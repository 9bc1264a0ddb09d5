// Split-precision variant of the two contraction passes for the bilinear models (gfx950).
//
// Every fp32 operand is written as the sum of two bf16 numbers, v = hi + lo with hi = bf16(v) and
// lo = bf16(v - hi) (v - hi is exact in fp32), and every product a b is taken as
//     a_hi b_hi + a_lo b_hi + a_hi b_lo
// on the bf16 matrix pipe (v_mfma_f32_16x16x32_bf16, fp32 accumulation), which runs at 16 times the fp32 matrix
// rate.  The dropped term a_lo b_lo and the rounding of the lo parts are of relative size 2^-16 .. 2^-17 per
// product, far inside the 1e-4 bars of the step.  The passes write what k_flash / k_flash_bwd write (softmax
// statistics, unnormalised operand gradients, gradient rows of the negatives), so everything around them is shared;
// they keep no weights between them (pass 2 computes the scores again, see k_split).
//
// Operand images (mar_split.h).  The gather writes both operand matrices (the chunk's negatives, the chunk's
// edge-side operands) as "images": per chunk-side and tile of 32 rows a hi plane and a lo plane, [32][PA bytes] each,
// row = 32 NS bf16 values (the row padded with zeros to a multiple of 32 columns) at a pitch PA chosen so that both
// kinds of LDS read below are free of bank conflicts.  An image is one contiguous block; the images of the matrix a
// pass streams (pass 1: the negatives, pass 2: the edge-side operands) are copied into LDS by buffer loads that
// write LDS directly, one tile ahead, in two alternating buffers; the stationary rows' fragments are read from
// their own images once.
//
// Lane layouts (lane = 16 g + m):
//   v_mfma_f32_16x16x32_bf16: A lane holds row m, contraction slots 8g .. 8g+7; B lane holds column m, the same
//   slots; D lane holds column m, rows 4g .. 4g+3.  Which contraction index a slot stands for is free as long as A
//   and B agree.
//   Score product S^T[y][x] = sum_c Y[y][c] X[x][c]: A = Y from LDS (16-byte read of row y = m, columns 32 s + 8g ..),
//   B = X fragments held in registers.  D: lane (g, m) gets S^T[4g + r][x = m], for the two 16-row blocks of a tile.
//   Second product O^T[c][x] += sum_y Y[y][c] W[y][x] over the tile's 32 rows: B = W built from the lane's own 8
//   score registers, slot kk <-> y = 4g + kk (kk < 4), 16 + 4g + kk - 4 (kk >= 4).  A = Y^T: lane (g, m) needs
//   Y[y of slot kk][16 cb + m] -- a column access of a row-major plane, which the LDS transpose read
//   (ds_read_b64_tr_b16) provides: within a group of 16 lanes, lane i passes the address of 4 consecutive 16-bit
//   values and receives, as its j-th value, value (i % 4) of lane 4j + i / 4.  With lane i pointing at row
//   4g + i / 4 (+ 16 for the second block), columns 16 cb + 4 (i % 4) .. +3, lane m receives Y[4g + j][16 cb + m].
#include <type_traits>

#include "mar_common.h"
#include "mar_flash.h"
#include "mar_split.h"

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef __bf16 v4bf __attribute__((ext_vector_type(4)));
typedef short v4s __attribute__((ext_vector_type(4)));

__device__ __forceinline__ v4f mfma_bf(v8bf a, v8bf b, v4f c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// v = hi + lo, both bf16 (round to nearest even); converted two at a time (one packed conversion per pair)
typedef float v2f __attribute__((ext_vector_type(2)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void split8(const float (&v)[8], v8bf& hi, v8bf& lo) {
#pragma unroll
  for (int i = 0; i < 8; i += 2) {
    const v2f p = {v[i], v[i + 1]};
    const v2bf h = __builtin_convertvector(p, v2bf);
    const v2f r = p - __builtin_convertvector(h, v2f);
    const v2bf l = __builtin_convertvector(r, v2bf);
    hi[i] = h[0]; hi[i + 1] = h[1];
    lo[i] = l[0]; lo[i + 1] = l[1];
  }
}

template <int NS>
struct SplitGeom {
  static constexpr int PA = sp_pitch(64 * NS);
  static constexpr int PLANE = sp_plane(NS);
  static constexpr int IMG = sp_image(NS);
  static constexpr int NCH = IMG / 1024;                   // 1 KB pieces of an image
  static constexpr int NCW = (NCH + 3) / 4;                // pieces per wave
  static constexpr size_t LDS_BYTES = 2 * (size_t)IMG;
};

__device__ __forceinline__ unsigned lds_address_b(const char* p) {
  return (unsigned)(unsigned long long)(__attribute__((address_space(3))) const char*)p;
}
__device__ __forceinline__ v4s lds_read_tr(const char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)p);
}
__device__ __forceinline__ v8bf join8(v4s a, v4s b) {
  return __builtin_bit_cast(v8bf, __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7));
}

// O^T[c][x] += sum over the tile's 32 rows of Y[y][c] W[y][x] for the 16-column blocks cb0 .. cb0 + ncb - 1 (ncb <= NCB,
// uniform over the wave); W is given split.  Blocks are taken a few at a time so that consecutive matrix instructions
// write different accumulators.
template <int NCB, int XB, int PA>
__device__ __forceinline__ void second_product(const char* hi, const char* lo, int trofs, int cb0, int ncb, const v8bf (&wh)[XB],
                                               const v8bf (&wl)[XB], v4f (&oacc)[XB][NCB]) {
  constexpr int CG = XB >= 2 ? 2 : 4;
  hi += trofs + 32 * cb0; lo += trofs + 32 * cb0;
#pragma unroll
  for (int c0 = 0; c0 < NCB; c0 += CG) {
    v8bf ah[CG], al[CG];
#pragma unroll
    for (int j = 0; j < CG; ++j) {
      if (c0 + j < NCB && (c0 + j < NCB - 1 || c0 + j < ncb)) {   // only the last block may be absent
        ah[j] = join8(lds_read_tr(hi + 32 * (c0 + j)), lds_read_tr(hi + 16 * PA + 32 * (c0 + j)));
        al[j] = join8(lds_read_tr(lo + 32 * (c0 + j)), lds_read_tr(lo + 16 * PA + 32 * (c0 + j)));
      }
    }
#pragma unroll
    for (int k = 0; k < 3; ++k) {
#pragma unroll
      for (int j = 0; j < CG; ++j) {
        if (c0 + j < NCB && (c0 + j < NCB - 1 || c0 + j < ncb)) {
#pragma unroll
          for (int b = 0; b < XB; ++b) oacc[b][c0 + j] = mfma_bf(k == 1 ? al[j] : ah[j], k == 2 ? wl[b] : wh[b], oacc[b][c0 + j]);
        }
      }
    }
  }
}

// ------------------------------------------------------------------- the two passes -----
// PASS 1: scores, online softmax and gQ = P K for 64 XB edges of one chunk-side against the chunk's negatives; the
// unit numbering, the split of the last round's stripes and the lazily updated softmax reference are k_flash's, and
// so are the statistics and gradient rows written.  No weights are kept for pass 2:
// PASS 2: gK = P^T Q for 64 XB negatives of one chunk-side against the chunk's edges, with the scores computed again
// (the same three bf16 products) and P = exp(score - lse) from the finished log-sum-exp.  Writing the weights out
// and reading them back costs 8 bytes of memory traffic per pair, computing a score again 6 d bf16 flops: at this
// matrix rate the second is several times cheaper (the fp32 passes, whose matrix rate is 16 times lower, store them).
// The unit numbering and the gradient rows written are k_flash_bwd's.
// CSP = 2 (widest rows): two waves share each 16-row block, each taking half of the columns -- half of the
// contraction steps of the score product (the partial scores are exchanged through LDS and added, so both waves go
// on with the same scores, weights and softmax statistics) and half of the second product's output blocks.  A wave
// then holds half of the stationary fragments and half of the accumulators, and a workgroup of eight waves puts two
// waves on every SIMD where the four-wave form has registers for one.
template <int NS, int NCB, int XB, int PASS, int CSP, int NW>
__global__ void __launch_bounds__(64 * NW) MAR_WAVES_PER_SIMD((NW == 8 || NS <= 8 ? 2 : 1))
k_split(FlashArgs a) {
  typedef SplitGeom<NS> SG;
  constexpr int PA = SG::PA, PLANE = SG::PLANE, IMG = SG::IMG;
  constexpr int TY = SP_TY;
  constexpr int SR = (NW / CSP) * XB * 16;                 // stationary rows per workgroup
  constexpr int NSA = (NS + CSP - 1) / CSP, NCBA = (NCB + CSP - 1) / CSP;   // steps and output blocks per wave
  constexpr int NCW = (SG::NCH + NW - 1) / NW;             // 1 KB pieces of an image per wave
  constexpr float LOG2E = 1.44269504088896341f;
  static_assert(SR == 64 * (NS <= 4 ? 2 : 1), "stripe rows the launch planning assumes");
  extern __shared__ __attribute__((aligned(16))) char smem[];
  float* const aux_all = reinterpret_cast<float*>(smem + 2 * IMG);   // PASS 2: [2][TY] log-sum-exp of the tile's edges
  float* const xch = aux_all + 2 * TY;                     // CSP = 2: [NW][8 XB][64] partial scores

  const int lane = threadIdx.x & 63, wave_all = threadIdx.x >> 6;
  const int wave = wave_all / CSP, half = wave_all % CSP;  // row block of the workgroup, half of the columns
  const int s0 = half * NSA, ns = min(NSA, NS - s0);       // this wave's contraction steps s0 .. s0 + ns - 1
  const int cb0 = half * NCBA, ncb = min(NCBA, NCB - cb0); // and output blocks
  const int g = lane >> 4, m = lane & 15;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  int part, cs, stripe, tps = a.tps;
  if (slot < a.whole_slots) {
    part = slot % a.sy;
    const int slot2 = slot / a.sy;
    cs = (slot2 / a.nstripes) * 8 + xcd;
    stripe = slot2 % a.nstripes;
  } else {                                                // a part of a split stripe (see k_flash)
    const int r = (slot - a.whole_slots) * 8 + xcd;
    const int unit = r / a.rem_k;
    part = r % a.rem_k;
    cs = a.rem_cs0 + unit / a.nstripes;
    stripe = unit % a.nstripes;
    tps = a.rem_tps;
  }
  const int csl = cs;                                      // chunk-side in launch order
  if (PASS == 2) cs = 2 * a.nchunks - 1 - cs;              // reverse of pass 1's order (see k_flash_bwd)
  if (cs < 0 || cs >= 2 * a.nchunks) return;
  const int side = cs & 1, c = cs >> 1;
  const int ne = min(a.S, a.n - c * a.S);                 // edges in this chunk
  const int n_x = PASS == 1 ? ne : a.N;                   // stationary rows
  const int n_y = PASS == 1 ? a.N : ne;                   // streamed rows
  if (stripe * SR >= n_x) return;
  const size_t q_base = (size_t)side * a.B + (size_t)c * a.S;        // first Q row of the chunk
  const size_t k_base = (size_t)side * a.C * a.N + (size_t)c * a.N;  // first K row of the chunk
  const size_t x_base = PASS == 1 ? q_base : k_base;
  const int dk = a.dk;

  // ---- stationary fragments from the rows' own images: slots of step s = columns 32 s + 8g .. +7 of row x
  int x[XB]; bool xv[XB];
  v8bf xh[XB][NSA], xl[XB][NSA];
#pragma unroll
  for (int b = 0; b < XB; ++b) {
    x[b] = stripe * SR + (wave * XB + b) * 16 + m;
    xv[b] = x[b] < n_x;
    const char* xrow = a.ximg + ((size_t)cs * a.ximg_tiles + x[b] / TY) * IMG + (x[b] % TY) * PA + 16 * g + 64 * s0;
#pragma unroll
    for (int s = 0; s < NSA; ++s) {
      xh[b][s] = (v8bf){0, 0, 0, 0, 0, 0, 0, 0};
      xl[b][s] = (v8bf){0, 0, 0, 0, 0, 0, 0, 0};
      if (xv[b] && s < ns) {
        xh[b][s] = *reinterpret_cast<const v8bf*>(xrow + 64 * s);
        xl[b][s] = *reinterpret_cast<const v8bf*>(xrow + PLANE + 64 * s);
      }
    }
  }

  v4f oacc[XB][NCBA];
  float mrun[XB], lrun[XB];
#pragma unroll
  for (int b = 0; b < XB; ++b) {
#pragma unroll
    for (int cb = 0; cb < NCBA; ++cb) oacc[b][cb] = (v4f){0.f, 0.f, 0.f, 0.f};
    mrun[b] = -3.0e38f; lrun[b] = 0.f;
  }

  const int ntiles_all = (n_y + TY - 1) / TY;
  const int t_begin = part * tps;
  const int ntiles = min(ntiles_all, t_begin + tps);

  // ---- images of the streamed rows, copied into LDS one tile ahead (see k_flash's DMA path); a register load issued
  // behind the copies is the fence: once its value is there the image is in LDS.  PASS 2's fence is the load of the
  // softmax statistics of streamed edge threadIdx % TY.
  const char* ybase = a.yimg + (size_t)cs * a.yimg_tiles * IMG;
  const uint32_t ybytes = (uint32_t)a.yimg_tiles * IMG;
  const v4i ywords = buf_words(ybase, ybytes);
  const BufRsrc ysrc = buf_rsrc(ybase, ybytes);
  const BufRsrc mlsrc = buf_rsrc(a.ml + q_base * 2, PASS == 2 ? (uint32_t)ne * 8 : 0u);
  const int wave_s = __builtin_amdgcn_readfirstlane(wave_all);
  const int f_row = threadIdx.x % TY;
  const size_t ml_stride = (size_t)2 * a.B;               // rows per part of pass 1's statistics
  float fence = 0.f;
  float2 st_ml = make_float2(0.f, 0.f);
  int token = 0;
  auto dma_tile = [&](int t, int buf) {
    const int tofs = t * IMG;
#pragma unroll
    for (int q = 0; q < NCW; ++q) {
      const int pc = NW * q + wave_s;
      if (pc < SG::NCH) buf_load4_to_lds(ywords, lds_address_b(smem) + buf * IMG + pc * 1024, lane * 16, tofs + pc * 1024, token);
    }
    if (PASS == 2) st_ml = buf_load2(mlsrc, f_row * 8 + token, t * TY * 8);
    else fence = buf_load1(ysrc, token, tofs);
  };
  auto dma_land = [&](int t, int buf) {
    if (PASS == 2) {
      const int yr = t * TY + f_row;
      float mm = st_ml.x, ll = st_ml.y;
      if (a.sy_ml > 1 && yr < n_y) {                       // pass 1 was split (small batches): merge the parts
        const float2* __restrict__ mlp = reinterpret_cast<const float2*>(a.ml) + q_base + yr;
        for (int p = 1; p < a.sy_ml; ++p) mm = fmaxf(mm, mlp[p * ml_stride].x);
        ll *= __expf(st_ml.x - mm);
        for (int p = 1; p < a.sy_ml; ++p) { const float2 v = mlp[p * ml_stride]; ll += v.y * __expf(v.x - mm); }
      }
      // rows beyond the chunk: +inf, so that their weights are exp(-inf) = 0
      // (times log2(e): the weights are formed as 2^(score log2(e) - this); threads that share a row write the same value)
      aux_all[buf * TY + f_row] = yr < n_y ? (mm + logf(ll)) * LOG2E : __builtin_inff();
    } else {
      asm volatile("" : : "v"(fence));
    }
  };
  if (t_begin < ntiles) {
    dma_tile(t_begin, 0);
    dma_land(t_begin, 0);
    __syncthreads();
  }

  const int trofs = (4 * g + (m >> 2)) * PA + 8 * (m & 3);
  for (int t = t_begin; t < ntiles; ++t) {
    const int buf = (t - t_begin) & 1;
    const char* hi = smem + buf * IMG;
    const char* lo = hi + PLANE;
    const bool has_next = t + 1 < ntiles;                  // uniform
    if (has_next) dma_tile(t + 1, buf ^ 1);
    const int y0 = t * TY;
    const bool masked = PASS == 1 && y0 + TY > n_y;

    // -- scores of the tile's two 16-row blocks.  The fragments of the streamed rows are read PD groups (one group =
    // one contraction step of one block) ahead of the matrix instructions that consume them.
    v4f sacc[2][XB];
#pragma unroll
    for (int yb = 0; yb < 2; ++yb) {
#pragma unroll
      for (int b = 0; b < XB; ++b) sacc[yb][b] = (v4f){0.f, 0.f, 0.f, 0.f};
    }
    {
      constexpr int NG = 2 * NSA, PD = NG < 4 ? NG : 4;
      const int fofs = m * PA + 16 * g + 64 * s0;
      v8bf fh[PD], fl[PD];
#pragma unroll
      for (int q = 0; q < PD; ++q) {                       // group q: step q / 2, block q % 2
        fh[q] = *reinterpret_cast<const v8bf*>(hi + fofs + (q % 2) * 16 * PA + (q / 2) * 64);
        fl[q] = *reinterpret_cast<const v8bf*>(lo + fofs + (q % 2) * 16 * PA + (q / 2) * 64);
      }
#pragma unroll
      for (int q = 0; q < NG; ++q) {
        const int s = q / 2, yb = q % 2;
        if (CSP > 1 && s == NSA - 1 && s >= ns) break;       // the second half may have one step less (uniform over the wave)
        const v8bf ah = fh[q % PD], al = fl[q % PD];
        if (q + PD < NG) {
          fh[q % PD] = *reinterpret_cast<const v8bf*>(hi + fofs + ((q + PD) % 2) * 16 * PA + ((q + PD) / 2) * 64);
          fl[q % PD] = *reinterpret_cast<const v8bf*>(lo + fofs + ((q + PD) % 2) * 16 * PA + ((q + PD) / 2) * 64);
        }
#pragma unroll
        for (int b = 0; b < XB; ++b) sacc[yb][b] = mfma_bf(ah, xh[b][s], sacc[yb][b]);
#pragma unroll
        for (int b = 0; b < XB; ++b) sacc[yb][b] = mfma_bf(al, xh[b][s], sacc[yb][b]);
#pragma unroll
        for (int b = 0; b < XB; ++b) sacc[yb][b] = mfma_bf(ah, xl[b][s], sacc[yb][b]);
        __builtin_amdgcn_sched_barrier(0);                 // keeps the reads PD groups ahead of their use
      }
    }
    if (CSP == 2) {                                        // add the other half's partial scores
      float* mine = xch + (wave_all * 8 * XB) * 64 + lane;
#pragma unroll
      for (int b = 0; b < XB; ++b) {
#pragma unroll
        for (int yb = 0; yb < 2; ++yb) {
#pragma unroll
          for (int r = 0; r < 4; ++r) mine[(8 * b + 4 * yb + r) * 64] = sacc[yb][b][r];
        }
      }
      __syncthreads();
      const float* other = xch + ((wave_all ^ 1) * 8 * XB) * 64 + lane;
#pragma unroll
      for (int b = 0; b < XB; ++b) {
#pragma unroll
        for (int yb = 0; yb < 2; ++yb) {
#pragma unroll
          for (int r = 0; r < 4; ++r) sacc[yb][b][r] += other[(8 * b + 4 * yb + r) * 64];
        }
      }
    }
    // -- weights of the lane's 8 pairs per x-block: slot kk <-> y = y0 + (kk < 4 ? 4g + kk : 16 + 4g + kk - 4)
    float lse8[8];
    if (PASS == 2) {
      const float4 l0 = *reinterpret_cast<const float4*>(aux_all + buf * TY + 4 * g);
      const float4 l1 = *reinterpret_cast<const float4*>(aux_all + buf * TY + 16 + 4 * g);
      lse8[0] = l0.x; lse8[1] = l0.y; lse8[2] = l0.z; lse8[3] = l0.w; lse8[4] = l1.x; lse8[5] = l1.y; lse8[6] = l1.z; lse8[7] = l1.w;
    }
    v8bf wh[XB], wl[XB];
#pragma unroll
    for (int b = 0; b < XB; ++b) {
      float sc[8], w[8];
#pragma unroll
      for (int yb = 0; yb < 2; ++yb) {
#pragma unroll
        for (int r = 0; r < 4; ++r) sc[4 * yb + r] = sacc[yb][b][r];
      }
      if (masked) {                                        // the chunk's last, partial tile (uniform): rows beyond it weigh nothing
#pragma unroll
        for (int yb = 0; yb < 2; ++yb) {
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            if (y0 + 16 * yb + 4 * g + r >= n_y) sc[4 * yb + r] = -__builtin_inff();
          }
        }
      }
      if (PASS == 1) {
        const float mloc = fmaxf(fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3])), fmaxf(fmaxf(sc[4], sc[5]), fmaxf(sc[6], sc[7])));
        if (__any(mloc > mrun[b] + 16.f)) {
          float mall = fmaxf(mloc, __shfl_xor(mloc, 16));
          mall = fmaxf(mall, __shfl_xor(mall, 32));
          const float mnew = fmaxf(mrun[b], mall);
          float alpha = __expf(mrun[b] - mnew);
          asm volatile("" : "+v"(alpha));                  // a real branch: keeps the rescale from being executed speculatively
          lrun[b] *= alpha;
#pragma unroll
          for (int cb = 0; cb < NCBA; ++cb) oacc[b][cb] *= alpha;
          mrun[b] = mnew;
        }
        const float nm2 = -LOG2E * mrun[b];
#pragma unroll
        for (int k = 0; k < 8; ++k) w[k] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[k], LOG2E, nm2));
        lrun[b] += ((w[0] + w[1]) + (w[2] + w[3])) + ((w[4] + w[5]) + (w[6] + w[7]));
      } else {
#pragma unroll
        for (int k = 0; k < 8; ++k) w[k] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[k], LOG2E, -lse8[k]));
      }
      split8(w, wh[b], wl[b]);
    }
    // -- O^T[c][x] += sum_y Y[y][c] W[y][x]
    second_product<NCBA, XB, PA>(hi, lo, trofs, cb0, ncb, wh, wl, oacc);
    if (has_next) {
      dma_land(t + 1, buf ^ 1);
      __syncthreads();                                     // tile t + 1 is in LDS; every wave is done with tile t
    }
  }

  // ---- epilogue
  if (PASS == 1) {                                         // the part's statistics and unnormalised gradient rows
    float* ml_out = a.ml + ((size_t)part * 2 * a.B + x_base) * 2;
    float* o_out = a.out + ((size_t)part * 2 * a.B + x_base) * dk;
    if (slot >= a.whole_slots && part > 0) {
      const size_t xr = (size_t)(part - 1) * a.rem_rows + (size_t)(cs - a.rem_cs0) * a.trows;
      ml_out = a.mlx + xr * 2;
      o_out = a.outx + xr * dk;
    } else if (slot >= a.whole_slots) {
      ml_out = a.ml + x_base * 2;
      o_out = a.out + x_base * dk;
    }
#pragma unroll
    for (int b = 0; b < XB; ++b) {
      float ltot = lrun[b] + __shfl_xor(lrun[b], 16);
      ltot += __shfl_xor(ltot, 32);
      if (!xv[b]) continue;
      if (g == 0 && half == 0) *reinterpret_cast<float2*>(ml_out + (size_t)x[b] * 2) = make_float2(mrun[b], ltot);
      float* orow = o_out + (size_t)x[b] * dk;
#pragma unroll
      for (int cb = 0; cb < NCBA; ++cb) {
        const int col = 16 * (cb0 + cb) + 4 * g;
        if (cb < ncb && col < dk) *reinterpret_cast<float4*>(orow + col) = make_float4(oacc[b][cb][0], oacc[b][cb][1], oacc[b][cb][2], oacc[b][cb][3]);
      }
    }
  } else {                                                 // gradient row of part `part` of each negative's occurrence
#pragma unroll
    for (int b = 0; b < XB; ++b) {
      if (!xv[b]) continue;
      float* orow = a.out + (a.roles * (size_t)a.n + ((side == MAR_SIDE_DST ? 0 : (size_t)a.cn) + (size_t)c * a.N + x[b]) * a.sy +
                             (slot >= a.whole_slots ? 0 : part)) * dk;
      if (slot >= a.whole_slots && part > 0)               // parts 1.. of a split stripe: added to the regular row afterwards
        orow = a.outx + ((size_t)(part - 1) * a.rem_rows + (size_t)(csl - a.rem_cs0) * (a.nstripes * SR) + x[b]) * dk;
#pragma unroll
      for (int cb = 0; cb < NCBA; ++cb) {
        const int col = 16 * (cb0 + cb) + 4 * g;
        if (cb < ncb && col < dk) *reinterpret_cast<float4*>(orow + col) = make_float4(oacc[b][cb][0], oacc[b][cb][1], oacc[b][cb][2], oacc[b][cb][3]);
      }
    }
  }
}

// Adds parts 1.. of pass 2's split stripes to the gradient rows that part 0 wrote, in the parts' order.  One group of
// 32 lanes per row.
__global__ void __launch_bounds__(256) k_split_merge2(FlashArgs a, int stripe_rows) {
  const int grp = threadIdx.x >> 5, l = threadIdx.x & 31;
  const long rrow = (long)blockIdx.x * 8 + grp;
  if (rrow >= a.rem_rows) return;
  const int pitch = a.nstripes * stripe_rows;
  const int cs = 2 * a.nchunks - 1 - (a.rem_cs0 + (int)(rrow / pitch)), x = (int)(rrow % pitch);
  if (cs < 0 || x >= a.N) return;
  const int side = cs & 1, c = cs >> 1;
  float* o0 = a.out + (a.roles * (size_t)a.n + ((side == MAR_SIDE_DST ? 0 : (size_t)a.cn) + (size_t)c * a.N + x)) * a.dk;
  for (int k = 4 * l; k < a.dk; k += 128) {
    float4 o = *reinterpret_cast<const float4*>(o0 + k);
    for (int p = 1; p < a.rem_k; ++p) {
      const float4 q = *reinterpret_cast<const float4*>(a.outx + ((size_t)(p - 1) * a.rem_rows + rrow) * a.dk + k);
      o.x += q.x; o.y += q.y; o.z += q.z; o.w += q.w;
    }
    *reinterpret_cast<float4*>(o0 + k) = o;
  }
}

// ------------------------------------------------------------------- launchers -----
// Form of the widest instantiation (d > 256): row blocks per wave and waves per workgroup (two waves share a block).
#ifndef SP_WIDE_XB
#define SP_WIDE_XB 1
#endif
#ifndef SP_WIDE_NW
#define SP_WIDE_NW 8
#endif
int mar_split_supported(int dk) { return dk >= 4 && dk <= 400; }
int mar_split_stripe_rows(int dk, int pass) { (void)pass; return sp_ns(dk) <= 4 ? 128 : 64; }
int mar_split_tile_rows() { return SP_TY; }
int mar_split_wgs_per_cu(int dk, int pass) { (void)pass; return sp_ns(dk) <= 8 ? 2 : 1; }
size_t mar_split_image_bytes(int dk) { return (size_t)sp_image(sp_ns(dk)); }

// LDS of a launch: two image buffers, the log-sum-exp of a tile's edges (pass 2), the exchange area (CSP = 2)
template <int NS, int XB, int CSP, int NW>
constexpr size_t sp_lds() { return SplitGeom<NS>::LDS_BYTES + 2 * SP_TY * 4 + (CSP == 2 ? NW * 8 * XB * 64 * 4 : 0); }

template <int NS, int NCB, int XB, int CSP, int NW>
static hipError_t sp_prepare() {
  constexpr size_t lds = sp_lds<NS, XB, CSP, NW>();
  hipError_t e = hipSuccess;
  if (lds > 64 * 1024) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_split<NS, NCB, XB, 1, CSP, NW>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_split<NS, NCB, XB, 2, CSP, NW>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  }
  return e;
}
hipError_t mar_split_prepare() {
  hipError_t e = sp_prepare<8, 13, 1, 1, 4>();
  if (e == hipSuccess) e = sp_prepare<8, 16, 1, 1, 4>();
  if (e == hipSuccess) e = sp_prepare<13, 25, SP_WIDE_XB, 2, SP_WIDE_NW>();
  return e;
}

template <int NS, int NCB, int XB, int CSP, int NW>
static hipError_t sp_launch(const FlashArgs& a, int pass, dim3 grid, hipStream_t st) {
  constexpr size_t lds = sp_lds<NS, XB, CSP, NW>();
  if (pass == 1) hipLaunchKernelGGL((k_split<NS, NCB, XB, 1, CSP, NW>), grid, dim3(64 * NW), lds, st, a);
  else hipLaunchKernelGGL((k_split<NS, NCB, XB, 2, CSP, NW>), grid, dim3(64 * NW), lds, st, a);
  return hipGetLastError();
}

// `a` is filled by mar_launch_flash (units, parts, buffers); this picks the instantiation for a.dk.
static hipError_t sp_launch_sized(const FlashArgs& a, int pass, dim3 grid, hipStream_t st);

hipError_t mar_split_launch(const FlashArgs& a, int pass, dim3 grid, hipStream_t st) {
  hipError_t e = sp_launch_sized(a, pass, grid, st);
  if (e == hipSuccess && pass == 2 && a.rem_k > 1) {
    hipLaunchKernelGGL(k_split_merge2, dim3((unsigned)((a.rem_rows + 7) / 8)), dim3(256), 0, st, a, mar_split_stripe_rows(a.dk, 2));
    e = hipGetLastError();
  }
  return e;
}

static hipError_t sp_launch_sized(const FlashArgs& a, int pass, dim3 grid, hipStream_t st) {
  const int ns = sp_ns(a.dk), ncb = sp_ncb(a.dk);
  if (ns == 2) return sp_launch<2, 4, 2, 1, 4>(a, pass, grid, st);
  if (ns == 4) return ncb == 7 ? sp_launch<4, 7, 2, 1, 4>(a, pass, grid, st) : sp_launch<4, 8, 2, 1, 4>(a, pass, grid, st);
  if (ns == 8) return ncb == 13 ? sp_launch<8, 13, 1, 1, 4>(a, pass, grid, st) : sp_launch<8, 16, 1, 1, 4>(a, pass, grid, st);
  return sp_launch<13, 25, SP_WIDE_XB, 2, SP_WIDE_NW>(a, pass, grid, st);
}

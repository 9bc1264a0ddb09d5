// Row-wise (bandwidth-bound) kernels of the training step (gfx950): gather of the batch's
// rows into dense contraction operands, the chain rule from operand gradients back to the
// source / relation / destination rows, the per-row gradient reduction over the row-sorted
// order, and the sparse Adagrad scatter.
#include "mar_common.h"
#include "mar_split.h"

struct RowArgs {
  const float *node_emb, *rel_emb;
  const int32_t *src, *rel, *dst, *neg_src, *neg_dst;
  int32_t n, cn, B, C, N, S, dim, dk, model;
  int64_t n_occ;
  int32_t num_nodes;
  int32_t sy1, sy2;      // parts per stripe in the two contraction passes
  int32_t roles;         // 3, or 2 for the relation-free Dot score
};

template <int GL> __device__ __forceinline__ float group_sum(float v) {
#pragma unroll
  for (int o = GL / 2; o >= 1; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// ---------------------------------------------------------------------- gather -----
// Edge blocks: one lane group per PREP_EDGES edges builds the two edge-side operands of each
//     side DST (negatives replace d): a_ej = <q, n_j>,  q = s*r (DistMult), s.r complex (ComplEx)
//     side SRC (negatives replace s): b_ej = <q, m_j>,  q = r*d,            conj(r).d
//   for TransE the scores are -|q - n_j| with q = s + r and q = d - r; also the positive score.
// Negative blocks: one lane group per PREP_NEGS negatives copies their rows into the dense per-chunk matrix.
// A group issues the loads of all its rows before the first use: the gathers are bound by the latency of
// scattered row reads (address translation included), so bytes in flight per lane are what counts.
// VEC: dim is a multiple of 4, rows are moved as float4 (float2 pairs for the two halves of a ComplEx row) and
// a lane holds all its pieces of a row (NV per row); otherwise one element per lane and step.
// MODEL: the score function, resolved at compile time.
#ifndef PREP_EDGES
#define PREP_EDGES 2
#endif
#ifndef PREP_NEGS
#define PREP_NEGS 4
#endif

template <int GL, int NV, bool VEC, int MODEL>
__global__ void __launch_bounds__(256)
k_prep(RowArgs a, int nbB, float* __restrict__ Q, float* __restrict__ Km, float* __restrict__ qq,
       float* __restrict__ kk, float* __restrict__ pos, float* __restrict__ pos_user, SplitImages qi, SplitImages ki) {
  const int blk = blockIdx.x;
  constexpr int GPB = 256 / GL;                  // lane groups per block
  const int grp = threadIdx.x / GL, l = threadIdx.x % GL;
  const int dim = a.dim, dk = a.dk;
  if (blk < nbB) {
    const int e0 = (blk * GPB + grp) * PREP_EDGES;
    if (e0 >= a.n) return;
    const float *s_row[PREP_EDGES], *r_row[PREP_EDGES], *d_row[PREP_EDGES];
#pragma unroll
    for (int j = 0; j < PREP_EDGES; ++j) {
      const int e = min(e0 + j, a.n - 1);                        // a group's surplus edge repeats the last one (not stored)
      s_row[j] = a.node_emb + (size_t)a.src[e] * dim;
      r_row[j] = a.rel_emb + (size_t)(MODEL == MAR_MODEL_DOT ? 0 : a.rel[e]) * dim;     // unused by Dot
      d_row[j] = a.node_emb + (size_t)a.dst[e] * dim;
    }
    float acc[PREP_EDGES], nd[PREP_EDGES], ns[PREP_EDGES];
#pragma unroll
    for (int j = 0; j < PREP_EDGES; ++j) acc[j] = nd[j] = ns[j] = 0.f;
    if (VEC && MODEL == MAR_MODEL_COMPLEX) {
      const int h = dim >> 1;
      float2 sr[PREP_EDGES][NV], si[PREP_EDGES][NV], rr[PREP_EDGES][NV], ri[PREP_EDGES][NV], dr[PREP_EDGES][NV], di[PREP_EDGES][NV];
#pragma unroll
      for (int j = 0; j < PREP_EDGES; ++j) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
          const int k = 2 * (l + GL * v);
          if (k < h) {
            sr[j][v] = *reinterpret_cast<const float2*>(s_row[j] + k); si[j][v] = *reinterpret_cast<const float2*>(s_row[j] + h + k);
            rr[j][v] = *reinterpret_cast<const float2*>(r_row[j] + k); ri[j][v] = *reinterpret_cast<const float2*>(r_row[j] + h + k);
            dr[j][v] = *reinterpret_cast<const float2*>(d_row[j] + k); di[j][v] = *reinterpret_cast<const float2*>(d_row[j] + h + k);
          }
        }
      }
#pragma unroll
      for (int j = 0; j < PREP_EDGES; ++j) {
        if (e0 + j < a.n) {
          float* qd = Q + ((size_t)MAR_SIDE_DST * a.B + e0 + j) * dk;
          float* qs = Q + ((size_t)MAR_SIDE_SRC * a.B + e0 + j) * dk;
          char* id_ = nullptr; char* is_ = nullptr;          // split precision: the rows' places in the images
          if (qi.base) {
            const int ch = (e0 + j) / a.S, er = (e0 + j) % a.S;
            id_ = sp_row(qi, 2 * ch + MAR_SIDE_DST, er); is_ = sp_row(qi, 2 * ch + MAR_SIDE_SRC, er);
            for (int k = dim + 4 * l; k < qi.dkp; k += 4 * GL) {        // zero columns up to the images' width
              sp_store4(id_, qi.plane, k, make_float4(0.f, 0.f, 0.f, 0.f)); sp_store4(is_, qi.plane, k, make_float4(0.f, 0.f, 0.f, 0.f));
            }
          }
#pragma unroll
          for (int v = 0; v < NV; ++v) {
            const int k = 2 * (l + GL * v);
            if (k < h) {
              const float2 ure = make_float2(sr[j][v].x * rr[j][v].x - si[j][v].x * ri[j][v].x, sr[j][v].y * rr[j][v].y - si[j][v].y * ri[j][v].y);
              const float2 uim = make_float2(sr[j][v].x * ri[j][v].x + si[j][v].x * rr[j][v].x, sr[j][v].y * ri[j][v].y + si[j][v].y * rr[j][v].y);
              const float2 wre = make_float2(rr[j][v].x * dr[j][v].x + ri[j][v].x * di[j][v].x, rr[j][v].y * dr[j][v].y + ri[j][v].y * di[j][v].y);
              const float2 wim = make_float2(rr[j][v].x * di[j][v].x - ri[j][v].x * dr[j][v].x, rr[j][v].y * di[j][v].y - ri[j][v].y * dr[j][v].y);
              acc[j] += (ure.x * dr[j][v].x + uim.x * di[j][v].x) + (ure.y * dr[j][v].y + uim.y * di[j][v].y);
              if (qi.base) {
                sp_store2(id_, qi.plane, k, ure); sp_store2(id_, qi.plane, h + k, uim);
                sp_store2(is_, qi.plane, k, wre); sp_store2(is_, qi.plane, h + k, wim);
              } else {
                *reinterpret_cast<float2*>(qd + k) = ure; *reinterpret_cast<float2*>(qd + h + k) = uim;
                *reinterpret_cast<float2*>(qs + k) = wre; *reinterpret_cast<float2*>(qs + h + k) = wim;
              }
            }
          }
        }
      }
    } else if (VEC) {
      float4 s4[PREP_EDGES][NV], r4[PREP_EDGES][NV], d4[PREP_EDGES][NV];
#pragma unroll
      for (int j = 0; j < PREP_EDGES; ++j) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
          const int k = 4 * (l + GL * v);
          if (k < dim) {
            s4[j][v] = *reinterpret_cast<const float4*>(s_row[j] + k); d4[j][v] = *reinterpret_cast<const float4*>(d_row[j] + k);
            r4[j][v] = MODEL == MAR_MODEL_DOT ? make_float4(0.f, 0.f, 0.f, 0.f) : *reinterpret_cast<const float4*>(r_row[j] + k);
          }
        }
      }
#pragma unroll
      for (int j = 0; j < PREP_EDGES; ++j) {
        if (e0 + j < a.n) {
          float* qd = Q + ((size_t)MAR_SIDE_DST * a.B + e0 + j) * dk;
          float* qs = Q + ((size_t)MAR_SIDE_SRC * a.B + e0 + j) * dk;
          char* id_ = nullptr; char* is_ = nullptr;
          if (qi.base) {
            const int ch = (e0 + j) / a.S, er = (e0 + j) % a.S;
            id_ = sp_row(qi, 2 * ch + MAR_SIDE_DST, er); is_ = sp_row(qi, 2 * ch + MAR_SIDE_SRC, er);
            for (int k = dim + 4 * l; k < qi.dkp; k += 4 * GL) {
              sp_store4(id_, qi.plane, k, make_float4(0.f, 0.f, 0.f, 0.f)); sp_store4(is_, qi.plane, k, make_float4(0.f, 0.f, 0.f, 0.f));
            }
          }
#pragma unroll
          for (int v = 0; v < NV; ++v) {
            const int k = 4 * (l + GL * v);
            if (k < dim) {
              const float4 s = s4[j][v], r = r4[j][v], d = d4[j][v];
              float4 u, w;
              if (MODEL == MAR_MODEL_DISTMULT) {
                u = make_float4(s.x * r.x, s.y * r.y, s.z * r.z, s.w * r.w);
                w = make_float4(r.x * d.x, r.y * d.y, r.z * d.z, r.w * d.w);
                acc[j] += (u.x * d.x + u.y * d.y) + (u.z * d.z + u.w * d.w);
              } else if (MODEL == MAR_MODEL_DOT) {
                u = s; w = d;
                acc[j] += (s.x * d.x + s.y * d.y) + (s.z * d.z + s.w * d.w);
              } else {
                u = make_float4(s.x + r.x, s.y + r.y, s.z + r.z, s.w + r.w);
                w = make_float4(d.x - r.x, d.y - r.y, d.z - r.z, d.w - r.w);
                const float4 df = make_float4(u.x - d.x, u.y - d.y, u.z - d.z, u.w - d.w);
                acc[j] += (df.x * df.x + df.y * df.y) + (df.z * df.z + df.w * df.w);
                nd[j] += (u.x * u.x + u.y * u.y) + (u.z * u.z + u.w * u.w);
                ns[j] += (w.x * w.x + w.y * w.y) + (w.z * w.z + w.w * w.w);
              }
              if (qi.base) { sp_store4(id_, qi.plane, k, u); sp_store4(is_, qi.plane, k, w); }
              else { *reinterpret_cast<float4*>(qd + k) = u; *reinterpret_cast<float4*>(qs + k) = w; }
            }
          }
        }
      }
    } else {
      for (int j = 0; j < PREP_EDGES; ++j) {
        if (e0 + j >= a.n) break;
        float* qd = Q + ((size_t)MAR_SIDE_DST * a.B + e0 + j) * dk;
        float* qs = Q + ((size_t)MAR_SIDE_SRC * a.B + e0 + j) * dk;
        char* id_ = nullptr; char* is_ = nullptr;
        if (qi.base) {
          const int ch = (e0 + j) / a.S, er = (e0 + j) % a.S;
          id_ = sp_row(qi, 2 * ch + MAR_SIDE_DST, er); is_ = sp_row(qi, 2 * ch + MAR_SIDE_SRC, er);
          for (int k = dim + l; k < qi.dkp; k += GL) { sp_store1(id_, qi.plane, k, 0.f); sp_store1(is_, qi.plane, k, 0.f); }
        }
        if (MODEL == MAR_MODEL_COMPLEX) {
          const int h = dim >> 1;
          for (int k = l; k < h; k += GL) {
            const float sr = s_row[j][k], si = s_row[j][h + k], rr = r_row[j][k], ri = r_row[j][h + k], dr = d_row[j][k], di = d_row[j][h + k];
            const float ure = sr * rr - si * ri, uim = sr * ri + si * rr;
            const float wre = rr * dr + ri * di, wim = rr * di - ri * dr;
            acc[j] += ure * dr + uim * di;
            if (qi.base) {
              sp_store1(id_, qi.plane, k, ure); sp_store1(id_, qi.plane, h + k, uim);
              sp_store1(is_, qi.plane, k, wre); sp_store1(is_, qi.plane, h + k, wim);
            } else { qd[k] = ure; qd[h + k] = uim; qs[k] = wre; qs[h + k] = wim; }
          }
        } else {
          for (int k = l; k < dim; k += GL) {
            const float s = s_row[j][k], r = MODEL == MAR_MODEL_DOT ? 0.f : r_row[j][k], d = d_row[j][k];
            float u, w;
            if (MODEL == MAR_MODEL_DISTMULT) { u = s * r; w = r * d; acc[j] += u * d; }
            else if (MODEL == MAR_MODEL_DOT) { u = s; w = d; acc[j] += s * d; }
            else { u = s + r; w = d - r; const float df = u - d; acc[j] += df * df; nd[j] += u * u; ns[j] += w * w; }
            if (qi.base) { sp_store1(id_, qi.plane, k, u); sp_store1(is_, qi.plane, k, w); }
            else { qd[k] = u; qs[k] = w; }
          }
        }
        if (!qi.base) { for (int k = dim + l; k < dk; k += GL) { qd[k] = 0.f; qs[k] = 0.f; } }
      }
    }
#pragma unroll
    for (int j = 0; j < PREP_EDGES; ++j) {
      const int e = e0 + j;
      float sc = group_sum<GL>(acc[j]);
      if (MODEL == MAR_MODEL_TRANSE) {
        const float sd = group_sum<GL>(nd[j]), ss = group_sum<GL>(ns[j]);
        sc = -sqrtf(sc);
        if (l == 0 && e < a.n) { qq[(size_t)MAR_SIDE_DST * a.B + e] = sd; qq[(size_t)MAR_SIDE_SRC * a.B + e] = ss; }
      }
      if (l == 0 && e < a.n) { pos[e] = sc; if (pos_user) pos_user[e] = sc; }
    }
    return;
  }
  {
    const int rr0 = ((blk - nbB) * GPB + grp) * PREP_NEGS;       // first row among the 2*cn negatives
    if (rr0 >= 2 * a.cn) return;
    const float* row[PREP_NEGS];
    size_t krow[PREP_NEGS];
    char* irow[PREP_NEGS];                                       // split precision: the rows' places in the images
#pragma unroll
    for (int j = 0; j < PREP_NEGS; ++j) {
      const int rr = min(rr0 + j, 2 * a.cn - 1);
      const int side = rr >= a.cn ? MAR_SIDE_DST : MAR_SIDE_SRC;
      const int cj = rr - (side == MAR_SIDE_DST ? a.cn : 0);    // chunk*N + j
      const int32_t id = side == MAR_SIDE_DST ? a.neg_dst[cj] : a.neg_src[cj];
      row[j] = a.node_emb + (size_t)id * dim;
      krow[j] = (size_t)side * a.C * a.N + cj;
      irow[j] = ki.base ? sp_row(ki, 2 * (cj / a.N) + side, cj % a.N) : nullptr;
    }
    if (VEC) {
      float4 v4[PREP_NEGS][NV];
#pragma unroll
      for (int j = 0; j < PREP_NEGS; ++j) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
          const int k = 4 * (l + GL * v);
          if (k < dim) v4[j][v] = *reinterpret_cast<const float4*>(row[j] + k);
        }
      }
#pragma unroll
      for (int j = 0; j < PREP_NEGS; ++j) {
        float nn = 0.f;
        if (rr0 + j < 2 * a.cn) {
          if (ki.base) {
            for (int k = dim + 4 * l; k < ki.dkp; k += 4 * GL) sp_store4(irow[j], ki.plane, k, make_float4(0.f, 0.f, 0.f, 0.f));
          }
#pragma unroll
          for (int v = 0; v < NV; ++v) {
            const int k = 4 * (l + GL * v);
            if (k < dim) {
              const float4 x = v4[j][v];
              nn += (x.x * x.x + x.y * x.y) + (x.z * x.z + x.w * x.w);
              if (ki.base) sp_store4(irow[j], ki.plane, k, x);
              else *reinterpret_cast<float4*>(Km + krow[j] * dk + k) = x;
            }
          }
        }
        if (MODEL == MAR_MODEL_TRANSE) {
          nn = group_sum<GL>(nn);
          if (l == 0 && rr0 + j < 2 * a.cn) kk[krow[j]] = nn;
        }
      }
    } else {
      for (int j = 0; j < PREP_NEGS; ++j) {
        float nn = 0.f;
        if (rr0 + j < 2 * a.cn) {
          for (int k = l; k < (ki.base ? ki.dkp : dk); k += GL) {
            const float x = k < dim ? row[j][k] : 0.f;
            nn += x * x;
            if (ki.base) sp_store1(irow[j], ki.plane, k, x);
            else Km[krow[j] * dk + k] = x;
          }
        }
        if (MODEL == MAR_MODEL_TRANSE) {
          nn = group_sum<GL>(nn);
          if (l == 0 && rr0 + j < 2 * a.cn) kk[krow[j]] = nn;
        }
      }
    }
  }
}

// ------------------------------------------------------------------ chain rule -----
// From the gradients w.r.t. the two edge-side operands (gq_dst w.r.t. the DST-side q, gq_src
// w.r.t. the SRC-side q) and the positive term -2 f(e) to gradient rows of s, r, d, written at
// the occurrences' fixed places.  Also the per-edge loss terms, summed per block in a fixed order.
//
// Pass 1 leaves, per part p of a stripe, the softmax reference m_p, the sum l_p and the unnormalised
// O_p = sum_j exp(a_j - m_p) n_j.  merge_parts turns them into the log-sum-exp and one factor per part,
// fac_p = exp(m_p - m) / l with m = max m_p and l = sum_p l_p exp(m_p - m), so that gq = sum_p fac_p O_p.

__device__ __forceinline__ float merge_parts(const float* __restrict__ ml, size_t row, size_t part_rows, int sy1,
                                             float (&fac)[MAR_MAX_PARTS]) {
  const float2* __restrict__ p2 = reinterpret_cast<const float2*>(ml) + row;
  float2 v[MAR_MAX_PARTS];
#pragma unroll
  for (int p = 0; p < MAR_MAX_PARTS; ++p) v[p] = p < sy1 ? p2[p * part_rows] : make_float2(-3.0e38f, 0.f);
  float mx = v[0].x;
#pragma unroll
  for (int p = 1; p < MAR_MAX_PARTS; ++p) mx = fmaxf(mx, v[p].x);
  float ls = 0.f;
#pragma unroll
  for (int p = 0; p < MAR_MAX_PARTS; ++p) { fac[p] = __expf(v[p].x - mx); ls += fac[p] * v[p].y; }
  const float il = 1.f / ls;
#pragma unroll
  for (int p = 0; p < MAR_MAX_PARTS; ++p) fac[p] *= il;
  return mx + logf(ls);
}

// Chain rule of one element: from s, r, d, the merged operand gradients u (DST side) and w (SRC side).
template <int MODEL>
__device__ __forceinline__ void chain1(float s, float r, float d, float u, float w, float inv2, float& gs, float& gd, float& gr) {
  if (MODEL == MAR_MODEL_DISTMULT) {
    gs = r * (u - 2.f * d); gd = r * (w - 2.f * s); gr = s * u + d * w - 2.f * s * d;
  } else if (MODEL == MAR_MODEL_DOT) {
    gs = u - 2.f * d; gd = w - 2.f * s; gr = 0.f;
  } else {                                               // TransE: inv2 = 2 / distance (0 at distance 0)
    const float dl = (s + r - d) * inv2;                 // 2 * unit(s + r - d)
    gs = u + dl; gr = u - w + dl; gd = w - dl;
  }
}

// ComplEx, one complex element: g_s = conj(r) (gU - 2 d), g_d = r (gW - 2 s), g_r = conj(s) gU + conj(gW) d - 2 conj(s) d.
__device__ __forceinline__ void chain_complex(float sr, float si, float rr, float ri, float dr, float di, float ure, float uim,
                                              float wre, float wim, float& gsr, float& gsi, float& gdr, float& gdi,
                                              float& grr, float& gri) {
  const float zr = ure - 2.f * dr, zi = uim - 2.f * di;
  gsr = rr * zr + ri * zi;  gsi = rr * zi - ri * zr;
  const float yr = wre - 2.f * sr, yi = wim - 2.f * si;
  gdr = rr * yr - ri * yi;  gdi = rr * yi + ri * yr;
  grr = sr * ure + si * uim + wre * dr + wim * di - 2.f * (sr * dr + si * di);
  gri = sr * uim - si * ure + wre * di - wim * dr - 2.f * (sr * di - si * dr);
}

// One group of GL lanes per edge.  VEC (dim % 4 == 0): a lane moves NV float4s per row (for ComplEx NV float2s of
// the real half and the matching float2s of the imaginary half), every load of the edge is issued before the
// first use; SY1 > 0: pass 1 was split into exactly SY1 parts (1 for the large batch shapes), SY1 = 0: a.sy1 parts.
template <int GL, int NV, int MODEL, bool VEC, int SY1>
__global__ void __launch_bounds__(256)
k_chain(RowArgs a, const float* __restrict__ gQ, const float* __restrict__ ml, const float* __restrict__ pos,
        float* __restrict__ lse, float* __restrict__ G, float* __restrict__ loss_part) {
  constexpr int GPB = 256 / GL;
  constexpr int P = SY1 ? SY1 : MAR_MAX_PARTS;
  __shared__ float lsum[GPB];
  const int grp = threadIdx.x / GL, l = threadIdx.x % GL;
  const int e = blockIdx.x * GPB + grp;
  const int dim = a.dim, dk = a.dk;
  const int sy1 = SY1 ? SY1 : a.sy1;
  const size_t part_rows = (size_t)2 * a.B;
  float le = 0.f;
  if (e < a.n) {
    // every lane of the group merges the parts of both sides (same addresses: one broadcast load each)
    float facu[MAR_MAX_PARTS], facw[MAR_MAX_PARTS];
    const size_t row_u = (size_t)MAR_SIDE_DST * a.B + e, row_w = (size_t)MAR_SIDE_SRC * a.B + e;
    const float lse_u = merge_parts(ml, row_u, part_rows, sy1, facu);
    const float lse_w = merge_parts(ml, row_w, part_rows, sy1, facw);
    const float pe = pos[e];
    if (l == 0) { lse[row_u] = lse_u; lse[row_w] = lse_w; }
    le = -2.f * pe + lse_u + lse_w;
    const float* gu0 = gQ + row_u * dk;
    const float* gw0 = gQ + row_w * dk;
    const size_t pstride = part_rows * dk;
    const float* s_row = a.node_emb + (size_t)a.src[e] * dim;
    const float* r_row = a.rel_emb + (size_t)(MODEL == MAR_MODEL_DOT ? 0 : a.rel[e]) * dim;
    const float* d_row = a.node_emb + (size_t)a.dst[e] * dim;
    float* gs = G + (size_t)e * dk;                              // gradient row of occurrence k is row k
    float* gd = G + ((size_t)a.n + e) * dk;
    float* gr = G + (2 * (size_t)a.n + e) * dk;
    float inv2 = 0.f;
    if (MODEL == MAR_MODEL_TRANSE) { const float dist = -pe; inv2 = dist > 0.f ? 2.f / dist : 0.f; }
    if (VEC && MODEL == MAR_MODEL_COMPLEX) {
      const int h = dim >> 1;
      float2 sr[NV], si[NV], rr[NV], ri[NV], dr[NV], di[NV], ur[NV], ui[NV], wr[NV], wi[NV];
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const int k = 2 * (l + GL * v);
        if (k < h) {
          sr[v] = *reinterpret_cast<const float2*>(s_row + k); si[v] = *reinterpret_cast<const float2*>(s_row + h + k);
          rr[v] = *reinterpret_cast<const float2*>(r_row + k); ri[v] = *reinterpret_cast<const float2*>(r_row + h + k);
          dr[v] = *reinterpret_cast<const float2*>(d_row + k); di[v] = *reinterpret_cast<const float2*>(d_row + h + k);
          ur[v] = ui[v] = wr[v] = wi[v] = make_float2(0.f, 0.f);
#pragma unroll
          for (int p = 0; p < P; ++p) {
            if (SY1 || p < sy1) {
              const float2 a0 = *reinterpret_cast<const float2*>(gu0 + p * pstride + k), a1 = *reinterpret_cast<const float2*>(gu0 + p * pstride + h + k);
              const float2 b0 = *reinterpret_cast<const float2*>(gw0 + p * pstride + k), b1 = *reinterpret_cast<const float2*>(gw0 + p * pstride + h + k);
              ur[v].x += facu[p] * a0.x; ur[v].y += facu[p] * a0.y; ui[v].x += facu[p] * a1.x; ui[v].y += facu[p] * a1.y;
              wr[v].x += facw[p] * b0.x; wr[v].y += facw[p] * b0.y; wi[v].x += facw[p] * b1.x; wi[v].y += facw[p] * b1.y;
            }
          }
        }
      }
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const int k = 2 * (l + GL * v);
        if (k < h) {
          float2 osr, osi, odr, odi, orr, ori;
          chain_complex(sr[v].x, si[v].x, rr[v].x, ri[v].x, dr[v].x, di[v].x, ur[v].x, ui[v].x, wr[v].x, wi[v].x, osr.x, osi.x, odr.x, odi.x, orr.x, ori.x);
          chain_complex(sr[v].y, si[v].y, rr[v].y, ri[v].y, dr[v].y, di[v].y, ur[v].y, ui[v].y, wr[v].y, wi[v].y, osr.y, osi.y, odr.y, odi.y, orr.y, ori.y);
          *reinterpret_cast<float2*>(gs + k) = osr; *reinterpret_cast<float2*>(gs + h + k) = osi;
          *reinterpret_cast<float2*>(gd + k) = odr; *reinterpret_cast<float2*>(gd + h + k) = odi;
          *reinterpret_cast<float2*>(gr + k) = orr; *reinterpret_cast<float2*>(gr + h + k) = ori;
        }
      }
    } else if (VEC) {
      float4 s4[NV], r4[NV], d4[NV], u4[NV], w4[NV];
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const int k = 4 * (l + GL * v);
        if (k < dim) {
          s4[v] = *reinterpret_cast<const float4*>(s_row + k); d4[v] = *reinterpret_cast<const float4*>(d_row + k);
          r4[v] = MODEL == MAR_MODEL_DOT ? make_float4(0.f, 0.f, 0.f, 0.f) : *reinterpret_cast<const float4*>(r_row + k);
          u4[v] = w4[v] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
          for (int p = 0; p < P; ++p) {
            if (SY1 || p < sy1) {
              const float4 a0 = *reinterpret_cast<const float4*>(gu0 + p * pstride + k), b0 = *reinterpret_cast<const float4*>(gw0 + p * pstride + k);
              u4[v].x += facu[p] * a0.x; u4[v].y += facu[p] * a0.y; u4[v].z += facu[p] * a0.z; u4[v].w += facu[p] * a0.w;
              w4[v].x += facw[p] * b0.x; w4[v].y += facw[p] * b0.y; w4[v].z += facw[p] * b0.z; w4[v].w += facw[p] * b0.w;
            }
          }
        }
      }
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const int k = 4 * (l + GL * v);
        if (k < dim) {
          float4 os, od, og;
          chain1<MODEL>(s4[v].x, r4[v].x, d4[v].x, u4[v].x, w4[v].x, inv2, os.x, od.x, og.x);
          chain1<MODEL>(s4[v].y, r4[v].y, d4[v].y, u4[v].y, w4[v].y, inv2, os.y, od.y, og.y);
          chain1<MODEL>(s4[v].z, r4[v].z, d4[v].z, u4[v].z, w4[v].z, inv2, os.z, od.z, og.z);
          chain1<MODEL>(s4[v].w, r4[v].w, d4[v].w, u4[v].w, w4[v].w, inv2, os.w, od.w, og.w);
          *reinterpret_cast<float4*>(gs + k) = os; *reinterpret_cast<float4*>(gd + k) = od;
          if (MODEL != MAR_MODEL_DOT) *reinterpret_cast<float4*>(gr + k) = og;
        }
      }
    } else {
      // any width: one element (ComplEx: one complex element) per lane and step
      auto merged = [&](const float* base, const float (&f)[MAR_MAX_PARTS], int k) {
        float v = 0.f;
#pragma unroll
        for (int p = 0; p < P; ++p) if (SY1 || p < sy1) v += f[p] * base[p * pstride + k];
        return v;
      };
      if (MODEL == MAR_MODEL_COMPLEX) {
        const int h = dim >> 1;
        for (int k = l; k < h; k += GL) {
          chain_complex(s_row[k], s_row[h + k], r_row[k], r_row[h + k], d_row[k], d_row[h + k], merged(gu0, facu, k), merged(gu0, facu, h + k),
                        merged(gw0, facw, k), merged(gw0, facw, h + k), gs[k], gs[h + k], gd[k], gd[h + k], gr[k], gr[h + k]);
        }
      } else {
        for (int k = l; k < dim; k += GL) {
          float os, od, og;
          chain1<MODEL>(s_row[k], MODEL == MAR_MODEL_DOT ? 0.f : r_row[k], d_row[k], merged(gu0, facu, k), merged(gw0, facw, k), inv2, os, od, og);
          gs[k] = os; gd[k] = od;
          if (MODEL != MAR_MODEL_DOT) gr[k] = og;
        }
      }
      for (int k = dim + l; k < dk; k += GL) { gs[k] = 0.f; gd[k] = 0.f; if (MODEL != MAR_MODEL_DOT) gr[k] = 0.f; }
    }
  }
  if (l == 0) lsum[grp] = le;
  __syncthreads();
  if (threadIdx.x == 0) {
    float t = 0.f;
    for (int i = 0; i < GPB; ++i) t += lsum[i];
    loss_part[blockIdx.x] = t;
  }
}

// ------------------------------------------------------------ filtered evaluation -----
// Score f(s, r, d) of one triple by one lane group, in the operation order of the positive score above.
template <int GL, bool VEC>
__device__ __forceinline__ float group_score(int model, int dim, const float* __restrict__ s_row,
                                             const float* __restrict__ r_row, const float* __restrict__ d_row, int l) {
  float acc = 0.f;
  if (VEC && model == MAR_MODEL_COMPLEX) {
    const int h = dim >> 1;
    for (int k = 2 * l; k < h; k += 2 * GL) {
      const float2 sr = *reinterpret_cast<const float2*>(s_row + k), si = *reinterpret_cast<const float2*>(s_row + h + k);
      const float2 rr = *reinterpret_cast<const float2*>(r_row + k), ri = *reinterpret_cast<const float2*>(r_row + h + k);
      const float2 dr = *reinterpret_cast<const float2*>(d_row + k), di = *reinterpret_cast<const float2*>(d_row + h + k);
      const float2 ure = make_float2(sr.x * rr.x - si.x * ri.x, sr.y * rr.y - si.y * ri.y);
      const float2 uim = make_float2(sr.x * ri.x + si.x * rr.x, sr.y * ri.y + si.y * rr.y);
      acc += (ure.x * dr.x + uim.x * di.x) + (ure.y * dr.y + uim.y * di.y);
    }
  } else if (VEC) {
    for (int k = 4 * l; k < dim; k += 4 * GL) {
      const float4 s = *reinterpret_cast<const float4*>(s_row + k), d = *reinterpret_cast<const float4*>(d_row + k);
      float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
      if (model != MAR_MODEL_DOT) r = *reinterpret_cast<const float4*>(r_row + k);
      if (model == MAR_MODEL_DISTMULT) {
        const float4 u = make_float4(s.x * r.x, s.y * r.y, s.z * r.z, s.w * r.w);
        acc += (u.x * d.x + u.y * d.y) + (u.z * d.z + u.w * d.w);
      } else if (model == MAR_MODEL_DOT) {
        acc += (s.x * d.x + s.y * d.y) + (s.z * d.z + s.w * d.w);
      } else {
        const float4 u = make_float4(s.x + r.x, s.y + r.y, s.z + r.z, s.w + r.w);
        const float4 df = make_float4(u.x - d.x, u.y - d.y, u.z - d.z, u.w - d.w);
        acc += (df.x * df.x + df.y * df.y) + (df.z * df.z + df.w * df.w);
      }
    }
  } else if (model == MAR_MODEL_COMPLEX) {
    const int h = dim >> 1;
    for (int k = l; k < h; k += GL) {
      const float sr = s_row[k], si = s_row[h + k], rr = r_row[k], ri = r_row[h + k], dr = d_row[k], di = d_row[h + k];
      const float ure = sr * rr - si * ri, uim = sr * ri + si * rr;
      acc += ure * dr + uim * di;
    }
  } else {
    for (int k = l; k < dim; k += GL) {
      const float s = s_row[k], r = r_row[k], d = d_row[k];
      if (model == MAR_MODEL_DISTMULT) { const float u = s * r; acc += u * d; }
      else if (model == MAR_MODEL_DOT) acc += s * d;
      else { const float u = s + r; const float df = u - d; acc += df * df; }
    }
  }
  acc = group_sum<GL>(acc);
  return model == MAR_MODEL_TRANSE ? -sqrtf(acc) : acc;
}

// One lane group per (edge, corrupted side): takes the listed true candidates that outscore the edge
// out of its rank.
template <int GL, bool VEC>
__global__ void __launch_bounds__(256)
k_filter(RowArgs a, const int64_t* __restrict__ dst_off, const int32_t* __restrict__ dst_ids,
         const int64_t* __restrict__ src_off, const int32_t* __restrict__ src_ids, const float* __restrict__ pos,
         int32_t* __restrict__ rank_dst, int32_t* __restrict__ rank_src) {
  constexpr int GPB = 256 / GL;
  const int grp = threadIdx.x / GL, l = threadIdx.x % GL;
  const int idx = blockIdx.x * GPB + grp;
  if (idx >= 2 * a.n) return;
  const int side = idx >= a.n ? MAR_SIDE_DST : MAR_SIDE_SRC;
  const int e = side == MAR_SIDE_DST ? idx - a.n : idx;
  const int dim = a.dim;
  const float* s_row = a.node_emb + (size_t)a.src[e] * dim;
  const float* r_row = a.rel_emb + (size_t)(a.model == MAR_MODEL_DOT ? 0 : a.rel[e]) * dim;
  const float* d_row = a.node_emb + (size_t)a.dst[e] * dim;
  const float p = pos[e];
  const int64_t* off = side == MAR_SIDE_DST ? dst_off : src_off;
  const int32_t* ids = side == MAR_SIDE_DST ? dst_ids : src_ids;
  int better = 0;
  for (int64_t k = off[e]; k < off[e + 1]; ++k) {
    const float* c_row = a.node_emb + (size_t)ids[k] * dim;
    const float f = side == MAR_SIDE_DST ? group_score<GL, VEC>(a.model, dim, s_row, r_row, c_row, l)
                                         : group_score<GL, VEC>(a.model, dim, c_row, r_row, d_row, l);
    better += f > p ? 1 : 0;
  }
  // The unfiltered rank comes from the matrix cores, this count from the vector ALU: a candidate within rounding
  // of the edge's score can be counted here and not there, so the difference is kept at 1 or above.
  if (l == 0 && better) {
    int32_t* rk = (side == MAR_SIDE_DST ? rank_dst : rank_src) + e;
    const int32_t v = *rk - better;
    *rk = v < 1 ? 1 : v;
  }
}

// ------------------------------------------------- per-row reduce + Adagrad scatter -----
// The gradient rows are summed per table row over the row-sorted order (a stable sort, so a row's
// occurrences are always added in the same order and the sums are bit-reproducible) and the Adagrad
// update (Sec. 5.1; one update per touched row and step) is applied where the sum becomes complete.
struct ReduceArgs {
  float *node_emb, *node_state, *rel_emb, *rel_state;
  const float* G;            // [n_rows][dk] gradient rows
  float* carry;              // [blocks][2][dk] partial sums of segments that cross block borders
  const int32_t* rank_sorted;
  const int32_t* perm;       // position in row-sorted order -> gradient row
  const uint32_t* seg_off;
  const int32_t* uniq;
  int32_t* scalars;          // [2] = number of entries in `owners`
  int32_t* owners;           // blocks in which a segment begins that continues into later blocks
  float* dbg_grad;           // [unique rows][dim] summed gradients (debug output), or NULL
  float* defer_grad;         // [unique rows][dk], or NULL: if set, a node row's summed gradient is stored here and the row is
                             // left alone (its update is applied later, by k_stage_apply); relation rows are updated as usual
  int64_t n_rows;
  int32_t num_nodes, dim, dk;
  float lr, eps;
};

__device__ __forceinline__ void add4(float4& a, const float4& b) { a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w; }

// Four consecutive floats of a table row starting at column `col`.  VEC: rows are 16-byte aligned (dim % 4 == 0).
template <bool VEC> __device__ __forceinline__ float4 load_row4(const float* __restrict__ row, int col, int dim) {
  if (VEC) return *reinterpret_cast<const float4*>(row + col);
  float4 v;
  v.x = col + 0 < dim ? row[col + 0] : 0.f; v.y = col + 1 < dim ? row[col + 1] : 0.f;
  v.z = col + 2 < dim ? row[col + 2] : 0.f; v.w = col + 3 < dim ? row[col + 3] : 0.f;
  return v;
}

template <bool VEC> __device__ __forceinline__ void store_row4(float* __restrict__ row, int col, int dim, const float4& v) {
  if (VEC) { *reinterpret_cast<float4*>(row + col) = v; return; }
  if (col + 0 < dim) row[col + 0] = v.x;
  if (col + 1 < dim) row[col + 1] = v.y;
  if (col + 2 < dim) row[col + 2] = v.z;
  if (col + 3 < dim) row[col + 3] = v.w;
}

__device__ __forceinline__ void table_rows(const ReduceArgs& a, int32_t id, float*& emb, float*& st) {
  if (id < a.num_nodes) { emb = a.node_emb + (size_t)id * a.dim; st = a.node_state + (size_t)id * a.dim; }
  else { emb = a.rel_emb + (size_t)(id - a.num_nodes) * a.dim; st = a.rel_state + (size_t)(id - a.num_nodes) * a.dim; }
}

// state += g^2; theta -= lr * g / (sqrt(state) + eps) on four columns whose old values are th, s0 (Sec. 5.1: Adagrad).
// The one place where the update is spelled out: every kernel that applies it goes through here.
__device__ __forceinline__ void adagrad_math(const float4& g, const float4& th, const float4& s0, float lr, float eps, float4& e1, float4& s1) {
  s1.x = s0.x + g.x * g.x; s1.y = s0.y + g.y * g.y; s1.z = s0.z + g.z * g.z; s1.w = s0.w + g.w * g.w;
  e1.x = th.x - lr * g.x / (sqrtf(s1.x) + eps); e1.y = th.y - lr * g.y / (sqrtf(s1.y) + eps);
  e1.z = th.z - lr * g.z / (sqrtf(s1.z) + eps); e1.w = th.w - lr * g.w / (sqrtf(s1.w) + eps);
}

__device__ __forceinline__ bool row_deferred(const ReduceArgs& a, int32_t id) { return a.defer_grad != nullptr && id < a.num_nodes; }

// Finishes a table row whose summed gradient over four columns is g: Adagrad on the row (old values th, s0), or,
// for a deferred node row, the gradient goes to defer_grad and the table is not touched.
template <bool VEC>
__device__ __forceinline__ void adagrad4(const ReduceArgs& a, int32_t id, float* __restrict__ emb, float* __restrict__ st, int rank, int col,
                                         const float4& g, const float4& th, const float4& s0) {
  if (a.dbg_grad) store_row4<VEC>(a.dbg_grad + (size_t)rank * a.dim, col, a.dim, g);
  if (row_deferred(a, id)) { *reinterpret_cast<float4*>(a.defer_grad + (size_t)rank * a.dk + col) = g; return; }
  float4 s1, e1;
  adagrad_math(g, th, s0, a.lr, a.eps, e1, s1);
  store_row4<VEC>(st, col, a.dim, s1);
  store_row4<VEC>(emb, col, a.dim, e1);
}

// Old values of four columns of a table row; a deferred row is not read.
template <bool VEC>
__device__ __forceinline__ void load_old4(const ReduceArgs& a, int32_t id, const float* emb, const float* st, int col, float4& th, float4& s0) {
  if (row_deferred(a, id)) { th = s0 = make_float4(0.f, 0.f, 0.f, 0.f); return; }
  th = load_row4<VEC>(emb, col, a.dim); s0 = load_row4<VEC>(st, col, a.dim);
}

// A workgroup takes MAR_REDUCE_BLOCK consecutive positions, a group of GL lanes GL of them (a "task"; the
// lanes of a group move one row as float4s, NV per lane).  Each lane first fetches the rank, gradient row,
// segment bounds and table row id of one position of its task, so that no later load depends on another.
// The task's rows are then fetched BATCH at a time -- together with the table row and accumulator row of
// every position at which a segment ends that also began inside the task -- and added up in position
// order; such a segment is finished by the Adagrad update right there.  A segment that crosses the task's
// borders leaves a partial sum in LDS (head: began earlier, tail: continues); the workgroup then chains the
// partials of its tasks in order, finishes the segments that lie inside the workgroup, and writes those
// that cross its own borders to `carry` (slot 0: began in an earlier workgroup, slot 1: continues into the
// next; a workgroup with a slot-1 partial appends itself to `owners`).
template <int GL, int NV, int BATCH, bool VEC>
__global__ void __launch_bounds__(256) k_reduce_apply(ReduceArgs a) {
  constexpr int GPB = 256 / GL;
  __shared__ float4 s_head[GPB][GL * NV], s_tail[GPB][GL * NV];
  __shared__ int s_hs[GPB], s_tf[GPB];       // head: 0 none, 1 ends inside the task, 2 runs through it; tail: 0 / 1
  __shared__ int s_fin[GPB];                 // the head slot of this task holds a finished sum (set by the chaining step)
  const int grp = threadIdx.x / GL, l = threadIdx.x % GL;
  const int64_t P0 = (int64_t)blockIdx.x * MAR_REDUCE_BLOCK;
  const int64_t p0 = P0 + (int64_t)grp * GL;
  const int64_t left = a.n_rows - p0;
  const int cnt = left < 0 ? 0 : (left < GL ? (int)left : GL);
  const int64_t p1 = p0 + cnt;
  const int nq = a.dk >> 2;

  int my_rank = 0, my_row = 0, my_id = 0, my_kind = 0;     // kind: 0 no segment end, 1 end of a segment inside the task,
  int64_t my_lo = 0, my_hi = 0;                            //       2 end of a segment that began before the task
  if (l < cnt) {
    my_rank = a.rank_sorted[p0 + l];
    my_row = a.perm[p0 + l];
    my_lo = a.seg_off[my_rank];
    my_hi = a.seg_off[my_rank + 1];
    my_id = a.uniq[my_rank];
    if (p0 + l == my_hi - 1) my_kind = my_lo >= p0 ? 1 : 2;
  }
  float4 acc[NV];
#pragma unroll
  for (int v = 0; v < NV; ++v) acc[v] = make_float4(0.f, 0.f, 0.f, 0.f);

  for (int i0 = 0; i0 < cnt; i0 += BATCH) {
    float4 g[BATCH][NV], th[BATCH][NV], s0[BATCH][NV];
    int kind[BATCH];
#pragma unroll
    for (int j = 0; j < BATCH; ++j) {
      const int pj = (i0 + j) & (GL - 1);
      const bool valid = i0 + j < cnt;
      const int row = __shfl(my_row, pj, GL);
      const int id = __shfl(my_id, pj, GL);
      kind[j] = valid ? __shfl(my_kind, pj, GL) : 0;
      const float* grow = a.G + (size_t)row * a.dk;
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const int q = l + GL * v;
        g[j][v] = (valid && q < nq) ? *reinterpret_cast<const float4*>(grow + 4 * q) : make_float4(0.f, 0.f, 0.f, 0.f);
      }
      if (kind[j] == 1) {
        float *emb, *st;
        table_rows(a, id, emb, st);
#pragma unroll
        for (int v = 0; v < NV; ++v) {
          const int q = l + GL * v;
          if (q < nq) load_old4<VEC>(a, id, emb, st, 4 * q, th[j][v], s0[j][v]);
        }
      }
    }
#pragma unroll
    for (int j = 0; j < BATCH; ++j) {
      if (i0 + j < cnt) {
#pragma unroll
        for (int v = 0; v < NV; ++v) add4(acc[v], g[j][v]);
        if (kind[j] != 0) {
          const int pj = (i0 + j) & (GL - 1);
          if (kind[j] == 1) {
            float *emb, *st;
            const int32_t fid = __shfl(my_id, pj, GL);
            table_rows(a, fid, emb, st);
            const int rank = __shfl(my_rank, pj, GL);
#pragma unroll
            for (int v = 0; v < NV; ++v) {
              const int q = l + GL * v;
              if (q < nq) adagrad4<VEC>(a, fid, emb, st, rank, 4 * q, acc[v], th[j][v], s0[j][v]);
            }
          } else {
#pragma unroll
            for (int v = 0; v < NV; ++v) s_head[grp][l + GL * v] = acc[v];
          }
#pragma unroll
          for (int v = 0; v < NV; ++v) acc[v] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
      }
    }
  }
  // what is left in acc belongs to the segment of the task's last position, if that segment continues
  int hs = 0, tf = 0;
  if (cnt > 0) {
    const int64_t lo_first = __shfl(my_lo, 0, GL), hi_first = __shfl(my_hi, 0, GL);
    const int64_t lo_last = __shfl(my_lo, cnt - 1, GL), hi_last = __shfl(my_hi, cnt - 1, GL);
    if (lo_first < p0) hs = hi_first <= p1 ? 1 : 2;
    if (hi_last > p1) {
      if (lo_last >= p0) tf = 1;
#pragma unroll
      for (int v = 0; v < NV; ++v) (tf ? s_tail : s_head)[grp][l + GL * v] = acc[v];
    }
  }
  if (l == 0) { s_hs[grp] = hs; s_tf[grp] = tf; s_fin[grp] = 0; }
  __syncthreads();

  // Chain the tasks' partial sums in task order: thread q owns column block q and walks the tasks (LDS only).
  // A segment that ends inside the workgroup and also began inside it leaves its sum in the head slot of the
  // task it ends in (s_fin marks it); those sums are then turned into Adagrad updates by all lane groups at
  // once -- group g takes task g -- so that their table reads do not queue up behind one another.
  const int q = threadIdx.x;
  float4 run = make_float4(0.f, 0.f, 0.f, 0.f);
  bool active = false, inside = false;                     // a segment is open / it began inside this workgroup
  for (int gi = 0; gi < GPB; ++gi) {
    const int h = s_hs[gi];                                // uniform over the workgroup
    if (h) {
      const float4 hv = q < nq ? s_head[gi][q] : make_float4(0.f, 0.f, 0.f, 0.f);
      if (active) add4(run, hv); else { run = hv; active = true; inside = false; }
      if (h == 1) {
        if (inside) {
          if (q < nq) s_head[gi][q] = run;
          if (q == 0) s_fin[gi] = 1;
        } else if (q < nq) {
          *reinterpret_cast<float4*>(a.carry + ((size_t)blockIdx.x * 2 + 0) * a.dk + 4 * q) = run;
        }
        active = false;
      }
    }
    if (s_tf[gi]) {
      run = q < nq ? s_tail[gi][q] : make_float4(0.f, 0.f, 0.f, 0.f);
      active = true; inside = true;
    }
  }
  if (active) {
    if (q < nq) *reinterpret_cast<float4*>(a.carry + ((size_t)blockIdx.x * 2 + (inside ? 1 : 0)) * a.dk + 4 * q) = run;
    if (inside && threadIdx.x == 0) a.owners[atomicAdd(&a.scalars[2], 1)] = (int32_t)blockIdx.x;
  }
  __syncthreads();
  if (s_fin[grp]) {                                        // uniform over the lane group
    const int rank = __shfl(my_rank, 0, GL);               // the segment that ends in task grp is the one its first position belongs to
    float *emb, *st;
    const int32_t fid = __shfl(my_id, 0, GL);
    table_rows(a, fid, emb, st);
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      const int qq = l + GL * v;
      if (qq < nq) {
        float4 th, s0;
        load_old4<VEC>(a, fid, emb, st, 4 * qq, th, s0);
        adagrad4<VEC>(a, fid, emb, st, rank, 4 * qq, s_head[grp][qq], th, s0);
      }
    }
  }
}

// Finishes the segments that span several workgroups of k_reduce_apply: a workgroup of SPAN_WAVES waves takes an
// entry of `owners` (in any order: every entry is a different table row), adds that block's slot-1 partial
// and the slot-0 partials of the following blocks up to the segment's end -- wave w takes every SPAN_WAVES-th,
// FB at a time, then the waves' sums are combined through LDS in wave order: a fixed tree -- and applies
// the Adagrad update.  Block 0 first adds up the per-block loss terms, also in a fixed order.
#define SPAN_WAVES 16
template <int NV, bool VEC>
__global__ void __launch_bounds__(64 * SPAN_WAVES)
k_span_apply(ReduceArgs a, const float* __restrict__ loss_part, int n_loss_part, float* __restrict__ loss_out) {
  constexpr int NT = 64 * SPAN_WAVES;
  __shared__ float4 part[SPAN_WAVES][64 * NV];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (blockIdx.x == 0 && loss_out) {                        // uniform over the workgroup
    // thread t adds terms t, t + NT, ..., then lanes, then the waves in order
    __shared__ float wsum[SPAN_WAVES];
    float t = 0.f;
    for (int i = threadIdx.x; i < n_loss_part; i += NT) t += loss_part[i];
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) t += __shfl_xor(t, o);
    if (lane == 0) wsum[wave] = t;
    __syncthreads();
    if (threadIdx.x == 0) {
      float s = 0.f;
      for (int w = 0; w < SPAN_WAVES; ++w) s += wsum[w];
      *loss_out = s;
    }
  }
  const int nq = a.dk >> 2;
  const int n_owners = a.scalars[2];
  for (int o = blockIdx.x; o < n_owners; o += gridDim.x) {  // uniform over the workgroup
    const int64_t blk = a.owners[o];
    const int64_t pe = (blk + 1) * MAR_REDUCE_BLOCK < a.n_rows ? (blk + 1) * MAR_REDUCE_BLOCK : a.n_rows;
    const int rank = a.rank_sorted[pe - 1];
    const int64_t hi = a.seg_off[rank + 1];
    const int64_t last_blk = (hi - 1) / MAR_REDUCE_BLOCK;
    float4 acc[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      const int q = lane + 64 * v;
      acc[v] = (wave == 0 && q < nq) ? *reinterpret_cast<const float4*>(a.carry + ((size_t)blk * 2 + 1) * a.dk + 4 * q)
                                     : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    constexpr int FB = 4;                                   // partial rows in flight per wave
    for (int64_t t = blk + 1 + wave; t <= last_blk; t += SPAN_WAVES * FB) {
      float4 rows[FB][NV];
#pragma unroll
      for (int j = 0; j < FB; ++j) {
        const int64_t tt = t + SPAN_WAVES * j;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
          const int q = lane + 64 * v;
          rows[j][v] = (tt <= last_blk && q < nq) ? *reinterpret_cast<const float4*>(a.carry + ((size_t)tt * 2) * a.dk + 4 * q)
                                                  : make_float4(0.f, 0.f, 0.f, 0.f);
        }
      }
#pragma unroll
      for (int j = 0; j < FB; ++j) {
#pragma unroll
        for (int v = 0; v < NV; ++v) add4(acc[v], rows[j][v]);
      }
    }
    __syncthreads();                                        // the previous entry's sums have been read
#pragma unroll
    for (int v = 0; v < NV; ++v) part[wave][lane + 64 * v] = acc[v];
    __syncthreads();
    if (wave == 0) {
      float *emb, *st;
      const int32_t fid = a.uniq[rank];
      table_rows(a, fid, emb, st);
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const int q = lane + 64 * v;
        if (q < nq) {
          float4 s = part[0][q], th, s0;
          for (int w = 1; w < SPAN_WAVES; ++w) add4(s, part[w][q]);
          load_old4<VEC>(a, fid, emb, st, 4 * q, th, s0);
          adagrad4<VEC>(a, fid, emb, st, rank, 4 * q, s, th, s0);
        }
      }
    }
  }
}

// ------------------------------------------------ staging for out-of-memory training -----
// Training with the node table outside device memory (Sec. 3: the table lives in CPU memory, batches move through
// gather / transfer / compute / transfer / update stages).  Here the table is pinned host memory that the GPU reads
// and writes directly; a batch's unique node rows are staged into a compact device table (row = rank of the node
// among the batch's unique rows), the step runs on that table with ids replaced by ranks, and the summed node
// gradients are applied to the host table afterwards.
struct StageArgs {
  const float* host_emb;     // [num_nodes][dim] pinned host memory, device-accessible
  float* host_state;         // [num_nodes][dim] (k_stage_apply)
  float* host_emb_rw;        // same table, writable (k_stage_apply)
  float* compact;            // [unique rows][dim] device
  const float* gsum;         // [unique rows][dk] summed gradients per unique row
  const int32_t* uniq;       // ascending unified ids of the batch's rows: the node ids come first
  const int32_t* scalars;    // [1] = number of unique nodes
  const uint32_t* keys0;     // gradient row -> rank
  int32_t *c_src, *c_dst, *c_neg_dst, *c_neg_src;   // ids replaced by ranks
  int32_t n, cn, roles, sy2, dim, dk;
  float lr, eps;
};

// Ranks in place of node ids, in the layout the step's entry arrays have.
__global__ void __launch_bounds__(256) k_stage_ids(StageArgs a) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t n3 = (int64_t)a.roles * a.n;
  if (i < a.n) { a.c_src[i] = (int32_t)a.keys0[i]; a.c_dst[i] = (int32_t)a.keys0[a.n + i]; }
  if (i < a.cn) {
    a.c_neg_dst[i] = (int32_t)a.keys0[n3 + i * a.sy2];
    a.c_neg_src[i] = (int32_t)a.keys0[n3 + ((int64_t)a.cn + i) * a.sy2];
  }
}

#define STAGE_ROWS 4   // rows in flight per lane group

// compact[rank] = host table row of the rank-th unique node.  One lane group per STAGE_ROWS rows.
template <int GL, int NV, bool VEC>
__global__ void __launch_bounds__(256) k_stage_gather(StageArgs a) {
  constexpr int GPB = 256 / GL;
  const int grp = threadIdx.x / GL, l = threadIdx.x % GL;
  const int un = a.scalars[1];
  const int r0 = (blockIdx.x * GPB + grp) * STAGE_ROWS;
  if (r0 >= un) return;
  float4 v4[STAGE_ROWS][NV];
#pragma unroll
  for (int j = 0; j < STAGE_ROWS; ++j) {
    const float* row = a.host_emb + (size_t)a.uniq[min(r0 + j, un - 1)] * a.dim;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      const int k = 4 * (l + GL * v);
      if (k < a.dim) v4[j][v] = load_row4<VEC>(row, k, a.dim);
    }
  }
#pragma unroll
  for (int j = 0; j < STAGE_ROWS; ++j) {
    if (r0 + j < un) {
      float* out = a.compact + (size_t)(r0 + j) * a.dim;
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const int k = 4 * (l + GL * v);
        if (k < a.dim) store_row4<VEC>(out, k, a.dim, v4[j][v]);
      }
    }
  }
}

// Adagrad on the host table rows of the batch's unique nodes with the summed gradients the step left in gsum
// (Sec. 3, last stage: the update is applied to whatever the table holds now, in batch order).
template <int GL, int NV, bool VEC>
__global__ void __launch_bounds__(256) k_stage_apply(StageArgs a) {
  constexpr int GPB = 256 / GL;
  const int grp = threadIdx.x / GL, l = threadIdx.x % GL;
  const int un = a.scalars[1];
  const int r0 = (blockIdx.x * GPB + grp) * STAGE_ROWS;
  if (r0 >= un) return;
  float4 th[STAGE_ROWS][NV], s0[STAGE_ROWS][NV], g[STAGE_ROWS][NV];
  size_t off[STAGE_ROWS];
#pragma unroll
  for (int j = 0; j < STAGE_ROWS; ++j) {
    const int r = min(r0 + j, un - 1);
    off[j] = (size_t)a.uniq[r] * a.dim;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      const int k = 4 * (l + GL * v);
      if (k < a.dim) {
        th[j][v] = load_row4<VEC>(a.host_emb_rw + off[j], k, a.dim);
        s0[j][v] = load_row4<VEC>(a.host_state + off[j], k, a.dim);
        g[j][v] = *reinterpret_cast<const float4*>(a.gsum + (size_t)r * a.dk + k);
      }
    }
  }
#pragma unroll
  for (int j = 0; j < STAGE_ROWS; ++j) {
    if (r0 + j < un) {
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const int k = 4 * (l + GL * v);
        if (k < a.dim) {
          float4 e1, s1;
          adagrad_math(g[j][v], th[j][v], s0[j][v], a.lr, a.eps, e1, s1);
          store_row4<VEC>(a.host_state + off[j], k, a.dim, s1);
          store_row4<VEC>(a.host_emb_rw + off[j], k, a.dim, e1);
        }
      }
    }
  }
}

// ------------------------------------------------------------------- launchers -----
static RowArgs row_args(const mar_ctx* c, const MarBatch& b) {
  const MarDims& d = c->dm;
  RowArgs a;
  a.node_emb = c->node_emb; a.rel_emb = c->rel_emb;
  a.src = b.src; a.rel = b.rel; a.dst = b.dst; a.neg_src = b.neg_src; a.neg_dst = b.neg_dst;
  a.n = b.n; a.cn = b.cn; a.B = d.B; a.C = d.C; a.N = d.N; a.S = d.S; a.dim = d.dim; a.dk = d.dk; a.model = c->cfg.model;
  a.n_occ = b.n_occ; a.num_nodes = (int32_t)d.num_nodes;
  a.sy1 = d.sy1; a.sy2 = d.sy2; a.roles = d.roles;
  return a;
}

hipError_t mar_launch_prep(const mar_ctx* c, const MarBatch& b, float* pos_out, int images, hipStream_t st) {
  const MarLayout& L = c->L;
  RowArgs a = row_args(c, b);
  const SplitImages qi = sp_images(images ? L.Qimg : nullptr, a.dk, c->dm.S), ki = sp_images(images ? L.Kimg : nullptr, a.dk, c->dm.N);
  const int GL = mar_lane_group(a.dk), gpb = 256 / GL;
  const int nbB = (b.n + gpb * PREP_EDGES - 1) / (gpb * PREP_EDGES);
  const int nbC = (2 * b.cn + gpb * PREP_NEGS - 1) / (gpb * PREP_NEGS);
  const dim3 grid(nbB + nbC), blk(256);
#define PREP3(GLV, NVV, V, M) hipLaunchKernelGGL((k_prep<GLV, NVV, V, M>), grid, blk, 0, st, a, nbB, L.Q, L.Km, L.qq, L.kk, L.pos, pos_out, qi, ki)
#define PREP(GLV, NVV, V) do { switch (a.model) { \
    case MAR_MODEL_DISTMULT: PREP3(GLV, NVV, V, MAR_MODEL_DISTMULT); break; \
    case MAR_MODEL_COMPLEX: PREP3(GLV, NVV, V, MAR_MODEL_COMPLEX); break; \
    case MAR_MODEL_TRANSE: PREP3(GLV, NVV, V, MAR_MODEL_TRANSE); break; \
    default: PREP3(GLV, NVV, V, MAR_MODEL_DOT); break; } } while (0)
  // lanes x float4s per lane cover a row (ComplEx: lanes x float2s cover half a row)
  if (a.dim % 4 == 0) {
    if (GL == 16) PREP(16, 1, true); else if (GL == 32) PREP(32, 1, true); else if (a.dk <= 256) PREP(64, 1, true); else PREP(64, 2, true);
  } else {
    if (GL == 16) PREP(16, 1, false); else if (GL == 32) PREP(32, 1, false); else PREP(64, 1, false);
  }
#undef PREP
#undef PREP3
  return hipGetLastError();
}

hipError_t mar_launch_filter(const mar_ctx* c, const MarBatch& b, const int64_t* dst_off, const int32_t* dst_ids,
                             const int64_t* src_off, const int32_t* src_ids, const float* pos, int32_t* rank_dst,
                             int32_t* rank_src, hipStream_t st) {
  RowArgs a = row_args(c, b);
  const int GL = mar_lane_group(a.dk), gpb = 256 / GL;
  const dim3 grid((2 * b.n + gpb - 1) / gpb), blk(256);
#define FILT(GLV, V) hipLaunchKernelGGL((k_filter<GLV, V>), grid, blk, 0, st, a, dst_off, dst_ids, src_off, src_ids, pos, rank_dst, rank_src)
  if (a.dim % 4 == 0) { if (GL == 16) FILT(16, true); else if (GL == 32) FILT(32, true); else FILT(64, true); }
  else { if (GL == 16) FILT(16, false); else if (GL == 32) FILT(32, false); else FILT(64, false); }
#undef FILT
  return hipGetLastError();
}

template <int GL, int NV, int MODEL>
static void launch_chain(const RowArgs& a, const MarLayout& L, dim3 grid, hipStream_t st) {
#define CHAIN(V, S) hipLaunchKernelGGL((k_chain<GL, NV, MODEL, V, S>), grid, dim3(256), 0, st, a, L.gQ, L.ml, L.pos, L.lse, L.G, L.loss_part)
  if (a.dim % 4 == 0) { if (a.sy1 == 1) CHAIN(true, 1); else if (a.sy1 == 2) CHAIN(true, 2); else CHAIN(true, 0); }
  else CHAIN(false, 0);
#undef CHAIN
}

template <int GL, int NV>
static void launch_chain_model(const RowArgs& a, const MarLayout& L, dim3 grid, hipStream_t st) {
  switch (a.model) {
    case MAR_MODEL_DISTMULT: launch_chain<GL, NV, MAR_MODEL_DISTMULT>(a, L, grid, st); break;
    case MAR_MODEL_COMPLEX:  launch_chain<GL, NV, MAR_MODEL_COMPLEX>(a, L, grid, st); break;
    case MAR_MODEL_TRANSE:   launch_chain<GL, NV, MAR_MODEL_TRANSE>(a, L, grid, st); break;
    default:                 launch_chain<GL, NV, MAR_MODEL_DOT>(a, L, grid, st); break;
  }
}

hipError_t mar_launch_chain(const mar_ctx* c, const MarBatch& b, hipStream_t st) {
  const MarLayout& L = c->L;
  RowArgs a = row_args(c, b);
  const int GL = mar_lane_group(a.dk), gpb = 256 / GL;
  const dim3 grid((b.n + gpb - 1) / gpb);
  // lanes x float4s per lane cover a row (ComplEx: lanes x float2s cover half a row)
  if (GL == 16) launch_chain_model<16, 1>(a, L, grid, st);
  else if (GL == 32) launch_chain_model<32, 1>(a, L, grid, st);
  else if (a.dk <= 256) launch_chain_model<64, 1>(a, L, grid, st);
  else launch_chain_model<64, 2>(a, L, grid, st);
  return hipGetLastError();
}

hipError_t mar_launch_reduce(const mar_ctx* c, const MarBatch& b, float* loss_out, float* dbg_grad, float* defer_grad, hipStream_t st) {
  const MarLayout& L = c->L;
  const MarDims& d = c->dm;
  ReduceArgs a;
  a.node_emb = c->node_emb; a.node_state = c->node_state; a.rel_emb = c->rel_emb; a.rel_state = c->rel_state;
  a.G = L.G; a.carry = L.carry; a.rank_sorted = L.rank_sorted; a.perm = L.perm; a.seg_off = L.seg_off; a.uniq = L.uniq;
  a.scalars = L.scalars; a.owners = L.owners; a.dbg_grad = dbg_grad; a.defer_grad = defer_grad; a.n_rows = b.n_pos;
  a.num_nodes = (int32_t)d.num_nodes; a.dim = d.dim; a.dk = d.dk; a.lr = c->cfg.lr; a.eps = c->cfg.eps;
  const int64_t blocks = (b.n_pos + MAR_REDUCE_BLOCK - 1) / MAR_REDUCE_BLOCK;
  const dim3 grid((unsigned)blocks), grids((unsigned)(blocks < 512 ? blocks : 512)), blk(256), blks(64 * SPAN_WAVES);
  const int GL = mar_lane_group(d.dk), gpb = 256 / GL;
  const int n_loss_part = (b.n + gpb - 1) / gpb;
  const bool vec = d.dim % 4 == 0;
#define RED(GLV, NVV, BT) do { \
    if (vec) hipLaunchKernelGGL((k_reduce_apply<GLV, NVV, BT, true>), grid, blk, 0, st, a); \
    else hipLaunchKernelGGL((k_reduce_apply<GLV, NVV, BT, false>), grid, blk, 0, st, a); } while (0)
  if (GL == 16) RED(16, 1, 8); else if (GL == 32) RED(32, 1, 8); else if (d.dk <= 256) RED(64, 1, 8); else RED(64, 2, 4);
#undef RED
  if (d.dk <= 256) {
    if (vec) hipLaunchKernelGGL((k_span_apply<1, true>), grids, blks, 0, st, a, L.loss_part, n_loss_part, loss_out);
    else hipLaunchKernelGGL((k_span_apply<1, false>), grids, blks, 0, st, a, L.loss_part, n_loss_part, loss_out);
  } else {
    if (vec) hipLaunchKernelGGL((k_span_apply<2, true>), grids, blks, 0, st, a, L.loss_part, n_loss_part, loss_out);
    else hipLaunchKernelGGL((k_span_apply<2, false>), grids, blks, 0, st, a, L.loss_part, n_loss_part, loss_out);
  }
  return hipGetLastError();
}

static StageArgs stage_args(const mar_ctx* c, const MarBatch& b, const MarStage& sg) {
  const MarDims& d = c->dm;
  StageArgs a;
  a.host_emb = sg.host_emb; a.host_emb_rw = sg.host_emb; a.host_state = sg.host_state;
  a.compact = sg.compact; a.gsum = sg.gsum; a.uniq = c->L.uniq; a.scalars = c->L.scalars; a.keys0 = c->L.keys0;
  a.c_src = sg.c_src; a.c_dst = sg.c_dst; a.c_neg_dst = sg.c_neg_dst; a.c_neg_src = sg.c_neg_src;
  a.n = b.n; a.cn = b.cn; a.roles = d.roles; a.sy2 = d.sy2; a.dim = d.dim; a.dk = d.dk;
  a.lr = c->cfg.lr; a.eps = c->cfg.eps;
  return a;
}

// most unique nodes a batch can have: the grids of the staging kernels are sized for it, the kernels read the count
static int64_t stage_rows_max(const mar_ctx* c, const MarBatch& b) {
  const int64_t occ = 2 * (int64_t)b.n + 2 * (int64_t)b.cn;
  return occ < c->dm.num_nodes ? occ : c->dm.num_nodes;
}

#define STAGE_LAUNCH(KERNEL) do { \
    const int GL = mar_lane_group(a.dk), gpb = 256 / GL; \
    const dim3 grid((unsigned)((stage_rows_max(c, b) + gpb * STAGE_ROWS - 1) / (gpb * STAGE_ROWS))), blk(256); \
    const bool vec = a.dim % 4 == 0; \
    if (GL == 16) { if (vec) hipLaunchKernelGGL((KERNEL<16, 1, true>), grid, blk, 0, st, a); else hipLaunchKernelGGL((KERNEL<16, 1, false>), grid, blk, 0, st, a); } \
    else if (GL == 32) { if (vec) hipLaunchKernelGGL((KERNEL<32, 1, true>), grid, blk, 0, st, a); else hipLaunchKernelGGL((KERNEL<32, 1, false>), grid, blk, 0, st, a); } \
    else if (a.dk <= 256) { if (vec) hipLaunchKernelGGL((KERNEL<64, 1, true>), grid, blk, 0, st, a); else hipLaunchKernelGGL((KERNEL<64, 1, false>), grid, blk, 0, st, a); } \
    else { if (vec) hipLaunchKernelGGL((KERNEL<64, 2, true>), grid, blk, 0, st, a); else hipLaunchKernelGGL((KERNEL<64, 2, false>), grid, blk, 0, st, a); } \
  } while (0)

hipError_t mar_launch_stage_in(const mar_ctx* c, const MarBatch& b, const MarStage& sg, hipStream_t st) {
  StageArgs a = stage_args(c, b, sg);
  const int64_t work = b.n > b.cn ? b.n : b.cn;
  hipLaunchKernelGGL(k_stage_ids, dim3((unsigned)((work + 255) / 256)), dim3(256), 0, st, a);
  STAGE_LAUNCH(k_stage_gather);
  return hipGetLastError();
}

hipError_t mar_launch_stage_out(const mar_ctx* c, const MarBatch& b, const MarStage& sg, hipStream_t st) {
  StageArgs a = stage_args(c, b, sg);
  STAGE_LAUNCH(k_stage_apply);
  return hipGetLastError();
}

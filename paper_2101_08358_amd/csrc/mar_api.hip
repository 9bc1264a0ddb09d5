// C ABI of the training-step library: argument checks, workspace carve-up, launch order.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <new>

#include "mar_common.h"

static thread_local char g_err[512] = "";

void mar_set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

extern "C" const char* mar_last_error(const mar_ctx*) { return g_err; }

static int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

static int hip_fail(hipError_t e, const char* what) {
  return fail(MAR_EHIP, "%s: %s", what, hipGetErrorString(e));
}

// ------------------------------------------------------------------ configuration -----
#ifndef MAR_FLASH_TARGET_WGS1
#define MAR_FLASH_TARGET_WGS1 640
#endif
#ifndef MAR_FLASH_TARGET_WGS2
#define MAR_FLASH_TARGET_WGS2 640
#endif

static int check_config(const mar_config* cfg, MarDims* d) {
  if (!cfg) return fail(MAR_EINVAL, "config is NULL");
  if (cfg->num_nodes < 1 || cfg->num_rels < 1) return fail(MAR_EINVAL, "num_nodes and num_rels must be >= 1");
  if (cfg->num_nodes + (int64_t)cfg->num_rels >= ((int64_t)1 << 31))
    return fail(MAR_ERANGE, "num_nodes + num_rels must be below 2^31");
  if (cfg->model < MAR_MODEL_DISTMULT || cfg->model > MAR_MODEL_DOT) return fail(MAR_EINVAL, "unknown model %d", cfg->model);
  if (cfg->dim < 1 || cfg->dim > MAR_MAX_DIM) return fail(MAR_ERANGE, "dim %d outside 1..%d", cfg->dim, MAR_MAX_DIM);
  if (cfg->model == MAR_MODEL_COMPLEX && (cfg->dim & 1)) return fail(MAR_EINVAL, "ComplEx needs an even dim");
  if (cfg->precision != MAR_PRECISION_FP32 && cfg->precision != MAR_PRECISION_SPLIT_BF16) return fail(MAR_EINVAL, "unknown precision %d", cfg->precision);
  if (cfg->precision == MAR_PRECISION_SPLIT_BF16 && cfg->model == MAR_MODEL_TRANSE)
    return fail(MAR_EINVAL, "the split-precision contraction serves the bilinear models (DistMult, ComplEx, Dot) only");
  if (cfg->reserved != 0) return fail(MAR_EINVAL, "reserved must be 0");
  if (cfg->batch_size < 1 || cfg->num_chunks < 1 || cfg->negs_per_chunk < 1)
    return fail(MAR_EINVAL, "batch_size, num_chunks and negs_per_chunk must be >= 1");
  if (cfg->batch_size % cfg->num_chunks) return fail(MAR_ERANGE, "batch_size must be a multiple of num_chunks");
  if (cfg->deg_negs_per_chunk < 0 || cfg->deg_negs_per_chunk > cfg->negs_per_chunk)
    return fail(MAR_EINVAL, "deg_negs_per_chunk outside 0..negs_per_chunk");
  if (!(cfg->lr > 0.f) || !(cfg->eps >= 0.f)) return fail(MAR_EINVAL, "lr must be > 0 and eps >= 0");
  const int64_t cn = (int64_t)cfg->num_chunks * cfg->negs_per_chunk;
  const int roles = cfg->model == MAR_MODEL_DOT ? 2 : 3;
  const int64_t n_occ = roles * (int64_t)cfg->batch_size + 2 * cn;
  if (3 * (int64_t)cfg->batch_size + 2 * cn >= ((int64_t)1 << 30)) return fail(MAR_ERANGE, "batch too large: 3*batch_size + 2*chunks*negatives must be below 2^30");
  d->dim = cfg->dim;
  d->dk = (cfg->dim + 3) & ~3;
  d->B = cfg->batch_size; d->C = cfg->num_chunks; d->S = cfg->batch_size / cfg->num_chunks;
  d->N = cfg->negs_per_chunk; d->Ndeg = cfg->deg_negs_per_chunk; d->roles = roles;
  d->num_nodes = cfg->num_nodes; d->num_rels = cfg->num_rels;
  d->n_occ_max = n_occ;
  const int64_t ids = cfg->num_nodes + cfg->num_rels;
  d->u_max = ids < n_occ ? ids : n_occ;
  d->ipw_log2 = ids <= ((int64_t)1 << 22) ? 2 : 5;       // small id spaces: one byte per id, no atomics
  d->nwords = (ids + (1 << d->ipw_log2) - 1) >> d->ipw_log2;
  if (!mar_flash_supported(d->dk)) return fail(MAR_ERANGE, "row width %d not supported by the contraction kernels", d->dk);
  d->split = cfg->precision == MAR_PRECISION_SPLIT_BF16;
  if (d->split && !mar_split_supported(d->dk)) return fail(MAR_ERANGE, "row width %d not supported by the split-precision kernels", d->dk);
  // The contraction kernels address one chunk-side's rows of either operand, and its block of weights, with 32-bit
  // byte offsets.
  {
    const int64_t rows = d->S > d->N ? d->S : d->N;
    const int64_t tp = (d->N + 127) & ~(int64_t)127, tr_ = (d->S + 63) & ~(int64_t)63;
    if (rows * d->dk * 4 >= ((int64_t)1 << 31) || tp * tr_ * 4 >= ((int64_t)1 << 31))
      return fail(MAR_ERANGE, "chunk too large: rows x row bytes of a chunk's edges or negatives, and chunk edges x negatives x 4, must be below 2^31");
    if (d->split && ((rows + 31) / 32) * (int64_t)mar_split_image_bytes(d->dk) >= ((int64_t)1 << 31))
      return fail(MAR_ERANGE, "chunk too large for the split-precision operand images (2^31 bytes per chunk and side)");
  }
  const int sp = d->split;
  auto stripe_rows = [&](int pass) { return sp ? mar_split_stripe_rows(d->dk, pass) : mar_flash_stripe_rows(d->dk, pass); };
  auto tile_rows = [&](int pass) { return sp ? mar_split_tile_rows() : mar_flash_tile_rows(d->dk, pass); };
  auto wgs_per_cu = [&](int pass) { return sp ? mar_split_wgs_per_cu(d->dk, pass) : mar_flash_wgs_per_cu(d->dk, pass); };
  // Small batches give too few (chunk-side, 64-row stripe) workgroups to fill 256 CUs: let several
  // workgroups share a stripe, each streaming a slice of the other matrix, until a pass has at least
  // MAR_FLASH_TARGET_WGS workgroups (measured best for a 10,000-edge batch; the 50,000-edge shapes have
  // enough stripes and are not split).
  // Split precision: into how many parts to cut the (chunk-side, stripe) units beyond the last whole round.  The
  // units are fewer and longer than the fp32 passes', and the remainder often exceeds half a round, so the parts may
  // take several rounds of their own; every part beyond the first costs a write and a read of the stripes' output
  // rows.  Estimated in microseconds from the rates these passes reach (about 600 TFLOP/s of bf16 work over all
  // workgroup slots, 4.5 TB/s of memory traffic): the time of the last rounds plus the merge.
  auto split_parts = [&](long rem_units, long slots, long ntiles, int sr, int n_y, long rows_per_cs) -> long {
    const double unit_us = 12.0 * sr * (double)n_y * d->dk * (double)slots / 6.0e8;
    const double rows = (double)rem_units / (double)((rows_per_cs + sr - 1) / sr) * (double)rows_per_cs;
    long k = 1;
    double best = 1e30;
    for (long kk = 1; kk <= MAR_MAX_PARTS && kk <= ntiles; ++kk) {
      const double cost = (double)((rem_units * kk + slots - 1) / slots) / (double)kk * unit_us
                        + (double)(kk - 1) * rows * d->dk * 8.0 / 4.5e6;
      if (cost < best) { best = cost; k = kk; }
    }
    return k;
  };
  auto split = [&](int pass, int n_x, int n_y, int32_t* sy, int32_t* tps) {
    const long target = pass == 1 ? MAR_FLASH_TARGET_WGS1 : MAR_FLASH_TARGET_WGS2;
    const int sr = stripe_rows(pass);
    const long wgs = 2L * d->C * ((n_x + sr - 1) / sr);
    const int ty = tile_rows(pass);
    const int ntiles = (n_y + ty - 1) / ty;
    long want = (target + wgs - 1) / wgs;
    if (want > 8) want = 8;
    if (want > ntiles) want = ntiles;
    if (want < 1) want = 1;
    *tps = (int32_t)((ntiles + want - 1) / want);
    *sy = (int32_t)((ntiles + *tps - 1) / *tps);
  };
  split(1, d->S, d->N, &d->sy1, &d->tps1);
  split(2, d->N, d->S, &d->sy2, &d->tps2);
  // Large batches: the (chunk-side, stripe) units of pass 1 rarely fill a whole number of rounds of the chip's
  // workgroup slots (256 CUs x workgroups per CU), and the last, partly filled round costs as much time as a full
  // one.  Chunk-sides are dealt to the 8 XCDs in groups of 8; the groups beyond the last whole round have every
  // stripe split into rem_k parts (each streaming rem_tps tiles), so that the last round is short.
  d->rem_cs0 = 2 * d->C; d->rem_k = 1; d->rem_tps = 0; d->rem_rows = 0;
  if (d->sy1 == 1) {
    const long slots = 256L * wgs_per_cu(1);
    const int sr1 = stripe_rows(1);
    const long nstripes = (d->S + sr1 - 1) / sr1, groups = (2L * d->C + 7) / 8, per_group = 8 * nstripes;
    const int ty = tile_rows(1);
    const long ntiles = (d->N + ty - 1) / ty;
    const long full_rounds = groups * per_group / slots;
    const long whole_groups = full_rounds * slots / per_group;
    if (full_rounds >= 1 && whole_groups < groups) {
      const long rem_units = (2L * d->C - 8 * whole_groups) * nstripes;
      long k = slots / rem_units;
      if (k > MAR_MAX_PARTS) k = MAR_MAX_PARTS;
      if (k > ntiles) k = ntiles;
      if (sp) k = split_parts(rem_units, slots, ntiles, sr1, d->N, nstripes * sr1);
      if (k >= 2) {
        d->rem_cs0 = (int32_t)(8 * whole_groups);
        d->rem_tps = (int32_t)((ntiles + k - 1) / k);
        d->rem_k = (int32_t)((ntiles + d->rem_tps - 1) / d->rem_tps);
        d->rem_rows = (int64_t)(2 * d->C - d->rem_cs0) * ((d->S + 63) & ~63);
      }
    }
  }
  d->rem2_cs0 = 2 * d->C; d->rem2_k = 1; d->rem2_tps = 0; d->rem2_rows = 0;
  if (sp && d->sy2 == 1) {                                 // the same for pass 2 (split precision only)
    const long slots = 256L * wgs_per_cu(2);
    const int sr2 = stripe_rows(2);
    const long nstripes = (d->N + sr2 - 1) / sr2, groups = (2L * d->C + 7) / 8, per_group = 8 * nstripes;
    const long ntiles = (d->S + tile_rows(2) - 1) / tile_rows(2);
    const long full_rounds = groups * per_group / slots;
    const long whole_groups = full_rounds * slots / per_group;
    if (full_rounds >= 1 && whole_groups < groups) {
      const long rem_units = (2L * d->C - 8 * whole_groups) * nstripes;
      const long k = split_parts(rem_units, slots, ntiles, sr2, d->S, nstripes * sr2);
      if (k >= 2) {
        d->rem2_cs0 = (int32_t)(8 * whole_groups);
        d->rem2_tps = (int32_t)((ntiles + k - 1) / k);
        d->rem2_k = (int32_t)((ntiles + d->rem2_tps - 1) / d->rem2_tps);
        d->rem2_rows = (int64_t)(2 * d->C - d->rem2_cs0) * (nstripes * sr2);
      }
    }
  }
  d->n_pos_max = roles * (int64_t)cfg->batch_size + 2 * cn * d->sy2;
  // Sort keys are ranks below u_max: as few passes as digits of at most MAR_SORT_MAX_BITS bits allow.
  int nbits = 1;
  while (((int64_t)1 << nbits) < d->u_max) ++nbits;
  d->sort_passes = (nbits + MAR_SORT_MAX_BITS - 1) / MAR_SORT_MAX_BITS;
  d->sort_bits = (nbits + d->sort_passes - 1) / d->sort_passes;
  // score pairs x row width per step: above ~2e9 the contraction passes are long enough to hide the index build
  d->index_after_gather = (double)cfg->batch_size * cfg->negs_per_chunk * d->dk >= 2.0e9;
  return MAR_OK;
}

// Carves the workspace; with base == NULL only measures.
static size_t carve(const MarDims& d, char* base, MarLayout* L) {
  size_t off = 0;
  auto take = [&](size_t bytes) -> void* {
    void* p = base ? base + off : nullptr;
    off += (bytes + 255) & ~(size_t)255;
    return p;
  };
  const size_t n_pos = (size_t)d.n_pos_max, u1 = (size_t)d.u_max + 1;
  const size_t B = d.B, CN = (size_t)d.C * d.N, dk = d.dk;
  const size_t scan_elems = (size_t)d.nwords > u1 ? (size_t)d.nwords : u1;
  const size_t blocks = (n_pos + MAR_REDUCE_BLOCK - 1) / MAR_REDUCE_BLOCK;
  const size_t tiles = (n_pos + MAR_SORT_TILE - 1) / MAR_SORT_TILE;
  MarLayout l;
  l.scalars = (int32_t*)take(16 * 4);
  l.bitmap = (uint32_t*)take((size_t)d.nwords * 4);
  l.word_prefix = (uint32_t*)take((size_t)d.nwords * 4);
  l.bsum = (uint32_t*)take((scan_elems / 4096 + 2) * 4);
  l.uniq = (int32_t*)take(u1 * 4);
  l.seg_off = (uint32_t*)take((u1 + 1) * 4);
  l.keys0 = (uint32_t*)take(n_pos * 4);
  for (int i = 0; i < 2; ++i) {
    l.kbuf[i] = (uint32_t*)take(d.sort_passes > i + 1 ? n_pos * 4 : 0);
    l.vbuf[i] = (int32_t*)take(d.sort_passes > i + 1 ? n_pos * 4 : 0);
  }
  l.hist = (uint32_t*)take((tiles << d.sort_bits) * 4);
  l.perm = (int32_t*)take(n_pos * 4);
  l.rank_sorted = (int32_t*)take(n_pos * 4);
  l.owners = (int32_t*)take(blocks * 4);
  l.Q = (float*)take(2 * B * dk * 4);
  l.Km = (float*)take(2 * CN * dk * 4);
  l.qq = (float*)take(2 * B * 4);
  l.kk = (float*)take(2 * CN * 4);
  l.pos = (float*)take(B * 4);
  l.lse = (float*)take(2 * B * 4);
  l.gQ = (float*)take((size_t)d.sy1 * 2 * B * dk * 4);
  l.ml = (float*)take((size_t)d.sy1 * 2 * B * 2 * 4);
  l.gQx = (float*)take((size_t)(d.rem_k - 1) * (size_t)d.rem_rows * dk * 4);
  l.mlx = (float*)take((size_t)(d.rem_k - 1) * (size_t)d.rem_rows * 2 * 4);
  // the split-precision passes keep no weights: pass 2 computes the scores again
  l.T = (float*)take(d.split ? 0 : 2 * (size_t)d.C * (size_t)((d.S + 63) & ~63) * (size_t)((d.N + 127) & ~127) * 4);
  l.R = (float*)take(d.split ? 0 : 2 * (size_t)d.C * (size_t)((d.S + 63) & ~63) * (size_t)(((d.N + 127) & ~127) / 16) * 4);
  l.Kimg = (char*)take(d.split ? 2 * (size_t)d.C * (size_t)((d.N + 31) / 32) * mar_split_image_bytes(d.dk) : 0);
  l.Qimg = (char*)take(d.split ? 2 * (size_t)d.C * (size_t)((d.S + 31) / 32) * mar_split_image_bytes(d.dk) : 0);
  l.Gx = (float*)take((size_t)(d.rem2_k - 1) * (size_t)d.rem2_rows * dk * 4);
  l.G = (float*)take(n_pos * dk * 4);
  l.carry = (float*)take(blocks * 2 * dk * 4);
  l.loss_part = (float*)take((B / 4 + 2) * 4);
  l.metric_part = take((size_t)MAR_METRIC_MAX_PARTS * MAR_METRIC_PART_BYTES);
  if (L) *L = l;
  return off;
}

extern "C" int mar_workspace_bytes(const mar_config* cfg, size_t* out_bytes) {
  MarDims d;
  const int rc = check_config(cfg, &d);
  if (rc) return rc;
  if (!out_bytes) return fail(MAR_EINVAL, "out_bytes is NULL");
  *out_bytes = carve(d, nullptr, nullptr);
  return MAR_OK;
}

extern "C" int mar_init_tables(const mar_config* cfg, float* node_emb, float* node_state, float* rel_emb,
                               float* rel_state, void* workspace, size_t workspace_bytes, int fill,
                               void* hip_stream, mar_ctx** out) {
  MarDims d;
  const int rc = check_config(cfg, &d);
  if (rc) return rc;
  if (!out) return fail(MAR_EINVAL, "out is NULL");
  if (!node_emb || !node_state || !rel_emb || !rel_state) return fail(MAR_EINVAL, "a table pointer is NULL");
  if (((uintptr_t)node_emb | (uintptr_t)node_state | (uintptr_t)rel_emb | (uintptr_t)rel_state) & 15)
    return fail(MAR_EINVAL, "table pointers must be 16-byte aligned");
  if (!workspace || ((uintptr_t)workspace & 255)) return fail(MAR_EINVAL, "workspace must be non-NULL and 256-byte aligned");
  const size_t need = carve(d, nullptr, nullptr);
  if (workspace_bytes < need) return fail(MAR_ENOMEM, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
  { const hipError_t e_ = mar_flash_prepare(); if (e_ != hipSuccess) return hip_fail(e_, "kernel attributes"); }
  { const hipError_t e_ = mar_split_prepare(); if (e_ != hipSuccess) return hip_fail(e_, "kernel attributes"); }
  mar_ctx* c = new (std::nothrow) mar_ctx();
  if (!c) return fail(MAR_ENOMEM, "out of host memory");
  c->cfg = *cfg; c->dm = d;
  c->node_emb = node_emb; c->node_state = node_state; c->rel_emb = rel_emb; c->rel_state = rel_state;
  c->workspace = workspace; c->workspace_bytes = workspace_bytes;
  carve(d, (char*)workspace, &c->L);
  c->bitmap_dirty = 0; c->prof_max = 0; c->prof_steps = 0; c->prof_mask = 0; c->prof_events = nullptr;
  c->aux = nullptr; c->ev_fork = c->ev_index = c->ev_pass1 = c->ev_chain = nullptr;
  hipError_t e = hipStreamCreateWithFlags(&c->aux, hipStreamNonBlocking);
  hipEvent_t* evs[4] = {&c->ev_fork, &c->ev_index, &c->ev_pass1, &c->ev_chain};
  for (int i = 0; i < 4 && e == hipSuccess; ++i) e = hipEventCreateWithFlags(evs[i], hipEventDisableTiming);
  if (e == hipSuccess) e = mar_launch_init(c, fill, (hipStream_t)hip_stream);
  if (e == hipSuccess && d.split) {
    // the images' padding rows (beyond a chunk's rows, up to whole tiles of 32) are never written again: zeros
    const size_t kb = 2 * (size_t)d.C * (size_t)((d.N + 31) / 32) * mar_split_image_bytes(d.dk);
    const size_t qb = 2 * (size_t)d.C * (size_t)((d.S + 31) / 32) * mar_split_image_bytes(d.dk);
    e = mar_launch_fill_u32((uint32_t*)c->L.Kimg, (int64_t)(kb / 4), 0u, (hipStream_t)hip_stream);
    if (e == hipSuccess) e = mar_launch_fill_u32((uint32_t*)c->L.Qimg, (int64_t)(qb / 4), 0u, (hipStream_t)hip_stream);
  }
  if (e != hipSuccess) { mar_destroy(c); return hip_fail(e, "context set-up"); }
  *out = c;
  return MAR_OK;
}

extern "C" int mar_destroy(mar_ctx* c) {
  if (!c) return MAR_OK;
  if (c->prof_events) {
    for (int i = 0; i < c->prof_max * 2 * MAR_NUM_PHASES; ++i) (void)hipEventDestroy(c->prof_events[i]);
    free(c->prof_events);
  }
  hipEvent_t evs[4] = {c->ev_fork, c->ev_index, c->ev_pass1, c->ev_chain};
  for (int i = 0; i < 4; ++i) if (evs[i]) (void)hipEventDestroy(evs[i]);
  if (c->aux) { (void)hipStreamSynchronize(c->aux); (void)hipStreamDestroy(c->aux); }
  delete c;
  return MAR_OK;
}

extern "C" int mar_sample_negatives(mar_ctx* c, uint64_t step, const int32_t* edge_src, const int32_t* edge_dst,
                                    int64_t num_edges, int32_t* neg_src, int32_t* neg_dst, void* hip_stream) {
  if (!c) return fail(MAR_EINVAL, "context is NULL");
  if (!neg_src || !neg_dst) return fail(MAR_EINVAL, "an output pointer is NULL");
  if (step >> 63) return fail(MAR_ERANGE, "step must be below 2^63");
  if (c->dm.Ndeg > 0) {
    if (!edge_src || !edge_dst) return fail(MAR_EINVAL, "degree-based negatives need the edge list");
    if (num_edges < 1) return fail(MAR_EINVAL, "degree-based negatives need num_edges >= 1");
  }
  if (num_edges < 0) return fail(MAR_EINVAL, "num_edges is negative");
  const hipError_t e = mar_launch_sample(c, step, edge_src, edge_dst, num_edges, neg_src, neg_dst, (hipStream_t)hip_stream);
  return e == hipSuccess ? MAR_OK : hip_fail(e, "sampling kernel");
}

static int make_batch(const mar_ctx* c, const int32_t* src, const int32_t* rel, const int32_t* dst, int32_t n,
                      const int32_t* neg_src, const int32_t* neg_dst, MarBatch* b) {
  if (!c) return fail(MAR_EINVAL, "context is NULL");
  if (n < 0 || n > c->dm.B) return fail(MAR_ERANGE, "n_edges %d outside 0..batch_size %d", n, c->dm.B);
  if (n > 0 && (!src || (!rel && c->dm.roles == 3) || !dst || !neg_src || !neg_dst)) return fail(MAR_EINVAL, "an id array is NULL");
  b->src = src; b->rel = rel; b->dst = dst; b->neg_src = neg_src; b->neg_dst = neg_dst;
  b->n = n;
  b->nchunks = (n + c->dm.S - 1) / c->dm.S;
  b->cn = b->nchunks * c->dm.N;
  b->n_occ = c->dm.roles * (int64_t)n + 2 * (int64_t)b->cn;
  b->n_pos = c->dm.roles * (int64_t)n + 2 * (int64_t)b->cn * c->dm.sy2;
  return MAR_OK;
}

#define HIP_TRY(expr, what) do { const hipError_t e_ = (expr); if (e_ != hipSuccess) { c->bitmap_dirty = 1; return hip_fail(e_, what); } } while (0)

extern "C" int mar_train_batch(mar_ctx* c, const int32_t* src, const int32_t* rel, const int32_t* dst, int32_t n_edges,
                               const int32_t* neg_src, const int32_t* neg_dst, float* loss_sum_out,
                               const mar_debug_out* dbg, void* hip_stream) {
  MarBatch b;
  const int rc = make_batch(c, src, rel, dst, n_edges, neg_src, neg_dst, &b);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  if (n_edges == 0) {
    if (loss_sum_out) HIP_TRY(mar_launch_fill_u32((uint32_t*)loss_sum_out, 1, 0u, st), "loss reset");
    if (dbg && dbg->num_uniq) HIP_TRY(mar_launch_fill_u32((uint32_t*)dbg->num_uniq, 2, 0u, st), "debug reset");
    return MAR_OK;
  }
  if (c->bitmap_dirty) {
    HIP_TRY(mar_launch_clear_bitmap(c, st), "bitmap reset");
    c->bitmap_dirty = 0;
  }
  // Two streams: the caller's carries the gather and the two contraction passes; the index build
  // (needed only by the per-row reduce) and the chain rule (needs pass 1 only) run beside them on `aux`.
  hipStream_t ax = c->aux;
  hipEvent_t* ev = nullptr;
  if (c->prof_events && c->prof_steps < c->prof_max) ev = c->prof_events + (size_t)c->prof_steps * 2 * MAR_NUM_PHASES;
#define MARK(phase, end, stream) do { if (ev && (c->prof_mask >> (phase) & 1u)) HIP_TRY(hipEventRecord(ev[2 * (phase) + (end)], stream), "event record"); } while (0)
  // Two orders of the first launches.  Large batches: the gather runs alone at memory speed and the index build
  // starts behind it, beside the first contraction pass that hides it.  Small batches: the index build is the
  // longer path to the reduce, so it starts first and the gather runs beside it.
  if (c->dm.index_after_gather) {
    MARK(1, 0, st);
    HIP_TRY(mar_launch_prep(c, b, dbg ? dbg->pos : nullptr, c->dm.split, st), "gather kernel");
    MARK(1, 1, st);
  }
  HIP_TRY(hipEventRecord(c->ev_fork, st), "fork");
  HIP_TRY(hipStreamWaitEvent(ax, c->ev_fork, 0), "fork");
  MARK(0, 0, ax);
  HIP_TRY(mar_launch_index(c, b, ax), "index kernels");
  if (dbg) HIP_TRY(mar_launch_debug_copy(c, b, dbg, ax), "debug copy");
  MARK(0, 1, ax);
  HIP_TRY(hipEventRecord(c->ev_index, ax), "join");
  if (!c->dm.index_after_gather) {
    MARK(1, 0, st);
    HIP_TRY(mar_launch_prep(c, b, dbg ? dbg->pos : nullptr, c->dm.split, st), "gather kernel");
    MARK(1, 1, st);
  }
  MARK(2, 0, st);
  HIP_TRY(mar_launch_flash(c, b, 1, nullptr, nullptr, st), "score/softmax kernel");
  MARK(2, 1, st);
  HIP_TRY(mar_launch_flash_merge(c, b, st), "stripe merge kernel");
  // The chain rule needs pass 1 only.  Large batches run it on `aux` beside pass 2, which leaves memory bandwidth
  // unused; for small batches `aux` is the longer path to the reduce (the index build), so it stays on the
  // caller's stream.
  if (c->dm.index_after_gather) {
    HIP_TRY(hipEventRecord(c->ev_pass1, st), "fork");
    HIP_TRY(hipStreamWaitEvent(ax, c->ev_pass1, 0), "fork");
    MARK(4, 0, ax);
    HIP_TRY(mar_launch_chain(c, b, ax), "chain-rule kernel");
    MARK(4, 1, ax);
    HIP_TRY(hipEventRecord(c->ev_chain, ax), "join");
  } else {
    MARK(4, 0, st);
    HIP_TRY(mar_launch_chain(c, b, st), "chain-rule kernel");
    MARK(4, 1, st);
    HIP_TRY(hipEventRecord(c->ev_chain, st), "join");
  }
  MARK(3, 0, st);
  HIP_TRY(mar_launch_flash(c, b, 2, nullptr, nullptr, st), "negative-gradient kernel");
  MARK(3, 1, st);
  HIP_TRY(hipStreamWaitEvent(st, c->ev_index, 0), "join");
  HIP_TRY(hipStreamWaitEvent(st, c->ev_chain, 0), "join");
  MARK(5, 0, st);
  HIP_TRY(mar_launch_reduce(c, b, loss_sum_out, dbg ? dbg->grad_rows : nullptr, nullptr, st), "reduce/Adagrad kernels");
  MARK(5, 1, st);
#undef MARK
  if (ev) c->prof_steps++;
  if (dbg) {
    const size_t nb = (size_t)n_edges * sizeof(float);
    if (dbg->lse_dst) HIP_TRY(hipMemcpyAsync(dbg->lse_dst, c->L.lse + (size_t)MAR_SIDE_DST * c->dm.B, nb, hipMemcpyDeviceToDevice, st), "debug copy");
    if (dbg->lse_src) HIP_TRY(hipMemcpyAsync(dbg->lse_src, c->L.lse + (size_t)MAR_SIDE_SRC * c->dm.B, nb, hipMemcpyDeviceToDevice, st), "debug copy");
  }
  return MAR_OK;
}

extern "C" int mar_eval_scores(mar_ctx* c, const int32_t* src, const int32_t* rel, const int32_t* dst, int32_t n_edges,
                               const int32_t* neg_src, const int32_t* neg_dst, float* pos_scores, int32_t* rank_dst,
                               int32_t* rank_src, void* hip_stream) {
  MarBatch b;
  const int rc = make_batch(c, src, rel, dst, n_edges, neg_src, neg_dst, &b);
  if (rc) return rc;
  if (!rank_dst || !rank_src) return fail(MAR_EINVAL, "a rank output pointer is NULL");
  if (n_edges == 0) return MAR_OK;
  hipStream_t st = (hipStream_t)hip_stream;
  HIP_TRY(mar_launch_prep(c, b, pos_scores, 0, st), "gather kernel");
  HIP_TRY(mar_launch_flash(c, b, 3, rank_dst, rank_src, st), "rank kernel");
  return MAR_OK;
}

extern "C" int mar_eval_filter(mar_ctx* c, const int32_t* src, const int32_t* rel, const int32_t* dst, int32_t n_edges,
                               const int64_t* dst_off, const int32_t* dst_ids, const int64_t* src_off,
                               const int32_t* src_ids, const float* pos_scores, int32_t* rank_dst, int32_t* rank_src,
                               void* hip_stream) {
  if (!c) return fail(MAR_EINVAL, "context is NULL");
  if (n_edges < 0 || n_edges > c->dm.B) return fail(MAR_ERANGE, "n_edges %d outside 0..batch_size %d", n_edges, c->dm.B);
  if (n_edges == 0) return MAR_OK;
  if (!src || (!rel && c->dm.roles == 3) || !dst) return fail(MAR_EINVAL, "an id array is NULL");
  if (!dst_off || !src_off || !pos_scores || !rank_dst || !rank_src) return fail(MAR_EINVAL, "an argument is NULL");
  MarBatch b;
  b.src = src; b.rel = rel; b.dst = dst; b.neg_src = nullptr; b.neg_dst = nullptr;
  b.n = n_edges; b.nchunks = 0; b.cn = 0; b.n_occ = 0; b.n_pos = 0;
  HIP_TRY(mar_launch_filter(c, b, dst_off, dst_ids, src_off, src_ids, pos_scores, rank_dst, rank_src, (hipStream_t)hip_stream),
          "filter kernel");
  return MAR_OK;
}

extern "C" int mar_rank_metrics(mar_ctx* c, const int32_t* ranks, int64_t n_ranks, const int32_t* ks, int32_t num_k,
                                double* out, void* hip_stream) {
  if (!c) return fail(MAR_EINVAL, "context is NULL");
  if (!out) return fail(MAR_EINVAL, "out is NULL");
  if (n_ranks < 0 || (n_ranks > 0 && !ranks)) return fail(MAR_EINVAL, "ranks is NULL or n_ranks negative");
  if (num_k < 0 || num_k > 8 || (num_k > 0 && !ks)) return fail(MAR_ERANGE, "num_k outside 0..8 or ks NULL");
  for (int j = 0; j < num_k; ++j) if (ks[j] < 1) return fail(MAR_EINVAL, "thresholds must be >= 1");
  HIP_TRY(mar_launch_rank_metrics(ranks, n_ranks, ks, num_k, out, c->L.metric_part, (hipStream_t)hip_stream), "metrics kernel");
  return MAR_OK;
}

// ------------------------------------------------------- out-of-memory pipelined training -----
// Sec. 3: node embeddings and their optimiser state live outside device memory; a batch goes through
//   in   : unique set + staging of its node rows into a compact device table          (stream s_in)
//   step : gather / score / loss / backward on the staged rows, relation rows updated  (caller's stream)
//   out  : Adagrad on the host table with the batch's summed node gradients            (stream s_out)
// and up to `depth` batches are in flight.  Events order the stages so that batch j stages its rows after the
// updates of batches <= j - depth and before the update of batch j - depth + 1: the staleness is exactly
// depth - 1 batches in every run.
struct PipeSlot {
  mar_ctx* ctx;                // context over the compact table (node_emb = compact) and the resident relation tables
  MarStage sg;
  int32_t *src, *rel, *dst, *neg_src, *neg_dst;    // the slot's copy of the batch's ids
  MarBatch b_ids, b_rank;      // the batch over real ids (index build) and over ranks (gather, chain rule)
  hipEvent_t ev_in, ev_step, ev_out;
};

struct mar_pipe {
  mar_config cfg; MarDims dm;
  int32_t depth;
  float *host_emb, *host_state, *rel_emb, *rel_state;
  hipStream_t s_in, s_out;
  hipEvent_t ev_call;
  PipeSlot* slots;
  int64_t submitted, applied;  // batches submitted / batches whose update has been enqueued
};

static size_t pipe_slot_extra(const MarDims& d, char* base, PipeSlot* ps) {
  size_t off = 0;
  auto take = [&](size_t bytes) -> void* {
    void* p = base ? base + off : nullptr;
    off += (bytes + 255) & ~(size_t)255;
    return p;
  };
  const size_t B = d.B, CN = (size_t)d.C * d.N;
  const size_t rows = (size_t)(2 * B + 2 * CN < (size_t)d.num_nodes ? 2 * B + 2 * CN : (size_t)d.num_nodes);
  PipeSlot t;
  t.sg.compact = (float*)take(rows * d.dim * 4 + 16);
  t.sg.gsum = (float*)take((size_t)d.u_max * d.dk * 4);
  t.sg.c_src = (int32_t*)take(B * 4); t.sg.c_dst = (int32_t*)take(B * 4);
  t.sg.c_neg_dst = (int32_t*)take(CN * 4); t.sg.c_neg_src = (int32_t*)take(CN * 4);
  t.src = (int32_t*)take(B * 4); t.rel = (int32_t*)take(B * 4); t.dst = (int32_t*)take(B * 4);
  t.neg_src = (int32_t*)take(CN * 4); t.neg_dst = (int32_t*)take(CN * 4);
  if (ps) { ps->sg.compact = t.sg.compact; ps->sg.gsum = t.sg.gsum; ps->sg.c_src = t.sg.c_src; ps->sg.c_dst = t.sg.c_dst;
            ps->sg.c_neg_dst = t.sg.c_neg_dst; ps->sg.c_neg_src = t.sg.c_neg_src; ps->src = t.src; ps->rel = t.rel; ps->dst = t.dst;
            ps->neg_src = t.neg_src; ps->neg_dst = t.neg_dst; }
  return off;
}

static int pipe_check(const mar_config* cfg, int32_t depth, MarDims* d) {
  const int rc = check_config(cfg, d);
  if (rc) return rc;
  if (depth < 1 || depth > MAR_PIPE_MAX_DEPTH) return fail(MAR_ERANGE, "depth %d outside 1..%d", depth, MAR_PIPE_MAX_DEPTH);
  return MAR_OK;
}

extern "C" int mar_pipe_workspace_bytes(const mar_config* cfg, int32_t depth, size_t* out_bytes) {
  MarDims d;
  const int rc = pipe_check(cfg, depth, &d);
  if (rc) return rc;
  if (!out_bytes) return fail(MAR_EINVAL, "out_bytes is NULL");
  *out_bytes = (size_t)depth * (carve(d, nullptr, nullptr) + pipe_slot_extra(d, nullptr, nullptr));
  return MAR_OK;
}

extern "C" int mar_pipe_destroy(mar_pipe* p) {
  if (!p) return MAR_OK;
  if (p->s_in) { (void)hipStreamSynchronize(p->s_in); (void)hipStreamDestroy(p->s_in); }
  if (p->s_out) { (void)hipStreamSynchronize(p->s_out); (void)hipStreamDestroy(p->s_out); }
  if (p->ev_call) (void)hipEventDestroy(p->ev_call);
  if (p->slots) {
    for (int i = 0; i < p->depth; ++i) {
      hipEvent_t evs[3] = {p->slots[i].ev_in, p->slots[i].ev_step, p->slots[i].ev_out};
      for (int k = 0; k < 3; ++k) if (evs[k]) (void)hipEventDestroy(evs[k]);
      mar_destroy(p->slots[i].ctx);
    }
    delete[] p->slots;
  }
  delete p;
  return MAR_OK;
}

extern "C" int mar_pipe_create(const mar_config* cfg, float* host_node_emb, float* host_node_state, float* rel_emb,
                               float* rel_state, void* workspace, size_t workspace_bytes, int32_t depth, void* hip_stream,
                               mar_pipe** out) {
  MarDims d;
  const int rc = pipe_check(cfg, depth, &d);
  if (rc) return rc;
  if (!out) return fail(MAR_EINVAL, "out is NULL");
  if (!host_node_emb || !host_node_state || !rel_emb || !rel_state) return fail(MAR_EINVAL, "a table pointer is NULL");
  if (((uintptr_t)host_node_emb | (uintptr_t)host_node_state | (uintptr_t)rel_emb | (uintptr_t)rel_state) & 15)
    return fail(MAR_EINVAL, "table pointers must be 16-byte aligned");
  if (!workspace || ((uintptr_t)workspace & 255)) return fail(MAR_EINVAL, "workspace must be non-NULL and 256-byte aligned");
  // the host tables must be memory the GPU can address; kernels use the device-side alias the runtime reports
  float* host_tabs[2] = {host_node_emb, host_node_state};
  for (int i = 0; i < 2; ++i) {
    hipPointerAttribute_t at;
    const hipError_t pe = hipPointerGetAttributes(&at, host_tabs[i]);
    if (pe != hipSuccess) { (void)hipGetLastError(); return fail(MAR_EINVAL, "host table %d is not memory known to the HIP runtime (allocate it pinned)", i); }
    if (at.type != hipMemoryTypeHost || !at.devicePointer) return fail(MAR_EINVAL, "host table %d is not pinned, device-accessible host memory", i);
    host_tabs[i] = (float*)at.devicePointer;
  }
  host_node_emb = host_tabs[0]; host_node_state = host_tabs[1];
  const size_t ctx_bytes = carve(d, nullptr, nullptr), extra = pipe_slot_extra(d, nullptr, nullptr);
  if (workspace_bytes < (size_t)depth * (ctx_bytes + extra))
    return fail(MAR_ENOMEM, "workspace has %zu bytes, %zu needed", workspace_bytes, (size_t)depth * (ctx_bytes + extra));
  mar_pipe* p = new (std::nothrow) mar_pipe();
  if (!p) return fail(MAR_ENOMEM, "out of host memory");
  p->cfg = *cfg; p->dm = d; p->depth = depth;
  p->host_emb = host_node_emb; p->host_state = host_node_state; p->rel_emb = rel_emb; p->rel_state = rel_state;
  p->s_in = p->s_out = nullptr; p->ev_call = nullptr; p->submitted = p->applied = 0;
  p->slots = new (std::nothrow) PipeSlot[depth]();
  if (!p->slots) { delete p; return fail(MAR_ENOMEM, "out of host memory"); }
  hipError_t e = hipStreamCreateWithFlags(&p->s_in, hipStreamNonBlocking);
  if (e == hipSuccess) e = hipStreamCreateWithFlags(&p->s_out, hipStreamNonBlocking);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&p->ev_call, hipEventDisableTiming);
  char* base = (char*)workspace;
  for (int i = 0; i < depth && e == hipSuccess; ++i) {
    PipeSlot& ps = p->slots[i];
    char* sb = base + (size_t)i * (ctx_bytes + extra);
    pipe_slot_extra(d, sb + ctx_bytes, &ps);
    ps.sg.host_emb = host_node_emb; ps.sg.host_state = host_node_state;
    // the slot's context: the compact table stands in for the node table (no fill; its accumulators are never used)
    const int rc2 = mar_init_tables(cfg, ps.sg.compact, ps.sg.compact, rel_emb, rel_state, sb, ctx_bytes, 0, hip_stream, &ps.ctx);
    if (rc2) { mar_pipe_destroy(p); return rc2; }
    hipEvent_t* evs[3] = {&ps.ev_in, &ps.ev_step, &ps.ev_out};
    for (int k = 0; k < 3 && e == hipSuccess; ++k) e = hipEventCreateWithFlags(evs[k], hipEventDisableTiming);
  }
  if (e != hipSuccess) { mar_pipe_destroy(p); return hip_fail(e, "pipeline set-up"); }
  *out = p;
  return MAR_OK;
}

__global__ void __launch_bounds__(256)
k_copy_ids(const int32_t* __restrict__ s0, const int32_t* __restrict__ r0, const int32_t* __restrict__ d0,
           const int32_t* __restrict__ ns0, const int32_t* __restrict__ nd0, int n, int cn, int32_t* __restrict__ s1,
           int32_t* __restrict__ r1, int32_t* __restrict__ d1, int32_t* __restrict__ ns1, int32_t* __restrict__ nd1) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) { s1[i] = s0[i]; d1[i] = d0[i]; if (r0) r1[i] = r0[i]; }
  if (i < cn) { ns1[i] = ns0[i]; nd1[i] = nd0[i]; }
}

#define PIPE_TRY(expr, what) do { const hipError_t e_ = (expr); if (e_ != hipSuccess) return hip_fail(e_, what); } while (0)

// Enqueues the update stage of batch i on s_out; `gather_of` >= 0: it must also wait for the staging of that batch.
static int pipe_enqueue_update(mar_pipe* p, int64_t i, int64_t gather_of) {
  PipeSlot& ps = p->slots[i % p->depth];
  PIPE_TRY(hipStreamWaitEvent(p->s_out, ps.ev_step, 0), "update stage");
  if (gather_of >= 0) PIPE_TRY(hipStreamWaitEvent(p->s_out, p->slots[gather_of % p->depth].ev_in, 0), "update stage");
  PIPE_TRY(mar_launch_stage_out(ps.ctx, ps.b_ids, ps.sg, p->s_out), "update kernel");
  PIPE_TRY(hipEventRecord(ps.ev_out, p->s_out), "update stage");
  p->applied = i + 1;
  return MAR_OK;
}

extern "C" int mar_pipe_submit(mar_pipe* p, const int32_t* src, const int32_t* rel, const int32_t* dst, int32_t n_edges,
                               const int32_t* neg_src, const int32_t* neg_dst, float* loss_sum_out, void* ids_stream,
                               void* hip_stream) {
  if (!p) return fail(MAR_EINVAL, "pipeline is NULL");
  if (n_edges < 1) return fail(MAR_EINVAL, "n_edges must be >= 1");
  const int64_t j = p->submitted;
  PipeSlot& ps = p->slots[j % p->depth];
  mar_ctx* c = ps.ctx;
  int rc = make_batch(c, src, rel, dst, n_edges, neg_src, neg_dst, &ps.b_ids);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  const int roles = c->dm.roles;
  // ---- in: after the work enqueued so far on the stream the ids come from, and after the update of the batch that
  // used this slot before (batch j - depth: its buffers are free, and its update is the newest one batch j may see)
  PIPE_TRY(hipEventRecord(p->ev_call, (hipStream_t)ids_stream), "submit");
  PIPE_TRY(hipStreamWaitEvent(p->s_in, p->ev_call, 0), "submit");
  if (j >= p->depth) PIPE_TRY(hipStreamWaitEvent(p->s_in, ps.ev_out, 0), "stage in");
  const int work = n_edges > ps.b_ids.cn ? n_edges : ps.b_ids.cn;
  hipLaunchKernelGGL(k_copy_ids, dim3((work + 255) / 256), dim3(256), 0, p->s_in, src, roles == 3 ? rel : nullptr, dst, neg_src, neg_dst,
                     n_edges, ps.b_ids.cn, ps.src, ps.rel, ps.dst, ps.neg_src, ps.neg_dst);
  PIPE_TRY(hipGetLastError(), "id copy");
  ps.b_ids.src = ps.src; ps.b_ids.rel = ps.rel; ps.b_ids.dst = ps.dst; ps.b_ids.neg_src = ps.neg_src; ps.b_ids.neg_dst = ps.neg_dst;
  ps.b_rank = ps.b_ids;
  ps.b_rank.src = ps.sg.c_src; ps.b_rank.dst = ps.sg.c_dst; ps.b_rank.neg_src = ps.sg.c_neg_src; ps.b_rank.neg_dst = ps.sg.c_neg_dst;
  if (c->bitmap_dirty) { PIPE_TRY(mar_launch_clear_bitmap(c, p->s_in), "bitmap reset"); c->bitmap_dirty = 0; }
  PIPE_TRY(mar_launch_index(c, ps.b_ids, p->s_in), "index kernels");
  PIPE_TRY(mar_launch_stage_in(c, ps.b_ids, ps.sg, p->s_in), "staging kernels");
  PIPE_TRY(hipEventRecord(ps.ev_in, p->s_in), "stage in");
  // ---- step on the caller's stream: staged rows, ranks as ids; node gradients are left in gsum, relation rows updated
  PIPE_TRY(hipStreamWaitEvent(st, ps.ev_in, 0), "step");
  PIPE_TRY(mar_launch_prep(c, ps.b_rank, nullptr, c->dm.split, st), "gather kernel");
  PIPE_TRY(mar_launch_flash(c, ps.b_rank, 1, nullptr, nullptr, st), "score/softmax kernel");
  PIPE_TRY(mar_launch_flash_merge(c, ps.b_rank, st), "stripe merge kernel");
  PIPE_TRY(mar_launch_chain(c, ps.b_rank, st), "chain-rule kernel");
  PIPE_TRY(mar_launch_flash(c, ps.b_rank, 2, nullptr, nullptr, st), "negative-gradient kernel");
  PIPE_TRY(mar_launch_reduce(c, ps.b_ids, loss_sum_out, nullptr, ps.sg.gsum, st), "reduce kernels");
  PIPE_TRY(hipEventRecord(ps.ev_step, st), "step");
  p->submitted = j + 1;
  // ---- out: the update of batch j - depth + 1 goes behind this batch's staging
  const int64_t i = j - p->depth + 1;
  if (i >= 0) { rc = pipe_enqueue_update(p, i, j); if (rc) return rc; }
  return MAR_OK;
}

extern "C" int mar_pipe_drain(mar_pipe* p, void* hip_stream) {
  if (!p) return fail(MAR_EINVAL, "pipeline is NULL");
  for (int64_t i = p->applied; i < p->submitted; ++i) { const int rc = pipe_enqueue_update(p, i, -1); if (rc) return rc; }
  if (p->submitted > 0)
    PIPE_TRY(hipStreamWaitEvent((hipStream_t)hip_stream, p->slots[(p->submitted - 1) % p->depth].ev_out, 0), "drain");
  return MAR_OK;
}

// ----------------------------------------------------------------------- profiling -----
extern "C" int mar_profile_enable(mar_ctx* c, int32_t max_steps, uint32_t phase_mask) {
  if (!c) return fail(MAR_EINVAL, "context is NULL");
  if (max_steps < 0 || max_steps > MAR_MAX_PROFILE_STEPS) return fail(MAR_ERANGE, "max_steps outside 0..%d", MAR_MAX_PROFILE_STEPS);
  if (c->prof_events) {
    for (int i = 0; i < c->prof_max * 2 * MAR_NUM_PHASES; ++i) (void)hipEventDestroy(c->prof_events[i]);
    free(c->prof_events);
    c->prof_events = nullptr;
  }
  c->prof_max = 0; c->prof_steps = 0; c->prof_mask = phase_mask & ((1u << MAR_NUM_PHASES) - 1u);
  if (max_steps == 0) return MAR_OK;
  const size_t ne = (size_t)max_steps * 2 * MAR_NUM_PHASES;
  c->prof_events = (hipEvent_t*)calloc(ne, sizeof(hipEvent_t));
  if (!c->prof_events) return fail(MAR_ENOMEM, "out of host memory");
  for (size_t i = 0; i < ne; ++i) {
    const hipError_t e = hipEventCreate(&c->prof_events[i]);
    if (e != hipSuccess) {
      for (size_t j = 0; j < i; ++j) (void)hipEventDestroy(c->prof_events[j]);
      free(c->prof_events); c->prof_events = nullptr;
      return hip_fail(e, "event create");
    }
  }
  c->prof_max = max_steps;
  return MAR_OK;
}

extern "C" int mar_profile_read(mar_ctx* c, double* ms, int32_t* steps) {
  if (!c || !ms || !steps) return fail(MAR_EINVAL, "an argument is NULL");
  for (int p = 0; p < MAR_NUM_PHASES; ++p) ms[p] = 0.0;
  *steps = c->prof_steps;
  for (int s = 0; s < c->prof_steps; ++s) {
    hipEvent_t* ev = c->prof_events + (size_t)s * 2 * MAR_NUM_PHASES;
    for (int p = 0; p < MAR_NUM_PHASES; ++p) {
      if (!(c->prof_mask >> p & 1u)) continue;
      hipError_t e = hipEventSynchronize(ev[2 * p + 1]);
      if (e != hipSuccess) return hip_fail(e, "event synchronize");
      float t = 0.f;
      e = hipEventElapsedTime(&t, ev[2 * p], ev[2 * p + 1]);
      if (e != hipSuccess) return hip_fail(e, "event elapsed time");
      ms[p] += t;
    }
  }
  c->prof_steps = 0;
  return MAR_OK;
}

// Internal declarations shared by the library's translation units (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/marius_hip.h"

// Side index of a corrupted endpoint; also the generator's "side" counter bit.
#define MAR_SIDE_SRC 0   // negatives replace the source
#define MAR_SIDE_DST 1   // negatives replace the destination

// Workspace carve-up (device pointers).
struct MarLayout {
  int32_t*  scalars;      // [16]: 0 = unique rows (nodes + relations), 1 = unique nodes, 2 = number of entries in `owners`
  uint32_t* bitmap;       // touched-id map over unified ids (node id, or num_nodes + relation id): one bit or
                          // one byte per id, see ipw_log2
  uint32_t* word_prefix;  // marked ids before each word of the map
  uint32_t* bsum;         // scan scratch (block sums)
  int32_t*  uniq;         // ascending unified ids of the touched rows
  uint32_t* seg_off;      // [unique rows + 1] first position of each row's segment in the row-sorted order
  uint32_t* keys0;        // [n_pos] gradient row -> rank of its table row among the unique rows (sort keys)
  uint32_t* kbuf[2];      // [n_pos] each: keys between two passes of the radix sort
  int32_t*  vbuf[2];      // [n_pos] each: gradient row numbers between two passes
  uint32_t* hist;         // [sort tiles][bins] digit counts of the current pass
  int32_t*  perm;         // position in row-sorted order -> gradient row
  int32_t*  rank_sorted;  // position -> rank
  int32_t*  owners;       // [reduce blocks] workgroups of the reduce in which a segment begins that continues into later ones
  float*    Q;            // [2][batch][dk] edge-side operands (side-major)
  float*    Km;           // [2][chunks][N][dk] gathered negative rows
  float*    qq;           // [2][batch] squared norms of Q rows (TransE)
  float*    kk;           // [2][chunks*N] squared norms of Km rows (TransE)
  float*    pos;          // [batch] positive scores
  float*    lse;          // [2][batch] log-sum-exp per edge and side
  float*    gQ;           // [sy1][2][batch][dk] per-part unnormalised gradient w.r.t. Q rows
  float*    ml;           // [sy1][2][batch][2] per-part softmax reference and sum
  float*    gQx;          // [rem_k - 1][rem_rows][dk] parts 1.. of the chunk-sides whose stripes are split to fill the last round
  float*    mlx;          // [rem_k - 1][rem_rows][2]
  float*    T;            // [2*chunks][S rounded up to 64][N rounded up to 128] softmax weights exp(score - reference)
                          // (TransE: divided by the distance), pass 1 -> pass 2
  float*    R;            // [2*chunks][N rounded up to 128, / 16][S rounded up to 64] the reference each 16-negative block of T was written with
  char*     Kimg;         // split precision: [2*chunks][N / 32 rounded up][image] bf16 hi/lo planes of Km's rows
  char*     Qimg;         // split precision: [2*chunks][S / 32 rounded up][image] the same of Q's rows
  float*    Gx;           // [rem2_k - 1][rem2_rows][dk] parts 1.. of pass 2's split stripes (split precision)
  float*    G;            // [roles*n + 2*cn*sy2][dk] gradient rows: edge-side occurrence k < roles*n at row k, part i
                          // of negative occurrence k at row roles*n + (k - roles*n)*sy2 + i
  float*    carry;        // [reduce blocks][2][dk] partial sums of segments that cross workgroup borders
  float*    loss_part;    // per-block partial loss sums
  void*     metric_part;  // [MAR_METRIC_MAX_PARTS] partial records of the rank metrics
};

struct MarDims {
  int32_t dim, dk;                 // row width and its multiple-of-4 padding
  int32_t B, C, S, N, Ndeg;
  int32_t roles;                   // edge-side occurrences per edge: source, destination and (unless Dot) relation
  int64_t num_nodes; int32_t num_rels;
  int64_t n_occ_max;               // roles*B + 2CN
  int64_t n_pos_max;               // roles*B + 2CN*sy2: gradient rows per step
  int32_t sy1, sy2;                // how many workgroups share the streamed rows of one stripe (pass 1 / 2)
  int32_t tps1, tps2;              // streamed tiles per workgroup
  // Pass 1 of a full batch: (chunk-side, stripe) units beyond the last whole round of workgroups -- all stripes of the
  // chunk-sides from rem_cs0 on -- are each split into rem_k parts of rem_tps tiles, which a small kernel merges.
  int32_t rem_cs0, rem_k, rem_tps;
  int64_t rem_rows;                // (2C - rem_cs0) * (S rounded up to 64)
  // The same for pass 2 in split precision (chunk-sides counted in that pass's launch order): parts 1.. of a split
  // stripe write their gradient rows to Gx, and a small kernel adds them to the regular rows.
  int32_t rem2_cs0, rem2_k, rem2_tps;
  int64_t rem2_rows;               // (2C - rem2_cs0) * (N rounded up to whole stripes)
  int64_t u_max;                   // min(num_nodes + num_rels, n_occ_max)
  int64_t nwords;                  // words of the touched-id map
  int32_t ipw_log2;                // ids per word: 5 = one bit per id (atomic marks), 2 = one byte per id (plain stores)
  int32_t sort_passes, sort_bits;  // radix sort of the gradient rows by rank: passes, bits per pass
  int32_t split;                   // the contraction passes run in split precision (bf16 hi + lo operands)
  int32_t index_after_gather;      // launch order of a step: gather first, index build behind it (large batches)
};

#define MAR_MAX_PARTS 8                   // most parts a stripe of pass 1 is split into
#define MAR_MAX_PROFILE_STEPS 4096

struct mar_ctx {
  mar_config cfg;
  MarDims dm;
  float *node_emb, *node_state, *rel_emb, *rel_state;
  void* workspace; size_t workspace_bytes;
  MarLayout L;
  int bitmap_dirty;                // a failed step may leave bits set
  // second stream for work that is independent of the contraction passes, and its fork/join events
  hipStream_t aux;
  hipEvent_t ev_fork, ev_index, ev_pass1, ev_chain;
  // profiling
  int32_t prof_max, prof_steps;
  uint32_t prof_mask;
  hipEvent_t* prof_events;         // 2 * MAR_NUM_PHASES per step (begin, end of each phase)
};

void mar_set_error(const char* fmt, ...);

// Radix sort of the gradient rows: elements per workgroup tile and the widest digit.
#define MAR_SORT_TILE 4096
#define MAR_SORT_MAX_BITS 10

// Rank metrics: ranks per partial record, records a scratch area holds, bytes per record.
#define MAR_METRIC_TILE 4096
#define MAR_METRIC_MAX_PARTS 4096
#define MAR_METRIC_PART_BYTES 72

// Positions of the row-sorted order per workgroup of the reduce.
#define MAR_REDUCE_BLOCK 256

// Lanes that move one table row as float4s.
static inline int mar_lane_group(int dk) { return dk <= 64 ? 16 : (dk <= 128 ? 32 : 64); }

// ---- launchers (each returns a hipError_t from the launch) --------------------------
hipError_t mar_launch_init(const mar_ctx* c, int fill, hipStream_t st);
hipError_t mar_launch_sample(const mar_ctx* c, uint64_t step, const int32_t* es, const int32_t* ed,
                             int64_t num_edges, int32_t* neg_src, int32_t* neg_dst, hipStream_t st);
hipError_t mar_launch_clear_bitmap(const mar_ctx* c, hipStream_t st);
hipError_t mar_launch_fill_u32(uint32_t* p, int64_t n, uint32_t v, hipStream_t st);

struct MarBatch {
  const int32_t *src, *rel, *dst, *neg_src, *neg_dst;
  int32_t n;        // edges
  int32_t nchunks;  // ceil(n / S)
  int32_t cn;       // nchunks * N
  int64_t n_occ;    // roles*n + 2cn
  int64_t n_pos;    // roles*n + 2cn*sy2 gradient rows
};

hipError_t mar_launch_index(const mar_ctx* c, const MarBatch& b, hipStream_t st);
// images != 0 (split-precision training): the operands are written as bf16 hi/lo images instead of fp32 rows
hipError_t mar_launch_prep(const mar_ctx* c, const MarBatch& b, float* pos_out, int images, hipStream_t st);
hipError_t mar_launch_flash(const mar_ctx* c, const MarBatch& b, int pass, int32_t* rank_dst, int32_t* rank_src,
                            hipStream_t st);
hipError_t mar_launch_chain(const mar_ctx* c, const MarBatch& b, hipStream_t st);
hipError_t mar_launch_filter(const mar_ctx* c, const MarBatch& b, const int64_t* dst_off, const int32_t* dst_ids,
                             const int64_t* src_off, const int32_t* src_ids, const float* pos, int32_t* rank_dst,
                             int32_t* rank_src, hipStream_t st);
hipError_t mar_launch_reduce(const mar_ctx* c, const MarBatch& b, float* loss_out, float* dbg_grad, float* defer_grad, hipStream_t st);

// Staging buffers of one batch of out-of-memory training (see mar_rows.hip).
struct MarStage {
  float *host_emb, *host_state;                      // node table and accumulators in pinned host memory
  float *compact, *gsum;                             // [unique rows][dim] staged rows, [unique rows][dk] summed gradients
  int32_t *c_src, *c_dst, *c_neg_dst, *c_neg_src;    // the batch's node ids replaced by ranks
};
hipError_t mar_launch_stage_in(const mar_ctx* c, const MarBatch& b, const MarStage& sg, hipStream_t st);
hipError_t mar_launch_stage_out(const mar_ctx* c, const MarBatch& b, const MarStage& sg, hipStream_t st);
hipError_t mar_launch_debug_copy(const mar_ctx* c, const MarBatch& b, const mar_debug_out* dbg, hipStream_t st);
hipError_t mar_launch_rank_metrics(const int32_t* ranks, int64_t n, const int32_t* ks, int num_k, double* out, void* part,
                                   hipStream_t st);
int mar_flash_supported(int dk);
int mar_flash_tile_rows(int dk, int pass);
int mar_flash_stripe_rows(int dk, int pass);
hipError_t mar_flash_prepare();   // once per process and device before the first contraction launch (LDS size limits)
int mar_flash_wgs_per_cu(int dk, int pass);        // workgroups of a pass that a CU holds at once
hipError_t mar_launch_flash_merge(const mar_ctx* c, const MarBatch& b, hipStream_t st);   // after pass 1: merges split stripes
// Split-precision passes (mar_split.hip): geometry for the planning of a configuration, and the launches.
int mar_split_supported(int dk);
int mar_split_stripe_rows(int dk, int pass);
int mar_split_tile_rows();
int mar_split_wgs_per_cu(int dk, int pass);
size_t mar_split_image_bytes(int dk);
hipError_t mar_split_prepare();

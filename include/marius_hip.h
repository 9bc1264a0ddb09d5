/*
 * marius_hip.h -- C ABI of the MI355X (gfx950) graph-embedding training step.
 *
 * One call of mar_train_batch is one iteration of the paper's synchronous training
 * loop (Alg. 1) with every table resident in device memory: form the batch from edge
 * ids, evaluate the contrastive loss of Eq. 1 with sampled negatives (Sec. 2.1),
 * differentiate it, and apply Adagrad (Sec. 5.1, "Hyperparameters") to the touched
 * node and relation rows.
 *
 * Conventions for every entry point
 *   - "device" pointers are HIP device memory owned by the caller; the library never
 *     allocates or frees device memory and keeps no pointer except the four tables and
 *     the workspace handed to mar_init_tables.
 *   - Calls only enqueue work on `hip_stream` (a hipStream_t cast to void*, NULL = the
 *     default stream); they do not synchronise.  Scalar results land in device memory.
 *     mar_train_batch also runs part of its work on a second stream owned by the context,
 *     forked from and joined back into `hip_stream` with events (default priority), so for the
 *     caller everything is ordered on `hip_stream`.
 *   - Return value: MAR_OK (0) or a negative MAR_E* code.  Nothing is enqueued when an
 *     argument check fails.  mar_last_error gives a text for the last failure of the
 *     calling thread.
 *   - Node and relation ids are NOT range-checked on the device: ids outside
 *     [0, num_nodes) / [0, num_rels) are undefined behaviour.
 *   - Calls on one context must not overlap (one stream at a time): they share the
 *     workspace.
 */
#ifndef MARIUS_HIP_H
#define MARIUS_HIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MAR_OK        0
#define MAR_EINVAL   -1   /* null / misaligned pointer, unknown model, bad count          */
#define MAR_ERANGE   -2   /* a size is outside what the kernels support                   */
#define MAR_ENOMEM   -3   /* workspace too small                                          */
#define MAR_EHIP     -4   /* a HIP runtime call or kernel launch failed                   */

/* Score functions f(theta_s, theta_r, theta_d) (Sec. 2.1). */
#define MAR_MODEL_DISTMULT 0   /* theta_s^T diag(theta_r) theta_d, as printed in Sec. 2.1             */
#define MAR_MODEL_COMPLEX  1   /* Re sum_k s_k r_k conj(d_k); row = [re(0..dim/2) | im(0..dim/2)]      */
#define MAR_MODEL_TRANSE   2   /* -|| s + r - d ||_2                                                   */
#define MAR_MODEL_DOT      3   /* theta_s . theta_d (Sec. 5.1, "Embedding Models"): no relation parameters; */
                               /* rel ids are ignored (may be NULL) and relation rows are never touched  */

/* Arithmetic of the two training contractions (scores with softmax and the edge-side gradient; the negatives'
 * gradient).  The paper trains in fp32 (Sec. 5.1).  SPLIT_BF16 writes every fp32 operand as the sum of two bf16
 * numbers and takes each product as three bf16 matrix products accumulated in fp32 (relative error of a product
 * about 2^-16, i.e. an absolute error of a score q.n of about 2^-17 sum_k |q_k n_k|: as accurate as fp32 to the
 * 1e-4 level while |q| |n| stays below about 10); it serves the bilinear models (DistMult, ComplEx, Dot) only, and
 * evaluation always runs in fp32. */
#define MAR_PRECISION_FP32        0
#define MAR_PRECISION_SPLIT_BF16  1

#define MAR_MAX_DIM 400        /* largest supported row width in floats                              */

/* Problem statement (Sec. 2.1; hyperparameters of Table 1). */
typedef struct mar_config {
  int64_t  num_nodes;           /* |V|; num_nodes + num_rels must be < 2^31                          */
  int32_t  num_rels;            /* |R| >= 1                                                          */
  int32_t  dim;                 /* d: floats per row, 1..MAR_MAX_DIM (even for ComplEx)              */
  int32_t  model;               /* MAR_MODEL_*                                                       */
  int32_t  batch_size;          /* b: most edges one mar_train_batch call may carry                  */
  int32_t  num_chunks;          /* the batch is cut into this many contiguous chunks;                */
                                /* batch_size must be a multiple of num_chunks                       */
  int32_t  negs_per_chunk;      /* n_t: negatives per chunk and corrupted side, shared by the chunk  */
                                /* (one chunk's rows x dim x 4 bytes, and chunk edges x n_t x 4 bytes,   */
                                /* must stay below 2^31: MAR_ERANGE otherwise)                           */
  int32_t  deg_negs_per_chunk;  /* round(alpha_nt * n_t): how many of them are drawn by degree       */
  float    lr;                  /* Adagrad learning rate                                             */
  float    eps;                 /* Adagrad epsilon, added outside the square root                    */
  float    init_std;            /* standard deviation of the N(0, std^2) initialisation              */
  uint64_t seed;                /* key of the counter-based generator                                */
  int32_t  precision;           /* MAR_PRECISION_*: arithmetic of the two training contractions      */
  int32_t  reserved;            /* must be 0                                                         */
} mar_config;

typedef struct mar_ctx mar_ctx;  /* opaque: host-side metadata only */

/* Optional per-step outputs for checking a step against a reference.  Every member
 * is a device pointer and may be NULL.  Capacities: uniq_* and grad_rows hold up to
 * min(num_nodes + num_rels, 3*batch_size + 2*num_chunks*negs_per_chunk) rows. */
typedef struct mar_debug_out {
  int32_t* num_uniq;    /* [2]: number of unique touched nodes, unique touched relations            */
  int32_t* uniq_nodes;  /* ascending unique node ids                                                */
  int32_t* uniq_rels;   /* ascending unique relation ids                                            */
  float*   pos;         /* [n_edges] positive scores f(e)                                           */
  float*   lse_dst;     /* [n_edges] log sum_j exp f(s, r, n_j)  (destination corrupted)            */
  float*   lse_src;     /* [n_edges] log sum_j exp f(m_j, r, d)  (source corrupted)                 */
  float*   grad_rows;   /* [(num_uniq[0] + num_uniq[1]) * dim] summed gradient of the batch loss    */
                        /* per unique row: nodes in uniq_nodes order, then relations                */
} mar_debug_out;

/* Bytes of device workspace a context for `cfg` needs.  Host only. */
int mar_workspace_bytes(const mar_config* cfg, size_t* out_bytes);

/*
 * Creates a context over caller-owned tables (Sec. 2.1: d(|V| + |R|) parameters; Sec. 5.1:
 * Adagrad keeps one accumulator per parameter).
 *   node_emb, node_state : device, [num_nodes * dim] floats, row-major, 16-byte aligned
 *   rel_emb,  rel_state  : device, [num_rels  * dim] floats
 *   workspace            : device, >= mar_workspace_bytes, 256-byte aligned; owned by the
 *                          caller, used by every later call until mar_destroy
 *   fill                 : 1 = embeddings ~ N(0, init_std^2) from the counter-based
 *                          generator (key = seed), accumulators = 0; 0 = adopt contents
 * The context is returned in *out.
 */
int mar_init_tables(const mar_config* cfg, float* node_emb, float* node_state,
                    float* rel_emb, float* rel_state, void* workspace, size_t workspace_bytes,
                    int fill, void* hip_stream, mar_ctx** out);

/*
 * Draws the negative node ids of training step `step` (Sec. 2.1: negative sampling; Table 1:
 * alpha_nt): for each chunk c and each side, negs_per_chunk ids; the first
 * deg_negs_per_chunk are the matching endpoint of a uniformly drawn edge of the given edge
 * list (degree-proportional), the rest uniform over [0, num_nodes).  Ids depend only on
 * (seed, step, side, chunk, slot) through Philox4x32-10 and a 64-bit multiply-high.
 *   edge_src, edge_dst : device, [num_edges] int32 (may be NULL when deg_negs_per_chunk = 0)
 *   neg_src, neg_dst   : device, out, [num_chunks * negs_per_chunk] int32: ids that replace
 *                        the source / the destination
 */
int mar_sample_negatives(mar_ctx* ctx, uint64_t step, const int32_t* edge_src, const int32_t* edge_dst,
                         int64_t num_edges, int32_t* neg_src, int32_t* neg_dst, void* hip_stream);

/*
 * One training step on edges (src[i], rel[i], dst[i]), i < n_edges <= batch_size (Alg. 1 body;
 * loss: Eq. 1 with the log term over the sampled negatives of the edge's chunk, once per
 * corrupted side; optimiser: Adagrad, one update per touched row with the gradient summed
 * over all of the row's occurrences).  Chunk c covers edges [c*S, (c+1)*S), S =
 * batch_size / num_chunks; a short batch uses the first ceil(n_edges / S) chunks.
 *   src, rel, dst    : device, [n_edges] int32
 *   neg_src, neg_dst : device, [num_chunks * negs_per_chunk] int32
 *   loss_sum_out     : device, 1 float: the loss summed over the batch (may be NULL)
 *   dbg              : host pointer to a struct of device pointers, or NULL
 */
int mar_train_batch(mar_ctx* ctx, const int32_t* src, const int32_t* rel, const int32_t* dst,
                    int32_t n_edges, const int32_t* neg_src, const int32_t* neg_dst,
                    float* loss_sum_out, const mar_debug_out* dbg, void* hip_stream);

/*
 * Link-prediction scores (Sec. 5.1, "Evaluation Task and Metrics"): the positive score of
 * each edge and its rank among the chunk's negatives per corrupted side, rank = 1 + number
 * of negatives scoring strictly higher.  Tables are not modified.
 *   pos_scores : device, out, [n_edges] float (may be NULL)
 *   rank_dst, rank_src : device, out, [n_edges] int32
 */
int mar_eval_scores(mar_ctx* ctx, const int32_t* src, const int32_t* rel, const int32_t* dst,
                    int32_t n_edges, const int32_t* neg_src, const int32_t* neg_dst,
                    float* pos_scores, int32_t* rank_dst, int32_t* rank_src, void* hip_stream);

/*
 * Filtered ranks (Sec. 5.1: "false negatives ... will not be used in filtered evaluation").  Call after
 * mar_eval_scores on a context whose negatives are ALL nodes, each exactly once (num_chunks chunks that
 * all carry 0..num_nodes-1).  For edge i the caller lists the OTHER true destinations of (src[i], rel[i], .)
 * in dst_ids[dst_off[i] .. dst_off[i+1]) and the other true sources of (., rel[i], dst[i]) in src_ids
 * likewise; every listed candidate that scores strictly higher than the edge itself is taken out of the rank:
 *     rank_dst[i] -= #{k : f(s, r, dst_ids[k]) > f(s, r, d)},   rank_src[i] likewise.
 * Scores are evaluated per candidate on the vector ALU in the same operation order as the positive score
 * (a candidate equal to the edge's own endpoint never counts); the ranks from mar_eval_scores come from the
 * matrix cores, so a candidate within rounding of the positive can be counted on one side and not the other;
 * a filtered rank never goes below 1.
 *   dst_off, src_off : device, [n_edges + 1] int64, non-decreasing, off[0] = 0
 *   dst_ids, src_ids : device, node ids
 *   pos_scores       : device, [n_edges], as written by mar_eval_scores
 *   rank_dst, rank_src : device, in/out
 */
int mar_eval_filter(mar_ctx* ctx, const int32_t* src, const int32_t* rel, const int32_t* dst, int32_t n_edges,
                    const int64_t* dst_off, const int32_t* dst_ids, const int64_t* src_off, const int32_t* src_ids,
                    const float* pos_scores, int32_t* rank_dst, int32_t* rank_src, void* hip_stream);

/*
 * Link-prediction metrics from ranks (Sec. 5.1): MRR = mean of 1/r_i and Hits@k = fraction of ranks
 * r_i <= k over the candidate set (pass the ranks of both corrupted sides as one array of 2n
 * candidates, or one side alone).
 *   ranks : device, [n_ranks] int32, every rank >= 1
 *   ks    : HOST array of num_k thresholds, 0 <= num_k <= 8
 *   out   : device, out, [1 + num_k] doubles: MRR, then Hits@ks[0], Hits@ks[1], ...
 * n_ranks = 0 writes zeros.  The sums are formed in a fixed order that depends on n_ranks alone
 * (bit-reproducible).  Partial sums go through the context's workspace.
 */
int mar_rank_metrics(mar_ctx* ctx, const int32_t* ranks, int64_t n_ranks, const int32_t* ks, int32_t num_k,
                     double* out, void* hip_stream);

/*
 * mar_rank_metrics for callers that cannot allocate device memory and therefore have no context and no
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels and the same results bit for bit; the partial sums go through an array built into
 * the library (MAR_RANK_METRICS_STATIC_MAX / 4096 records of 72 bytes = 288 KiB per GPU, held until the process
 * ends).  The call allocates nothing and frees nothing; its first call on a device looks the array's address
 * up.  It runs on the CURRENT device, to which hip_stream must belong.
 *   n_ranks > MAR_RANK_METRICS_STATIC_MAX : MAR_ERANGE, nothing is enqueued (use mar_rank_metrics).
 * All calls on one GPU share the array and overwrite what the previous call left in it (nothing has to start
 * at zero: every record that is read was written by the same call); two calls that overlap in time on one GPU
 * -- different streams, or different threads -- race and give undefined results.
 */
#define MAR_RANK_METRICS_STATIC_MAX ((int64_t)4096 * 4096)
int mar_rank_metrics_static(const int32_t* ranks, int64_t n_ranks, const int32_t* ks, int32_t num_k,
                            double* out, void* hip_stream);

/*
 * Edge-bucket ordering for out-of-memory training (Sec. 4.1).  Host-only: all pointers are HOST memory.
 *   mar_beta_buffer_sequence  : Alg. 3.  Writes the sequence of partition buffers, row r = the c partition
 *                               ids in the buffer at step r; successive rows differ by one swapped
 *                               partition.  buffers == NULL only reports the number of rows.
 *   mar_beta_edge_bucket_order: Alg. 3 + Alg. 4.  Writes all p*p edge buckets (i, j) as pairs[2k], pairs[2k+1]
 *                               in processing order: every bucket the first time both partitions share the
 *                               buffer; shuffle != 0 permutes the buckets of one buffer (Fisher-Yates from
 *                               the back, j = mulhi64(x, k+1), x = words 0,1 of Philox4x32-10 with key =
 *                               seed and counter (k, buffer index, 0, 0x40000000)).
 *   mar_buffer_simulate       : Alg. 2 without the training: replays an order through a buffer of c
 *                               partitions that evicts the partition needed furthest in the future and
 *                               reports the number of partition loads (swaps = loads - c, the first fill
 *                               of the buffer is not a swap).
 *   mar_swap_lower_bound      : Eq. 2.     mar_beta_swap_count: Eq. 3.   (-1 unless 2 <= c <= p)
 */
int mar_beta_buffer_sequence(int32_t p, int32_t c, int32_t* buffers, int64_t capacity_rows, int64_t* num_rows);
int mar_beta_edge_bucket_order(int32_t p, int32_t c, int32_t shuffle, uint64_t seed, int32_t* pairs);
int mar_buffer_simulate(int32_t p, int32_t c, const int32_t* pairs, int64_t n_pairs, int64_t* loads);
int64_t mar_swap_lower_bound(int32_t p, int32_t c);
int64_t mar_beta_swap_count(int32_t p, int32_t c);

/*
 * Training with the node table outside device memory (Sec. 3: "Pipelined training architecture" and "Bounded
 * Staleness").  The node embeddings and their Adagrad accumulators live in pinned host memory that the GPU can
 * address (hipHostMalloc); relation tables stay in device memory.  A batch passes through three stages on three
 * streams -- in: unique set of the batch and staging of its node rows into a compact device table; step: gather,
 * scores, loss and gradients on the staged rows, relation rows updated at once (relations are never stale); out:
 * Adagrad on the host table with the batch's summed node gradients -- and up to `depth` batches are in flight.
 * The stages are ordered so that batch j reads the node table after the updates of batches 0 .. j - depth and
 * before the update of batch j - depth + 1: every run has the same staleness of exactly depth - 1 batches, and
 * depth = 1 reproduces mar_train_batch bit for bit.  A batch's node gradient is applied to whatever the host table
 * holds when its turn comes (updates are applied in batch order).
 *   host_node_emb, host_node_state : [num_nodes * dim] floats in pinned, device-accessible host memory
 *   rel_emb, rel_state             : device, [num_rels * dim]
 *   workspace                      : device, >= mar_pipe_workspace_bytes(cfg, depth), 256-byte aligned
 *   depth                          : 1 .. MAR_PIPE_MAX_DEPTH batches in flight
 * mar_pipe_submit enqueues one batch (arguments as mar_train_batch, n_edges >= 1).  The id arrays are copied by the
 * first stage, which waits for the work enqueued so far on ids_stream (the stream that wrote them; hip_stream itself
 * is allowed, but then the staging of a batch also waits for the step of the batch before it and nothing overlaps);
 * they may be reused once hip_stream has passed this call.  loss_sum_out receives the batch's loss on hip_stream.  mar_pipe_drain enqueues the updates
 * still outstanding and makes hip_stream wait for them: after it, work on hip_stream sees the final host tables.
 * Between the first submit and the drain the host tables must not be touched by anyone else.
 */
#define MAR_PIPE_MAX_DEPTH 32
typedef struct mar_pipe mar_pipe;
int mar_pipe_workspace_bytes(const mar_config* cfg, int32_t depth, size_t* out_bytes);
int mar_pipe_create(const mar_config* cfg, float* host_node_emb, float* host_node_state, float* rel_emb,
                    float* rel_state, void* workspace, size_t workspace_bytes, int32_t depth, void* hip_stream,
                    mar_pipe** out);
int mar_pipe_submit(mar_pipe* pipe, const int32_t* src, const int32_t* rel, const int32_t* dst, int32_t n_edges,
                    const int32_t* neg_src, const int32_t* neg_dst, float* loss_sum_out, void* ids_stream, void* hip_stream);
int mar_pipe_drain(mar_pipe* pipe, void* hip_stream);
int mar_pipe_destroy(mar_pipe* pipe);

/*
 * Per-phase device timing of mar_train_batch with HIP events on the stream each phase runs on
 * (phases 0 and 4 run on the context's second stream beside phases 1-3, so the six times
 * overlap and do not add up to the step time).
 * Phases: 0 index build (unique set, occurrence order), 1 row gather and operand build,
 * 2 score + softmax + gradient w.r.t. the edge side (MFMA), 3 gradient w.r.t. the
 * negatives (MFMA), 4 chain rule, 5 per-row reduce + Adagrad scatter.
 * mar_profile_enable(ctx, max_steps, phase_mask) starts recording the phases whose bit is set in
 * phase_mask (max_steps <= 4096; 0 stops; every recorded phase costs two event records per step);
 * mar_profile_read synchronises with the recorded events, adds each recorded phase's elapsed
 * milliseconds over the recorded steps into ms[MAR_NUM_PHASES], reports how many steps
 * were recorded, and resets the recording.
 */
#define MAR_NUM_PHASES 6
int mar_profile_enable(mar_ctx* ctx, int32_t max_steps, uint32_t phase_mask);
int mar_profile_read(mar_ctx* ctx, double* ms, int32_t* steps);

/* Releases the host-side context (device memory stays with the caller). */
int mar_destroy(mar_ctx* ctx);

/* Text of the calling thread's most recent failure ("" if none).  ctx may be NULL. */
const char* mar_last_error(const mar_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* MARIUS_HIP_H */

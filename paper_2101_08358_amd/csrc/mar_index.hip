// Integer side of the training step: counter-based sampling and table fill, the batch's
// unique-row set, and the row-sorted order of all row occurrences (gfx950).
//
// The unique set comes from a bitmap over "unified ids" (a node id, or num_nodes + relation
// id): mark bits, pop-count scan -> rank of every touched row and the ascending id list.
// The gradient rows (one per occurrence of a row in the batch) are then put in row-sorted order by
// a stable radix sort on the rank, so that every table row owns a contiguous segment of positions
// whose order -- the occurrence order -- is the same in every run: the per-row sums that follow
// are bit-reproducible.
#include "mar_common.h"

// ---------------------------------------------------------------- Philox4x32-10 -----
// Salmon, Moraes, Dror, Shaw, "Parallel random numbers: as easy as 1, 2, 3" (SC'11).
__device__ __forceinline__ void philox4x32_10(uint32_t& c0, uint32_t& c1, uint32_t& c2, uint32_t& c3,
                                              uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
}

// Negative sampling (Sec. 2.1; degree-based fraction of Table 1).  One thread per pair of
// slots: counter = (slot >> 1, 2*chunk + side, step lo, step hi), key = seed; even slot takes
// output words 0,1 and odd slot words 2,3 as a 64-bit value x; id = mulhi64(x, range).
__global__ void __launch_bounds__(256)
k_sample(uint64_t seed, uint64_t step, int64_t num_nodes, const int32_t* __restrict__ es,
         const int32_t* __restrict__ ed, int64_t num_edges, int C, int N, int Ndeg,
         int32_t* __restrict__ neg_src, int32_t* __restrict__ neg_dst) {
  const int pairs = (N + 1) >> 1;
  const int64_t total = (int64_t)2 * C * pairs;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int pr = (int)(i % pairs);
  const int cs = (int)(i / pairs);            // 2*chunk + side
  const int side = cs & 1, chunk = cs >> 1;
  uint32_t c0 = (uint32_t)pr, c1 = (uint32_t)cs, c2 = (uint32_t)step, c3 = (uint32_t)(step >> 32);
  philox4x32_10(c0, c1, c2, c3, (uint32_t)seed, (uint32_t)(seed >> 32));
  const uint64_t x[2] = {(uint64_t)c0 | ((uint64_t)c1 << 32), (uint64_t)c2 | ((uint64_t)c3 << 32)};
  int32_t* out = (side == MAR_SIDE_SRC ? neg_src : neg_dst) + (size_t)chunk * N;
  const int32_t* endpoint = side == MAR_SIDE_SRC ? es : ed;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int slot = 2 * pr + h;
    if (slot >= N) break;
    int32_t id;
    if (slot < Ndeg) id = endpoint[__umul64hi(x[h], (uint64_t)num_edges)];
    else id = (int32_t)__umul64hi(x[h], (uint64_t)num_nodes);
    out[slot] = id;
  }
}

// N(0, std^2) fill: counter = (block lo, block hi, 0, 0x80000000 | table) gives elements
// 4*block .. 4*block+3 by two Box-Muller pairs on 24-bit uniforms.
__global__ void __launch_bounds__(256)
k_init_normal(float* __restrict__ tab, int64_t n, uint64_t seed, uint32_t table, float std) {
  const int64_t nblocks = (n + 3) >> 2;
  for (int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; b < nblocks; b += (int64_t)gridDim.x * blockDim.x) {
    uint32_t c0 = (uint32_t)b, c1 = (uint32_t)((uint64_t)b >> 32), c2 = 0u, c3 = 0x80000000u | table;
    philox4x32_10(c0, c1, c2, c3, (uint32_t)seed, (uint32_t)(seed >> 32));
    const uint32_t o[4] = {c0, c1, c2, c3};
    float z[4];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const float u1 = (float)((o[2 * p] >> 8) + 1u) * (1.0f / 16777216.0f);
      const float u2 = (float)(o[2 * p + 1] >> 8) * (1.0f / 16777216.0f);
      const float r = sqrtf(-2.0f * logf(u1));
      float sn, cs;
      sincospif(2.0f * u2, &sn, &cs);
      z[2 * p] = r * cs * std;
      z[2 * p + 1] = r * sn * std;
    }
    const int64_t e = b << 2;
    if (e + 3 < n) {
      *reinterpret_cast<float4*>(tab + e) = make_float4(z[0], z[1], z[2], z[3]);
    } else {
      for (int k = 0; k < 4 && e + k < n; ++k) tab[e + k] = z[k];
    }
  }
}

__global__ void __launch_bounds__(256) k_fill_u32(uint32_t* __restrict__ p, int64_t n, uint32_t v) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = v;
}

// ------------------------------------------------------------ occurrence numbering -----
// Occurrence k of a batch with n edges and cn = chunks*N negatives per side (roles = 3, or 2 for
// the relation-free Dot score, which has no relation occurrences):
//   [0,n) source of edge k | [n,2n) destination | [2n,3n) relation (roles = 3 only) |
//   [roles*n, +cn) destination-replacing negatives | then cn source-replacing negatives
struct OccArgs {
  const int32_t *src, *rel, *dst, *neg_src, *neg_dst;
  int32_t n, cn;
  int32_t num_nodes;
  int32_t roles;
};

__device__ __forceinline__ int32_t occ_unified_id(const OccArgs& a, int64_t k) {
  const int64_t n = a.n;
  if (k < n) return a.src[k];
  if (k < 2 * n) return a.dst[k - n];
  if (k < a.roles * n) return a.num_nodes + a.rel[k - 2 * n];
  k -= a.roles * n;
  if (k < a.cn) return a.neg_dst[k];
  return a.neg_src[k - a.cn];
}

// ------------------------------------------------------------- touched-id map -----
// One word holds 2^L ids: L = 5 is a bitmap (marks need atomics), L = 2 one byte per id
// (marks are plain byte stores).  Same-address -- in practice same-cache-line -- atomics
// serialise at tens of ns each, so the bitmap is only used when the id space is large and
// therefore sparse; small dense id spaces take the byte map.
__device__ __forceinline__ uint32_t map_bitpos(uint32_t id, int L) { return (id & ((1u << L) - 1u)) * (32u >> L); }

// Block-wide grouping of equal keys through an LDS hash table (open addressing).
// Blocks of the index kernels stay at 256 threads: they run beside the contraction kernel on
// a second stream and have to fit into the wave slots and registers it leaves free on a CU.
#define AGG_THREADS 256
#define AGG_SLOTS 512
struct BlockAgg {
  int key[AGG_SLOTS];
  uint32_t cnt[AGG_SLOTS];
  uint32_t base[AGG_SLOTS];
};

__device__ __forceinline__ void agg_clear(BlockAgg& t) {
  for (int i = threadIdx.x; i < AGG_SLOTS; i += AGG_THREADS) { t.key[i] = -1; t.cnt[i] = 0u; }
}

// Inserts key, adds mult to its group; returns the slot through `h` and the group-local offset.
__device__ __forceinline__ uint32_t agg_insert(BlockAgg& t, int key, uint32_t mult, int* h_out) {
  int h = (int)(((uint32_t)key * 2654435761u) >> 23);          // 9 bits
  for (;;) {
    const int prev = atomicCAS(&t.key[h], -1, key);
    if (prev == -1 || prev == key) break;
    h = (h + 1) & (AGG_SLOTS - 1);
  }
  *h_out = h;
  return atomicAdd(&t.cnt[h], mult);
}

// Marks the touched-id map.
__global__ void __launch_bounds__(AGG_THREADS)
k_mark(OccArgs a, int64_t n_occ, int L, uint32_t* __restrict__ bitmap) {
  __shared__ BlockAgg tab;
  const int64_t stride = (int64_t)gridDim.x * AGG_THREADS;
  const int64_t t0 = (int64_t)blockIdx.x * AGG_THREADS + threadIdx.x;
  if (L == 2) {
    unsigned char* bytes = reinterpret_cast<unsigned char*>(bitmap);
    for (int64_t k = t0; k < n_occ; k += stride) bytes[(uint32_t)occ_unified_id(a, k)] = 1;
    return;
  }
  // bitmap: one atomic per distinct id of the block, and none if the bit is already visible
  const int64_t rounds = (n_occ + stride - 1) / stride;
  for (int64_t it = 0; it < rounds; ++it) {
    agg_clear(tab);
    __syncthreads();
    const int64_t k = it * stride + t0;
    if (k < n_occ) { int h; agg_insert(tab, occ_unified_id(a, k), 0u, &h); }
    __syncthreads();
    for (int i = threadIdx.x; i < AGG_SLOTS; i += AGG_THREADS) {
      const int key = tab.key[i];
      if (key >= 0) {
        const uint32_t id = (uint32_t)key, bit = 1u << (id & 31u);
        uint32_t* w = bitmap + (id >> 5);
        if (!(__hip_atomic_load(w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & bit)) atomicOr(w, bit);
      }
    }
    __syncthreads();
  }
}

// ------------------------------------------------------------------------- scans -----
// Exclusive prefix sums over f(in[i]); f = popcount for the touched-id map, identity for counts.
template <int POPC> __device__ __forceinline__ uint32_t scan_f(uint32_t v) { return POPC ? (uint32_t)__popc(v) : v; }

// Block-wide exclusive scan of one value per thread (BT threads); returns the exclusive
// prefix and the block total through `total`.
template <int BT>
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* total) {
  __shared__ uint32_t wave_tot[BT / 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t t = __shfl_up(inc, o);
    if (lane >= o) inc += t;
  }
  __syncthreads();                    // protects wave_tot across successive calls
  if (lane == 63) wave_tot[wave] = inc;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < BT / 64; ++w) {
    const uint32_t t = wave_tot[w];
    if (w < wave) base += t;
    tot += t;
  }
  *total = tot;
  return base + inc - v;
}

#define SCAN_PER_THREAD 16
#define SCAN_BLOCK_ELEMS (256 * SCAN_PER_THREAD)

template <int POPC>
__global__ void __launch_bounds__(256)
k_scan_block_sums(const uint32_t* __restrict__ in, int64_t n, uint32_t* __restrict__ bsum) {
  const int64_t base = (int64_t)blockIdx.x * SCAN_BLOCK_ELEMS + (int64_t)threadIdx.x * SCAN_PER_THREAD;
  uint32_t s = 0;
#pragma unroll
  for (int j = 0; j < SCAN_PER_THREAD; ++j) if (base + j < n) s += scan_f<POPC>(in[base + j]);
  uint32_t tot;
  block_exclusive_scan<256>(s, &tot);
  if (threadIdx.x == 0) bsum[blockIdx.x] = tot;
}

// One block: exclusive scan of bsum[0..nb) in place.
__global__ void __launch_bounds__(256) k_scan_bsum(uint32_t* __restrict__ bsum, int64_t nb) {
  uint32_t carry = 0;
  for (int64_t b0 = 0; b0 < nb; b0 += 256) {
    const int64_t i = b0 + threadIdx.x;
    const uint32_t v = i < nb ? bsum[i] : 0u;
    uint32_t tot;
    const uint32_t ex = block_exclusive_scan<256>(v, &tot);
    if (i < nb) bsum[i] = carry + ex;
    carry += tot;
  }
}

// Writes out[i] = exclusive prefix.  With POPC: also emits the ascending ids of the marked
// positions (L = log2 ids per word), the unique-row total into scalars[0] and the number of
// marks below `split_id` (the first relation's unified id) into scalars[1].  With
// `single_block` the kernel loops over the whole input itself and needs no block sums.
template <int POPC, int BT, int PER>
__global__ void __launch_bounds__(BT, 8)
k_scan_apply(const uint32_t* __restrict__ in, int64_t n, const uint32_t* __restrict__ bsum, int single_block, int L,
             uint32_t* __restrict__ out, int32_t* __restrict__ uniq, int32_t* __restrict__ scalars, int64_t split_id) {
  constexpr int ELEMS = BT * PER;
  const int64_t nblk = (n + ELEMS - 1) / ELEMS;
  const int bpi = 32 >> L;                                   // bits per id
  uint32_t carry = 0;
  for (int64_t blk = single_block ? 0 : blockIdx.x; blk < nblk; blk += single_block ? 1 : gridDim.x) {
    const int64_t base = blk * ELEMS + (int64_t)threadIdx.x * PER;
    uint32_t v[PER];
    uint32_t s = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      v[j] = base + j < n ? in[base + j] : 0u;
      s += scan_f<POPC>(v[j]);
    }
    uint32_t tot;
    uint32_t run = block_exclusive_scan<BT>(s, &tot) + (single_block ? carry : bsum[blk]);
    carry += tot;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      if (base + j < n) {
        out[base + j] = run;
        if (POPC) {
          uint32_t w = v[j];
          const int64_t id0 = (base + j) << L;
          if (id0 <= split_id && split_id < id0 + (1 << L))
            scalars[1] = (int32_t)(run + __popc(w & ((1u << ((split_id - id0) * bpi)) - 1u)));
          uint32_t r = run;
          while (w) {
            const int b = __ffs(w) - 1;
            uniq[r++] = (int32_t)(id0 + b / bpi);
            w &= w - 1;
          }
        }
        run += scan_f<POPC>(v[j]);
      }
    }
    if (POPC && base <= n - 1 && n - 1 < base + PER) scalars[0] = (int32_t)run;   // thread owning the last word
  }
}

template <int POPC>
static hipError_t scan_u32(const uint32_t* in, int64_t n, int L, uint32_t* out, uint32_t* bsum, int32_t* uniq,
                           int32_t* scalars, int64_t split_id, hipStream_t st) {
  if (n <= 256) {
    hipLaunchKernelGGL((k_scan_apply<POPC, 256, 1>), dim3(1), dim3(256), 0, st, in, n, bsum, 1, L, out, uniq, scalars, split_id);
  } else if (n <= 1024 * 4) {
    hipLaunchKernelGGL((k_scan_apply<POPC, 256, 4>), dim3(1), dim3(256), 0, st, in, n, bsum, 1, L, out, uniq, scalars, split_id);
  } else if (n <= 4096 * 8) {
    hipLaunchKernelGGL((k_scan_apply<POPC, 256, 16>), dim3(1), dim3(256), 0, st, in, n, bsum, 1, L, out, uniq, scalars, split_id);
  } else {
    const int64_t nblk = (n + SCAN_BLOCK_ELEMS - 1) / SCAN_BLOCK_ELEMS;
    hipLaunchKernelGGL(k_scan_block_sums<POPC>, dim3((unsigned)nblk), dim3(256), 0, st, in, n, bsum);
    hipLaunchKernelGGL(k_scan_bsum, dim3(1), dim3(256), 0, st, bsum, nblk);
    hipLaunchKernelGGL((k_scan_apply<POPC, 256, SCAN_PER_THREAD>), dim3((unsigned)nblk), dim3(256), 0, st, in, n, bsum, 0, L, out,
                       uniq, scalars, split_id);
  }
  return hipGetLastError();
}

// ------------------------------------------------ row-sorted order of the gradient rows -----
// Gradient row gr belongs to occurrence k = gr (edge side, gr < roles*n) or to part (gr - roles*n) % sy2
// of negative occurrence roles*n + (gr - roles*n) / sy2; its sort key is the rank of the occurrence's
// table row among the unique rows.  A least-significant-digit radix sort with digits of `bits` bits puts
// the gradient rows in key order; every pass is stable, so equal keys stay in gradient-row order.
// One pass = k_sort_hist (digit counts per tile of MAR_SORT_TILE elements) + k_sort_scatter (each tile
// derives its digits' global offsets from the counts of all tiles and scatters its elements).

// Lanes of the wave that hold the same digit as this lane (valid lanes only).
__device__ __forceinline__ uint64_t match_digit(uint32_t digit, int bits, bool valid) {
  uint64_t mask = __ballot(valid);
  for (int b = 0; b < bits; ++b) {
    const bool bit = (digit >> b) & 1u;
    const uint64_t bal = __ballot(bit);
    mask &= bit ? bal : ~bal;
  }
  return mask;
}

// FIRST: computes the keys from the touched-id map and its prefix sums and stores them.
template <int FIRST>
__global__ void __launch_bounds__(256)
k_sort_hist(OccArgs a, int64_t n_pos, int sy2, int L, const uint32_t* __restrict__ bitmap,
            const uint32_t* __restrict__ word_prefix, const uint32_t* __restrict__ keys_in,
            uint32_t* __restrict__ keys_out, int shift, int bits, uint32_t* __restrict__ hist) {
  __shared__ uint32_t h[1 << MAR_SORT_MAX_BITS];
  const int bins = 1 << bits;
  const int lane = threadIdx.x & 63;
  for (int i = threadIdx.x; i < bins; i += 256) h[i] = 0u;
  __syncthreads();
  const int64_t base = (int64_t)blockIdx.x * MAR_SORT_TILE;
  const int64_t n3 = a.roles * (int64_t)a.n;
  constexpr int ITEMS = MAR_SORT_TILE / 256;
  // keys of this thread's elements; the three dependent loads behind a key (id, map word, prefix) are issued
  // level by level for all elements, so the kernel pays three memory round trips, not three per element
  uint32_t key[ITEMS];
  if (FIRST) {
    uint32_t id[ITEMS], word[ITEMS];
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
      const int64_t gr = base + j * 256 + threadIdx.x;
      const int64_t grc = gr < n_pos ? gr : n_pos - 1;
      id[j] = (uint32_t)occ_unified_id(a, grc < n3 ? grc : n3 + (grc - n3) / sy2);
    }
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) { word[j] = bitmap[id[j] >> L]; key[j] = word_prefix[id[j] >> L]; }
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
      key[j] += __popc(word[j] & ((1u << map_bitpos(id[j], L)) - 1u));
      const int64_t gr = base + j * 256 + threadIdx.x;
      if (gr < n_pos) keys_out[gr] = key[j];
    }
  } else {
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
      const int64_t gr = base + j * 256 + threadIdx.x;
      key[j] = gr < n_pos ? keys_in[gr] : 0u;
    }
  }
#pragma unroll
  for (int j = 0; j < ITEMS; ++j) {
    const bool valid = base + j * 256 + threadIdx.x < n_pos;
    // one LDS atomic per distinct digit of the wave (a hot row fills whole waves with one key)
    const uint32_t digit = (key[j] >> shift) & (uint32_t)(bins - 1);
    const uint64_t same = match_digit(digit, bits, valid);
    if (valid && (same & ((1ull << lane) - 1ull)) == 0ull) atomicAdd(&h[digit], (uint32_t)__popcll(same));
  }
  __syncthreads();
  for (int i = threadIdx.x; i < bins; i += 256) hist[(size_t)blockIdx.x * bins + i] = h[i];
}

// Scatters the tile's elements to their places in digit order.  Global place of an element =
// (elements with a smaller digit anywhere) + (same digit in earlier tiles) + (same digit earlier in this
// tile).  Inside the tile wave w owns a contiguous quarter and walks it 64 consecutive elements at a time,
// so "earlier in this tile" = same digit in earlier waves + earlier rounds of this wave + lower lanes.
// vals_in == NULL: the values are the element indices (first pass).
__global__ void __launch_bounds__(256)
k_sort_scatter(const uint32_t* __restrict__ keys_in, const int32_t* __restrict__ vals_in,
               uint32_t* __restrict__ keys_out, int32_t* __restrict__ vals_out, const uint32_t* __restrict__ hist,
               int64_t n, int shift, int bits, int ntiles) {
  constexpr int ITEMS = MAR_SORT_TILE / 256;
  __shared__ uint32_t wcnt[4][1 << MAR_SORT_MAX_BITS];      // per wave: elements per digit, then their exclusive prefix over waves
  __shared__ uint32_t gbase[1 << MAR_SORT_MAX_BITS];        // global place of the tile's first element of each digit
  const int bins = 1 << bits;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int i = threadIdx.x; i < 4 * bins; i += 256) wcnt[i / bins][i % bins] = 0u;

  // keys of this wave's quarter, round r = 64 consecutive elements
  const int64_t q0 = (int64_t)blockIdx.x * MAR_SORT_TILE + (int64_t)wave * (MAR_SORT_TILE / 4) + lane;
  uint32_t key[ITEMS];
#pragma unroll
  for (int r = 0; r < ITEMS; ++r) key[r] = q0 + 64 * r < n ? keys_in[q0 + 64 * r] : 0u;

  // digit offsets: thread t owns digits [t*per, (t+1)*per)
  const int per = (bins + 255) / 256;
  uint32_t before[4] = {0u, 0u, 0u, 0u}, total[4] = {0u, 0u, 0u, 0u};
  const int d0 = threadIdx.x * per;
  // the tiles' counts are fetched eight tiles at a time (independent loads), summed in tile order
  for (int b0 = 0; b0 < ntiles; b0 += 8) {
    uint32_t v[8][4];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const uint32_t* hrow = hist + (size_t)(b0 + i) * bins;
#pragma unroll
      for (int j = 0; j < 4; ++j) v[i][j] = (b0 + i < ntiles && j < per && d0 + j < bins) ? hrow[d0 + j] : 0u;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        total[j] += v[i][j];
        if (b0 + i < (int)blockIdx.x) before[j] += v[i][j];
      }
    }
  }
  uint32_t tot_all;
  uint32_t run = block_exclusive_scan<256>((total[0] + total[1]) + (total[2] + total[3]), &tot_all);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if (j < per && d0 + j < bins) { gbase[d0 + j] = run + before[j]; run += total[j]; }
  }
  __syncthreads();                                          // counters cleared, gbase written

  uint32_t loc[ITEMS];
#pragma unroll
  for (int r = 0; r < ITEMS; ++r) {
    const bool valid = q0 + 64 * r < n;
    const uint32_t digit = (key[r] >> shift) & (uint32_t)(bins - 1);
    const uint64_t same = match_digit(digit, bits, valid);
    const uint32_t lower = (uint32_t)__popcll(same & ((1ull << lane) - 1ull));
    loc[r] = 0u;
    if (valid) {
      // every lane of a group reads the wave's counter before the group's first lane advances it: one wave
      // executes both accesses in program order
      const uint32_t old = wcnt[wave][digit];
      loc[r] = old + lower;
      if (lower == 0u) wcnt[wave][digit] = old + (uint32_t)__popcll(same);
    }
  }
  __syncthreads();
  for (int d = threadIdx.x; d < bins; d += 256) {
    const uint32_t c0 = wcnt[0][d], c1 = wcnt[1][d], c2 = wcnt[2][d];
    wcnt[0][d] = 0u; wcnt[1][d] = c0; wcnt[2][d] = c0 + c1; wcnt[3][d] = c0 + c1 + c2;
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < ITEMS; ++r) {
    const int64_t idx = q0 + 64 * r;
    if (idx < n) {
      const uint32_t digit = (key[r] >> shift) & (uint32_t)(bins - 1);
      const uint32_t p = gbase[digit] + wcnt[wave][digit] + loc[r];
      keys_out[p] = key[r];
      vals_out[p] = vals_in ? vals_in[idx] : (int32_t)idx;
    }
  }
}

// Segment starts of the row-sorted order (every unique row has at least one position), the end sentinel,
// the reset of the owner list's counter, and the reset of the touched-id map for the next step.
__global__ void __launch_bounds__(256)
k_segments(OccArgs a, int64_t n_occ, int64_t n_pos, int L, const int32_t* __restrict__ rank_sorted,
           uint32_t* __restrict__ seg_off, uint32_t* __restrict__ bitmap, int32_t* __restrict__ scalars) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i == 0) scalars[2] = 0;
  if (i < n_pos) {
    const int r = rank_sorted[i];
    if (i == 0 || rank_sorted[i - 1] != r) seg_off[r] = (uint32_t)i;
    if (i == n_pos - 1) seg_off[r + 1] = (uint32_t)n_pos;
  }
  if (i < n_occ) bitmap[(uint32_t)occ_unified_id(a, i) >> L] = 0u;
}

// Copies the unique id lists into the caller's debug buffers.
__global__ void __launch_bounds__(256)
k_debug_uniq(const int32_t* __restrict__ uniq, const int32_t* __restrict__ scalars, int32_t num_nodes,
             int32_t* __restrict__ num_uniq, int32_t* __restrict__ uniq_nodes, int32_t* __restrict__ uniq_rels) {
  const int total = scalars[0], un = scalars[1];
  if (blockIdx.x == 0 && threadIdx.x == 0 && num_uniq) { num_uniq[0] = un; num_uniq[1] = total - un; }
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
    if (i < un) { if (uniq_nodes) uniq_nodes[i] = uniq[i]; }
    else if (uniq_rels) uniq_rels[i - un] = uniq[i] - num_nodes;
  }
}

// ------------------------------------------------------------------- launchers -----
static inline unsigned grid_for(int64_t n, int threads, unsigned cap) {
  int64_t g = (n + threads - 1) / threads;
  if (g < 1) g = 1;
  if (g > cap) g = cap;
  return (unsigned)g;
}

hipError_t mar_launch_init(const mar_ctx* c, int fill, hipStream_t st) {
  const MarDims& d = c->dm;
  hipLaunchKernelGGL(k_fill_u32, dim3(grid_for(d.nwords, 256, 4096)), dim3(256), 0, st, c->L.bitmap, d.nwords, 0u);
  hipLaunchKernelGGL(k_fill_u32, dim3(1), dim3(64), 0, st, (uint32_t*)c->L.scalars, (int64_t)16, 0u);
  if (fill) {
    const int64_t nn = d.num_nodes * d.dim, nr = (int64_t)d.num_rels * d.dim;
    hipLaunchKernelGGL(k_init_normal, dim3(grid_for((nn + 3) / 4, 256, 1 << 16)), dim3(256), 0, st,
                       c->node_emb, nn, c->cfg.seed, 0u, c->cfg.init_std);
    hipLaunchKernelGGL(k_init_normal, dim3(grid_for((nr + 3) / 4, 256, 1 << 16)), dim3(256), 0, st,
                       c->rel_emb, nr, c->cfg.seed, 1u, c->cfg.init_std);
    hipLaunchKernelGGL(k_fill_u32, dim3(grid_for(nn, 256, 1 << 16)), dim3(256), 0, st, (uint32_t*)c->node_state, nn, 0u);
    hipLaunchKernelGGL(k_fill_u32, dim3(grid_for(nr, 256, 1 << 16)), dim3(256), 0, st, (uint32_t*)c->rel_state, nr, 0u);
  }
  return hipGetLastError();
}

hipError_t mar_launch_clear_bitmap(const mar_ctx* c, hipStream_t st) {
  hipLaunchKernelGGL(k_fill_u32, dim3(grid_for(c->dm.nwords, 256, 4096)), dim3(256), 0, st, c->L.bitmap, c->dm.nwords, 0u);
  return hipGetLastError();
}

hipError_t mar_launch_fill_u32(uint32_t* p, int64_t n, uint32_t v, hipStream_t st) {
  hipLaunchKernelGGL(k_fill_u32, dim3(grid_for(n, 256, 4096)), dim3(256), 0, st, p, n, v);
  return hipGetLastError();
}

hipError_t mar_launch_sample(const mar_ctx* c, uint64_t step, const int32_t* es, const int32_t* ed,
                             int64_t num_edges, int32_t* neg_src, int32_t* neg_dst, hipStream_t st) {
  const MarDims& d = c->dm;
  const int64_t total = (int64_t)2 * d.C * ((d.N + 1) / 2);
  hipLaunchKernelGGL(k_sample, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, c->cfg.seed, step,
                     d.num_nodes, es, ed, num_edges, d.C, d.N, d.Ndeg, neg_src, neg_dst);
  return hipGetLastError();
}

hipError_t mar_launch_index(const mar_ctx* c, const MarBatch& b, hipStream_t st) {
  const MarDims& d = c->dm;
  const MarLayout& L = c->L;
  OccArgs a{b.src, b.rel, b.dst, b.neg_src, b.neg_dst, b.n, b.cn, (int32_t)d.num_nodes, d.roles};
  hipLaunchKernelGGL(k_mark, dim3(grid_for(b.n_occ, AGG_THREADS, 2048)), dim3(AGG_THREADS), 0, st, a, b.n_occ, (int)d.ipw_log2,
                     L.bitmap);
  hipError_t e = scan_u32<1>(L.bitmap, d.nwords, d.ipw_log2, L.word_prefix, L.bsum, L.uniq, L.scalars, d.num_nodes, st);
  if (e != hipSuccess) return e;
  // stable radix sort of the gradient rows by rank; the last pass writes rank_sorted / perm
  const int ntiles = (int)((b.n_pos + MAR_SORT_TILE - 1) / MAR_SORT_TILE);
  const uint32_t* kin = L.keys0;
  const int32_t* vin = nullptr;
  for (int p = 0; p < d.sort_passes; ++p) {
    const bool last = p == d.sort_passes - 1;
    uint32_t* kout = last ? (uint32_t*)L.rank_sorted : L.kbuf[p & 1];
    int32_t* vout = last ? L.perm : L.vbuf[p & 1];
    const int shift = p * d.sort_bits;
    if (p == 0)
      hipLaunchKernelGGL(k_sort_hist<1>, dim3(ntiles), dim3(256), 0, st, a, b.n_pos, (int)d.sy2, (int)d.ipw_log2, L.bitmap,
                         L.word_prefix, nullptr, L.keys0, shift, (int)d.sort_bits, L.hist);
    else
      hipLaunchKernelGGL(k_sort_hist<0>, dim3(ntiles), dim3(256), 0, st, a, b.n_pos, (int)d.sy2, (int)d.ipw_log2, L.bitmap,
                         L.word_prefix, kin, nullptr, shift, (int)d.sort_bits, L.hist);
    hipLaunchKernelGGL(k_sort_scatter, dim3(ntiles), dim3(256), 0, st, kin, vin, kout, vout, L.hist, b.n_pos, shift,
                       (int)d.sort_bits, ntiles);
    kin = kout; vin = vout;
  }
  const int64_t work = b.n_pos > b.n_occ ? b.n_pos : b.n_occ;
  hipLaunchKernelGGL(k_segments, dim3((unsigned)((work + 255) / 256)), dim3(256), 0, st, a, b.n_occ, b.n_pos, (int)d.ipw_log2,
                     L.rank_sorted, L.seg_off, L.bitmap, L.scalars);
  return hipGetLastError();
}

hipError_t mar_launch_debug_copy(const mar_ctx* c, const MarBatch& b, const mar_debug_out* dbg, hipStream_t st) {
  (void)b;
  if (dbg->num_uniq || dbg->uniq_nodes || dbg->uniq_rels)
    hipLaunchKernelGGL(k_debug_uniq, dim3(64), dim3(256), 0, st, c->L.uniq, c->L.scalars, (int32_t)c->dm.num_nodes,
                       dbg->num_uniq, dbg->uniq_nodes, dbg->uniq_rels);
  return hipGetLastError();
}

// Host-side edge-bucket ordering (no device code): the BETA buffer sequence (Alg. 3), its
// conversion to an edge-bucket order (Alg. 4), and a partition-buffer simulator that replays an
// order with furthest-in-future eviction (Alg. 2) and counts partition loads.  Closed forms of
// Sec. 4.1: lower bound on swaps (Eq. 2) and the swap count of BETA (Eq. 3).
#include <stdint.h>
#include <stdlib.h>
#include <algorithm>
#include <vector>

#include "mar_common.h"

namespace {

int order_fail(int code, const char* msg) {
  mar_set_error("%s", msg);
  return code;
}

// Philox4x32-10 on the host (Salmon et al., SC'11); only words 0 and 1 of the block are used.
uint64_t philox_word01(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint64_t seed) {
  uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c0 = n0; c1 = (uint32_t)p1; c2 = n2; c3 = (uint32_t)p0;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  return (uint64_t)c0 | ((uint64_t)c1 << 32);
}

// The BETA buffer sequence (Alg. 3) as a stream of swaps.  The walk keeps c - 1 "fixed" slots and one "cycling"
// slot (the last).  A round over the m partitions still outside the buffer is a rotation: each of them passes
// through the cycling slot in order (m swaps), which leaves the slot holding the last of them and the outside
// pool holding [what the slot held before, then all but the last of them]; the fixed partitions have then met
// everybody and the first min(c - 1, m) of the pool take their places one by one (they leave the pool; the
// partitions they replace are done for good).  visit(slot, incoming) is called once per swap, in order.
template <class Visit>
void beta_walk(int p, int c, Visit visit) {
  std::vector<int32_t> pool(p - c);
  for (int i = 0; i < p - c; ++i) pool[i] = c + i;
  int32_t cycling = c - 1;                                   // partition in the cycling slot
  while (!pool.empty()) {
    const size_t m = pool.size();
    for (size_t i = 0; i < m; ++i) visit(c - 1, pool[i]);
    const int32_t came_last = pool[m - 1];
    for (size_t i = m - 1; i > 0; --i) pool[i] = pool[i - 1];   // rotate: the slot's old content heads the pool
    pool[0] = cycling;
    cycling = came_last;
    const size_t n = std::min<size_t>((size_t)c - 1, m);
    for (size_t i = 0; i < n; ++i) visit((int)i, pool[i]);
    pool.erase(pool.begin(), pool.begin() + n);
  }
}

// Who has shared a buffer with whom: one bit row per partition.
struct MetMatrix {
  int p; size_t words;
  std::vector<uint64_t> bits;
  explicit MetMatrix(int p_) : p(p_), words(((size_t)p_ + 63) / 64), bits(words * (size_t)p_, 0) {}
  bool test_and_set(int i, int j) {
    uint64_t& w = bits[(size_t)i * words + ((size_t)j >> 6)];
    const uint64_t m = 1ull << (j & 63);
    const bool was = (w & m) != 0;
    w |= m;
    return was;
  }
};

}  // namespace

extern "C" int64_t mar_swap_lower_bound(int32_t p, int32_t c) {
  if (c < 2 || p < c) return -1;
  const int64_t pairs = (int64_t)p * (p - 1) / 2 - (int64_t)c * (c - 1) / 2;
  return (pairs + (c - 2)) / (c - 1);
}

extern "C" int64_t mar_beta_swap_count(int32_t p, int32_t c) {
  if (c < 2 || p < c) return -1;
  const int64_t x = (p - c) / (c - 1);
  return (2 * (int64_t)(p - c) + (x + 1) * (2 * (int64_t)(p - c) - x * (c - 1))) / 2;
}

extern "C" int mar_beta_buffer_sequence(int32_t p, int32_t c, int32_t* buffers, int64_t capacity_rows, int64_t* num_rows) {
  if (c < 2 || p < c) return order_fail(MAR_EINVAL, "need 2 <= c <= p");
  if (!num_rows) return order_fail(MAR_EINVAL, "num_rows is NULL");
  const int64_t rows = mar_beta_swap_count(p, c) + 1;        // one row per swap (Eq. 3) after the first buffer
  *num_rows = rows;
  if (!buffers) return MAR_OK;                              // size query
  if (capacity_rows < rows) return order_fail(MAR_ENOMEM, "buffer sequence does not fit");
  for (int i = 0; i < c; ++i) buffers[i] = i;
  int64_t r = 0;
  beta_walk(p, c, [&](int slot, int32_t incoming) {          // row r + 1 = row r with one slot replaced
    int32_t* next = buffers + (r + 1) * c;
    std::copy(buffers + r * c, buffers + (r + 1) * c, next);
    next[slot] = incoming;
    ++r;
  });
  return r + 1 == rows ? MAR_OK : order_fail(MAR_ERANGE, "internal: swap count does not match Eq. 3");
}

extern "C" int mar_beta_edge_bucket_order(int32_t p, int32_t c, int32_t shuffle, uint64_t seed, int32_t* pairs) {
  if (c < 2 || p < c) return order_fail(MAR_EINVAL, "need 2 <= c <= p");
  if (!pairs) return order_fail(MAR_EINVAL, "pairs is NULL");
  if ((int64_t)p * p > ((int64_t)1 << 30)) return order_fail(MAR_ERANGE, "too many edge buckets");
  // Alg. 4 asks for every bucket (i, j) the first time both partitions are in the buffer.  After a swap the only
  // new candidates involve the partition that came in, so each buffer's group is emitted from that partition's
  // row of the who-met-whom matrix, in the order a row-major scan of the buffer's slots would find them: (x' , x)
  // for the slots before the swapped one, then (x, .) for all slots, then (x', x) for the slots behind it.
  MetMatrix met(p);
  std::vector<int32_t> buf(c);
  size_t out = 0, buffer_index = 0;
  auto emit = [&](int32_t i, int32_t j) {
    if (!met.test_and_set(i, j)) { pairs[2 * out] = i; pairs[2 * out + 1] = j; ++out; }
  };
  auto close_group = [&](size_t first) {
    if (shuffle) {
      // Fisher-Yates from the back, j = high 64 bits of x * (k + 1)
      const size_t m = out - first;
      for (size_t k = m; k-- > 1;) {
        const uint64_t x = philox_word01((uint32_t)k, (uint32_t)buffer_index, 0u, 0x40000000u, seed);
        const size_t j = (size_t)(((unsigned __int128)x * (k + 1)) >> 64);
        std::swap(pairs[2 * (first + k)], pairs[2 * (first + j)]);
        std::swap(pairs[2 * (first + k) + 1], pairs[2 * (first + j) + 1]);
      }
    }
    ++buffer_index;
  };
  for (int i = 0; i < c; ++i) buf[i] = i;
  for (int i = 0; i < c; ++i)
    for (int j = 0; j < c; ++j) emit(buf[i], buf[j]);
  close_group(0);
  beta_walk(p, c, [&](int slot, int32_t x) {
    const size_t first = out;
    buf[slot] = x;
    for (int i = 0; i < slot; ++i) emit(buf[i], x);
    for (int j = 0; j < c; ++j) emit(x, buf[j]);
    for (int i = slot + 1; i < c; ++i) emit(buf[i], x);
    close_group(first);
  });
  return out == (size_t)p * p ? MAR_OK : order_fail(MAR_ERANGE, "internal: not every bucket was emitted");
}

extern "C" int mar_buffer_simulate(int32_t p, int32_t c, const int32_t* pairs, int64_t n_pairs, int64_t* loads) {
  if (c < 2 || p < c) return order_fail(MAR_EINVAL, "need 2 <= c <= p");
  if (!pairs || !loads || n_pairs < 0) return order_fail(MAR_EINVAL, "bad arguments");
  for (int64_t k = 0; k < 2 * n_pairs; ++k)
    if (pairs[k] < 0 || pairs[k] >= p) return order_fail(MAR_ERANGE, "partition id out of range");
  // next_use[k][side]: next position after k at which the same partition is needed again
  std::vector<int64_t> next_of((size_t)2 * n_pairs), last((size_t)p, n_pairs);
  for (int64_t k = n_pairs - 1; k >= 0; --k) {
    // the two endpoints of bucket k are used at position k; process the second endpoint first so that a
    // self bucket (i, i) links to the later use
    for (int s = 1; s >= 0; --s) {
      const int32_t x = pairs[2 * k + s];
      next_of[2 * k + s] = last[x] == k ? next_of[2 * k + 1] : last[x];
      last[x] = k;
    }
  }
  std::vector<int64_t> next_use((size_t)p, n_pairs);       // for partitions in the buffer: next position needed
  std::vector<uint8_t> in_buf((size_t)p, 0);
  int64_t size = 0, cnt = 0;
  for (int64_t k = 0; k < n_pairs; ++k) {
    const int32_t i = pairs[2 * k], j = pairs[2 * k + 1];
    for (int s = 0; s < 2; ++s) {
      const int32_t x = s == 0 ? i : j;
      if (!in_buf[x]) {
        if (size == c) {
          int32_t victim = -1; int64_t far = -1;
          for (int32_t y = 0; y < p; ++y)
            if (in_buf[y] && y != i && y != j && next_use[y] > far) { far = next_use[y]; victim = y; }
          in_buf[victim] = 0; --size;
        }
        in_buf[x] = 1; ++size; ++cnt;
      }
    }
    // both endpoints are now in use at k: their next use is after k
    next_use[i] = next_of[2 * k];
    next_use[j] = next_of[2 * k + 1];
  }
  *loads = cnt;
  return MAR_OK;
}

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

std::vector<std::vector<int32_t>> buffer_sequence(int p, int c) {
  std::vector<std::vector<int32_t>> seq;
  std::vector<int32_t> cur(c), disk;
  for (int i = 0; i < c; ++i) cur[i] = i;
  for (int i = c; i < p; ++i) disk.push_back(i);
  seq.push_back(cur);
  while (!disk.empty()) {
    // the leading c-1 partitions stay; every partition on disk passes through the last slot
    for (size_t i = 0; i < disk.size(); ++i) {
      std::swap(cur[c - 1], disk[i]);
      seq.push_back(cur);
    }
    // the leading partitions have met every other one: bring in fresh ones
    size_t n = 0;
    for (int i = 0; i < c - 1 && (size_t)i < disk.size(); ++i) {
      cur[i] = disk[i];
      seq.push_back(cur);
      ++n;
    }
    disk.erase(disk.begin(), disk.begin() + n);
  }
  return seq;
}

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
  const auto seq = buffer_sequence(p, c);
  *num_rows = (int64_t)seq.size();
  if (!buffers) return MAR_OK;                              // size query
  if (capacity_rows < (int64_t)seq.size()) return order_fail(MAR_ENOMEM, "buffer sequence does not fit");
  for (size_t r = 0; r < seq.size(); ++r)
    for (int i = 0; i < c; ++i) buffers[r * c + i] = seq[r][i];
  return MAR_OK;
}

extern "C" int mar_beta_edge_bucket_order(int32_t p, int32_t c, int32_t shuffle, uint64_t seed, int32_t* pairs) {
  if (c < 2 || p < c) return order_fail(MAR_EINVAL, "need 2 <= c <= p");
  if (!pairs) return order_fail(MAR_EINVAL, "pairs is NULL");
  if ((int64_t)p * p > ((int64_t)1 << 30)) return order_fail(MAR_ERANGE, "too many edge buckets");
  const auto seq = buffer_sequence(p, c);
  std::vector<uint8_t> seen((size_t)p * p, 0);
  size_t out = 0;
  for (size_t b = 0; b < seq.size(); ++b) {
    const size_t first = out;
    for (int i : seq[b])
      for (int j : seq[b])
        if (!seen[(size_t)i * p + j]) {
          seen[(size_t)i * p + j] = 1;
          pairs[2 * out] = i; pairs[2 * out + 1] = j;
          ++out;
        }
    if (shuffle) {
      // Fisher-Yates from the back, j = high 64 bits of x * (k + 1)
      const size_t m = out - first;
      for (size_t k = m; k-- > 1;) {
        const uint64_t x = philox_word01((uint32_t)k, (uint32_t)b, 0u, 0x40000000u, seed);
        const size_t j = (size_t)(((unsigned __int128)x * (k + 1)) >> 64);
        std::swap(pairs[2 * (first + k)], pairs[2 * (first + j)]);
        std::swap(pairs[2 * (first + k) + 1], pairs[2 * (first + j) + 1]);
      }
    }
  }
  return MAR_OK;
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

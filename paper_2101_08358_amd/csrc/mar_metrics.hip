// Link-prediction metrics from ranks (Sec. 5.1, "Evaluation Task and Metrics"): MRR and Hits@k (gfx950).
//
// Two kernels: k_rank_partial sums 1/rank and the hit counts of MAR_METRIC_TILE ranks per workgroup into
// one partial record, k_rank_final adds the records.  Every sum follows a fixed tree that depends only on
// the number of ranks, so the result is bit-reproducible.  The partial records live in the context's
// workspace.
#include "mar_common.h"

struct MetricKs { int32_t k[8]; int32_t num; };
struct MetricPart { double rr; unsigned long long hit[8]; };
static_assert(sizeof(MetricPart) == MAR_METRIC_PART_BYTES, "partial record size");

// Workgroup b sums the ranks of tiles b, b + gridDim.x, ...: thread t takes elements t, t + 256, ... of a
// tile, then the 256 threads' sums are combined by a binary tree in LDS.
__global__ void __launch_bounds__(256)
k_rank_partial(const int32_t* __restrict__ ranks, int64_t n, MetricKs ks, MetricPart* __restrict__ part) {
  __shared__ double s_rr[256];
  __shared__ unsigned long long s_hit[8][256];
  double rr = 0.0;
  unsigned long long hit[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int64_t t0 = (int64_t)blockIdx.x * MAR_METRIC_TILE; t0 < n; t0 += (int64_t)gridDim.x * MAR_METRIC_TILE) {
#pragma unroll 4
    for (int j = 0; j < MAR_METRIC_TILE / 256; ++j) {
      const int64_t i = t0 + j * 256 + threadIdx.x;
      if (i < n) {
        const int r = ranks[i];
        rr += 1.0 / (double)r;
#pragma unroll
        for (int q = 0; q < 8; ++q) if (q < ks.num && r <= ks.k[q]) hit[q]++;
      }
    }
  }
  s_rr[threadIdx.x] = rr;
#pragma unroll
  for (int q = 0; q < 8; ++q) s_hit[q][threadIdx.x] = hit[q];
  __syncthreads();
  for (int o = 128; o >= 1; o >>= 1) {
    if ((int)threadIdx.x < o) {
      s_rr[threadIdx.x] += s_rr[threadIdx.x + o];
#pragma unroll
      for (int q = 0; q < 8; ++q) s_hit[q][threadIdx.x] += s_hit[q][threadIdx.x + o];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    MetricPart p;
    p.rr = s_rr[0];
    for (int q = 0; q < 8; ++q) p.hit[q] = s_hit[q][0];
    part[blockIdx.x] = p;
  }
}

// One workgroup: thread t adds records t, t + 256, ..., then the same tree; writes MRR and Hits@k.
__global__ void __launch_bounds__(256)
k_rank_final(const MetricPart* __restrict__ part, int nparts, int64_t n, MetricKs ks, double* __restrict__ out) {
  __shared__ double s_rr[256];
  __shared__ unsigned long long s_hit[8][256];
  double rr = 0.0;
  unsigned long long hit[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int i = threadIdx.x; i < nparts; i += 256) {
    const MetricPart p = part[i];
    rr += p.rr;
#pragma unroll
    for (int q = 0; q < 8; ++q) hit[q] += p.hit[q];
  }
  s_rr[threadIdx.x] = rr;
#pragma unroll
  for (int q = 0; q < 8; ++q) s_hit[q][threadIdx.x] = hit[q];
  __syncthreads();
  for (int o = 128; o >= 1; o >>= 1) {
    if ((int)threadIdx.x < o) {
      s_rr[threadIdx.x] += s_rr[threadIdx.x + o];
#pragma unroll
      for (int q = 0; q < 8; ++q) s_hit[q][threadIdx.x] += s_hit[q][threadIdx.x + o];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    out[0] = n > 0 ? s_rr[0] / (double)n : 0.0;
    for (int q = 0; q < ks.num; ++q) out[1 + q] = n > 0 ? (double)s_hit[q][0] / (double)n : 0.0;
  }
}

// `part` holds MAR_METRIC_MAX_PARTS records.  Every record the second kernel reads is written by the first
// in the same call, so the buffer needs no clearing.
hipError_t mar_launch_rank_metrics(const int32_t* ranks, int64_t n, const int32_t* ks, int num_k, double* out, void* part,
                                   hipStream_t st) {
  MetricKs m;
  m.num = num_k;
  for (int j = 0; j < 8; ++j) m.k[j] = j < num_k ? ks[j] : 0;
  int64_t nparts = (n + MAR_METRIC_TILE - 1) / MAR_METRIC_TILE;
  if (nparts > MAR_METRIC_MAX_PARTS) nparts = MAR_METRIC_MAX_PARTS;
  MetricPart* p = reinterpret_cast<MetricPart*>(part);
  if (nparts > 0) hipLaunchKernelGGL(k_rank_partial, dim3((unsigned)nparts), dim3(256), 0, st, ranks, n, m, p);
  hipLaunchKernelGGL(k_rank_final, dim3(1), dim3(256), 0, st, p, (int)nparts, n, m, out);
  return hipGetLastError();
}

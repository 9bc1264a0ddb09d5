// Link-prediction metrics from ranks (Sec. 5.1, "Evaluation Task and Metrics"): MRR and Hits@k (gfx950).
//
// Two kernels: k_rank_partial sums 1/rank and the hit counts of MAR_METRIC_TILE ranks per workgroup into
// one partial record, k_rank_final adds the records.  Every sum follows a fixed tree that depends only on
// the number of ranks, so the result is bit-reproducible.  The partial records live either in the
// context's workspace (mar_rank_metrics) or in a file-scope device array (mar_rank_metrics_static, for
// callers that have no workspace and may not allocate one).
#include <mutex>

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

// ------------------------------------------------ entry point that allocates nothing -----
// Partial records of mar_rank_metrics_static.  One copy per GPU, held until the process ends; in host code
// the name is only a handle for hipGetSymbolAddress, the device address is looked up once per device.
static __device__ __align__(256) unsigned char scratch[MAR_METRIC_MAX_PARTS * MAR_METRIC_PART_BYTES];

#define MAR_MAX_DEVICES 64
static std::mutex g_scratch_mu;
static void* g_scratch_ptr[MAR_MAX_DEVICES];

extern "C" int mar_rank_metrics_static(const int32_t* ranks, int64_t n_ranks, const int32_t* ks, int32_t num_k,
                                       double* out, void* hip_stream) {
  if (!out) { mar_set_error("out is NULL"); return MAR_EINVAL; }
  if (n_ranks < 0 || (n_ranks > 0 && !ranks)) { mar_set_error("ranks is NULL or n_ranks negative"); return MAR_EINVAL; }
  if (num_k < 0 || num_k > 8 || (num_k > 0 && !ks)) { mar_set_error("num_k outside 0..8 or ks NULL"); return MAR_ERANGE; }
  for (int j = 0; j < num_k; ++j) if (ks[j] < 1) { mar_set_error("thresholds must be >= 1"); return MAR_EINVAL; }
  if (n_ranks > MAR_RANK_METRICS_STATIC_MAX) {
    mar_set_error("n_ranks %lld exceeds the %lld ranks the built-in scratch array serves; use mar_rank_metrics with a context",
                  (long long)n_ranks, (long long)MAR_RANK_METRICS_STATIC_MAX);
    return MAR_ERANGE;
  }
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) { mar_set_error("hipGetDevice: %s", hipGetErrorString(e)); return MAR_EHIP; }
  if (dev < 0 || dev >= MAR_MAX_DEVICES) { mar_set_error("device index %d outside 0..%d", dev, MAR_MAX_DEVICES - 1); return MAR_ERANGE; }
  void* part = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
      void* p = nullptr;
      e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !p) { mar_set_error("hipGetSymbolAddress(scratch): %s", hipGetErrorString(e)); return MAR_EHIP; }
      g_scratch_ptr[dev] = p;
    }
    part = g_scratch_ptr[dev];
  }
  e = mar_launch_rank_metrics(ranks, n_ranks, ks, num_k, out, part, (hipStream_t)hip_stream);
  if (e != hipSuccess) { mar_set_error("metrics kernels: %s", hipGetErrorString(e)); return MAR_EHIP; }
  return MAR_OK;
}

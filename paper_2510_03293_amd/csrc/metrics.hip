// Imbalance metrics of per-layer assignment counts (Problem statement: imbalance
// factor I_L = max_e N / mean_e N, its weighted aggregate over layers, and the
// GPU-level version under a placement matrix A; Evaluation, Metrics: max violation,
// the relative excess of the most loaded expert over the average, I_L - 1).
// fp64 on the device; one workgroup per layer, then one wavefront for the aggregates.
#include "../../include/laser.h"
#include "laser_internal.h"

namespace laser {

constexpr int kMetricThreads = 256;

__device__ __forceinline__ double wave_max(double v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v = fmax(v, __shfl_xor(v, d, 64));
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  return v;
}

// max and sum over the workgroup; result valid in every thread
__device__ void block_max_sum(double& mx, double& sum, double* sh) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  mx = wave_max(mx);
  sum = wave_sum(sum);
  __syncthreads();  // sh may still be read from the previous call
  if (lane == 0) {
    sh[wave] = mx;
    sh[4 + wave] = sum;
  }
  __syncthreads();
  mx = fmax(fmax(sh[0], sh[1]), fmax(sh[2], sh[3]));
  sum = ((sh[4] + sh[5]) + sh[6]) + sh[7];
}

__global__ __launch_bounds__(kMetricThreads) void imbalance_layers_kernel(
    const int32_t* __restrict__ counts, int E, const float* __restrict__ placement, int G,
    double* __restrict__ I, double* __restrict__ MV, double* __restrict__ Igpu) {
  __shared__ double sh[8];
  extern __shared__ double gload[];  // [G] when a placement is given
  const int l = blockIdx.x;
  const int32_t* n = counts + (size_t)l * E;
  double mx = 0.0, sum = 0.0;
  for (int e = threadIdx.x; e < E; e += kMetricThreads) {
    const double v = (double)n[e];
    mx = fmax(mx, v);
    sum += v;
  }
  block_max_sum(mx, sum, sh);
  const double il = sum > 0.0 ? mx / (sum / (double)E) : 1.0;
  if (threadIdx.x == 0) {
    I[l] = il;
    if (MV) MV[l] = il - 1.0;
  }
  if (placement == nullptr) {
    if (Igpu && threadIdx.x == 0) Igpu[l] = 1.0;
    return;
  }
  // load of GPU g: one wavefront per g, lanes over the experts
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  for (int g = wave; g < G; g += kMetricThreads / 64) {
    double acc = 0.0;
    for (int e = lane; e < E; e += 64) acc += (double)placement[(size_t)g * E + e] * (double)n[e];
    acc = wave_sum(acc);
    if (lane == 0) gload[g] = acc;
  }
  __syncthreads();
  double gmx = 0.0, gsum = 0.0;
  for (int g = threadIdx.x; g < G; g += kMetricThreads) {
    gmx = fmax(gmx, gload[g]);
    gsum += gload[g];
  }
  block_max_sum(gmx, gsum, sh);
  if (Igpu && threadIdx.x == 0) Igpu[l] = gsum > 0.0 ? gmx / (gsum / (double)G) : 1.0;
}

// agg[0] = sum_l w_l I[l], agg[1] = sum_l w_l Igpu[l]; sequential in l (one lane), so
// the result does not depend on the launch shape
__global__ void imbalance_aggregate_kernel(const double* __restrict__ I, const double* __restrict__ Igpu,
                                           const float* __restrict__ weights, int L,
                                           double* __restrict__ agg) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  double a0 = 0.0, a1 = 0.0;
  for (int l = 0; l < L; ++l) {
    const double w = weights ? (double)weights[l] : 1.0 / (double)L;
    a0 += w * I[l];
    a1 += w * (Igpu ? Igpu[l] : 1.0);
  }
  agg[0] = a0;
  agg[1] = a1;
}

// Percentiles of n values: every value's rank by counting (value, then index, so equal
// values get distinct ranks), the sorted list in LDS, then one lane per percentile reads
// its two neighbours.  One workgroup; n <= kMaxPercentileValues.
constexpr int kMaxPercentileValues = 4096;
constexpr int kMaxPercentiles = 16;
struct PercentileArgs {
  double q[kMaxPercentiles];
  int nq;
};

__global__ __launch_bounds__(kMetricThreads) void percentile_kernel(const double* __restrict__ values, int n,
                                                                    const PercentileArgs pa,
                                                                    double* __restrict__ out) {
  __shared__ double raw[kMaxPercentileValues], sorted[kMaxPercentileValues];
  for (int i = threadIdx.x; i < n; i += kMetricThreads) raw[i] = values[i];
  __syncthreads();
  for (int i = threadIdx.x; i < n; i += kMetricThreads) {
    const double v = raw[i];
    int rank = 0;
    for (int j = 0; j < n; ++j) {
      const double u = raw[j];
      rank += (u < v || (u == v && j < i)) ? 1 : 0;
    }
    sorted[rank] = v;
  }
  __syncthreads();
  if ((int)threadIdx.x < pa.nq) {
    const double h = (double)(n - 1) * pa.q[threadIdx.x] / 100.0;
    int lo = (int)h;
    lo = lo > n - 1 ? n - 1 : lo;
    const int hi = lo + 1 < n ? lo + 1 : lo;
    out[threadIdx.x] = sorted[lo] + (h - (double)lo) * (sorted[hi] - sorted[lo]);
  }
}

// Mean and percentiles of n fp32 values (a layer's per-token statistic): one workgroup,
// no scratch memory.  An order statistic is found exactly by radix selection on the
// values' order-preserving 32-bit codes, a byte at a time from the top: histogram of the
// byte among the values that share the prefix found so far, then the bin that holds the
// wanted rank.  The mean is a fixed-shape fp64 sum (per thread in index order, then a
// tree), so it does not depend on anything but n.
constexpr int kSummaryThreads = 1024;

__device__ __forceinline__ unsigned order_code(float v) {  // a < b  <=>  code(a) < code(b)
  const unsigned u = __float_as_uint(v);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float code_value(unsigned c) {
  return __uint_as_float((c & 0x80000000u) ? (c & 0x7FFFFFFFu) : ~c);
}

// rank-th smallest (rank in [0, n)) of the values; called by the whole workgroup
__device__ unsigned select_code(const float* __restrict__ values, int n, int rank, unsigned* hist,
                                unsigned* sh) {
  unsigned prefix = 0, mask = 0;
  int want = rank;
  for (int shift = 24; shift >= 0; shift -= 8) {
    for (int i = threadIdx.x; i < 256; i += kSummaryThreads) hist[i] = 0;
    __syncthreads();
    for (int i = threadIdx.x; i < n; i += kSummaryThreads) {
      const unsigned c = order_code(values[i]);
      if ((c & mask) == prefix) atomicAdd(&hist[(c >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      unsigned cum = 0;
      int bin = 0;
      for (; bin < 255; ++bin) {
        if (cum + hist[bin] > (unsigned)want) break;
        cum += hist[bin];
      }
      sh[0] = (unsigned)bin;
      sh[1] = cum;
    }
    __syncthreads();
    prefix |= sh[0] << shift;
    mask |= 255u << shift;
    want -= (int)sh[1];
    __syncthreads();  // sh and hist are reused
  }
  return prefix;
}

__global__ __launch_bounds__(kSummaryThreads) void summary_f32_kernel(const float* __restrict__ values, int n,
                                                                      const PercentileArgs pa,
                                                                      double* __restrict__ mean,
                                                                      double* __restrict__ out) {
  __shared__ unsigned hist[256], sh[2];
  __shared__ double part[kSummaryThreads];
  if (mean != nullptr) {
    double acc = 0.0;
    for (int i = threadIdx.x; i < n; i += kSummaryThreads) acc += (double)values[i];
    part[threadIdx.x] = acc;
    __syncthreads();
    for (int s = kSummaryThreads / 2; s >= 1; s >>= 1) {
      if ((int)threadIdx.x < s) part[threadIdx.x] += part[threadIdx.x + s];
      __syncthreads();
    }
    if (threadIdx.x == 0) *mean = part[0] / (double)n;
  }
  for (int i = 0; i < pa.nq; ++i) {
    const double h = (double)(n - 1) * pa.q[i] / 100.0;
    int lo = (int)h;
    lo = lo > n - 1 ? n - 1 : lo;
    const int hi = lo + 1 < n ? lo + 1 : lo;
    const double xlo = (double)code_value(select_code(values, n, lo, hist, sh));
    const double xhi = hi == lo ? xlo : (double)code_value(select_code(values, n, hi, hist, sh));
    if (threadIdx.x == 0) out[i] = xlo + (h - (double)lo) * (xhi - xlo);
  }
}

}  // namespace laser

using namespace laser;

extern "C" int laser_summary_f32(const float* values, int32_t n, const double* q, int32_t nq,
                                 double* mean, double* out, void* hip_stream) {
  if (n < 1 || nq < 0 || nq > kMaxPercentiles) return LASER_E_RANGE;
  if (!values || (nq > 0 && (!q || !out))) return LASER_E_NULL;
  if (nq == 0 && !mean) return LASER_OK;
  PercentileArgs pa;
  pa.nq = nq;
  for (int i = 0; i < kMaxPercentiles; ++i) {
    pa.q[i] = i < nq ? q[i] : 0.0;
    if (i < nq && !(q[i] >= 0.0 && q[i] <= 100.0)) return LASER_E_RANGE;
  }
  (void)hipGetLastError();  // (an earlier call's error is not this launch's)
  hipLaunchKernelGGL(summary_f32_kernel, dim3(1), dim3(kSummaryThreads), 0,
                     static_cast<hipStream_t>(hip_stream), values, n, pa, mean, out);
  return hipGetLastError() == hipSuccess ? LASER_OK : LASER_E_LAUNCH;
}

extern "C" int laser_percentiles(const double* values, int32_t n, const double* q, int32_t nq,
                                 double* out, void* hip_stream) {
  if (n < 1 || nq < 0 || nq > kMaxPercentiles) return LASER_E_RANGE;
  if (n > kMaxPercentileValues) return LASER_E_UNSUPPORTED;
  if (nq == 0) return LASER_OK;
  if (!values || !q || !out) return LASER_E_NULL;
  PercentileArgs pa;
  pa.nq = nq;
  for (int i = 0; i < kMaxPercentiles; ++i) {
    pa.q[i] = i < nq ? q[i] : 0.0;
    if (i < nq && !(q[i] >= 0.0 && q[i] <= 100.0)) return LASER_E_RANGE;
  }
  (void)hipGetLastError();  // (an earlier call's error is not this launch's)
  hipLaunchKernelGGL(percentile_kernel, dim3(1), dim3(kMetricThreads), 0, static_cast<hipStream_t>(hip_stream),
                     values, n, pa, out);
  return hipGetLastError() == hipSuccess ? LASER_OK : LASER_E_LAUNCH;
}

extern "C" int laser_imbalance(const int32_t* counts, int32_t L, int32_t E, const float* placement,
                               int32_t G, const float* layer_weights, double* I, double* MV,
                               double* I_gpu, double* agg, void* hip_stream) {
  if (L < 0 || E < 1 || E > (1 << 20)) return LASER_E_RANGE;
  if (placement && (G < 1 || G > 4096)) return LASER_E_RANGE;
  if (!agg || (L > 0 && (!counts || !I))) return LASER_E_NULL;
  if (placement && !I_gpu) return LASER_E_NULL;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (L > 0) {
    const size_t lds = placement ? (size_t)G * sizeof(double) : 0;
    (void)hipGetLastError();  // (an earlier call's error is not this launch's)
    hipLaunchKernelGGL(imbalance_layers_kernel, dim3(L), dim3(kMetricThreads), lds, s, counts, E,
                       placement, G, I, MV, I_gpu);
    if (hipGetLastError() != hipSuccess) return LASER_E_LAUNCH;
  }
  (void)hipGetLastError();  // (an earlier call's error is not this launch's)
  hipLaunchKernelGGL(imbalance_aggregate_kernel, dim3(1), dim3(64), 0, s, I, placement ? I_gpu : nullptr,
                     layer_weights, L, agg);
  return hipGetLastError() == hipSuccess ? LASER_OK : LASER_E_LAUNCH;
}

// libsmfg consumer kernel: GraphSAGE mean aggregation over one MFG block.
#ifndef SMFG_KERNELS_AGGREGATE_H_
#define SMFG_KERNELS_AGGREGATE_H_

#include "device_common.h"

namespace smfg_dev {

// 16 lanes per destination; a lane owns V consecutive columns per round of 16 * V columns and
// accumulates its destination's sampled source rows in float, slot order, two rows in flight.
// Offsets are clamped to [0, max_edges] and source ids outside [0, max_src) read row 0, so the
// arrays of a batch that ended with a status (contents unspecified) cannot cause a stray read.
constexpr int kAggLanes = 16;
constexpr int kAggRows = kThreads / kAggLanes;

template <typename T, int V>
struct alignas(sizeof(T) * V) RowVec {
  T v[V];
};

__device__ __forceinline__ float to_float(_Float16 h) { return static_cast<float>(h); }
__device__ __forceinline__ float to_float(float f) { return f; }

template <typename T, int V>
__global__ void __launch_bounds__(kThreads) k_mean_aggregate(const int32_t* __restrict__ indptr,
                                                             const int32_t* __restrict__ indices,
                                                             int64_t max_edges,
                                                             const int64_t* __restrict__ num_dst, int64_t max_dst,
                                                             const T* __restrict__ x, int64_t max_src, int dim,
                                                             float* __restrict__ out) {
  int64_t n = *num_dst;
  if (n > max_dst) n = max_dst;
  const int64_t i = static_cast<int64_t>(blockIdx.x) * kAggRows + threadIdx.x / kAggLanes;
  if (i >= n) return;
  const int lane = threadIdx.x & (kAggLanes - 1);
  int e0 = indptr[i], e1 = indptr[i + 1];
  if (e0 < 0) e0 = 0;
  if (e1 > max_edges) e1 = static_cast<int>(max_edges);
  if (e1 < e0) e1 = e0;
  const float k = static_cast<float>(e1 - e0);
  typedef RowVec<T, V> Vec;
  const uint32_t nsrc = static_cast<uint32_t>(max_src);
  auto row = [&](int e) -> const T* {
    uint32_t s = static_cast<uint32_t>(indices[e]);
    if (s >= nsrc) s = 0;
    return x + static_cast<int64_t>(s) * dim;
  };
  for (int c = lane * V; c < dim; c += kAggLanes * V) {
    float acc[V];
#pragma unroll
    for (int t = 0; t < V; ++t) acc[t] = 0.f;
    int e = e0;
    for (; e + 1 < e1; e += 2) {
      const Vec a = *reinterpret_cast<const Vec*>(row(e) + c);
      const Vec b = *reinterpret_cast<const Vec*>(row(e + 1) + c);
#pragma unroll
      for (int t = 0; t < V; ++t) acc[t] = (acc[t] + to_float(a.v[t])) + to_float(b.v[t]);
    }
    if (e < e1) {
      const Vec a = *reinterpret_cast<const Vec*>(row(e) + c);
#pragma unroll
      for (int t = 0; t < V; ++t) acc[t] += to_float(a.v[t]);
    }
    float* o = out + i * dim + c;
#pragma unroll
    for (int t = 0; t < V; ++t) o[t] = e1 > e0 ? acc[t] / k : 0.f;
  }
}

}  // namespace smfg_dev

#endif  // SMFG_KERNELS_AGGREGATE_H_

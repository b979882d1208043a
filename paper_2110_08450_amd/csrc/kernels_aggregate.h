// libsmfg consumer kernel: GraphSAGE mean aggregation over one MFG block.
#ifndef SMFG_KERNELS_AGGREGATE_H_
#define SMFG_KERNELS_AGGREGATE_H_

#include "device_common.h"

namespace smfg_dev {

// A group of 16 lanes walks the samples of kAggSpan consecutive destinations, which are one
// contiguous range of the block's indices array; a lane owns V consecutive columns per round of
// 16 * V columns.  kAggDepth source rows are requested before the first is used, whichever
// destination they belong to, so a short destination (fanout 5) does not limit the loads in
// flight.  Each destination's rows are added in float, in slot order, then divided once.
// Offsets are clamped to [0, max_edges] and source ids outside [0, max_src) read row 0, so the
// arrays of a batch that ended with a status (contents unspecified) cannot cause a stray read.
constexpr int kAggLanes = 16;
constexpr int kAggSpan = 2;
constexpr int kAggDepth = 10;
constexpr int kAggGroups = kThreads / kAggLanes;
constexpr int kAggRows = kAggGroups * kAggSpan;  // destinations per block

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
  __shared__ int s_off[kAggGroups][kAggSpan + 1];
  int64_t n = *num_dst;
  if (n > max_dst) n = max_dst;
  const int grp = threadIdx.x / kAggLanes, lane = threadIdx.x & (kAggLanes - 1);
  const int64_t i0 = static_cast<int64_t>(blockIdx.x) * kAggRows + static_cast<int64_t>(grp) * kAggSpan;
  if (static_cast<int64_t>(blockIdx.x) * kAggRows >= n) return;  // whole block past the end
  // offsets of the group's destinations: entry r of a destination past the end repeats the last one
  if (lane <= kAggSpan) {
    int64_t i = i0 + lane;
    if (i > n) i = n;
    int o = i0 <= n ? indptr[i] : 0;
    if (o < 0) o = 0;
    if (o > max_edges) o = static_cast<int>(max_edges);
    s_off[grp][lane] = o;
  }
  __syncthreads();
  if (i0 >= n) return;
  const int rows_here = static_cast<int>(n - i0 < kAggSpan ? n - i0 : kAggSpan);
  const int e_begin = s_off[grp][0];
  typedef RowVec<T, V> Vec;
  const uint32_t nsrc = static_cast<uint32_t>(max_src);
  for (int c = lane * V; c < dim; c += kAggLanes * V) {
    float acc[V];
#pragma unroll
    for (int t = 0; t < V; ++t) acc[t] = 0.f;
    int r = 0;               // destination being summed
    int r_begin = e_begin;   // its first sample
    int r_end = s_off[grp][1];
    if (r_end < r_begin) r_end = r_begin;
    int e_end = r_end;       // end of the group's range, kept non-decreasing
    for (int q = 2; q <= rows_here; ++q) {
      const int o = s_off[grp][q];
      if (o > e_end) e_end = o;
    }
    // closes destination r (mean or zeros) and moves to the next one
    auto close_row = [&]() {
      const float k = static_cast<float>(r_end - r_begin);
      float* o = out + (i0 + r) * dim + c;
#pragma unroll
      for (int t = 0; t < V; ++t) {
        o[t] = r_end > r_begin ? acc[t] / k : 0.f;
        acc[t] = 0.f;
      }
      ++r;
      r_begin = r_end;
      if (r < rows_here) {
        const int o2 = s_off[grp][r + 1];
        r_end = o2 > r_begin ? o2 : r_begin;
      }
    };
    for (int e = e_begin; e < e_end; e += kAggDepth) {
      Vec rows[kAggDepth];
      uint32_t ids[kAggDepth];
#pragma unroll
      for (int u = 0; u < kAggDepth; ++u) {
        const int ee = e + u < e_end ? e + u : e_end - 1;
        ids[u] = static_cast<uint32_t>(indices[ee]);
      }
#pragma unroll
      for (int u = 0; u < kAggDepth; ++u) {
        const uint32_t sidx = ids[u] < nsrc ? ids[u] : 0u;
        rows[u] = *reinterpret_cast<const Vec*>(x + static_cast<int64_t>(sidx) * dim + c);
      }
#pragma unroll
      for (int u = 0; u < kAggDepth; ++u) {
        if (e + u < e_end) {
          while (e + u >= r_end && r < rows_here) close_row();
#pragma unroll
          for (int t = 0; t < V; ++t) acc[t] += to_float(rows[u].v[t]);
        }
      }
    }
    while (r < rows_here) close_row();
  }
}

}  // namespace smfg_dev

#endif  // SMFG_KERNELS_AGGREGATE_H_

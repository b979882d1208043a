// libsmfg consumer kernels: GraphSAGE mean aggregation over one MFG block, alone and fused into
// the layer's linear transform on the matrix cores.
#ifndef SMFG_KERNELS_AGGREGATE_H_
#define SMFG_KERNELS_AGGREGATE_H_

#include "device_common.h"

namespace smfg_dev {

// A group of 16 lanes walks the samples of SPAN consecutive destinations, which are one
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
constexpr int kAggRows = kAggGroups * kAggSpan;  // destinations per block of k_mean_aggregate

template <typename T, int V>
struct alignas(sizeof(T) * V) RowVec {
  T v[V];
};

__device__ __forceinline__ float to_float(_Float16 h) { return static_cast<float>(h); }
__device__ __forceinline__ float to_float(float f) { return f; }

// Offsets of the SPAN + 1 boundaries of a group's destinations i0 .. i0 + SPAN into off[] (LDS);
// a destination past the end n repeats the last boundary.  Call with all lanes of the group, then
// synchronise before walk_group_means reads them.
template <int SPAN>
__device__ __forceinline__ void load_group_offsets(int* off, const int32_t* __restrict__ indptr, int64_t i0,
                                                   int64_t n, int64_t max_edges, int lane) {
  if (lane <= SPAN) {
    int64_t i = i0 + lane;
    if (i > n) i = n;
    int o = i0 <= n ? indptr[i] : 0;
    if (o < 0) o = 0;
    if (o > max_edges) o = static_cast<int>(max_edges);
    off[lane] = o;
  }
}

// Means of the group's rows_here (<= SPAN) destinations; emit(r, c, mean) receives, once per
// destination r and column round, the V means of columns c .. c + V (zeros for an empty row).
template <typename T, int V, typename Emit>
__device__ __forceinline__ void walk_group_means(const int* off, int rows_here,
                                                 const int32_t* __restrict__ indices, const T* __restrict__ x,
                                                 uint32_t nsrc, int dim, int lane, Emit emit) {
  typedef RowVec<T, V> Vec;
  const int e_begin = off[0];
  for (int c = lane * V; c < dim; c += kAggLanes * V) {
    float acc[V];
#pragma unroll
    for (int t = 0; t < V; ++t) acc[t] = 0.f;
    int r = 0;               // destination being summed
    int r_begin = e_begin;   // its first sample
    int r_end = off[1];
    if (r_end < r_begin) r_end = r_begin;
    int e_end = r_end;       // end of the group's range, kept non-decreasing
    for (int q = 2; q <= rows_here; ++q) {
      const int o = off[q];
      if (o > e_end) e_end = o;
    }
    // closes destination r (mean or zeros) and moves to the next one
    auto close_row = [&]() {
      const float k = static_cast<float>(r_end - r_begin);
      float mean[V];
#pragma unroll
      for (int t = 0; t < V; ++t) {
        mean[t] = r_end > r_begin ? acc[t] / k : 0.f;
        acc[t] = 0.f;
      }
      emit(r, c, mean);
      ++r;
      r_begin = r_end;
      if (r < rows_here) {
        const int o2 = off[r + 1];
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
  load_group_offsets<kAggSpan>(s_off[grp], indptr, i0, n, max_edges, lane);
  __syncthreads();
  if (i0 >= n) return;
  const int rows_here = static_cast<int>(n - i0 < kAggSpan ? n - i0 : kAggSpan);
  walk_group_means<T, V>(s_off[grp], rows_here, indices, x, static_cast<uint32_t>(max_src), dim, lane,
                         [&](int r, int c, const float* mean) {
                           float* o = out + (i0 + r) * dim + c;
#pragma unroll
                           for (int t = 0; t < V; ++t) o[t] = mean[t];
                         });
}

// ---- one GraphSAGE layer: out = act([x_dst | mean] W^T + b) -------------------------------------
//
// A block owns ROWS consecutive destinations.  It first builds the layer input of its rows
// in LDS as halfs: columns [0, dim) the destination's own row (destination i is source i, so
// these are contiguous rows of x), columns [dim, 2 dim) the neighbour means from the walk above,
// rounded to half.  Then each wave multiplies the tile by 32-column slices of W^T with
// v_mfma_f32_32x32x16_f16 (one 32 x 32 accumulator per 32 rows), adds the bias, applies the ReLU
// and stores.  W comes pre-arranged in the lanes' operand order (k_sage_pack_weights).
// ROWS is 64 for dim <= 128 and 32 above, which keeps the tile within 64 KB of LDS.
constexpr int kLayerPad = 8;  // halfs of padding per LDS row
constexpr int kLayerMaxDim = 256;
constexpr int kLayerAhead = 8;  // vectors of W requested ahead of their use

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));

// Weights in the order the layer kernel's lanes consume them: for column slice sl (32 output
// columns), vector q (16 reduction indices) and lane (hi, col): the 8 halfs
// w[32 sl + col][16 q + 8 hi .. + 8), zeros for columns past out_dim.
__global__ void __launch_bounds__(kThreads) k_sage_pack_weights(const _Float16* __restrict__ w, int K, int out_dim,
                                                                half8_t* __restrict__ packed, int64_t vectors) {
  const int nq = K / 16;
  for (int64_t v = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; v < vectors;
       v += static_cast<int64_t>(gridDim.x) * kThreads) {
    const int l = static_cast<int>(v & 63);
    const int64_t sq = v >> 6;
    const int q = static_cast<int>(sq % nq);
    const int sl = static_cast<int>(sq / nq);
    const int row = sl * 32 + (l & 31);
    half8_t o = {0, 0, 0, 0, 0, 0, 0, 0};
    if (row < out_dim) o = *reinterpret_cast<const half8_t*>(w + static_cast<int64_t>(row) * K + q * 16 + (l >> 5) * 8);
    packed[v] = o;
  }
}

template <typename OutT, int ROWS>
__global__ void __launch_bounds__(kThreads, 4) k_sage_layer(const int32_t* __restrict__ indptr,
                                                         const int32_t* __restrict__ indices, int64_t max_edges,
                                                         const int64_t* __restrict__ num_dst, int64_t max_dst,
                                                         const _Float16* __restrict__ x, int64_t max_src, int dim,
                                                         const _Float16* __restrict__ w,
                                                         const float* __restrict__ bias, int out_dim, int relu,
                                                         OutT* __restrict__ out) {
  static_assert(ROWS == 32 || ROWS == 64, "one or two 32-row accumulators");
  constexpr int kLayerRows = ROWS;
  constexpr int kLayerSpan = ROWS / kAggGroups;  // destinations per lane group
  extern __shared__ __align__(16) unsigned char lds_raw[];
  __shared__ int s_off[kAggGroups][kLayerSpan + 1];
  _Float16* a_lds = reinterpret_cast<_Float16*>(lds_raw);  // [ROWS][2 dim + kLayerPad]
  int64_t n = *num_dst;
  if (n > max_dst) n = max_dst;
  if (n > max_src) n = max_src;  // a destination's own row is row i of x
  const int64_t tile0 = static_cast<int64_t>(blockIdx.x) * kLayerRows;
  if (tile0 >= n) return;
  const int rows_tile = static_cast<int>(n - tile0 < kLayerRows ? n - tile0 : kLayerRows);
  const int K = 2 * dim;
  const int lda = K + kLayerPad;
  const int grp = threadIdx.x / kAggLanes, lane = threadIdx.x & (kAggLanes - 1);
  const int64_t i0 = tile0 + static_cast<int64_t>(grp) * kLayerSpan;
  load_group_offsets<kLayerSpan>(s_off[grp], indptr, i0, n, max_edges, lane);

  // own rows -> columns [0, dim); rows past the end of the block become zeros (both halves)
  {
    const int vec_per_row = dim / 8;
    const half8_t zero = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int idx = threadIdx.x; idx < kLayerRows * vec_per_row; idx += kThreads) {
      const int r = idx / vec_per_row, cv = idx - r * vec_per_row;
      half8_t v = zero;
      if (r < rows_tile) v = *reinterpret_cast<const half8_t*>(x + (tile0 + r) * dim + cv * 8);
      *reinterpret_cast<half8_t*>(a_lds + r * lda + cv * 8) = v;
      if (r >= rows_tile) *reinterpret_cast<half8_t*>(a_lds + r * lda + dim + cv * 8) = zero;
    }
  }
  __syncthreads();
  if (i0 < n) {
    const int rows_here = static_cast<int>(n - i0 < kLayerSpan ? n - i0 : kLayerSpan);
    _Float16* a_grp = a_lds + (grp * kLayerSpan) * lda + dim;
    walk_group_means<_Float16, 8>(s_off[grp], rows_here, indices, x, static_cast<uint32_t>(max_src), dim, lane,
                                  [&](int r, int c, const float* mean) {
                                    half8_t h;
#pragma unroll
                                    for (int t = 0; t < 8; ++t) h[t] = static_cast<_Float16>(mean[t]);
                                    *reinterpret_cast<half8_t*>(a_grp + r * lda + c) = h;
                                  });
  }
  __syncthreads();

  // tile [ROWS x K] times W^T: wave wv takes the column slices wv, wv + 4, ...  The packed
  // weights hold, for every slice and every 16 reduction indices, the 64 lanes' operands side by
  // side, so one load instruction of the wave reads 1 KB of consecutive memory (W stays in the L2);
  // kLayerAhead such vectors are always on their way.
  const int wv = threadIdx.x >> 6, l = threadIdx.x & 63;
  const int col = l & 31, hi = l >> 5;
  const int nq = K / 16;
  for (int n0 = wv * 32; n0 < out_dim; n0 += 4 * 32) {
    const half8_t* wp = reinterpret_cast<const half8_t*>(w) + static_cast<int64_t>(n0 / 32) * nq * 64 + l;
    const _Float16* ap0 = a_lds + col * lda + hi * 8;
    const _Float16* ap1 = ap0 + 32 * lda;
    float16_t acc0, acc1;
#pragma unroll
    for (int t = 0; t < 16; ++t) {
      acc0[t] = 0.f;
      acc1[t] = 0.f;
    }
    half8_t bq[kLayerAhead];
#pragma unroll
    for (int u = 0; u < kLayerAhead; ++u) bq[u] = wp[(u < nq ? u : 0) * 64];
    // one v_mfma_f32_32x32x16_f16 per vector: lane half hi supplies reduction indices 16 q + 8 hi .. + 8
    // of both operands (any assignment works as long as it is the same on both sides)
    // The body is free of branches (a vector past the end multiplies zeros), so the LDS reads of
    // the unrolled steps can be issued ahead of the MFMAs that use them.
    for (int qb = 0; qb < nq; qb += kLayerAhead) {
#pragma unroll
      for (int u = 0; u < kLayerAhead; ++u) {
        const int q = qb + u;
        const half8_t zero = {0, 0, 0, 0, 0, 0, 0, 0};
        const half8_t b = q < nq ? bq[u] : zero;
        const int qn = q + kLayerAhead;
        bq[u] = wp[(qn < nq ? qn : 0) * 64];
        const int k0 = (q < nq ? q : 0) * 16;
        const half8_t a0 = *reinterpret_cast<const half8_t*>(ap0 + k0);
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, b, acc0, 0, 0, 0);
        if constexpr (ROWS == 64) {
          const half8_t a1 = *reinterpret_cast<const half8_t*>(ap1 + k0);
          acc1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, b, acc1, 0, 0, 0);
        }
      }
    }
    // element t of a lane's accumulator: row 8 (t / 4) + 4 hi + t % 4, column col.  The row term
    // that depends on t is the same for all lanes, so a store is one lane pointer plus a uniform
    // offset.
    if (n0 + col < out_dim) {
      const float bj = bias ? bias[n0 + col] : 0.f;
      OutT* o0 = out + (tile0 + 4 * hi) * out_dim + n0 + col;
      const int rows_left = rows_tile - 4 * hi;  // rows of the tile at or after the lane's first
      OutT r0[16], r1[16];
#pragma unroll
      for (int t = 0; t < 16; ++t) {
        float v0 = acc0[t] + bj, v1 = acc1[t] + bj;
        if (relu) {
          v0 = v0 > 0.f ? v0 : 0.f;
          v1 = v1 > 0.f ? v1 : 0.f;
        }
        r0[t] = static_cast<OutT>(v0);
        r1[t] = static_cast<OutT>(v1);
      }
      if (rows_tile == ROWS) {  // full tile: all stores in one go, nothing to test
#pragma unroll
        for (int t = 0; t < 16; ++t) {
          const int rt = 8 * (t / 4) + (t % 4);
          o0[static_cast<int64_t>(rt) * out_dim] = r0[t];
          if (ROWS == 64) o0[static_cast<int64_t>(rt + 32) * out_dim] = r1[t];
        }
      } else {
#pragma unroll
        for (int t = 0; t < 16; ++t) {
          const int rt = 8 * (t / 4) + (t % 4);
          if (rt < rows_left) o0[static_cast<int64_t>(rt) * out_dim] = r0[t];
          if (ROWS == 64 && rt + 32 < rows_left) o0[static_cast<int64_t>(rt + 32) * out_dim] = r1[t];
        }
      }
    }
  }
}

}  // namespace smfg_dev

#endif  // SMFG_KERNELS_AGGREGATE_H_

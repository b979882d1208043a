// libsmfg feature gather xs = x[ids] (Listing 1).
#ifndef SMFG_KERNELS_GATHER_H_
#define SMFG_KERNELS_GATHER_H_

#include "device_common.h"

namespace smfg_dev {

// Rows are moved as vectors of sizeof(V) bytes.  A block copies ROWS consecutive output rows (32,
// or 64 when a row has fewer than 256 bytes: the 200-byte rows of the products-shaped workload
// copy 6 % faster that way, 256- and 512-byte rows 2-5 % slower) and exits: many short-lived blocks
// reach a higher copy rate on this chip than a persistent grid-stride loop.  Inside a block the output chunk is addressed as one flat vector array, so
// stores are fully coalesced and the lanes that share a row read one contiguous span of it.
// A row id outside [0, num_nodes) is read as row 0, so that no id can cause a read outside x.
constexpr int gather_rows_per_block(int64_t row_bytes) { return row_bytes < 256 ? 64 : 32; }

// The copy's loads and stores are written out as instructions, for two reasons.  Cache policy:
// rows are read once and written once, and the compiler's non-temporal builtins set `nt` alone.
// `nt` keeps the rows from displacing what the sampling kernels beside the copy have in the
// caches (without it the whole path loses 8-13 %); stores with `sc0` on top measured +2.5 to +3 %
// on the papers100M-, arxiv- and products-shaped workloads, loads at system scope (`sc0 sc1`)
// another +1.4 % on the first (means of six interleaved runs).  Issue order: the two loads of a
// round leave together and its two stores leave back to back after one wait; the compiler put a
// wait between the stores, which cost the 200-byte rows of the products-shaped workload 3 %.
// Which level a line is kept in does not change what is copied: the table is read-only, and the
// kernel's end makes every store visible to what follows.  The wait is part of the load
// statements because the compiler does not track loads it did not emit; for the same reason a
// store is followed by two idle cycles: the hardware reads a wide store's data registers a
// moment after issue and wants no vector write to them in between, a gap the compiler only
// inserts after stores of its own.
template <typename V>
__device__ __forceinline__ void store_streaming(V v, V* p) {
  if constexpr (sizeof(V) == 16) {
    asm volatile("global_store_dwordx4 %0, %1, off sc0 nt\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
  } else if constexpr (sizeof(V) == 8) {
    asm volatile("global_store_dwordx2 %0, %1, off sc0 nt\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
  } else if constexpr (sizeof(V) == 4) {
    asm volatile("global_store_dword %0, %1, off sc0 nt\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
  } else {
    __builtin_nontemporal_store(v, p);
  }
}
template <typename V>
__device__ __forceinline__ V load_streaming(const V* p) {
  V v;
  if constexpr (sizeof(V) == 16) {
    asm volatile("global_load_dwordx4 %0, %1, off sc0 sc1 nt\n\ts_waitcnt vmcnt(0)" : "=&v"(v) : "v"(p) : "memory");
  } else if constexpr (sizeof(V) == 8) {
    asm volatile("global_load_dwordx2 %0, %1, off sc0 sc1 nt\n\ts_waitcnt vmcnt(0)" : "=&v"(v) : "v"(p) : "memory");
  } else if constexpr (sizeof(V) == 4) {
    asm volatile("global_load_dword %0, %1, off sc0 sc1 nt\n\ts_waitcnt vmcnt(0)" : "=&v"(v) : "v"(p) : "memory");
  } else {
    v = __builtin_nontemporal_load(p);
  }
  return v;
}
template <typename V>
__device__ __forceinline__ void load_pair_streaming(const V* p0, const V* p1, V& v0, V& v1) {
  if constexpr (sizeof(V) == 16) {
    asm volatile(
        "global_load_dwordx4 %0, %2, off sc0 sc1 nt\n\t"
        "global_load_dwordx4 %1, %3, off sc0 sc1 nt\n\t"
        "s_waitcnt vmcnt(0)"
        : "=&v"(v0), "=&v"(v1)
        : "v"(p0), "v"(p1)
        : "memory");
  } else if constexpr (sizeof(V) == 8) {
    asm volatile(
        "global_load_dwordx2 %0, %2, off sc0 sc1 nt\n\t"
        "global_load_dwordx2 %1, %3, off sc0 sc1 nt\n\t"
        "s_waitcnt vmcnt(0)"
        : "=&v"(v0), "=&v"(v1)
        : "v"(p0), "v"(p1)
        : "memory");
  } else if constexpr (sizeof(V) == 4) {
    asm volatile(
        "global_load_dword %0, %2, off sc0 sc1 nt\n\t"
        "global_load_dword %1, %3, off sc0 sc1 nt\n\t"
        "s_waitcnt vmcnt(0)"
        : "=&v"(v0), "=&v"(v1)
        : "v"(p0), "v"(p1)
        : "memory");
  } else {
    v0 = __builtin_nontemporal_load(p0);
    v1 = __builtin_nontemporal_load(p1);
  }
}

template <typename V, int ROWS>
__device__ __forceinline__ void gather_rows(const uint8_t* __restrict__ feat, int64_t row_stride,
                                            uint32_t vec_per_row, int64_t num_nodes,
                                            const int32_t* __restrict__ ids, int64_t n,
                                            uint8_t* __restrict__ out) {
  static_assert(ROWS <= kThreads, "a thread per row fetches its id");
  __shared__ int64_t row_byte[ROWS];  // byte offset of each source row
  const int64_t r0 = static_cast<int64_t>(blockIdx.x) * ROWS;
  if (r0 >= n) return;
  const uint32_t rows = static_cast<uint32_t>(n - r0 < ROWS ? n - r0 : ROWS);
  const uint32_t cnt = rows * vec_per_row;
  if (threadIdx.x < ROWS) {
    int64_t id = threadIdx.x < rows ? ids[r0 + threadIdx.x] : 0;
    if (id < 0 || id >= num_nodes) id = 0;
    row_byte[threadIdx.x] = id * row_stride;
  }
  __syncthreads();
  V* __restrict__ o = reinterpret_cast<V*>(out) + static_cast<uint64_t>(r0) * vec_per_row;
  // (row, column) of a vector of the chunk by multiplication: ceil(2^32 / vec_per_row) gives the
  // exact quotient as long as index * vec_per_row < 2^32, which holds for every index of a chunk
  // when a row has at most 8192 vectors; longer rows divide
  const bool by_mul = vec_per_row <= 8192u;
  const uint64_t inv = 0xFFFFFFFFull / vec_per_row + 1ull;
  const auto source = [&](uint32_t idx) {
    const uint32_t jrow = by_mul ? static_cast<uint32_t>((idx * inv) >> 32) : idx / vec_per_row;
    return reinterpret_cast<const V*>(feat + row_byte[jrow]) + (idx - jrow * vec_per_row);
  };
  // a round: two independent row reads per thread, then the two stores; the last round of a
  // thread may hold one vector only
  for (uint32_t base = threadIdx.x; base < cnt; base += kThreads * 2) {
    if (base + kThreads < cnt) {
      V v0, v1;
      load_pair_streaming(source(base), source(base + kThreads), v0, v1);
      store_streaming(v0, o + base);
      store_streaming(v1, o + base + kThreads);
    } else {
      store_streaming(load_streaming(source(base)), o + base);
    }
  }
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <typename V, int ROWS>
__global__ void __launch_bounds__(kThreads) k_gather(const Launch P) {
  const BatchCtx& B = P.b[blockIdx.y];
  if (B.features == nullptr || status_of(B, P.L) != 0) return;
  int64_t n = B.counts[P.L];
  if (n > B.node_capacity) n = B.node_capacity;
  gather_rows<V, ROWS>(P.feat, P.row_stride, static_cast<uint32_t>(P.row_bytes / sizeof(V)), P.num_nodes,
                 B.node_ids, n, B.features);
}

template <typename V, int ROWS>
__global__ void __launch_bounds__(kThreads) k_gather_plain(const uint8_t* feat, int64_t row_bytes,
                                                           int64_t row_stride, int64_t num_nodes,
                                                           const int32_t* ids, const int64_t* num_rows,
                                                           int64_t max_rows, uint8_t* out) {
  int64_t n = *num_rows;
  if (n > max_rows) n = max_rows;
  if (n < 0) n = 0;
  gather_rows<V, ROWS>(feat, row_stride, static_cast<uint32_t>(row_bytes / sizeof(V)), num_nodes, ids, n, out);
}

}  // namespace smfg_dev

#endif  // SMFG_KERNELS_GATHER_H_

// libsmfg input check: one streaming pass over the CSR arrays of a graph handle.
#ifndef SMFG_KERNELS_VALIDATE_H_
#define SMFG_KERNELS_VALIDATE_H_

#include "device_common.h"

namespace smfg_dev {

// flags |= SMFG_BAD_INDPTR_* for every violated condition on indptr[0 .. n] (n + 1 entries).
__global__ void __launch_bounds__(kThreads) k_validate_indptr(const int64_t* __restrict__ indptr, int64_t n,
                                                              int64_t m, uint32_t* __restrict__ flags) {
  uint32_t bad = 0;
  const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
  const int64_t t = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (t == 0) {
    if (indptr[0] != 0) bad |= SMFG_BAD_INDPTR_START;
    if (indptr[n] != m) bad |= SMFG_BAD_INDPTR_END;
  }
  for (int64_t i = t; i < n; i += stride) {
    const int64_t a = indptr[i], b = indptr[i + 1];
    if (b < a || b - a >= (1ll << 31)) bad |= SMFG_BAD_INDPTR_ORDER;
  }
  if (bad) atomicOr(flags, bad);
}

// flags |= SMFG_BAD_INDEX_RANGE if any indices[e], e < m, lies outside [0, n).
__global__ void __launch_bounds__(kThreads) k_validate_indices(const int32_t* __restrict__ indices, int64_t m,
                                                               int64_t n, uint32_t* __restrict__ flags) {
  bool bad = false;
  const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
  for (int64_t e = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; e < m; e += stride) {
    const int32_t v = __builtin_nontemporal_load(indices + e);
    bad |= v < 0 || static_cast<int64_t>(v) >= n;
  }
  if (bad) atomicOr(flags, static_cast<uint32_t>(SMFG_BAD_INDEX_RANGE));
}

}  // namespace smfg_dev

#endif  // SMFG_KERNELS_VALIDATE_H_

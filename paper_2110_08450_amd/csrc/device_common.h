// libsmfg device code shared by all kernels: launch parameters, status word, Philox4x32-10,
// the dedup table insert and the block scan.
#ifndef SMFG_DEVICE_COMMON_H_
#define SMFG_DEVICE_COMMON_H_

#include <hip/hip_runtime.h>

#include <cstdint>

#include "smfg.h"

namespace smfg_dev {

constexpr int kThreads = 256;
constexpr int kTileRows = 256;              // destinations per scan tile
constexpr uint32_t kPend = 0x80000000u;     // table value / entry tag: a position of this hop
constexpr uint32_t kSlot = 0x40000000u;     // entry tag: index of the sample's table slot
constexpr uint32_t kTagMask = 0xC0000000u;
constexpr uint64_t kEmpty = ~0ull;

struct BatchCtx {
  const int32_t* seeds;
  int64_t* counts;       // [2L+2]
  uint64_t* table;
  int32_t* node_ids;
  uint32_t* ent;         // per (destination, s): final local id | kSlot+slot (owner) | kPend+position
  uint32_t* lostto;      // per (destination, s): 0, or kPend+position of the sample that displaced it
  int64_t lostto_entries;
  int32_t* gsrc;         // per (destination, s): global id of the sampled neighbour
  int32_t* rowk;         // samples per destination
  uint2* rowmn;          // per destination: .x first-appearance bits, .y new nodes of the tile before its first new node
  int32_t* rowoff;       // samples of the tile before this destination
  uint64_t* tile_sums;   // per tile: (edges << 32 | new nodes), later their exclusive scan
  int64_t* rowstart;     // wide path: first CSR position of the destination's row
  int32_t* rowdeg;       // wide path: degree of the destination
  uint32_t* rank;        // wide path, table strategy: new nodes of the sample's tile before this sample
  uint4* grp;            // wide path, partition strategy: per 64 samples (.x, .y) first-appearance bits,
                         // .z new nodes of the tile before the group
  uint64_t* stile_sums;  // wide path: per sample tile, new nodes, later their exclusive scan
  int32_t* blk_indptr;   // hop h
  int32_t* blk_indices;  // hop h
  uint8_t* features;
  uint8_t* labels;       // [num_seeds x label bytes] or null
  int64_t edge_capacity; // hop h
  int32_t node_capacity;
  int32_t num_seeds;
  uint32_t key0, key1;
  uint32_t table_shift;  // slot = hash >> shift
  uint32_t table_mask;
  // partition path (no table): records of a hop grouped by hash bucket
  uint64_t* rec;         // (node << 32 | value) per known node and per sample, bucket by bucket
  uint32_t* hist;        // [blocks x buckets] records per (row block, bucket), later their offsets
  uint32_t* bstart;      // [buckets + 1] first record of each bucket; [buckets + 1 .. 2 buckets + 1) bucket sizes
  uint64_t* rec2;        // the records once more, each bucket split into sub-buckets (hops with lg2 > 0)
  uint32_t* bstart2;     // [buckets * sub-buckets + 1] first record of each sub-bucket in rec2
};

struct Launch {
  const int64_t* indptr;
  const int32_t* indices;
  const uint8_t* feat;
  const uint8_t* labels;  // y, label_bytes per node, or null
  int64_t row_bytes;
  int64_t row_stride;
  int64_t num_nodes;
  int32_t label_bytes;
  int32_t L;       // hops of this call (counts layout)
  int32_t h;       // current hop
  int32_t d;       // its fanout
  int32_t G;       // batches
  int32_t lgB;     // partition path: log2 of the hash buckets of this hop
  int32_t lg2;     // partition path: log2 of the sub-buckets each bucket is split into (0: not split)
  int32_t block_rows;  // partition path: destinations per row block of this hop
  int32_t flat;    // partition path over exact offsets: lgB / lg2 are upper bounds, the hop's own
                   // shape follows from its record count on the device (hop_shape)
  BatchCtx b[SMFG_MAX_BATCHES];
};
static_assert(sizeof(Launch) <= 4096, "kernel arguments are limited to 4 KB");

// Grids are one-dimensional with the batch as the fastest-varying part of the block index:
// consecutive workgroups go to consecutive XCDs, so with 8 batches per call the blocks of one
// batch share one XCD and its L2 (a locality preference only, nothing depends on it).
__device__ __forceinline__ int batch_of_block(const Launch& P) { return static_cast<int>(blockIdx.x % static_cast<unsigned>(P.G)); }
__device__ __forceinline__ int block_in_batch(const Launch& P) { return static_cast<int>(blockIdx.x / static_cast<unsigned>(P.G)); }
__device__ __forceinline__ int blocks_per_batch(const Launch& P) { return static_cast<int>(gridDim.x / static_cast<unsigned>(P.G)); }

__device__ __forceinline__ int64_t status_of(const BatchCtx& B, int L) {
  return __hip_atomic_load(&B.counts[2 * L + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The same answer for every thread of the block (other blocks may set the status while this one
// starts, and kernels that synchronise must leave as whole blocks).
__device__ __forceinline__ bool block_has_status(const BatchCtx& B, int L) {
  __shared__ int st_lds;
  if (threadIdx.x == 0) st_lds = status_of(B, L) != 0 ? 1 : 0;
  __syncthreads();
  const bool r = st_lds != 0;
  __syncthreads();
  return r;
}

__device__ __forceinline__ void set_status(const BatchCtx& B, int L, int64_t code) {
  unsigned long long* p = reinterpret_cast<unsigned long long*>(&B.counts[2 * L + 1]);
  atomicCAS(p, 0ull, static_cast<unsigned long long>(code));
}

// ---- Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11) -------------------------------------
// Returns word `w` (0..3) of the block with counter (c0, c1, c2, 0) and key (k0, k1).
__device__ __forceinline__ uint32_t philox_word(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t k0,
                                                uint32_t k1, uint32_t w) {
  constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
  uint32_t c3 = 0u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
    const uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
    const uint32_t n0 = hi1 ^ c1 ^ k0;
    const uint32_t n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return w == 0 ? c0 : (w == 1 ? c1 : (w == 2 ? c2 : c3));
}

// ---- dedup table ----------------------------------------------------------------------------
__device__ __forceinline__ uint32_t hash_slot(uint32_t key, uint32_t shift) {
  return (key * 0x9E3779B1u) >> shift;
}

// Inserts key with value `val`, or lowers the stored value to `val`.  Returns the value that
// stood in the table just before this sample's own update took effect (0xFFFFFFFF when the key
// was new) and the slot in `slot`.  The first access of a probe is the compare-and-swap itself:
// on the common paths (key new, or key present with a smaller value) it is the only access.
// If the returned value is larger than `val`, this call is the one and only update that
// replaced exactly that value.
__device__ __forceinline__ uint32_t table_insert_min(const BatchCtx& B, uint32_t key, uint32_t val,
                                                     uint32_t& slot, bool& full) {
  unsigned long long* T = reinterpret_cast<unsigned long long*>(B.table);
  const unsigned long long mine = (static_cast<unsigned long long>(key) << 32) | val;
  uint32_t s = hash_slot(key, B.table_shift);
  full = false;
  // A probe run that has seen every slot means more distinct nodes than slots, i.e. more than
  // twice the node capacity: only then is the table reported as full.  (Node ids whose hashes
  // share their leading bits make long runs, which cost time but never a wrong answer.)
  for (uint64_t probes = 0; probes <= B.table_mask; ++probes) {
    unsigned long long old = atomicCAS(&T[s], kEmpty, mine);
    if (old == kEmpty) {
      slot = s;
      return 0xFFFFFFFFu;
    }
    if (static_cast<uint32_t>(old >> 32) == key) {
      slot = s;
      if (static_cast<uint32_t>(old) > val) old = atomicMin(&T[s], mine);
      return static_cast<uint32_t>(old);
    }
    s = (s + 1) & B.table_mask;
  }
  full = true;
  slot = 0;
  return 0u;
}

// Small fill kernel (used instead of a memset node where a caller may capture the stream).
__global__ void __launch_bounds__(kThreads) k_fill_u32(uint32_t* p, int64_t n, uint32_t value) {
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; i < n;
       i += static_cast<int64_t>(gridDim.x) * kThreads)
    p[i] = value;
}

// ---- block scan ------------------------------------------------------------------------------
// Exclusive scan over a block of kThreads values; returns the exclusive prefix, total in `total`.
__device__ __forceinline__ unsigned long long block_exscan(unsigned long long x, unsigned long long* lds,
                                                            unsigned long long& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  unsigned long long inc = x;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const unsigned long long y = __shfl_up(inc, o, 64);
    if (lane >= o) inc += y;
  }
  __syncthreads();
  if (lane == 63) lds[wave] = inc;
  __syncthreads();
  unsigned long long base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kThreads / 64; ++w) {
    const unsigned long long v = lds[w];
    if (w < wave) base += v;
    tot += v;
  }
  total = tot;
  return base + inc - x;
}

}  // namespace smfg_dev

#endif  // SMFG_DEVICE_COMMON_H_

// libsmfg: sampled mini-batch preparation on gfx950 (MI355X).  Implements include/smfg.h.
//
// One hop h of one batch is four launches (all batches of a call share each launch through
// blockIdx.y):
//   sample_insert  per destination: degree, Floyd/Philox row positions, neighbour ids, and an
//                  insert of each neighbour into the batch's dedup table carrying the sample's
//                  scan position (section 4.1 "fusing sampling and MFG construction": the edge
//                  is recorded the moment the neighbour is picked).  The insert's own return
//                  values settle everything: a known node yields its final local id; a sample
//                  that claims a slot or lowers its value is the node's owner for now; a sample
//                  that finds a smaller position keeps that position as a pointer; a sample that
//                  lowers the value tells the one it displaced (`lostto`), exactly once;
//   flag_rows      streaming, one block per tile of 256 destinations: owner samples that were
//                  not displaced are the first appearances; one bit mask per destination, the
//                  in-tile exclusive scan of (samples, new nodes) per destination, per-tile
//                  totals; displaced owners turn into pointers and `lostto` is cleared again;
//   scan_tiles     exclusive scan of the tile totals, E_h and n_{h+1};
//   assemble       streaming, one block per tile: block indptr; final local id of every sample
//                  -> block indices; first appearances also write node_ids and (unless this is
//                  the last hop) the final id into the table (the auto-increment of procedure
//                  OneHopMFG, made order-independent: the id is the rank of the first appearance
//                  in (destination, slot) order); the other samples of a new node follow their
//                  pointer (positions only decrease along it) to the first appearance.
// Then one gather launch copies the feature rows of the final node list (Listing 1, xs = x[ids]).
//
// The dedup table is open addressing over 64-bit slots (key << 32 | value).  A known node holds
// its local id; a node met in the current hop holds kPend | position until it is published.
// Claims use compare-and-swap on the whole slot, later samples of the same node use a 64-bit
// atomic minimum, so the surviving value is the smallest position whatever the schedule.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <new>

#include "smfg.h"

namespace {

constexpr int kThreads = 256;
constexpr int kTileRows = 256;              // destinations per scan tile
constexpr uint32_t kPend = 0x80000000u;     // table value / entry tag: a position of this hop
constexpr uint32_t kSlot = 0x40000000u;     // entry tag: index of the sample's table slot
constexpr uint32_t kTagMask = 0xC0000000u;
constexpr uint64_t kEmpty = ~0ull;
constexpr uint32_t kMaxProbes = 4096;      // longest probe run before the table counts as full

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
  uint32_t* rowmask;     // first-appearance bits per destination
  int32_t* newrank;      // new nodes of the tile before this destination's first new node
  int32_t* rowoff;       // samples of the tile before this destination
  uint64_t* tile_sums;   // per tile: (edges << 32 | new nodes), later their exclusive scan
  int64_t* rowstart;     // wide path: first CSR position of the destination's row
  int32_t* rowdeg;       // wide path: degree of the destination
  uint32_t* rank;        // wide path: new nodes of the sample's tile before this sample
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
  BatchCtx b[SMFG_MAX_BATCHES];
};

__device__ __forceinline__ int64_t status_of(const BatchCtx& B, int L) {
  return __hip_atomic_load(&B.counts[2 * L + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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
  // The table has at least two slots per node of capacity, so a probe run this long only occurs
  // when far more distinct nodes arrive than the capacity allows: report the table as full.
  const uint32_t max_probes = B.table_mask < kMaxProbes ? B.table_mask + 1u : kMaxProbes;
  for (uint32_t probes = 0; probes < max_probes; ++probes) {
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

// ---- kernels --------------------------------------------------------------------------------

__global__ void __launch_bounds__(kThreads) k_clear(const Launch P) {
  const BatchCtx& B = P.b[blockIdx.y];
  const size_t n = static_cast<size_t>(B.table_mask) + 1;
  for (size_t i = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x; i < n;
       i += static_cast<size_t>(gridDim.x) * kThreads)
    B.table[i] = kEmpty;
  if (blockIdx.x == 0) {
    const int m = 2 * P.L + 2;
    for (int q = threadIdx.x; q < m; q += kThreads) B.counts[q] = (q == 0) ? B.num_seeds : 0;
  }
}

// M starts with the destination nodes of hop 0 in the order given (procedure OneHopMFG).
__global__ void __launch_bounds__(kThreads) k_insert_seeds(const Launch P) {
  const BatchCtx& B = P.b[blockIdx.y];
  for (int i = blockIdx.x * kThreads + threadIdx.x; i < B.num_seeds; i += gridDim.x * kThreads) {
    const int32_t v = B.seeds[i];
    if (v < 0 || static_cast<int64_t>(v) >= P.num_nodes) {
      set_status(B, P.L, SMFG_ST_SEED_OUT_OF_RANGE);
      continue;
    }
    uint32_t slot;
    bool full;
    const uint32_t prev = table_insert_min(B, static_cast<uint32_t>(v), static_cast<uint32_t>(i), slot, full);
    if (full) set_status(B, P.L, SMFG_ST_TABLE_FULL);
    else if (prev != 0xFFFFFFFFu) set_status(B, P.L, SMFG_ST_DUPLICATE_SEED);
    B.node_ids[i] = v;
    if (B.labels) {  // ys = y[ids[:batch_size]] (Listing 1): the seeds are the first ids
      const uint8_t* src = P.labels + static_cast<int64_t>(v) * P.label_bytes;
      uint8_t* dst = B.labels + static_cast<int64_t>(i) * P.label_bytes;
      switch (P.label_bytes) {
        case 8: *reinterpret_cast<uint64_t*>(dst) = *reinterpret_cast<const uint64_t*>(src); break;
        case 4: *reinterpret_cast<uint32_t*>(dst) = *reinterpret_cast<const uint32_t*>(src); break;
        case 2: *reinterpret_cast<uint16_t*>(dst) = *reinterpret_cast<const uint16_t*>(src); break;
        default: *dst = *src; break;
      }
    }
  }
}

// d lanes cooperate on one destination, lane s of the group owns slot s; a wave holds
// floor(64 / d) groups (its last 64 mod d lanes idle).
__global__ void __launch_bounds__(kThreads) k_sample_insert(const Launch P) {
  const BatchCtx& B = P.b[blockIdx.y];
  if (status_of(B, P.L) != 0) return;
  const int n = static_cast<int>(B.counts[P.h]);
  const int d = P.d;
  const int lane = threadIdx.x & 63;
  const int per_wave = 64 / d;                 // destinations per wave
  const int per_block = per_wave * (kThreads / 64);
  const int grp = lane / d;
  const int s = lane - grp * d;
  const bool lane_used = grp < per_wave;
  const int gbase = grp * d;                   // first lane of the group within the wave
  const unsigned long long gmask = (1ull << d) - 1ull;
  const int row_in_block = (threadIdx.x >> 6) * per_wave + grp;

  for (int i0 = blockIdx.x * per_block; i0 < n; i0 += gridDim.x * per_block) {
    const int i = i0 + row_in_block;
    const bool row = lane_used && i < n;
    uint32_t v = 0, deg = 0;
    int64_t a = 0;
    if (row) {
      v = static_cast<uint32_t>(B.node_ids[i]);
      a = P.indptr[v];
      deg = static_cast<uint32_t>(P.indptr[v + 1] - a);
    }
    const bool floyd = row && deg > static_cast<uint32_t>(d);
    const uint32_t k = floyd ? static_cast<uint32_t>(d) : deg;
    uint32_t p = static_cast<uint32_t>(s);  // whole row in CSR order when deg <= d
    uint32_t t = 0, j = 0;
    if (floyd) {
      const uint32_t w = philox_word(v, static_cast<uint32_t>(P.h), static_cast<uint32_t>(s) >> 2,
                                     B.key0, B.key1, static_cast<uint32_t>(s) & 3u);
      j = deg - static_cast<uint32_t>(d) + static_cast<uint32_t>(s);
      t = __umulhi(w, j + 1u);  // index in [0, j]
    }
    // Floyd's subset algorithm, resolved slot by slot: pick t_s unless an earlier slot holds it,
    // then pick j_s.  The membership test is a linear search over the lanes (the array set).
    if (__any(floyd)) {
      for (int q = 0; q < d; ++q) {
        const uint32_t tq = __shfl(t, gbase + q, 64);
        const bool hit = floyd && s < q && p == tq;
        const unsigned long long bal = (__ballot(hit) >> gbase) & gmask;
        if (floyd && s == q) p = bal ? j : tq;
      }
    }
    if (row && static_cast<uint32_t>(s) < k) {
      const uint32_t g = static_cast<uint32_t>(P.indices[a + p]);
      const uint32_t pos = static_cast<uint32_t>(i) * static_cast<uint32_t>(d) + static_cast<uint32_t>(s);
      uint32_t slot;
      bool full;
      const uint32_t prev = table_insert_min(B, g, kPend | pos, slot, full);
      if (full) set_status(B, P.L, SMFG_ST_TABLE_FULL);
      // prev < kPend      : a node known before this hop, prev is its final local id
      // prev < kPend|pos  : an earlier sample of this hop holds the node: keep it as a pointer
      // prev > kPend|pos  : this sample now holds the node; it displaced the sample at prev
      //                     (unless the node was new), which is told so through lostto
      uint32_t e = prev;
      if (prev > (kPend | pos)) {
        e = kSlot | slot;
        if (prev != 0xFFFFFFFFu) B.lostto[prev & ~kTagMask] = kPend | pos;
      }
      B.ent[pos] = e;
      B.gsrc[pos] = static_cast<int32_t>(g);
    }
    if (row && s == 0) B.rowk[i] = static_cast<int32_t>(k);
  }
}

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

// (destination, slot) of the idx-th padded sample of a tile: idx = r * d + s.
struct DivD {
  uint64_t inv;  // ceil(2^32 / d); the quotient is exact for idx < 2^27
  uint32_t d;
  __device__ __forceinline__ explicit DivD(uint32_t d_) : inv((0xFFFFFFFFull / d_) + 1ull), d(d_) {}
  __device__ __forceinline__ void split(uint32_t idx, uint32_t& r, uint32_t& s) const {
    r = static_cast<uint32_t>((static_cast<uint64_t>(idx) * inv) >> 32);
    s = idx - r * d;
  }
};

// One block per tile of kTileRows destinations.  The padded samples of a tile are one contiguous
// span of ent / lostto, read flat and coalesced.
__global__ void __launch_bounds__(kThreads) k_flag_rows(const Launch P) {
  __shared__ unsigned long long lds[kThreads / 64];
  __shared__ int k_lds[kTileRows];
  __shared__ unsigned int mask_lds[kTileRows];
  static_assert(kTileRows == kThreads, "one row per thread");
  const BatchCtx& B = P.b[blockIdx.y];
  if (status_of(B, P.L) != 0) {
    // a failed sample_insert may have left displacement notes behind: wipe them all
    for (int64_t q = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; q < B.lostto_entries;
         q += static_cast<int64_t>(gridDim.x) * kThreads)
      B.lostto[q] = 0u;
    return;
  }
  const int n = static_cast<int>(B.counts[P.h]);
  const uint32_t d = static_cast<uint32_t>(P.d);
  const DivD div(d);
  const int tiles = (n + kTileRows - 1) / kTileRows;
  for (int tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    const int i0 = tile * kTileRows;
    const int nrows = n - i0 < kTileRows ? n - i0 : kTileRows;
    const int tr = threadIdx.x;
    __syncthreads();
    k_lds[tr] = tr < nrows ? B.rowk[i0 + tr] : 0;
    mask_lds[tr] = 0u;
    __syncthreads();
    const uint32_t pos0 = static_cast<uint32_t>(i0) * d;
    const uint32_t cnt = static_cast<uint32_t>(nrows) * d;
    constexpr int U = 4;
    for (uint32_t base = threadIdx.x; base < cnt; base += kThreads * U) {
      uint32_t lost[U], e[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t idx = base + u * kThreads;
        lost[u] = idx < cnt ? B.lostto[pos0 + idx] : 0u;
        e[u] = idx < cnt ? B.ent[pos0 + idx] : 0u;
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t idx = base + u * kThreads;
        if (idx < cnt) {
          uint32_t r, sl;
          div.split(idx, r, sl);
          if (sl < static_cast<uint32_t>(k_lds[r])) {
            if (lost[u] != 0u) {  // displaced by the sample at lost[u]: follow it later
              B.ent[pos0 + idx] = lost[u];
              B.lostto[pos0 + idx] = 0u;
            } else if ((e[u] & kTagMask) == kSlot) {
              atomicOr(&mask_lds[r], 1u << sl);
            }
          }
        }
      }
    }
    __syncthreads();
    const int k = k_lds[tr];
    const uint32_t m = mask_lds[tr];
    const unsigned long long x = (static_cast<unsigned long long>(k) << 32) | static_cast<unsigned long long>(__popc(m));
    unsigned long long total;
    const unsigned long long pre = block_exscan(x, lds, total);
    if (tr < nrows) {
      B.rowmask[i0 + tr] = m;
      B.rowoff[i0 + tr] = static_cast<int32_t>(pre >> 32);
      B.newrank[i0 + tr] = static_cast<int32_t>(pre & 0xFFFFFFFFull);
    }
    if (tr == 0) B.tile_sums[tile] = total;
  }
}

__global__ void __launch_bounds__(kThreads) k_scan_tiles(const Launch P) {
  __shared__ unsigned long long lds[kThreads / 64];
  const BatchCtx& B = P.b[blockIdx.y];
  if (status_of(B, P.L) != 0) return;
  const int n = static_cast<int>(B.counts[P.h]);
  const int tiles = (n + kTileRows - 1) / kTileRows;
  unsigned long long carry = 0;
  for (int t0 = 0; t0 < tiles; t0 += kThreads) {
    const int t = t0 + threadIdx.x;
    const unsigned long long x = t < tiles ? B.tile_sums[t] : 0ull;
    unsigned long long total;
    const unsigned long long ex = block_exscan(x, lds, total);
    if (t < tiles) B.tile_sums[t] = carry + ex;
    carry += total;
  }
  if (threadIdx.x == 0) {
    const int64_t edges = static_cast<int64_t>(carry >> 32);
    const int64_t nodes = static_cast<int64_t>(n) + static_cast<int64_t>(carry & 0xFFFFFFFFull);
    B.counts[P.L + 1 + P.h] = edges;
    B.counts[P.h + 1] = nodes;
    B.blk_indptr[n] = static_cast<int32_t>(edges);
    if (nodes > B.node_capacity) set_status(B, P.L, SMFG_ST_NODE_CAPACITY);
    else if (edges > B.edge_capacity) set_status(B, P.L, SMFG_ST_EDGE_CAPACITY);
  }
}

// One block per tile of kTileRows destinations; samples are walked flat like in k_flag_rows.
__global__ void __launch_bounds__(kThreads) k_assemble(const Launch P) {
  __shared__ int k_lds[kTileRows];
  __shared__ unsigned int mask_lds[kTileRows];
  __shared__ unsigned int off_lds[kTileRows];   // global edge offset of the destination
  __shared__ unsigned int rank_lds[kTileRows];  // local id of the destination's first new node
  const BatchCtx& B = P.b[blockIdx.y];
  if (status_of(B, P.L) != 0) return;
  const int n = static_cast<int>(B.counts[P.h]);
  const uint32_t d = static_cast<uint32_t>(P.d);
  const DivD div(d);
  const bool last = P.h == P.L - 1;  // nodes found in the last hop are never looked up again
  const int tiles = (n + kTileRows - 1) / kTileRows;
  for (int tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    const int i0 = tile * kTileRows;
    const int nrows = n - i0 < kTileRows ? n - i0 : kTileRows;
    const int tr = threadIdx.x;
    const unsigned long long tpre = B.tile_sums[tile];
    __syncthreads();
    if (tr < nrows) {
      const uint32_t off = static_cast<uint32_t>(tpre >> 32) + static_cast<uint32_t>(B.rowoff[i0 + tr]);
      k_lds[tr] = B.rowk[i0 + tr];
      mask_lds[tr] = B.rowmask[i0 + tr];
      off_lds[tr] = off;
      rank_lds[tr] = static_cast<uint32_t>(n) + static_cast<uint32_t>(tpre & 0xFFFFFFFFull) +
                     static_cast<uint32_t>(B.newrank[i0 + tr]);
      B.blk_indptr[i0 + tr] = static_cast<int32_t>(off);
    } else {
      k_lds[tr] = 0;
    }
    __syncthreads();
    const uint32_t pos0 = static_cast<uint32_t>(i0) * d;
    const uint32_t cnt = static_cast<uint32_t>(nrows) * d;
    constexpr int U = 4;
    for (uint32_t base = threadIdx.x; base < cnt; base += kThreads * U) {
      uint32_t e[U], g[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t idx = base + u * kThreads;
        e[u] = idx < cnt ? B.ent[pos0 + idx] : 0u;
        g[u] = idx < cnt ? static_cast<uint32_t>(B.gsrc[pos0 + idx]) : 0u;
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t idx = base + u * kThreads;
        if (idx >= cnt) continue;
        uint32_t r, sl;
        div.split(idx, r, sl);
        if (sl >= static_cast<uint32_t>(k_lds[r])) continue;
        const uint32_t tag = e[u] & kTagMask;
        uint32_t local = e[u];
        if (tag == kSlot) {  // first appearance: rank among the new nodes of this hop
          local = rank_lds[r] + __popc(mask_lds[r] & ((1u << sl) - 1u));
          B.node_ids[local] = static_cast<int32_t>(g[u]);
          if (!last) B.table[e[u] & ~kTagMask] = (static_cast<uint64_t>(g[u]) << 32) | local;
        } else if (tag != 0u) {  // kPend: same node as the sample at position q < own position
          uint32_t q = e[u] & ~kTagMask;
          for (;;) {
            const uint32_t qi = q / d, qs = q - qi * d;
            const uint32_t m = B.rowmask[qi];
            if ((m >> qs) & 1u) {  // q is the node's first appearance
              local = static_cast<uint32_t>(n) +
                      static_cast<uint32_t>(B.tile_sums[qi / kTileRows] & 0xFFFFFFFFull) +
                      static_cast<uint32_t>(B.newrank[qi]) + __popc(m & ((1u << qs) - 1u));
              break;
            }
            const uint32_t nxt = B.ent[q] & ~kTagMask;  // strictly smaller position
            if (nxt >= q) break;                        // cannot happen; guards the loop
            q = nxt;
          }
        }
        B.blk_indices[off_lds[r] + sl] = static_cast<int32_t>(local);
      }
    }
  }
}

// Rows are moved as vectors of sizeof(V) bytes.  A block copies kGatherRows consecutive output
// rows and exits: many short-lived blocks reach a higher copy rate on this chip than a persistent
// grid-stride loop.  Inside a block the output chunk is addressed as one flat vector array, so
// stores are fully coalesced and the lanes that share a row read one contiguous span of it.
constexpr int kGatherRows = 32;
template <typename V>
__device__ __forceinline__ void gather_rows(const uint8_t* __restrict__ feat, int64_t row_stride,
                                            uint32_t vec_per_row, const int32_t* __restrict__ ids,
                                            int64_t n, uint8_t* __restrict__ out) {
  constexpr int U = 2;
  __shared__ int64_t row_byte[kGatherRows];  // byte offset of each source row
  const int64_t r0 = static_cast<int64_t>(blockIdx.x) * kGatherRows;
  if (r0 >= n) return;
  const uint32_t rows = static_cast<uint32_t>(n - r0 < kGatherRows ? n - r0 : kGatherRows);
  const uint32_t cnt = rows * vec_per_row;
  if (threadIdx.x < kGatherRows)
    row_byte[threadIdx.x] = threadIdx.x < rows ? static_cast<int64_t>(ids[r0 + threadIdx.x]) * row_stride : 0;
  __syncthreads();
  V* __restrict__ o = reinterpret_cast<V*>(out) + static_cast<uint64_t>(r0) * vec_per_row;
  uint32_t base = threadIdx.x;
  // full rounds: U independent row reads in flight per thread, then the U stores
  for (; base + (U - 1) * kThreads < cnt; base += kThreads * U) {
    V val[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t idx = base + u * kThreads;
      const uint32_t jrow = idx / vec_per_row;
      const uint32_t c = idx - jrow * vec_per_row;
      val[u] = __builtin_nontemporal_load(reinterpret_cast<const V*>(feat + row_byte[jrow]) + c);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) __builtin_nontemporal_store(val[u], o + base + u * kThreads);
  }
  for (; base < cnt; base += kThreads) {
    const uint32_t jrow = base / vec_per_row;
    const uint32_t c = base - jrow * vec_per_row;
    __builtin_nontemporal_store(
        __builtin_nontemporal_load(reinterpret_cast<const V*>(feat + row_byte[jrow]) + c), o + base);
  }
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <typename V>
__global__ void __launch_bounds__(kThreads) k_gather(const Launch P) {
  const BatchCtx& B = P.b[blockIdx.y];
  if (status_of(B, P.L) != 0) return;
  int64_t n = B.counts[P.L];
  if (n > B.node_capacity) n = B.node_capacity;
  gather_rows<V>(P.feat, P.row_stride, static_cast<uint32_t>(P.row_bytes / sizeof(V)), B.node_ids, n,
                 B.features);
}

template <typename V>
__global__ void __launch_bounds__(kThreads) k_gather_plain(const uint8_t* feat, int64_t row_bytes,
                                                           int64_t row_stride, const int32_t* ids,
                                                           const int64_t* num_rows, int64_t max_rows,
                                                           uint8_t* out) {
  int64_t n = *num_rows;
  if (n > max_rows) n = max_rows;
  if (n < 0) n = 0;
  gather_rows<V>(feat, row_stride, static_cast<uint32_t>(row_bytes / sizeof(V)), ids, n, out);
}

// ---- wide path: fanouts above 32, or every neighbour (SMFG_FANOUT_ALL) ------------------------
// Samples sit at their exact block offsets (pos = block indptr[i] + s), so a count + scan pass
// comes first and the later passes walk the samples flat, four consecutive samples per thread.
constexpr int kWideTile = 4 * kThreads;  // samples per flat tile

// Degree, sample count and row start per destination; in-tile scan of the sample counts.
__global__ void __launch_bounds__(kThreads) k_count_rows(const Launch P) {
  __shared__ unsigned long long lds[kThreads / 64];
  const BatchCtx& B = P.b[blockIdx.y];
  if (status_of(B, P.L) != 0) return;
  const int n = static_cast<int>(B.counts[P.h]);
  const int d = P.d;
  const int tiles = (n + kTileRows - 1) / kTileRows;
  for (int tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    const int i = tile * kTileRows + threadIdx.x;
    uint32_t k = 0;
    if (i < n) {
      const uint32_t v = static_cast<uint32_t>(B.node_ids[i]);
      const int64_t a = P.indptr[v];
      const uint32_t deg = static_cast<uint32_t>(P.indptr[v + 1] - a);
      k = (d < 0 || deg <= static_cast<uint32_t>(d)) ? deg : static_cast<uint32_t>(d);
      B.rowstart[i] = a;
      B.rowdeg[i] = deg;
      B.rowk[i] = static_cast<int32_t>(k);
    }
    unsigned long long total;
    const unsigned long long pre = block_exscan(k, lds, total);
    if (i < n) B.rowoff[i] = static_cast<int32_t>(pre);
    if (threadIdx.x == 0) B.tile_sums[tile] = total;
    __syncthreads();
  }
}

// Exclusive scan of the per-tile sample counts; E_h and its capacity checks.
__global__ void __launch_bounds__(kThreads) k_scan_count_tiles(const Launch P) {
  __shared__ unsigned long long lds[kThreads / 64];
  const BatchCtx& B = P.b[blockIdx.y];
  if (status_of(B, P.L) != 0) return;
  const int n = static_cast<int>(B.counts[P.h]);
  const int tiles = (n + kTileRows - 1) / kTileRows;
  unsigned long long carry = 0;
  for (int t0 = 0; t0 < tiles; t0 += kThreads) {
    const int t = t0 + threadIdx.x;
    const unsigned long long x = t < tiles ? B.tile_sums[t] : 0ull;
    unsigned long long total;
    const unsigned long long ex = block_exscan(x, lds, total);
    if (t < tiles) B.tile_sums[t] = carry + ex;
    carry += total;
  }
  if (threadIdx.x == 0) {
    const bool fits = carry <= static_cast<unsigned long long>(B.edge_capacity) &&
                      carry <= static_cast<unsigned long long>(B.lostto_entries);
    B.counts[P.L + 1 + P.h] = static_cast<int64_t>(carry);
    if (fits) B.blk_indptr[n] = static_cast<int32_t>(carry);
    else set_status(B, P.L, SMFG_ST_EDGE_CAPACITY);
  }
}

// One wave per destination; lane l of round r owns slot s = 64 r + l.
__global__ void __launch_bounds__(kThreads) k_sample_insert_wide(const Launch P) {
  __shared__ uint32_t picks_lds[kThreads / 64][SMFG_MAX_WIDE_FANOUT];
  const BatchCtx& B = P.b[blockIdx.y];
  if (status_of(B, P.L) != 0) return;
  const int n = static_cast<int>(B.counts[P.h]);
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  uint32_t* picks = picks_lds[wave];
  const int waves_total = gridDim.x * (kThreads / 64);
  for (int i = blockIdx.x * (kThreads / 64) + wave; i < n; i += waves_total) {
    const uint32_t v = static_cast<uint32_t>(B.node_ids[i]);
    const int64_t a = B.rowstart[i];
    const uint32_t deg = static_cast<uint32_t>(B.rowdeg[i]);
    const uint32_t k = static_cast<uint32_t>(B.rowk[i]);
    const uint32_t base = static_cast<uint32_t>(B.tile_sums[i / kTileRows]) + static_cast<uint32_t>(B.rowoff[i]);
    if (lane == 0) B.blk_indptr[i] = static_cast<int32_t>(base);
    const bool floyd = deg > k;  // only then are positions drawn (k = fanout <= SMFG_MAX_WIDE_FANOUT)
    for (uint32_t s0 = 0; s0 < k; s0 += 64) {
      const uint32_t s = s0 + static_cast<uint32_t>(lane);
      const bool active = s < k;
      uint32_t p = s;  // whole row in CSR order when nothing is drawn
      if (floyd) {
        uint32_t t = 0, j = 0;
        if (active) {
          const uint32_t w = philox_word(v, static_cast<uint32_t>(P.h), s >> 2, B.key0, B.key1, s & 3u);
          j = deg - k + s;
          t = __umulhi(w, j + 1u);  // index in [0, j]
        }
        // Floyd's rule slot by slot; the array set is picks[0, s0) in LDS plus the lanes of this round
        const uint32_t round = k - s0 < 64u ? k - s0 : 64u;
        for (uint32_t q = 0; q < round; ++q) {
          const uint32_t tq = __shfl(t, static_cast<int>(q), 64);
          bool hit = static_cast<uint32_t>(lane) < q && p == tq;
          for (uint32_t l = static_cast<uint32_t>(lane); l < s0; l += 64) hit = hit || picks[l] == tq;
          const bool any = __ballot(hit) != 0ull;
          if (static_cast<uint32_t>(lane) == q) p = any ? j : tq;
        }
        if (active) picks[s] = p;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");  // later rounds read all lanes' picks
        __builtin_amdgcn_wave_barrier();
      }
      if (active) {
        const uint32_t g = static_cast<uint32_t>(P.indices[a + p]);
        const uint32_t pos = base + s;
        uint32_t slot;
        bool full;
        const uint32_t prev = table_insert_min(B, g, kPend | pos, slot, full);
        if (full) set_status(B, P.L, SMFG_ST_TABLE_FULL);
        uint32_t e = prev;  // see k_sample_insert for the three cases
        if (prev > (kPend | pos)) {
          e = kSlot | slot;
          if (prev != 0xFFFFFFFFu) B.lostto[prev & ~kTagMask] = kPend | pos;
        }
        B.ent[pos] = e;
        B.gsrc[pos] = static_cast<int32_t>(g);
      }
    }
  }
}

// Flat over the samples: first appearances, their in-tile ranks, per-tile totals.
__global__ void __launch_bounds__(kThreads) k_flag_flat(const Launch P) {
  __shared__ unsigned long long lds[kThreads / 64];
  const BatchCtx& B = P.b[blockIdx.y];
  if (status_of(B, P.L) != 0) {
    for (int64_t q = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; q < B.lostto_entries;
         q += static_cast<int64_t>(gridDim.x) * kThreads)
      B.lostto[q] = 0u;
    return;
  }
  const uint32_t E = static_cast<uint32_t>(B.counts[P.L + 1 + P.h]);
  const uint32_t tiles = (E + kWideTile - 1) / kWideTile;
  for (uint32_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    const uint32_t p0 = tile * kWideTile + threadIdx.x * 4;
    uint32_t first[4];
    uint32_t mine = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      first[u] = 0;
      const uint32_t pos = p0 + u;
      if (pos < E) {
        const uint32_t lost = B.lostto[pos];
        if (lost != 0u) {
          B.ent[pos] = lost;
          B.lostto[pos] = 0u;
        } else {
          first[u] = (B.ent[pos] & kTagMask) == kSlot ? 1u : 0u;
        }
      }
      mine += first[u];
    }
    unsigned long long total;
    uint32_t pre = static_cast<uint32_t>(block_exscan(mine, lds, total));
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (p0 + u < E) B.rank[p0 + u] = pre;
      pre += first[u];
    }
    if (threadIdx.x == 0) B.stile_sums[tile] = total;
    __syncthreads();
  }
}

// Exclusive scan of the per-tile counts of new nodes; n_{h+1} and its capacity check.
__global__ void __launch_bounds__(kThreads) k_scan_flat_tiles(const Launch P) {
  __shared__ unsigned long long lds[kThreads / 64];
  const BatchCtx& B = P.b[blockIdx.y];
  if (status_of(B, P.L) != 0) return;
  const int n = static_cast<int>(B.counts[P.h]);
  const uint32_t E = static_cast<uint32_t>(B.counts[P.L + 1 + P.h]);
  const uint32_t tiles = (E + kWideTile - 1) / kWideTile;
  unsigned long long carry = 0;
  for (uint32_t t0 = 0; t0 < tiles; t0 += kThreads) {
    const uint32_t t = t0 + threadIdx.x;
    const unsigned long long x = t < tiles ? B.stile_sums[t] : 0ull;
    unsigned long long total;
    const unsigned long long ex = block_exscan(x, lds, total);
    if (t < tiles) B.stile_sums[t] = carry + ex;
    carry += total;
  }
  if (threadIdx.x == 0) {
    const int64_t nodes = static_cast<int64_t>(n) + static_cast<int64_t>(carry);
    B.counts[P.h + 1] = nodes;
    if (nodes > B.node_capacity) set_status(B, P.L, SMFG_ST_NODE_CAPACITY);
  }
}

// Flat over the samples: final local ids -> block indices; first appearances publish themselves.
__global__ void __launch_bounds__(kThreads) k_assemble_flat(const Launch P) {
  const BatchCtx& B = P.b[blockIdx.y];
  if (status_of(B, P.L) != 0) return;
  const uint32_t n = static_cast<uint32_t>(B.counts[P.h]);
  const uint32_t E = static_cast<uint32_t>(B.counts[P.L + 1 + P.h]);
  const bool last = P.h == P.L - 1;
  const uint32_t tiles = (E + kWideTile - 1) / kWideTile;
  for (uint32_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    const uint32_t tpre = n + static_cast<uint32_t>(B.stile_sums[tile]);
    const uint32_t p0 = tile * kWideTile + threadIdx.x * 4;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint32_t pos = p0 + u;
      if (pos >= E) continue;
      const uint32_t e = B.ent[pos];
      const uint32_t tag = e & kTagMask;
      uint32_t local = e;
      if (tag == kSlot) {
        local = tpre + B.rank[pos];
        const uint32_t g = static_cast<uint32_t>(B.gsrc[pos]);
        B.node_ids[local] = static_cast<int32_t>(g);
        if (!last) B.table[e & ~kTagMask] = (static_cast<uint64_t>(g) << 32) | local;
      } else if (tag != 0u) {  // kPend: same node as the sample at position q < pos
        uint32_t q = e & ~kTagMask;
        for (;;) {
          const uint32_t eq = B.ent[q];
          if ((eq & kTagMask) == kSlot) {  // q is the node's first appearance
            local = n + static_cast<uint32_t>(B.stile_sums[q / kWideTile]) + B.rank[q];
            break;
          }
          const uint32_t nxt = eq & ~kTagMask;  // strictly smaller position
          if (nxt >= q) break;                  // cannot happen; guards the loop
          q = nxt;
        }
      }
      B.blk_indices[pos] = static_cast<int32_t>(local);
    }
  }
}

// ---- a consumer: GraphSAGE mean aggregation over one block -------------------------------------
// 16 lanes per destination; a lane owns V consecutive columns per round of 16 * V columns and
// accumulates its destination's sampled source rows in float, slot order, two rows in flight.
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
                                                             const int64_t* __restrict__ num_dst, int64_t max_dst,
                                                             const T* __restrict__ x, int dim,
                                                             float* __restrict__ out) {
  int64_t n = *num_dst;
  if (n > max_dst) n = max_dst;
  const int64_t i = static_cast<int64_t>(blockIdx.x) * kAggRows + threadIdx.x / kAggLanes;
  if (i >= n) return;
  const int lane = threadIdx.x & (kAggLanes - 1);
  const int e0 = indptr[i], e1 = indptr[i + 1];
  const float k = static_cast<float>(e1 - e0);
  typedef RowVec<T, V> Vec;
  for (int c = lane * V; c < dim; c += kAggLanes * V) {
    float acc[V];
#pragma unroll
    for (int t = 0; t < V; ++t) acc[t] = 0.f;
    int e = e0;
    for (; e + 1 < e1; e += 2) {
      const Vec a = *reinterpret_cast<const Vec*>(x + static_cast<int64_t>(indices[e]) * dim + c);
      const Vec b = *reinterpret_cast<const Vec*>(x + static_cast<int64_t>(indices[e + 1]) * dim + c);
#pragma unroll
      for (int t = 0; t < V; ++t) acc[t] = (acc[t] + to_float(a.v[t])) + to_float(b.v[t]);
    }
    if (e < e1) {
      const Vec a = *reinterpret_cast<const Vec*>(x + static_cast<int64_t>(indices[e]) * dim + c);
#pragma unroll
      for (int t = 0; t < V; ++t) acc[t] += to_float(a.v[t]);
    }
    float* o = out + i * dim + c;
#pragma unroll
    for (int t = 0; t < V; ++t) o[t] = e1 > e0 ? acc[t] / k : 0.f;
  }
}

// ---- host side --------------------------------------------------------------------------------

inline int hip_err(hipError_t e) { return e == hipSuccess ? SMFG_OK : SMFG_ERR_HIP_BASE - static_cast<int>(e); }


inline int vec_bytes(uintptr_t a, uintptr_t b, int64_t row_bytes, int64_t row_stride) {
  const uint64_t x = static_cast<uint64_t>(a) | static_cast<uint64_t>(b) | static_cast<uint64_t>(row_bytes) |
                     static_cast<uint64_t>(row_stride);
  if ((x & 15) == 0) return 16;
  if ((x & 7) == 0) return 8;
  if ((x & 3) == 0) return 4;
  if ((x & 1) == 0) return 2;
  return 1;
}

// Optional event bracketing of launches (smfg_profile_begin / smfg_profile_end).
struct Profiler {
  int level = 0;
  int max_records = 0;
  int used = 0;
  hipEvent_t* ev = nullptr;  // 2 per record
  int* stage = nullptr;
} g_prof;

struct StageTimer {
  int rec = -1;
  hipStream_t st;
  StageTimer(int stage, hipStream_t s) : st(s) {
    if (g_prof.level == 0) return;
    if (g_prof.level == 1 && stage != SMFG_STAGE_GATHER) return;
    if (g_prof.used >= g_prof.max_records) return;
    rec = g_prof.used++;
    g_prof.stage[rec] = stage;
    (void)hipEventRecord(g_prof.ev[2 * rec], st);
  }
  ~StageTimer() {
    if (rec >= 0) (void)hipEventRecord(g_prof.ev[2 * rec + 1], st);
  }
};

void profiler_free() {
  for (int i = 0; i < 2 * g_prof.max_records; ++i)
    if (g_prof.ev && g_prof.ev[i]) (void)hipEventDestroy(g_prof.ev[i]);
  std::free(g_prof.ev);
  std::free(g_prof.stage);
  g_prof = Profiler();
}

inline unsigned blocks_for(int64_t work_items, int64_t per_block, unsigned cap) {
  int64_t b = (work_items + per_block - 1) / per_block;
  if (b < 1) b = 1;
  if (b > cap) b = cap;
  return static_cast<unsigned>(b);
}

}  // namespace

struct smfg_graph {
  int64_t num_nodes, num_edges;
  const int64_t* indptr;
  const int32_t* indices;
  const uint8_t* feat;
  int64_t row_bytes, row_stride;
  const uint8_t* labels;
  int32_t label_bytes;
  int device;
};

struct smfg_workspace {
  int device;
  int32_t max_seeds, L;
  int32_t fanouts[SMFG_MAX_LAYERS];
  int64_t node_capacity;
  int64_t slot_entries;  // capacity of `slot`
  int64_t bytes;
  uint32_t table_log2;
  void* slab;
  uint64_t* table;
  uint32_t* ent;
  uint32_t* lostto;
  int32_t* gsrc;
  int32_t* rowk;
  uint32_t* rowmask;
  int32_t* newrank;
  int32_t* rowoff;
  uint64_t* tile_sums;
  int64_t* rowstart;
  int32_t* rowdeg;
  uint32_t* rank;
  uint64_t* stile_sums;
};

namespace {

// Largest (destination, slot) index space any hop can need, given a node capacity; -1 when a hop
// takes every neighbour (no bound without the degrees).
int64_t slot_entries_needed(int32_t num_seeds, int32_t L, const int32_t* fanouts, int64_t num_nodes,
                            int64_t node_capacity) {
  int64_t n = num_seeds < num_nodes ? num_seeds : num_nodes, need = 0;
  for (int h = 0; h < L; ++h) {
    if (fanouts[h] < 0) return -1;
    if (n > node_capacity) n = node_capacity;
    const int64_t e = n * fanouts[h];
    if (e > need) need = e;
    n = n + e;
    if (n > num_nodes) n = num_nodes;
  }
  return need;
}

// Valid fanouts; `wide` tells whether the call needs the exact-offset path.
int check_fanouts(int32_t L, const int32_t* fanouts, bool* wide = nullptr) {
  if (L < 1 || L > SMFG_MAX_LAYERS) return SMFG_ERR_TOO_MANY_LAYERS;
  if (!fanouts) return SMFG_ERR_NULL_PTR;
  bool w = false;
  for (int h = 0; h < L; ++h) {
    const int d = fanouts[h];
    if (d != SMFG_FANOUT_ALL && (d < 1 || d > SMFG_MAX_WIDE_FANOUT)) return SMFG_ERR_BAD_FANOUT;
    if (d == SMFG_FANOUT_ALL || d > SMFG_MAX_FANOUT) w = true;
  }
  if (wide) *wide = w;
  return SMFG_OK;
}

// The gather launch shared by smfg_sample_mfg_many and smfg_gather_many.
void launch_gather(const Launch& P, int64_t max_rows, int vb, unsigned G, hipStream_t st) {
  const unsigned gb = blocks_for(max_rows, kGatherRows, 0x7FFFFFFFu);
  StageTimer t_(SMFG_STAGE_GATHER, st);
  switch (vb) {
    case 16: k_gather<u32x4><<<dim3(gb, G), kThreads, 0, st>>>(P); break;
    case 8: k_gather<u32x2><<<dim3(gb, G), kThreads, 0, st>>>(P); break;
    case 4: k_gather<uint32_t><<<dim3(gb, G), kThreads, 0, st>>>(P); break;
    case 2: k_gather<uint16_t><<<dim3(gb, G), kThreads, 0, st>>>(P); break;
    default: k_gather<uint8_t><<<dim3(gb, G), kThreads, 0, st>>>(P); break;
  }
}

}  // namespace

extern "C" {

int smfg_graph_create(smfg_graph_t** out, int64_t num_nodes, int64_t num_edges, const int64_t* d_indptr,
                      const int32_t* d_indices, const void* d_feat, int32_t feat_dim, int32_t elem_bytes,
                      int64_t row_stride_bytes) {
  if (!out) return SMFG_ERR_NULL_PTR;
  *out = nullptr;
  if (!d_indptr || (num_edges > 0 && !d_indices)) return SMFG_ERR_NULL_PTR;
  if (num_nodes < 0 || num_nodes >= (1ll << 31) || num_edges < 0) return SMFG_ERR_INVALID_ARG;
  int64_t row_bytes = 0;
  if (d_feat) {
    if (feat_dim < 1 || elem_bytes < 1) return SMFG_ERR_INVALID_ARG;
    row_bytes = static_cast<int64_t>(feat_dim) * elem_bytes;
    if (row_stride_bytes < row_bytes) return SMFG_ERR_INVALID_ARG;
  }
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_err(e);
  smfg_graph* g = new (std::nothrow) smfg_graph;
  if (!g) return SMFG_ERR_OOM;
  g->num_nodes = num_nodes;
  g->num_edges = num_edges;
  g->indptr = d_indptr;
  g->indices = d_indices;
  g->feat = static_cast<const uint8_t*>(d_feat);
  g->row_bytes = row_bytes;
  g->row_stride = d_feat ? row_stride_bytes : 0;
  g->labels = nullptr;
  g->label_bytes = 0;
  g->device = dev;
  *out = g;
  return SMFG_OK;
}

int smfg_graph_destroy(smfg_graph_t* g) {
  delete g;
  return SMFG_OK;
}

int smfg_graph_set_labels(smfg_graph_t* g, const void* d_labels, int32_t elem_bytes) {
  if (!g) return SMFG_ERR_NULL_PTR;
  if (!d_labels) {
    g->labels = nullptr;
    g->label_bytes = 0;
    return SMFG_OK;
  }
  if (elem_bytes != 1 && elem_bytes != 2 && elem_bytes != 4 && elem_bytes != 8) return SMFG_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(d_labels) % static_cast<uintptr_t>(elem_bytes) != 0) return SMFG_ERR_INVALID_ARG;
  g->labels = static_cast<const uint8_t*>(d_labels);
  g->label_bytes = elem_bytes;
  return SMFG_OK;
}

int smfg_bounds(int32_t num_seeds, int32_t L, const int32_t* fanouts, int64_t num_nodes, int64_t* max_nodes,
                int64_t* max_edges) {
  int rc = check_fanouts(L, fanouts);
  if (rc != SMFG_OK) return rc;
  if (!max_nodes || !max_edges) return SMFG_ERR_NULL_PTR;
  if (num_seeds < 0 || num_nodes < 0) return SMFG_ERR_INVALID_ARG;
  int64_t n = num_seeds < num_nodes ? num_seeds : num_nodes;
  max_nodes[0] = n;
  bool all = false;
  for (int h = 0; h < L; ++h) {
    all = all || fanouts[h] == SMFG_FANOUT_ALL;
    if (all) {
      max_edges[h] = fanouts[h] == SMFG_FANOUT_ALL ? -1 : num_nodes * fanouts[h];
      n = num_nodes;
    } else {
      max_edges[h] = n * fanouts[h];
      n = n + max_edges[h];
      if (n > num_nodes) n = num_nodes;
    }
    max_nodes[h + 1] = n;
  }
  return SMFG_OK;
}

int smfg_workspace_create(smfg_workspace_t** out, const smfg_graph_t* g, int32_t max_seeds, int32_t L,
                          const int32_t* fanouts, int64_t node_capacity) {
  return smfg_workspace_create_sized(out, g, max_seeds, L, fanouts, node_capacity, 0);
}

int smfg_workspace_create_sized(smfg_workspace_t** out, const smfg_graph_t* g, int32_t max_seeds, int32_t L,
                                const int32_t* fanouts, int64_t node_capacity, int64_t sample_capacity) {
  if (!out) return SMFG_ERR_NULL_PTR;
  *out = nullptr;
  if (!g) return SMFG_ERR_NULL_PTR;
  int rc = check_fanouts(L, fanouts);
  if (rc != SMFG_OK) return rc;
  if (max_seeds < 0 || node_capacity < 0 || sample_capacity < 0) return SMFG_ERR_INVALID_ARG;
  int64_t mn[SMFG_MAX_LAYERS + 1], me[SMFG_MAX_LAYERS];
  smfg_bounds(max_seeds, L, fanouts, g->num_nodes, mn, me);
  if (node_capacity == 0 || node_capacity > mn[L]) node_capacity = mn[L];
  if (node_capacity < 1) node_capacity = 1;
  if (node_capacity < mn[0]) return SMFG_ERR_TOO_MANY_SEEDS;
  int64_t slots = slot_entries_needed(max_seeds, L, fanouts, g->num_nodes, node_capacity);
  if (sample_capacity > 0) slots = sample_capacity;
  if (slots < 0) return SMFG_ERR_INVALID_ARG;  // SMFG_FANOUT_ALL needs an explicit sample capacity
  if (slots >= (1ll << 30) || node_capacity > (1ll << 29)) return SMFG_ERR_CAPACITY;

  uint32_t lg = 10;
  while ((1ll << lg) < 2 * node_capacity) ++lg;

  smfg_workspace* ws = new (std::nothrow) smfg_workspace;
  if (!ws) return SMFG_ERR_OOM;
  std::memset(ws, 0, sizeof(*ws));
  ws->device = g->device;
  ws->max_seeds = max_seeds;
  ws->L = L;
  for (int h = 0; h < L; ++h) ws->fanouts[h] = fanouts[h];
  ws->node_capacity = node_capacity;
  ws->slot_entries = slots > 0 ? slots : 1;
  ws->table_log2 = lg;

  auto align = [](int64_t x) { return (x + 255) & ~int64_t(255); };
  const int64_t tiles = (node_capacity + kTileRows - 1) / kTileRows + 1;
  const int64_t b_table = align((int64_t(1) << lg) * 8);
  const int64_t b_slot = align(ws->slot_entries * 4);
  const int64_t b_rowk = align((node_capacity + 4) * 4);
  const int64_t b_mask = align((node_capacity + 4) * 4);
  const int64_t b_tiles = align(tiles * 8);
  const int64_t b_start = align((node_capacity + 4) * 8);
  const int64_t b_stiles = align((ws->slot_entries / kWideTile + 2) * 8);
  ws->bytes = b_table + 4 * b_slot + 5 * b_rowk + b_tiles + b_start + b_stiles;
  int cur = 0;
  (void)hipGetDevice(&cur);
  if (cur != g->device) (void)hipSetDevice(g->device);
  hipError_t e = hipMalloc(&ws->slab, static_cast<size_t>(ws->bytes));
  if (e != hipSuccess) {
    (void)hipGetLastError();
    if (cur != g->device) (void)hipSetDevice(cur);
    delete ws;
    return SMFG_ERR_OOM;
  }
  uint8_t* p = static_cast<uint8_t*>(ws->slab);
  ws->table = reinterpret_cast<uint64_t*>(p); p += b_table;
  ws->ent = reinterpret_cast<uint32_t*>(p); p += b_slot;
  ws->lostto = reinterpret_cast<uint32_t*>(p); p += b_slot;
  ws->gsrc = reinterpret_cast<int32_t*>(p); p += b_slot;
  ws->rowk = reinterpret_cast<int32_t*>(p); p += b_rowk;
  ws->rowmask = reinterpret_cast<uint32_t*>(p); p += b_mask;
  ws->newrank = reinterpret_cast<int32_t*>(p); p += b_rowk;
  ws->rowoff = reinterpret_cast<int32_t*>(p); p += b_rowk;
  ws->tile_sums = reinterpret_cast<uint64_t*>(p); p += b_tiles;
  ws->rowstart = reinterpret_cast<int64_t*>(p); p += b_start;
  ws->rowdeg = reinterpret_cast<int32_t*>(p); p += b_rowk;
  ws->rank = reinterpret_cast<uint32_t*>(p); p += b_slot;
  ws->stile_sums = reinterpret_cast<uint64_t*>(p);
  // displacement notes start out clear; flag_rows clears whatever a call writes
  e = hipMemset(ws->lostto, 0, static_cast<size_t>(b_slot));
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (cur != g->device) (void)hipSetDevice(cur);
  if (e != hipSuccess) {
    (void)hipFree(ws->slab);
    delete ws;
    return hip_err(e);
  }
  *out = ws;
  return SMFG_OK;
}

int smfg_workspace_destroy(smfg_workspace_t* ws) {
  if (!ws) return SMFG_OK;
  hipError_t e = hipFree(ws->slab);
  delete ws;
  return hip_err(e);
}

int64_t smfg_workspace_bytes(const smfg_workspace_t* ws) { return ws ? ws->bytes : 0; }

int smfg_sample_mfg_many(const smfg_graph_t* g, smfg_workspace_t* const* ws, const int32_t* const* d_seeds,
                         const int32_t* num_seeds, const int32_t* fanouts, int32_t L, const uint64_t* rng_keys,
                         const smfg_output_t* outs, int32_t num_batches, void* hip_stream) {
  if (!g || !ws || !d_seeds || !num_seeds || !rng_keys || !outs) return SMFG_ERR_NULL_PTR;
  bool wide = false;
  int rc = check_fanouts(L, fanouts, &wide);
  if (rc != SMFG_OK) return rc;
  if (num_batches < 1 || num_batches > SMFG_MAX_BATCHES) return SMFG_ERR_INVALID_ARG;

  Launch P;
  std::memset(&P, 0, sizeof(P));
  P.indptr = g->indptr;
  P.indices = g->indices;
  P.feat = g->feat;
  P.row_bytes = g->row_bytes;
  P.row_stride = g->row_stride;
  P.num_nodes = g->num_nodes;
  P.labels = g->labels;
  P.label_bytes = g->label_bytes;
  P.L = L;
  P.G = num_batches;

  int64_t max_n[SMFG_MAX_LAYERS + 1];  // per hop, the largest destination count over the batches
  for (int h = 0; h <= L; ++h) max_n[h] = 0;
  uint32_t max_table_log2 = 0;
  int32_t max_seeds = 0;
  int64_t max_entries = 0;
  bool want_feat = false;
  int vb = 16;

  for (int b = 0; b < num_batches; ++b) {
    const smfg_workspace* w = ws[b];
    const smfg_output_t& o = outs[b];
    if (!w) return SMFG_ERR_NULL_PTR;
    for (int c = 0; c < b; ++c)
      if (ws[c] == w) return SMFG_ERR_INVALID_ARG;
    if (w->device != g->device) return SMFG_ERR_INVALID_ARG;
    if (num_seeds[b] < 0) return SMFG_ERR_INVALID_ARG;
    if (num_seeds[b] > 0 && !d_seeds[b]) return SMFG_ERR_NULL_PTR;
    if (!o.node_ids || !o.counts) return SMFG_ERR_NULL_PTR;
    for (int h = 0; h < L; ++h) {
      if (!o.indptr[h] || !o.indices[h]) return SMFG_ERR_NULL_PTR;
      if (o.edge_capacity[h] < 0) return SMFG_ERR_INVALID_ARG;
    }
    if (o.node_capacity < 1) return SMFG_ERR_INVALID_ARG;
    if (num_seeds[b] > w->max_seeds || num_seeds[b] > o.node_capacity) return SMFG_ERR_TOO_MANY_SEEDS;
    if (o.node_capacity > w->node_capacity) return SMFG_ERR_CAPACITY;
    // fast path: padded positions must fit; wide path: E_h is checked on the device
    if (!wide && slot_entries_needed(num_seeds[b], L, fanouts, g->num_nodes, o.node_capacity) > w->slot_entries)
      return SMFG_ERR_CAPACITY;
    if (w->slot_entries > max_entries) max_entries = w->slot_entries;
    if (g->feat && o.features) {
      want_feat = true;
      const int v = vec_bytes(reinterpret_cast<uintptr_t>(g->feat), reinterpret_cast<uintptr_t>(o.features),
                              g->row_bytes, g->row_stride);
      if (v < vb) vb = v;
    } else if (b > 0 && want_feat) {
      return SMFG_ERR_INVALID_ARG;  // either every batch gathers or none
    }
    if (b > 0 && !want_feat && g->feat && o.features) return SMFG_ERR_INVALID_ARG;

    BatchCtx& B = P.b[b];
    B.seeds = d_seeds[b];
    B.counts = o.counts;
    B.table = w->table;
    B.node_ids = o.node_ids;
    B.ent = w->ent;
    B.lostto = w->lostto;
    B.lostto_entries = w->slot_entries;
    B.gsrc = w->gsrc;
    B.rowk = w->rowk;
    B.rowmask = w->rowmask;
    B.newrank = w->newrank;
    B.rowoff = w->rowoff;
    B.tile_sums = w->tile_sums;
    B.rowstart = w->rowstart;
    B.rowdeg = w->rowdeg;
    B.rank = w->rank;
    B.stile_sums = w->stile_sums;
    B.features = static_cast<uint8_t*>(o.features);
    if (o.labels) {
      if (!g->labels) return SMFG_ERR_INVALID_ARG;
      if (reinterpret_cast<uintptr_t>(o.labels) % static_cast<uintptr_t>(g->label_bytes) != 0)
        return SMFG_ERR_INVALID_ARG;
    }
    B.labels = static_cast<uint8_t*>(o.labels);
    B.node_capacity = static_cast<int32_t>(o.node_capacity);
    B.num_seeds = num_seeds[b];
    B.key0 = static_cast<uint32_t>(rng_keys[b]);
    B.key1 = static_cast<uint32_t>(rng_keys[b] >> 32);
    B.table_shift = 32u - w->table_log2;
    B.table_mask = static_cast<uint32_t>((1ull << w->table_log2) - 1ull);
    if (w->table_log2 > max_table_log2) max_table_log2 = w->table_log2;
    if (num_seeds[b] > max_seeds) max_seeds = num_seeds[b];

    int64_t n = num_seeds[b] < g->num_nodes ? num_seeds[b] : g->num_nodes;
    for (int h = 0; h <= L; ++h) {
      if (n > o.node_capacity) n = o.node_capacity;
      if (n > max_n[h]) max_n[h] = n;
      if (h < L) {
        n = fanouts[h] < 0 ? g->num_nodes : n + n * fanouts[h];
        if (n > g->num_nodes) n = g->num_nodes;
      }
    }
  }

  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  int cur = 0;
  (void)hipGetDevice(&cur);
  if (cur != g->device) (void)hipSetDevice(g->device);
  const unsigned G = static_cast<unsigned>(num_batches);
  constexpr unsigned kCap = 4096;

  { StageTimer t_(SMFG_STAGE_CLEAR, st);
  k_clear<<<dim3(blocks_for(int64_t(1) << max_table_log2, kThreads * 8, 2048), G), kThreads, 0, st>>>(P); }
  { StageTimer t_(SMFG_STAGE_SEEDS, st);
  k_insert_seeds<<<dim3(blocks_for(max_seeds, kThreads, kCap), G), kThreads, 0, st>>>(P); }
  for (int h = 0; h < L; ++h) {
    P.h = h;
    P.d = fanouts[h];
    for (int b = 0; b < num_batches; ++b) {
      P.b[b].blk_indptr = outs[b].indptr[h];
      P.b[b].blk_indices = outs[b].indices[h];
      P.b[b].edge_capacity = outs[b].edge_capacity[h];
    }
    const int64_t rows = max_n[h];
    const unsigned tile_blocks = blocks_for(rows, kTileRows, kCap);
    if (wide) {
      int64_t samples = P.d < 0 ? max_entries : rows * P.d;  // upper bound of E_h
      if (samples > max_entries) samples = max_entries;
      const unsigned flat_blocks = blocks_for(samples, kWideTile, kCap);
      {
        StageTimer t_(SMFG_STAGE_SCAN_TILES, st);
        k_count_rows<<<dim3(tile_blocks, G), kThreads, 0, st>>>(P);
        k_scan_count_tiles<<<dim3(1, G), kThreads, 0, st>>>(P);
      }
      {
        StageTimer t_(SMFG_STAGE_SAMPLE, st);
        k_sample_insert_wide<<<dim3(blocks_for(rows, kThreads / 64, 2 * kCap), G), kThreads, 0, st>>>(P);
      }
      {
        StageTimer t_(SMFG_STAGE_FLAG, st);
        k_flag_flat<<<dim3(flat_blocks, G), kThreads, 0, st>>>(P);
      }
      {
        StageTimer t_(SMFG_STAGE_SCAN_TILES, st);
        k_scan_flat_tiles<<<dim3(1, G), kThreads, 0, st>>>(P);
      }
      {
        StageTimer t_(SMFG_STAGE_ASSEMBLE, st);
        k_assemble_flat<<<dim3(flat_blocks, G), kThreads, 0, st>>>(P);
      }
      continue;
    }
    const unsigned row_blocks = blocks_for(rows, (64 / P.d) * (kThreads / 64), kCap);
    {
      StageTimer t_(SMFG_STAGE_SAMPLE, st);
      k_sample_insert<<<dim3(row_blocks, G), kThreads, 0, st>>>(P);
    }
    {
      StageTimer t_(SMFG_STAGE_FLAG, st);
      k_flag_rows<<<dim3(tile_blocks, G), kThreads, 0, st>>>(P);
    }
    {
      StageTimer t_(SMFG_STAGE_SCAN_TILES, st);
      k_scan_tiles<<<dim3(1, G), kThreads, 0, st>>>(P);
    }
    {
      StageTimer t_(SMFG_STAGE_ASSEMBLE, st);
      k_assemble<<<dim3(tile_blocks, G), kThreads, 0, st>>>(P);
    }
  }
  if (want_feat) launch_gather(P, max_n[L], vb, G, st);
  hipError_t e = hipGetLastError();
  if (cur != g->device) (void)hipSetDevice(cur);
  return hip_err(e);
}

int smfg_sample_mfg(const smfg_graph_t* g, smfg_workspace_t* ws, const int32_t* d_seeds, int32_t num_seeds,
                    const int32_t* fanouts, int32_t L, uint64_t rng_key, const smfg_output_t* out,
                    void* hip_stream) {
  if (!out) return SMFG_ERR_NULL_PTR;
  return smfg_sample_mfg_many(g, &ws, &d_seeds, &num_seeds, fanouts, L, &rng_key, out, 1, hip_stream);
}

int smfg_gather_many(const smfg_graph_t* g, const smfg_output_t* outs, int32_t num_batches, int32_t L,
                     void* hip_stream) {
  if (!g || !outs) return SMFG_ERR_NULL_PTR;
  if (!g->feat) return SMFG_ERR_INVALID_ARG;
  if (L < 1 || L > SMFG_MAX_LAYERS) return SMFG_ERR_TOO_MANY_LAYERS;
  if (num_batches < 1 || num_batches > SMFG_MAX_BATCHES) return SMFG_ERR_INVALID_ARG;
  Launch P;
  std::memset(&P, 0, sizeof(P));
  P.feat = g->feat;
  P.row_bytes = g->row_bytes;
  P.row_stride = g->row_stride;
  P.num_nodes = g->num_nodes;
  P.L = L;
  P.G = num_batches;
  int vb = 16;
  int64_t max_rows = 1;
  for (int b = 0; b < num_batches; ++b) {
    const smfg_output_t& o = outs[b];
    if (!o.node_ids || !o.counts || !o.features) return SMFG_ERR_NULL_PTR;
    if (o.node_capacity < 1 || o.node_capacity > (1ll << 29)) return SMFG_ERR_INVALID_ARG;
    const int v = vec_bytes(reinterpret_cast<uintptr_t>(g->feat), reinterpret_cast<uintptr_t>(o.features),
                            g->row_bytes, g->row_stride);
    if (v < vb) vb = v;
    if (o.node_capacity > max_rows) max_rows = o.node_capacity;
    P.b[b].counts = o.counts;
    P.b[b].node_ids = o.node_ids;
    P.b[b].features = static_cast<uint8_t*>(o.features);
    P.b[b].node_capacity = static_cast<int32_t>(o.node_capacity);
  }
  int cur = 0;
  (void)hipGetDevice(&cur);
  if (cur != g->device) (void)hipSetDevice(g->device);
  launch_gather(P, max_rows, vb, static_cast<unsigned>(num_batches), static_cast<hipStream_t>(hip_stream));
  hipError_t e = hipGetLastError();
  if (cur != g->device) (void)hipSetDevice(cur);
  return hip_err(e);
}

int smfg_gather_rows(const smfg_graph_t* g, const int32_t* d_node_ids, const int64_t* d_num_rows,
                     int64_t max_rows, void* d_out, void* hip_stream) {
  if (!g || !d_node_ids || !d_num_rows || !d_out) return SMFG_ERR_NULL_PTR;
  if (!g->feat) return SMFG_ERR_INVALID_ARG;
  if (max_rows < 0 || max_rows >= (1ll << 31)) return SMFG_ERR_INVALID_ARG;
  if (max_rows == 0) return SMFG_OK;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int vb = vec_bytes(reinterpret_cast<uintptr_t>(g->feat), reinterpret_cast<uintptr_t>(d_out), g->row_bytes,
                           g->row_stride);
  const unsigned gb = blocks_for(max_rows, kGatherRows, 0x7FFFFFFFu);
  uint8_t* o = static_cast<uint8_t*>(d_out);
  int cur = 0;
  (void)hipGetDevice(&cur);
  if (cur != g->device) (void)hipSetDevice(g->device);
  switch (vb) {
    case 16: k_gather_plain<u32x4><<<gb, kThreads, 0, st>>>(g->feat, g->row_bytes, g->row_stride, d_node_ids, d_num_rows, max_rows, o); break;
    case 8: k_gather_plain<u32x2><<<gb, kThreads, 0, st>>>(g->feat, g->row_bytes, g->row_stride, d_node_ids, d_num_rows, max_rows, o); break;
    case 4: k_gather_plain<uint32_t><<<gb, kThreads, 0, st>>>(g->feat, g->row_bytes, g->row_stride, d_node_ids, d_num_rows, max_rows, o); break;
    case 2: k_gather_plain<uint16_t><<<gb, kThreads, 0, st>>>(g->feat, g->row_bytes, g->row_stride, d_node_ids, d_num_rows, max_rows, o); break;
    default: k_gather_plain<uint8_t><<<gb, kThreads, 0, st>>>(g->feat, g->row_bytes, g->row_stride, d_node_ids, d_num_rows, max_rows, o); break;
  }
  hipError_t e = hipGetLastError();
  if (cur != g->device) (void)hipSetDevice(cur);
  return hip_err(e);
}

int smfg_mean_aggregate(const int32_t* d_indptr, const int32_t* d_indices, const int64_t* d_num_dst,
                        int64_t max_dst, const void* d_x, int32_t dim, int32_t elem_bytes, float* d_out,
                        void* hip_stream) {
  if (!d_indptr || !d_indices || !d_num_dst || !d_x || !d_out) return SMFG_ERR_NULL_PTR;
  if (dim < 1 || (elem_bytes != 2 && elem_bytes != 4) || max_dst < 0 || max_dst >= (1ll << 31))
    return SMFG_ERR_INVALID_ARG;
  if (max_dst == 0) return SMFG_OK;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const unsigned gb = blocks_for(max_dst, kAggRows, 0x7FFFFFFFu);
  const uintptr_t ax = reinterpret_cast<uintptr_t>(d_x);
  {
    StageTimer t_(SMFG_STAGE_AGGREGATE, st);
    if (elem_bytes == 2) {
      const _Float16* x = static_cast<const _Float16*>(d_x);
      if (dim % 8 == 0 && ax % 16 == 0)
        k_mean_aggregate<_Float16, 8><<<gb, kThreads, 0, st>>>(d_indptr, d_indices, d_num_dst, max_dst, x, dim, d_out);
      else if (dim % 2 == 0 && ax % 4 == 0)
        k_mean_aggregate<_Float16, 2><<<gb, kThreads, 0, st>>>(d_indptr, d_indices, d_num_dst, max_dst, x, dim, d_out);
      else
        k_mean_aggregate<_Float16, 1><<<gb, kThreads, 0, st>>>(d_indptr, d_indices, d_num_dst, max_dst, x, dim, d_out);
    } else {
      const float* x = static_cast<const float*>(d_x);
      if (dim % 4 == 0 && ax % 16 == 0)
        k_mean_aggregate<float, 4><<<gb, kThreads, 0, st>>>(d_indptr, d_indices, d_num_dst, max_dst, x, dim, d_out);
      else
        k_mean_aggregate<float, 1><<<gb, kThreads, 0, st>>>(d_indptr, d_indices, d_num_dst, max_dst, x, dim, d_out);
    }
  }
  return hip_err(hipGetLastError());
}

int smfg_read_counts(const smfg_output_t* out, int32_t L, int64_t* h_counts, void* hip_stream) {
  if (!out || !out->counts || !h_counts) return SMFG_ERR_NULL_PTR;
  if (L < 1 || L > SMFG_MAX_LAYERS) return SMFG_ERR_TOO_MANY_LAYERS;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  hipError_t e = hipMemcpyAsync(h_counts, out->counts, sizeof(int64_t) * (2 * L + 2), hipMemcpyDeviceToHost, st);
  if (e != hipSuccess) return hip_err(e);
  e = hipStreamSynchronize(st);
  if (e != hipSuccess) return hip_err(e);
  return static_cast<int>(h_counts[2 * L + 1]);
}

int smfg_profile_begin(int32_t level, int32_t max_records) {
  if (level < 0 || level > 2 || max_records < 0) return SMFG_ERR_INVALID_ARG;
  profiler_free();
  if (level == 0 || max_records == 0) return SMFG_OK;
  g_prof.ev = static_cast<hipEvent_t*>(std::calloc(2 * static_cast<size_t>(max_records), sizeof(hipEvent_t)));
  g_prof.stage = static_cast<int*>(std::calloc(static_cast<size_t>(max_records), sizeof(int)));
  if (!g_prof.ev || !g_prof.stage) {
    profiler_free();
    return SMFG_ERR_OOM;
  }
  g_prof.max_records = max_records;
  for (int i = 0; i < 2 * max_records; ++i) {
    hipError_t e = hipEventCreate(&g_prof.ev[i]);
    if (e != hipSuccess) {
      profiler_free();
      return hip_err(e);
    }
  }
  g_prof.level = level;
  return SMFG_OK;
}

int smfg_profile_end(double* stage_ms, int64_t* stage_launches) {
  if (!stage_ms || !stage_launches) return SMFG_ERR_NULL_PTR;
  for (int s = 0; s < SMFG_NUM_STAGES; ++s) {
    stage_ms[s] = 0.0;
    stage_launches[s] = 0;
  }
  hipError_t e = hipDeviceSynchronize();
  if (e != hipSuccess) {
    profiler_free();
    return hip_err(e);
  }
  for (int r = 0; r < g_prof.used; ++r) {
    float ms = 0.f;
    e = hipEventElapsedTime(&ms, g_prof.ev[2 * r], g_prof.ev[2 * r + 1]);
    if (e != hipSuccess) {
      profiler_free();
      return hip_err(e);
    }
    stage_ms[g_prof.stage[r]] += ms;
    stage_launches[g_prof.stage[r]] += 1;
  }
  profiler_free();
  return SMFG_OK;
}

const char* smfg_strerror(int code) {
  switch (code) {
    case SMFG_OK: return "ok";
    case SMFG_ERR_INVALID_ARG: return "invalid argument";
    case SMFG_ERR_NULL_PTR: return "null pointer";
    case SMFG_ERR_BAD_FANOUT: return "fanout is neither SMFG_FANOUT_ALL nor in [1, SMFG_MAX_WIDE_FANOUT]";
    case SMFG_ERR_TOO_MANY_LAYERS: return "number of hops out of range [1, SMFG_MAX_LAYERS]";
    case SMFG_ERR_TOO_MANY_SEEDS: return "more seeds than the workspace or output capacity";
    case SMFG_ERR_OOM: return "out of memory";
    case SMFG_ERR_CAPACITY: return "requested capacity exceeds what the workspace supports";
    case SMFG_ST_NODE_CAPACITY: return "device: node capacity exceeded";
    case SMFG_ST_EDGE_CAPACITY: return "device: edge capacity exceeded";
    case SMFG_ST_TABLE_FULL: return "device: dedup table full";
    case SMFG_ST_SEED_OUT_OF_RANGE: return "device: seed out of range";
    case SMFG_ST_DUPLICATE_SEED: return "device: duplicate seed";
    default: return code <= SMFG_ERR_HIP_BASE ? "HIP runtime error" : "unknown code";
  }
}

}  // extern "C"

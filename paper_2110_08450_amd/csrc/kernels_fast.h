// libsmfg fast path (fanouts up to SMFG_MAX_FANOUT), samples at padded positions pos = i * d + s.
// This file: the per-destination draw shared by both dedup strategies, the table strategy's
// clear / seed insert / sample_insert, and the flag_rows / scan_tiles / assemble passes that turn
// first-appearance information into local ids (shared by both strategies).
#ifndef SMFG_KERNELS_FAST_H_
#define SMFG_KERNELS_FAST_H_

#include "device_common.h"

namespace smfg_dev {

__global__ void __launch_bounds__(kThreads) k_clear(const Launch P) {
  const BatchCtx& B = P.b[batch_of_block(P)];
  const size_t n = static_cast<size_t>(B.table_mask) + 1;
  const size_t stride = static_cast<size_t>(blocks_per_batch(P)) * kThreads;
  for (size_t i = static_cast<size_t>(block_in_batch(P)) * kThreads + threadIdx.x; i < n; i += stride)
    B.table[i] = kEmpty;
  if (block_in_batch(P) == 0) {
    const int m = 2 * P.L + 2;
    for (int q = threadIdx.x; q < m; q += kThreads) B.counts[q] = (q == 0) ? B.num_seeds : 0;
  }
}

// ys = y[ids[:batch_size]] (Listing 1): the seeds are the first ids.
__device__ __forceinline__ void copy_label(const Launch& P, const BatchCtx& B, int i, int32_t v) {
  const uint8_t* src = P.labels + static_cast<int64_t>(v) * P.label_bytes;
  uint8_t* dst = B.labels + static_cast<int64_t>(i) * P.label_bytes;
  switch (P.label_bytes) {
    case 8: *reinterpret_cast<uint64_t*>(dst) = *reinterpret_cast<const uint64_t*>(src); break;
    case 4: *reinterpret_cast<uint32_t*>(dst) = *reinterpret_cast<const uint32_t*>(src); break;
    case 2: *reinterpret_cast<uint16_t*>(dst) = *reinterpret_cast<const uint16_t*>(src); break;
    default: *dst = *src; break;
  }
}

// M starts with the destination nodes of hop 0 in the order given (procedure OneHopMFG).
__global__ void __launch_bounds__(kThreads) k_insert_seeds(const Launch P) {
  const BatchCtx& B = P.b[batch_of_block(P)];
  const int stride = blocks_per_batch(P) * kThreads;
  for (int i = block_in_batch(P) * kThreads + threadIdx.x; i < B.num_seeds; i += stride) {
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
    if (B.labels) copy_label(P, B, i, v);
  }
}

// d lanes cooperate on one destination, lane s of the group owns slot s; a wave holds
// floor(64 / d) groups (its last 64 mod d lanes idle).
struct LaneGroups {
  int d, per_wave, per_block, grp, s, gbase, row_in_block;
  bool lane_used;
  unsigned long long gmask;
  __device__ __forceinline__ explicit LaneGroups(int d_) {
    const int lane = threadIdx.x & 63;
    d = d_;
    per_wave = 64 / d;                 // destinations per wave
    per_block = per_wave * (kThreads / 64);
    grp = lane / d;
    s = lane - grp * d;
    lane_used = grp < per_wave;
    gbase = grp * d;                   // first lane of the group within the wave
    gmask = (1ull << d) - 1ull;
    row_in_block = (threadIdx.x >> 6) * per_wave + grp;
  }
};

// The draw for destination i (section 2.2: at most d neighbours, uniformly, without replacement):
// lane s of the destination's group ends up with the global id g of the s-th pick, if s < k.
// `row` tells whether this lane's group has a destination at all; the whole wave must call.
// Returns true for lanes that hold a sample.
__device__ __forceinline__ bool draw_neighbour(const Launch& P, const BatchCtx& B, const LaneGroups& G, int i,
                                               bool row, uint32_t& v, uint32_t& k, uint32_t& g) {
  const int d = G.d, s = G.s;
  uint32_t deg = 0;
  int64_t a = 0;
  v = 0;
  if (row) {
    v = static_cast<uint32_t>(B.node_ids[i]);
    a = P.indptr[v];
    deg = static_cast<uint32_t>(P.indptr[v + 1] - a);
  }
  const bool floyd = row && deg > static_cast<uint32_t>(d);
  k = floyd ? static_cast<uint32_t>(d) : deg;
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
      const uint32_t tq = __shfl(t, G.gbase + q, 64);
      const bool hit = floyd && s < q && p == tq;
      const unsigned long long bal = (__ballot(hit) >> G.gbase) & G.gmask;
      if (floyd && s == q) p = bal ? j : tq;
    }
  }
  const bool has = row && static_cast<uint32_t>(s) < k;
  g = 0;
  // a neighbour id is read once per batch: keep it out of the way of data that is reused
  if (has) g = static_cast<uint32_t>(__builtin_nontemporal_load(P.indices + (a + p)));
  return has;
}

__global__ void __launch_bounds__(kThreads) k_sample_insert(const Launch P) {
  const BatchCtx& B = P.b[batch_of_block(P)];
  // other blocks of this launch may set the status at any time: leave as whole waves only, the
  // lanes below talk to each other
  if (__any(status_of(B, P.L) != 0)) return;
  const int n = static_cast<int>(B.counts[P.h]);
  const LaneGroups G(P.d);
  const int stride = blocks_per_batch(P) * G.per_block;
  for (int i0 = block_in_batch(P) * G.per_block; i0 < n; i0 += stride) {
    const int i = i0 + G.row_in_block;
    const bool row = G.lane_used && i < n;
    uint32_t v, k, g;
    if (draw_neighbour(P, B, G, i, row, v, k, g)) {
      const uint32_t pos = static_cast<uint32_t>(i) * static_cast<uint32_t>(G.d) + static_cast<uint32_t>(G.s);
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
    if (row && G.s == 0) B.rowk[i] = static_cast<int32_t>(k);
  }
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
// span of ent (and lostto), read flat and coalesced.  NOTES: the table strategy's displacement
// notes are applied (a displaced owner becomes a pointer) and cleared; the partition strategy
// writes final states into ent and has no notes.
template <bool NOTES>
__global__ void __launch_bounds__(kThreads) k_flag_rows(const Launch P) {
  __shared__ unsigned long long lds[kThreads / 64];
  __shared__ int k_lds[kTileRows];
  __shared__ unsigned int mask_lds[kTileRows];
  static_assert(kTileRows == kThreads, "one row per thread");
  const BatchCtx& B = P.b[batch_of_block(P)];
  const int nblocks = blocks_per_batch(P);
  if (block_has_status(B, P.L)) {
    if (NOTES) {
      // a failed sample_insert may have left displacement notes behind: wipe them all
      for (int64_t q = static_cast<int64_t>(block_in_batch(P)) * kThreads + threadIdx.x; q < B.lostto_entries;
           q += static_cast<int64_t>(nblocks) * kThreads)
        B.lostto[q] = 0u;
    }
    return;
  }
  const int n = static_cast<int>(B.counts[P.h]);
  const uint32_t d = static_cast<uint32_t>(P.d);
  const DivD div(d);
  const int tiles = (n + kTileRows - 1) / kTileRows;
  for (int tile = block_in_batch(P); tile < tiles; tile += nblocks) {
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
        lost[u] = (NOTES && idx < cnt) ? B.lostto[pos0 + idx] : 0u;
        e[u] = idx < cnt ? B.ent[pos0 + idx] : 0u;
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t idx = base + u * kThreads;
        if (idx < cnt) {
          uint32_t r, sl;
          div.split(idx, r, sl);
          if (sl < static_cast<uint32_t>(k_lds[r])) {
            if (NOTES && lost[u] != 0u) {  // displaced by the sample at lost[u]: follow it later
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
      B.rowmn[i0 + tr] = make_uint2(m, static_cast<uint32_t>(pre & 0xFFFFFFFFull));
      B.rowoff[i0 + tr] = static_cast<int32_t>(pre >> 32);
    }
    if (tr == 0) B.tile_sums[tile] = total;
  }
}

__global__ void __launch_bounds__(kThreads) k_scan_tiles(const Launch P) {
  __shared__ unsigned long long lds[kThreads / 64];
  const BatchCtx& B = P.b[batch_of_block(P)];
  if (block_has_status(B, P.L)) return;
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
// PUBLISH: first appearances also write their final id into their slot of the dedup table (the
// table strategy, all hops but the last); then the tag-01 entries carry that slot.
template <bool PUBLISH>
__global__ void __launch_bounds__(kThreads) k_assemble(const Launch P) {
  __shared__ int k_lds[kTileRows];
  __shared__ unsigned int mask_lds[kTileRows];
  __shared__ unsigned int off_lds[kTileRows];   // global edge offset of the destination
  __shared__ unsigned int rank_lds[kTileRows];  // local id of the destination's first new node
  const BatchCtx& B = P.b[batch_of_block(P)];
  if (block_has_status(B, P.L)) return;
  const int n = static_cast<int>(B.counts[P.h]);
  const uint32_t d = static_cast<uint32_t>(P.d);
  const DivD div(d);
  const int tiles = (n + kTileRows - 1) / kTileRows;
  const int nblocks = blocks_per_batch(P);
  for (int tile = block_in_batch(P); tile < tiles; tile += nblocks) {
    const int i0 = tile * kTileRows;
    const int nrows = n - i0 < kTileRows ? n - i0 : kTileRows;
    const int tr = threadIdx.x;
    const unsigned long long tpre = B.tile_sums[tile];
    __syncthreads();
    if (tr < nrows) {
      const uint32_t off = static_cast<uint32_t>(tpre >> 32) + static_cast<uint32_t>(B.rowoff[i0 + tr]);
      const uint2 mn = B.rowmn[i0 + tr];
      k_lds[tr] = B.rowk[i0 + tr];
      mask_lds[tr] = mn.x;
      off_lds[tr] = off;
      rank_lds[tr] = static_cast<uint32_t>(n) + static_cast<uint32_t>(tpre & 0xFFFFFFFFull) + mn.y;
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
      // Samples that repeat a node found earlier in this hop point at the position q of another
      // sample of it.  The row record of q is fetched for all U samples of the thread before any
      // is used (a sample without such a pointer fetches the tile's first row instead), so the
      // scattered reads of a thread overlap.
      uint32_t r[U], sl[U], q[U], qi[U];
      bool live[U], dup[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t idx = base + u * kThreads;
        r[u] = 0u;
        sl[u] = 0u;
        if (idx < cnt) div.split(idx, r[u], sl[u]);
        live[u] = idx < cnt && sl[u] < static_cast<uint32_t>(k_lds[r[u]]);
        const uint32_t tag = e[u] & kTagMask;
        dup[u] = live[u] && tag != 0u && tag != kSlot;
        q[u] = dup[u] ? (e[u] & ~kTagMask) : pos0;
        qi[u] = q[u] / d;
      }
      uint2 mn[U];
      uint32_t ts[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        mn[u] = B.rowmn[qi[u]];
        ts[u] = static_cast<uint32_t>(B.tile_sums[qi[u] / kTileRows] & 0xFFFFFFFFull);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (!live[u]) continue;
        uint32_t local = e[u];
        if ((e[u] & kTagMask) == kSlot) {  // first appearance: rank among the new nodes of this hop
          local = rank_lds[r[u]] + __popc(mask_lds[r[u]] & ((1u << sl[u]) - 1u));
          B.node_ids[local] = static_cast<int32_t>(g[u]);
          if (PUBLISH) B.table[e[u] & ~kTagMask] = (static_cast<uint64_t>(g[u]) << 32) | local;
        } else if (dup[u]) {
          uint32_t qq = q[u], qqi = qi[u];
          uint2 m = mn[u];
          uint32_t t = ts[u];
          for (;;) {
            const uint32_t qs = qq - qqi * d;
            if ((m.x >> qs) & 1u) {  // qq is the node's first appearance
              local = static_cast<uint32_t>(n) + t + m.y + __popc(m.x & ((1u << qs) - 1u));
              break;
            }
            // Positions strictly decrease along a chain (a sample only ever points at an earlier
            // one), so the walk ends at a first appearance; anything else means the scratch arrays
            // were disturbed, which is reported rather than turned into a wrong index.
            const uint32_t nxt = B.ent[qq] & ~kTagMask;
            if (nxt >= qq) {
              set_status(B, P.L, SMFG_ST_INTERNAL);
              local = 0u;
              break;
            }
            qq = nxt;
            qqi = qq / d;
            m = B.rowmn[qqi];
            t = static_cast<uint32_t>(B.tile_sums[qqi / kTileRows] & 0xFFFFFFFFull);
          }
        }
        B.blk_indices[off_lds[r[u]] + sl[u]] = static_cast<int32_t>(local);
      }
    }
  }
}

}  // namespace smfg_dev

#endif  // SMFG_KERNELS_FAST_H_

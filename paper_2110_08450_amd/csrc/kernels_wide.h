// libsmfg wide path: fanouts above SMFG_MAX_FANOUT and SMFG_FANOUT_ALL, samples at exact block offsets.
// count_rows / scan_count_tiles fix the offsets; then either the table strategy (sample_wide<true>,
// flag_flat, scan_flat_tiles, assemble_flat) or the partition strategy (sample_wide<false>, hist_flat,
// scan_hist, scatter_flat, [split_buckets], dedup_buckets, flag_flat_part, scan_flat_tiles,
// assemble_flat_part) turns the samples into local ids.
#ifndef SMFG_KERNELS_WIDE_H_
#define SMFG_KERNELS_WIDE_H_

#include "device_common.h"
#include "kernels_part.h"

namespace smfg_dev {

// Samples sit at their exact block offsets (pos = block indptr[i] + s), so a count + scan pass
// comes first and the later passes walk the samples flat, four consecutive samples per thread.
constexpr int kWideTile = 4 * kThreads;  // samples per flat tile

// Degree, sample count and row start per destination; in-tile scan of the sample counts.
__global__ void __launch_bounds__(kThreads) k_count_rows(const Launch P) {
  __shared__ unsigned long long lds[kThreads / 64];
  const BatchCtx& B = P.b[batch_of_block(P)];
  if (block_has_status(B, P.L)) return;
  const int n = static_cast<int>(B.counts[P.h]);
  const int d = P.d;
  const int tiles = (n + kTileRows - 1) / kTileRows;
  for (int tile = block_in_batch(P); tile < tiles; tile += blocks_per_batch(P)) {
    const int i = tile * kTileRows + threadIdx.x;
    uint32_t k = 0;
    if (i < n) {
      const int32_t id = B.node_ids[i];
      int64_t a = 0;
      uint32_t deg = 0;
      // the seeds are caller data: none may index the graph unchecked (later hops only hold
      // neighbour ids read from the graph)
      if (P.h == 0 && (id < 0 || static_cast<int64_t>(id) >= P.num_nodes)) {
        set_status(B, P.L, SMFG_ST_SEED_OUT_OF_RANGE);
      } else {
        a = P.indptr[id];
        deg = static_cast<uint32_t>(P.indptr[id + 1] - a);
      }
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
    const bool fits = carry <= static_cast<unsigned long long>(B.edge_capacity) &&
                      carry <= static_cast<unsigned long long>(B.lostto_entries);
    B.counts[P.L + 1 + P.h] = static_cast<int64_t>(carry);
    if (fits) B.blk_indptr[n] = static_cast<int32_t>(carry);
    else set_status(B, P.L, SMFG_ST_EDGE_CAPACITY);
  }
}

// A wave takes up to kWideRows consecutive destinations (fewer when the hop has fewer destinations
// than that per wave of the grid: a hop of few, long rows then still spreads over the chip): lane l
// first fetches the row record of destination l (start, degree, sample count, block offset:
// coalesced, once per group of rows), then the wave walks the rows, lane l of round r owning slot
// s = 64 r + l: first the rows that are one plain round (whole row taken, at most 64 samples; several
// in flight), then the others one by one - a row taken whole kWideCopyRounds rounds at a time, a
// row with drawn positions after Floyd's rule has settled them in the wave's part of the LDS
// (two arrays of the fanout rounded up to 64 words per wave, sized by the launch; none for
// SMFG_FANOUT_ALL, where nothing is drawn).  INSERT: the sample goes into
// the dedup table at once (table strategy); else only its node id is stored (partition strategy).
constexpr int kWideRows = 16;
constexpr int kWideCopyRounds = 8;
constexpr uint32_t wide_lds_words(int d) { return d < 0 ? 0u : (static_cast<uint32_t>(d) + 63u) & ~63u; }
constexpr size_t wide_lds_bytes(int d) { return sizeof(uint32_t) * 2 * (kThreads / 64) * wide_lds_words(d); }

// What happens to a drawn sample: recorded (partition strategy), or also inserted into the dedup
// table right away (table strategy; see k_sample_insert for the three cases).
template <bool INSERT>
__device__ __forceinline__ void wide_emit(const Launch& P, const BatchCtx& B, uint32_t g, uint32_t pos) {
  if (INSERT) {
    uint32_t slot;
    bool full;
    const uint32_t prev = table_insert_min(B, g, kPend | pos, slot, full);
    if (full) set_status(B, P.L, SMFG_ST_TABLE_FULL);
    uint32_t e = prev;
    if (prev > (kPend | pos)) {
      e = kSlot | slot;
      if (prev != 0xFFFFFFFFu) B.lostto[prev & ~kTagMask] = kPend | pos;
    }
    B.ent[pos] = e;
  }
  B.gsrc[pos] = static_cast<int32_t>(g);
}

// Floyd's subset algorithm for one destination with k > 32 slots, by one wave (lane l owns slots
// l, l + 64, ...).  Slot s draws t_s in [0, j_s], j_s = deg - k + s, and takes t_s unless an
// earlier slot holds that position, else j_s.  Settled without walking the slots one by one:
// an earlier slot holds t_s exactly if (a) an earlier slot drew the same value - whether that slot
// kept it or not, the value was in the set by then - or (b) t_s is the j of an earlier slot q (only
// q = t_s - (deg - k) can be) and slot q took its j, i.e. was itself refused.  (a) needs no other
// slot's outcome; (b) refers to one earlier slot.  So every slot is refused outright, accepted
// outright, or "as slot q": chains of such references are shortcut by pointer jumping, at most
// log2 k + 1 passes.  `draws` keeps the t_s, `picks` the states and in the end the positions p_s
// (both LDS, k entries, private to the wave).
__device__ __forceinline__ void floyd_positions(const Launch& P, const BatchCtx& B, uint32_t v, uint32_t deg,
                                                uint32_t k, uint32_t* picks, uint32_t* draws) {
  constexpr uint32_t kKnown = 0x80000000u, kRefused = 0x40000000u, kRefMask = 0x3FFFFFFFu;
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t j0 = deg - k;
  for (uint32_t s = lane; s < k; s += 64u) {
    const uint32_t w = philox_word(v, static_cast<uint32_t>(P.h), s >> 2, B.key0, B.key1, s & 3u);
    draws[s] = __umulhi(w, j0 + s + 1u);  // index in [0, j_s]
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  const uint4* draws4 = reinterpret_cast<const uint4*>(draws);
  for (uint32_t s0 = 0; s0 < k; s0 += 64u) {
    const uint32_t s = s0 + lane;
    const bool active = s < k;
    const uint32_t t = active ? draws[s] : 0u;
    bool dup = false;
    const uint32_t upto = s0 + 64u < k ? s0 + 64u : k;
    // every lane reads the same four draws at a time (a broadcast read); entries at or beyond s
    // are masked out, so the read may run past k inside the array
#pragma unroll 4
    for (uint32_t q = 0; q + 1u < upto; q += 4u) {
      const uint4 x = draws4[q >> 2];
      dup = dup | ((q < s) & (x.x == t)) | ((q + 1u < s) & (x.y == t)) | ((q + 2u < s) & (x.z == t)) |
            ((q + 3u < s) & (x.w == t));
    }
    const bool refers = !dup && t >= j0 && t - j0 < s;
    if (active) picks[s] = dup ? (kKnown | kRefused) : (refers ? t - j0 : kKnown);
  }
  for (;;) {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    bool open = false;
    for (uint32_t s = lane; s < k; s += 64u) {
      const uint32_t st = picks[s];
      if ((st & kKnown) == 0u) {
        // as slot q: take its outcome if it has one, else refer to what it refers to (a word is read
        // and written whole, and a state only ever moves forward along its chain, so the order in
        // which lanes get here does not matter)
        const uint32_t sq = picks[st & kRefMask];
        picks[s] = (sq & kKnown) ? sq : (sq & kRefMask);
        open = open || (sq & kKnown) == 0u;
      }
    }
    if (__ballot(open) == 0ull) break;
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  for (uint32_t s = lane; s < k; s += 64u) picks[s] = (picks[s] & kRefused) ? j0 + s : draws[s];
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

template <bool INSERT>
__global__ void __launch_bounds__(kThreads) k_sample_wide(const Launch P) {
  extern __shared__ __align__(16) uint32_t wide_lds[];
  const BatchCtx& B = P.b[batch_of_block(P)];
  if (__any(status_of(B, P.L) != 0)) return;  // whole waves only: the lanes below cooperate
  const int n = static_cast<int>(B.counts[P.h]);
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  uint32_t* draws = wide_lds + 2 * wave * wide_lds_words(P.d);
  uint32_t* picks = draws + wide_lds_words(P.d);
  const int waves_total = blocks_per_batch(P) * (kThreads / 64);
  int per = (n + waves_total - 1) / waves_total;  // destinations per wave and turn
  per = per < 1 ? 1 : (per > kWideRows ? kWideRows : per);
  for (int i0 = (block_in_batch(P) * (kThreads / 64) + wave) * per; i0 < n; i0 += waves_total * per) {
    const int il = i0 + lane;
    uint32_t v_l = 0, deg_l = 0, k_l = 0, base_l = 0, a_lo = 0, a_hi = 0;
    if (lane < per && il < n) {
      v_l = static_cast<uint32_t>(B.node_ids[il]);
      const int64_t a = B.rowstart[il];
      a_lo = static_cast<uint32_t>(a);
      a_hi = static_cast<uint32_t>(static_cast<uint64_t>(a) >> 32);
      deg_l = static_cast<uint32_t>(B.rowdeg[il]);
      k_l = static_cast<uint32_t>(B.rowk[il]);
      base_l = static_cast<uint32_t>(B.tile_sums[il / kTileRows]) + static_cast<uint32_t>(B.rowoff[il]);
      B.blk_indptr[il] = static_cast<int32_t>(base_l);
    }
    const int rows = n - i0 < per ? n - i0 : per;
    static_assert(kWideRows % 4 == 0 && kWideRows <= 64, "rows are walked four at a time, a lane per row record");
    for (int r0 = 0; r0 < rows; r0 += 4) {  // lanes beyond the last row hold k = 0
      uint32_t g[4], pos[4];
      bool on[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int r = r0 + u;
        const int64_t a = static_cast<int64_t>((static_cast<uint64_t>(__shfl(a_hi, r, 64)) << 32) | __shfl(a_lo, r, 64));
        const uint32_t deg = __shfl(deg_l, r, 64);
        const uint32_t k = __shfl(k_l, r, 64);
        pos[u] = __shfl(base_l, r, 64) + static_cast<uint32_t>(lane);
        on[u] = deg == k && k <= 64u && static_cast<uint32_t>(lane) < k;
        g[u] = on[u] ? static_cast<uint32_t>(__builtin_nontemporal_load(P.indices + (a + lane))) : 0u;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (on[u]) wide_emit<INSERT>(P, B, g[u], pos[u]);
    }
    for (int r = 0; r < rows; ++r) {
      const uint32_t v = __shfl(v_l, r, 64);
      const int64_t a = static_cast<int64_t>((static_cast<uint64_t>(__shfl(a_hi, r, 64)) << 32) | __shfl(a_lo, r, 64));
      const uint32_t deg = __shfl(deg_l, r, 64);
      const uint32_t k = __shfl(k_l, r, 64);
      const uint32_t base = __shfl(base_l, r, 64);
      const bool floyd = deg > k;  // only then are positions drawn (k = fanout <= SMFG_MAX_WIDE_FANOUT)
      if (!floyd && k <= 64u) continue;  // done above
      if (!floyd) {  // the whole row in CSR order; every read of a turn leaves before a result is used
        for (uint32_t s0 = static_cast<uint32_t>(lane); s0 < k; s0 += 64u * kWideCopyRounds) {
          uint32_t gv[kWideCopyRounds];
#pragma unroll
          for (int u = 0; u < kWideCopyRounds; ++u) {
            const uint32_t sl = s0 + 64u * u;
            gv[u] = sl < k ? static_cast<uint32_t>(__builtin_nontemporal_load(P.indices + (a + sl))) : 0u;
          }
#pragma unroll
          for (int u = 0; u < kWideCopyRounds; ++u) {
            const uint32_t sl = s0 + 64u * u;
            if (sl < k) wide_emit<INSERT>(P, B, gv[u], base + sl);
          }
        }
        continue;
      }
      floyd_positions(P, B, v, deg, k, picks, draws);
      for (uint32_t s0 = 0; s0 < k; s0 += 128) {  // two rounds at a time
        const uint32_t sa = s0 + static_cast<uint32_t>(lane), sb = sa + 64u;
        uint32_t ga = 0, gb = 0;
        if (sa < k) ga = static_cast<uint32_t>(__builtin_nontemporal_load(P.indices + (a + picks[sa])));
        if (sb < k) gb = static_cast<uint32_t>(__builtin_nontemporal_load(P.indices + (a + picks[sb])));
        if (sa < k) wide_emit<INSERT>(P, B, ga, base + sa);
        if (sb < k) wide_emit<INSERT>(P, B, gb, base + sb);
      }
      // the next row's draws must not overwrite picks a lane has yet to read
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
  }
}

// ---- partition strategy over exact offsets ----------------------------------------------------
// The records of a hop as one stream: element e < n is known node e, element n + pos the sample
// at position pos.  A flat block owns kFlatBlock consecutive elements.
__device__ __forceinline__ unsigned long long flat_record(const BatchCtx& B, uint32_t e, uint32_t n) {
  if (e < n) return (static_cast<unsigned long long>(static_cast<uint32_t>(B.node_ids[e])) << 32) | e;
  const uint32_t pos = e - n;
  return (static_cast<unsigned long long>(static_cast<uint32_t>(B.gsrc[pos])) << 32) | (kPend | pos);
}

// Per flat block: records per bucket -> hist row.
__global__ void __launch_bounds__(kThreads) k_hist_flat(const Launch P) {
  __shared__ uint32_t hist[1 << kPartMaxLgB];
  const BatchCtx& B = P.b[batch_of_block(P)];
  if (block_has_status(B, P.L)) return;
  const uint32_t n = static_cast<uint32_t>(B.counts[P.h]);
  const uint32_t total = n + static_cast<uint32_t>(B.counts[P.L + 1 + P.h]);
  const int lgB = hop_shape(P, B).lgB;
  const int nB = 1 << lgB;
  const int blocks = hop_blocks(P, B);
  for (int blk = block_in_batch(P); blk < blocks; blk += blocks_per_batch(P)) {
    __syncthreads();
    for (int b = threadIdx.x; b < nB; b += kThreads) hist[b] = 0u;
    __syncthreads();
    const uint32_t e0 = static_cast<uint32_t>(blk) * kFlatBlock;
    constexpr int U = 8;
    for (uint32_t c0 = e0; c0 < e0 + kFlatBlock && c0 < total; c0 += kThreads * U) {
      unsigned long long r[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t e = c0 + u * kThreads + threadIdx.x;
        r[u] = e < total ? flat_record(B, e, n) : kEmpty;
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (r[u] != kEmpty) atomicAdd(&hist[part_bucket(static_cast<uint32_t>(r[u] >> 32), lgB)], 1u);
    }
    __syncthreads();
    uint32_t* out = B.hist + static_cast<size_t>(blk) * nB;
    for (int b = threadIdx.x; b < nB; b += kThreads) out[b] = hist[b];
  }
}

// Records of a flat block -> their buckets, in the staged rounds of k_scatter.
__global__ void __launch_bounds__(kThreads) k_scatter_flat(const Launch P) {
  __shared__ StageLds L;
  const BatchCtx& B = P.b[batch_of_block(P)];
  if (block_has_status(B, P.L)) return;
  const uint32_t n = static_cast<uint32_t>(B.counts[P.h]);
  const uint32_t total_e = n + static_cast<uint32_t>(B.counts[P.L + 1 + P.h]);
  const int lgB = hop_shape(P, B).lgB;
  const int nB = 1 << lgB;
  const int blocks = hop_blocks(P, B);
  for (int blk = block_in_batch(P); blk < blocks; blk += blocks_per_batch(P)) {
    __syncthreads();  // the previous flat block is done with the LDS arrays
    stage_bucket_bases(L, B, nB, blk);
    const uint32_t e0 = static_cast<uint32_t>(blk) * kFlatBlock;
    for (uint32_t c0 = e0; c0 < e0 + kFlatBlock && c0 < total_e; c0 += kScatterRound) {
      unsigned long long r[kScatterPer];
#pragma unroll
      for (int u = 0; u < kScatterPer; ++u) {
        const uint32_t e = c0 + u * kThreads + threadIdx.x;
        r[u] = e < total_e ? flat_record(B, e, n) : kEmpty;
      }
      stage_round(L, nB, r, [&](uint32_t node) { return part_bucket(node, lgB); }, B.rec);
    }
  }
}

// flag_flat for the entries dedup_buckets leaves (a sample whose gsrc entry still is a node id is a
// first appearance).  Instead of a rank per sample, every group of 64 consecutive samples gets one
// 16-byte record: the 64 first-appearance bits and the number of new nodes of the tile before the
// group.  For a hop of millions of samples that is about a megabyte, which stays in the L2, so the
// lookups of the samples that repeat a node (scattered over the hop) do not go to memory.
__global__ void __launch_bounds__(kThreads) k_flag_flat_part(const Launch P) {
  __shared__ unsigned long long lds[kThreads / 64];
  const BatchCtx& B = P.b[batch_of_block(P)];
  if (block_has_status(B, P.L)) return;
  const uint32_t E = static_cast<uint32_t>(B.counts[P.L + 1 + P.h]);
  const uint32_t tiles = (E + kWideTile - 1) / kWideTile;
  const int sub = threadIdx.x & 15;  // 16 threads x 4 samples = one group of 64
  for (uint32_t tile = block_in_batch(P); tile < tiles; tile += blocks_per_batch(P)) {
    const uint32_t p0 = tile * kWideTile + threadIdx.x * 4;
    uint32_t nibble = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint32_t pos = p0 + u;
      if (pos < E && (static_cast<uint32_t>(B.gsrc[pos]) & kResolved) == 0u) nibble |= 1u << u;
    }
    unsigned long long total;
    const uint32_t pre = static_cast<uint32_t>(block_exscan(__popc(nibble), lds, total));
    // the 16 nibbles of a group, OR-ed over its lanes
    unsigned long long bits = static_cast<unsigned long long>(nibble) << (4 * sub);
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) bits |= __shfl_xor(bits, o, 64);
    if (sub == 0 && p0 < E)
      B.grp[p0 >> 6] = make_uint4(static_cast<uint32_t>(bits), static_cast<uint32_t>(bits >> 32), pre, 0u);
    if (threadIdx.x == 0) B.stile_sums[tile] = total;
    __syncthreads();
  }
}

// New nodes of the hop before the sample at position q (a first appearance or not).
__device__ __forceinline__ uint32_t flat_rank(const uint4 g, uint32_t tile_before, uint32_t q) {
  const unsigned long long bits = (static_cast<unsigned long long>(g.y) << 32) | g.x;
  return tile_before + g.z + __popcll(bits & ((1ull << (q & 63u)) - 1ull));
}

// assemble_flat for those entries.
__global__ void __launch_bounds__(kThreads) k_assemble_flat_part(const Launch P) {
  const BatchCtx& B = P.b[batch_of_block(P)];
  if (status_of(B, P.L) != 0) return;
  const uint32_t n = static_cast<uint32_t>(B.counts[P.h]);
  const uint32_t E = static_cast<uint32_t>(B.counts[P.L + 1 + P.h]);
  const uint32_t tiles = (E + kWideTile - 1) / kWideTile;
  for (uint32_t tile = block_in_batch(P); tile < tiles; tile += blocks_per_batch(P)) {
    const uint32_t tpre = static_cast<uint32_t>(B.stile_sums[tile]);
    const uint32_t p0 = tile * kWideTile + threadIdx.x * 4;
    if (p0 >= E) continue;
    const uint4 own = B.grp[p0 >> 6];  // the thread's four samples share a group
    uint32_t e[4], q[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint32_t pos = p0 + u;
      e[u] = pos < E ? static_cast<uint32_t>(B.gsrc[pos]) : kResolved;
      q[u] = (e[u] & kPointer) == kPointer ? (e[u] & ~kPointer) : p0;
    }
    // what the pointers name is fetched for all four samples before any is used
    uint4 qg[4];
    uint32_t qtile[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      qg[u] = B.grp[q[u] >> 6];
      qtile[u] = static_cast<uint32_t>(B.stile_sums[q[u] / kWideTile]);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const uint32_t pos = p0 + u;
      if (pos >= E) continue;
      uint32_t local;
      if ((e[u] & kResolved) == 0u) {  // first appearance
        local = n + flat_rank(own, tpre, pos);
        B.node_ids[local] = static_cast<int32_t>(e[u]);
      } else if ((e[u] & kPointer) == kPointer) {
        local = n + flat_rank(qg[u], qtile[u], q[u]);  // a pointer always names a first appearance
      } else {
        local = e[u] & ~kPointer;
      }
      B.blk_indices[pos] = static_cast<int32_t>(local);
    }
  }
}

// ---- table strategy over exact offsets ---------------------------------------------------------
// Flat over the samples: first appearances, their in-tile ranks, per-tile totals.
__global__ void __launch_bounds__(kThreads) k_flag_flat(const Launch P) {
  __shared__ unsigned long long lds[kThreads / 64];
  const BatchCtx& B = P.b[batch_of_block(P)];
  if (block_has_status(B, P.L)) {
    for (int64_t q = static_cast<int64_t>(block_in_batch(P)) * kThreads + threadIdx.x; q < B.lostto_entries;
         q += static_cast<int64_t>(blocks_per_batch(P)) * kThreads)
      B.lostto[q] = 0u;
    return;
  }
  const uint32_t E = static_cast<uint32_t>(B.counts[P.L + 1 + P.h]);
  const uint32_t tiles = (E + kWideTile - 1) / kWideTile;
  for (uint32_t tile = block_in_batch(P); tile < tiles; tile += blocks_per_batch(P)) {
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
  const BatchCtx& B = P.b[batch_of_block(P)];
  if (block_has_status(B, P.L)) return;
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
  const BatchCtx& B = P.b[batch_of_block(P)];
  if (status_of(B, P.L) != 0) return;
  const uint32_t n = static_cast<uint32_t>(B.counts[P.h]);
  const uint32_t E = static_cast<uint32_t>(B.counts[P.L + 1 + P.h]);
  const bool last = P.h == P.L - 1;
  const uint32_t tiles = (E + kWideTile - 1) / kWideTile;
  for (uint32_t tile = block_in_batch(P); tile < tiles; tile += blocks_per_batch(P)) {
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
          const uint32_t nxt = eq & ~kTagMask;  // strictly smaller position, or the scratch was disturbed
          if (nxt >= q) {
            set_status(B, P.L, SMFG_ST_INTERNAL);
            local = 0u;
            break;
          }
          q = nxt;
        }
      }
      B.blk_indices[pos] = static_cast<int32_t>(local);
    }
  }
}

}  // namespace smfg_dev

#endif  // SMFG_KERNELS_WIDE_H_

// libsmfg partition strategy for the dedup of a hop (fanouts up to SMFG_MAX_FANOUT).
//
// Procedure OneHopMFG keeps one map from global to local ids and gives a node its local id at the
// first encounter.  Here the map never exists as one structure in memory.  Per hop:
//   sample_hist   draws the neighbours (as k_sample_insert does) into gsrc and counts, per block
//                 of destinations, how many records fall into each hash bucket; a record is
//                 (node, value): one per known node (value = its local id) and one per sample
//                 (value = tag | scan position);
//   scan_hist     turns the counts of a bucket over the row blocks into offsets, bucket sizes;
//   scatter       moves the records into their buckets (one contiguous range of `rec` each);
//   split_buckets only for hops with more records than 1024 buckets of the target size hold (such
//                 a hop starts with fewer, larger buckets, see part_levels): one block per bucket
//                 orders the bucket's records by further hash bits into sub-buckets (`rec2`),
//                 which then take the place of the buckets;
//   dedup_buckets one block per bucket builds a hash table of the bucket's nodes in LDS, keeping
//                 the smallest value per node (a known node's local id always wins, else the
//                 earliest scan position).  A sample that is its node's first appearance keeps
//                 its gsrc entry (the node id, bit 31 clear); every other sample's entry is
//                 overwritten with kResolved | final local id (known node) or kPointer | position
//                 of the first appearance.  In the outer hops most samples are first appearances,
//                 so few entries are rewritten.
// flag_rows_part / scan_tiles / assemble_part then number the first appearances in scan order,
// exactly the ids the serial first-encounter rule gives.  Which thread inserts first never
// matters: only minima are kept.  All global traffic but the neighbour reads and those scattered
// 4-byte rewrites is streaming, and there are no global atomics.
#ifndef SMFG_KERNELS_PART_H_
#define SMFG_KERNELS_PART_H_

#include "device_common.h"
#include "kernels_fast.h"

namespace smfg_dev {

constexpr int kPartMaxLgB = 10;                     // at most 1024 buckets per hop and level ...
constexpr int kPartMaxLg2 = 10;                     // ... each split into at most 1024 sub-buckets
constexpr int kPartTableLg = 12;                    // LDS table: 4096 slots of 8 bytes
constexpr uint32_t kPartSlots = 1u << kPartTableLg;
constexpr int kPartBucketRecords = 2048;            // buckets are sized for at most this many on average
constexpr int64_t kPartMaxRecords = static_cast<int64_t>(kPartBucketRecords) << (kPartMaxLgB + kPartMaxLg2);
constexpr uint32_t kPartHash = 0x9E3779B1u;         // odd: node -> node * kPartHash is a bijection on 32 bits
constexpr uint32_t kResolved = 0x80000000u;         // gsrc entry: low 30 bits = final local id of a known node
constexpr uint32_t kPointer = 0xC0000000u;          // gsrc entry: low 30 bits = position of the first appearance

__device__ __forceinline__ uint32_t part_bucket(uint32_t node, int lgB) {
  return lgB == 0 ? 0u : (node * kPartHash) >> (32 - lgB);
}

// Buckets (2^lgB) and sub-buckets per bucket (2^lg2) of the current hop.  Padded positions: as the
// host planned them from the worst case.  Exact offsets (P.flat): the worst case of a hop that
// takes whole neighbourhoods is far above what a batch draws, so the shape follows the hop's
// actual record count (known nodes + samples, both final before the first kernel that asks) and
// the host's figures only bound it; grids are sized for the bound and surplus blocks leave.
constexpr int kFlatBlock = 8192;  // stream elements (known nodes, then samples) per block of the flat kernels
struct HopShape {
  int lgB, lg2;
};
// 2^lg buckets in all: one level up to 2^kPartMaxLgB of them; beyond that two levels, the first of
// only 2^kPartSplitLgB buckets (more if the second would exceed 2^kPartMaxLg2), so that what a
// block sends to a bucket per round is a run of a sector or more and the lines it is filling stay
// in the L2 until they are full.
constexpr int kPartSplitLgB = 7;
__host__ __device__ inline void part_levels(int lg, int& lgB, int& lg2) {
  if (lg <= kPartMaxLgB) {
    lgB = lg;
    lg2 = 0;
    return;
  }
  lgB = lg - kPartMaxLg2 > kPartSplitLgB ? lg - kPartMaxLg2 : kPartSplitLgB;
  lg2 = lg - lgB;
}
__device__ __forceinline__ HopShape hop_shape(const Launch& P, const BatchCtx& B) {
  HopShape s{P.lgB, P.lg2};
  if (P.flat) {
    const long long records = B.counts[P.h] + B.counts[P.L + 1 + P.h];
    int lg = 0;
    while (lg < P.lgB + P.lg2 && (records >> lg) > kPartBucketRecords) ++lg;
    part_levels(lg, s.lgB, s.lg2);
  }
  return s;
}
// Row blocks (padded positions) or flat blocks (exact offsets) of the current hop.
__device__ __forceinline__ int hop_blocks(const Launch& P, const BatchCtx& B) {
  if (P.flat) return static_cast<int>((B.counts[P.h] + B.counts[P.L + 1 + P.h] + kFlatBlock - 1) / kFlatBlock);
  return static_cast<int>((B.counts[P.h] + P.block_rows - 1) / P.block_rows);
}

// counts <- (n_0, 0, ..., status 0); node_ids[0, n_0) <- seeds; labels of the seeds.  Seeds are
// range-checked by the first hop's k_sample_hist, which runs after the status word is zero.
__global__ void __launch_bounds__(kThreads) k_begin(const Launch P) {
  const BatchCtx& B = P.b[batch_of_block(P)];
  if (block_in_batch(P) == 0) {
    const int m = 2 * P.L + 2;
    for (int q = threadIdx.x; q < m; q += kThreads) B.counts[q] = (q == 0) ? B.num_seeds : 0;
  }
  const int stride = blocks_per_batch(P) * kThreads;
  for (int i = block_in_batch(P) * kThreads + threadIdx.x; i < B.num_seeds; i += stride) {
    const int32_t v = B.seeds[i];
    B.node_ids[i] = v;
    if (B.labels && v >= 0 && static_cast<int64_t>(v) < P.num_nodes) copy_label(P, B, i, v);
  }
}

// Samples of the block's destinations -> gsrc, rowk; per-bucket record counts -> hist row.
__global__ void __launch_bounds__(kThreads) k_sample_hist(const Launch P) {
  __shared__ uint32_t hist[1 << kPartMaxLgB];
  const BatchCtx& B = P.b[batch_of_block(P)];
  const int blk = block_in_batch(P);
  if (block_has_status(B, P.L)) return;
  const int n = static_cast<int>(B.counts[P.h]);
  const int r0 = blk * P.block_rows;
  if (r0 >= n) return;
  const int r1 = r0 + P.block_rows < n ? r0 + P.block_rows : n;
  const int nB = 1 << P.lgB;
  for (int b = threadIdx.x; b < nB; b += kThreads) hist[b] = 0u;
  __syncthreads();
  const LaneGroups G(P.d);
  for (int i0 = r0; i0 < r1; i0 += G.per_block) {
    const int i = i0 + G.row_in_block;
    bool row = G.lane_used && i < r1;
    if (P.h == 0 && row) {  // the seeds are caller data: none may index the graph unchecked
      const int32_t seed = B.node_ids[i];
      if (seed < 0 || static_cast<int64_t>(seed) >= P.num_nodes) {
        set_status(B, P.L, SMFG_ST_SEED_OUT_OF_RANGE);
        row = false;
      }
    }
    uint32_t v, k, g;
    if (draw_neighbour(P, B, G, i, row, v, k, g)) {
      B.gsrc[static_cast<uint32_t>(i) * static_cast<uint32_t>(G.d) + static_cast<uint32_t>(G.s)] = static_cast<int32_t>(g);
      atomicAdd(&hist[part_bucket(g, P.lgB)], 1u);
    }
    if (row && G.s == 0) {
      B.rowk[i] = static_cast<int32_t>(k);
      atomicAdd(&hist[part_bucket(v, P.lgB)], 1u);  // the destination itself, a known node
    }
  }
  __syncthreads();
  uint32_t* out = B.hist + static_cast<size_t>(blk) * nB;
  for (int b = threadIdx.x; b < nB; b += kThreads) out[b] = hist[b];
}

// Counts of a bucket over the row blocks -> exclusive offsets, and the bucket's size.  A thread
// block takes kScanCols buckets; kScanSegs threads share a bucket, each a contiguous range of the
// row blocks (sum, then the ranges' exclusive scan in LDS, then the offsets).
constexpr int kScanCols = 32;
constexpr int kScanSegs = kThreads / kScanCols;
__global__ void __launch_bounds__(kThreads) k_scan_hist(const Launch P) {
  __shared__ uint32_t part[kScanSegs][kScanCols];
  const BatchCtx& B = P.b[batch_of_block(P)];
  if (block_has_status(B, P.L)) return;
  const int blocks = hop_blocks(P, B);
  const int nB = 1 << hop_shape(P, B).lgB;
  const int c = threadIdx.x % kScanCols, seg = threadIdx.x / kScanCols;
  const int b = block_in_batch(P) * kScanCols + c;
  const int per = (blocks + kScanSegs - 1) / kScanSegs;
  const int j0 = seg * per < blocks ? seg * per : blocks;
  const int j1 = j0 + per < blocks ? j0 + per : blocks;
  uint32_t* col = B.hist + (b < nB ? b : 0);
  uint32_t sum = 0;
  if (b < nB) {
    int j = j0;
    constexpr int U = 8;
    for (; j + U <= j1; j += U) {
      uint32_t t[U];
#pragma unroll
      for (int u = 0; u < U; ++u) t[u] = col[static_cast<size_t>(j + u) * nB];
#pragma unroll
      for (int u = 0; u < U; ++u) sum += t[u];
    }
    for (; j < j1; ++j) sum += col[static_cast<size_t>(j) * nB];
  }
  part[seg][c] = sum;
  __syncthreads();
  if (b >= nB) return;
  uint32_t run = 0, total = 0;
#pragma unroll
  for (int q = 0; q < kScanSegs; ++q) {
    const uint32_t v = part[q][c];
    if (q < seg) run += v;
    total += v;
  }
  if (seg == 0) B.bstart[nB + 1 + b] = total;  // bucket size
  int j = j0;
  constexpr int U = 8;
  for (; j + U <= j1; j += U) {
    uint32_t t[U];
#pragma unroll
    for (int u = 0; u < U; ++u) t[u] = col[static_cast<size_t>(j + u) * nB];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      col[static_cast<size_t>(j + u) * nB] = run;
      run += t[u];
    }
  }
  for (; j < j1; ++j) {
    const uint32_t t = col[static_cast<size_t>(j) * nB];
    col[static_cast<size_t>(j) * nB] = run;
    run += t;
  }
}

// ---- records to buckets, in rounds staged through LDS ------------------------------------------
// A block that moves records to buckets takes them in rounds of kScatterRound (kScatterPer per
// thread): the round's records are counted per bucket (each gets its rank within its bucket by an
// LDS atomicAdd), the counts are scanned, the records are put in bucket order into a staging
// array in LDS and written out in that order, so that what a bucket receives from a round leaves
// as one run of consecutive addresses.  gbase[b] is where the block's next record of bucket b goes.
constexpr int kScatterPer = 8;
constexpr int kScatterRound = kScatterPer * kThreads;
constexpr int kStageBuckets = 1 << (kPartMaxLgB > kPartMaxLg2 ? kPartMaxLgB : kPartMaxLg2);
constexpr int kStagePer = kStageBuckets / kThreads;  // buckets per thread in the block scans

struct StageLds {
  uint32_t gbase[kStageBuckets];
  uint32_t cnt[kStageBuckets];
  uint32_t lstart[kStageBuckets];
  unsigned long long stage[kScatterRound];
  unsigned long long scan[kThreads / 64];
};

// gbase[b] <- first + exclusive scan of sizes[b] (+ offs[b] if given), b < nb; returns the total
// of the sizes.  `write_starts`, if given, also receives first + the exclusive scan.
template <typename SizeOf, typename OffOf, typename StartTo>
__device__ __forceinline__ uint32_t stage_set_bases(StageLds& L, int nb, uint32_t first, SizeOf size_of, OffOf off_of,
                                                     StartTo start_to) {
  uint32_t sz[kStagePer];
  uint32_t mine = 0;
#pragma unroll
  for (int u = 0; u < kStagePer; ++u) {
    const int b = threadIdx.x * kStagePer + u;
    sz[u] = b < nb ? size_of(b) : 0u;
    mine += sz[u];
  }
  unsigned long long total;
  uint32_t pre = first + static_cast<uint32_t>(block_exscan(mine, L.scan, total));
#pragma unroll
  for (int u = 0; u < kStagePer; ++u) {
    const int b = threadIdx.x * kStagePer + u;
    if (b < nb) {
      L.gbase[b] = pre + off_of(b);
      start_to(b, pre);
    }
    pre += sz[u];
  }
  __syncthreads();
  return static_cast<uint32_t>(total);
}

// One round: r[u] are this thread's records (kEmpty = none), bucket_of maps a node to its bucket
// in [0, nb).  All threads of the block call.
template <typename BucketOf>
__device__ __forceinline__ void stage_round(StageLds& L, int nb, const unsigned long long (&r)[kScatterPer],
                                            BucketOf bucket_of, uint64_t* __restrict__ dst) {
  __syncthreads();  // the previous round has been written out
  for (int b = threadIdx.x; b < nb; b += kThreads) L.cnt[b] = 0u;
  __syncthreads();
  uint32_t bk[kScatterPer], rk[kScatterPer];
#pragma unroll
  for (int u = 0; u < kScatterPer; ++u) {
    bk[u] = 0u;
    rk[u] = 0u;
    if (r[u] != kEmpty) {
      bk[u] = bucket_of(static_cast<uint32_t>(r[u] >> 32));
      rk[u] = atomicAdd(&L.cnt[bk[u]], 1u);
    }
  }
  __syncthreads();
  uint32_t c[kStagePer];
  uint32_t mine = 0;
#pragma unroll
  for (int u = 0; u < kStagePer; ++u) {
    const int b = threadIdx.x * kStagePer + u;
    c[u] = b < nb ? L.cnt[b] : 0u;
    mine += c[u];
  }
  unsigned long long total;
  uint32_t pre = static_cast<uint32_t>(block_exscan(mine, L.scan, total));
#pragma unroll
  for (int u = 0; u < kStagePer; ++u) {
    const int b = threadIdx.x * kStagePer + u;
    if (b < nb) L.lstart[b] = pre;
    pre += c[u];
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < kScatterPer; ++u)
    if (r[u] != kEmpty) L.stage[L.lstart[bk[u]] + rk[u]] = r[u];
  __syncthreads();
  const uint32_t staged = static_cast<uint32_t>(total);
  for (uint32_t t = threadIdx.x; t < staged; t += kThreads) {
    const unsigned long long x = L.stage[t];
    const uint32_t b = bucket_of(static_cast<uint32_t>(x >> 32));
    dst[L.gbase[b] + (t - L.lstart[b])] = x;
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < kStagePer; ++u) {
    const int b = threadIdx.x * kStagePer + u;
    if (b < nb) L.gbase[b] += c[u];
  }
}

// The first record of every bucket (exclusive scan of the bucket sizes k_scan_hist left) plus this
// block's offset within each bucket; block 0 also stores the bucket starts for k_dedup_buckets.
__device__ __forceinline__ void stage_bucket_bases(StageLds& L, const BatchCtx& B, int nB, int blk) {
  const uint32_t* offs = B.hist + static_cast<size_t>(blk) * nB;
  const uint32_t total = stage_set_bases(
      L, nB, 0u, [&](int b) { return B.bstart[nB + 1 + b]; }, [&](int b) { return offs[b]; },
      [&](int b, uint32_t start) {
        if (blk == 0) B.bstart[b] = start;
      });
  if (blk == 0 && threadIdx.x == 0) B.bstart[nB] = total;
}

// Records of the block's destinations (its known nodes first, then its samples in position
// order) -> their buckets.
__global__ void __launch_bounds__(kThreads) k_scatter(const Launch P) {
  __shared__ StageLds L;
  const BatchCtx& B = P.b[batch_of_block(P)];
  if (block_has_status(B, P.L)) return;
  const int blk = block_in_batch(P);
  const int n = static_cast<int>(B.counts[P.h]);
  const int r0 = blk * P.block_rows;
  if (r0 >= n) return;
  const int r1 = r0 + P.block_rows < n ? r0 + P.block_rows : n;
  const int nB = 1 << P.lgB;
  stage_bucket_bases(L, B, nB, blk);
  const uint32_t d = static_cast<uint32_t>(P.d);
  const DivD div(d);
  const uint32_t known = static_cast<uint32_t>(r1 - r0);
  const uint32_t pos0 = static_cast<uint32_t>(r0) * d;
  const uint32_t stream = known + known * d;  // known nodes, then the padded sample positions
  for (uint32_t c0 = 0; c0 < stream; c0 += kScatterRound) {
    unsigned long long rec[kScatterPer];
    uint32_t k[kScatterPer], sl[kScatterPer], g[kScatterPer];
#pragma unroll
    for (int u = 0; u < kScatterPer; ++u) {
      const uint32_t e = c0 + u * kThreads + threadIdx.x;
      k[u] = 0u;
      sl[u] = 0u;
      g[u] = 0u;
      if (e < known) {
        g[u] = static_cast<uint32_t>(B.node_ids[r0 + static_cast<int>(e)]);
        k[u] = 1u;
      } else if (e < stream) {
        uint32_t r;
        div.split(e - known, r, sl[u]);
        k[u] = static_cast<uint32_t>(B.rowk[r0 + static_cast<int>(r)]);
        g[u] = static_cast<uint32_t>(B.gsrc[pos0 + (e - known)]);
      }
    }
#pragma unroll
    for (int u = 0; u < kScatterPer; ++u) {
      const uint32_t e = c0 + u * kThreads + threadIdx.x;
      rec[u] = kEmpty;
      if (e < stream && sl[u] < k[u]) {
        // a known node (destination i has local id i), or a sample: tag | position
        const uint32_t val = e < known ? static_cast<uint32_t>(r0) + e : (kPend | (pos0 + (e - known)));
        rec[u] = (static_cast<unsigned long long>(g[u]) << 32) | val;
      }
    }
    stage_round(L, nB, rec, [&](uint32_t node) { return part_bucket(node, P.lgB); }, B.rec);
  }
}

// Grid-stride over the buckets: a bucket's records, ordered by the lg2 hash bits below the
// bucket's, go to the same range of rec2; the sub-buckets' first records go to bstart2.  A counting
// pass over the bucket, then the staged rounds.
__global__ void __launch_bounds__(kThreads) k_split_buckets(const Launch P) {
  __shared__ StageLds L;
  const BatchCtx& B = P.b[batch_of_block(P)];
  if (block_has_status(B, P.L)) return;
  const HopShape hs = hop_shape(P, B);
  if (hs.lg2 == 0) return;
  const uint32_t nB1 = 1u << hs.lgB;
  const int n2 = 1 << hs.lg2;
  const int shift = 32 - hs.lgB - hs.lg2;
  const uint32_t mask = static_cast<uint32_t>(n2 - 1);
  const auto sub_of = [&](uint32_t node) { return ((node * kPartHash) >> shift) & mask; };
  for (uint32_t b1 = static_cast<uint32_t>(block_in_batch(P)); b1 < nB1;
       b1 += static_cast<uint32_t>(blocks_per_batch(P))) {
    const uint32_t rec0 = B.bstart[b1];
    const uint32_t rec1 = rec0 + B.bstart[nB1 + 1 + b1];
    __syncthreads();  // the previous bucket is done with the LDS arrays
    for (int b = threadIdx.x; b < n2; b += kThreads) L.cnt[b] = 0u;
    __syncthreads();
    for (uint32_t c0 = rec0; c0 < rec1; c0 += kScatterRound) {
      unsigned long long r[kScatterPer];
#pragma unroll
      for (int u = 0; u < kScatterPer; ++u) {
        const uint32_t q = c0 + u * kThreads + threadIdx.x;
        r[u] = q < rec1 ? B.rec[q] : kEmpty;
      }
#pragma unroll
      for (int u = 0; u < kScatterPer; ++u)
        if (r[u] != kEmpty) atomicAdd(&L.cnt[sub_of(static_cast<uint32_t>(r[u] >> 32))], 1u);
    }
    __syncthreads();
    stage_set_bases(
        L, n2, rec0, [&](int b) { return L.cnt[b]; }, [](int) { return 0u; },
        [&](int b, uint32_t start) { B.bstart2[(static_cast<size_t>(b1) << hs.lg2) + b] = start; });
    if (b1 == nB1 - 1 && threadIdx.x == 0) B.bstart2[static_cast<size_t>(nB1) << hs.lg2] = rec1;
    for (uint32_t c0 = rec0; c0 < rec1; c0 += kScatterRound) {
      unsigned long long r[kScatterPer];
#pragma unroll
      for (int u = 0; u < kScatterPer; ++u) {
        const uint32_t q = c0 + u * kThreads + threadIdx.x;
        r[u] = q < rec1 ? B.rec[q] : kEmpty;
      }
      stage_round(L, n2, r, sub_of, B.rec2);
    }
  }
}

// Grid-stride over the (sub-)buckets, a block at a time.  All records of a node are in one bucket,
// so the bucket's table in LDS sees every occurrence of its nodes.  A bucket with more records than the table takes is
// handled in 2^lgR rounds, round r taking the nodes whose next lgR hash bits equal r; should a
// round still overflow (skewed bits), the bucket starts over with one more bit.  With
// 32 - lgB - lgR <= kPartTableLg bits left every node of a round has a slot of its own (the hash
// is a bijection), so the retries end.
// One record into the bucket's table: the slot of its node keeps the smallest value.  False if the
// table has no slot left.
__device__ __forceinline__ bool dedup_insert(unsigned long long* tab, unsigned long long rec, uint32_t sl) {
  const uint32_t node = static_cast<uint32_t>(rec >> 32);
  // A plain read first: a node sampled thousands of times (a hub) would otherwise queue
  // thousands of atomics on one LDS word, while most of its records only need to see that
  // a smaller value is there already.  Slots never lose their node, values only fall.
  for (uint32_t probes = 0; probes < kPartSlots; ++probes) {
    unsigned long long old = tab[sl];
    if (old == kEmpty) old = atomicCAS(&tab[sl], kEmpty, rec);
    if (old == kEmpty) return true;
    if (static_cast<uint32_t>(old >> 32) == node) {
      if (old > rec) atomicMin(&tab[sl], rec);
      return true;
    }
    sl = (sl + 1u) & (kPartSlots - 1u);
  }
  return false;
}

// What the filled table says about one record: a known node must be alone with its id; a sample
// that is not its node's smallest value learns the node's local id or the position of its first
// appearance.
__device__ __forceinline__ void dedup_settle(const Launch& P, const BatchCtx& B, const unsigned long long* tab,
                                             unsigned long long rec, uint32_t sl) {
  const uint32_t node = static_cast<uint32_t>(rec >> 32);
  const uint32_t val = static_cast<uint32_t>(rec);
  uint32_t least = 0u;
  uint32_t probes = 0;
  for (; probes < kPartSlots; ++probes) {
    const unsigned long long t = tab[sl];
    if (static_cast<uint32_t>(t >> 32) == node) {
      least = static_cast<uint32_t>(t);
      break;
    }
    sl = (sl + 1u) & (kPartSlots - 1u);
  }
  if (probes == kPartSlots) {  // every inserted node is found again
    set_status(B, P.L, SMFG_ST_INTERNAL);
    return;
  }
  if (val < kPend) {
    // a known node: two of them with one id can only be a repeated seed
    if (least != val) set_status(B, P.L, SMFG_ST_DUPLICATE_SEED);
  } else if (least != val) {
    // least < kPend: the node's final local id; else least names the position of the first
    // appearance (least == val: this sample is that first appearance, its entry stays)
    B.gsrc[val & ~kTagMask] =
        static_cast<int32_t>(least < kPend ? (kResolved | least) : (kPointer | (least & ~kTagMask)));
  }
}

__global__ void __launch_bounds__(kThreads) k_dedup_buckets(const Launch P) {
  __shared__ unsigned long long tab[kPartSlots];
  __shared__ int overflow_lds;
  const BatchCtx& B = P.b[batch_of_block(P)];
  if (block_has_status(B, P.L)) return;
  const HopShape hs = hop_shape(P, B);
  const uint32_t nB = 1u << hs.lgB;
  const uint64_t* __restrict__ recs = hs.lg2 == 0 ? B.rec : B.rec2;
  const int free_bits = 32 - hs.lgB - hs.lg2;  // hash bits below the (sub-)bucket's
  const int max_lgR = free_bits > kPartTableLg ? free_bits - kPartTableLg : 0;
  constexpr int U = 8;  // records in flight per thread
  for (uint32_t bucket = static_cast<uint32_t>(block_in_batch(P)); bucket < (nB << hs.lg2);
       bucket += static_cast<uint32_t>(blocks_per_batch(P))) {
    // the (sub-)bucket's records
    const uint32_t rec0 = hs.lg2 == 0 ? B.bstart[bucket] : B.bstart2[bucket];
    const uint32_t rec1 = hs.lg2 == 0 ? rec0 + B.bstart[nB + 1 + bucket] : B.bstart2[bucket + 1];
    const uint32_t cnt = rec1 - rec0;
    if (cnt == 0) continue;
    if (cnt <= kThreads * U && cnt <= kPartSlots / 2) {
      // the usual bucket: its records stay in registers between the two passes, and a table at most
      // half full cannot overflow
      static_assert(kThreads * U <= kPartSlots, "a resident bucket always fits its table");
      unsigned long long mine[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t r = rec0 + u * kThreads + threadIdx.x;
        mine[u] = r < rec1 ? recs[r] : kEmpty;
      }
      for (uint32_t q = threadIdx.x; q < kPartSlots; q += kThreads) tab[q] = kEmpty;
      __syncthreads();
      const int down = free_bits > kPartTableLg ? free_bits - kPartTableLg : 0;
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (mine[u] != kEmpty)
          dedup_insert(tab, mine[u], ((static_cast<uint32_t>(mine[u] >> 32) * kPartHash) >> down) & (kPartSlots - 1u));
      __syncthreads();
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (mine[u] != kEmpty)
          dedup_settle(P, B, tab, mine[u],
                       ((static_cast<uint32_t>(mine[u] >> 32) * kPartHash) >> down) & (kPartSlots - 1u));
      __syncthreads();
      continue;
    }
    int lgR = 0;
    while (lgR < max_lgR && (cnt >> lgR) > kPartSlots / 2) ++lgR;
    for (;;) {
      bool failed = false;
      const int rem = free_bits - lgR;  // hash bits below the round's
      const int down = rem > kPartTableLg ? rem - kPartTableLg : 0;
      const uint32_t rounds = 1u << lgR;
      for (uint32_t round = 0; round < rounds && !failed; ++round) {
        for (uint32_t q = threadIdx.x; q < kPartSlots; q += kThreads) tab[q] = kEmpty;
        if (threadIdx.x == 0) overflow_lds = 0;
        __syncthreads();
        for (int pass = 0; pass < 2 && !failed; ++pass) {  // insert, then settle
          for (uint32_t c0 = rec0; c0 < rec1; c0 += kThreads * U) {
            unsigned long long mine[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
              const uint32_t r = c0 + u * kThreads + threadIdx.x;
              mine[u] = r < rec1 ? recs[r] : kEmpty;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
              if (mine[u] == kEmpty) continue;
              const uint32_t hsh = static_cast<uint32_t>(mine[u] >> 32) * kPartHash;
              if (lgR != 0 && ((hsh >> rem) & (rounds - 1u)) != round) continue;
              const uint32_t sl = (hsh >> down) & (kPartSlots - 1u);
              if (pass == 0) {
                if (!dedup_insert(tab, mine[u], sl)) overflow_lds = 1;
              } else {
                dedup_settle(P, B, tab, mine[u], sl);
              }
            }
          }
          __syncthreads();
          failed = overflow_lds != 0;
        }
      }
      if (!failed) break;
      if (lgR >= max_lgR) {  // cannot overflow with a slot per node
        if (threadIdx.x == 0) set_status(B, P.L, SMFG_ST_INTERNAL);
        break;
      }
      __syncthreads();  // every thread has read the overflow word before the next attempt clears it
      ++lgR;
    }
  }
}

// flag_rows for the entries dedup_buckets leaves: a valid sample whose entry still is a node id
// (bit 31 clear) is a first appearance.  Per destination: bit mask of its first appearances; in-tile
// exclusive scan of (samples, new nodes); per-tile totals.
__global__ void __launch_bounds__(kThreads) k_flag_rows_part(const Launch P) {
  __shared__ unsigned long long lds[kThreads / 64];
  __shared__ int k_lds[kTileRows];
  __shared__ unsigned int mask_lds[kTileRows];
  const BatchCtx& B = P.b[batch_of_block(P)];
  if (block_has_status(B, P.L)) return;
  const int nblocks = blocks_per_batch(P);
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
      uint32_t e[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t idx = base + u * kThreads;
        e[u] = idx < cnt ? static_cast<uint32_t>(B.gsrc[pos0 + idx]) : kResolved;
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t idx = base + u * kThreads;
        if (idx < cnt && (e[u] & kResolved) == 0u) {
          uint32_t r, sl;
          div.split(idx, r, sl);
          if (sl < static_cast<uint32_t>(k_lds[r])) atomicOr(&mask_lds[r], 1u << sl);
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

// assemble for those entries: block indptr; block indices = final local ids; node ids of the
// first appearances.  A pointer always names a first appearance, so one lookup of that
// destination's record settles it.
__global__ void __launch_bounds__(kThreads) k_assemble_part(const Launch P) {
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
      uint32_t e[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t idx = base + u * kThreads;
        e[u] = idx < cnt ? static_cast<uint32_t>(B.gsrc[pos0 + idx]) : 0u;
      }
      // the records of the destinations that pointers name are fetched for all U samples of the
      // thread before any is used (other samples fetch the tile's first record), so the scattered
      // reads of a thread overlap
      uint32_t r[U], sl[U], q[U], qi[U];
      bool live[U], dup[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t idx = base + u * kThreads;
        r[u] = 0u;
        sl[u] = 0u;
        if (idx < cnt) div.split(idx, r[u], sl[u]);
        live[u] = idx < cnt && sl[u] < static_cast<uint32_t>(k_lds[r[u]]);
        dup[u] = live[u] && (e[u] & kPointer) == kPointer;
        q[u] = dup[u] ? (e[u] & ~kPointer) : pos0;
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
        uint32_t local;
        if ((e[u] & kResolved) == 0u) {  // first appearance: rank among the new nodes of this hop
          local = rank_lds[r[u]] + __popc(mask_lds[r[u]] & ((1u << sl[u]) - 1u));
          B.node_ids[local] = static_cast<int32_t>(e[u]);
        } else if (dup[u]) {
          const uint32_t qs = q[u] - qi[u] * d;
          local = static_cast<uint32_t>(n) + ts[u] + mn[u].y + __popc(mn[u].x & ((1u << qs) - 1u));
          if (((mn[u].x >> qs) & 1u) == 0u) {  // the named sample is not a first appearance: scratch disturbed
            set_status(B, P.L, SMFG_ST_INTERNAL);
            local = 0u;
          }
        } else {
          local = e[u] & ~kPointer;
        }
        B.blk_indices[off_lds[r[u]] + sl[u]] = static_cast<int32_t>(local);
      }
    }
  }
}

}  // namespace smfg_dev

#endif  // SMFG_KERNELS_PART_H_

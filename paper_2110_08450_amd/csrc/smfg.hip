// libsmfg: sampled mini-batch preparation on gfx950 (MI355X).  Implements include/smfg.h.
// This file is the host side (handles, validation, launch sequences); the kernels live in
// device_common.h (launch parameters, Philox, dedup table), kernels_fast.h (fanouts up to 32),
// kernels_wide.h (larger fanouts, full neighbourhoods), kernels_gather.h, kernels_aggregate.h,
// kernels_validate.h (the optional check of the input arrays).
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

#include <atomic>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

#include "smfg.h"

#include "device_common.h"
#include "kernels_aggregate.h"
#include "kernels_fast.h"
#include "kernels_gather.h"
#include "kernels_part.h"
#include "kernels_validate.h"
#include "kernels_wide.h"

// Scratch of smfg_sample_mfg_static: one copy per GPU, held until the process ends.  In host code
// this name is only a handle for hipGetSymbolAddress; the device address is looked up once per
// device (static_scratch_of) and that pointer is what the kernels and the fill receive.
static __device__ __align__(256) unsigned char scratch[SMFG_STATIC_SCRATCH_BYTES];

namespace {

using namespace smfg_dev;

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
  std::atomic<int> used{0};  // launches may be issued from several threads while a profile is open
  hipEvent_t* ev = nullptr;  // 2 per record
  int* stage = nullptr;
} g_prof;

struct StageTimer {
  int rec = -1;
  hipStream_t st;
  StageTimer(int stage, hipStream_t s) : st(s) {
    if (g_prof.level == 0) return;
    if (g_prof.level == 1 && stage != SMFG_STAGE_GATHER) return;
    const int r = g_prof.used.fetch_add(1, std::memory_order_relaxed);
    if (r >= g_prof.max_records) return;
    rec = r;
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
  g_prof.level = 0;
  g_prof.max_records = 0;
  g_prof.used.store(0);
  g_prof.ev = nullptr;
  g_prof.stage = nullptr;
}

// Typed device pointers must be multiples of their element size (atomics and vector accesses on a
// misaligned address are undefined).
inline bool misaligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

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
  int64_t slot_entries;  // capacity of the per-sample arrays
  int64_t bytes;
  // partition strategy (no dedup table) or table strategy; fixed when the workspace is planned
  bool part;
  bool flat;             // partition strategy also over exact offsets (wide fanouts): group records, row starts etc. present
  int64_t rec_entries;   // capacity of rec: known nodes + samples of a hop
  int64_t hist_entries;  // capacity of hist: row blocks x buckets of a hop
  int split_lg;          // log2 of the most sub-buckets a hop needs (0: no hop splits its buckets)
  int64_t b_table, b_slot, b_row, b_tiles, b_stiles, b_rec, b_hist, b_bstart, b_bstart2, b_grp;  // byte sizes of the slab's parts
  uint32_t table_log2;
  void* slab;
  uint64_t* table;
  uint32_t* ent;
  uint32_t* lostto;
  int32_t* gsrc;
  int32_t* rowk;
  uint2* rowmn;
  int32_t* rowoff;
  uint64_t* tile_sums;
  int64_t* rowstart;
  int32_t* rowdeg;
  uint32_t* rank;
  uint4* grp;
  uint64_t* stile_sums;
  uint64_t* rec;
  uint32_t* hist;
  uint32_t* bstart;
  uint64_t* rec2;
  uint32_t* bstart2;
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

// Blocks per batch of k_dedup_buckets.  A hop of one level: a block per bucket.  A hop of two
// levels has thousands of sub-buckets per batch: about 4096 blocks over the whole launch, each
// taking several sub-buckets one after the other - the scattered writes a sub-bucket leaves behind
// then drain while the block is busy with its next one, instead of holding the block's LDS until
// they are done.
inline unsigned dedup_blocks(int lgB, int lg2, unsigned batches) {
  if (lg2 == 0) return 1u << lgB;
  const unsigned cap = 4096u / batches > 512u ? 4096u / batches : 512u;
  return blocks_for(int64_t(1) << (lgB + lg2), 1, cap);
}
inline int64_t align256(int64_t x) { return (x + 255) & ~int64_t(255); }

// Launch shape of one hop under the partition strategy: 2^lgB hash buckets (at most 1024) sized for
// kPartBucketRecords records on average in the worst case; a hop that needs more buckets than that
// takes two levels, 2^lgB buckets each split into 2^lg2 (part_levels); destinations cut into row blocks that are whole
// multiples of what a thread block draws at once, at most 512 of them (128 in a launch of more than
// 8 batches; more for hops beyond 256 K destinations, up to 4096).
struct HopPlan {
  int lgB, lg2;
  int block_rows;
  int64_t row_blocks;
};

HopPlan plan_hop(int64_t max_rows, int d, int batches) {
  HopPlan hp;
  const int64_t records = max_rows * (1 + d);
  int lg = 0;
  while (lg < kPartMaxLgB + kPartMaxLg2 && (records >> lg) > kPartBucketRecords) ++lg;
  part_levels(lg, hp.lgB, hp.lg2);
  int64_t cap = (max_rows + 511) / 512;
  const int64_t least = batches > 8 ? 128 : 512;  // fewer, longer row blocks when many batches fill the chip anyway
  cap = cap < least ? least : (cap > 4096 ? 4096 : cap);
  hp.block_rows = (64 / d) * (kThreads / 64);
  while ((max_rows + hp.block_rows - 1) / hp.block_rows > cap) hp.block_rows *= 2;
  hp.row_blocks = (max_rows + hp.block_rows - 1) / hp.block_rows;
  if (hp.row_blocks < 1) hp.row_blocks = 1;
  return hp;
}

// Destinations each hop can have at most: seeds, then everything known so far, capped by the node
// capacity and the graph.  False if a fanout takes whole neighbourhoods (no bound without degrees).
bool hop_row_bounds(int32_t num_seeds, int32_t L, const int32_t* fanouts, int64_t num_nodes, int64_t node_capacity,
                    int64_t* rows /*[L]*/) {
  int64_t n = num_seeds < num_nodes ? num_seeds : num_nodes;
  for (int h = 0; h < L; ++h) {
    if (fanouts[h] < 0) return false;
    if (n > node_capacity) n = node_capacity;
    rows[h] = n;
    n = n + n * fanouts[h];
    if (n > num_nodes) n = num_nodes;
  }
  return true;
}

// Whether every hop of a call can take the partition strategy; if so, what it needs of a workspace.
// The environment variable SMFG_DEDUP=table makes new workspaces use the table strategy even
// where the partition strategy applies (for measuring one against the other).
bool table_forced() {
  const char* e = std::getenv("SMFG_DEDUP");
  return e && std::strcmp(e, "table") == 0;
}
// ... and SMFG_DEDUP=partition the partition strategy also for calls so small that the table
// strategy would be chosen (so that tests reach it with small inputs).
bool part_forced() {
  const char* e = std::getenv("SMFG_DEDUP");
  return e && std::strcmp(e, "partition") == 0;
}

// Calls whose largest hop stays below kPartMinRecords keep the table strategy: its four launches per
// hop cost less than the partition strategy's seven when every kernel is launch-bound anyway.
constexpr int64_t kPartMinRecords = 32768;

bool part_needs(int32_t num_seeds, int32_t L, const int32_t* fanouts, int64_t num_nodes, int64_t node_capacity,
                int64_t* rec_entries, int64_t* hist_entries, int* split_lg) {
  int64_t rows[SMFG_MAX_LAYERS];
  *rec_entries = 1;
  *hist_entries = 1;
  *split_lg = 0;
  for (int h = 0; h < L; ++h)
    if (fanouts[h] < 1 || fanouts[h] > SMFG_MAX_FANOUT) return false;
  if (!hop_row_bounds(num_seeds, L, fanouts, num_nodes, node_capacity, rows)) return false;
  for (int h = 0; h < L; ++h) {
    const int64_t records = rows[h] * (1 + fanouts[h]);
    if (records > kPartMaxRecords) return false;
    const HopPlan hp = plan_hop(rows[h], fanouts[h], 1);  // the most row blocks any launch will use
    if (records > *rec_entries) *rec_entries = records;
    // a call with fewer seeds may take one level of up to 2^kPartMaxLgB buckets where this bound takes two
    const int lg1 = hp.lgB + hp.lg2 < kPartMaxLgB ? hp.lgB + hp.lg2 : kPartMaxLgB;
    if ((hp.row_blocks << lg1) > *hist_entries) *hist_entries = hp.row_blocks << lg1;
    if (hp.lg2 > 0 && hp.lgB + hp.lg2 > *split_lg) *split_lg = hp.lgB + hp.lg2;
  }
  if (*rec_entries < kPartMinRecords && !part_forced()) return false;
  return true;
}

// Sizes of a workspace for up to max_seeds seeds, the given fanouts and capacities: fills every
// field of *ws but the pointers (slab stays null).  Host only.
int plan_workspace(smfg_workspace* ws, const smfg_graph* g, int32_t max_seeds, int32_t L, const int32_t* fanouts,
                   int64_t node_capacity, int64_t sample_capacity) {
  std::memset(ws, 0, sizeof(*ws));
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
  ws->device = g->device;
  ws->max_seeds = max_seeds;
  ws->L = L;
  for (int h = 0; h < L; ++h) ws->fanouts[h] = fanouts[h];
  ws->node_capacity = node_capacity;
  ws->slot_entries = slots > 0 ? slots : 1;
  ws->table_log2 = lg;
  bool wide = false;
  check_fanouts(L, fanouts, &wide);
  if (wide && !table_forced()) {
    // partition strategy over exact offsets: a hop holds at most node_capacity known nodes and
    // slot_entries samples
    ws->part = ws->flat = true;
    ws->rec_entries = node_capacity + ws->slot_entries;
    int lg = 0;
    while (lg < kPartMaxLgB + kPartMaxLg2 && (ws->rec_entries >> lg) > kPartBucketRecords) ++lg;
    const int lgB = lg < kPartMaxLgB ? lg : kPartMaxLgB;
    ws->split_lg = lg > lgB ? lg : 0;
    int64_t rows = (ws->rec_entries + kFlatBlock - 1) / kFlatBlock + 1;
    if (rows < 520) rows = 520;  // a later call with fanouts up to SMFG_MAX_FANOUT uses row blocks instead
    ws->hist_entries = rows << lgB;
  } else {
    ws->part = !table_forced() &&
               part_needs(max_seeds, L, fanouts, g->num_nodes, node_capacity, &ws->rec_entries, &ws->hist_entries,
                          &ws->split_lg) &&
               slot_entries_needed(max_seeds, L, fanouts, g->num_nodes, node_capacity) <= ws->slot_entries;
  }
  const int64_t tiles = (node_capacity + kTileRows - 1) / kTileRows + 1;
  ws->b_slot = align256(ws->slot_entries * 4);
  ws->b_row = align256((node_capacity + 4) * 4);
  ws->b_tiles = align256(tiles * 8);
  ws->b_stiles = align256((ws->slot_entries / kWideTile + 2) * 8);
  if (ws->part) {
    ws->b_rec = align256(ws->rec_entries * 8);
    ws->b_hist = align256(ws->hist_entries * 4);
    ws->b_bstart = align256((2 * (int64_t(1) << kPartMaxLgB) + 2) * 4);
    ws->b_bstart2 = ws->split_lg > 0 ? align256(((int64_t(1) << ws->split_lg) + 2) * 4) : 0;
    ws->bytes = ws->b_slot + 4 * ws->b_row + ws->b_tiles + (ws->split_lg > 0 ? 2 : 1) * ws->b_rec + ws->b_hist +
                ws->b_bstart + ws->b_bstart2;
    ws->b_grp = ws->flat ? align256((ws->slot_entries / 64 + 2) * 16) : 0;
    if (ws->flat) ws->bytes += ws->b_grp + 3 * ws->b_row + ws->b_stiles;
  } else {
    ws->b_table = align256((int64_t(1) << lg) * 8);
    ws->bytes = ws->b_table + 4 * ws->b_slot + 8 * ws->b_row + ws->b_tiles + ws->b_stiles;
  }
  return SMFG_OK;
}

// Points the arrays of a planned workspace into `base` (ws->bytes bytes, 256-byte aligned).
void bind_workspace(smfg_workspace* ws, void* base) {
  uint8_t* p = static_cast<uint8_t*>(base);
  ws->gsrc = reinterpret_cast<int32_t*>(p); p += ws->b_slot;
  ws->rowk = reinterpret_cast<int32_t*>(p); p += ws->b_row;
  ws->rowmn = reinterpret_cast<uint2*>(p); p += 2 * ws->b_row;
  ws->rowoff = reinterpret_cast<int32_t*>(p); p += ws->b_row;
  ws->tile_sums = reinterpret_cast<uint64_t*>(p); p += ws->b_tiles;
  if (ws->part) {
    ws->rec = reinterpret_cast<uint64_t*>(p); p += ws->b_rec;
    ws->hist = reinterpret_cast<uint32_t*>(p); p += ws->b_hist;
    ws->bstart = reinterpret_cast<uint32_t*>(p); p += ws->b_bstart;
    if (ws->split_lg > 0) {
      ws->bstart2 = reinterpret_cast<uint32_t*>(p); p += ws->b_bstart2;
      ws->rec2 = reinterpret_cast<uint64_t*>(p); p += ws->b_rec;
    }
    if (ws->flat) {
      ws->grp = reinterpret_cast<uint4*>(p); p += ws->b_grp;
      ws->rowstart = reinterpret_cast<int64_t*>(p); p += 2 * ws->b_row;
      ws->rowdeg = reinterpret_cast<int32_t*>(p); p += ws->b_row;
      ws->stile_sums = reinterpret_cast<uint64_t*>(p);
    }
    return;
  }
  ws->table = reinterpret_cast<uint64_t*>(p); p += ws->b_table;
  ws->ent = reinterpret_cast<uint32_t*>(p); p += ws->b_slot;
  ws->lostto = reinterpret_cast<uint32_t*>(p); p += ws->b_slot;
  ws->rank = reinterpret_cast<uint32_t*>(p); p += ws->b_slot;
  ws->rowstart = reinterpret_cast<int64_t*>(p); p += 2 * ws->b_row;
  ws->rowdeg = reinterpret_cast<int32_t*>(p); p += ws->b_row;
  p += ws->b_row;  // spare
  ws->stile_sums = reinterpret_cast<uint64_t*>(p);
}

// Device address of this GPU's copy of `scratch`, looked up at the first call on the device (the
// device must be current).  Each GPU has its own copy at its own address.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch_of(int device, void** out) {
  if (device < 0 || device >= kMaxDevices) return SMFG_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_err(e);
    if (!p) return SMFG_ERR_HIP_BASE;
    g_scratch_ptr[device] = p;
  }
  *out = g_scratch_ptr[device];
  return SMFG_OK;
}

// The gather launch shared by smfg_sample_mfg_many and smfg_gather_many.
template <int ROWS>
void launch_gather_rows(const Launch& P, int64_t max_rows, int vb, unsigned G, hipStream_t st) {
  const unsigned gb = blocks_for(max_rows, ROWS, 0x7FFFFFFFu);
  switch (vb) {
    case 16: k_gather<u32x4, ROWS><<<dim3(gb, G), kThreads, 0, st>>>(P); break;
    case 8: k_gather<u32x2, ROWS><<<dim3(gb, G), kThreads, 0, st>>>(P); break;
    case 4: k_gather<uint32_t, ROWS><<<dim3(gb, G), kThreads, 0, st>>>(P); break;
    case 2: k_gather<uint16_t, ROWS><<<dim3(gb, G), kThreads, 0, st>>>(P); break;
    default: k_gather<uint8_t, ROWS><<<dim3(gb, G), kThreads, 0, st>>>(P); break;
  }
}
template <int ROWS>
void launch_gather_plain(const smfg_graph* g, int vb, const int32_t* d_node_ids, const int64_t* d_num_rows,
                         int64_t max_rows, uint8_t* o, hipStream_t st) {
  const unsigned gb = blocks_for(max_rows, ROWS, 0x7FFFFFFFu);
  switch (vb) {
    case 16: k_gather_plain<u32x4, ROWS><<<gb, kThreads, 0, st>>>(g->feat, g->row_bytes, g->row_stride, g->num_nodes, d_node_ids, d_num_rows, max_rows, o); break;
    case 8: k_gather_plain<u32x2, ROWS><<<gb, kThreads, 0, st>>>(g->feat, g->row_bytes, g->row_stride, g->num_nodes, d_node_ids, d_num_rows, max_rows, o); break;
    case 4: k_gather_plain<uint32_t, ROWS><<<gb, kThreads, 0, st>>>(g->feat, g->row_bytes, g->row_stride, g->num_nodes, d_node_ids, d_num_rows, max_rows, o); break;
    case 2: k_gather_plain<uint16_t, ROWS><<<gb, kThreads, 0, st>>>(g->feat, g->row_bytes, g->row_stride, g->num_nodes, d_node_ids, d_num_rows, max_rows, o); break;
    default: k_gather_plain<uint8_t, ROWS><<<gb, kThreads, 0, st>>>(g->feat, g->row_bytes, g->row_stride, g->num_nodes, d_node_ids, d_num_rows, max_rows, o); break;
  }
}
void launch_gather(const Launch& P, int64_t max_rows, int vb, unsigned G, hipStream_t st) {
  StageTimer t_(SMFG_STAGE_GATHER, st);
  if (gather_rows_per_block(P.row_bytes) == 64) launch_gather_rows<64>(P, max_rows, vb, G, st);
  else launch_gather_rows<32>(P, max_rows, vb, G, st);
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
  if (misaligned(d_indptr, 8) || misaligned(d_indices, 4)) return SMFG_ERR_INVALID_ARG;
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

int smfg_graph_validate(const smfg_graph_t* g, uint32_t* h_flags, void* hip_stream) {
  if (h_flags) *h_flags = 0;
  if (!g) return SMFG_ERR_NULL_PTR;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  int cur = 0;
  (void)hipGetDevice(&cur);
  if (cur != g->device) (void)hipSetDevice(g->device);
  uint32_t* d_flags = nullptr;
  uint32_t flags = 0;
  hipError_t e = hipMalloc(reinterpret_cast<void**>(&d_flags), sizeof(uint32_t));
  if (e == hipSuccess) {
    e = hipMemsetAsync(d_flags, 0, sizeof(uint32_t), st);
    if (e == hipSuccess) {
      k_validate_indptr<<<blocks_for(g->num_nodes, kThreads * 4, 4096), kThreads, 0, st>>>(g->indptr, g->num_nodes,
                                                                                          g->num_edges, d_flags);
      if (g->num_edges > 0)
        k_validate_indices<<<blocks_for(g->num_edges, kThreads * 16, 8192), kThreads, 0, st>>>(
            g->indices, g->num_edges, g->num_nodes, d_flags);
      e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipMemcpyAsync(&flags, d_flags, sizeof(uint32_t), hipMemcpyDeviceToHost, st);
    const hipError_t es = hipStreamSynchronize(st);
    if (e == hipSuccess) e = es;
    (void)hipFree(d_flags);
  }
  if (cur != g->device) (void)hipSetDevice(cur);
  if (e != hipSuccess) return hip_err(e);
  if (h_flags) *h_flags = flags;
  return flags ? SMFG_ERR_BAD_GRAPH : SMFG_OK;
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
  smfg_workspace* ws = new (std::nothrow) smfg_workspace;
  if (!ws) return SMFG_ERR_OOM;
  int rc = plan_workspace(ws, g, max_seeds, L, fanouts, node_capacity, sample_capacity);
  if (rc != SMFG_OK) {
    delete ws;
    return rc;
  }
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
  bind_workspace(ws, ws->slab);
  // displacement notes (table strategy) start out clear; flag_rows clears whatever a call writes
  e = ws->lostto ? hipMemset(ws->lostto, 0, static_cast<size_t>(ws->slot_entries) * 4) : hipSuccess;
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

int smfg_workspace_strategy(const smfg_workspace_t* ws) {
  return ws ? (ws->part ? SMFG_STRATEGY_PARTITION : SMFG_STRATEGY_TABLE) : -1;
}

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
  // either every batch gathers or none: the gather is one launch over all of them
  const bool want_feat = g->feat && outs[0].features;
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
    if (misaligned(d_seeds[b], 4) || misaligned(o.node_ids, 4) || misaligned(o.counts, 8))
      return SMFG_ERR_INVALID_ARG;
    for (int h = 0; h < L; ++h) {
      if (!o.indptr[h] || !o.indices[h]) return SMFG_ERR_NULL_PTR;
      if (misaligned(o.indptr[h], 4) || misaligned(o.indices[h], 4)) return SMFG_ERR_INVALID_ARG;
      if (o.edge_capacity[h] < 0) return SMFG_ERR_INVALID_ARG;
    }
    if (o.node_capacity < 1) return SMFG_ERR_INVALID_ARG;
    if (num_seeds[b] > w->max_seeds || num_seeds[b] > o.node_capacity) return SMFG_ERR_TOO_MANY_SEEDS;
    // the nodes this call can reach at most; a roomier output buffer does not ask more of the workspace
    int64_t bn[SMFG_MAX_LAYERS + 1], be[SMFG_MAX_LAYERS];
    smfg_bounds(num_seeds[b], L, fanouts, g->num_nodes, bn, be);
    const int64_t ncap = o.node_capacity < bn[L] ? o.node_capacity : (bn[L] > 0 ? bn[L] : 1);
    if (ncap > w->node_capacity) return SMFG_ERR_CAPACITY;
    // fast path: padded positions must fit; wide path: E_h is checked on the device
    if (!wide && slot_entries_needed(num_seeds[b], L, fanouts, g->num_nodes, ncap) > w->slot_entries)
      return SMFG_ERR_CAPACITY;
    if (w->slot_entries > max_entries) max_entries = w->slot_entries;
    if ((g->feat && o.features) != want_feat) return SMFG_ERR_INVALID_ARG;
    if (want_feat) {
      const int v = vec_bytes(reinterpret_cast<uintptr_t>(g->feat), reinterpret_cast<uintptr_t>(o.features),
                              g->row_bytes, g->row_stride);
      if (v < vb) vb = v;
    }

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
    B.rowmn = w->rowmn;
    B.rowoff = w->rowoff;
    B.tile_sums = w->tile_sums;
    B.rowstart = w->rowstart;
    B.rowdeg = w->rowdeg;
    B.rank = w->rank;
    B.grp = w->grp;
    B.stile_sums = w->stile_sums;
    B.rec = w->rec;
    B.hist = w->hist;
    B.bstart = w->bstart;
    B.rec2 = w->rec2;
    B.bstart2 = w->bstart2;
    B.features = static_cast<uint8_t*>(o.features);
    if (o.labels) {
      if (!g->labels) return SMFG_ERR_INVALID_ARG;
      if (reinterpret_cast<uintptr_t>(o.labels) % static_cast<uintptr_t>(g->label_bytes) != 0)
        return SMFG_ERR_INVALID_ARG;
    }
    B.labels = static_cast<uint8_t*>(o.labels);
    B.node_capacity = static_cast<int32_t>(ncap);
    B.num_seeds = num_seeds[b];
    B.key0 = static_cast<uint32_t>(rng_keys[b]);
    B.key1 = static_cast<uint32_t>(rng_keys[b] >> 32);
    B.table_shift = 32u - w->table_log2;
    B.table_mask = static_cast<uint32_t>((1ull << w->table_log2) - 1ull);
    if (w->table_log2 > max_table_log2) max_table_log2 = w->table_log2;
    if (num_seeds[b] > max_seeds) max_seeds = num_seeds[b];

    int64_t n = num_seeds[b] < g->num_nodes ? num_seeds[b] : g->num_nodes;
    for (int h = 0; h <= L; ++h) {
      if (n > ncap) n = ncap;
      if (n > max_n[h]) max_n[h] = n;
      if (h < L) {
        n = fanouts[h] < 0 ? g->num_nodes : n + n * fanouts[h];
        if (n > g->num_nodes) n = g->num_nodes;
      }
    }
  }

  // Dedup strategy of the call: the partition strategy if every workspace was planned for it and
  // the call's hops fit what they hold; the table strategy if every workspace holds a table.
  bool part = true, table = true;
  for (int b = 0; b < num_batches; ++b) {
    part = part && ws[b]->part;
    table = table && !ws[b]->part;
  }
  if (!part && !table) return SMFG_ERR_INVALID_ARG;  // workspaces of one call must be planned alike
  HopPlan plan[SMFG_MAX_LAYERS];
  HopPlan flat_plan = {0, 0, 0, 1};
  if (part && wide) {
    // exact offsets: every workspace must have been planned for wide fanouts; the shape of a hop
    // is settled on the device, the host only bounds it by the roomiest workspace
    int64_t bound = 1;
    for (int b = 0; b < num_batches; ++b) {
      if (!ws[b]->flat) return SMFG_ERR_CAPACITY;
      if (ws[b]->rec_entries > bound) bound = ws[b]->rec_entries;
    }
    int lg = 0;
    while (lg < kPartMaxLgB + kPartMaxLg2 && (bound >> lg) > kPartBucketRecords) ++lg;
    flat_plan.lgB = lg < kPartMaxLgB ? lg : kPartMaxLgB;
    flat_plan.lg2 = lg - flat_plan.lgB;
    flat_plan.row_blocks = (bound + kFlatBlock - 1) / kFlatBlock;
  } else if (part) {
    for (int h = 0; h < L; ++h) {
      plan[h] = plan_hop(max_n[h], fanouts[h], num_batches);
      const int64_t records = max_n[h] * (1 + fanouts[h]);
      for (int b = 0; b < num_batches; ++b)
        if (records > ws[b]->rec_entries || (plan[h].row_blocks << plan[h].lgB) > ws[b]->hist_entries ||
            (plan[h].lg2 > 0 && plan[h].lgB + plan[h].lg2 > ws[b]->split_lg))
          return SMFG_ERR_CAPACITY;
    }
  }

  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  int cur = 0;
  (void)hipGetDevice(&cur);
  if (cur != g->device) (void)hipSetDevice(g->device);
  const unsigned G = static_cast<unsigned>(num_batches);
  constexpr unsigned kCap = 4096;  // blocks per batch of the grid-stride kernels

  if (part) {
    StageTimer t_(SMFG_STAGE_SEEDS, st);
    k_begin<<<blocks_for(max_seeds, kThreads, kCap) * G, kThreads, 0, st>>>(P);
  } else {
    { StageTimer t_(SMFG_STAGE_CLEAR, st);
    k_clear<<<blocks_for(int64_t(1) << max_table_log2, kThreads * 8, 2048) * G, kThreads, 0, st>>>(P); }
    { StageTimer t_(SMFG_STAGE_SEEDS, st);
    k_insert_seeds<<<blocks_for(max_seeds, kThreads, kCap) * G, kThreads, 0, st>>>(P); }
  }
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
    if (part && !wide) {
      P.lgB = plan[h].lgB;
      P.lg2 = plan[h].lg2;
      P.block_rows = plan[h].block_rows;
      const unsigned row_blocks = static_cast<unsigned>(plan[h].row_blocks);
      const unsigned buckets = 1u << P.lgB;
      {
        StageTimer t_(SMFG_STAGE_SAMPLE, st);
        k_sample_hist<<<row_blocks * G, kThreads, 0, st>>>(P);
      }
      {
        StageTimer t_(SMFG_STAGE_PARTITION, st);
        k_scan_hist<<<((buckets + kScanCols - 1) / kScanCols) * G, kThreads, 0, st>>>(P);
        k_scatter<<<row_blocks * G, kThreads, 0, st>>>(P);
        if (P.lg2 > 0) k_split_buckets<<<buckets * G, kThreads, 0, st>>>(P);
      }
      {
        StageTimer t_(SMFG_STAGE_DEDUP, st);
        k_dedup_buckets<<<dedup_blocks(P.lgB, P.lg2, G) * G, kThreads, 0, st>>>(P);
      }
      {
        StageTimer t_(SMFG_STAGE_FLAG, st);
        k_flag_rows_part<<<tile_blocks * G, kThreads, 0, st>>>(P);
      }
      {
        StageTimer t_(SMFG_STAGE_SCAN_TILES, st);
        k_scan_tiles<<<G, kThreads, 0, st>>>(P);
      }
      {
        StageTimer t_(SMFG_STAGE_ASSEMBLE, st);
        k_assemble_part<<<tile_blocks * G, kThreads, 0, st>>>(P);
      }
      continue;
    }
    if (wide) {
      int64_t samples = P.d < 0 ? max_entries : rows * P.d;  // upper bound of E_h
      if (samples > max_entries) samples = max_entries;
      const unsigned flat_blocks = blocks_for(samples, kWideTile, kCap);
      // a wave per destination while the grid allows; beyond that a wave takes several (see k_sample_wide)
      const unsigned wave_blocks = blocks_for(rows, kThreads / 64, 2 * kCap);
      {
        StageTimer t_(SMFG_STAGE_SCAN_TILES, st);
        k_count_rows<<<tile_blocks * G, kThreads, 0, st>>>(P);
        k_scan_count_tiles<<<G, kThreads, 0, st>>>(P);
      }
      if (part) {
        P.flat = 1;
        P.lgB = flat_plan.lgB;
        P.lg2 = flat_plan.lg2;
        int64_t stream_bound = rows + samples;  // known nodes + samples of this hop, at most
        const unsigned stream_blocks = blocks_for(stream_bound, kFlatBlock, kCap);
        const unsigned buckets = 1u << P.lgB;
        {
          StageTimer t_(SMFG_STAGE_SAMPLE, st);
          k_sample_wide<false><<<wave_blocks * G, kThreads, wide_lds_bytes(P.d), st>>>(P);
        }
        {
          StageTimer t_(SMFG_STAGE_PARTITION, st);
          k_hist_flat<<<stream_blocks * G, kThreads, 0, st>>>(P);
          k_scan_hist<<<((buckets + kScanCols - 1) / kScanCols) * G, kThreads, 0, st>>>(P);
          k_scatter_flat<<<stream_blocks * G, kThreads, 0, st>>>(P);
          if (P.lg2 > 0) k_split_buckets<<<buckets * G, kThreads, 0, st>>>(P);
        }
        {
          StageTimer t_(SMFG_STAGE_DEDUP, st);
          k_dedup_buckets<<<dedup_blocks(P.lgB, P.lg2, G) * G, kThreads, 0, st>>>(P);
        }
        {
          StageTimer t_(SMFG_STAGE_FLAG, st);
          k_flag_flat_part<<<flat_blocks * G, kThreads, 0, st>>>(P);
        }
        {
          StageTimer t_(SMFG_STAGE_SCAN_TILES, st);
          k_scan_flat_tiles<<<G, kThreads, 0, st>>>(P);
        }
        {
          StageTimer t_(SMFG_STAGE_ASSEMBLE, st);
          k_assemble_flat_part<<<flat_blocks * G, kThreads, 0, st>>>(P);
        }
        continue;
      }
      {
        StageTimer t_(SMFG_STAGE_SAMPLE, st);
        k_sample_wide<true><<<wave_blocks * G, kThreads, wide_lds_bytes(P.d), st>>>(P);
      }
      {
        StageTimer t_(SMFG_STAGE_FLAG, st);
        k_flag_flat<<<flat_blocks * G, kThreads, 0, st>>>(P);
      }
      {
        StageTimer t_(SMFG_STAGE_SCAN_TILES, st);
        k_scan_flat_tiles<<<G, kThreads, 0, st>>>(P);
      }
      {
        StageTimer t_(SMFG_STAGE_ASSEMBLE, st);
        k_assemble_flat<<<flat_blocks * G, kThreads, 0, st>>>(P);
      }
      continue;
    }
    const unsigned row_blocks = blocks_for(rows, (64 / P.d) * (kThreads / 64), kCap);
    {
      StageTimer t_(SMFG_STAGE_SAMPLE, st);
      k_sample_insert<<<row_blocks * G, kThreads, 0, st>>>(P);
    }
    {
      StageTimer t_(SMFG_STAGE_FLAG, st);
      k_flag_rows<true><<<tile_blocks * G, kThreads, 0, st>>>(P);
    }
    {
      StageTimer t_(SMFG_STAGE_SCAN_TILES, st);
      k_scan_tiles<<<G, kThreads, 0, st>>>(P);
    }
    {
      StageTimer t_(SMFG_STAGE_ASSEMBLE, st);
      if (h == L - 1) k_assemble<false><<<tile_blocks * G, kThreads, 0, st>>>(P);
      else k_assemble<true><<<tile_blocks * G, kThreads, 0, st>>>(P);
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

int smfg_sample_mfg_static(const smfg_graph_t* g, const int32_t* d_seeds, int32_t num_seeds, const int32_t* fanouts,
                           int32_t L, uint64_t rng_key, const smfg_output_t* out, void* hip_stream) {
  if (!g || !out) return SMFG_ERR_NULL_PTR;
  if (num_seeds < 0 || out->node_capacity < 1) return SMFG_ERR_INVALID_ARG;
  // the workspace this call needs: the caller's node capacity bounds it, as in smfg_workspace_create
  smfg_workspace ws;
  int rc = plan_workspace(&ws, g, num_seeds, L, fanouts, out->node_capacity, 0);
  if (rc != SMFG_OK) return rc;
  if (ws.bytes > static_cast<int64_t>(SMFG_STATIC_SCRATCH_BYTES)) return SMFG_ERR_CAPACITY;
  int cur = 0;
  hipError_t e = hipGetDevice(&cur);
  if (e != hipSuccess) return hip_err(e);
  if (cur != g->device) (void)hipSetDevice(g->device);
  void* base = nullptr;
  rc = static_scratch_of(g->device, &base);
  if (rc == SMFG_OK) {
    bind_workspace(&ws, base);
    // the array keeps what the last call left: the displacement notes of the table strategy must
    // start out clear (nothing of the partition strategy's scratch is read before it is written)
    if (ws.lostto) {
      hipStream_t st = static_cast<hipStream_t>(hip_stream);
      k_fill_u32<<<blocks_for(ws.slot_entries, kThreads * 4, 1024), kThreads, 0, st>>>(ws.lostto, ws.slot_entries, 0u);
      rc = hip_err(hipGetLastError());
    }
  }
  if (cur != g->device) (void)hipSetDevice(cur);
  if (rc != SMFG_OK) return rc;
  smfg_workspace* wsp = &ws;
  return smfg_sample_mfg_many(g, &wsp, &d_seeds, &num_seeds, fanouts, L, &rng_key, out, 1, hip_stream);
}

int smfg_gather_many(const smfg_graph_t* g, const smfg_output_t* outs, int32_t num_batches, int32_t L,
                     void* hip_stream) {
  if (!g || !outs) return SMFG_ERR_NULL_PTR;
  if (!g->feat || g->num_nodes < 1) return SMFG_ERR_INVALID_ARG;
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
    if (misaligned(o.node_ids, 4) || misaligned(o.counts, 8)) return SMFG_ERR_INVALID_ARG;
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
  if (!g->feat || g->num_nodes < 1) return SMFG_ERR_INVALID_ARG;
  if (max_rows < 0 || max_rows >= (1ll << 31)) return SMFG_ERR_INVALID_ARG;
  if (misaligned(d_node_ids, 4) || misaligned(d_num_rows, 8)) return SMFG_ERR_INVALID_ARG;
  if (max_rows == 0) return SMFG_OK;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int vb = vec_bytes(reinterpret_cast<uintptr_t>(g->feat), reinterpret_cast<uintptr_t>(d_out), g->row_bytes,
                           g->row_stride);
  uint8_t* o = static_cast<uint8_t*>(d_out);
  int cur = 0;
  (void)hipGetDevice(&cur);
  if (cur != g->device) (void)hipSetDevice(g->device);
  if (gather_rows_per_block(g->row_bytes) == 64) launch_gather_plain<64>(g, vb, d_node_ids, d_num_rows, max_rows, o, st);
  else launch_gather_plain<32>(g, vb, d_node_ids, d_num_rows, max_rows, o, st);
  hipError_t e = hipGetLastError();
  if (cur != g->device) (void)hipSetDevice(cur);
  return hip_err(e);
}

int smfg_mean_aggregate(const int32_t* d_indptr, const int32_t* d_indices, int64_t max_edges,
                        const int64_t* d_num_dst, int64_t max_dst, const void* d_x, int64_t max_src, int32_t dim,
                        int32_t elem_bytes, float* d_out, void* hip_stream) {
  if (!d_indptr || !d_indices || !d_num_dst || !d_x || !d_out) return SMFG_ERR_NULL_PTR;
  if (dim < 1 || (elem_bytes != 2 && elem_bytes != 4) || max_dst < 0 || max_dst >= (1ll << 31) || max_edges < 0 ||
      max_edges >= (1ll << 31) || max_src < 1 || max_src >= (1ll << 31))
    return SMFG_ERR_INVALID_ARG;
  if (misaligned(d_indptr, 4) || misaligned(d_indices, 4) || misaligned(d_num_dst, 8) ||
      misaligned(d_x, static_cast<uintptr_t>(elem_bytes)) || misaligned(d_out, 4))
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
        k_mean_aggregate<_Float16, 8><<<gb, kThreads, 0, st>>>(d_indptr, d_indices, max_edges, d_num_dst, max_dst, x, max_src, dim, d_out);
      else if (dim % 4 == 0 && ax % 8 == 0)
        k_mean_aggregate<_Float16, 4><<<gb, kThreads, 0, st>>>(d_indptr, d_indices, max_edges, d_num_dst, max_dst, x, max_src, dim, d_out);
      else if (dim % 2 == 0 && ax % 4 == 0)
        k_mean_aggregate<_Float16, 2><<<gb, kThreads, 0, st>>>(d_indptr, d_indices, max_edges, d_num_dst, max_dst, x, max_src, dim, d_out);
      else
        k_mean_aggregate<_Float16, 1><<<gb, kThreads, 0, st>>>(d_indptr, d_indices, max_edges, d_num_dst, max_dst, x, max_src, dim, d_out);
    } else {
      const float* x = static_cast<const float*>(d_x);
      if (dim % 4 == 0 && ax % 16 == 0)
        k_mean_aggregate<float, 4><<<gb, kThreads, 0, st>>>(d_indptr, d_indices, max_edges, d_num_dst, max_dst, x, max_src, dim, d_out);
      else
        k_mean_aggregate<float, 1><<<gb, kThreads, 0, st>>>(d_indptr, d_indices, max_edges, d_num_dst, max_dst, x, max_src, dim, d_out);
    }
  }
  return hip_err(hipGetLastError());
}

int64_t smfg_sage_packed_bytes(int32_t dim, int32_t out_dim) {
  if (dim < 8 || dim % 8 != 0 || dim > kLayerMaxDim || out_dim < 1) return 0;
  const int64_t slices = (static_cast<int64_t>(out_dim) + 31) / 32;
  return slices * 32 * 2 * dim * static_cast<int64_t>(sizeof(_Float16));
}

int smfg_sage_pack_weights(const void* d_w, int32_t dim, int32_t out_dim, void* d_packed, void* hip_stream) {
  if (!d_w || !d_packed) return SMFG_ERR_NULL_PTR;
  const int64_t bytes = smfg_sage_packed_bytes(dim, out_dim);
  if (bytes == 0) return SMFG_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(d_w) % 16 != 0 || reinterpret_cast<uintptr_t>(d_packed) % 16 != 0)
    return SMFG_ERR_INVALID_ARG;
  const int64_t vectors = bytes / 16;
  k_sage_pack_weights<<<blocks_for(vectors, kThreads, 4096), kThreads, 0, static_cast<hipStream_t>(hip_stream)>>>(
      static_cast<const _Float16*>(d_w), 2 * dim, out_dim, static_cast<half8_t*>(d_packed), vectors);
  return hip_err(hipGetLastError());
}

int smfg_sage_layer(const int32_t* d_indptr, const int32_t* d_indices, int64_t max_edges, const int64_t* d_num_dst,
                    int64_t max_dst, const void* d_x, int64_t max_src, int32_t dim, const void* d_w_packed,
                    const float* d_bias, int32_t out_dim, int32_t relu, void* d_out, int32_t out_elem_bytes,
                    void* hip_stream) {
  if (!d_indptr || !d_indices || !d_num_dst || !d_x || !d_w_packed || !d_out) return SMFG_ERR_NULL_PTR;
  if (dim < 8 || dim % 8 != 0 || dim > kLayerMaxDim || out_dim < 1 || (out_elem_bytes != 2 && out_elem_bytes != 4) ||
      max_dst < 0 || max_dst >= (1ll << 31) || max_edges < 0 || max_edges >= (1ll << 31) || max_src < 1 ||
      max_src >= (1ll << 31))
    return SMFG_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(d_x) % 16 != 0 || reinterpret_cast<uintptr_t>(d_w_packed) % 16 != 0 ||
      reinterpret_cast<uintptr_t>(d_out) % static_cast<uintptr_t>(out_elem_bytes) != 0)
    return SMFG_ERR_INVALID_ARG;
  if (misaligned(d_indptr, 4) || misaligned(d_indices, 4) || misaligned(d_num_dst, 8) || misaligned(d_bias, 4))
    return SMFG_ERR_INVALID_ARG;
  if (max_dst == 0) return SMFG_OK;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const _Float16* x = static_cast<const _Float16*>(d_x);
  const _Float16* w = static_cast<const _Float16*>(d_w_packed);
  const int rows = dim <= 128 ? 64 : 32;
  const unsigned gb = blocks_for(max_dst, rows, 0x7FFFFFFFu);
  const size_t lds = static_cast<size_t>(rows) * static_cast<size_t>(2 * dim + kLayerPad) * sizeof(_Float16);
  {
    StageTimer t_(SMFG_STAGE_LAYER, st);
    if (out_elem_bytes == 2) {
      _Float16* o = static_cast<_Float16*>(d_out);
      if (rows == 64)
        k_sage_layer<_Float16, 64><<<gb, kThreads, lds, st>>>(d_indptr, d_indices, max_edges, d_num_dst, max_dst, x, max_src, dim, w, d_bias, out_dim, relu, o);
      else
        k_sage_layer<_Float16, 32><<<gb, kThreads, lds, st>>>(d_indptr, d_indices, max_edges, d_num_dst, max_dst, x, max_src, dim, w, d_bias, out_dim, relu, o);
    } else {
      float* o = static_cast<float*>(d_out);
      if (rows == 64)
        k_sage_layer<float, 64><<<gb, kThreads, lds, st>>>(d_indptr, d_indices, max_edges, d_num_dst, max_dst, x, max_src, dim, w, d_bias, out_dim, relu, o);
      else
        k_sage_layer<float, 32><<<gb, kThreads, lds, st>>>(d_indptr, d_indices, max_edges, d_num_dst, max_dst, x, max_src, dim, w, d_bias, out_dim, relu, o);
    }
  }
  return hip_err(hipGetLastError());
}

int smfg_read_counts(const smfg_output_t* out, int32_t L, int64_t* h_counts, void* hip_stream) {
  if (!out || !out->counts || !h_counts) return SMFG_ERR_NULL_PTR;
  if (L < 1 || L > SMFG_MAX_LAYERS) return SMFG_ERR_TOO_MANY_LAYERS;
  if (misaligned(out->counts, 8)) return SMFG_ERR_INVALID_ARG;
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
  const int used = g_prof.used.load() < g_prof.max_records ? g_prof.used.load() : g_prof.max_records;
  for (int r = 0; r < used; ++r) {
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
    case SMFG_ERR_BAD_GRAPH: return "the graph's CSR arrays are inconsistent";
    case SMFG_ST_NODE_CAPACITY: return "device: node capacity exceeded";
    case SMFG_ST_EDGE_CAPACITY: return "device: edge capacity exceeded";
    case SMFG_ST_TABLE_FULL: return "device: dedup table full";
    case SMFG_ST_SEED_OUT_OF_RANGE: return "device: seed out of range";
    case SMFG_ST_DUPLICATE_SEED: return "device: duplicate seed";
    case SMFG_ST_INTERNAL: return "device: internal inconsistency (scratch memory disturbed during the call?)";
    default: return code <= SMFG_ERR_HIP_BASE ? "HIP runtime error" : "unknown code";
  }
}

}  // extern "C"

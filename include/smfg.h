/*
 * smfg - sampled mini-batch preparation for GNN training / inference on one AMD MI355X.
 *
 * C ABI of libsmfg.so.  The library computes, on the GPU, what the paper's batch-preparation
 * step computes on CPU cores (paper section 4.1 and Listing 1, lines 2-3):
 *
 *   1. node-wise neighbour sampling: for every destination node take at most d_h of its
 *      neighbours, uniformly, without replacement (section 2.2, "node-wise sampling";
 *      section 4.1, first paragraph), one fanout d_h per hop;
 *   2. construction of one bipartite block per hop with compact local node ids: destination
 *      nodes keep the first local ids in their given order, every other node gets the next id
 *      at its first appearance when scanning destinations in order and each destination's
 *      samples in slot order (the MFG construction algorithm, procedure OneHopMFG); hops are
 *      chained, the node list of hop h being the destination list of hop h+1 (section 4.1);
 *   3. the feature slice xs = x[ids] for the final node list (Listing 1).
 *
 * A fanout may also be SMFG_FANOUT_ALL: the full neighbourhood, as the paper's inference
 * experiments use it next to sampled fanouts (section 5, Table 6).
 *
 * Conventions fixed where the paper is silent:
 *   - fanouts[0] belongs to hop 0, whose destinations are the seeds;
 *   - a node with degree <= d_h contributes its whole CSR row in CSR order (no random draw);
 *     otherwise d_h distinct row positions are chosen by Floyd's subset algorithm, slot s
 *     holding the s-th pick;
 *   - random words come from Philox4x32-10 (Salmon et al., SC'11) with key = (low, high) 32-bit
 *     halves of rng_key and counter = (destination node, hop, s / 4, 0), word s % 4; a word r
 *     gives an index in [0, m) as floor(r * m / 2^32);
 *   - block h is a CSR keyed by destination: indptr[h] has n_h + 1 entries, indices[h] holds the
 *     local ids of the sampled source nodes; destination i and source i are the same node.
 * The result is a pure function of (graph, seeds, fanouts, rng_key).
 *
 * All "device" pointers are HIP device memory on the device that was current when the graph
 * handle was created.  The caller allocates and frees every input and output buffer; handles
 * own only their private scratch.  No function throws or aborts; every function returns SMFG_OK
 * or a negative SMFG_ERR_* code.  Conditions only the GPU can see are reported as a positive
 * SMFG_ST_* value in counts[2L+1]; outputs are then unspecified but nothing is written out of
 * bounds.
 */
#ifndef SMFG_H_
#define SMFG_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SMFG_MAX_LAYERS 8
#define SMFG_MAX_FANOUT 32         /* fanouts up to here take the fast path (one lane per slot)   */
#define SMFG_MAX_WIDE_FANOUT 1024  /* larger fanouts, up to here, take the wide path               */
#define SMFG_FANOUT_ALL (-1)       /* every neighbour (full neighbourhood, no draw); wide path     */
#define SMFG_MAX_BATCHES 16 /* batches per smfg_sample_mfg_many call */

/* host-detected errors (return values) */
#define SMFG_OK 0
#define SMFG_ERR_INVALID_ARG (-1)
#define SMFG_ERR_NULL_PTR (-2)
#define SMFG_ERR_BAD_FANOUT (-3)      /* d is neither SMFG_FANOUT_ALL nor in [1, SMFG_MAX_WIDE_FANOUT] */
#define SMFG_ERR_TOO_MANY_LAYERS (-4) /* L < 1 or L > SMFG_MAX_LAYERS */
#define SMFG_ERR_TOO_MANY_SEEDS (-5)  /* more seeds than the workspace / output was sized for */
#define SMFG_ERR_OOM (-6)             /* scratch allocation failed */
#define SMFG_ERR_CAPACITY (-7)        /* output capacities exceed what the workspace supports */
#define SMFG_ERR_BAD_GRAPH (-8)       /* smfg_graph_validate found a broken CSR array */
#define SMFG_ERR_HIP_BASE (-1000)     /* a HIP call failed: code = SMFG_ERR_HIP_BASE - hipError_t */

/* device-detected conditions (value of counts[2L+1]) */
#define SMFG_ST_OK 0
#define SMFG_ST_NODE_CAPACITY 1     /* more distinct nodes than out->node_capacity */
#define SMFG_ST_EDGE_CAPACITY 2     /* a block has more edges than out->edge_capacity[h] */
#define SMFG_ST_TABLE_FULL 3        /* dedup table exhausted (only if node capacity is too) */
#define SMFG_ST_SEED_OUT_OF_RANGE 4 /* a seed is < 0 or >= num_nodes */
#define SMFG_ST_DUPLICATE_SEED 5    /* the seed list holds a node twice */
#define SMFG_ST_INTERNAL 6          /* a kernel met a state its own invariants exclude (a defect, or
                                       scratch memory overwritten from outside during the call) */

typedef struct smfg_graph smfg_graph_t;         /* opaque; BORROWS the device arrays given to it */
typedef struct smfg_workspace smfg_workspace_t; /* opaque; OWNS the scratch of one in-flight batch */

/*
 * Input graph G and feature matrix X (section 2.1: X is n x f, row v the features of node v;
 * N(v) = {u : (u,v) in E}).  CSR row v = the neighbours N(v) of v; rows must not contain
 * duplicates (else "without replacement" holds for positions, not neighbours).
 *   d_indptr   device, int64 [num_nodes + 1], non-decreasing, d_indptr[0] = 0; each degree < 2^31
 *   d_indices  device, int32 [num_edges], values in [0, num_nodes)
 *              (both naturally aligned, like every typed pointer of this interface: a pointer that
 *              is not a multiple of its element size is refused with SMFG_ERR_INVALID_ARG)
 *   d_feat     device, row-major, row v at byte offset v * row_stride_bytes, the first
 *              feat_dim * elem_bytes bytes of a row are its features (any elem_bytes >= 1;
 *              rows are moved as opaque bytes, no conversion).  May be NULL: no gather then.
 * num_nodes < 2^31.  The arrays are not copied and must outlive the handle.
 */
int smfg_graph_create(smfg_graph_t **out, int64_t num_nodes, int64_t num_edges,
                      const int64_t *d_indptr, const int32_t *d_indices, const void *d_feat,
                      int32_t feat_dim, int32_t elem_bytes, int64_t row_stride_bytes);
int smfg_graph_destroy(smfg_graph_t *g);

/*
 * Optional check of the borrowed CSR arrays against the conditions above, for callers that do
 * not trust their input: the sampling calls themselves check seeds, not the graph, and follow a
 * bad offset or neighbour id out of bounds.  One streaming pass over d_indptr and d_indices on
 * hip_stream, then a synchronisation of that stream; allocates and frees 4 bytes of device memory
 * (not for use inside a stream capture).  Returns SMFG_OK, or SMFG_ERR_BAD_GRAPH with the OR of
 * the SMFG_BAD_* bits below in *h_flags (host, may be NULL).  Duplicates inside a row are not
 * looked for.
 */
#define SMFG_BAD_INDPTR_START 1u /* d_indptr[0] != 0 */
#define SMFG_BAD_INDPTR_ORDER 2u /* some d_indptr[v+1] < d_indptr[v], or a degree >= 2^31 */
#define SMFG_BAD_INDPTR_END 4u   /* d_indptr[num_nodes] != num_edges */
#define SMFG_BAD_INDEX_RANGE 8u  /* some d_indices[e] outside [0, num_nodes) */
int smfg_graph_validate(const smfg_graph_t *g, uint32_t *h_flags, void *hip_stream);

/*
 * Optional label vector y (Listing 1: ys = y[ids[:batch_size]], the labels of the seed nodes).
 * d_labels: device, num_nodes elements of elem_bytes (1, 2, 4 or 8) each, borrowed like the other
 * arrays; NULL removes it.  A batch whose output has a non-NULL `labels` buffer then receives
 * labels[i] = y[seed i], copied as opaque bytes.
 */
int smfg_graph_set_labels(smfg_graph_t *g, const void *d_labels, int32_t elem_bytes);

/*
 * Worst-case sizes (host only, pure).  With disjoint neighbourhoods (section 3 draft text on
 * neighbourhood expansion) n_{h+1} <= min(num_nodes, n_h (1 + d_h)) and E_h <= n_h d_h.
 *   max_nodes host [L + 1], max_edges host [L].  From the first hop with SMFG_FANOUT_ALL on, the
 * bounds are num_nodes nodes and -1 (unknown without the degrees) edges; E_h never exceeds the
 * graph's num_edges, because destinations are distinct.
 */
int smfg_bounds(int32_t num_seeds, int32_t L, const int32_t *fanouts, int64_t num_nodes,
                int64_t *max_nodes, int64_t *max_edges);

/*
 * Scratch for one batch in flight: per-sample and per-row state, scan partials and, by dedup
 * strategy (smfg_workspace_strategy), the records of a hop with their bucket counts and offsets,
 * or a dedup table (>= 2 slots per node of capacity).  Sized for up to max_seeds seeds, the given
 * fanouts (a later call may use the same or smaller fanouts / fewer hops) and node_capacity
 * distinct nodes (0 = the worst case of smfg_bounds).  Allocates device memory with hipMalloc,
 * zeroes part of it and synchronises the device once; not for use inside a stream capture.
 */
int smfg_workspace_create(smfg_workspace_t **out, const smfg_graph_t *g, int32_t max_seeds,
                          int32_t L, const int32_t *fanouts, int64_t node_capacity);
/*
 * The same with an explicit bound on the samples of a single hop (sample_capacity >= max_h E_h;
 * 0 = derive it from the fanouts as smfg_workspace_create does).  Needed when a fanout is
 * SMFG_FANOUT_ALL, or when the derived worst case (destinations x fanout) would exceed the 2^30
 * positions a hop can address.  A hop that draws more samples ends with SMFG_ST_EDGE_CAPACITY.
 * Calls whose fanouts are all <= SMFG_MAX_FANOUT address samples at padded positions
 * (destination x fanout + slot): for them the capacity must cover destinations x fanout of every
 * hop, else the call returns SMFG_ERR_CAPACITY.
 */
int smfg_workspace_create_sized(smfg_workspace_t **out, const smfg_graph_t *g, int32_t max_seeds,
                                int32_t L, const int32_t *fanouts, int64_t node_capacity,
                                int64_t sample_capacity);
int smfg_workspace_destroy(smfg_workspace_t *ws);
/* Bytes of device scratch the workspace holds (0 for NULL). */
int64_t smfg_workspace_bytes(const smfg_workspace_t *ws);
/*
 * How calls on this workspace remove duplicates and number new nodes (the global-to-local map of
 * procedure OneHopMFG); both give the same, serial-order result.
 *   SMFG_STRATEGY_PARTITION  the records of a hop (known nodes, samples) are grouped by node hash
 *                            and every group is settled in a hash table in on-chip memory: no
 *                            table in device memory, no device-wide atomics.  The default.
 *   SMFG_STRATEGY_TABLE      one open-addressing table in device memory per batch, claimed with
 *                            atomics.  Chosen when no hop of the planned size reaches 32768
 *                            records (fewer launches per hop; such calls are launch bound).
 * The environment variable SMFG_DEDUP=table or =partition, read when a workspace is created,
 * overrides the choice (for measurements and tests).  Returns -1 for NULL.
 */
#define SMFG_STRATEGY_TABLE 0
#define SMFG_STRATEGY_PARTITION 1
int smfg_workspace_strategy(const smfg_workspace_t *ws);

/* Output of one batch.  Every pointer is a caller-owned DEVICE buffer. */
typedef struct {
  int32_t *indptr[SMFG_MAX_LAYERS];  /* hop h: [node_capacity + 1]; n_h + 1 entries are written   */
  int32_t *indices[SMFG_MAX_LAYERS]; /* hop h: [edge_capacity[h]]; E_h local source ids written   */
  int32_t *node_ids;                 /* [node_capacity] global ids; N_h = the first n_h entries   */
  void *features;                    /* [node_capacity x feat_dim*elem_bytes] dense rows, or NULL */
  int64_t *counts;                   /* [2L+2]: n_0..n_L, E_0..E_{L-1}, status                    */
  int64_t node_capacity;
  int64_t edge_capacity[SMFG_MAX_LAYERS];
  void *labels;                      /* [num_seeds x label elem_bytes], or NULL (needs graph labels) */
} smfg_output_t;

/*
 * sample_mfg(graph, seeds, fanouts, rng_key) -> per-hop MFG blocks + node ids + gathered features.
 * Enqueues all work on `hip_stream` (a hipStream_t, NULL = the default stream) and returns
 * without waiting; nothing is copied to the host.  d_seeds: device int32 [num_seeds], distinct,
 * in [0, num_nodes).  fanouts: host int32 [L].  `out` is read during the call only (the struct
 * itself is host memory).  The workspace must not be used by another call until this one has
 * finished on the GPU.  num_seeds = 0 is allowed (all counts 0).
 */
int smfg_sample_mfg(const smfg_graph_t *g, smfg_workspace_t *ws, const int32_t *d_seeds,
                    int32_t num_seeds, const int32_t *fanouts, int32_t L, uint64_t rng_key,
                    const smfg_output_t *out, void *hip_stream);

/*
 * smfg_sample_mfg for callers that cannot allocate device memory or hold a workspace handle: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs,
 * outputs and results as smfg_sample_mfg, but the scratch lives in a fixed array inside the
 * library (SMFG_STATIC_SCRATCH_BYTES per GPU, held from the library's load until the process
 * ends) and the call allocates and frees nothing.  The scratch needed grows with
 * out->node_capacity and the fanouts exactly as smfg_workspace_bytes reports for a workspace
 * created with (num_seeds, fanouts, out->node_capacity); a call that needs more than the array
 * holds returns SMFG_ERR_CAPACITY and launches nothing (pass a smaller out->node_capacity - a
 * batch that outgrows it ends with SMFG_ST_NODE_CAPACITY - or use a workspace).  Fanouts must be
 * in [1, SMFG_MAX_WIDE_FANOUT] (SMFG_FANOUT_ALL has no size bound without a workspace:
 * SMFG_ERR_INVALID_ARG).  All calls on one GPU share the array: two calls that overlap in time
 * on the same GPU, on any streams, race; order them (one stream, or events).
 */
#define SMFG_STATIC_SCRATCH_BYTES (64u << 20)
int smfg_sample_mfg_static(const smfg_graph_t *g, const int32_t *d_seeds, int32_t num_seeds,
                           const int32_t *fanouts, int32_t L, uint64_t rng_key,
                           const smfg_output_t *out, void *hip_stream);

/*
 * The same for num_batches (1..SMFG_MAX_BATCHES) independent batches in one set of launches:
 * batch b uses ws[b], d_seeds[b], num_seeds[b], rng_keys[b], outs[b]; all share the fanouts.
 * Batches are independent units (section 4.2), so this is how several are kept in flight.
 * Results are identical to num_batches separate smfg_sample_mfg calls.
 */
int smfg_sample_mfg_many(const smfg_graph_t *g, smfg_workspace_t *const *ws,
                         const int32_t *const *d_seeds, const int32_t *num_seeds,
                         const int32_t *fanouts, int32_t L, const uint64_t *rng_keys,
                         const smfg_output_t *outs, int32_t num_batches, void *hip_stream);

/*
 * Only the gather xs = x[ids] (Listing 1): out rows j < *d_num_rows (a device int64) are copied
 * from the graph's feature rows d_node_ids[j].  max_rows bounds the launch.  Asynchronous.
 * An id outside [0, num_nodes) yields a copy of row 0: never a read outside the feature matrix.
 */
int smfg_gather_rows(const smfg_graph_t *g, const int32_t *d_node_ids, const int64_t *d_num_rows,
                     int64_t max_rows, void *d_out, void *hip_stream);

/*
 * The gather stage of smfg_sample_mfg_many on its own, for callers that run it on another stream
 * than the sampling stages (a call with outs[b].features == NULL skips the gather; this function
 * does it later): for every batch b, rows j < counts[L] of outs[b].features are copied from the
 * feature rows outs[b].node_ids[j] (an id outside [0, num_nodes) reads row 0); a batch whose
 * status word is non-zero is skipped.  One launch for all batches.  The caller orders it after the sampling call (same stream, or an event).
 */
int smfg_gather_many(const smfg_graph_t *g, const smfg_output_t *outs, int32_t num_batches,
                     int32_t L, void *hip_stream);

/*
 * A consumer of one MFG block: the mean aggregation of a GraphSAGE layer (Appendix C, GraphSAGE
 * listing: x_target = x[:size[1]], conv((x, x_target), edge_index); equation 1 with agg = mean):
 *   out[i, :] = (1 / k_i) * sum over e in [indptr[i], indptr[i+1]) of float(x[indices[e], :]),
 * k_i = indptr[i+1] - indptr[i]; a destination without samples gets zeros.  i < *d_num_dst (a device
 * int64, e.g. &counts[h]); max_dst bounds the launch (d_indptr holds at least max_dst + 1 entries,
 * d_indices max_edges).  x: device, row-major [max_src x dim], dense, max_src >= 1,
 * elem_bytes 2 (IEEE half) or 4 (float); out: device float [max_dst x dim].  Offsets beyond
 * max_edges and source ids outside [0, max_src) - which only the unspecified arrays of a batch
 * that ended with a status can hold - are clamped (row 0 is read): no read leaves the buffers.  Sums run in float in
 * slot order, then one division: the error of an output is at most k_i * 2^-24 times the mean of
 * the magnitudes added (k_i - 1 rounded additions and one rounded division).  Asynchronous on
 * hip_stream.
 */
int smfg_mean_aggregate(const int32_t *d_indptr, const int32_t *d_indices, int64_t max_edges,
                        const int64_t *d_num_dst, int64_t max_dst, const void *d_x, int64_t max_src,
                        int32_t dim, int32_t elem_bytes, float *d_out, void *hip_stream);

/*
 * One whole GraphSAGE layer over a block, with the aggregation fused into the linear transform
 * (equation 1 with the choices section 2.1 names for GraphSAGE: agg = mean, upd = a linear layer
 * on the concatenation of the node's own representation and the mean; ReLU between layers as in
 * the model listing of Appendix C):
 *   out[i, j] = act(bias[j] + sum_c w[j, c] x[i, c] + sum_c w[j, dim + c] mean_i[c]),  i < *d_num_dst,
 * mean_i as in smfg_mean_aggregate, act = max(., 0) if relu != 0 else the identity.
 *   d_x     device, IEEE half, row-major [max_src x dim], dense, 16-byte aligned; dim a multiple of
 *           8, at most 256.  Destination i is source i, so row i is also the node's own row
 *           (destinations beyond max_src are not computed).
 *   w       IEEE half, row-major [out_dim x 2 dim] (a linear layer's weight: columns [0, dim)
 *           act on the own row, [dim, 2 dim) on the mean); out_dim >= 1.  The layer call takes
 *           it re-arranged for the matrix cores: smfg_sage_pack_weights writes that arrangement
 *           (smfg_sage_packed_bytes bytes, 0 for unsupported sizes; both buffers device, 16-byte
 *           aligned; asynchronous) once per set of weights.
 *   d_bias  device, float [out_dim], or NULL.
 *   d_out   device, row-major [max_dst x out_dim] of out_elem_bytes 2 (half, round to nearest) or
 *           4 (float).
 * Arithmetic: the mean is summed in float in slot order, divided once and rounded to half; the
 * products of halfs are exact and are added in float on the matrix cores in an unspecified order.
 * With S = |bias[j]| + sum_c |w||x| + sum_c |w| mean|x| the error of an output is at most
 * S * (2^-11 + (2 dim + k_i + 2) * 2^-24), plus half an ulp of the half result if out is half.
 * Offsets and source ids are clamped as in smfg_mean_aggregate.  Asynchronous on hip_stream.
 */
int64_t smfg_sage_packed_bytes(int32_t dim, int32_t out_dim);
int smfg_sage_pack_weights(const void *d_w, int32_t dim, int32_t out_dim, void *d_packed,
                           void *hip_stream);
int smfg_sage_layer(const int32_t *d_indptr, const int32_t *d_indices, int64_t max_edges,
                    const int64_t *d_num_dst, int64_t max_dst, const void *d_x, int64_t max_src,
                    int32_t dim, const void *d_w_packed, const float *d_bias, int32_t out_dim, int32_t relu,
                    void *d_out, int32_t out_elem_bytes, void *hip_stream);

/* Copies counts[0 .. 2L+2) to the host after synchronising the stream; returns SMFG_OK or, if the
 * status word is non-zero, its (positive) SMFG_ST_* value. */
int smfg_read_counts(const smfg_output_t *out, int32_t L, int64_t *h_counts, void *hip_stream);

/*
 * Stage timing for measurement.  One profile at a time per process; begin and end must not run
 * while another thread is inside any other call of this library (the record list is process-wide
 * state that the sampling calls append to).
 * Between begin and end, launches are bracketed by HIP events on the call's own stream:
 * level 1 = only the feature gather launch, level 2 = every launch.  At most max_records
 * launches are recorded, later ones run untimed.  smfg_profile_end synchronises the device,
 * adds up the event-to-event milliseconds and the launch count per stage, and frees the events.
 */
#define SMFG_STAGE_CLEAR 0
#define SMFG_STAGE_SEEDS 1
#define SMFG_STAGE_SAMPLE 2
#define SMFG_STAGE_FLAG 3
#define SMFG_STAGE_SCAN_TILES 4
#define SMFG_STAGE_ASSEMBLE 5
#define SMFG_STAGE_GATHER 6
#define SMFG_STAGE_AGGREGATE 7
#define SMFG_STAGE_LAYER 8
#define SMFG_STAGE_PARTITION 9
#define SMFG_STAGE_DEDUP 10
#define SMFG_NUM_STAGES 11
int smfg_profile_begin(int32_t level, int32_t max_records);
int smfg_profile_end(double *stage_ms /* host [SMFG_NUM_STAGES] */,
                     int64_t *stage_launches /* host [SMFG_NUM_STAGES] */);

const char *smfg_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* SMFG_H_ */

/*
 * ripple.h - C ABI of the MI355X incremental GNN inference library.
 *
 * The library keeps, resident on one GPU, a directed graph (out- and in-
 * adjacency), the vertex features H^0 and every layer's embeddings H^1..H^L
 * of an L-layer GNN, plus one cached un-normalised neighbourhood sum X^l per
 * layer. After a batch of graph updates it refreshes only the embeddings the
 * batch can affect, by propagating embedding deltas hop by hop (paper Sec. 3.3),
 * and the result equals layer-wise recomputation on the updated graph up to
 * floating-point rounding (Sec. 3.3.3; Sec. 5, last paragraph).
 *
 * Conventions for every call:
 *   - returns a ripple_status; nothing throws or aborts across this boundary;
 *     ripple_last_error() gives a text for the last failure on that context;
 *   - input pointers are borrowed for the duration of the call only; outputs
 *     are caller-allocated; the context owns all device memory it needs;
 *   - "host or device" pointers may be pageable/pinned host memory or memory of
 *     the context's GPU; "host" pointers must be host memory;
 *   - all GPU work is enqueued on the stream given at init and the call returns
 *     after that stream has been synchronised (trigger-based inference,
 *     Sec. 2.2: results are available as soon as the batch is done);
 *   - a context is not thread-safe; call order is
 *     init_graph -> load_model -> full_infer -> (apply_updates | get_*)*,
 *     violations return RIPPLE_ESTATE.
 *   - matrices are row-major; vertex ids are 0 .. vertex_capacity-1.
 */
#ifndef RIPPLE_H
#define RIPPLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ripple_ctx ripple_ctx;   /* opaque */

typedef enum {
    RIPPLE_OK = 0,
    RIPPLE_EINVAL = 1,      /* bad argument (null pointer, id out of range, bad enum, bad shape) */
    RIPPLE_ESTATE = 2,      /* call order violated */
    RIPPLE_ECAPACITY = 3,   /* vertex/edge capacity exceeded; the piece of the batch that hit it changed nothing */
    RIPPLE_ENOMEM = 4,      /* device or host allocation failed */
    RIPPLE_EDEVICE = 5,     /* a HIP call failed */
    RIPPLE_ERANGE = 6       /* an attention layer's exponentials left the float range (scores above about 88): the call did
                               its work, but the rows ripple_last_error counts hold non-finite values */
} ripple_status;

/* The five update types of Sec. 3.1, and the replacement of an edge's weight (weighted graphs; Sec. 3.3.3,
 * "Other linear aggregators": a message is alpha_uv times the source's embedding, so a new alpha_uv reaches
 * the sink as (alpha_new - alpha_old) h_u). */
typedef enum {
    RIPPLE_EDGE_ADD = 0,      /* edge u -> v */
    RIPPLE_EDGE_DEL = 1,      /* edge u -> v */
    RIPPLE_VERTEX_ADD = 2,    /* vertex u, features = payload row feat_row */
    RIPPLE_VERTEX_DEL = 3,    /* vertex u and all its incident edges (Sec. 3.2) */
    RIPPLE_FEAT_UPDATE = 4,   /* h^0_u = payload row feat_row */
    RIPPLE_EDGE_REWEIGHT = 5  /* existing edge u -> v of a weighted graph: alpha_uv = the float32 whose bits are in feat_row;
                                 rejected when the edge is missing or the graph has no weights. The sink is affected at
                                 every hop, like the sink of an added or deleted edge. */
} ripple_op_kind;

typedef struct {
    uint32_t kind;       /* ripple_op_kind */
    uint32_t u;
    uint32_t v;          /* sink of an edge op; ignored otherwise */
    uint32_t feat_row;   /* row of the batch's feature payload; ignored for EDGE_DEL and VERTEX_DEL; weighted graphs: the
                            float32 bits of alpha_uv for EDGE_ADD and EDGE_REWEIGHT */
} ripple_update;         /* 16 bytes */

typedef enum {
    RIPPLE_AGG_SUM = 0, RIPPLE_AGG_MEAN = 1, RIPPLE_AGG_WSUM = 2,   /* linear (Table 1, Sec. 3.3.3) */
    RIPPLE_AGG_MAX = 3, RIPPLE_AGG_MIN = 4,                         /* monotonic (Table 1, Sec. 3.4.2) */
    RIPPLE_AGG_ATTN = 5                                             /* graph attention (Sec. 3.4.1, Eq. 3) */
} ripple_agg;
typedef enum {
    RIPPLE_SELF_NONE = 0,    /* GraphConv:  h = act(x W0 + b0)                               */
    RIPPLE_SELF_CONCAT = 1,  /* GraphSAGE:  h = act([h_self | x] W0 + b0), W0 is [2 d_in x .] */
    RIPPLE_SELF_ADD = 2      /* GIN:        h = act(MLP((1+eps) h_self + x))                  */
} ripple_self;
typedef enum { RIPPLE_ACT_NONE = 0, RIPPLE_ACT_RELU = 1 } ripple_act;
typedef enum { RIPPLE_STORE_F32 = 0, RIPPLE_STORE_BF16 = 1 } ripple_store;

/* One GNN layer (Eq. 1-2). x is the sum (RIPPLE_AGG_SUM) or the mean
 * (RIPPLE_AGG_MEAN; zero for a vertex without in-neighbours) of the previous
 * layer's embeddings of the vertex's in-neighbours. With d_hidden == 0 the
 * update is one linear map W0 [K x d_out], K = d_in (2*d_in for SELF_CONCAT);
 * with d_hidden > 0 it is W0 [K x d_hidden], act_inner, W1 [d_hidden x d_out].
 * act_out is applied last. Weights and biases are float32 host arrays.
 * RIPPLE_AGG_MAX / RIPPLE_AGG_MIN take the element-wise extreme over the in-neighbours' rows (zero
 * for a vertex without in-neighbours) and are maintained with the hybrid scheme of Sec. 3.4.2: a
 * vertex that hears from a changed in-neighbour keeps its aggregate, raises it from the message, or
 * recomputes it from all its in-neighbours; a vertex whose in-edges changed always recomputes. Such
 * layers are not handled project-first and are refused in the deterministic mode (they need none:
 * their result does not depend on any order).
 * RIPPLE_AGG_ATTN is a single-head graph attention layer: with p_u = h_u W0,
 * z_uv = LeakyReLU_0.2(a_src . p_u + a_dst . p_v), alpha_uv = softmax of z_uv over v's in-neighbours,
 * h_v = act_out(sum_u alpha_uv p_u + b0), act_out(b0) for a vertex without in-neighbours; att holds
 * a_src followed by a_dst (d_out floats each); self_mode must be RIPPLE_SELF_NONE and d_hidden 0. It
 * is maintained with the hybrid scheme of Sec. 3.4.1: a vertex already in the previous hop's set, or
 * with a changed in-edge, recomputes numerator and denominator from all its in-neighbours, any
 * other receives numerator / denominator differences. Exponentials are taken without subtracting a
 * maximum (the incremental form needs a fixed reference), so scores must stay below about 80; a row whose
 * sums overflow all the same is detected when it is updated, and ripple_full_infer / ripple_apply_updates
 * then return RIPPLE_ERANGE. */
typedef struct {
    uint32_t d_in, d_hidden, d_out;
    uint32_t agg;          /* ripple_agg  */
    uint32_t self_mode;    /* ripple_self */
    float    eps;          /* SELF_ADD only */
    uint32_t act_inner;    /* ripple_act, used when d_hidden > 0 */
    uint32_t act_out;      /* ripple_act */
    const float *W0, *b0;  /* host */
    const float *W1, *b1;  /* host; NULL when d_hidden == 0 */
    const float *att;      /* host; RIPPLE_AGG_ATTN only: 2 * d_out floats, else NULL */
} ripple_layer_desc;

#define RIPPLE_MAX_LAYERS 8

/* Filled by ripple_apply_updates. */
typedef struct {
    uint32_t n_ops;                               /* operations submitted                        */
    uint32_t n_applied;                           /* accepted and applied                        */
    uint32_t n_rejected;                          /* individually invalid, skipped               */
    uint32_t n_sub_batches;                       /* 1 unless operations of the batch conflicted */
    uint32_t n_compactions;                       /* graph-store compactions run by this call    */
    uint32_t n_alive;                             /* live vertices after the batch               */
    uint64_t n_edges;                             /* edges after the batch                       */
    uint32_t affected[RIPPLE_MAX_LAYERS + 1];     /* a_l = |A_l|, l = 0..L (Sec. 3.5)            */
    uint64_t messages[RIPPLE_MAX_LAYERS + 1];     /* delta messages sent into layer l (index 0 unused) */
    uint32_t n_structural;                        /* added / removed / re-weighted edges incl. those of deleted vertices */
    /* max / min layers only (Sec. 3.4.2): vertices that received a message or had an in-edge changed at
     * hop l, split by what was done with them; unchanged ones are not in A_l and send nothing on */
    uint32_t mono_unchanged[RIPPLE_MAX_LAYERS + 1];
    uint32_t mono_incremental[RIPPLE_MAX_LAYERS + 1];
    uint32_t mono_recomputed[RIPPLE_MAX_LAYERS + 1];
    /* sum, mean and weighted-sum layers: how hop l moved its messages (Sec. 3.5 compares the costs): 1 pushed
     * along the out-edges of A_{l-1}, 2 pulled through the in-rows of A_l, 3 one scan of all in-rows that also
     * found A_l, 4 gathered from the list of the hop's messages sorted by destination (RIPPLE_OPT_SORTED_MESSAGES);
     * 0 where no such kernel ran (no messages, other aggregators, deterministic mode). A batch that
     * was cut into pieces reports its last piece. */
    uint32_t hop_mode[RIPPLE_MAX_LAYERS + 1];
    /* operations of the batch, counted from its start, that took effect: n_ops on success; on a capacity or
     * device error in a batch that had to be cut into pieces, the end of the last piece that went through */
    uint32_t n_ops_done;
} ripple_batch_result;

/* Accumulated per-kernel-class timing and work counters (RIPPLE_OPT_TIMING). */
#define RIPPLE_N_PHASES 8
enum { RIPPLE_PH_INGEST = 0, RIPPLE_PH_STRUCT = 1, RIPPLE_PH_FRONTIER = 2, RIPPLE_PH_SCATTER = 3,
       RIPPLE_PH_COMPACT = 4, RIPPLE_PH_TRANSFORM = 5, RIPPLE_PH_OTHER = 6, RIPPLE_PH_TOTAL = 7 };
typedef struct {
    uint64_t batches;
    double   ms[RIPPLE_N_PHASES][RIPPLE_MAX_LAYERS + 1];       /* summed HIP-event time per phase and layer */
    uint64_t launches[RIPPLE_N_PHASES][RIPPLE_MAX_LAYERS + 1];
    uint64_t rows[RIPPLE_MAX_LAYERS + 1];                      /* sum of a_l                                 */
    uint64_t msgs[RIPPLE_MAX_LAYERS + 1];                      /* sum of messages into layer l               */
    uint64_t touched[RIPPLE_MAX_LAYERS + 1];                   /* sum of distinct destinations of those messages */
} ripple_stats;

typedef enum {
    RIPPLE_OPT_TIMING = 0,        /* 0/1: record HIP events around every kernel class (default 0) */
    RIPPLE_OPT_SCATTER_MODE = 1,  /* 0 auto per hop, 1 push (float atomics), 2 pull (segmented reduction over the in-rows of A_l),
                                     3 discover from hop 2 on (one scan of all in-rows gathers the messages and finds A_l) */
    RIPPLE_OPT_PULL_RATIO = 2,    /* auto mode pulls when messages * row_bytes * ratio >= 8 * scanned in-edges (default 1) */
    RIPPLE_OPT_BF16_MFMA = 4,     /* 0/1 (default 1): with bf16 storage, multiply on the bf16 matrix cores (fp32 accumulation);
                                     0 keeps the fp32 matrix path on bf16-rounded inputs */
    RIPPLE_OPT_PROJECT_FIRST = 3, /* 0/1 (default 1), before load_model: layers with one linear map and d_out <= d_in/2
                                     cache sum_u H[u] W_neigh instead of sum_u H[u] and scatter d_out-wide messages */
    RIPPLE_OPT_SELF_CACHE = 5,    /* 0/1 (default 1), before load_model: layers that concatenate the vertex's own embedding
                                     (one linear map) keep H[v] W_self per vertex, recomputed only where H[v] changed */
    RIPPLE_OPT_SPLIT_MFMA = 7,    /* 0/1 (default 0), before load_model, fp32 storage only: the dense products run on the bf16 matrix
                                     cores with every fp32 operand split exactly into three bf16 numbers and the six
                                     largest of the nine partial products kept (what is dropped is below 2^-24 of a
                                     product); results agree with the fp32 matrix path to rounding */
    RIPPLE_OPT_SPARSE_FRONTIER = 8, /* 0/1 (default 1): a hop whose set was small in the previous batch enters vertices into
                                     its list as they are marked instead of scanning the whole bitmap afterwards */
    RIPPLE_OPT_ROW_SEGMENTS = 9,  /* >= 0 (default: what the graph's edge capacity can need, at most 262144): max / min and attention
                                     layers recompute a very long in-row in 512-entry segments, a workgroup each; this is the
                                     most segments a hop may have queued at a time. Rows that find the queue full are read by
                                     one workgroup, as all are with 0. Results do not depend on it (sums: up to rounding order). */
    RIPPLE_OPT_PACKED_MESSAGES = 10, /* 0/1 (default 1), before load_model: a project-first layer whose rows have 33 to 48 columns
                                     sends every message as one 128-byte line instead of two (a random gather costs per line
                                     touched): block floating point, three 19-bit integers and their common power of two per
                                     8 bytes, so that a number is off by at most 2^-19 of the largest of its three. What the
                                     rounding takes from a message is carried into the sender's next one: the cached
                                     aggregates stay the exact sum of what was sent and nothing accumulates. */
    RIPPLE_OPT_STREAM_TRANSFORM = 11, /* 0/1/2 (default 1): large row updates of 256 -> 256 layers (fp32 rows) run in persistent
                                     workgroups that write a finished tile while the next one is being multiplied; 0 keeps
                                     the one-tile-per-workgroup kernel; 2 takes the streaming kernel whatever the number of
                                     rows (for tests). Same arithmetic up to rounding order. */
    RIPPLE_OPT_SORTED_MESSAGES = 12, /* 0/1/2 (default 1): a hop that would be pulled while few of the scanned in-row entries
                                      carry a message is scattered from the list of its messages instead, which the out-edge
                                      walk writes down and a radix sort orders by destination; 1 where the previous batch's
                                      counts say so, 2 wherever a hop is pulled (tests), 0 never. Same results up to the order
                                      of the sums. Not used in the deterministic mode, by weighted-sum layers or packed rows. */
    RIPPLE_OPT_DETERMINISTIC = 6  /* 0/1 (default 0), before load_model: every sum is taken in an order that is a function of
                                     the graph and the batches alone (no float atomics: in-rows keep a reproducible order,
                                     hops are gathered along them, rows that several wavefronts read are finished in
                                     wavefront order, changed edges are sorted), so that two runs over the same
                                     operations on the same device model give the same bits. About 1.3x the time.
                                     Sum and mean layers only. */
} ripple_option;

/* Build the graph store and upload features (the state the paper's Sec. 3.1
 * assumes before updates stream in). Vertices 0..n_vertices-1 are live, ids up
 * to vertex_capacity-1 may be created later. src/dst: host, n_edges entries,
 * distinct edges src[i] -> dst[i] between live vertices (self-loops allowed,
 * duplicates are a precondition violation). features: host float32
 * [n_vertices x d0]. store: RIPPLE_STORE_F32 or RIPPLE_STORE_BF16 (embeddings
 * kept in bfloat16; cached sums and all accumulation stay float32).
 * hip_stream: a hipStream_t (NULL = the default stream). */
ripple_status ripple_init_graph(ripple_ctx **out, uint32_t n_vertices, uint32_t vertex_capacity,
                                uint64_t n_edges, uint64_t edge_capacity,
                                const uint32_t *src, const uint32_t *dst,
                                const float *features, uint32_t d0, int store, void *hip_stream);

/* The same with a weight alpha_uv per edge (edge_weights: host, float32 [n_edges], borrowed; Table 1's
 * weighted sum, Sec. 3.3.3 "Other linear aggregators"): layers with RIPPLE_AGG_WSUM aggregate
 * sum_u alpha_uv h_u, other layers ignore the weights. A weight is fixed when its edge is created: an
 * EDGE_ADD operation on such a graph carries the float32 bits of alpha_uv in its feat_row word, and
 * RIPPLE_EDGE_REWEIGHT replaces it later. Weighted graphs always gather along in-edges (no push kernel) and do
 * not combine with RIPPLE_OPT_DETERMINISTIC. */
ripple_status ripple_init_graph_weighted(ripple_ctx **out, uint32_t n_vertices, uint32_t vertex_capacity,
                                         uint64_t n_edges, uint64_t edge_capacity,
                                         const uint32_t *src, const uint32_t *dst, const float *edge_weights,
                                         const float *features, uint32_t d0, int store, void *hip_stream);

/* Copy the model to the GPU: L layers, each an AGGREGATE over the in-neighbours followed by an UPDATE with
 * learned weights (Sec. 2.1, Eq. 1-2; ripple_layer_desc above says which of Table 1's aggregators and which
 * update each layer takes). layers: host array of n_layers descriptors whose weight pointers are host memory,
 * all borrowed for the call; layers[0].d_in must equal d0 and the widths must chain, else RIPPLE_EINVAL.
 * Allocates every per-layer array (H^l, X^l, caches) at vertex_capacity rows; RIPPLE_ENOMEM when that fails. */
ripple_status ripple_load_model(ripple_ctx *ctx, uint32_t n_layers, const ripple_layer_desc *layers);

/* Bootstrap: compute X^l and H^l for all layers and all live vertices on the
 * current graph (Sec. 3.1: initial embeddings exist before updates arrive). */
ripple_status ripple_full_infer(ripple_ctx *ctx);

/* Apply one batch (Sec. 3.3): operations take effect in array order; invalid
 * ones (dead endpoint, existing edge added, missing edge deleted or re-weighted, live vertex
 * added, dead vertex deleted/updated) are rejected one by one and counted; ids
 * >= vertex_capacity, unknown kinds or feat_row >= n_feat_rows fail the whole
 * call with RIPPLE_EINVAL before anything changes. Then deltas are propagated
 * through all layers. ops: host or device. feat_payload: host or device
 * float32 [n_feat_rows x d0]. res may be NULL.
 * A batch whose operations depend on one another (the same edge twice, a vertex used after the batch
 * deleted it, ...) is cut into pieces that run one after another (ripple_plan_batch shows the cut). If a
 * piece exceeds the edge capacity, or the adjacency pool even after compaction, that piece changes nothing
 * and the call returns RIPPLE_ECAPACITY; earlier pieces stay applied and fully propagated, so graph and
 * embeddings are those of the batch's first res->n_ops_done operations, which res then describes
 * (n_applied, n_rejected, n_edges, n_alive, affected). A batch that needed no cut is all or nothing. */
ripple_status ripple_apply_updates(ripple_ctx *ctx, const ripple_update *ops, uint32_t n_ops,
                                   const float *feat_payload, uint32_t n_feat_rows,
                                   ripple_batch_result *res);

/* Rows ids[0..n_ids) of H^layer (layer 0 = features) as float32 into out
 * [n_ids x d_layer] (host or device). ids: host or device, or NULL for rows
 * 0..n_ids-1. Rows of dead vertices are zero. This is the read side of trigger-based
 * inference (Sec. 2.2): every embedding is kept current by ripple_apply_updates, so a
 * query is a row copy, with no computation at request time; layer L holds the predictions. */
ripple_status ripple_get_embeddings(ripple_ctx *ctx, uint32_t layer, const uint32_t *ids,
                                    uint32_t n_ids, float *out);

/* Same for the cached un-normalised neighbourhood sums X^layer, layer = 1..L; used to
 * check the invariant X^l[v] = sum of H^{l-1} over v's in-neighbours. The row width is
 * d_{layer-1}, except for project-first layers (see ripple_get_layer_info), whose rows hold
 * sum of H^{l-1}[u] W_neigh and are d_layer wide. */
ripple_status ripple_get_aggregates(ripple_ctx *ctx, uint32_t layer, const uint32_t *ids,
                                    uint32_t n_ids, float *out);

/* Width of layer's cached aggregate rows and how the layer's linear map is split: *flags bit 0:
 * handled project-first; bit 1: the self term H^{l-1}[v] W_self is cached per vertex and refreshed
 * only where H^{l-1} changed; bit 2: the layer's messages travel packed (RIPPLE_OPT_PACKED_MESSAGES)
 * (either output pointer may be NULL). */
ripple_status ripple_get_layer_info(ripple_ctx *ctx, uint32_t layer, uint32_t *aggregate_width, int *flags);

/* Vertices the last batch could affect at `layer` (0..L), ascending, into
 * ids_out (host, room for cap ids); *n_out receives the set size even when it
 * exceeds cap (then only cap ids are written). At and below a max / min layer the
 * set is pruned (Sec. 3.4.2): it holds the vertices whose aggregate changed (plus
 * created vertices and, for layers with a self term, the previous hop's set), a
 * subset of the topological set and a superset of the rows whose value changed. */
ripple_status ripple_get_affected(ripple_ctx *ctx, uint32_t layer, uint32_t *ids_out, uint32_t cap,
                                  uint32_t *n_out);

/* ripple_get_affected for callers that cannot allocate (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the same ascending set, written straight into ids_out (device memory of
 * the context's GPU, room for cap ids; ids beyond cap are counted but not written) with the set size in
 * *n_out (device memory, 4 bytes). The call allocates and frees nothing, on the host or on the device: the
 * block sums of its two-pass compaction live in a static device array of 192 KiB that each GPU the library
 * runs on holds until the process ends. That bounds the graph: vertex_capacity beyond 134,217,728
 * (16,384 blocks of 8,192 vertices) returns RIPPLE_EINVAL. All contexts on a GPU share the array, so calls
 * that overlap on one GPU (two contexts on different streams or host threads) race; calls in sequence do
 * not, since every call writes the entries it reads. Returns after the context's stream has been
 * synchronised. */
ripple_status ripple_get_affected_static(ripple_ctx *ctx, uint32_t layer, uint32_t *ids_out, uint32_t cap,
                                         uint32_t *n_out);

/* Current edge set read back from the out-adjacency (direction 0) or the
 * in-adjacency (direction 1) as src -> dst pairs, in storage order (host
 * arrays with room for cap edges). */
ripple_status ripple_export_edges(ripple_ctx *ctx, int direction, uint32_t *src_out, uint32_t *dst_out,
                                  uint64_t cap, uint64_t *n_out);

/* In-degree (direction 1) or out-degree (direction 0) of every vertex id, and
 * the live flag (0/1) per id; host arrays of vertex_capacity entries; either may be NULL. */
ripple_status ripple_get_degrees(ripple_ctx *ctx, int direction, uint32_t *deg_out, uint8_t *alive_out);

/* Rebuild both adjacency pools without holes (also runs by itself when a pool fills up). */
ripple_status ripple_compact(ripple_ctx *ctx);

ripple_status ripple_set_option(ripple_ctx *ctx, int option, int64_t value);
ripple_status ripple_get_stats(ripple_ctx *ctx, ripple_stats *out, int reset);

/* Host only, no GPU and no context needed: how ripple_apply_updates cuts a batch (host array) into pieces
 * whose operations do not depend on one another, so that each piece can be applied in parallel with
 * the result of applying it in array order (operations of a batch take effect in array order; the
 * paper batches updates and applies them, Sec. 3.1, without saying more). piece_end (host, room for cap
 * entries) receives, per piece, the index one past its last operation; *n_pieces the number of pieces
 * even when it exceeds cap. An operation with an unknown kind, a vertex id >= vertex_capacity or a
 * payload row >= n_feat_rows makes the call return RIPPLE_EINVAL, as it does in ripple_apply_updates. */
ripple_status ripple_plan_batch(const ripple_update *ops, uint32_t n_ops, uint32_t vertex_capacity,
                                uint32_t n_feat_rows, uint32_t *piece_end, uint32_t cap, uint32_t *n_pieces);

/* What this GPU reaches on the operations the kernels above are bound by (the cost model of Sec. 3.5 counts
 * messages and rows; these are the chip's prices for them), measured with plain kernels of known size on the
 * current device: no context needed. Takes about 50 ms and 2 GiB of device memory, which it frees again. */
typedef struct {
    double hbm_copy_gbps;      /* streaming copy of 1 GiB: bytes read + written per second, in 1e9 bytes/s             */
    double hbm_read_gbps;      /* streaming read of 1 GiB, in 1e9 bytes/s                                              */
    double gather_glines;      /* gathers of random 128-byte lines from a 512 MiB table, in 1e9 lines/s                */
    double atomic_gops;        /* float atomic additions to rows of 47 numbers in ascending order, in 1e9 additions/s  */
    double mfma_f32_tflops;    /* register-only loop of 32x32x2 fp32 matrix-core instructions, in 1e12 flop/s          */
    double mfma_bf16_tflops;   /* the same with 32x32x16 bf16 instructions                                             */
    uint32_t compute_units;
    uint32_t reserved;
} ripple_peaks;
ripple_status ripple_measure_peaks(ripple_peaks *out, void *hip_stream);

void ripple_destroy(ripple_ctx *ctx);
const char *ripple_last_error(const ripple_ctx *ctx);   /* never NULL; "" when ctx is NULL */

#ifdef __cplusplus
}
#endif
#endif /* RIPPLE_H */

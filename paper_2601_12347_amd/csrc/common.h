// Internal definitions shared by the host code and the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <stdint.h>
#include <string>
#include <vector>

#include "../../include/ripple.h"

#define RP_TOMB 0xFFFFFFFFu          // hole left in an adjacency row by a deletion
#define RP_WAVE 64

// per-vertex scratch bits kept in vstate[] while a batch is being applied
#define VS_TOUCH_OUT 1u              // out-row is on the touched list
#define VS_TOUCH_IN 2u
#define VS_ADDING 4u                 // created by this (sub-)batch
#define VS_DYING 8u                  // deleted by this (sub-)batch

// expanded edge of a deleted vertex
#define EXP_NONE 0u
#define EXP_OUT 1u                   // (w -> y): erase w from y's in-row
#define EXP_IN 2u                    // (x -> w): erase w from x's out-row

struct DevCtr {                      // device-resident counters, one instance per context
    uint32_t a[RIPPLE_MAX_LAYERS + 1];        // |A_l|
    uint32_t m[RIPPLE_MAX_LAYERS + 1];        // out-edges walked from A_{l-1}
    uint32_t touched[RIPPLE_MAX_LAYERS + 1];  // distinct live destinations of those edges
    uint32_t isum[RIPPLE_MAX_LAYERS + 1];     // sum of in-degrees over A_l
    uint32_t n_struct;
    uint32_t n_touch_out, n_touch_in;
    uint32_t n_exp;                           // expanded edges of deleted vertices
    uint32_t need_exp;                        // upper bound of n_exp computed while validating
    uint32_t n_applied, n_rejected;
    uint32_t n_add, n_del;                    // accepted edge adds / deletes (ops only)
    uint32_t need_out, need_in;               // pool entries relocation will take
    uint32_t out_top, in_top;                 // first free pool entry
    uint32_t n_alive;
    uint32_t n_vadd;
    uint32_t abort_flag;                      // written by k_capacity's last workgroup: 0 ok, bit0 pool, bit1 edges, bit2 scratch
    uint32_t n_all;                           // live vertices listed for a discovering hop
    uint32_t n_long[RIPPLE_MAX_LAYERS + 1];   // max / min and attention hops: vertices with long in-rows queued for the workgroup kernel
    uint32_t cand[RIPPLE_MAX_LAYERS + 1];     // max / min hops: candidates listed while they were marked (small hops)
    uint32_t n_big[RIPPLE_MAX_LAYERS + 1];    // very long in-rows whose recomputation was split into segments
    uint32_t n_seg[RIPPLE_MAX_LAYERS + 1];    // segments queued for them
    uint32_t mono[3][RIPPLE_MAX_LAYERS + 1];  // max / min hops: candidates left unchanged / raised from the messages / recomputed
    uint32_t hop_mode[RIPPLE_MAX_LAYERS + 1]; // 1 + RP_HOP_* of the scatter kernel that moved hop l's messages (0: none ran)
    uint32_t range_rows;                      // attention layers: rows updated from sums that were not finite
    unsigned long long n_edges;
    uint32_t blocks_done;                     // workgroups of k_capacity that have finished (0 between launches)
    uint32_t n_tail_q;                        // deterministic mode: in-rows whose appended entries a workgroup puts in order
    uint32_t error;                           // sticky consistency error seen by a kernel
    uint32_t tail_top;                        // ... and the part of the copy buffer they have taken
    uint32_t pull_next[RIPPLE_MAX_LAYERS + 1];// pull scatter of hop l: runs of chunks handed out so far
};

#define RP_MONO_LISTED_LONG 64u        // small max / min and attention hops: in-rows longer than this are queued for a workgroup while the hop's vertices are listed
#define ROW_SPLIT_MIN 512u
#define ROW_SEG 512u
#define ROW_SEG_MAX (1u << 18)           // segments queued at a time; rows that find the queue full are read by one workgroup
#define SEG_NONE 0xffffffffu

struct LayerDev {
    uint32_t d_in, d_hidden, d_out, K;        // K = rows of W0
    uint32_t agg, self_mode, act_inner, act_out;
    float eps;
    // weights padded to [Kpad x Npad] (Kpad multiple of 32, Npad multiple of 64), zero filled
    float *W0, *b0, *W1, *b1;
    __hip_bfloat16 *W0h, *W1h;                // bf16 copy of W0, transposed [N0pad x K0pad] (bf16 store only); W1h unused
    uint32_t K0pad, N0pad, K1pad, N1pad;
    // project-first layers: the cached aggregate holds sum_u H[u] W_neigh (d_out wide)
    uint32_t proj;
    // What the receivers of such a layer have been sent so far: T[u] (d_out floats) is the sum of all messages u
    // has ever sent, so the cached aggregate is X[v] = sum over v's in-neighbours of T[u] at all times. A message
    // is m = H[u] W_neigh - T[u] in the form it travels in (rounded to 19-bit block floating point when
    // the row is packed into one 128-byte line) and T[u] += m: what rounding takes away from one message is part
    // of the next, so nothing accumulates. Changed edges add or remove T[u] itself.
    float *T;
    uint32_t packed;                          // 0: messages travel as fp32 rows of PD; 1: as packed rows of MSG
    float *Wn;                                // neighbour weights padded to [roundup(d_in,32) x N0pad] (may alias W0)
    float *bzero;                             // N0pad zeros
    // concat layers with one linear map: PS[v] = H^{l-1}[v] W_self (d_out wide, fp32) is cached and
    // refreshed only where H^{l-1} changed, so the row transform multiplies the aggregate alone
    uint32_t selfc;
    float *PS;
    // project-first layers with a cached self term: [W_self | W_neigh] as one matrix [roundup(d_in,32) x 128] (W_neigh
    // from column 64 on) and 128 zeros, so that one pass over the rows of A_{l-1} yields both products; else null.
    // Wc96: the same for d_out <= 48 as [roundup(d_in,32) x 96] with W_neigh from column 48 on (a quarter fewer
    // matrix-core operations; used when many rows are expected), else null
    // Wc96p: the 96 columns permuted for k_project_both_stream, [256][32][3] (d_in = 256 only), else null
    float *Wc, *bzero_c, *Wc96, *Wc96p;
    // attention layers: projected rows P[v] = H^{l-1}[v] W0 [n x d_out], scores a_src . P[v] and a_dst . P[v],
    // denominators of the softmax (the numerators are the layer's X rows); att = a_src then a_dst on the device
    float *att, *P, *ssrc, *sdst, *den;
    // fp32 storage: W0, Wn, W1 as three transposed bf16 planes each (their sum is the matrix), or null
    unsigned short *W0s, *Wns, *W1s;
    uint32_t Wns_ld;                          // row stride of the Wn planes (those of W0: K0pad, of W1: K1pad)
};

struct PhaseTimer;

struct ripple_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    std::string err;
    int state = 0;                             // 1 graph, 2 model, 3 inferred
    uint32_t n_cap = 0, n_words = 0;           // vertex capacity, bitmap words
    uint64_t e_cap = 0;
    uint64_t pool_cap = 0;
    int store = 0;                             // ripple_store
    uint32_t L = 0;
    uint32_t d[RIPPLE_MAX_LAYERS + 1] = {0};
    uint32_t dmax = 0, hmax = 0;               // widest layer / widest hidden
    LayerDev layers[RIPPLE_MAX_LAYERS];

    // graph store
    uint2 *out_meta = nullptr, *in_meta = nullptr;      // {start, len} per vertex
    uint32_t *out_capv = nullptr, *in_capv = nullptr;   // row capacity
    uint32_t *out_pool = nullptr, *in_pool = nullptr;
    float *in_w = nullptr;                              // edge weights, parallel to in_pool (weighted graphs only)
    uint32_t *alive = nullptr;                          // bitmap
    uint32_t *vstate = nullptr;                         // VS_* bits, zero between batches
    uint32_t *pend_out = nullptr, *pend_in = nullptr;   // appended this batch
    uint32_t *dead_out = nullptr, *dead_in = nullptr;   // tombstones this batch
    uint32_t *hole_out = nullptr, *hole_in = nullptr;   // where a row's latest tombstone sits

    // embeddings and cached sums
    void *H[RIPPLE_MAX_LAYERS + 1] = {nullptr};
    float *X[RIPPLE_MAX_LAYERS + 1] = {nullptr};
    float *D[2] = {nullptr, nullptr};                   // delta rows D^l[v] (valid for v in A_l), ping-pong
    float *tmp = nullptr;                               // hidden activations of two-stage updates
    float *PD = nullptr;                                // project-first layers: projected rows, then fp32 messages (by vertex)
    uint32_t *MSG = nullptr;                            // project-first layers with packed messages: 32 words per vertex
    // max / min (and attention) hops: in-rows of ROW_SPLIT_MIN entries or more are recomputed in segments of ROW_SEG
    // entries, one workgroup each. Per split row: vertex, segments finished, first segment; per segment: its row's
    // slot and its partial result (seg_ld floats)
    uint32_t *seg_v = nullptr, *seg_done = nullptr, *seg_base = nullptr, *seg_r = nullptr;
    float *seg_part = nullptr;
    uint32_t big_cap = 0, seg_cap = 0, seg_ld = 0;
    uint32_t seg_limit = 0xffffffffu;                   // RIPPLE_OPT_ROW_SEGMENTS: segments a hop may queue (<= seg_cap is used)
    float *Pold = nullptr, *sold = nullptr;             // attention hops: projected rows / source scores of A_{l-1} before the batch
    uint32_t xw[RIPPLE_MAX_LAYERS + 1] = {0};           // width of X^l (d_{l-1}, or d_l when projected)
    uint32_t pd_ld = 0;                                 // row stride of PD (64-byte multiple)

    // frontier
    uint32_t *bm[RIPPLE_MAX_LAYERS + 1] = {nullptr};    // dirty bitmap per layer
    uint32_t *bm_sink = nullptr, *bm_vadd = nullptr;    // S and V_added
    uint8_t *mk = nullptr;                              // one byte per vertex: marks of the hop in progress (zero between hops)
    uint32_t *rep[RIPPLE_MAX_LAYERS + 1] = {nullptr};   // union over sub-batches (reporting)
    uint32_t *list[RIPPLE_MAX_LAYERS + 1] = {nullptr};  // A_l, ascending (l >= 1); op order for l = 0
    uint32_t *eoff[RIPPLE_MAX_LAYERS + 1] = {nullptr};  // exclusive scan of out-degrees over A_l, +1 entry
    uint32_t *part_cnt = nullptr, *part_deg = nullptr, *part_ideg = nullptr;  // per-block partial sums
    uint32_t *ioff[RIPPLE_MAX_LAYERS + 1] = {nullptr};  // exclusive scan of in-degrees over A_l, +1 entry
    uint32_t n_part = 0;
    uint32_t *all_list = nullptr;                       // scratch list (live vertices): full inference, discovering hops
    uint32_t *ioff_all = nullptr;                       // exclusive scan of in-degrees over all_list, +1 entry

    // batch staging
    uint32_t ops_cap = 0, feat_cap = 0;
    ripple_update *ops_d = nullptr;
    float *payload_d = nullptr;
    uint32_t *op_status = nullptr, *op_pos_out = nullptr, *op_pos_in = nullptr;
    uint32_t *op_touch = nullptr;                        // per operation: accepted / add / first touch of its rows
    uint32_t *touch_out = nullptr, *touch_in = nullptr;  // touched row lists
    uint32_t touch_cap = 0;
    uint32_t exp_cap = 0;
    uint32_t *exp_kind = nullptr, *exp_a = nullptr, *exp_b = nullptr, *exp_s = nullptr;
    uint32_t struct_cap = 0;
    uint32_t *st_src = nullptr, *st_dst = nullptr;
    float *st_sign = nullptr;                           // per changed edge: what its sink's weighted sums gain, +alpha / -alpha / alpha_new - alpha_old
    float *st_unit = nullptr;                           // the same for aggregates that ignore weights: +1 added, -1 deleted, 0 re-weighted
    // deterministic mode: appended in-row entries are put in id order through these (ops_cap entries each; queue: touch_cap)
    uint32_t *tail_ids = nullptr, *tail_q = nullptr;
    float *tail_w = nullptr;
    // ... and the pull kernels leave the sums of rows whose in-edges lie in more than one run of chunks here (two entries per run)
    uint32_t *side_v = nullptr;
    float *side_acc = nullptr;
    uint32_t side_runs = 0;                             // runs there is room for
    // ... and the changed edges are sorted by (sink, source) before their structural terms are added (struct_cap entries each)
    unsigned long long *sk_in = nullptr, *sk_out = nullptr;
    float *sv_in = nullptr, *sv_out = nullptr;
    void *sort_tmp = nullptr;
    size_t sort_tmp_bytes = 0;
    DevCtr *ctr = nullptr;
    DevCtr *ctr_host = nullptr;                         // pinned mirror
    ripple_update *ops_pin = nullptr;                   // pinned staging for ops
    float *payload_pin = nullptr;
    uint32_t pin_ops_cap = 0, pin_feat_cap = 0;

    // gather staging for get_* calls
    float *gather_d = nullptr;
    uint32_t *gather_ids = nullptr;
    size_t gather_cap = 0, gather_ids_cap = 0;

    // last batch's sets (reporting)
    uint32_t last_a[RIPPLE_MAX_LAYERS + 1] = {0};
    bool hints_valid = false;                           // last_a / last_cand describe a batch (not the state after the bootstrap)
    uint32_t last_cand[RIPPLE_MAX_LAYERS + 1] = {0};
    uint32_t last_m[RIPPLE_MAX_LAYERS + 1] = {0};       // messages per hop of the last batch (a size hint)
    uint32_t last_isum[RIPPLE_MAX_LAYERS + 1] = {0};    // in-row entries a pull of that hop would have scanned
    uint32_t last_hop_mode[RIPPLE_MAX_LAYERS + 1] = {0};// 1 + RP_HOP_* of the kernel that moved that hop's messages
    // messages of a hop as (destination, source) pairs, as the out-edge walk lists them and sorted by destination
    uint32_t *pk_a = nullptr, *pk_b = nullptr, *pv_a = nullptr, *pv_b = nullptr;
    uint32_t pair_cap = 0;
    void *pair_tmp = nullptr;
    size_t pair_tmp_bytes = 0;
    unsigned pair_bits = 32;                            // key bits that tell vertex ids and the filler key apart
    int opt_sorted = 1;                                 // 0 never, 1 where the last batch says it pays, 2 wherever a hop is pulled
    uint32_t last_n_ops = 0;                            // operations of the last single-piece batch    // candidates of the last batch's max / min hops (a size hint)
    bool last_from_rep = false;
    bool push_margin[RIPPLE_MAX_LAYERS + 1] = {false};  // last batch pushed at this hop by a wide margin
    bool disc_near[RIPPLE_MAX_LAYERS + 1] = {false};    // last batch's hop was within reach of the discovering mode

    // options
    int opt_timing = 0;
    int opt_scatter = 0;
    int opt_bf16_mfma = 1;                      // bf16 storage: multiply on the bf16 matrix cores
    int opt_project = 1;                        // allow project-first layers (read by load_model)
    int opt_selfcache = 1;                      // allow cached self projections (read by load_model)
    int opt_sparse = 1;                         // small frontiers are listed as they are marked (no bitmap scan)
    int opt_stream = 1;                         // large 256 -> 256 row updates: persistent workgroups, tiles written while the next is multiplied (2: any size)
    int opt_split = 0;                          // fp32 storage: products on the bf16 matrix cores, operands split in three (read by load_model)
    int opt_deterministic = 0;                  // bit-reproducible aggregation (owner kernels, no float atomics)
    int opt_pull_ratio = 1;                     // pull when messages * width * ratio >= scanned in-edges
    int opt_pack = 1;                           // project-first layers of 33..48 columns send one-line packed messages (read by load_model)
    ripple_stats stats;
    PhaseTimer *timer = nullptr;
    uint32_t n_cu = 256;
};

// ---- host helpers -----------------------------------------------------------------
#define RP_HIP(ctx, call)                                                              \
    do {                                                                               \
        hipError_t e__ = (call);                                                       \
        if (e__ != hipSuccess) {                                                       \
            (ctx)->err = std::string(#call) + ": " + hipGetErrorString(e__);          \
            return RIPPLE_EDEVICE;                                                     \
        }                                                                              \
    } while (0)

// scatter policy of hop l as the kernels see it (see rp_hop_mode)
// |A_l| of the previous batch as a hint for launch shapes (tile sizes, grids, which compaction kernel); before
// the first batch nothing is known and the shapes for large sets are taken, which are never far off
static inline uint32_t rp_rows_hint(const ripple_ctx *c, uint32_t l) { return c->hints_valid ? c->last_a[l] : c->n_cap; }
static inline bool rp_layer_mono(const ripple_ctx *c, uint32_t l) {      // layer l (1-based) aggregates with max or min
    return l >= 1 && l <= c->L && (c->layers[l - 1].agg == RIPPLE_AGG_MAX || c->layers[l - 1].agg == RIPPLE_AGG_MIN);
}
static inline bool rp_layer_attn(const ripple_ctx *c, uint32_t l) {
    return l >= 1 && l <= c->L && c->layers[l - 1].agg == RIPPLE_AGG_ATTN;
}
static inline int rp_layer_mode(const ripple_ctx *c, uint32_t l) {
    return c->layers[l - 1].agg == RIPPLE_AGG_WSUM ? 4 : c->opt_scatter;
}
static inline uint32_t rp_div_up(uint64_t a, uint64_t b) { return (uint32_t)((a + b - 1) / b); }
static inline uint32_t rp_round_up(uint32_t a, uint32_t b) { return (a + b - 1) / b * b; }

// ---- device helpers -----------------------------------------------------------------
#ifdef __HIPCC__
__device__ __forceinline__ int rp_lane() { return threadIdx.x & 63; }
__device__ __forceinline__ bool rp_bit(const uint32_t *bm, uint32_t v) { return (bm[v >> 5] >> (v & 31)) & 1u; }
__device__ __forceinline__ void rp_set_bit(uint32_t *bm, uint32_t v) {
    uint32_t m = 1u << (v & 31);
    if (!(bm[v >> 5] & m)) atomicOr(&bm[v >> 5], m);
}
__device__ __forceinline__ float rp_bf2f(__hip_bfloat16 x) { return __bfloat162float(x); }
__device__ __forceinline__ float rp_load_h(const void *H, int store, size_t idx) {
    return store ? __bfloat162float(((const __hip_bfloat16 *)H)[idx]) : ((const float *)H)[idx];
}
__device__ __forceinline__ uint32_t rp_row_cap(uint32_t need) {   // capacity given to a relocated row
    uint32_t c = need + (need >> 1) + 4u;
    return (c + 3u) & ~3u;
}
// largest i in [lo, hi] with off[i] <= e   (off is non-decreasing, off[lo] <= e)
__device__ __forceinline__ uint32_t rp_seg_search(const uint32_t *off, uint32_t lo, uint32_t hi, uint32_t e) {
    while (lo < hi) {
        const uint32_t mid = (lo + hi + 1) >> 1;
        if (off[mid] <= e) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}
// The same for a value that all 64 lanes share, found by the wavefront together: 64 probes per round
// trip instead of one, so a list of up to 4096 rows takes two dependent reads and not twelve. To be
// called by all 64 lanes.
__device__ __forceinline__ uint32_t rp_seg_search_wave(const uint32_t *off, uint32_t lo, uint32_t hi, uint32_t e) {
    const uint32_t lane = (uint32_t)rp_lane();
    while (hi - lo >= 64u) {
        const uint32_t step = (hi - lo) / 64u + 1u;        // probes at lo + step, lo + 2 step, ... (clipped to hi)
        const uint32_t p = min(hi, lo + (lane + 1u) * step);
        const uint32_t k = (uint32_t)__popcll(__ballot(off[p] <= e));   // the probes that are <= e come first
        const uint32_t nlo = k ? min(hi, lo + k * step) : lo;
        const uint32_t nhi = (k == 64u) ? hi : min(hi, lo + (k + 1u) * step) - 1u;
        lo = nlo;
        hi = max(nlo, nhi);
    }
    const uint32_t p = lo + lane;
    return lo + (uint32_t)__popcll(__ballot(p <= hi && p > lo && off[p] <= e));
}
// the same over [lo, last], for an answer expected close to lo: doubling steps, then bisection
__device__ __forceinline__ uint32_t rp_seg_forward(const uint32_t *off, uint32_t lo, uint32_t last, uint32_t e) {
    uint32_t step = 1;
    while (lo + step <= last && off[lo + step] <= e) {
        lo += step;
        step <<= 1;
    }
    return rp_seg_search(off, lo, min(last, lo + step), e);
}
// number of lanes whose value b (ascending over the lanes) is <= e, found with shuffles; to be
// called by all 64 lanes together
__device__ __forceinline__ uint32_t rp_count_le(uint32_t b, uint32_t e) {
    const uint32_t top = __shfl(b, 63);
    uint32_t lo = 0;                                        // b of every lane below lo is <= e
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) {
        const uint32_t v = __shfl(b, (int)(lo + s - 1));
        if (v <= e) lo += s;
    }
    if (lo == 63 && top <= e) lo = 64;
    return lo;
}

// ---- packed messages ------------------------------------------------------------------
// A message row of 33..48 numbers as one 128-byte line of sixteen 8-byte chunks. Chunk c holds columns
// c, 16 + c and 32 + c as 19-bit two's-complement integers q (bits 0-18, 19-37, 38-56) that share a power of
// two: the 7-bit code E in bits 57-63 stands for the factor 2^(E - 82) (E = 0: the three numbers are zero). The
// largest of the three keeps 18 significant bits, so a number is off by at most 2^-19 of the largest in its
// chunk. A chunk is all a lane needs to decode its three columns: nothing is exchanged between lanes.
// Magnitudes of 2^63 and above are clipped; below 2^-82 they round to zero.
#define RP_MSG_WORDS 32u
#define RP_MSG_QBITS 19
static inline uint32_t rp_msg_packed(uint32_t d) { return (d > 32u && d <= 48u) ? 1u : 0u; }   // up to 32 floats are one line as they are
#ifdef __HIPCC__
__device__ __forceinline__ uint2 rp_msg_encode(float m0, float m1, float m2, float &v0, float &v1, float &v2) {
    const float big = fmaxf(fabsf(m0), fmaxf(fabsf(m1), fabsf(m2)));
    int e = 0;
    (void)frexpf(big, &e);                                  // big < 2^e
    const int se = max(-81, min(45, e - (RP_MSG_QBITS - 1)));   // the factor is 2^se
    const bool zero = !(big > 0.0f);
    const int lim = (1 << (RP_MSG_QBITS - 1)) - 1;
    const int q0 = zero ? 0 : max(-lim - 1, min(lim, __float2int_rn(ldexpf(m0, -se))));
    const int q1 = zero ? 0 : max(-lim - 1, min(lim, __float2int_rn(ldexpf(m1, -se))));
    const int q2 = zero ? 0 : max(-lim - 1, min(lim, __float2int_rn(ldexpf(m2, -se))));
    const float f = ldexpf(1.0f, se);
    v0 = (float)q0 * f;                                     // the values the integers stand for (exact products)
    v1 = (float)q1 * f;
    v2 = (float)q2 * f;
    const unsigned long long mask = (1ull << RP_MSG_QBITS) - 1ull;
    const unsigned long long bits = ((unsigned long long)(uint32_t)q0 & mask) | (((unsigned long long)(uint32_t)q1 & mask) << 19) |
                                    (((unsigned long long)(uint32_t)q2 & mask) << 38) |
                                    ((unsigned long long)(zero ? 0u : (uint32_t)(se + 82)) << 57);
    return make_uint2((uint32_t)bits, (uint32_t)(bits >> 32));
}
__device__ __forceinline__ void rp_msg_decode(uint2 c, float &v0, float &v1, float &v2) {
    const float f = __uint_as_float(((c.y >> 25) + 45u) << 23);           // 2^(E - 82); E = 0 meets q = 0
    const int q0 = ((int)(c.x << 13)) >> 13;
    const int q1 = ((int)(__builtin_amdgcn_alignbit(c.y, c.x, 19) << 13)) >> 13;
    const int q2 = ((int)(c.y << 7)) >> 13;
    v0 = (float)q0 * f;
    v1 = (float)q1 * f;
    v2 = (float)q2 * f;
}
// the same in parts: the three integers as floats and the chunk's factor; (float)q * f is exact, so a fused
// multiply-add of the two into a sum rounds as the sum of the decoded value would
__device__ __forceinline__ void rp_msg_decode_parts(uint2 c, float &q0, float &q1, float &q2, float &f) {
    f = __uint_as_float(((c.y >> 25) + 45u) << 23);
    q0 = (float)(((int)(c.x << 13)) >> 13);
    q1 = (float)(((int)(__builtin_amdgcn_alignbit(c.y, c.x, 19) << 13)) >> 13);
    q2 = (float)(((int)(c.y << 7)) >> 13);
}
// column `col` alone (kernels that give every lane one column)
__device__ __forceinline__ float rp_msg_decode_col(uint2 c, uint32_t col) {
    float v0, v1, v2;
    rp_msg_decode(c, v0, v1, v2);
    return col < 16u ? v0 : (col < 32u ? v1 : v2);
}
#endif

// How hop l (1-based) moves its messages, decided on the device from the hop's own counters so
// that no host round trip is needed. 0 push: walk the out-edges of A_{l-1}, one atomic row update
// per message. 1 pull: scan the in-rows of A_l (index + dirty-bit probe per in-edge) and gather each
// message once. 2 discover: when A_{l-1} sends along a large share of all edges nearly every vertex
// is hit, so the in-rows of all live vertices are scanned once, which both gathers the messages and
// finds A_l, and the out-edge walk that would have marked A_l is skipped.
// mode: 0 automatic, 1 push, 2 pull, 3 discover wherever it is allowed, 4 automatic without push (layers whose
// messages carry an edge weight, which is stored with the in-rows only).
#define RP_HOP_PUSH 0
#define RP_HOP_PULL 1
#define RP_HOP_DISCOVER 2
#define RP_HOP_SORTED 3                 // a pull whose messages were listed by the out-edge walk and sorted by destination (reported only)
__device__ __forceinline__ int rp_hop_mode(const DevCtr *ctr, uint32_t l, uint32_t d, int mode, int ratio, int allow_disc) {
    const unsigned long long m = ctr->m[l];
    if (allow_disc && m > 0 && (mode == 3 || ((mode == 0 || mode == 4) && m * 8ull >= ctr->n_edges))) return RP_HOP_DISCOVER;
    if (mode == 1) return RP_HOP_PUSH;
    if (mode >= 2) return RP_HOP_PULL;
    return (m > 0 && m * d * 4ull * (unsigned long long)ratio >= 8ull * ctr->isum[l]) ? RP_HOP_PULL : RP_HOP_PUSH;
}

// A hop that would be pulled is taken from the sorted list of its messages instead when the list was made (M fits
// the `cap` entries the host sorted) and it pays (force: whenever the list was made): sorting a pair costs about as
// much as eight tests of an in-neighbour, and the sort's launches as much as six million of them, so the in-rows
// that a pull would scan have to hold more than 8 M + 6 * 2^20 entries. M: out-edges of A_{l-1}.
#define RP_SORTED_FACTOR 8ull
#define RP_SORTED_FIXED (6ull << 20)
static inline bool rp_sorted_pays(unsigned long long m, unsigned long long in_entries) {
    return RP_SORTED_FACTOR * m + RP_SORTED_FIXED <= in_entries;
}
__device__ __forceinline__ bool rp_hop_sorted(const DevCtr *ctr, uint32_t l, uint32_t M, uint32_t cap, int force) {
    return cap && M > 0 && M <= cap && (force || RP_SORTED_FACTOR * M + RP_SORTED_FIXED <= ctr->isum[l]);
}

// position of `target` in row[0..len), searched by one wavefront; -1 when absent. Long (hub) rows
// are read sixteen 64-entry blocks per round, short ones four, so that a row is not paced by one
// memory round trip per 64 entries.
template <int T>
__device__ __forceinline__ int rp_wave_find_blocks(const uint32_t *row, uint32_t base, uint32_t len, uint32_t target) {
    const int lane = rp_lane();
    uint32_t v[T];
#pragma unroll
    for (int t = 0; t < T; ++t) {
        const uint32_t i = base + 64 * t + lane;
        v[t] = (i < len) ? row[i] : RP_TOMB;                // a tombstone never equals a vertex id
    }
#pragma unroll
    for (int t = 0; t < T; ++t) {
        const unsigned long long m = __ballot(v[t] == target);
        if (m) return (int)(base + 64 * t + __ffsll((long long)m) - 1);
    }
    return -1;
}
__device__ __forceinline__ int rp_wave_find(const uint32_t *row, uint32_t len, uint32_t target) {
    uint32_t base = 0;
    for (; base + 1024 <= len; base += 1024) {
        const int p = rp_wave_find_blocks<16>(row, base, len, target);
        if (p >= 0) return p;
    }
    for (; base < len; base += 256) {
        const int p = rp_wave_find_blocks<4>(row, base, len, target);
        if (p >= 0) return p;
    }
    return -1;
}
#endif

// Delta aggregation (the Send / Aggregate steps of Sec. 3.3): every vertex u of
// A_{l-1} sends m = h_u(new) - h_u(old) (Sec. 3.3.3, sum) along its out-edges
// of the updated graph and the messages arriving at v are added into the cached
// un-normalised sum X^l[v] (the vertex's hop-l inbox, Sec. 3.3.2). Mean needs
// no separate message: X stays a plain sum and the in-degree divides it when
// the row is transformed.
//
// Push kernel: the flattened (source, out-edge) space is cut into equal chunks
// via the out-degree prefix, one wavefront walks a chunk, holds the source's
// delta row in registers across that source's edges and adds it to the
// destination rows with hardware float atomics (order-free, Sec. 3.3.3).
//
// Bootstrap kernel: X^l[v] = sum over v's in-row of H^{l-1}, one wavefront per row.
#include "common.h"
#include "kernels.h"


#define PUSH_CHUNK 64
#define PULL_CHUNK 256

// PK = 1 (NJ = 1 only): the message rows are packed 128-byte lines (D points at them)
typedef uint32_t uintx2 __attribute__((ext_vector_type(2)));

template <int NJ, int PK>
__global__ __launch_bounds__(256) void k_scatter_push(const uint32_t *list, const uint32_t *count_ptr,
                                                      const uint32_t *eoff, const float *D, uint32_t ldd, uint32_t d,
                                                      const uint2 *out_meta, const uint32_t *out_pool, float *X,
                                                      DevCtr *ctr, uint32_t l, int may_pull, int mode, int ratio, int allow_disc) {
    constexpr int G = (NJ <= 2) ? 8 : (NJ <= 4 ? 4 : (NJ <= 8 ? 2 : 1));   // edges per round
    const int hm = rp_hop_mode(ctr, l, d, mode, ratio, allow_disc);
    if (hm == RP_HOP_DISCOVER || (may_pull && hm == RP_HOP_PULL)) return;
    const uint32_t count = *count_ptr;
    if (count == 0) return;
    if (blockIdx.x == 0 && threadIdx.x == 0) ctr->hop_mode[l] = 1u + RP_HOP_PUSH;
    const int lane = rp_lane();
    const uint32_t M = eoff[count];
    const uint32_t chunk = (M <= 16384u) ? 16u : PUSH_CHUNK;   // few messages: spread them over more wavefronts
    const uint32_t n_chunks = (M + chunk - 1) / chunk;
    const uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    for (uint32_t c = gw; c < n_chunks; c += nw) {
        const uint32_t e0 = c * chunk, e1 = min(M, e0 + chunk);
        // the chunk's first row by the wavefront together; the 64 rows from there on (vertex, pool position,
        // end) one per lane, so an edge finds its row with shuffles instead of a chain of dependent reads
        const uint32_t i_lo = rp_seg_search_wave(eoff, 0, count - 1, e0);
        const uint32_t ri = min(count - 1, i_lo + (uint32_t)lane);
        const uint32_t rv = list[ri];
        const uint32_t rbase = out_meta[rv].x - eoff[ri];      // pool position of edge e: rbase + e (mod 2^32)
        const uint32_t bnd = eoff[min(count, i_lo + 1u + (uint32_t)lane)];
        const uint32_t e = min(e0 + (uint32_t)lane, e1 - 1);    // lanes past the chunk repeat its last edge (not used)
        const uint32_t k = rp_count_le(bnd, e);
        uint32_t my_i = i_lo + k, my_u = __shfl(rv, (int)min(k, 63u)), pos = __shfl(rbase, (int)min(k, 63u)) + e;
        if (k >= 64u) {                                         // more than 64 rows in 64 edges (rows without out-edges)
            my_i = rp_seg_search(eoff, i_lo + 64u, count - 1, e);
            my_u = list[my_i];
            pos = out_meta[my_u].x + (e - eoff[my_i]);
        }
        const uint32_t my_v = out_pool[pos];
        const int n_here = (int)(e1 - e0);
        // G edges per round: their sources' delta rows are requested together (consecutive edges mostly share
        // the source: the repeats are cache hits), then the additions go out
        for (int k0 = 0; k0 < n_here; k0 += G) {
            float dreg[G][NJ];
            uint32_t vk[G];
            if constexpr (PK) {                              // lane = column: its chunk is lane mod 16
                uint2 ch[G];
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    const int k = min(k0 + g, n_here - 1);
                    const uint32_t uk = __shfl(my_u, k);
                    vk[g] = __shfl(my_v, k);
                    ch[g] = *(const uint2 *)((const uint32_t *)D + (size_t)uk * RP_MSG_WORDS + 2u * ((uint32_t)lane & 15u));
                }
#pragma unroll
                for (int g = 0; g < G; ++g) dreg[g][0] = ((uint32_t)lane < d) ? rp_msg_decode_col(ch[g], (uint32_t)lane) : 0.0f;
            } else {
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    const int k = min(k0 + g, n_here - 1);
                    const uint32_t uk = __shfl(my_u, k);
                    vk[g] = __shfl(my_v, k);
#pragma unroll
                    for (int j = 0; j < NJ; ++j) {
                        const uint32_t col = lane + 64 * j;
                        dreg[g][j] = (col < d) ? D[(size_t)uk * ldd + col] : 0.0f;
                    }
                }
            }
#pragma unroll
            for (int g = 0; g < G; ++g) {
                if (k0 + g < n_here) {
                    bool any = false;
#pragma unroll
                    for (int j = 0; j < NJ; ++j) any |= dreg[g][j] != 0.0f;
                    if (__ballot(any) != 0ull) {                // an all-zero delta changes nothing
                        float *xr = X + (size_t)vk[g] * d;
#pragma unroll
                        for (int j = 0; j < NJ; ++j) {
                            const uint32_t col = lane + 64 * j;
                            if (col < d) unsafeAtomicAdd(&xr[col], dreg[g][j]);
                        }
                    }
                }
            }
        }
    }
}

void rp_launch_scatter_push(ripple_ctx *c, uint32_t l, bool may_pull, bool allow_disc) {
    const bool proj = c->layers[l - 1].proj != 0;           // project-first: messages are already d_out wide
    const uint32_t d = c->xw[l];
    const bool packed = proj && c->layers[l - 1].packed;
    const float *D = packed ? (const float *)c->MSG : (proj ? c->PD : c->D[(l - 1) & 1]);
    const uint32_t ldd = proj ? c->pd_ld : d;
    dim3 grid(c->n_cu * 8), block(256);
#define PUSH_CASE_PK(NJ, PK)                                                                                       \
    hipLaunchKernelGGL((k_scatter_push<NJ, PK>), grid, block, 0, c->stream, c->list[l - 1], &c->ctr->a[l - 1],     \
                       c->eoff[l - 1], D, ldd, d, c->out_meta, c->out_pool, c->X[l], c->ctr, l, may_pull ? 1 : 0,  \
                       c->opt_scatter, c->opt_pull_ratio, allow_disc ? 1 : 0)
#define PUSH_CASE(NJ) PUSH_CASE_PK(NJ, 0)
    if (packed) PUSH_CASE_PK(1, 1);
    else if (d <= 64) PUSH_CASE(1);
    else if (d <= 128) PUSH_CASE(2);
    else if (d <= 256) PUSH_CASE(4);
    else if (d <= 512) PUSH_CASE(8);
    else PUSH_CASE(16);
#undef PUSH_CASE
#undef PUSH_CASE_PK
}

// ---------------------------------------------------------------------------------
// pull: segmented reduction over in-rows, keeping only the sources that are in A_{l-1}
// ---------------------------------------------------------------------------------
// The flattened in-edge space of the listed destinations is cut into 256-edge chunks and every
// wavefront takes a contiguous run of chunks, so the row of a chunk's first edge follows from the
// previous chunk instead of a search over the whole list. The 64 rows after that one (vertex, pool
// position, first edge) sit in registers, one per lane; an edge finds its row with shuffles. The next
// chunk's rows are requested before the gathers of the current one.
// DISC = 0: destinations are A_l. DISC = 1 (discovering hop): destinations are all live vertices and
// those that receive a message are marked in the hop's bitmap.
#define PULL_RUN 8                      // chunks a wavefront takes at a time on a large hop
// the next run's number, fetched by lane 0 for the wavefront
__device__ __forceinline__ uint32_t rp_next_run(uint32_t *counter, int lane) {
    uint32_t r = 0;
    if (lane == 0) r = atomicAdd(counter, 1u);
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)r);
}

struct PullArgs {
    const uint32_t *list;          // destinations, ascending
    const uint32_t *count_ptr;
    const uint32_t *ioff;          // in-degree prefix over the list
    const uint2 *in_meta;
    const uint32_t *in_pool;
    const float *in_w;             // edge weights parallel to in_pool (weighted-sum layers), or null
    const uint32_t *bm_prev;       // A_{l-1} as bitmap
    uint32_t *bm_cur;              // bitmap of A_l: receivers are marked here when discovering
    const float *D;                // delta rows, indexed by vertex
    uint32_t ldd;                  // their row stride
    uint32_t msg_bytes;            // packed message rows (k_scatter_pull4): size of the table in bytes, below 4 GB
    uint32_t d;
    float *X;
    DevCtr *ctr;
    uint32_t l;
    int mode, ratio, allow_disc;
    // the hop's messages may have been listed and sorted instead (rp_hop_sorted): then the pull leaves the hop alone
    const uint32_t *m_eoff, *m_count;   // out-degree prefix over A_{l-1} and |A_{l-1}|: the number of messages
    uint32_t sorted_cap;           // entries the host sorted (0: no list was made)
    int sorted_force;
    // deterministic variants only
    const uint32_t *bm_rec;        // destinations that are recomputed from all their in-neighbours (bootstrap inference), or null
    const void *Hprev;             // what a recomputed row sums: rows of H^{l-1} (storage format `store`) ...
    const float *R;                // ... or, for a project-first layer, of T (what every vertex has sent so far); stride d
    int store;
    uint32_t side_runs;            // runs the side entries have room for (two entries per run)
    uint32_t *side_v;              // per run: the destinations of its first and last in-edge, if it has sums for them
    float *side_acc;               // ... and those sums, d floats per entry
};

// The part both pull kernels share: which in-edges a chunk holds. Lane j describes row i_lo + j of the
// list: destination rv, pool position of edge e is rbase + e (mod 2^32), and bnd = first edge of row
// i_lo + j + 1 (the total beyond the list's end).
template <int T, int WT>
struct PullScan {
    uint32_t i_lo, rv, rbase, bnd;
    uint32_t i_nx, rv_n, rbase_n, bnd_n;

    __device__ __forceinline__ void begin(const PullArgs &a, uint32_t count, uint32_t c_begin, int lane) {
        const uint32_t last = count - 1;
        i_lo = rp_seg_search_wave(a.ioff, 0, last, c_begin * PULL_CHUNK);
        const uint32_t ri = min(last, i_lo + lane);
        rv = a.list[ri];
        rbase = a.in_meta[rv].x - a.ioff[ri];
        bnd = a.ioff[min(count, i_lo + 1 + lane)];
    }
    // edge e0 + 64 t + lane of the chunk [e0, e1): its destination, source, weight and whether the source is in
    // A_{l-1}; then requests the rows of the next chunk, which are in flight while this chunk's messages are gathered
    __device__ __forceinline__ void chunk(const PullArgs &a, uint32_t count, uint32_t e0, uint32_t e1, int lane,
                                          uint32_t (&my_v)[T], uint32_t (&my_u)[T], float (&my_w)[WT ? T : 1], bool (&dirty)[T]) {
        const uint32_t last = count - 1;
        const bool fits = __shfl(bnd, 63) > e1 - 1;         // every row of the chunk is among the 64 held
        if (fits) {
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const uint32_t e = e0 + 64 * t + lane;
                const int r = (int)min(63u, rp_count_le(bnd, e));
                my_v[t] = __shfl(rv, r);
                const uint32_t base = __shfl(rbase, r);
                my_u[t] = 0;
                dirty[t] = false;
                if (WT) my_w[t] = 0.0f;
                if (e < e1) {
                    my_u[t] = a.in_pool[base + e];
                    if (WT) my_w[t] = a.in_w[base + e];
                    dirty[t] = (a.bm_prev[my_u[t] >> 5] >> (my_u[t] & 31)) & 1u;
                }
            }
            i_nx = min(last, i_lo + rp_count_le(bnd, e1));
        } else {
            // Short rows (a stretch of vertices with fewer than four in-neighbours on average, e.g. vertices created
            // by earlier batches, which sit together at the end of the id range): the chunk is taken in pieces of
            // 64 rows, each like a chunk that fits. (A search per edge instead made such chunks several times as
            // slow as the others, and since a wavefront's chunks are neighbours, the wavefronts at the end of the
            // id range then held up the whole hop: 2.1 -> 3.8 ms after 400 batches that each create 100 vertices.)
#pragma unroll
            for (int t = 0; t < T; ++t) {
                my_v[t] = 0;
                my_u[t] = 0;
                if (WT) my_w[t] = 0.0f;
                dirty[t] = false;
            }
            uint32_t il = i_lo, rv_p = rv, rb_p = rbase, bn_p = bnd, es = e0;
            for (;;) {
                const uint32_t top = min(e1, (uint32_t)__shfl(bn_p, 63));   // edges [es, top) lie in the 64 rows held
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    const uint32_t e = e0 + 64 * t + lane;
                    const int r = (int)min(63u, rp_count_le(bn_p, e));
                    const uint32_t v = __shfl(rv_p, r);
                    const uint32_t base = __shfl(rb_p, r);
                    if (e >= es && e < top) {
                        my_v[t] = v;
                        my_u[t] = a.in_pool[base + e];
                        if (WT) my_w[t] = a.in_w[base + e];
                        dirty[t] = (a.bm_prev[my_u[t] >> 5] >> (my_u[t] & 31)) & 1u;
                    }
                }
                if (top >= e1) break;
                es = top;
                il = min(last, il + 64u);
                const uint32_t rp = min(last, il + lane);
                rv_p = a.list[rp];
                rb_p = a.in_meta[rv_p].x - a.ioff[rp];
                bn_p = a.ioff[min(count, il + 1 + lane)];
            }
            i_nx = min(last, il + rp_count_le(bn_p, e1));
        }
        const uint32_t ri = min(last, i_nx + lane);
        rv_n = a.list[ri];
        rbase_n = a.in_meta[rv_n].x - a.ioff[ri];
        bnd_n = a.ioff[min(count, i_nx + 1 + lane)];
    }
    __device__ __forceinline__ void advance() {
        i_lo = i_nx;
        rv = rv_n;
        rbase = rbase_n;
        bnd = bnd_n;
    }
};

// DET = 1, the deterministic mode's form of both pull kernels. Float addition does not commute bit for bit, so
// every sum has to be taken in an order that is a function of the graph and the batches alone:
//   * the graph store keeps the order of an in-row such a function (rows built in the order the edges were given,
//     appended entries put in id order, holes filled by a fixed rule), the list of destinations is ascending, and
//     the cut of the in-edge space into chunks and of the chunks into runs (every nw-th run is one wavefront's)
//     depends on their number and the grid only;
//   * within a run a wavefront carries a destination's partial sum from chunk to chunk, so a run finishes every
//     destination once. Only the destinations of a run's first and last in-edge can have in-edges in another run;
//     their sums go to two side entries per run instead of memory, and k_pull_fixup adds the entries of one
//     destination in run order. All other rows are written with plain loads and stores by their only writer.
// The changed edges' structural terms have been added before the first hop, in (sink, source) order (k_struct_ordered).
// Bootstrap inference runs the same kernels with every destination marked as recomputed: every in-edge of such a
// row contributes, with the source's current row (of H^{l-1}, or of T for a project-first layer) in place of a
// message, and the sum replaces the row. The hop is always pulled.
//
// WT = 1: every message is multiplied by its edge's weight (weighted sum, m = alpha (h - h_old), Sec. 3.3.3)
template <int NJ, int DISC, int WT, int DET>
__global__ __launch_bounds__(256) void k_scatter_pull(PullArgs a) {
    static_assert(!DET || (!DISC && !WT), "the deterministic form pulls into A_l, unweighted");
    if (!DET && rp_hop_mode(a.ctr, a.l, a.d, a.mode, a.ratio, a.allow_disc) != (DISC ? RP_HOP_DISCOVER : RP_HOP_PULL)) return;
    if (!DET && !DISC && a.sorted_cap) {
        const uint32_t cp = *a.m_count;
        if (rp_hop_sorted(a.ctr, a.l, cp ? a.m_eoff[cp] : 0u, a.sorted_cap, a.sorted_force)) return;
    }
    const uint32_t count = *a.count_ptr;
    if (count == 0) return;
    if (blockIdx.x == 0 && threadIdx.x == 0) a.ctr->hop_mode[a.l] = 1u + (DISC ? RP_HOP_DISCOVER : RP_HOP_PULL);
    // delta rows gathered per round trip; the weighted one-column kernel takes 12 so that it stays
    // within 64 registers (eight waves per SIMD), which matters more here than the deeper round
    constexpr int G = (NJ >= 8) ? 2 : (WT && NJ == 1) ? 12 : 16 / NJ;
    constexpr int T = PULL_CHUNK / 64;                      // in-edges examined per lane and chunk
    const int lane = rp_lane();
    const uint32_t d = a.d;
    const uint32_t total = a.ioff[count];
    const uint32_t n_chunks = (total + PULL_CHUNK - 1) / PULL_CHUNK;
    const uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    // The chunks are handed out in runs (PULL_RUN chunks on large hops, one chunk when there are fewer chunks than
    // wavefronts would need). A wavefront starts with the run of its own number; after that it fetches runs from a
    // counter until none is left, or, in the deterministic mode, takes every nw-th run (a cut that depends on the
    // number of chunks and the grid alone). One long contiguous run per wavefront is what the first version had:
    // chunks differ in cost (a stretch of short in-rows ends a sum every few edges), stretches of such chunks exist
    // (the vertices that earlier batches created sit together at the end of the id range), and the few wavefronts
    // that owned such a stretch held up the hop (3.4 instead of 2.1 ms after 400 batches that each create 100
    // vertices; in the deterministic mode 7.4 instead of 2.5 ms at hop 2).
    const uint32_t per = max(1u, min((uint32_t)PULL_RUN, n_chunks / (2u * nw)));
    const uint32_t n_runs = (n_chunks + per - 1) / per;
    uint32_t run = gw;                                      // the first run needs no counter
    if (DET && n_runs > a.side_runs) {                      // cannot happen: the side entries are sized for the in-row pool
        if (gw == 0 && lane == 0) a.ctr->error = 9;
        return;
    }
    if (run >= n_runs) {
        if (DET && lane == 0)
            for (; run < a.side_runs; run += nw) a.side_v[2 * run] = a.side_v[2 * run + 1] = 0xFFFFFFFFu;
        return;
    }
    uint32_t c_begin = run * per;
    uint32_t c_end = min(n_chunks, c_begin + per);
    PullScan<T, WT> scan;
    scan.begin(a, count, c_begin, lane);
    constexpr uint32_t NONE = 0xFFFFFFFFu;
    uint32_t cur = NONE;                                    // destination whose partial sum is held
    bool cur_rec = false;                                   // ... and whether it is recomputed (DET)
    float acc[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) acc[j] = 0.0f;
    // DET: the destinations of the current run's first and last in-edge, and whether a sum was left for them
    uint32_t v_head = NONE, v_tail = NONE;
    bool wrote_head = false, wrote_tail = false;
    if (DET) {
        v_head = (uint32_t)__shfl((int)scan.rv, 0);
        v_tail = a.list[rp_seg_search_wave(a.ioff, 0, count - 1, min(total, c_end * PULL_CHUNK) - 1u)];
    }
    auto flush = [&]() {
        float *xr = a.X + (size_t)cur * d;
        if (!DET) {
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const uint32_t col = lane + 64 * j;
                if (col < d && acc[j] != 0.0f) unsafeAtomicAdd(&xr[col], acc[j]);
                acc[j] = 0.0f;
            }
            if (DISC && lane == 0) atomicOr(&a.bm_cur[cur >> 5], 1u << (cur & 31));   // once per receiver and wavefront
            return;
        }
        if (cur == v_head || cur == v_tail) {
            const uint32_t slot = 2 * run + (cur == v_head ? 0u : 1u);
            if (cur == v_head) wrote_head = true;
            else wrote_tail = true;
            xr = a.side_acc + (size_t)slot * d;
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const uint32_t col = lane + 64 * j;
                if (col < d) xr[col] = acc[j];
                acc[j] = 0.0f;
            }
        } else {
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const uint32_t col = lane + 64 * j;
                if (col < d) xr[col] = cur_rec ? acc[j] : xr[col] + acc[j];
                acc[j] = 0.0f;
            }
        }
    };
    for (;;) {
    for (uint32_t c = c_begin; c < c_end; ++c) {
        const uint32_t e0 = c * PULL_CHUNK, e1 = min(total, e0 + PULL_CHUNK);
        uint32_t my_v[T], my_u[T];
        float my_w[WT ? T : 1];
        bool dirty[T];
        bool rec[DET ? T : 1];
        scan.chunk(a, count, e0, e1, lane, my_v, my_u, my_w, dirty);
        if (DET) {
#pragma unroll
            for (int t = 0; t < T; ++t) {
                rec[t] = a.bm_rec && e0 + 64 * t + lane < e1 && rp_bit(a.bm_rec, my_v[t]);
                dirty[t] = dirty[t] || rec[t];
            }
        }
#pragma unroll
        for (int t = 0; t < T; ++t) {
            unsigned long long mask = __ballot(dirty[t]);
            while (mask) {
                int kk[G];
                int n = 0;
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    kk[g] = 0;
                    if (mask) {
                        kk[g] = __ffsll((long long)mask) - 1;
                        mask &= mask - 1;
                        n = g + 1;
                    }
                }
                float r[G][NJ];
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    const uint32_t uk = __shfl(my_u[t], kk[g]);
                    const bool rk = DET && __shfl((int)rec[DET ? t : 0], kk[g]) != 0;
#pragma unroll
                    for (int j = 0; j < NJ; ++j) {
                        const uint32_t col = lane + 64 * j;
                        float x = 0.0f;
                        if (g < n && col < d) {
                            if (rk) x = a.R ? a.R[(size_t)uk * d + col] : rp_load_h(a.Hprev, a.store, (size_t)uk * d + col);
                            else x = a.D[(size_t)uk * a.ldd + col];
                        }
                        r[g][j] = x;
                    }
                }
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    if (g < n) {
                        const uint32_t vk = __shfl(my_v[t], kk[g]);
                        if (vk != cur) {                     // the destination changes: flush its partial sum
                            if (cur != NONE) flush();
                            cur = vk;
                            if (DET) cur_rec = __shfl((int)rec[DET ? t : 0], kk[g]) != 0;
                        }
                        // the weight is fetched again here rather than kept per row in flight (registers)
                        const float wk = WT ? __shfl(my_w[t], kk[g]) : 1.0f;
#pragma unroll
                        for (int j = 0; j < NJ; ++j) acc[j] += WT ? r[g][j] * wk : r[g][j];
                    }
                }
            }
        }
        scan.advance();                                      // the destination and its partial sum carry over to the next chunk
    }
    if (cur != NONE) flush();
    cur = NONE;
    if (DET) {
        if (lane == 0) {
            a.side_v[2 * run] = wrote_head ? v_head : NONE;
            a.side_v[2 * run + 1] = wrote_tail ? v_tail : NONE;
        }
        wrote_head = wrote_tail = false;
        run += nw;
    } else {
        if ((unsigned long long)nw * per >= n_chunks) break;      // every run was somebody's first
        run = nw + rp_next_run(&a.ctr->pull_next[a.l], lane);
    }
    if (run >= n_runs) break;
    c_begin = run * per;
    c_end = min(n_chunks, c_begin + per);
    scan.begin(a, count, c_begin, lane);
    if (DET) {
        v_head = (uint32_t)__shfl((int)scan.rv, 0);
        v_tail = a.list[rp_seg_search_wave(a.ioff, 0, count - 1, min(total, c_end * PULL_CHUNK) - 1u)];
    }
    }
    if (DET && lane == 0)                                         // the runs of this wavefront's numbers that do not exist
        for (; run < a.side_runs; run += nw) a.side_v[2 * run] = a.side_v[2 * run + 1] = NONE;
}

// The same hop from the list of its messages. A pull finds the messages by testing every in-neighbour of every vertex
// of A_l against the bitmap of A_{l-1}; when few of them carry a message (hop 2 of a large batch on the dense
// graph: 4.6 M of 110 M), those tests, each a request to the L2 that a compute unit can only have so many of in
// flight, are most of the hop. The out-edge walk that marks A_l has every message in its hands, so it writes them
// down as (destination, source) pairs (k_frontier_mark_pairs), a radix sort (rocPRIM) puts them in destination
// order, and this kernel is the pull's inner part over that list: every wavefront takes a contiguous run of pairs,
// gathers the sources' delta rows G at a time, sums while the destination stays and sends one row of atomic
// additions per destination and wavefront. The host sorts `cap` entries, a number it takes from the previous batch;
// whether the list is used is decided here, like the hop's mode, from the hop's own counters.
struct SortedArgs {
    const uint32_t *pk, *pv;       // sorted: destination, source
    const uint32_t *m_eoff, *m_count;
    uint32_t cap;
    int force;
    const float *D;
    uint32_t ldd, d;
    float *X;
    DevCtr *ctr;
    uint32_t l;
    int mode, ratio, allow_disc;
};

template <int NJ>
__global__ __launch_bounds__(256) void k_scatter_sorted(SortedArgs a) {
    if (rp_hop_mode(a.ctr, a.l, a.d, a.mode, a.ratio, a.allow_disc) != RP_HOP_PULL) return;
    const uint32_t cp = *a.m_count;
    const uint32_t M = cp ? a.m_eoff[cp] : 0u;
    if (!rp_hop_sorted(a.ctr, a.l, M, a.cap, a.force)) return;
    if (blockIdx.x == 0 && threadIdx.x == 0) a.ctr->hop_mode[a.l] = 1u + RP_HOP_SORTED;
    constexpr int G = (NJ >= 8) ? 2 : (NJ == 4 ? 4 : 8 / NJ);   // message rows per round trip (and up to as many destination rows)
    constexpr uint32_t NONE = 0xFFFFFFFFu;
    const int lane = rp_lane();
    const uint32_t d = a.d;
    const uint32_t n_chunks = (M + 63u) / 64u;
    const uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    const uint32_t per = (n_chunks + nw - 1) / nw;
    const uint32_t c_begin = min(n_chunks, gw * per), c_end = min(n_chunks, c_begin + per);
    if (c_begin >= c_end) return;
    // A destination whose pairs all lie inside this wavefront's run has no other writer: its row is read like one
    // more message when its first pair comes up, summed with the messages and stored with plain stores (a row of
    // float atomics costs the L2 one operation per number: 1.5 M rows of 256 took 0.9 ms that way, more than the
    // gathers). Only the destinations of the run's first and last pair can have pairs in a neighbour's run; their sums
    // go to memory as atomic additions.
    const uint32_t v_first = a.pk[c_begin * 64u], v_last = a.pk[min(M, c_end * 64u) - 1u];
    uint32_t cur = NONE;
    float acc[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) acc[j] = 0.0f;
    auto flush = [&]() {
        float *xr = a.X + (size_t)cur * d;
        const bool shared = cur == v_first || cur == v_last;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const uint32_t col = lane + 64 * j;
            if (col < d) {
                if (!shared) xr[col] = acc[j];
                else if (acc[j] != 0.0f) unsafeAtomicAdd(&xr[col], acc[j]);
            }
        }
    };
    uint32_t e = c_begin * 64u + lane;
    uint32_t nv = (e < M) ? a.pk[e] : NONE, nu = (e < M) ? a.pv[e] : 0u;
    for (uint32_t c = c_begin; c < c_end; ++c) {
        const uint32_t my_v = nv, my_u = nu;
        const uint32_t n = min(64u, M - c * 64u);
        e += 64u;                                            // the next chunk's pairs are on their way during the gathers
        nv = (c + 1 < c_end && e < M) ? a.pk[e] : NONE;
        nu = (c + 1 < c_end && e < M) ? a.pv[e] : 0u;
        for (uint32_t k0 = 0; k0 < n; k0 += G) {
            float r[G][NJ], rx[G][NJ];
            uint32_t vk[G];
            uint32_t prev = cur;                             // every pair before k0 has been summed: cur is pair k0 - 1's destination
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const int k = (int)min(k0 + g, 63u);
                const uint32_t uk = (uint32_t)__builtin_amdgcn_readlane((int)my_u, k);
                vk[g] = (uint32_t)__builtin_amdgcn_readlane((int)my_v, k);
                const bool live = k0 + g < n;
                const bool own = live && vk[g] != prev && vk[g] != v_first && vk[g] != v_last;   // first pair of an unshared destination
                prev = vk[g];
#pragma unroll
                for (int j = 0; j < NJ; ++j) {
                    const uint32_t col = lane + 64 * j;
                    r[g][j] = (live && col < d) ? a.D[(size_t)uk * a.ldd + col] : 0.0f;
                    rx[g][j] = (own && col < d) ? a.X[(size_t)vk[g] * d + col] : 0.0f;
                }
            }
#pragma unroll
            for (int g = 0; g < G; ++g) {
                if (k0 + g < n) {
                    if (vk[g] != cur) {
                        if (cur != NONE) flush();
                        cur = vk[g];
#pragma unroll
                        for (int j = 0; j < NJ; ++j) acc[j] = rx[g][j];
                    }
#pragma unroll
                    for (int j = 0; j < NJ; ++j) acc[j] += r[g][j];
                }
            }
        }
    }
    if (cur != NONE) flush();
}

// The same hop for packed message rows (one 128-byte line each, see rp_msg_encode). Decoding a row costs a dozen
// vector instructions whatever the number of lanes that take part, and a wavefront's instruction rate, not the
// memory system, is what bounds a one-line gather; so a row is handled by 16 lanes (8 bytes = three columns
// each) and a wavefront works on four messages, a quad, at a time. The dirty in-edges of a chunk are first
// compacted (source, destination, weight) into LDS in edge order, i.e. sorted by destination; quad k is entries
// 4k .. 4k+3, one per 16-lane group. While all four belong to the destination being summed, every group adds its
// message to its own partial sums. A quad in which the destination changes is taken entry by entry; a change
// first adds the four groups' partial sums together and sends the row to memory as one 47-lane atomic addition
// (the atomic units take about three cycles per lane, so the number of such rows, not of instructions, is what
// counts). The destination and the partial sums carry over from chunk to chunk: a wavefront adds to a row once,
// however many chunks the row's in-edges span.
#define PULL4_QUADS 4                                       // quads (16 rows) in flight per wavefront
#define PULL4_PAD 0xFFFFFFFEu                               // destination of the entries that fill a chunk's last round
template <int DISC, int WT, int DET>
__global__ __launch_bounds__(256) void k_scatter_pull4(PullArgs a) {
    static_assert(!DET || (!DISC && !WT), "the deterministic form pulls into A_l, unweighted");
    if (!DET && rp_hop_mode(a.ctr, a.l, a.d, a.mode, a.ratio, a.allow_disc) != (DISC ? RP_HOP_DISCOVER : RP_HOP_PULL)) return;
    const uint32_t count = *a.count_ptr;
    if (count == 0) return;
    if (blockIdx.x == 0 && threadIdx.x == 0) a.ctr->hop_mode[a.l] = 1u + (DISC ? RP_HOP_DISCOVER : RP_HOP_PULL);
    constexpr int T = PULL_CHUNK / 64;
    constexpr uint32_t NONE = 0xFFFFFFFFu;
    constexpr uint32_t LIST = PULL_CHUNK + 4 * PULL4_QUADS; // a round always reads 4 PULL4_QUADS entries
    // per dirty in-edge: (byte offset of the source's message row, destination); what the inner loop needs per quad
    // is then one 8-byte LDS read and one addition in front of the row's load
    __shared__ uint2 s_e[4][LIST];
    __shared__ float s_w[WT ? 4 : 1][WT ? LIST : 1];
    __shared__ uint8_t s_r[DET ? 4 : 1][DET ? LIST : 1];        // DET: the entry's destination is recomputed
    const int lane = rp_lane(), wave = threadIdx.x >> 6;
    const uint32_t grp = (uint32_t)lane >> 4, sub = (uint32_t)lane & 15u;
    const uint32_t d = a.d;
    const uint32_t total = a.ioff[count];
    const uint32_t n_chunks = (total + PULL_CHUNK - 1) / PULL_CHUNK;
    const uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    // runs of chunks: every nw-th one (DET) or fetched from a counter, see k_scatter_pull
    const uint32_t per = max(1u, min((uint32_t)PULL_RUN, n_chunks / (2u * nw)));
    const uint32_t n_runs = (n_chunks + per - 1) / per;
    uint32_t run = gw;                                      // the first run needs no counter
    if (DET && n_runs > a.side_runs) {                      // cannot happen: the side entries are sized for the in-row pool
        if (gw == 0 && lane == 0) a.ctr->error = 9;
        return;
    }
    if (run >= n_runs) {
        if (DET && lane == 0)
            for (; run < a.side_runs; run += nw) a.side_v[2 * run] = a.side_v[2 * run + 1] = NONE;
        return;
    }
    uint32_t c_begin = run * per;
    uint32_t c_end = min(n_chunks, c_begin + per);
    // message rows through a buffer descriptor: 32-bit byte offsets (row offset from LDS + this lane's chunk)
    const __amdgpu_buffer_rsrc_t mres = __builtin_amdgcn_make_buffer_rsrc((void *)a.D, 0, a.msg_bytes, 0x00020000u);
    const uint32_t sub8 = 8u * sub;
    const uint32_t my_col = 16u * grp + sub;                // the column this lane sends to memory
    const bool sends = grp < 3u && my_col < d;
    uint32_t cur = NONE;                                    // destination being summed (the same in all lanes)
    bool cur_rec = false;                                   // ... and whether it is recomputed (DET)
    float acc0 = 0.0f, acc1 = 0.0f, acc2 = 0.0f;            // this group's partial sums of columns sub, 16 + sub, 32 + sub
    PullScan<T, WT> scan;
    scan.begin(a, count, c_begin, lane);
    uint32_t v_head = NONE, v_tail = NONE;                  // DET: see k_scatter_pull
    bool wrote_head = false, wrote_tail = false;
    if (DET) {
        v_head = (uint32_t)__shfl((int)scan.rv, 0);
        v_tail = a.list[rp_seg_search_wave(a.ioff, 0, count - 1, min(total, c_end * PULL_CHUNK) - 1u)];
    }
    auto flush = [&]() {
        acc0 += __shfl_xor(acc0, 16);
        acc1 += __shfl_xor(acc1, 16);
        acc2 += __shfl_xor(acc2, 16);
        acc0 += __shfl_xor(acc0, 32);
        acc1 += __shfl_xor(acc1, 32);
        acc2 += __shfl_xor(acc2, 32);
        const float mine = grp == 0u ? acc0 : (grp == 1u ? acc1 : acc2);
        if (!DET) {
            if (sends && mine != 0.0f) unsafeAtomicAdd(&a.X[(size_t)cur * d + my_col], mine);
            if (DISC && lane == 0) atomicOr(&a.bm_cur[cur >> 5], 1u << (cur & 31));
        } else if (cur == v_head || cur == v_tail) {
            if (cur == v_head) wrote_head = true;
            else wrote_tail = true;
            if (sends) a.side_acc[(size_t)(2 * run + (cur == v_head ? 0u : 1u)) * d + my_col] = mine;
        } else if (sends) {
            float *x = &a.X[(size_t)cur * d + my_col];
            *x = cur_rec ? mine : *x + mine;
        }
        acc0 = acc1 = acc2 = 0.0f;
    };
    for (;;) {
    for (uint32_t c = c_begin; c < c_end; ++c) {
        const uint32_t e0 = c * PULL_CHUNK, e1 = min(total, e0 + PULL_CHUNK);
        uint32_t my_v[T], my_u[T];
        float my_w[WT ? T : 1];
        bool dirty[T];
        scan.chunk(a, count, e0, e1, lane, my_v, my_u, my_w, dirty);
        // compact the dirty edges, in edge order
        uint32_t n = 0;
#pragma unroll
        for (int t = 0; t < T; ++t) {
            bool rec = false;
            if (DET) {
                rec = a.bm_rec && e0 + 64 * t + lane < e1 && rp_bit(a.bm_rec, my_v[t]);
                dirty[t] = dirty[t] || rec;
            }
            const unsigned long long mask = __ballot(dirty[t]);
            const uint32_t pos = n + __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
            if (dirty[t]) {
                s_e[wave][pos] = make_uint2(my_u[t] << 7, my_v[t]);
                if (WT) s_w[wave][pos] = my_w[t];
                if (DET) s_r[wave][pos] = rec ? 1 : 0;
            }
            n += (uint32_t)__popcll(mask);
        }
        // the entries a round reads past the list's end: row 0 (valid memory), a destination that never matches
        if (lane < 4 * PULL4_QUADS) {
            s_e[wave][n + lane] = make_uint2(0u, PULL4_PAD);
            if (WT) s_w[wave][n + lane] = 0.0f;
            if (DET) s_r[DET ? wave : 0][DET ? n + lane : 0] = 0;
        }
        // LDS accesses of one wavefront are executed in order, so the loads below see the stores above without a
        // workgroup barrier; the fence keeps the compiler from moving them across each other
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const uint32_t n_quads = (n + 3u) >> 2;
        for (uint32_t k0 = 0; k0 < n_quads; k0 += PULL4_QUADS) {
            uint2 ent[PULL4_QUADS];
            float wk[PULL4_QUADS];
            uint2 ch[PULL4_QUADS];
            bool rk[PULL4_QUADS];
            float tv[DET ? PULL4_QUADS : 1][3];              // DET: the three columns of a recomputed row's source
#pragma unroll
            for (int r = 0; r < PULL4_QUADS; ++r) {
                const uint32_t idx = 4u * (k0 + r) + grp;
                ent[r] = s_e[wave][idx];
                if (WT) wk[r] = s_w[wave][idx];
                rk[r] = DET && s_r[DET ? wave : 0][DET ? idx : 0] != 0;
                if (DET && rk[r]) {
                    const float *t = a.R + (size_t)(ent[r].x >> 7) * d;
                    tv[DET ? r : 0][0] = t[sub];
                    tv[DET ? r : 0][1] = t[16u + sub];
                    tv[DET ? r : 0][2] = (32u + sub < d) ? t[32u + sub] : 0.0f;
                    ch[r] = make_uint2(0u, 0u);
                } else {
                    const uintx2 w2 = __builtin_bit_cast(uintx2, __builtin_amdgcn_raw_buffer_load_b64(mres, ent[r].x + sub8, 0, 0));
                    ch[r] = make_uint2(w2.x, w2.y);
                }
            }
#pragma unroll
            for (int r = 0; r < PULL4_QUADS; ++r) {
                const uint32_t k = k0 + r;
                if (k < n_quads) {
                    // the three columns as (integer, as a float) x (the chunk's power of two): one fused
                    // multiply-add per column takes them into the sums (the product is exact)
                    float q0, q1, q2, f;
                    rp_msg_decode_parts(ch[r], q0, q1, q2, f);
                    if (DET && rk[r]) {
                        q0 = tv[DET ? r : 0][0];
                        q1 = tv[DET ? r : 0][1];
                        q2 = tv[DET ? r : 0][2];
                        f = 1.0f;
                    }
                    if (WT) f *= wk[r];                      // a power of two times the weight: exact
                    if (!__any(ent[r].y != cur)) {           // the whole quad goes on
                        acc0 = __builtin_fmaf(q0, f, acc0);
                        acc1 = __builtin_fmaf(q1, f, acc1);
                        acc2 = __builtin_fmaf(q2, f, acc2);
                    } else {                                 // entry by entry (they are sorted by destination)
#pragma unroll
                        for (uint32_t g = 0; g < 4u; ++g) {
                            const uint32_t vg = (uint32_t)__builtin_amdgcn_readlane((int)ent[r].y, 16 * (int)g);
                            if (vg != PULL4_PAD) {
                                if (vg != cur) {
                                    if (cur != NONE) flush();
                                    cur = vg;
                                    if (DET) cur_rec = __builtin_amdgcn_readlane((int)rk[r], 16 * (int)g) != 0;
                                }
                                if (grp == g) {
                                    acc0 = __builtin_fmaf(q0, f, acc0);
                                    acc1 = __builtin_fmaf(q1, f, acc1);
                                    acc2 = __builtin_fmaf(q2, f, acc2);
                                }
                            }
                        }
                    }
                }
            }
        }
        __builtin_amdgcn_wave_barrier();                    // the next chunk overwrites the lists
        scan.advance();
    }
    if (cur != NONE) flush();
    cur = NONE;
    if (DET) {
        if (lane == 0) {
            a.side_v[2 * run] = wrote_head ? v_head : NONE;
            a.side_v[2 * run + 1] = wrote_tail ? v_tail : NONE;
        }
        wrote_head = wrote_tail = false;
        run += nw;
    } else {
        if ((unsigned long long)nw * per >= n_chunks) break;      // every run was somebody's first
        run = nw + rp_next_run(&a.ctr->pull_next[a.l], lane);
    }
    if (run >= n_runs) break;
    c_begin = run * per;
    c_end = min(n_chunks, c_begin + per);
    scan.begin(a, count, c_begin, lane);
    if (DET) {
        v_head = (uint32_t)__shfl((int)scan.rv, 0);
        v_tail = a.list[rp_seg_search_wave(a.ioff, 0, count - 1, min(total, c_end * PULL_CHUNK) - 1u)];
    }
    }
    if (DET && lane == 0)                                         // the runs of this wavefront's numbers that do not exist
        for (; run < a.side_runs; run += nw) a.side_v[2 * run] = a.side_v[2 * run + 1] = NONE;
}

// Deterministic mode, after a DET pull: the side entries (two per run of chunks, in run order; entries of one
// destination are neighbours, apart from empty ones between them) are added up per destination in that order
// and the sum is added to the row, or replaces it if the row is recomputed. One wavefront per entry; the one
// that holds a destination's first entry does the work. Recomputed rows without any in-edge are zeroed here too:
// no in-edge, so the pull never met them.
__global__ __launch_bounds__(256) void k_pull_fixup(PullArgs a, uint32_t n_entries, uint32_t pull_nw) {
    constexpr uint32_t NONE = 0xFFFFFFFFu;
    const uint32_t count = *a.count_ptr;
    if (count == 0) return;
    {   // only the entries of runs that exist can hold anything (the same cut as in the pull kernels)
        const uint32_t n_chunks = (a.ioff[count] + PULL_CHUNK - 1) / PULL_CHUNK;
        const uint32_t per = max(1u, min((uint32_t)PULL_RUN, n_chunks / (2u * pull_nw)));
        n_entries = min(n_entries, 2u * ((n_chunks + per - 1) / per));
    }
    const int lane = rp_lane();
    const uint32_t d = a.d;
    const uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    for (uint32_t i = gw * 64u + lane; a.bm_rec && i < count; i += nw * 64u) {
        const uint32_t v = a.list[i];
        if (a.in_meta[v].y == 0 && rp_bit(a.bm_rec, v))
            for (uint32_t c = 0; c < d; ++c) a.X[(size_t)v * d + c] = 0.0f;
    }
    for (uint32_t k = gw; k < n_entries; k += nw) {
        const uint32_t v = a.side_v[k];
        if (v == NONE) continue;
        // the nearest entry before k that is not empty: the same destination means k is not the first
        bool first = true;
        for (uint32_t b0 = k; b0 > 0;) {
            const uint32_t b = b0 - 1u - (uint32_t)lane;                 // lane 0 looks at the nearest one
            const uint32_t val = ((uint32_t)lane < b0) ? a.side_v[b] : NONE;
            const unsigned long long m = __ballot(val != NONE);
            if (m) {
                first = (uint32_t)__shfl((int)val, __ffsll((long long)m) - 1) != v;
                break;
            }
            b0 = b0 > 64u ? b0 - 64u : 0u;
        }
        if (!first) continue;
        const bool rec = a.bm_rec && rp_bit(a.bm_rec, v);
        for (uint32_t c0 = 0; c0 < d; c0 += 64) {
            const uint32_t col = c0 + lane;
            float t = (col < d) ? a.side_acc[(size_t)k * d + col] : 0.0f;
            bool more = true;
            for (uint32_t f0 = k + 1; f0 < n_entries && more; f0 += 64) {
                const uint32_t f = f0 + (uint32_t)lane;
                const uint32_t val = (f < n_entries) ? a.side_v[f] : NONE;
                unsigned long long same = __ballot(val == v);
                const unsigned long long other = __ballot(val != NONE && val != v);
                if (other) {                                             // entries past the first other destination are not ours
                    same &= (1ull << (__ffsll((long long)other) - 1)) - 1ull;
                    more = false;
                }
                while (same) {
                    const uint32_t e = f0 + (uint32_t)(__ffsll((long long)same) - 1);
                    same &= same - 1;
                    if (col < d) t += a.side_acc[(size_t)e * d + col];
                }
            }
            if (col < d) {
                float *x = &a.X[(size_t)v * d + col];
                *x = rec ? t : *x + t;
            }
        }
    }
}

// discover = false: pull into A_l (the hop's list). true: scan every live vertex (c->all_list and
// c->ioff_all must have been produced by rp_launch_alive_list) and mark the receivers in bm[l].
void rp_launch_scatter_pull(ripple_ctx *c, uint32_t l, bool discover, bool allow_disc, uint32_t pair_cap) {
    PullArgs a;
    a.m_eoff = c->eoff[l - 1];
    a.m_count = &c->ctr->a[l - 1];
    a.sorted_cap = discover ? 0u : pair_cap;
    a.sorted_force = c->opt_sorted == 2;
    a.side_runs = 0;
    a.list = discover ? c->all_list : c->list[l];
    a.count_ptr = discover ? &c->ctr->n_all : &c->ctr->a[l];
    a.ioff = discover ? c->ioff_all : c->ioff[l];
    a.in_meta = c->in_meta;
    a.in_pool = c->in_pool;
    a.bm_prev = c->bm[l - 1];
    a.bm_cur = c->bm[l];
    const bool packed = c->layers[l - 1].proj && c->layers[l - 1].packed;
    a.D = packed ? (const float *)c->MSG : (c->layers[l - 1].proj ? c->PD : c->D[(l - 1) & 1]);
    a.d = c->xw[l];
    a.ldd = c->layers[l - 1].proj ? c->pd_ld : a.d;
    a.msg_bytes = (uint32_t)(c->n_cap * (RP_MSG_WORDS * 4u));   // packed layers exist below 2^25 vertices only
    a.X = c->X[l];
    a.ctr = c->ctr;
    a.l = l;
    a.mode = rp_layer_mode(c, l);
    a.ratio = c->opt_pull_ratio;
    a.allow_disc = allow_disc ? 1 : 0;
    dim3 grid(c->n_cu * 8), block(256);
    const bool wt = c->layers[l - 1].agg == RIPPLE_AGG_WSUM;
    a.in_w = wt ? c->in_w : nullptr;
#define PULL_CASE(NJ)                                                                                      \
    do {                                                                                                   \
        if (discover && wt) hipLaunchKernelGGL((k_scatter_pull<NJ, 1, 1, 0>), grid, block, 0, c->stream, a);  \
        else if (discover) hipLaunchKernelGGL((k_scatter_pull<NJ, 1, 0, 0>), grid, block, 0, c->stream, a);   \
        else if (wt) hipLaunchKernelGGL((k_scatter_pull<NJ, 0, 1, 0>), grid, block, 0, c->stream, a);         \
        else hipLaunchKernelGGL((k_scatter_pull<NJ, 0, 0, 0>), grid, block, 0, c->stream, a);                 \
    } while (0)
    if (packed) {
        if (discover && wt) hipLaunchKernelGGL((k_scatter_pull4<1, 1, 0>), grid, block, 0, c->stream, a);
        else if (discover) hipLaunchKernelGGL((k_scatter_pull4<1, 0, 0>), grid, block, 0, c->stream, a);
        else if (wt) hipLaunchKernelGGL((k_scatter_pull4<0, 1, 0>), grid, block, 0, c->stream, a);
        else hipLaunchKernelGGL((k_scatter_pull4<0, 0, 0>), grid, block, 0, c->stream, a);
    } else if (a.d <= 64) PULL_CASE(1);
    else if (a.d <= 128) PULL_CASE(2);
    else if (a.d <= 256) PULL_CASE(4);
    else if (a.d <= 512) PULL_CASE(8);
    else PULL_CASE(16);
#undef PULL_CASE
}

// Sorts the pairs the out-edge walk wrote (pair_cap entries; the filler key sorts last) and enqueues the kernel that
// scatters from the sorted list. False, and nothing enqueued, if the sort could not be set up: the caller then has
// to launch the pull without a list (pair_cap 0).
bool rp_launch_scatter_sorted(ripple_ctx *c, uint32_t l, bool allow_disc, uint32_t pair_cap) {
    if (!rp_sort_pairs_u32(c, c->pk_a, c->pk_b, c->pv_a, c->pv_b, pair_cap, c->pair_bits, c->pair_tmp, c->pair_tmp_bytes)) return false;
    const LayerDev &ly = c->layers[l - 1];
    SortedArgs a;
    a.pk = c->pk_b;
    a.pv = c->pv_b;
    a.m_eoff = c->eoff[l - 1];
    a.m_count = &c->ctr->a[l - 1];
    a.cap = pair_cap;
    a.force = c->opt_sorted == 2;
    a.D = ly.proj ? c->PD : c->D[(l - 1) & 1];
    a.d = c->xw[l];
    a.ldd = ly.proj ? c->pd_ld : a.d;
    a.X = c->X[l];
    a.ctr = c->ctr;
    a.l = l;
    a.mode = rp_layer_mode(c, l);
    a.ratio = c->opt_pull_ratio;
    a.allow_disc = allow_disc ? 1 : 0;
    dim3 grid(c->n_cu * 8), block(256);
    if (a.d <= 64) hipLaunchKernelGGL((k_scatter_sorted<1>), grid, block, 0, c->stream, a);
    else if (a.d <= 128) hipLaunchKernelGGL((k_scatter_sorted<2>), grid, block, 0, c->stream, a);
    else if (a.d <= 256) hipLaunchKernelGGL((k_scatter_sorted<4>), grid, block, 0, c->stream, a);
    else if (a.d <= 512) hipLaunchKernelGGL((k_scatter_sorted<8>), grid, block, 0, c->stream, a);
    else hipLaunchKernelGGL((k_scatter_sorted<16>), grid, block, 0, c->stream, a);
    return true;
}

// Deterministic mode: the hop is pulled into A_l (bootstrap: into every live vertex, all of them recomputed;
// c->all_list and c->ioff_all must have been produced by rp_launch_alive_list), then the rows that more than
// one wavefront had in-edges of are finished.
void rp_launch_scatter_pull_det(ripple_ctx *c, uint32_t l, bool bootstrap) {
    const LayerDev &ly = c->layers[l - 1];
    PullArgs a;
    a.m_eoff = a.m_count = nullptr;
    a.sorted_cap = 0;
    a.sorted_force = 0;
    a.list = bootstrap ? c->all_list : c->list[l];
    a.count_ptr = bootstrap ? &c->ctr->n_all : &c->ctr->a[l];
    a.ioff = bootstrap ? c->ioff_all : c->ioff[l];
    a.in_meta = c->in_meta;
    a.in_pool = c->in_pool;
    a.in_w = nullptr;
    a.bm_prev = c->bm[l - 1];
    a.bm_cur = c->bm[l];
    const bool packed = ly.proj && ly.packed;
    a.D = packed ? (const float *)c->MSG : (ly.proj ? c->PD : c->D[(l - 1) & 1]);
    a.d = c->xw[l];
    a.ldd = ly.proj ? c->pd_ld : a.d;
    a.msg_bytes = (uint32_t)(c->n_cap * (RP_MSG_WORDS * 4u));
    a.X = c->X[l];
    a.ctr = c->ctr;
    a.l = l;
    a.mode = a.ratio = a.allow_disc = 0;
    a.bm_rec = bootstrap ? c->alive : nullptr;              // bootstrap: every listed vertex is recomputed; batches: none is
    a.Hprev = c->H[l - 1];
    a.R = ly.proj ? ly.T : nullptr;
    a.store = c->store;
    a.side_v = c->side_v;
    a.side_acc = c->side_acc;
    dim3 grid(c->n_cu * 8), block(256);
    a.side_runs = c->side_runs;
    const uint32_t n_entries = 2u * c->side_runs;           // two per run
    if (packed) hipLaunchKernelGGL((k_scatter_pull4<0, 0, 1>), grid, block, 0, c->stream, a);
    else if (a.d <= 64) hipLaunchKernelGGL((k_scatter_pull<1, 0, 0, 1>), grid, block, 0, c->stream, a);
    else if (a.d <= 128) hipLaunchKernelGGL((k_scatter_pull<2, 0, 0, 1>), grid, block, 0, c->stream, a);
    else if (a.d <= 256) hipLaunchKernelGGL((k_scatter_pull<4, 0, 0, 1>), grid, block, 0, c->stream, a);
    else if (a.d <= 512) hipLaunchKernelGGL((k_scatter_pull<8, 0, 0, 1>), grid, block, 0, c->stream, a);
    else hipLaunchKernelGGL((k_scatter_pull<16, 0, 0, 1>), grid, block, 0, c->stream, a);
    hipLaunchKernelGGL(k_pull_fixup, dim3(std::min<uint32_t>(rp_div_up(n_entries, 4), c->n_cu * 32)), block, 0, c->stream, a, n_entries,
                       grid.x * 4u);
}

// ---------------------------------------------------------------------------------
// messages of a project-first layer
// ---------------------------------------------------------------------------------
// For every vertex u of A_{l-1}: P[u] = H^{l-1}[u] W_neigh has just been written to PD[u]. The message is what
// the receivers are still missing, m = P[u] - T[u], in the form it travels in: an fp32 row (left in PD[u];
// T[u] = P[u]) or a packed row (written to MSG[u]; T[u] += the values the packed numbers stand for, so what the
// rounding took away is part of u's next message). 16 lanes per row, three columns (c, 16 + c, 32 + c) each for
// packed rows; four rows per wavefront and step, two steps in flight.
__global__ __launch_bounds__(256) void k_messages(const uint32_t *list, const uint32_t *count_ptr, float *PD, uint32_t ldd,
                                                  float *T, uint32_t d, uint32_t packed, uint32_t *MSG) {
    const uint32_t count = *count_ptr;
    const uint32_t lane = (uint32_t)rp_lane();
    const uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    if (!packed) {                                          // any width: one wavefront per row, element by element
        constexpr int R = 8;
        for (uint32_t s0 = gw * R; s0 < count; s0 += nw * R) {
            uint32_t u[R];
#pragma unroll
            for (int r = 0; r < R; ++r) u[r] = list[min(s0 + r, count - 1u)];
            for (uint32_t col = lane; col < d; col += 64) {
                float p[R], t[R];
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    p[r] = PD[(size_t)u[r] * ldd + col];
                    t[r] = T[(size_t)u[r] * d + col];
                }
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    if (s0 + r >= count) continue;
                    PD[(size_t)u[r] * ldd + col] = p[r] - t[r];
                    T[(size_t)u[r] * d + col] = p[r];
                }
            }
        }
        return;
    }
    constexpr int R = 2;
    const uint32_t grp = lane >> 4, sub = lane & 15u;
    const bool has1 = 16u + sub < d, has2 = 32u + sub < d;
    for (uint32_t s0 = gw * 4u * R; s0 < count; s0 += nw * 4u * R) {
        uint32_t u[R];
        float p[R][3], t[R][3];
#pragma unroll
        for (int r = 0; r < R; ++r) u[r] = list[min(s0 + 4u * r + grp, count - 1u)];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float *pr = PD + (size_t)u[r] * ldd;
            const float *tr = T + (size_t)u[r] * d;
            p[r][0] = pr[sub];
            t[r][0] = tr[sub];
            p[r][1] = has1 ? pr[16u + sub] : 0.0f;
            t[r][1] = has1 ? tr[16u + sub] : 0.0f;
            p[r][2] = has2 ? pr[32u + sub] : 0.0f;
            t[r][2] = has2 ? tr[32u + sub] : 0.0f;
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (s0 + 4u * r + grp >= count) continue;
            float v0, v1, v2;
            const uint2 ch = rp_msg_encode(p[r][0] - t[r][0], p[r][1] - t[r][1], p[r][2] - t[r][2], v0, v1, v2);
            *(uint2 *)(MSG + (size_t)u[r] * RP_MSG_WORDS + 2u * sub) = ch;
            float *tr = T + (size_t)u[r] * d;
            tr[sub] = t[r][0] + v0;
            if (has1) tr[16u + sub] = t[r][1] + v1;
            if (has2) tr[32u + sub] = t[r][2] + v2;
        }
    }
}

void rp_launch_messages(ripple_ctx *c, uint32_t l) {
    const LayerDev &ly = c->layers[l - 1];
    const uint32_t hint = rp_rows_hint(c, l - 1);
    const uint32_t grid = std::max<uint32_t>(1u, std::min<uint32_t>(c->n_cu * 8, rp_div_up(hint, 4 * 8) + 1));
    hipLaunchKernelGGL(k_messages, dim3(grid), dim3(256), 0, c->stream, c->list[l - 1], &c->ctr->a[l - 1], c->PD, c->pd_ld,
                       ly.T, c->xw[l], ly.packed, c->MSG);
}

// ---------------------------------------------------------------------------------
// max / min aggregation: keep, raise or recompute (Sec. 3.4.2)
// ---------------------------------------------------------------------------------
// A message carries the sender's old and new row. The owner of a candidate v (a vertex with a
// changed in-neighbour or a changed in-edge) decides, element by element:
//   * a new value that is at least as good as v's aggregate raises it (incremental case);
//   * an old value that equalled the aggregate and got worse may have been the one that set it; unless
//     another message reaches the aggregate again, the row is recomputed from all in-neighbours;
//   * anything else leaves the element alone.
// Recomputing is always right, so it is also taken where it is the cheaper way: for a created vertex
// and for a vertex with a short in-row whose in-edges changed, where reading the old and new rows of
// the changed in-neighbours would cost as much as reading every in-neighbour once, and as soon as one
// element is known to have lost its extreme. A vertex with a long in-row whose in-edges changed treats
// each changed edge as a message: an added edge sends its source's current row (no old value), a deleted
// one its source's pre-batch row as an old value that is gone.
// Rows whose aggregate ends up bit-equal to the old one are taken out of the hop's set again, so they
// are not transformed and send nothing on. There are no atomics on rows and the result does not
// depend on any order. One wavefront owns a candidate with up to long_min (at most MONO_LONG)
// in-neighbours; longer in-rows are queued and taken by a workgroup each, and a very long row that has
// to be recomputed is queued once more, in segments that a workgroup each reads.
#define MONO_LONG 256u
#define MONO_DIRTY_LIST 2048u     // changed in-neighbours of a long row remembered between counting and reading them
#define MONO_EDGE_HITS 1024u      // changed edges of one sink kept as messages; more: recompute
#define MONO_EDGE_SCAN 32768u     // longest list of changed edges a sink's workgroup searches; longer: recompute

struct MonoArgs {
    const uint32_t *list;          // candidates (ascending), or the queue of long rows
    const uint32_t *count_ptr;
    uint32_t *queue, *queue_count; // candidates with long in-rows, left to the workgroup kernel
    const uint2 *in_meta;
    const uint32_t *in_pool;
    const uint32_t *bm_prev;       // A_{l-1}: the in-neighbours whose row changed
    const uint32_t *bm_sink, *bm_vadd;
    uint32_t *bm_cur;              // the candidates on entry, the hop's set on exit
    const float *Dold;             // pre-batch rows of H^{l-1}, valid on A_{l-1}
    const void *Hprev;             // current H^{l-1}
    uint32_t d;
    float *X;
    int keep_prev;                 // the layer reads the vertex's own row: members of A_{l-1} stay in the set
    DevCtr *ctr;
    uint32_t l;
    // the batch's changed edges (source, sink, sign: < 0 deleted), read for sinks with long in-rows
    const uint32_t *st_src, *st_dst;
    const float *st_sign;
    uint32_t struct_cap;
    const uint32_t *alive;
    uint32_t long_min;             // in-rows longer than this (at most MONO_LONG) go to the workgroup kernel
    uint32_t split_min;            // in-rows of at least this many entries (at least ROW_SPLIT_MIN) are recomputed in segments
    uint32_t *out_list, *out_count; // small hops: the vertices that stay in the hop's set are appended here (or null)
    // very long rows that are recomputed: split into segments for k_scatter_mono_seg
    uint32_t *seg_v, *seg_done, *seg_base, *seg_r;
    float *seg_part;
    uint32_t big_cap, seg_cap, seg_ld;
};

template <int IS_MIN>
__device__ __forceinline__ bool mono_better(float a, float b) { return IS_MIN ? a < b : a > b; }

// Messages of the in-neighbours `mask` selects among the 64 ids held one per lane in my_u: inc becomes
// the best new value, lostm (bit j: column lane + 64 j) records elements whose old value equalled the
// aggregate and got worse. stop_early: return true as soon as such an element is not covered by inc.
template <int NJ, int IS_MIN, int STORE, int G>
__device__ __forceinline__ bool mono_messages(const MonoArgs &a, uint32_t my_u, unsigned long long mask, const float *xo,
                                              float *inc, uint32_t &lostm, bool stop_early) {
    const int lane = rp_lane();
    const uint32_t d = a.d;
    while (mask) {
        int kk[G];
        int n = 0;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            kk[g] = 0;
            if (mask) {
                kk[g] = __ffsll((long long)mask) - 1;
                mask &= mask - 1;
                n = g + 1;
            }
        }
        float ro[G][NJ], rn[G][NJ];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const uint32_t u = __shfl(my_u, kk[g]);
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const uint32_t col = lane + 64 * j;
                const bool on = g < n && col < d;
                ro[g][j] = on ? a.Dold[(size_t)u * d + col] : 0.0f;
                rn[g][j] = on ? rp_load_h(a.Hprev, STORE, (size_t)u * d + col) : 0.0f;
            }
        }
        bool need = false;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                if (g < n) {
                    if (mono_better<IS_MIN>(rn[g][j], inc[j])) inc[j] = rn[g][j];
                    if (ro[g][j] == xo[j] && mono_better<IS_MIN>(ro[g][j], rn[g][j])) lostm |= 1u << j;
                }
            }
            if (lane + 64 * j < (int)d && ((lostm >> j) & 1u) && mono_better<IS_MIN>(xo[j], inc[j])) need = true;
        }
        if (stop_early && __ballot(need) != 0ull) return true;
    }
    return false;
}

// Messages of changed in-edges of one sink, held one per lane (u = source, deleted = the edge went away)
// for the lanes in `mask`. A deleted edge sends its source's pre-batch row as a value that is gone: where
// it equalled the aggregate the element may have lost its extreme. An added edge sends the source's
// current row. Bit 31 of lostm: the pre-batch row is no longer there (the source was removed), recompute.
template <int NJ, int IS_MIN, int STORE>
__device__ __forceinline__ void mono_edge_messages(const MonoArgs &a, uint32_t my_u, bool my_deleted,
                                                   unsigned long long mask, const float *xo, float *inc, uint32_t &lostm) {
    const int lane = rp_lane();
    const uint32_t d = a.d;
    while (mask) {
        const int k = __ffsll((long long)mask) - 1;
        mask &= mask - 1;
        const uint32_t u = __shfl(my_u, k);
        const bool deleted = __shfl((int)my_deleted, k) != 0;
        if (deleted && !rp_bit(a.alive, u)) {
            lostm |= 1u << 31;
            continue;
        }
        const bool from_old = deleted && rp_bit(a.bm_prev, u);
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const uint32_t col = lane + 64 * j;
            if (col >= d) continue;
            const float r = from_old ? a.Dold[(size_t)u * d + col] : rp_load_h(a.Hprev, STORE, (size_t)u * d + col);
            if (deleted) {
                if (r == xo[j]) lostm |= 1u << j;
            } else if (mono_better<IS_MIN>(r, inc[j])) {
                inc[j] = r;
            }
        }
    }
}

// best value per column over the rows of the `n_here` in-neighbours held one per lane in my_u, taken
// from lane `first` on in steps of `step`
template <int NJ, int IS_MIN, int STORE, int G>
__device__ __forceinline__ void mono_gather(const MonoArgs &a, uint32_t my_u, int n_here, float *xn) {
    const int lane = rp_lane();
    const uint32_t d = a.d;
    for (int k0 = 0; k0 < n_here; k0 += G) {
        float r[G][NJ];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const bool on = k0 + g < n_here;
            const uint32_t u = __shfl(my_u, min(k0 + g, n_here - 1));
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const uint32_t col = lane + 64 * j;
                r[g][j] = (on && col < d) ? rp_load_h(a.Hprev, STORE, (size_t)u * d + col) : xn[j];
            }
        }
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
                if (mono_better<IS_MIN>(r[g][j], xn[j])) xn[j] = r[g][j];
    }
}

// store the row if it differs from the old one, else take v out of the hop's set; returns "changed"
template <int NJ>
__device__ __forceinline__ bool mono_finish(const MonoArgs &a, uint32_t v, bool created, const float *xo, const float *xn) {
    const int lane = rp_lane();
    const uint32_t d = a.d;
    bool diff = false;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const uint32_t col = lane + 64 * j;
        if (col < d && xn[j] != xo[j]) diff = true;
    }
    const bool changed = __ballot(diff) != 0ull;
    if (changed) {
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const uint32_t col = lane + 64 * j;
            if (col < d) a.X[(size_t)v * d + col] = xn[j];
        }
    }
    if (!changed && !created && !(a.keep_prev && rp_bit(a.bm_prev, v))) {
        if (lane == 0) atomicAnd(&a.bm_cur[v >> 5], ~(1u << (v & 31)));
    } else if (a.out_list && lane == 0) {
        a.out_list[atomicAdd(a.out_count, 1u)] = v;
    }
    return changed;
}

// wavefront gw of nw: the candidates gw, gw + nw, ... of the list
template <int NJ, int IS_MIN, int STORE>
__device__ __forceinline__ void mono_wave_role(const MonoArgs &a, uint32_t gw, uint32_t nw) {
    constexpr int GC = (NJ <= 4) ? 8 : 32 / NJ;                // senders in flight (two rows each)
    constexpr int GR = (NJ <= 2) ? 32 : 64 / NJ;               // rows in flight when recomputing: round trips pace a row
    constexpr int T = MONO_LONG / 64;
    const uint32_t count = *a.count_ptr;
    const int lane = rp_lane();
    const uint32_t d = a.d;
    const float ident = IS_MIN ? INFINITY : -INFINITY;
    uint32_t n_same = 0, n_inc = 0, n_rec = 0;
    for (uint32_t i = gw; i < count; i += nw) {
        const uint32_t v = a.list[i];
        const uint2 m = a.in_meta[v];
        if (m.y > a.long_min) {
            if (lane == 0) {
                if (a.queue) a.queue[atomicAdd(a.queue_count, 1u)] = v;
                else a.ctr->error = 9;                          // the long rows were meant to be sorted out already
            }
            continue;
        }
        const bool created = rp_bit(a.bm_vadd, v);
        float xo[NJ], xn[NJ];
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const uint32_t col = lane + 64 * j;
            xo[j] = (col < d) ? a.X[(size_t)v * d + col] : 0.0f;
        }
        uint32_t my_u[T];
        unsigned long long dmask[T];
        uint32_t nd = 0;
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const uint32_t e = 64 * t + lane;
            my_u[t] = (e < m.y) ? a.in_pool[m.x + e] : 0u;
            dmask[t] = __ballot(e < m.y && rp_bit(a.bm_prev, my_u[t]));
            nd += (uint32_t)__popcll(dmask[t]);
        }
        // reading old and new rows of nd senders against reading m.y rows once
        bool recompute = created || rp_bit(a.bm_sink, v) || 2 * nd >= m.y;
        if (!recompute) {
            float inc[NJ];
            uint32_t lostm = 0;
#pragma unroll
            for (int j = 0; j < NJ; ++j) inc[j] = ident;
#pragma unroll
            for (int t = 0; t < T; ++t)
                if (!recompute && dmask[t])
                    recompute = mono_messages<NJ, IS_MIN, STORE, GC>(a, my_u[t], dmask[t], xo, inc, lostm, true);
#pragma unroll
            for (int j = 0; j < NJ; ++j) xn[j] = mono_better<IS_MIN>(inc[j], xo[j]) ? inc[j] : xo[j];
        }
        if (recompute) {
#pragma unroll
            for (int j = 0; j < NJ; ++j) xn[j] = (m.y == 0) ? 0.0f : ident;     // no in-neighbours: zero
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const int n_here = (int)min(64u, m.y - min(m.y, 64u * t));
                if (n_here > 0) mono_gather<NJ, IS_MIN, STORE, GR>(a, my_u[t], n_here, xn);
            }
        }
        const bool changed = mono_finish<NJ>(a, v, created, xo, xn);
        if (recompute) ++n_rec;
        else if (changed) ++n_inc;
        else ++n_same;
    }
    if (lane == 0) {
        if (n_same) atomicAdd(&a.ctr->mono[0][a.l], n_same);
        if (n_inc) atomicAdd(&a.ctr->mono[1][a.l], n_inc);
        if (n_rec) atomicAdd(&a.ctr->mono[2][a.l], n_rec);
    }
}

template <int NJ, int IS_MIN, int STORE>
__global__ __launch_bounds__(256) void k_scatter_mono(MonoArgs a) {
    mono_wave_role<NJ, IS_MIN, STORE>(a, (blockIdx.x * blockDim.x + threadIdx.x) >> 6, (gridDim.x * blockDim.x) >> 6);
}

// One workgroup of TEAM wavefronts per candidate with a long in-row: wavefront w takes the 64-entry
// blocks w, w + TEAM, ...; the wavefronts' partial results meet in LDS and wavefront 0 finishes the row.
// Workgroup bid of nb: the rows bid, bid + nb, ... of the queue.
template <int NJ, int IS_MIN, int STORE, int TEAM>
__device__ __forceinline__ void mono_team_role(const MonoArgs &a, uint32_t bid, uint32_t nb) {
    constexpr int GC = (NJ <= 4) ? 8 : 32 / NJ;
    constexpr int GR = (NJ <= 2) ? 32 : 64 / NJ;               // rows in flight: a long row is paced by round trips
    __shared__ float s_val[TEAM][NJ * 64];
    __shared__ uint32_t s_lost[TEAM][64];
    constexpr int IDS = 4;                                     // blocks of in-neighbour ids in flight while counting
    __shared__ uint32_t s_dirty[MONO_DIRTY_LIST];              // the changed in-neighbours of the row (while they fit)
    __shared__ uint32_t s_nd;
    __shared__ uint32_t s_flag;
    __shared__ uint32_t s_hit[MONO_EDGE_HITS];                 // the sink's entries in the list of changed edges
    __shared__ uint32_t s_nhit;
    __shared__ uint32_t s_base, s_slot;
    const uint32_t count = *a.count_ptr;
    const uint32_t n_st = a.ctr->n_struct;
    const int lane = rp_lane(), wave = threadIdx.x >> 6;
    const uint32_t d = a.d;
    const float ident = IS_MIN ? INFINITY : -INFINITY;
    for (uint32_t i = bid; i < count; i += nb) {
        const uint32_t v = a.list[i];
        const uint2 m = a.in_meta[v];
        const bool created = rp_bit(a.bm_vadd, v);
        float xo[NJ], xn[NJ];
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const uint32_t col = lane + 64 * j;
            xo[j] = (col < d) ? a.X[(size_t)v * d + col] : 0.0f;
        }
        // the in-neighbours that changed: counted, and listed in LDS while they fit (several blocks of ids
        // are in flight per wavefront: the row is long and each block is two dependent reads)
        if (threadIdx.x == 0) {
            s_nd = 0;
            s_nhit = 0;
        }
        __syncthreads();
        for (uint32_t base = 64u * wave; base < m.y; base += 64u * TEAM * IDS) {
            uint32_t u[IDS];
            bool dirty[IDS];
#pragma unroll
            for (int t = 0; t < IDS; ++t) {
                const uint32_t e = base + 64u * TEAM * t + lane;
                u[t] = (e < m.y) ? a.in_pool[m.x + e] : 0u;
            }
#pragma unroll
            for (int t = 0; t < IDS; ++t) {
                const uint32_t e = base + 64u * TEAM * t + lane;
                dirty[t] = e < m.y && rp_bit(a.bm_prev, u[t]);
            }
#pragma unroll
            for (int t = 0; t < IDS; ++t) {
                const unsigned long long mask = __ballot(dirty[t]);
                if (!mask) continue;
                uint32_t pos = 0;
                if (lane == __ffsll((long long)mask) - 1) pos = atomicAdd(&s_nd, (uint32_t)__popcll(mask));
                pos = __shfl(pos, __ffsll((long long)mask) - 1) + (uint32_t)__popcll(mask & ((1ull << lane) - 1ull));
                if (dirty[t] && pos < MONO_DIRTY_LIST) s_dirty[pos] = u[t];
            }
        }
        __syncthreads();
        const uint32_t nd = s_nd;
        // A sink keeps its long row incremental when its changed edges can be looked up: each becomes a message.
        bool recompute = created;
        uint32_t ns = 0;
        if (!recompute && rp_bit(a.bm_sink, v)) {
            if (n_st > a.struct_cap || n_st > MONO_EDGE_SCAN) {
                recompute = true;
            } else {
                for (uint32_t s = threadIdx.x; s < n_st; s += TEAM * 64)
                    if (a.st_dst[s] == v && a.st_sign[s] != 0.0f) {
                        const uint32_t k = atomicAdd(&s_nhit, 1u);
                        if (k < MONO_EDGE_HITS) s_hit[k] = s;
                    }
                __syncthreads();
                ns = s_nhit;
                if (ns > MONO_EDGE_HITS) recompute = true;
            }
        }
        if (2 * (nd + ns) >= m.y) recompute = true;            // old and new rows of the senders against every row once
        if (!recompute) {                                      // every wavefront looks at its share of the messages
            float inc[NJ];
            uint32_t lostm = 0;
#pragma unroll
            for (int j = 0; j < NJ; ++j) inc[j] = ident;
            if (nd <= MONO_DIRTY_LIST) {
                for (uint32_t base = 64u * wave; base < nd; base += 64u * TEAM) {
                    const uint32_t k = base + lane;
                    const uint32_t u = (k < nd) ? s_dirty[k] : 0u;
                    mono_messages<NJ, IS_MIN, STORE, GC>(a, u, __ballot(k < nd), xo, inc, lostm, false);
                }
            } else {
                for (uint32_t base = 64u * wave; base < m.y; base += 64u * TEAM) {
                    const uint32_t e = base + lane;
                    const uint32_t u = (e < m.y) ? a.in_pool[m.x + e] : 0u;
                    const unsigned long long mask = __ballot(e < m.y && rp_bit(a.bm_prev, u));
                    if (mask) mono_messages<NJ, IS_MIN, STORE, GC>(a, u, mask, xo, inc, lostm, false);
                }
            }
            for (uint32_t base = 64u * wave; base < ns; base += 64u * TEAM) {
                const uint32_t k = base + lane;
                const uint32_t s = (k < ns) ? s_hit[k] : 0u;
                const uint32_t u = (k < ns) ? a.st_src[s] : 0u;
                const bool deleted = (k < ns) && a.st_sign[s] < 0.0f;
                mono_edge_messages<NJ, IS_MIN, STORE>(a, u, deleted, __ballot(k < ns), xo, inc, lostm);
            }
#pragma unroll
            for (int j = 0; j < NJ; ++j) s_val[wave][j * 64 + lane] = inc[j];
            s_lost[wave][lane] = lostm;
            __syncthreads();
            if (wave == 0) {
                lostm = 0;
                for (int w = 0; w < TEAM; ++w) lostm |= s_lost[w][lane];
                bool need = (lostm >> 31) != 0;
#pragma unroll
                for (int j = 0; j < NJ; ++j) {
                    float best = s_val[0][j * 64 + lane];
                    for (int w = 1; w < TEAM; ++w) {
                        const float x = s_val[w][j * 64 + lane];
                        if (mono_better<IS_MIN>(x, best)) best = x;
                    }
                    if (lane + 64 * j < (int)d && ((lostm >> j) & 1u) && mono_better<IS_MIN>(xo[j], best)) need = true;
                    xn[j] = mono_better<IS_MIN>(best, xo[j]) ? best : xo[j];
                }
                const bool rec = __ballot(need) != 0ull;
                if (lane == 0) s_flag = rec ? 1u : 0u;
            }
            __syncthreads();
            recompute = s_flag != 0;
            if (!recompute) {
                if (wave == 0) {
                    const bool changed = mono_finish<NJ>(a, v, created, xo, xn);
                    if (lane == 0) atomicAdd(&a.ctr->mono[changed ? 1 : 0][a.l], 1u);
                }
                __syncthreads();                               // the LDS arrays are reused by the next row
                continue;
            }
        }
        // recompute from all in-neighbours (m.y > long_min, so the row is not empty)
        if (m.y >= a.split_min) {
            // One compute unit reads a row of thousands of in-neighbours far too slowly: queue its segments,
            // a workgroup each takes one, the last to finish combines them (k_scatter_mono_seg).
            const uint32_t nseg = (m.y + ROW_SEG - 1) / ROW_SEG;
            if (threadIdx.x == 0) {
                const uint32_t r = atomicAdd(&a.ctr->n_big[a.l], 1u);
                const uint32_t base = atomicAdd(&a.ctr->n_seg[a.l], nseg);
                const bool fits = r < a.big_cap && base < a.seg_cap && nseg <= a.seg_cap - base;
                if (fits) {
                    a.seg_v[r] = v;
                    a.seg_done[r] = 0;
                    a.seg_base[r] = base;
                }
                s_base = base;
                s_slot = fits ? r : SEG_NONE;
            }
            __syncthreads();
            const uint32_t base = s_base, r = s_slot;
            for (uint32_t k = threadIdx.x; k < nseg; k += TEAM * 64)
                if (base < a.seg_cap && k < a.seg_cap - base) a.seg_r[base + k] = r;    // SEG_NONE: skipped there
            __syncthreads();
            if (r != SEG_NONE) continue;                       // (the capacities cover every row: not expected otherwise)
        }
#pragma unroll
        for (int j = 0; j < NJ; ++j) xn[j] = ident;
        const uint32_t chunk = (m.y <= 16u * 64u) ? 16u : 64u;  // shorter rows in finer pieces: every wavefront reads some
        for (uint32_t base = chunk * wave; base < m.y; base += chunk * TEAM) {
            const uint32_t e = base + lane;
            const uint32_t u = ((uint32_t)lane < chunk && e < m.y) ? a.in_pool[m.x + e] : 0u;
            mono_gather<NJ, IS_MIN, STORE, GR>(a, u, (int)min(chunk, m.y - base), xn);
        }
        __syncthreads();                                       // s_val may still be read by wavefront 0 (classification)
#pragma unroll
        for (int j = 0; j < NJ; ++j) s_val[wave][j * 64 + lane] = xn[j];
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                float best = s_val[0][j * 64 + lane];
                for (int w = 1; w < TEAM; ++w) {
                    const float x = s_val[w][j * 64 + lane];
                    if (mono_better<IS_MIN>(x, best)) best = x;
                }
                xn[j] = best;
            }
            mono_finish<NJ>(a, v, created, xo, xn);
            if (lane == 0) atomicAdd(&a.ctr->mono[2][a.l], 1u);
        }
        __syncthreads();
    }
}

template <int NJ, int IS_MIN, int STORE, int TEAM>
__global__ __launch_bounds__(TEAM * 64) void k_scatter_mono_long(MonoArgs a) {
    mono_team_role<NJ, IS_MIN, STORE, TEAM>(a, blockIdx.x, gridDim.x);
}

// Small hops, whose long rows were sorted out while the candidates were listed: both roles in one launch
// (the first team_blocks workgroups take a queued long row each, the wavefronts of the others a short
// candidate each), which saves one of the hop's dependent launches.
template <int NJ, int IS_MIN, int STORE, int TEAM>
__global__ __launch_bounds__(TEAM * 64) void k_scatter_mono_both(MonoArgs a, MonoArgs b, uint32_t team_blocks) {
    if (blockIdx.x < team_blocks) {
        mono_team_role<NJ, IS_MIN, STORE, TEAM>(b, blockIdx.x, team_blocks);
    } else {
        const uint32_t wb = blockIdx.x - team_blocks, nwb = gridDim.x - team_blocks;
        mono_wave_role<NJ, IS_MIN, STORE>(a, (wb * blockDim.x + threadIdx.x) >> 6, (nwb * blockDim.x) >> 6);
    }
}

// One workgroup per queued segment of a very long row that is recomputed: the extreme over the segment's
// ROW_SEG in-neighbours goes to the segment's partial row; the workgroup that finishes a row's last
// segment takes the extreme over the partial rows and finishes the row.
template <int NJ, int IS_MIN, int STORE, int TEAM>
__global__ __launch_bounds__(TEAM * 64) void k_scatter_mono_seg(MonoArgs a) {
    static_assert(TEAM * 64 == ROW_SEG, "one 64-entry block per wavefront");
    constexpr int GR = (NJ <= 2) ? 32 : 64 / NJ;
    __shared__ float s_val[TEAM][NJ * 64];
    const uint32_t n_seg = min(a.ctr->n_seg[a.l], a.seg_cap);
    const int lane = rp_lane(), wave = threadIdx.x >> 6;
    const uint32_t d = a.d;
    const float ident = IS_MIN ? INFINITY : -INFINITY;
    for (uint32_t e = blockIdx.x; e < n_seg; e += gridDim.x) {
        const uint32_t r = a.seg_r[e];
        if (r == SEG_NONE) continue;
        const uint32_t v = a.seg_v[r], first = a.seg_base[r];
        const uint2 m = a.in_meta[v];
        const uint32_t nseg = (m.y + ROW_SEG - 1) / ROW_SEG;
        const uint32_t lo = (e - first) * ROW_SEG, hi = min(m.y, lo + ROW_SEG);
        float xn[NJ];
#pragma unroll
        for (int j = 0; j < NJ; ++j) xn[j] = ident;
        const uint32_t b = lo + 64u * wave;
        if (b < hi) {
            const uint32_t u = (b + lane < hi) ? a.in_pool[m.x + b + lane] : 0u;
            mono_gather<NJ, IS_MIN, STORE, GR>(a, u, (int)min(64u, hi - b), xn);
        }
#pragma unroll
        for (int j = 0; j < NJ; ++j) s_val[wave][j * 64 + lane] = xn[j];
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                float best = s_val[0][j * 64 + lane];
                for (int w = 1; w < TEAM; ++w) {
                    const float x = s_val[w][j * 64 + lane];
                    if (mono_better<IS_MIN>(x, best)) best = x;
                }
                const uint32_t col = lane + 64 * j;
                if (col < d) a.seg_part[(size_t)e * a.seg_ld + col] = best;
            }
            __threadfence();                                   // the partial row is visible before the count moves
            uint32_t last = 0;
            if (lane == 0) last = (atomicAdd(&a.seg_done[r], 1u) == nseg - 1) ? 1u : 0u;
            last = __shfl(last, 0);
            if (last) {
                __threadfence();
                float xo[NJ];
#pragma unroll
                for (int j = 0; j < NJ; ++j) {
                    const uint32_t col = lane + 64 * j;
                    xo[j] = (col < d) ? a.X[(size_t)v * d + col] : 0.0f;
                    xn[j] = ident;
                }
                constexpr int GP = (NJ <= 4) ? 8 : 32 / NJ;     // partial rows requested per round trip
                for (uint32_t k0 = 0; k0 < nseg; k0 += GP) {
                    float x[GP][NJ];
#pragma unroll
                    for (int g = 0; g < GP; ++g) {
                        const float *part = a.seg_part + (size_t)(first + min(k0 + g, nseg - 1)) * a.seg_ld;
#pragma unroll
                        for (int j = 0; j < NJ; ++j) {          // written by other compute units: read past this one's cache
                            const uint32_t col = lane + 64 * j;
                            x[g][j] = (col < d) ? __hip_atomic_load(part + col, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : ident;
                        }
                    }
#pragma unroll
                    for (int g = 0; g < GP; ++g)
#pragma unroll
                        for (int j = 0; j < NJ; ++j)
                            if (mono_better<IS_MIN>(x[g][j], xn[j])) xn[j] = x[g][j];
                }
                mono_finish<NJ>(a, v, rp_bit(a.bm_vadd, v), xo, xn);
                if (lane == 0) atomicAdd(&a.ctr->mono[2][a.l], 1u);
            }
        }
        __syncthreads();
    }
}

// candidates in c->all_list, *count_ptr of them (rp_launch_candidates[_sparse]); D[(l-1)&1] holds the pre-batch rows of A_{l-1}
void rp_launch_scatter_mono(ripple_ctx *c, uint32_t l, const uint32_t *count_ptr, bool listed) {
    MonoArgs a;
    const bool few = c->hints_valid && c->last_cand[l] <= 8192u;
    // few candidates: one wavefront would read a row of 100+ in-neighbours for tens of microseconds with the chip idle
    a.long_min = (few || listed) ? RP_MONO_LISTED_LONG : MONO_LONG;   // (a listed hop's long rows were sorted out with this limit)
    // a full chip is busy whichever workgroup reads a row: only the longest rows are split, so that none is left running
    // alone; in between (up to 128 K candidates) a row of a few thousand entries would still outlast everything else
    const bool some = c->hints_valid && c->last_cand[l] <= 131072u;
    a.split_min = few ? ROW_SPLIT_MIN : (some ? 4u : 64u) * ROW_SPLIT_MIN;
    a.list = c->all_list;
    a.count_ptr = count_ptr;
    // listed: the long rows are in c->eoff[l] already (rp_launch_candidates_sparse), nothing is queued here
    a.queue = listed ? nullptr : c->list[l];    // not written before the hop's set is final
    a.out_list = listed ? c->list[l] : nullptr;
    a.out_count = &c->ctr->a[l];                // zero since the batch began
    a.queue_count = &c->ctr->n_long[l];         // zero since the batch began
    a.in_meta = c->in_meta;
    a.in_pool = c->in_pool;
    a.bm_prev = c->bm[l - 1];
    a.bm_sink = c->bm_sink;
    a.bm_vadd = c->bm_vadd;
    a.bm_cur = c->bm[l];
    a.Dold = c->D[(l - 1) & 1];
    a.Hprev = c->H[l - 1];
    a.d = c->xw[l];
    a.X = c->X[l];
    a.keep_prev = c->layers[l - 1].self_mode != RIPPLE_SELF_NONE ? 1 : 0;
    a.ctr = c->ctr;
    a.l = l;
    a.st_src = c->st_src;
    a.st_dst = c->st_dst;
    a.st_sign = c->st_unit;                         // +1 added, -1 deleted, 0 re-weighted (nothing to a max / min layer)
    a.struct_cap = c->in_w ? 0u : c->struct_cap;   // weighted graphs: the sign carries the weight, sinks recompute
    a.alive = c->alive;
    a.seg_v = c->seg_v;
    a.seg_done = c->seg_done;
    a.seg_base = c->seg_base;
    a.seg_r = c->seg_r;
    a.seg_part = c->seg_part;
    a.big_cap = c->big_cap;
    a.seg_cap = std::min(c->seg_cap, c->seg_limit);
    a.seg_ld = c->seg_ld;
    MonoArgs b = a;
    b.list = listed ? c->eoff[l] : a.queue;
    b.count_ptr = &c->ctr->n_long[l];
    const bool is_min = c->layers[l - 1].agg == RIPPLE_AGG_MIN;
    // few candidates: every workgroup resident at once, so none waits for a slot behind one that holds a long chain of reads
    dim3 grid(c->n_cu * (few ? 4 : 8)), block(256);
#define MONO_PAIR(NJ, MN, ST, TEAM)                                                                          \
    do {                                                                                                     \
        if (listed) {                                                                                        \
            /* every workgroup resident at once: half the compute units' worth for each role */              \
            hipLaunchKernelGGL((k_scatter_mono_both<NJ, MN, ST, TEAM>), dim3(c->n_cu / 2 + (c->n_cu / 2) * (16 / TEAM)), \
                               dim3(TEAM * 64), 0, c->stream, a, b, c->n_cu / 2);                            \
        } else {                                                                                             \
            hipLaunchKernelGGL((k_scatter_mono<NJ, MN, ST>), grid, block, 0, c->stream, a);                  \
            hipLaunchKernelGGL((k_scatter_mono_long<NJ, MN, ST, TEAM>), dim3(c->n_cu * 2), dim3(TEAM * 64), 0, c->stream, b); \
        }                                                                                                    \
        hipLaunchKernelGGL((k_scatter_mono_seg<NJ, MN, ST, ROW_SEG / 64>), dim3(c->n_cu * 4), dim3(ROW_SEG), 0, c->stream, b); \
    } while (0)
#define MONO_CASE(NJ, TEAM)                                                                                  \
    do {                                                                                                     \
        if (is_min && c->store) MONO_PAIR(NJ, 1, 1, TEAM);                                                   \
        else if (is_min) MONO_PAIR(NJ, 1, 0, TEAM);                                                          \
        else if (c->store) MONO_PAIR(NJ, 0, 1, TEAM);                                                        \
        else MONO_PAIR(NJ, 0, 0, TEAM);                                                                      \
    } while (0)
    if (a.d <= 64) MONO_CASE(1, 16);
    else if (a.d <= 128) MONO_CASE(2, 16);
    else if (a.d <= 256) MONO_CASE(4, 16);
    else if (a.d <= 512) MONO_CASE(8, 16);
    else MONO_CASE(16, 8);
#undef MONO_CASE
#undef MONO_PAIR
}

// ---------------------------------------------------------------------------------
// bootstrap aggregation: X[v] = sum (op 0), max (1) or min (2) over u in in-row(v) of H_prev[u]
// ---------------------------------------------------------------------------------
template <int NJ, int STORE>
__global__ __launch_bounds__(256) void k_pull_all(const uint2 *in_meta, const uint32_t *in_pool, const float *in_w,
                                                  uint32_t n_cap, const void *Hprev, uint32_t lds, uint32_t d, float *X,
                                                  int op) {
    const int lane = rp_lane();
    const uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    for (uint32_t v = gw; v < n_cap; v += nw) {
        const uint2 m = in_meta[v];
        float acc[NJ];
        const float start = (op == 0 || m.y == 0) ? 0.0f : (op == 1 ? -INFINITY : INFINITY);
#pragma unroll
        for (int j = 0; j < NJ; ++j) acc[j] = start;
        for (uint32_t base = 0; base < m.y; base += 64) {
            const uint32_t i = base + lane;
            const uint32_t my_u = (i < m.y) ? in_pool[m.x + i] : 0u;
            const float my_w = (in_w && i < m.y) ? in_w[m.x + i] : 1.0f;   // edge weight (weighted-sum layers)
            const int n_here = (int)min(64u, m.y - base);
            for (int k = 0; k < n_here; ++k) {
                const uint32_t u = __shfl(my_u, k);
                const float wk = __shfl(my_w, k);
#pragma unroll
                for (int j = 0; j < NJ; ++j) {
                    uint32_t col = lane + 64 * j;
                    if (col < d) {
                        size_t idx = (size_t)u * lds + col;
                        const float x = STORE ? __bfloat162float(((const __hip_bfloat16 *)Hprev)[idx])
                                              : ((const float *)Hprev)[idx];
                        acc[j] = op == 0 ? acc[j] + wk * x : (op == 1 ? fmaxf(acc[j], x) : fminf(acc[j], x));
                    }
                }
            }
        }
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            uint32_t col = lane + 64 * j;
            if (col < d) X[(size_t)v * d + col] = acc[j];
        }
    }
}

// X^l[v] = sum over v's in-row of the previous layer's rows (of their projections, kept in the layer's T,
// for project-first layers)
void rp_launch_pull_all(ripple_ctx *c, uint32_t l) {
    const bool proj = c->layers[l - 1].proj != 0;
    const uint32_t d = c->xw[l];
    const void *src = proj ? (const void *)c->layers[l - 1].T : c->H[l - 1];
    const int store = proj ? 0 : c->store;
    const uint32_t lds = d;
    const float *w = (c->layers[l - 1].agg == RIPPLE_AGG_WSUM) ? c->in_w : nullptr;
    const int op = c->layers[l - 1].agg == RIPPLE_AGG_MAX ? 1 : (c->layers[l - 1].agg == RIPPLE_AGG_MIN ? 2 : 0);
    dim3 grid(c->n_cu * 16), block(256);
#define PULL_CASE(NJ)                                                                                          \
    do {                                                                                                       \
        if (store)                                                                                             \
            hipLaunchKernelGGL((k_pull_all<NJ, 1>), grid, block, 0, c->stream, c->in_meta, c->in_pool, w, c->n_cap, \
                               src, lds, d, c->X[l], op);                                                          \
        else                                                                                                   \
            hipLaunchKernelGGL((k_pull_all<NJ, 0>), grid, block, 0, c->stream, c->in_meta, c->in_pool, w, c->n_cap, \
                               src, lds, d, c->X[l], op);                                                          \
    } while (0)
    if (d <= 64) PULL_CASE(1);
    else if (d <= 128) PULL_CASE(2);
    else if (d <= 256) PULL_CASE(4);
    else if (d <= 512) PULL_CASE(8);
    else PULL_CASE(16);
#undef PULL_CASE
}

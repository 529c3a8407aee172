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

#define seg_search2 rp_seg_search

#define PUSH_CHUNK 64
#define PULL_CHUNK 256

template <int NJ>
__global__ __launch_bounds__(256) void k_scatter_push(const uint32_t *list, const uint32_t *count_ptr,
                                                      const uint32_t *eoff, const float *D, uint32_t ldd, uint32_t d,
                                                      const uint2 *out_meta, const uint32_t *out_pool, float *X,
                                                      const DevCtr *ctr, uint32_t l, int may_pull, int mode, int ratio, int allow_disc) {
    const int hm = rp_hop_mode(ctr, l, d, mode, ratio, allow_disc);
    if (hm == RP_HOP_DISCOVER || (may_pull && hm == RP_HOP_PULL)) return;
    const uint32_t count = *count_ptr;
    if (count == 0) return;
    const int lane = rp_lane();
    const uint32_t M = eoff[count];
    const uint32_t n_chunks = (M + PUSH_CHUNK - 1) / PUSH_CHUNK;
    const uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    for (uint32_t c = gw; c < n_chunks; c += nw) {
        const uint32_t e0 = c * PUSH_CHUNK, e1 = min(M, e0 + PUSH_CHUNK);
        const uint32_t i_lo = seg_search2(eoff, 0, count - 1, e0);
        const uint32_t i_hi = seg_search2(eoff, i_lo, count - 1, e1 - 1);
        const uint32_t e = e0 + lane;
        uint32_t my_i = 0, my_v = 0;
        if (e < e1) {
            my_i = seg_search2(eoff, i_lo, i_hi, e);
            my_v = out_pool[out_meta[list[my_i]].x + (e - eoff[my_i])];
        }
        const int n_here = (int)(e1 - e0);
        uint32_t cur = 0xFFFFFFFFu;
        float dreg[NJ];
        bool nz = false;
        for (int k = 0; k < n_here; ++k) {
            const uint32_t ik = __shfl(my_i, k), vk = __shfl(my_v, k);
            if (ik != cur) {                                    // same for all lanes
                cur = ik;
                const uint32_t uk = list[ik];                   // delta rows are indexed by vertex
                bool any = false;
#pragma unroll
                for (int j = 0; j < NJ; ++j) {
                    uint32_t col = lane + 64 * j;
                    dreg[j] = (col < d) ? D[(size_t)uk * ldd + col] : 0.0f;
                    any |= dreg[j] != 0.0f;
                }
                nz = __ballot(any) != 0ull;
            }
            if (!nz) continue;                                  // an all-zero delta changes nothing
            float *xr = X + (size_t)vk * d;
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                uint32_t col = lane + 64 * j;
                if (col < d) unsafeAtomicAdd(&xr[col], dreg[j]);
            }
        }
    }
}

void rp_launch_scatter_push(ripple_ctx *c, uint32_t l, bool may_pull, bool allow_disc) {
    const bool proj = c->layers[l - 1].proj != 0;           // project-first: messages are already d_out wide
    const uint32_t d = c->xw[l];
    const float *D = proj ? c->PD : c->D[(l - 1) & 1];
    const uint32_t ldd = proj ? c->pd_ld : d;
    dim3 grid(c->n_cu * 8), block(256);
#define PUSH_CASE(NJ)                                                                                         \
    hipLaunchKernelGGL(k_scatter_push<NJ>, grid, block, 0, c->stream, c->list[l - 1], &c->ctr->a[l - 1],      \
                       c->eoff[l - 1], D, ldd, d, c->out_meta, c->out_pool, c->X[l], c->ctr, l, may_pull ? 1 : 0,          \
                       c->opt_scatter, c->opt_pull_ratio, allow_disc ? 1 : 0)
    if (d <= 64) PUSH_CASE(1);
    else if (d <= 128) PUSH_CASE(2);
    else if (d <= 256) PUSH_CASE(4);
    else if (d <= 512) PUSH_CASE(8);
    else PUSH_CASE(16);
#undef PUSH_CASE
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
struct PullArgs {
    const uint32_t *list;          // destinations, ascending
    const uint32_t *count_ptr;
    const uint32_t *ioff;          // in-degree prefix over the list
    const uint2 *in_meta;
    const uint32_t *in_pool;
    const uint32_t *bm_prev;       // A_{l-1} as bitmap
    uint32_t *bm_cur;              // bitmap of A_l: receivers are marked here when discovering
    const float *D;                // delta rows, indexed by vertex
    uint32_t ldd;                  // their row stride
    uint32_t d;
    float *X;
    const DevCtr *ctr;
    uint32_t l;
    int mode, ratio, allow_disc;
};

template <int NJ, int DISC>
__global__ __launch_bounds__(256) void k_scatter_pull(PullArgs a) {
    if (rp_hop_mode(a.ctr, a.l, a.d, a.mode, a.ratio, a.allow_disc) != (DISC ? RP_HOP_DISCOVER : RP_HOP_PULL)) return;
    const uint32_t count = *a.count_ptr;
    if (count == 0) return;
    constexpr int G = (NJ >= 8) ? 2 : 16 / NJ;              // delta rows gathered per round trip
    constexpr int T = PULL_CHUNK / 64;                      // in-edges examined per lane and chunk
    const int lane = rp_lane();
    const uint32_t d = a.d;
    const uint32_t total = a.ioff[count];
    const uint32_t n_chunks = (total + PULL_CHUNK - 1) / PULL_CHUNK;
    const uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    const uint32_t per = (n_chunks + nw - 1) / nw;
    const uint32_t c_begin = min(n_chunks, gw * per), c_end = min(n_chunks, c_begin + per);
    if (c_begin >= c_end) return;
    const uint32_t last = count - 1;
    uint32_t i_lo = rp_seg_search(a.ioff, 0, last, c_begin * PULL_CHUNK);
    // lane j describes row i_lo + j: destination, pool position of edge e is rbase + e (mod 2^32),
    // and bnd = first edge of row i_lo + j + 1 (the total beyond the list's end)
    uint32_t rv, rbase, bnd;
    {
        const uint32_t ri = min(last, i_lo + lane);
        rv = a.list[ri];
        rbase = a.in_meta[rv].x - a.ioff[ri];
        bnd = a.ioff[min(count, i_lo + 1 + lane)];
    }
    for (uint32_t c = c_begin; c < c_end; ++c) {
        const uint32_t e0 = c * PULL_CHUNK, e1 = min(total, e0 + PULL_CHUNK);
        const bool fits = __shfl(bnd, 63) > e1 - 1;         // every row of the chunk is among the 64 held
        uint32_t my_v[T], my_u[T];
        bool dirty[T];
        uint32_t i_nx;
        if (fits) {
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const uint32_t e = e0 + 64 * t + lane;
                const int r = (int)min(63u, rp_count_le(bnd, e));
                my_v[t] = __shfl(rv, r);
                const uint32_t base = __shfl(rbase, r);
                my_u[t] = 0;
                dirty[t] = false;
                if (e < e1) {
                    my_u[t] = a.in_pool[base + e];
                    dirty[t] = (a.bm_prev[my_u[t] >> 5] >> (my_u[t] & 31)) & 1u;
                }
            }
            i_nx = min(last, i_lo + rp_count_le(bnd, e1));
        } else {
            const uint32_t i_hi = rp_seg_forward(a.ioff, i_lo, last, e1 - 1);
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const uint32_t e = e0 + 64 * t + lane;
                my_v[t] = 0;
                my_u[t] = 0;
                dirty[t] = false;
                if (e < e1) {
                    const uint32_t i = rp_seg_search(a.ioff, i_lo, i_hi, e);
                    my_v[t] = a.list[i];
                    my_u[t] = a.in_pool[a.in_meta[my_v[t]].x + (e - a.ioff[i])];
                    dirty[t] = (a.bm_prev[my_u[t] >> 5] >> (my_u[t] & 31)) & 1u;
                }
            }
            i_nx = rp_seg_forward(a.ioff, i_hi, last, e1);
        }
        // rows of the next chunk: in flight while this chunk's messages are gathered
        uint32_t rv_n, rbase_n, bnd_n;
        {
            const uint32_t ri = min(last, i_nx + lane);
            rv_n = a.list[ri];
            rbase_n = a.in_meta[rv_n].x - a.ioff[ri];
            bnd_n = a.ioff[min(count, i_nx + 1 + lane)];
        }
        uint32_t cur = 0xFFFFFFFFu;                          // destination whose partial sum is held
        float acc[NJ];
#pragma unroll
        for (int j = 0; j < NJ; ++j) acc[j] = 0.0f;
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
#pragma unroll
                    for (int j = 0; j < NJ; ++j) {
                        const uint32_t col = lane + 64 * j;
                        r[g][j] = (g < n && col < d) ? a.D[(size_t)uk * a.ldd + col] : 0.0f;
                    }
                }
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    if (g < n) {
                        const uint32_t vk = __shfl(my_v[t], kk[g]);
                        if (vk != cur) {                     // the destination changes: flush its partial sum
                            if (cur != 0xFFFFFFFFu) {
                                float *xr = a.X + (size_t)cur * d;
#pragma unroll
                                for (int j = 0; j < NJ; ++j) {
                                    const uint32_t col = lane + 64 * j;
                                    if (col < d && acc[j] != 0.0f) unsafeAtomicAdd(&xr[col], acc[j]);
                                    acc[j] = 0.0f;
                                }
                                if (DISC && lane == 0) atomicOr(&a.bm_cur[cur >> 5], 1u << (cur & 31));   // once per receiver and chunk
                            }
                            cur = vk;
                        }
#pragma unroll
                        for (int j = 0; j < NJ; ++j) acc[j] += r[g][j];
                    }
                }
            }
        }
        if (cur != 0xFFFFFFFFu) {
            float *xr = a.X + (size_t)cur * d;
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const uint32_t col = lane + 64 * j;
                if (col < d && acc[j] != 0.0f) unsafeAtomicAdd(&xr[col], acc[j]);
            }
            if (DISC && lane == 0) atomicOr(&a.bm_cur[cur >> 5], 1u << (cur & 31));   // once per receiver and chunk
        }
        i_lo = i_nx;
        rv = rv_n;
        rbase = rbase_n;
        bnd = bnd_n;
    }
}

// discover = false: pull into A_l (the hop's list). true: scan every live vertex (c->all_list and
// c->ioff_all must have been produced by rp_launch_alive_list) and mark the receivers in bm[l].
void rp_launch_scatter_pull(ripple_ctx *c, uint32_t l, bool discover, bool allow_disc) {
    PullArgs a;
    a.list = discover ? c->all_list : c->list[l];
    a.count_ptr = discover ? &c->ctr->n_all : &c->ctr->a[l];
    a.ioff = discover ? c->ioff_all : c->ioff[l];
    a.in_meta = c->in_meta;
    a.in_pool = c->in_pool;
    a.bm_prev = c->bm[l - 1];
    a.bm_cur = c->bm[l];
    a.D = c->layers[l - 1].proj ? c->PD : c->D[(l - 1) & 1];
    a.d = c->xw[l];
    a.ldd = c->layers[l - 1].proj ? c->pd_ld : a.d;
    a.X = c->X[l];
    a.ctr = c->ctr;
    a.l = l;
    a.mode = c->opt_scatter;
    a.ratio = c->opt_pull_ratio;
    a.allow_disc = allow_disc ? 1 : 0;
    dim3 grid(c->n_cu * 8), block(256);
#define PULL_CASE(NJ)                                                                            \
    do {                                                                                         \
        if (discover) hipLaunchKernelGGL((k_scatter_pull<NJ, 1>), grid, block, 0, c->stream, a); \
        else hipLaunchKernelGGL((k_scatter_pull<NJ, 0>), grid, block, 0, c->stream, a);          \
    } while (0)
    if (a.d <= 64) PULL_CASE(1);
    else if (a.d <= 128) PULL_CASE(2);
    else if (a.d <= 256) PULL_CASE(4);
    else if (a.d <= 512) PULL_CASE(8);
    else PULL_CASE(16);
#undef PULL_CASE
}

// ---------------------------------------------------------------------------------
// bootstrap aggregation: X[v] = sum_{u in in-row(v)} H_prev[u]
// ---------------------------------------------------------------------------------
template <int NJ, int STORE>
__global__ __launch_bounds__(256) void k_pull_all(const uint2 *in_meta, const uint32_t *in_pool, uint32_t n_cap,
                                                  const void *Hprev, uint32_t lds, uint32_t d, float *X) {
    const int lane = rp_lane();
    const uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    for (uint32_t v = gw; v < n_cap; v += nw) {
        const uint2 m = in_meta[v];
        float acc[NJ];
#pragma unroll
        for (int j = 0; j < NJ; ++j) acc[j] = 0.0f;
        for (uint32_t base = 0; base < m.y; base += 64) {
            const uint32_t i = base + lane;
            const uint32_t my_u = (i < m.y) ? in_pool[m.x + i] : 0u;
            const int n_here = (int)min(64u, m.y - base);
            for (int k = 0; k < n_here; ++k) {
                const uint32_t u = __shfl(my_u, k);
#pragma unroll
                for (int j = 0; j < NJ; ++j) {
                    uint32_t col = lane + 64 * j;
                    if (col < d) {
                        size_t idx = (size_t)u * lds + col;
                        acc[j] += STORE ? __bfloat162float(((const __hip_bfloat16 *)Hprev)[idx])
                                        : ((const float *)Hprev)[idx];
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

// X^l[v] = sum over v's in-row of the previous layer's rows (of their projections, kept in PD,
// for project-first layers)
void rp_launch_pull_all(ripple_ctx *c, uint32_t l) {
    const bool proj = c->layers[l - 1].proj != 0;
    const uint32_t d = c->xw[l];
    const void *src = proj ? (const void *)c->PD : c->H[l - 1];
    const int store = proj ? 0 : c->store;
    const uint32_t lds = proj ? c->pd_ld : d;
    dim3 grid(c->n_cu * 16), block(256);
#define PULL_CASE(NJ)                                                                                          \
    do {                                                                                                       \
        if (store)                                                                                             \
            hipLaunchKernelGGL((k_pull_all<NJ, 1>), grid, block, 0, c->stream, c->in_meta, c->in_pool, c->n_cap, \
                               src, lds, d, c->X[l]);                                                          \
        else                                                                                                   \
            hipLaunchKernelGGL((k_pull_all<NJ, 0>), grid, block, 0, c->stream, c->in_meta, c->in_pool, c->n_cap, \
                               src, lds, d, c->X[l]);                                                          \
    } while (0)
    if (d <= 64) PULL_CASE(1);
    else if (d <= 128) PULL_CASE(2);
    else if (d <= 256) PULL_CASE(4);
    else if (d <= 512) PULL_CASE(8);
    else PULL_CASE(16);
#undef PULL_CASE
}

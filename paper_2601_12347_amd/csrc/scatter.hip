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

__device__ __forceinline__ uint32_t seg_search2(const uint32_t *off, uint32_t lo, uint32_t hi, uint32_t e) {
    while (lo < hi) {
        uint32_t mid = (lo + hi + 1) >> 1;
        if (off[mid] <= e) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}

#define PUSH_CHUNK 64
#define PULL_CHUNK 256

// Direction of hop l, decided on the device from the hop's own counters so that no host
// round trip is needed: pulling scans every in-edge of A_l (index + dirty-bit probe, ~8 bytes
// each) but gathers each message once without atomics; pushing touches only the messages but
// pays a read-modify-write per message.
__device__ __forceinline__ bool rp_use_pull(const DevCtr *ctr, uint32_t l, uint32_t d, int mode, int ratio) {
    if (mode == 2) return true;
    if (mode == 1) return false;
    const unsigned long long m = ctr->m[l], in_edges = ctr->isum[l];
    return m > 0 && m * d * 4ull * (unsigned long long)ratio >= 8ull * in_edges;
}

template <int NJ>
__global__ __launch_bounds__(256) void k_scatter_push(const uint32_t *list, const uint32_t *count_ptr,
                                                      const uint32_t *eoff, const float *D, uint32_t ldd, uint32_t d,
                                                      const uint2 *out_meta, const uint32_t *out_pool, float *X,
                                                      const DevCtr *ctr, uint32_t l, int may_pull, int mode, int ratio) {
    if (may_pull && rp_use_pull(ctr, l, d, mode, ratio)) return;
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

void rp_launch_scatter_push(ripple_ctx *c, uint32_t l, bool may_pull) {
    const bool proj = c->layers[l - 1].proj != 0;           // project-first: messages are already d_out wide
    const uint32_t d = c->xw[l];
    const float *D = proj ? c->PD : c->D[(l - 1) & 1];
    const uint32_t ldd = proj ? c->pd_ld : d;
    dim3 grid(c->n_cu * 8), block(256);
#define PUSH_CASE(NJ)                                                                                         \
    hipLaunchKernelGGL(k_scatter_push<NJ>, grid, block, 0, c->stream, c->list[l - 1], &c->ctr->a[l - 1],      \
                       c->eoff[l - 1], D, ldd, d, c->out_meta, c->out_pool, c->X[l], c->ctr, l, may_pull ? 1 : 0,          \
                       c->opt_scatter, c->opt_pull_ratio)
    if (d <= 64) PUSH_CASE(1);
    else if (d <= 128) PUSH_CASE(2);
    else if (d <= 256) PUSH_CASE(4);
    else if (d <= 512) PUSH_CASE(8);
    else PUSH_CASE(16);
#undef PUSH_CASE
}

// ---------------------------------------------------------------------------------
// pull: segmented reduction over the in-rows of A_l, keeping only dirty sources
// ---------------------------------------------------------------------------------
struct PullArgs {
    const uint32_t *list;          // A_l
    const uint32_t *count_ptr;
    const uint32_t *ioff;          // in-degree prefix over A_l
    const uint2 *in_meta;
    const uint32_t *in_pool;
    const uint32_t *bm_prev;       // A_{l-1} as bitmap
    const float *D;                // delta rows, indexed by vertex
    uint32_t ldd;                  // their row stride
    uint32_t d;
    float *X;
    const DevCtr *ctr;
    uint32_t l;
    int mode, ratio;
};

template <int NJ>
__global__ __launch_bounds__(256) void k_scatter_pull(PullArgs a) {
    if (!rp_use_pull(a.ctr, a.l, a.d, a.mode, a.ratio)) return;
    const uint32_t count = *a.count_ptr;
    if (count == 0) return;
    constexpr int G = (NJ >= 8) ? 2 : 16 / NJ;              // delta rows gathered per round trip
    constexpr int T = PULL_CHUNK / 64;                      // in-edges examined per lane and chunk
    const int lane = rp_lane();
    const uint32_t d = a.d;
    const uint32_t total = a.ioff[count];
    const uint32_t n_chunks = (total + PULL_CHUNK - 1) / PULL_CHUNK;
    const uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    for (uint32_t c = gw; c < n_chunks; c += nw) {
        const uint32_t e0 = c * PULL_CHUNK, e1 = min(total, e0 + PULL_CHUNK);
        const uint32_t i_lo = seg_search2(a.ioff, 0, count - 1, e0);
        const uint32_t i_hi = seg_search2(a.ioff, i_lo, count - 1, e1 - 1);
        // every lane resolves its T in-edges first (independent load chains), then the
        // wavefront walks the dirty ones in edge order
        uint32_t my_i[T], slot[T];
        bool dirty[T];
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const uint32_t e = e0 + 64 * t + lane;
            my_i[t] = 0;
            slot[t] = 0;
            dirty[t] = false;
            if (e < e1) {
                my_i[t] = (i_lo == i_hi) ? i_lo : seg_search2(a.ioff, i_lo, i_hi, e);
                const uint32_t u = a.in_pool[a.in_meta[a.list[my_i[t]]].x + (e - a.ioff[my_i[t]])];
                dirty[t] = (a.bm_prev[u >> 5] >> (u & 31)) & 1u;
                slot[t] = u;
            }
        }
        uint32_t cur = i_lo;
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
                    const uint32_t sk = __shfl(slot[t], kk[g]);
#pragma unroll
                    for (int j = 0; j < NJ; ++j) {
                        const uint32_t col = lane + 64 * j;
                        r[g][j] = (g < n && col < d) ? a.D[(size_t)sk * a.ldd + col] : 0.0f;
                    }
                }
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    if (g < n) {
                        const uint32_t ik = __shfl(my_i[t], kk[g]);
                        if (ik != cur) {                     // the destination changes: flush its partial sum
                            float *xr = a.X + (size_t)a.list[cur] * d;
#pragma unroll
                            for (int j = 0; j < NJ; ++j) {
                                const uint32_t col = lane + 64 * j;
                                if (col < d && acc[j] != 0.0f) unsafeAtomicAdd(&xr[col], acc[j]);
                                acc[j] = 0.0f;
                            }
                            cur = ik;
                        }
#pragma unroll
                        for (int j = 0; j < NJ; ++j) acc[j] += r[g][j];
                    }
                }
            }
        }
        float *xr = a.X + (size_t)a.list[cur] * d;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const uint32_t col = lane + 64 * j;
            if (col < d && acc[j] != 0.0f) unsafeAtomicAdd(&xr[col], acc[j]);
        }
    }
}

void rp_launch_scatter_pull(ripple_ctx *c, uint32_t l) {
    PullArgs a;
    a.list = c->list[l];
    a.count_ptr = &c->ctr->a[l];
    a.ioff = c->ioff[l];
    a.in_meta = c->in_meta;
    a.in_pool = c->in_pool;
    a.bm_prev = c->bm[l - 1];
    a.D = c->layers[l - 1].proj ? c->PD : c->D[(l - 1) & 1];
    a.d = c->xw[l];
    a.ldd = c->layers[l - 1].proj ? c->pd_ld : a.d;
    a.X = c->X[l];
    a.ctr = c->ctr;
    a.l = l;
    a.mode = c->opt_scatter;
    a.ratio = c->opt_pull_ratio;
    dim3 grid(c->n_cu * 8), block(256);
    if (a.d <= 64) hipLaunchKernelGGL(k_scatter_pull<1>, grid, block, 0, c->stream, a);
    else if (a.d <= 128) hipLaunchKernelGGL(k_scatter_pull<2>, grid, block, 0, c->stream, a);
    else if (a.d <= 256) hipLaunchKernelGGL(k_scatter_pull<4>, grid, block, 0, c->stream, a);
    else if (a.d <= 512) hipLaunchKernelGGL(k_scatter_pull<8>, grid, block, 0, c->stream, a);
    else hipLaunchKernelGGL(k_scatter_pull<16>, grid, block, 0, c->stream, a);
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

// Graph attention layers (Sec. 3.4.1, Eq. 3), hybrid-incremental.
//
// Layer l keeps, per vertex, the projected row P[v] = H^{l-1}[v] W, its two scores
// s_src[v] = a_src . P[v] and s_dst[v] = a_dst . P[v], and the un-normalised aggregate: the numerator
// X[v] = sum_u w_uv P[u] and the denominator den[v] = sum_u w_uv over v's in-neighbours u, with
// w_uv = exp(LeakyReLU(s_src[u] + s_dst[v])). The row transform is h_v = act(X[v] / den[v] + b).
// After a batch, a vertex of A_l that is itself in A_{l-1} (its own score moved, so every w_uv did), or
// whose in-edges changed, recomputes numerator and denominator from all its in-neighbours; any other
// vertex of A_l receives, per changed in-neighbour u, the message of the paper:
// <w_new P_new[u] - w_old P_old[u], w_new - w_old>. One owner per destination (a wavefront; a workgroup for long
// in-rows), no atomics, a fixed order of additions.
#include "kernels.h"

#define GAT_SLOPE 0.2f
#define GAT_LONG 256u

struct GatArgs {
    const uint32_t *list;          // A_l, or every live vertex (bootstrap), or the queue of long rows
    const uint32_t *count_ptr;
    uint32_t *queue, *queue_count;
    const uint2 *in_meta;
    const uint32_t *in_pool;
    const uint32_t *bm_prev;       // A_{l-1}
    const uint32_t *bm_sink, *bm_vadd;
    const float *P, *Pold;         // projected rows now / before the batch (the latter valid on A_{l-1})
    const float *ssrc, *sold, *sdst;
    uint32_t d;                    // d_out
    float *X, *den;
    int all;                       // bootstrap: recompute every listed row
};

__device__ __forceinline__ float gat_weight(float s_u, float t_v) {
    const float z = s_u + t_v;
    return __expf(z > 0.0f ? z : GAT_SLOPE * z);
}

// One block of up to 64 in-neighbours (id per lane in my_u, `valid` lanes hold one). recompute: all of them
// contribute w P[u]; otherwise the changed ones contribute w_new P[u] - w_old Pold[u]. acc: the wavefront's
// running numerator (column lane + 64 j); returns this lane's share of the denominator and adds the
// magnitude of what it patched (w_new + w_old) to mag.
template <int NJ, int G, bool recompute>
__device__ __forceinline__ float gat_block(const GatArgs &a, uint32_t my_u, bool valid, float t_v, float *acc, float &mag) {
    const int lane = rp_lane();
    const uint32_t d = a.d;
    const bool on = valid && (recompute || rp_bit(a.bm_prev, my_u));     // rp_bit is not evaluated when recomputing
    float wn = 0.0f, wo = 0.0f;
    if (on) {
        wn = gat_weight(a.ssrc[my_u], t_v);
        if (!recompute) wo = gat_weight(a.sold[my_u], t_v);
    }
    unsigned long long mask = __ballot(on);
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
        float rn[G][NJ], ro[recompute ? 1 : G][NJ];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const uint32_t u = __shfl(my_u, kk[g]);
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const uint32_t col = lane + 64 * j;
                const bool in = g < n && col < d;
                rn[g][j] = in ? a.P[(size_t)u * d + col] : 0.0f;
                if (!recompute) ro[g][j] = in ? a.Pold[(size_t)u * d + col] : 0.0f;
            }
        }
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (g < n) {
                const float wnk = __shfl(wn, kk[g]), wok = __shfl(wo, kk[g]);
#pragma unroll
                for (int j = 0; j < NJ; ++j) acc[j] += recompute ? wnk * rn[g][j] : wnk * rn[g][j] - wok * ro[g][j];
            }
        }
    }
    mag += wn + wo;
    return wn - wo;
}

// A patched denominator that is tiny against what was added and taken away has lost its small terms
// (a weight e^z that dropped by many orders of magnitude leaves only rounding residue of itself): such a
// row is recomputed from all its in-neighbours instead.
#define GAT_CANCEL 1e-3f

__device__ __forceinline__ float gat_wave_sum(float x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

template <int NJ>
__global__ __launch_bounds__(256) void k_gat_scatter(GatArgs a) {
    constexpr int G = (NJ <= 1) ? 8 : (NJ <= 2 ? 4 : (NJ <= 4 ? 2 : 1));     // senders in flight (old and new row each)
    constexpr int GR = (NJ <= 1) ? 16 : (NJ <= 16 ? 16 / NJ : 1);             // rows in flight when recomputing
    const uint32_t count = *a.count_ptr;
    const int lane = rp_lane();
    const uint32_t d = a.d;
    const uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    for (uint32_t i = gw; i < count; i += nw) {
        const uint32_t v = a.list[i];
        const uint2 m = a.in_meta[v];
        if (m.y > GAT_LONG) {
            if (lane == 0) a.queue[atomicAdd(a.queue_count, 1u)] = v;
            continue;
        }
        bool recompute = a.all || rp_bit(a.bm_prev, v) || rp_bit(a.bm_sink, v) || rp_bit(a.bm_vadd, v);
        const float t_v = a.sdst[v];
        float acc[NJ];
        float dsum;
        for (;;) {                                             // a second pass only after a cancelled patch
#pragma unroll
            for (int j = 0; j < NJ; ++j) acc[j] = 0.0f;
            dsum = 0.0f;
            float mag = 0.0f;
            for (uint32_t base = 0; base < m.y; base += 64) {
                const uint32_t e = base + lane;
                const uint32_t my_u = (e < m.y) ? a.in_pool[m.x + e] : 0u;
                dsum += recompute ? gat_block<NJ, GR, true>(a, my_u, e < m.y, t_v, acc, mag)
                                  : gat_block<NJ, G, false>(a, my_u, e < m.y, t_v, acc, mag);
            }
            dsum = gat_wave_sum(dsum);
            if (recompute) break;
            mag = gat_wave_sum(mag);
            if (a.den[v] + dsum > GAT_CANCEL * mag) break;
            recompute = true;
        }
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const uint32_t col = lane + 64 * j;
            if (col < d) {
                float *x = a.X + (size_t)v * d + col;
                *x = recompute ? acc[j] : *x + acc[j];
            }
        }
        if (lane == 0) a.den[v] = recompute ? dsum : a.den[v] + dsum;
    }
}

// one workgroup of TEAM wavefronts per long in-row; partial sums meet in LDS and are added in wavefront order
template <int NJ, int TEAM>
__global__ __launch_bounds__(TEAM * 64) void k_gat_scatter_long(GatArgs a) {
    constexpr int G = (NJ <= 1) ? 8 : (NJ <= 2 ? 4 : (NJ <= 4 ? 2 : 1));
    constexpr int GR = (NJ <= 2) ? 16 : 32 / NJ;               // a long row is paced by round trips
    __shared__ float s_val[TEAM][NJ * 64];
    __shared__ float s_den[TEAM], s_mag[TEAM];
    const uint32_t count = *a.count_ptr;
    const int lane = rp_lane(), wave = threadIdx.x >> 6;
    const uint32_t d = a.d;
    for (uint32_t i = blockIdx.x; i < count; i += gridDim.x) {
        const uint32_t v = a.list[i];
        const uint2 m = a.in_meta[v];
        bool recompute = a.all || rp_bit(a.bm_prev, v) || rp_bit(a.bm_sink, v) || rp_bit(a.bm_vadd, v);
        const float t_v = a.sdst[v];
        float acc[NJ];
        for (;;) {                                             // a second pass only after a cancelled patch
#pragma unroll
            for (int j = 0; j < NJ; ++j) acc[j] = 0.0f;
            float dsum = 0.0f, mag = 0.0f;
            for (uint32_t base = 64u * wave; base < m.y; base += 64u * TEAM) {
                const uint32_t e = base + lane;
                const uint32_t my_u = (e < m.y) ? a.in_pool[m.x + e] : 0u;
                dsum += recompute ? gat_block<NJ, GR, true>(a, my_u, e < m.y, t_v, acc, mag)
                                  : gat_block<NJ, G, false>(a, my_u, e < m.y, t_v, acc, mag);
            }
            dsum = gat_wave_sum(dsum);
            mag = gat_wave_sum(mag);
#pragma unroll
            for (int j = 0; j < NJ; ++j) s_val[wave][j * 64 + lane] = acc[j];
            if (lane == 0) {
                s_den[wave] = dsum;
                s_mag[wave] = mag;
            }
            __syncthreads();
            if (recompute) break;
            float dd = 0.0f, mm = 0.0f;                        // every thread takes the same decision
            for (int w = 0; w < TEAM; ++w) {
                dd += s_den[w];
                mm += s_mag[w];
            }
            if (a.den[v] + dd > GAT_CANCEL * mm) break;
            recompute = true;
            __syncthreads();                                   // the partial results are overwritten by the second pass
        }
        if (wave == 0) {
            float dd = 0.0f;
            for (int w = 0; w < TEAM; ++w) dd += s_den[w];
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                float t = 0.0f;
                for (int w = 0; w < TEAM; ++w) t += s_val[w][j * 64 + lane];
                const uint32_t col = lane + 64 * j;
                if (col < d) {
                    float *x = a.X + (size_t)v * d + col;
                    *x = recompute ? t : *x + t;
                }
            }
            if (lane == 0) a.den[v] = recompute ? dd : a.den[v] + dd;
        }
        __syncthreads();
    }
}

// bootstrap: every live vertex (c->all_list, count in ctr->a[0]) is recomputed
void rp_launch_gat_scatter(ripple_ctx *c, uint32_t l, bool bootstrap) {
    const LayerDev &ly = c->layers[l - 1];
    GatArgs a;
    a.list = bootstrap ? c->all_list : c->list[l];
    a.count_ptr = bootstrap ? &c->ctr->a[0] : &c->ctr->a[l];
    a.queue = bootstrap ? c->list[0] : c->all_list;     // scratch that is free at that point
    a.queue_count = &c->ctr->n_long[l];
    a.in_meta = c->in_meta;
    a.in_pool = c->in_pool;
    a.bm_prev = c->bm[l - 1];
    a.bm_sink = c->bm_sink;
    a.bm_vadd = c->bm_vadd;
    a.P = ly.P;
    a.Pold = c->Pold;
    a.ssrc = ly.ssrc;
    a.sold = c->sold;
    a.sdst = ly.sdst;
    a.d = ly.d_out;
    a.X = c->X[l];
    a.den = ly.den;
    a.all = bootstrap ? 1 : 0;
    if (bootstrap) hipMemsetAsync(&c->ctr->n_long[l], 0, 4, c->stream);   // a batch starts with it cleared
    GatArgs b = a;
    b.list = a.queue;
    b.count_ptr = &c->ctr->n_long[l];
    dim3 grid(c->n_cu * 8), block(256);
#define GAT_CASE(NJ, TEAM)                                                                                   \
    do {                                                                                                     \
        hipLaunchKernelGGL((k_gat_scatter<NJ>), grid, block, 0, c->stream, a);                               \
        hipLaunchKernelGGL((k_gat_scatter_long<NJ, TEAM>), dim3(c->n_cu * 2), dim3(TEAM * 64), 0, c->stream, b); \
    } while (0)
    if (a.d <= 64) GAT_CASE(1, 16);
    else if (a.d <= 128) GAT_CASE(2, 16);
    else if (a.d <= 256) GAT_CASE(4, 16);
    else if (a.d <= 512) GAT_CASE(8, 16);
    else GAT_CASE(16, 8);
#undef GAT_CASE
}

// before the projection of A_{l-1} is refreshed: keep the old rows and source scores for the messages
__global__ __launch_bounds__(256) void k_gat_save(const uint32_t *list, const uint32_t *count_ptr, const float *P,
                                                  const float *ssrc, uint32_t d, float *Pold, float *sold) {
    const uint32_t count = *count_ptr;
    const int lane = rp_lane();
    const uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    for (uint32_t i = gw; i < count; i += nw) {
        const uint32_t v = list[i];
        for (uint32_t col = lane; col < d; col += 64) Pold[(size_t)v * d + col] = P[(size_t)v * d + col];
        if (lane == 0) sold[v] = ssrc[v];
    }
}

// s_src[v] = a_src . P[v], s_dst[v] = a_dst . P[v] for the listed vertices (att: a_src then a_dst)
__global__ __launch_bounds__(256) void k_gat_scores(const uint32_t *list, const uint32_t *count_ptr, const float *P,
                                                    const float *att, uint32_t d, float *ssrc, float *sdst) {
    const uint32_t count = *count_ptr;
    const int lane = rp_lane();
    const uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    for (uint32_t i = gw; i < count; i += nw) {
        const uint32_t v = list[i];
        float s = 0.0f, t = 0.0f;
        for (uint32_t col = lane; col < d; col += 64) {
            const float p = P[(size_t)v * d + col];
            s += p * att[col];
            t += p * att[d + col];
        }
        s = gat_wave_sum(s);
        t = gat_wave_sum(t);
        if (lane == 0) {
            ssrc[v] = s;
            sdst[v] = t;
        }
    }
}

void rp_launch_gat_save(ripple_ctx *c, uint32_t l, const uint32_t *list, const uint32_t *count_d) {
    const LayerDev &ly = c->layers[l - 1];
    hipLaunchKernelGGL(k_gat_save, dim3(c->n_cu * 4), dim3(256), 0, c->stream, list, count_d, ly.P, ly.ssrc, ly.d_out,
                       c->Pold, c->sold);
}

void rp_launch_gat_scores(ripple_ctx *c, uint32_t l, const uint32_t *list, const uint32_t *count_d) {
    const LayerDev &ly = c->layers[l - 1];
    hipLaunchKernelGGL(k_gat_scores, dim3(c->n_cu * 4), dim3(256), 0, c->stream, list, count_d, ly.P, ly.att, ly.d_out,
                       ly.ssrc, ly.sdst);
}

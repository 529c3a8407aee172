// Graph attention layers (Sec. 3.4.1, Eq. 3), hybrid-incremental.
//
// Layer l keeps, per vertex, the projected row P[v] = H^{l-1}[v] W, its two scores
// s_src[v] = a_src . P[v] and s_dst[v] = a_dst . P[v], and the un-normalised aggregate: the numerator
// X[v] = sum_u w_uv P[u] and the denominator den[v] = sum_u w_uv over v's in-neighbours u, with
// w_uv = exp(LeakyReLU(s_src[u] + s_dst[v])). The row transform is h_v = act(X[v] / den[v] + b).
// After a batch, a vertex of A_l that is itself in A_{l-1} (its own score moved, so every w_uv did)
// recomputes numerator and denominator from all its in-neighbours; any other vertex of A_l receives, per
// changed in-neighbour u, the message of the paper: <w_new P_new[u] - w_old P_old[u], w_new - w_old>.
// A vertex whose in-edges changed recomputes if its in-row is short; with a long in-row each changed edge
// is a message too (its pre-batch weight and row, added or taken away). One owner per destination (a
// wavefront; a workgroup for long in-rows; a workgroup per 512-entry segment when a very long row is
// recomputed, the last of them adding the segments up in order), no atomics on rows.
#include "kernels.h"

#define GAT_SLOPE 0.2f
#define GAT_LONG 256u
#define GAT_EDGE_HITS 1024u       // changed edges of one sink kept as messages; more: recompute
#define GAT_EDGE_SCAN 32768u      // longest list of changed edges a sink's workgroup searches; longer: recompute

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
    int few;                       // few rows this hop: latency of the longest row matters, not throughput
    uint32_t long_min;             // in-rows longer than this (at most GAT_LONG) go to the workgroup kernel
    uint32_t split_min;            // in-rows of at least this many entries are recomputed in segments (k_gat_scatter_seg)
    uint32_t *n_big, *n_seg;       // split rows / queued segments of this hop
    uint32_t *seg_v, *seg_done, *seg_base, *seg_r;
    float *seg_part;               // per segment: partial numerator (d floats), then the partial denominator
    uint32_t big_cap, seg_cap, seg_ld;
    // the batch's changed edges (source, sink, sign: < 0 deleted), read for sinks with long in-rows
    const uint32_t *st_src, *st_dst;
    const float *st_sign;
    const uint32_t *n_struct;
    uint32_t struct_cap;
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

// Messages of changed in-edges of one sink whose own score stayed (u = source, sgn = +1 added, -1 deleted,
// one per valid lane): the edge's weight and row as they were before the batch. For a deleted edge that
// is what goes away; for an added edge whose source also changed it cancels the old part of the
// changed-source message, which was never in the sums; for an added edge from an unchanged source it is
// the edge's contribution itself.
template <int NJ>
__device__ __forceinline__ float gat_edge_block(const GatArgs &a, uint32_t my_u, float my_sgn, bool valid, float t_v,
                                                float *acc, float &mag) {
    const int lane = rp_lane();
    const uint32_t d = a.d;
    bool from_old = false;
    float w = 0.0f;
    if (valid) {
        from_old = rp_bit(a.bm_prev, my_u);
        w = gat_weight(from_old ? a.sold[my_u] : a.ssrc[my_u], t_v);
    }
    unsigned long long mask = __ballot(valid);
    while (mask) {
        const int k = __ffsll((long long)mask) - 1;
        mask &= mask - 1;
        const uint32_t u = __shfl(my_u, k);
        const float wk = __shfl(w, k) * __shfl(my_sgn, k);
        const float *row = (__shfl((int)from_old, k) ? a.Pold : a.P) + (size_t)u * d;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const uint32_t col = lane + 64 * j;
            if (col < d) acc[j] += wk * row[col];
        }
    }
    mag += w;
    return w * my_sgn;
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

// wavefront gw of nw: the vertices gw, gw + nw, ... of the list
template <int NJ>
__device__ __forceinline__ void gat_wave_role(const GatArgs &a, uint32_t gw, uint32_t nw) {
    constexpr int G = (NJ <= 1) ? 8 : (NJ <= 2 ? 4 : (NJ <= 4 ? 2 : 1));
    constexpr int GR = (NJ <= 1) ? 16 : (NJ <= 16 ? 16 / NJ : 1);
    const uint32_t count = *a.count_ptr;
    const int lane = rp_lane();
    const uint32_t d = a.d;
    for (uint32_t i = gw; i < count; i += nw) {
        const uint32_t v = a.list[i];
        const uint2 m = a.in_meta[v];
        if (m.y > a.long_min) {                                // queued here, or already when the hop's vertices were listed
            if (lane == 0 && a.queue) a.queue[atomicAdd(a.queue_count, 1u)] = v;
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

template <int NJ>
__global__ __launch_bounds__(256) void k_gat_scatter(GatArgs a) {
    gat_wave_role<NJ>(a, (blockIdx.x * blockDim.x + threadIdx.x) >> 6, (gridDim.x * blockDim.x) >> 6);
}

// one workgroup of TEAM wavefronts per long in-row; partial sums meet in LDS and are added in wavefront order.
// Workgroup bid of nb: the rows bid, bid + nb, ... of the queue.
template <int NJ, int TEAM>
__device__ __forceinline__ void gat_team_role(const GatArgs &a, uint32_t bid, uint32_t nb) {
    constexpr int G = (NJ <= 1) ? 8 : (NJ <= 2 ? 4 : (NJ <= 4 ? 2 : 1));
    constexpr int GR = (NJ <= 2) ? 16 : 32 / NJ;
    constexpr int IDS = 4;                                     // blocks of in-neighbour ids in flight while looking for changed ones
    __shared__ float s_val[TEAM][NJ * 64];
    __shared__ float s_den[TEAM], s_mag[TEAM];
    __shared__ uint32_t s_hit[GAT_EDGE_HITS];                  // the sink's entries in the list of changed edges
    __shared__ uint32_t s_nhit, s_base, s_slot;
    const uint32_t count = *a.count_ptr;
    const uint32_t n_st = *a.n_struct;
    const int lane = rp_lane(), wave = threadIdx.x >> 6;
    const uint32_t d = a.d;
    for (uint32_t i = bid; i < count; i += nb) {
        const uint32_t v = a.list[i];
        const uint2 m = a.in_meta[v];
        bool recompute = a.all || rp_bit(a.bm_prev, v) || rp_bit(a.bm_vadd, v);
        // a sink whose own score stayed keeps its long row incremental when its changed edges can be looked up
        uint32_t ns = 0;
        if (!recompute && rp_bit(a.bm_sink, v)) {
            if (n_st > a.struct_cap || n_st > GAT_EDGE_SCAN) {
                recompute = true;
            } else {
                if (threadIdx.x == 0) s_nhit = 0;
                __syncthreads();
                for (uint32_t s = threadIdx.x; s < n_st; s += TEAM * 64)
                    if (a.st_dst[s] == v && a.st_sign[s] != 0.0f) {
                        const uint32_t k = atomicAdd(&s_nhit, 1u);
                        if (k < GAT_EDGE_HITS) s_hit[k] = s;
                    }
                __syncthreads();
                ns = s_nhit;
                if (ns > GAT_EDGE_HITS || 2 * ns >= m.y) recompute = true;
            }
        }
        const float t_v = a.sdst[v];
        float acc[NJ];
        bool queued = false;
        for (;;) {                                             // a second pass only after a cancelled patch
            if (recompute && m.y >= a.split_min) {
                // One compute unit reads a row of thousands of in-neighbours far too slowly: queue its segments,
                // a workgroup each takes one, the last to finish adds them up (k_gat_scatter_seg).
                const uint32_t nseg = (m.y + ROW_SEG - 1) / ROW_SEG;
                if (threadIdx.x == 0) {
                    const uint32_t r = atomicAdd(a.n_big, 1u);
                    const uint32_t base = atomicAdd(a.n_seg, nseg);
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
                if (r != SEG_NONE) {                           // (the queue holds every row unless it is capped: then read it here)
                    queued = true;
                    break;
                }
            }
#pragma unroll
            for (int j = 0; j < NJ; ++j) acc[j] = 0.0f;
            float dsum = 0.0f, mag = 0.0f;
            if (recompute) {
                const uint32_t chunk = (m.y <= 16u * 64u) ? 16u : 64u;   // shorter rows in finer pieces: every wavefront reads some
                for (uint32_t base = chunk * wave; base < m.y; base += chunk * TEAM) {
                    const uint32_t e = base + lane;
                    const bool valid = (uint32_t)lane < chunk && e < m.y;
                    const uint32_t my_u = valid ? a.in_pool[m.x + e] : 0u;
                    dsum += gat_block<NJ, GR, true>(a, my_u, valid, t_v, acc, mag);
                }
            } else {
                if (!a.few) {                                  // the chip is full: block after block
                    for (uint32_t base = 64u * wave; base < m.y; base += 64u * TEAM) {
                        const uint32_t e = base + lane;
                        const uint32_t my_u = (e < m.y) ? a.in_pool[m.x + e] : 0u;
                        dsum += gat_block<NJ, G, false>(a, my_u, e < m.y, t_v, acc, mag);
                    }
                } else
                for (uint32_t base = 64u * wave; base < m.y; base += 64u * TEAM * IDS) {
                    uint32_t u[IDS];
                    bool any[IDS];
#pragma unroll
                    for (int t = 0; t < IDS; ++t) {
                        const uint32_t e = base + 64u * TEAM * t + lane;
                        u[t] = (e < m.y) ? a.in_pool[m.x + e] : 0u;
                    }
#pragma unroll
                    for (int t = 0; t < IDS; ++t) {
                        const uint32_t e = base + 64u * TEAM * t + lane;
                        any[t] = __ballot(e < m.y && rp_bit(a.bm_prev, u[t])) != 0ull;
                    }
#pragma unroll
                    for (int t = 0; t < IDS; ++t) {
                        const uint32_t e = base + 64u * TEAM * t + lane;
                        if (any[t]) dsum += gat_block<NJ, G, false>(a, u[t], e < m.y, t_v, acc, mag);
                    }
                }
                for (uint32_t base = 64u * wave; base < ns; base += 64u * TEAM) {
                    const uint32_t k = base + lane;
                    const uint32_t s = (k < ns) ? s_hit[k] : 0u;
                    const uint32_t u = (k < ns) ? a.st_src[s] : 0u;
                    const float sgn = (k < ns && a.st_sign[s] < 0.0f) ? -1.0f : 1.0f;
                    dsum += gat_edge_block<NJ>(a, u, sgn, k < ns, t_v, acc, mag);
                }
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
        if (queued) continue;
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

template <int NJ, int TEAM>
__global__ __launch_bounds__(TEAM * 64) void k_gat_scatter_long(GatArgs a) {
    gat_team_role<NJ, TEAM>(a, blockIdx.x, gridDim.x);
}

// Small hops, whose long rows were queued while the hop's vertices were listed: both roles in one launch
// (the first team_blocks workgroups take a long row each, the wavefronts of the others a short one each).
template <int NJ, int TEAM>
__global__ __launch_bounds__(TEAM * 64) void k_gat_scatter_both(GatArgs a, GatArgs b, uint32_t team_blocks) {
    if (blockIdx.x < team_blocks) {
        gat_team_role<NJ, TEAM>(b, blockIdx.x, team_blocks);
    } else {
        const uint32_t wb = blockIdx.x - team_blocks, nwb = gridDim.x - team_blocks;
        gat_wave_role<NJ>(a, (wb * blockDim.x + threadIdx.x) >> 6, (nwb * blockDim.x) >> 6);
    }
}

// One workgroup per queued segment of a very long row that is recomputed: numerator and denominator over
// the segment's ROW_SEG in-neighbours go to the segment's partial row; the workgroup that finishes a row's
// last segment adds the partial rows up in segment order and stores the row.
template <int NJ, int TEAM>
__global__ __launch_bounds__(TEAM * 64) void k_gat_scatter_seg(GatArgs a) {
    static_assert(TEAM * 64 == ROW_SEG, "one 64-entry block per wavefront");
    constexpr int GR = (NJ <= 2) ? 32 : 64 / NJ;
    __shared__ float s_val[TEAM][NJ * 64];
    __shared__ float s_den[TEAM];
    const uint32_t n_seg = min(*a.n_seg, a.seg_cap);
    const int lane = rp_lane(), wave = threadIdx.x >> 6;
    const uint32_t d = a.d;
    for (uint32_t e = blockIdx.x; e < n_seg; e += gridDim.x) {
        const uint32_t r = a.seg_r[e];
        if (r == SEG_NONE) continue;
        const uint32_t v = a.seg_v[r], first = a.seg_base[r];
        const uint2 m = a.in_meta[v];
        const uint32_t nseg = (m.y + ROW_SEG - 1) / ROW_SEG;
        const uint32_t lo = (e - first) * ROW_SEG, hi = min(m.y, lo + ROW_SEG);
        const float t_v = a.sdst[v];
        float acc[NJ];
#pragma unroll
        for (int j = 0; j < NJ; ++j) acc[j] = 0.0f;
        float dsum = 0.0f, mag = 0.0f;
        const uint32_t b = lo + 64u * wave;
        if (b < hi) {
            const bool valid = b + lane < hi;
            const uint32_t my_u = valid ? a.in_pool[m.x + b + lane] : 0u;
            dsum = gat_block<NJ, GR, true>(a, my_u, valid, t_v, acc, mag);
        }
        dsum = gat_wave_sum(dsum);
#pragma unroll
        for (int j = 0; j < NJ; ++j) s_val[wave][j * 64 + lane] = acc[j];
        if (lane == 0) s_den[wave] = dsum;
        __syncthreads();
        if (wave == 0) {
            float *part = a.seg_part + (size_t)e * a.seg_ld;
            float dd = 0.0f;
            for (int w = 0; w < TEAM; ++w) dd += s_den[w];
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                float t = 0.0f;
                for (int w = 0; w < TEAM; ++w) t += s_val[w][j * 64 + lane];
                const uint32_t col = lane + 64 * j;
                if (col < d) part[col] = t;
            }
            if (lane == 0) part[d] = dd;
            __threadfence();                                   // the partial row is visible before the count moves
            uint32_t last = 0;
            if (lane == 0) last = (atomicAdd(&a.seg_done[r], 1u) == nseg - 1) ? 1u : 0u;
            last = __shfl(last, 0);
            if (last) {
                __threadfence();
#pragma unroll
                for (int j = 0; j < NJ; ++j) acc[j] = 0.0f;
                dd = 0.0f;
                constexpr int GP = (NJ <= 4) ? 8 : 32 / NJ;     // partial rows requested per round trip
                for (uint32_t k0 = 0; k0 < nseg; k0 += GP) {   // written by other compute units: read past this one's cache
                    float x[GP][NJ], xd[GP];
#pragma unroll
                    for (int g = 0; g < GP; ++g) {
                        const bool on = k0 + g < nseg;
                        const float *p = a.seg_part + (size_t)(first + min(k0 + g, nseg - 1)) * a.seg_ld;
#pragma unroll
                        for (int j = 0; j < NJ; ++j) {
                            const uint32_t col = lane + 64 * j;
                            x[g][j] = (on && col < d) ? __hip_atomic_load(p + col, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.0f;
                        }
                        xd[g] = on ? __hip_atomic_load(p + d, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.0f;
                    }
#pragma unroll
                    for (int g = 0; g < GP; ++g) {              // in segment order
#pragma unroll
                        for (int j = 0; j < NJ; ++j) acc[j] += x[g][j];
                        dd += xd[g];
                    }
                }
#pragma unroll
                for (int j = 0; j < NJ; ++j) {
                    const uint32_t col = lane + 64 * j;
                    if (col < d) a.X[(size_t)v * d + col] = acc[j];
                }
                if (lane == 0) a.den[v] = dd;
            }
        }
        __syncthreads();
    }
}

// bootstrap: every live vertex (c->all_list, count in ctr->a[0]) is recomputed
void rp_launch_gat_scatter(ripple_ctx *c, uint32_t l, bool bootstrap, bool prequeued) {
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
    const bool few = !bootstrap && c->hints_valid && c->last_a[l] <= 8192u;
    // few rows: one wavefront would read a row of 100+ in-neighbours, one workgroup a row of thousands, with the chip idle
    a.few = (few || prequeued) ? 1 : 0;
    a.long_min = (few || prequeued) ? RP_MONO_LISTED_LONG : GAT_LONG;   // (the limit the long rows were queued with)
    const bool some = !bootstrap && c->hints_valid && c->last_a[l] <= 131072u;   // in between: split rows of a few thousand entries
    a.split_min = few ? ROW_SPLIT_MIN : (some ? 4u : 64u) * ROW_SPLIT_MIN;
    a.n_big = &c->ctr->n_big[l];
    a.n_seg = &c->ctr->n_seg[l];
    a.seg_v = c->seg_v;
    a.seg_done = c->seg_done;
    a.seg_base = c->seg_base;
    a.seg_r = c->seg_r;
    a.seg_part = c->seg_part;
    a.big_cap = c->big_cap;
    a.seg_cap = std::min(c->seg_cap, c->seg_limit);
    a.seg_ld = c->seg_ld;
    a.st_src = c->st_src;
    a.st_dst = c->st_dst;
    a.st_sign = c->st_unit;                         // +1 added, -1 deleted, 0 re-weighted (attention ignores edge weights)
    a.n_struct = &c->ctr->n_struct;
    a.struct_cap = (c->in_w || bootstrap) ? 0u : c->struct_cap;   // weighted graphs: the sign carries the weight, sinks recompute
    if (bootstrap) {                                     // a batch starts with them cleared
        hipMemsetAsync(&c->ctr->n_long[l], 0, 4, c->stream);
        hipMemsetAsync(&c->ctr->n_big[l], 0, 4, c->stream);
        hipMemsetAsync(&c->ctr->n_seg[l], 0, 4, c->stream);
    }
    GatArgs b = a;
    b.list = a.queue;
    if (prequeued) a.queue = nullptr;                    // the wavefront role skips the long rows: they are in the queue already
    b.count_ptr = &c->ctr->n_long[l];
    dim3 grid(c->n_cu * (few ? 4 : 8)), block(256);
#define GAT_CASE(NJ, TEAM)                                                                                   \
    do {                                                                                                     \
        if (prequeued) { /* every workgroup resident at once: half the compute units' worth for each role */ \
            hipLaunchKernelGGL((k_gat_scatter_both<NJ, TEAM>), dim3(c->n_cu / 2 + (c->n_cu / 2) * (16 / TEAM)),  \
                               dim3(TEAM * 64), 0, c->stream, a, b, c->n_cu / 2);                            \
        } else {                                                                                             \
            hipLaunchKernelGGL((k_gat_scatter<NJ>), grid, block, 0, c->stream, a);                           \
            hipLaunchKernelGGL((k_gat_scatter_long<NJ, TEAM>), dim3(c->n_cu * 2), dim3(TEAM * 64), 0, c->stream, b); \
        }                                                                                                    \
        hipLaunchKernelGGL((k_gat_scatter_seg<NJ, ROW_SEG / 64>), dim3(c->n_cu * 4), dim3(ROW_SEG), 0, c->stream, b); \
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

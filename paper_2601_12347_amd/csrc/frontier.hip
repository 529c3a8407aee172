// Frontier construction (the per-hop slice of the propagation tree, Sec. 3.3):
//   A_l = (S  u  Out(A_{l-1})  u  [A_{l-1} if the layer reads the vertex's own
//          embedding]  u  V_added)  n  Alive
// as a bitmap and as an ascending list, plus the exclusive scan of out-degrees
// over that list, which lets the next hop's edge walk be split evenly over
// wavefronts regardless of degree skew.
#include "common.h"
#include "kernels.h"

// largest i in [lo, hi] with off[i] <= e   (off is non-decreasing, off[lo] <= e)
__device__ __forceinline__ uint32_t seg_search(const uint32_t *off, uint32_t lo, uint32_t hi, uint32_t e) {
    while (lo < hi) {
        uint32_t mid = (lo + hi + 1) >> 1;
        if (off[mid] <= e) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}

#define MARK_CHUNK 256

// mark the out-neighbours of every vertex of A_{l-1}
__global__ __launch_bounds__(256) void k_frontier_mark(const uint32_t *list, const uint32_t *count_ptr,
                                                       const uint32_t *eoff, const uint2 *out_meta,
                                                       const uint32_t *out_pool, uint32_t *bm) {
    const uint32_t count = *count_ptr;
    if (count == 0) return;
    const int lane = rp_lane();
    const uint32_t gt = blockIdx.x * blockDim.x + threadIdx.x, nt = gridDim.x * blockDim.x;
    const uint32_t M = eoff[count];
    const uint32_t n_chunks = (M + MARK_CHUNK - 1) / MARK_CHUNK;
    const uint32_t gw = gt >> 6, nw = nt >> 6;
    for (uint32_t c = gw; c < n_chunks; c += nw) {
        uint32_t e0 = c * MARK_CHUNK, e1 = min(M, e0 + MARK_CHUNK);
        uint32_t i_lo = seg_search(eoff, 0, count - 1, e0);
        uint32_t i_hi = seg_search(eoff, i_lo, count - 1, e1 - 1);
        for (uint32_t e = e0 + lane; e < e1; e += 64) {
            uint32_t i = seg_search(eoff, i_lo, i_hi, e);
            uint32_t u = list[i];
            uint32_t v = out_pool[out_meta[u].x + (e - eoff[i])];
            rp_set_bit(bm, v);
        }
    }
}

// pass 1: merge the root sets (S, V_added, and the previous hop's set when the layer has a
// self term) into the layer's bitmap, restrict to live vertices, count vertices and
// (optionally) their out-degrees per block of 256 words
__global__ __launch_bounds__(256) void k_frontier_count(uint32_t *bm, const uint32_t *bm_prev, const uint32_t *bm_sink,
                                                        const uint32_t *bm_vadd, const uint32_t *alive, uint32_t n_words,
                                                        const uint2 *out_meta, int want_deg, uint32_t *part_cnt,
                                                        uint32_t *part_deg, uint32_t *rep, uint32_t *touched_out) {
    __shared__ uint32_t sh[12];
    const int tid = threadIdx.x;
    uint32_t idx = blockIdx.x * 256 + tid;
    uint32_t w = 0, tch = 0;
    if (idx < n_words) {
        const uint32_t live = alive[idx];
        w = bm[idx] & live;
        tch = __popc(w);                         // vertices that received at least one message
        if (bm_sink) w |= (bm_sink[idx] | bm_vadd[idx]) & live;
        if (bm_prev) w |= bm_prev[idx] & live;
        bm[idx] = w;
        if (rep && w) rep[idx] |= w;
    }
    uint32_t cnt = __popc(w), deg = 0;
    if (want_deg) {
        uint32_t t = w;
        while (t) {
            uint32_t b = __ffs(t) - 1;
            t &= t - 1;
            deg += out_meta[idx * 32 + b].y;
        }
    }
    for (int o = 32; o > 0; o >>= 1) {
        cnt += __shfl_down(cnt, o);
        deg += __shfl_down(deg, o);
        tch += __shfl_down(tch, o);
    }
    if ((tid & 63) == 0) {
        sh[tid >> 6] = cnt;
        sh[4 + (tid >> 6)] = deg;
        sh[8 + (tid >> 6)] = tch;
    }
    __syncthreads();
    if (tid == 0) {
        part_cnt[blockIdx.x] = sh[0] + sh[1] + sh[2] + sh[3];
        part_deg[blockIdx.x] = sh[4] + sh[5] + sh[6] + sh[7];
        const uint32_t t = sh[8] + sh[9] + sh[10] + sh[11];
        if (touched_out && t) atomicAdd(touched_out, t);
    }
}

// pass 2: write the ascending list and the out-degree prefix
__global__ __launch_bounds__(256) void k_frontier_emit(const uint32_t *bm, uint32_t n_words, const uint2 *out_meta,
                                                       int want_deg, const uint32_t *part_cnt, const uint32_t *part_deg,
                                                       uint32_t *list, uint32_t *eoff, uint32_t *count_out,
                                                       uint32_t *msgs_out) {
    __shared__ uint32_t sh[8];
    __shared__ uint32_t wc[4], wd[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t pc = 0, pd = 0;
    for (uint32_t b = tid; b < blockIdx.x; b += 256) {
        pc += part_cnt[b];
        pd += part_deg[b];
    }
    for (int o = 32; o > 0; o >>= 1) {
        pc += __shfl_down(pc, o);
        pd += __shfl_down(pd, o);
    }
    if (lane == 0) {
        sh[wave] = pc;
        sh[4 + wave] = pd;
    }
    __syncthreads();
    pc = sh[0] + sh[1] + sh[2] + sh[3];
    pd = sh[4] + sh[5] + sh[6] + sh[7];
    uint32_t idx = blockIdx.x * 256 + tid;
    uint32_t w = (idx < n_words) ? bm[idx] : 0u;
    uint32_t cnt = __popc(w), deg = 0;
    if (want_deg) {
        uint32_t t = w;
        while (t) {
            uint32_t b = __ffs(t) - 1;
            t &= t - 1;
            deg += out_meta[idx * 32 + b].y;
        }
    }
    uint32_t ic = cnt, id = deg;
    for (int o = 1; o < 64; o <<= 1) {
        uint32_t tc = __shfl_up(ic, o), td = __shfl_up(id, o);
        if (lane >= o) {
            ic += tc;
            id += td;
        }
    }
    if (lane == 63) {
        wc[wave] = ic;
        wd[wave] = id;
    }
    __syncthreads();
    uint32_t oc = pc + ic - cnt, od = pd + id - deg;
    for (int k = 0; k < wave; ++k) {
        oc += wc[k];
        od += wd[k];
    }
    uint32_t t = w;
    while (t) {
        uint32_t b = __ffs(t) - 1;
        t &= t - 1;
        uint32_t v = idx * 32 + b;
        list[oc] = v;
        if (want_deg) {
            eoff[oc] = od;
            od += out_meta[v].y;
        }
        ++oc;
    }
    if (blockIdx.x == gridDim.x - 1 && tid == 255) {     // oc/od now hold the grand totals
        *count_out = oc;
        if (want_deg) {
            eoff[oc] = od;
            if (msgs_out) *msgs_out = od;
        }
    }
}

// out-degree prefix over an arbitrary (unsorted) list, one workgroup; used for hop 0
__global__ __launch_bounds__(1024) void k_list_eoff(const uint32_t *list, const uint32_t *count_ptr,
                                                    const uint2 *out_meta, uint32_t *eoff, uint32_t *msgs_out) {
    __shared__ uint32_t ws[16];
    __shared__ uint32_t carry;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t count = *count_ptr;
    if (tid == 0) carry = 0;
    __syncthreads();
    for (uint32_t base = 0; base < count; base += 1024) {
        uint32_t i = base + tid;
        uint32_t deg = (i < count) ? out_meta[list[i]].y : 0u;
        uint32_t inc = deg;
        for (int o = 1; o < 64; o <<= 1) {
            uint32_t t = __shfl_up(inc, o);
            if (lane >= o) inc += t;
        }
        if (lane == 63) ws[wave] = inc;
        __syncthreads();
        uint32_t off = carry;
        for (int k = 0; k < wave; ++k) off += ws[k];
        if (i < count) eoff[i] = off + inc - deg;
        __syncthreads();
        if (tid == 1023) carry = off + inc;
        __syncthreads();
    }
    if (tid == 0) {
        eoff[count] = carry;
        if (msgs_out) *msgs_out = carry;
    }
}

void rp_launch_frontier_mark(ripple_ctx *c, uint32_t l) {
    hipLaunchKernelGGL(k_frontier_mark, dim3(c->n_cu * 4), dim3(256), 0, c->stream, c->list[l - 1], &c->ctr->a[l - 1],
                       c->eoff[l - 1], c->out_meta, c->out_pool, c->bm[l]);
}

// bitmap of layer l, merged with S, V_added (and A_{l-1} when self_term) -> list[l], eoff[l], ctr->a[l], ctr->m[l+1]
void rp_launch_frontier_compact(ripple_ctx *c, uint32_t l, bool self_term, bool want_deg, bool accumulate_rep) {
    uint32_t nb = rp_div_up(c->n_words, 256);
    hipLaunchKernelGGL(k_frontier_count, dim3(nb), dim3(256), 0, c->stream, c->bm[l],
                       self_term ? c->bm[l - 1] : (const uint32_t *)nullptr, c->bm_sink, c->bm_vadd, c->alive,
                       c->n_words, c->out_meta, want_deg ? 1 : 0, c->part_cnt, c->part_deg,
                       accumulate_rep ? c->rep[l] : (uint32_t *)nullptr, &c->ctr->touched[l]);
    hipLaunchKernelGGL(k_frontier_emit, dim3(nb), dim3(256), 0, c->stream, c->bm[l], c->n_words, c->out_meta,
                       want_deg ? 1 : 0, c->part_cnt, c->part_deg, c->list[l], c->eoff[l], &c->ctr->a[l],
                       (want_deg && l < RIPPLE_MAX_LAYERS) ? &c->ctr->m[l + 1] : (uint32_t *)nullptr);
}

// any bitmap & alive -> ascending list in `out_list`, count in *count_d (device)
void rp_launch_bitmap_to_list(ripple_ctx *c, uint32_t *bitmap, uint32_t *out_list, uint32_t *count_d) {
    uint32_t nb = rp_div_up(c->n_words, 256);
    hipLaunchKernelGGL(k_frontier_count, dim3(nb), dim3(256), 0, c->stream, bitmap, (const uint32_t *)nullptr,
                       (const uint32_t *)nullptr, (const uint32_t *)nullptr, c->alive, c->n_words, c->out_meta, 0,
                       c->part_cnt, c->part_deg, (uint32_t *)nullptr, (uint32_t *)nullptr);
    hipLaunchKernelGGL(k_frontier_emit, dim3(nb), dim3(256), 0, c->stream, bitmap, c->n_words, c->out_meta, 0,
                       c->part_cnt, c->part_deg, out_list, (uint32_t *)nullptr, count_d, (uint32_t *)nullptr);
}

void rp_launch_list_eoff(ripple_ctx *c, uint32_t l) {
    hipLaunchKernelGGL(k_list_eoff, dim3(1), dim3(1024), 0, c->stream, c->list[l], &c->ctr->a[l], c->out_meta,
                       c->eoff[l], l < RIPPLE_MAX_LAYERS ? &c->ctr->m[l + 1] : (uint32_t *)nullptr);
}

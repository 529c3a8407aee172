// GPU-resident graph store: out- and in-adjacency kept as per-vertex rows with
// slack inside two pools, built from a COO edge list, mutated by batches of
// updates (the Apply step of Sec. 3.3), and compacted when a pool fills up.
//
// A batch is applied in two phases. Validation decides, against the graph as
// it stands, which operations are accepted and how much pool space they need;
// nothing is modified. Only if everything fits does the commit phase run:
// deletions leave tombstones that one wavefront per touched row squeezes out,
// rows that would overflow move to fresh space at the pool's end, additions
// are appended. Deleting a vertex expands into deleting its incident edges
// (Sec. 3.2, vertex deletion). The host guarantees that operations inside one
// launch sequence never touch the same edge twice nor a vertex that the same
// sequence adds or deletes (other than a new vertex's own edges), so all
// operations can be handled in parallel without changing the array-order result.
#include "common.h"
#include "kernels.h"

// ---------------------------------------------------------------------------------
// exclusive scan over uint32 (two kernels: block sums, then per-block prefix + scan)
// ---------------------------------------------------------------------------------
#define SCAN_PER_BLOCK 1024

__device__ __forceinline__ uint32_t block_sum_256(uint32_t v, uint32_t *sh) {
    const int tid = threadIdx.x;
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o);
    if ((tid & 63) == 0) sh[tid >> 6] = v;
    __syncthreads();
    uint32_t t = sh[0] + sh[1] + sh[2] + sh[3];
    __syncthreads();
    return t;
}

__global__ __launch_bounds__(256) void k_scan_partial(const uint32_t *in, uint32_t n, uint32_t *part) {
    __shared__ uint32_t sh[4];
    uint32_t base = blockIdx.x * SCAN_PER_BLOCK + threadIdx.x * 4;
    uint32_t s = 0;
    for (int k = 0; k < 4; ++k)
        if (base + k < n) s += in[base + k];
    uint32_t t = block_sum_256(s, sh);
    if (threadIdx.x == 0) part[blockIdx.x] = t;
}

__global__ __launch_bounds__(256) void k_scan_final(const uint32_t *in, uint32_t *out, uint32_t n,
                                                    const uint32_t *part, uint32_t *total_out) {
    __shared__ uint32_t sh[4];
    __shared__ uint32_t wsum[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t pre = 0;
    for (uint32_t b = tid; b < blockIdx.x; b += 256) pre += part[b];
    pre = block_sum_256(pre, sh);
    uint32_t base = blockIdx.x * SCAN_PER_BLOCK + tid * 4;
    uint32_t v[4], s = 0;
    for (int k = 0; k < 4; ++k) {
        v[k] = (base + k < n) ? in[base + k] : 0u;
        s += v[k];
    }
    uint32_t incl = s;                                  // inclusive scan inside the wavefront
    for (int o = 1; o < 64; o <<= 1) {
        uint32_t t = __shfl_up(incl, o);
        if (lane >= o) incl += t;
    }
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    uint32_t woff = 0;
    for (int w = 0; w < wave; ++w) woff += wsum[w];
    uint32_t run = pre + woff + incl - s;
    for (int k = 0; k < 4; ++k) {
        if (base + k < n) out[base + k] = run;
        run += v[k];
    }
    if (total_out && blockIdx.x == gridDim.x - 1 && tid == 255) *total_out = run;
}

// out[i] = exclusive prefix of in[0..n); *total_out = sum. part: scratch of ceil(n/1024) words.
void rp_exclusive_scan(hipStream_t s, const uint32_t *in, uint32_t *out, uint32_t n, uint32_t *part,
                       uint32_t *total_out) {
    if (n == 0) return;
    uint32_t nb = rp_div_up(n, SCAN_PER_BLOCK);
    hipLaunchKernelGGL(k_scan_partial, dim3(nb), dim3(256), 0, s, in, n, part);
    hipLaunchKernelGGL(k_scan_final, dim3(nb), dim3(256), 0, s, in, out, n, part, total_out);
}

// ---------------------------------------------------------------------------------
// build from COO
// ---------------------------------------------------------------------------------
__global__ void k_degree_count(const uint32_t *src, const uint32_t *dst, uint64_t n_edges, uint32_t n_vertices,
                               uint32_t *deg_out, uint32_t *deg_in, uint32_t *err) {
    uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t e = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n_edges; e += stride) {
        uint32_t s = src[e], d = dst[e];
        if (s >= n_vertices || d >= n_vertices) {
            *err = 1;
            continue;
        }
        atomicAdd(&deg_out[s], 1u);
        atomicAdd(&deg_in[d], 1u);
    }
}

__global__ void k_fresh_caps(const uint32_t *len, const uint32_t *alive, uint32_t n_cap, uint32_t *capv) {
    uint32_t v = blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= n_cap) return;
    uint32_t l = len[v];
    bool live = rp_bit(alive, v);
    capv[v] = (live || l) ? ((l + (l >> 3) + 4u + 3u) & ~3u) : 0u;
}

__global__ void k_meta_len(const uint2 *meta, uint32_t n_cap, uint32_t *len) {
    uint32_t v = blockIdx.x * blockDim.x + threadIdx.x;
    if (v < n_cap) len[v] = meta[v].y;
}

__global__ void k_init_meta(const uint32_t *start, uint32_t n_cap, uint2 *meta) {
    uint32_t v = blockIdx.x * blockDim.x + threadIdx.x;
    if (v < n_cap) meta[v] = make_uint2(start[v], 0u);
}

__global__ void k_fill_rows(const uint32_t *key, const uint32_t *val, const float *wts, uint64_t n_edges,
                            uint2 *meta, uint32_t *pool, float *wpool) {
    uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t e = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n_edges; e += stride) {
        uint32_t k = key[e];
        uint32_t p = atomicAdd(&((uint32_t *)meta)[2 * (size_t)k + 1], 1u);
        pool[meta[k].x + p] = val[e];
        if (wpool) wpool[meta[k].x + p] = wts[e];
    }
}

// In-rows are filled in the order the edges were given (a stable sort by sink has put position e of the
// sorted sequence at offset e - first[sink] of the sink's row), so that their order is a function of the input.
__global__ void k_iota(uint32_t *out, uint64_t n) {
    uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t e = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += stride) out[e] = (uint32_t)e;
}

__global__ void k_fill_in_rows_ordered(const uint32_t *sorted_dst, const uint32_t *sorted_idx, const uint32_t *src,
                                       const float *wts, uint64_t n_edges, const uint32_t *first, const uint2 *meta,
                                       uint32_t *pool, float *wpool) {
    uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t e = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n_edges; e += stride) {
        const uint32_t k = sorted_dst[e], i = sorted_idx[e];
        const size_t at = (size_t)meta[k].x + ((uint32_t)e - first[k]);
        pool[at] = src[i];
        if (wpool) wpool[at] = wts[i];
    }
}

__global__ void k_set_len(uint2 *meta, const uint32_t *len, uint32_t n_cap) {
    uint32_t v = blockIdx.x * blockDim.x + threadIdx.x;
    if (v < n_cap) meta[v].y = len[v];
}

__global__ void k_set_alive_prefix(uint32_t *alive, uint32_t n_words, uint32_t n_vertices) {
    uint32_t w = blockIdx.x * blockDim.x + threadIdx.x;
    if (w >= n_words) return;
    uint32_t lo = w * 32u;
    uint32_t bits = 0;
    if (lo + 32u <= n_vertices) bits = 0xFFFFFFFFu;
    else if (lo < n_vertices) bits = (1u << (n_vertices - lo)) - 1u;
    alive[w] = bits;
}

ripple_status rp_build_graph(ripple_ctx *c, uint32_t n_vertices, uint64_t n_edges, const uint32_t *src_h,
                             const uint32_t *dst_h, const float *w_h) {
    hipStream_t s = c->stream;
    uint32_t *src_d = nullptr, *dst_d = nullptr, *tmp = nullptr, *err_d = nullptr;
    float *w_d = nullptr;
    size_t eb = (size_t)(n_edges ? n_edges : 1) * sizeof(uint32_t);
    RP_HIP(c, hipMalloc(&src_d, eb));
    RP_HIP(c, hipMalloc(&dst_d, eb));
    RP_HIP(c, hipMalloc(&tmp, (size_t)c->n_cap * 4 * 2 + 64));
    RP_HIP(c, hipMalloc(&err_d, 64));
    RP_HIP(c, hipMemsetAsync(err_d, 0, 64, s));
    if (n_edges) {
        RP_HIP(c, hipMemcpyAsync(src_d, src_h, eb, hipMemcpyHostToDevice, s));
        RP_HIP(c, hipMemcpyAsync(dst_d, dst_h, eb, hipMemcpyHostToDevice, s));
        if (w_h) {
            RP_HIP(c, hipMalloc(&w_d, eb));
            RP_HIP(c, hipMemcpyAsync(w_d, w_h, eb, hipMemcpyHostToDevice, s));
        }
    }
    uint32_t *deg_out = tmp, *deg_in = tmp + c->n_cap;
    RP_HIP(c, hipMemsetAsync(tmp, 0, (size_t)c->n_cap * 8, s));
    hipLaunchKernelGGL(k_set_alive_prefix, dim3(rp_div_up(c->n_words, 256)), dim3(256), 0, s, c->alive,
                       c->n_words, n_vertices);
    uint32_t gb = (uint32_t)std::min<uint64_t>(rp_div_up(n_edges ? n_edges : 1, 256), 65536);
    hipLaunchKernelGGL(k_degree_count, dim3(gb), dim3(256), 0, s, src_d, dst_d, n_edges, n_vertices, deg_out,
                       deg_in, err_d);
    uint32_t vb = rp_div_up(c->n_cap, 256);
    // caps -> starts, for both directions; pend_* serve as scratch for the scan output
    hipLaunchKernelGGL(k_fresh_caps, dim3(vb), dim3(256), 0, s, deg_out, c->alive, c->n_cap, c->out_capv);
    hipLaunchKernelGGL(k_fresh_caps, dim3(vb), dim3(256), 0, s, deg_in, c->alive, c->n_cap, c->in_capv);
    rp_exclusive_scan(s, c->out_capv, c->pend_out, c->n_cap, c->part_cnt, &c->ctr->out_top);
    rp_exclusive_scan(s, c->in_capv, c->pend_in, c->n_cap, c->part_deg, &c->ctr->in_top);
    hipLaunchKernelGGL(k_init_meta, dim3(vb), dim3(256), 0, s, c->pend_out, c->n_cap, c->out_meta);
    hipLaunchKernelGGL(k_init_meta, dim3(vb), dim3(256), 0, s, c->pend_in, c->n_cap, c->in_meta);
    uint32_t err_h = 0;
    RP_HIP(c, hipMemcpyAsync(&err_h, err_d, 4, hipMemcpyDeviceToHost, s));
    RP_HIP(c, hipMemcpyAsync(c->ctr_host, c->ctr, sizeof(DevCtr), hipMemcpyDeviceToHost, s));
    RP_HIP(c, hipStreamSynchronize(s));
    ripple_status rc = RIPPLE_OK;
    if (err_h) {
        c->err = "edge endpoint is not a live vertex (id >= n_vertices)";
        rc = RIPPLE_EINVAL;
    } else if (c->ctr_host->out_top > c->pool_cap || c->ctr_host->in_top > c->pool_cap) {
        c->err = "edge_capacity too small for the initial graph";
        rc = RIPPLE_ECAPACITY;
    } else if (n_edges) {
        hipLaunchKernelGGL(k_fill_rows, dim3(gb), dim3(256), 0, s, src_d, dst_d, (const float *)nullptr, n_edges,
                           c->out_meta, c->out_pool, (float *)nullptr);
        // in-rows: stable sort of the edge numbers by sink, then every edge knows its place
        uint32_t *ord = nullptr;
        unsigned key_bits = 1;
        while (key_bits < 32 && (1ull << key_bits) < (unsigned long long)n_vertices) ++key_bits;
        if (hipMalloc(&ord, 3 * eb + (size_t)c->n_cap * 4) != hipSuccess) {
            (void)hipGetLastError();
            c->err = "device allocation for the build failed";
            rc = RIPPLE_ENOMEM;
        } else {
            uint32_t *idx = ord, *sdst = ord + n_edges, *sidx = ord + 2 * n_edges, *first = ord + 3 * n_edges;
            hipLaunchKernelGGL(k_iota, dim3(gb), dim3(256), 0, s, idx, n_edges);
            rc = rp_stable_sort_pairs(c, dst_d, sdst, idx, sidx, (size_t)n_edges, key_bits);
            if (rc == RIPPLE_OK) {
                rp_exclusive_scan(s, deg_in, first, c->n_cap, c->part_deg, nullptr);
                hipLaunchKernelGGL(k_fill_in_rows_ordered, dim3(gb), dim3(256), 0, s, sdst, sidx, src_d, (const float *)w_d,
                                   n_edges, first, c->in_meta, c->in_pool, w_d ? c->in_w : (float *)nullptr);
                hipLaunchKernelGGL(k_set_len, dim3(vb), dim3(256), 0, s, c->in_meta, deg_in, c->n_cap);
            }
            hipStreamSynchronize(s);
            hipFree(ord);
        }
    }
    hipMemsetAsync(c->pend_out, 0, (size_t)c->n_cap * 4, s);
    hipMemsetAsync(c->pend_in, 0, (size_t)c->n_cap * 4, s);
    hipStreamSynchronize(s);
    hipFree(src_d);
    hipFree(dst_d);
    if (w_d) hipFree(w_d);
    hipFree(tmp);
    hipFree(err_d);
    if (rc == RIPPLE_OK) RP_HIP(c, hipGetLastError());
    return rc;
}

// ---------------------------------------------------------------------------------
// compaction: fresh caps, scan, copy every row into a new pool
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_copy_rows(uint2 *meta, const uint32_t *new_start, uint32_t n_cap,
                                                   const uint32_t *old_pool, uint32_t *new_pool, const float *old_w,
                                                   float *new_w) {
    const int lane = rp_lane();
    uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    for (uint32_t v = gw; v < n_cap; v += nw) {
        uint2 m = meta[v];
        uint32_t ns = new_start[v];
        for (uint32_t i = lane; i < m.y; i += 64) new_pool[ns + i] = old_pool[m.x + i];
        if (old_w)
            for (uint32_t i = lane; i < m.y; i += 64) new_w[ns + i] = old_w[m.x + i];
        if (lane == 0) meta[v] = make_uint2(ns, m.y);
    }
}

static ripple_status compact_one(ripple_ctx *c, uint2 *meta, uint32_t *capv, uint32_t **pool, float **wpool,
                                 uint32_t *top_d, uint32_t *scratch_len, uint32_t *scratch_start) {
    hipStream_t s = c->stream;
    uint32_t vb = rp_div_up(c->n_cap, 256);
    uint32_t *new_pool = nullptr;
    float *new_w = nullptr;
    RP_HIP(c, hipMalloc(&new_pool, (size_t)c->pool_cap * 4));
    if (wpool && *wpool) RP_HIP(c, hipMalloc(&new_w, (size_t)c->pool_cap * 4));
    hipLaunchKernelGGL(k_meta_len, dim3(vb), dim3(256), 0, s, meta, c->n_cap, scratch_len);
    hipLaunchKernelGGL(k_fresh_caps, dim3(vb), dim3(256), 0, s, scratch_len, c->alive, c->n_cap, capv);
    rp_exclusive_scan(s, capv, scratch_start, c->n_cap, c->part_cnt, top_d);
    hipLaunchKernelGGL(k_copy_rows, dim3(c->n_cu * 8), dim3(256), 0, s, meta, scratch_start, c->n_cap, *pool,
                       new_pool, (const float *)(new_w ? *wpool : nullptr), new_w);
    RP_HIP(c, hipStreamSynchronize(s));
    hipFree(*pool);
    *pool = new_pool;
    if (new_w) {
        hipFree(*wpool);
        *wpool = new_w;
    }
    return RIPPLE_OK;
}

ripple_status rp_compact(ripple_ctx *c) {
    // pend_* / dead_* are zero between batches and serve as scratch here
    ripple_status rc = compact_one(c, c->out_meta, c->out_capv, &c->out_pool, nullptr, &c->ctr->out_top, c->pend_out,
                                   c->dead_out);
    if (rc != RIPPLE_OK) return rc;
    rc = compact_one(c, c->in_meta, c->in_capv, &c->in_pool, &c->in_w, &c->ctr->in_top, c->pend_in, c->dead_in);
    if (rc != RIPPLE_OK) return rc;
    hipStream_t s = c->stream;
    RP_HIP(c, hipMemsetAsync(c->pend_out, 0, (size_t)c->n_cap * 4, s));
    RP_HIP(c, hipMemsetAsync(c->pend_in, 0, (size_t)c->n_cap * 4, s));
    RP_HIP(c, hipMemsetAsync(c->dead_out, 0, (size_t)c->n_cap * 4, s));
    RP_HIP(c, hipMemsetAsync(c->dead_in, 0, (size_t)c->n_cap * 4, s));
    RP_HIP(c, hipStreamSynchronize(s));
    return RIPPLE_OK;
}

// ---------------------------------------------------------------------------------
// batch application
// ---------------------------------------------------------------------------------
struct MutArgs {
    const ripple_update *ops;
    uint32_t n_ops;
    const float *payload;
    uint32_t *status, *pos_out, *pos_in;
    uint32_t *op_touch;                          // bit 0 accepted edge op, 1 it is an add, 2 / 3 first touch of out-row(u) / in-row(v)
    int defer_touch;                             // large batches: touched-row lists and counts come from k_touch_lists
    uint2 *out_meta, *in_meta;
    uint32_t *out_capv, *in_capv;
    uint32_t *out_pool, *in_pool;
    float *in_w;                                 // edge weights parallel to in_pool, or null
    uint32_t *alive, *vstate;
    uint32_t *pend_out, *pend_in, *dead_out, *dead_in;
    uint32_t *hole_out, *hole_in;                // position of a row's latest tombstone (exact when the row has one)
    uint32_t *touch_out, *touch_in;
    uint32_t touch_cap;
    uint32_t *exp_kind, *exp_a, *exp_b;
    uint32_t *exp_s;                             // structural-list slot of an expanded out-edge (weighted graphs)
    uint32_t exp_cap;
    uint32_t *st_src, *st_dst;
    float *st_sign, *st_unit;
    uint32_t struct_cap;
    uint32_t *bm0, *bm_sink, *bm_vadd;
    uint32_t *list0;
    float *D0;
    DevCtr *ctr;
    uint32_t n_cap;
    unsigned long long e_cap, pool_cap;
    int store;
    uint32_t L;
    uint32_t d[RIPPLE_MAX_LAYERS + 1];
    uint32_t xw[RIPPLE_MAX_LAYERS + 1];          // width of X^l
    void *H[RIPPLE_MAX_LAYERS + 1];
    float *X[RIPPLE_MAX_LAYERS + 1];
    float *T[RIPPLE_MAX_LAYERS + 1];             // project-first layers: what every vertex has sent so far (xw[l] floats per vertex), else null
    uint32_t mono_mask;                          // bit l: layer l takes max / min or attention (no structural terms)
    uint32_t wsum_mask;                          // bit l: layer l aggregates with the edge weights
    int d0_old;                                  // layer 1 does: D0 receives the old feature row instead of the difference
    int det;                                     // deterministic mode: appended in-row entries are put in id order
    uint32_t *tail_ids, *tail_q;                 // ... through a copy (tail_cap entries) and a queue of rows with many of them
    float *tail_w;
    uint32_t tail_cap;
    unsigned long long *sk_in;                   // ... and the changed edges sorted by (sink, source): keys before / after,
    const unsigned long long *sk_out;
    float *sv_in;                                // ... with what each adds to its sink's aggregates (+1 / -1 / 0)
    const float *sv_out;
    uint32_t n_sort;                             // entries the sort takes (those past n_struct hold the largest key)
};

__device__ __forceinline__ void touch_row(const MutArgs &a, uint32_t x, uint32_t bit) {
    uint32_t old = atomicOr(&a.vstate[x], bit);
    if (old & bit) return;
    uint32_t *cnt = (bit == VS_TOUCH_OUT) ? &a.ctr->n_touch_out : &a.ctr->n_touch_in;
    uint32_t *lst = (bit == VS_TOUCH_OUT) ? a.touch_out : a.touch_in;
    uint32_t p = atomicAdd(cnt, 1u);
    if (p < a.touch_cap) lst[p] = x;
    else a.ctr->error = 2;
}

__global__ void k_vertex_validate(MutArgs a) {
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= a.n_ops) return;
    ripple_update op = a.ops[i];
    uint32_t st = 0;
    if (op.kind == RIPPLE_VERTEX_ADD) {
        if (!rp_bit(a.alive, op.u)) {
            st = 1;
            atomicOr(&a.vstate[op.u], VS_ADDING);
        }
    } else if (op.kind == RIPPLE_VERTEX_DEL) {
        if (rp_bit(a.alive, op.u)) {
            st = 1;
            atomicOr(&a.vstate[op.u], VS_DYING);
            atomicAdd(&a.ctr->need_exp, a.out_meta[op.u].y + a.in_meta[op.u].y);
        }
    } else {
        return;                                   // edge operations and feature updates: k_edge_validate
    }
    a.status[i] = st;
}

__global__ __launch_bounds__(256) void k_edge_validate(MutArgs a) {
    const int lane = rp_lane();
    uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    for (uint32_t i = gw; i < a.n_ops; i += nw) {
        ripple_update op = a.ops[i];
        if (op.kind == RIPPLE_FEAT_UPDATE) {               // needs the live flag only
            if (lane == 0) {
                a.status[i] = rp_bit(a.alive, op.u) ? 1u : 0u;
                if (a.defer_touch) a.op_touch[i] = 0;
            }
            continue;
        }
        if (op.kind == RIPPLE_EDGE_REWEIGHT) {             // the edge must exist; nothing about the rows' shape changes
            int p = -1;
            if (a.in_w && rp_bit(a.alive, op.u) && rp_bit(a.alive, op.v)) {
                const uint2 mi = a.in_meta[op.v];
                p = rp_wave_find(a.in_pool + mi.x, mi.y, op.u);
            }
            if (lane == 0) {
                a.status[i] = p >= 0 ? 1u : 0u;
                if (p >= 0) a.pos_in[i] = (uint32_t)p;
                if (a.defer_touch) a.op_touch[i] = 0;
            }
            continue;
        }
        if (op.kind != RIPPLE_EDGE_ADD && op.kind != RIPPLE_EDGE_DEL) {
            if (lane == 0 && a.defer_touch) a.op_touch[i] = 0;
            continue;
        }
        uint32_t u = op.u, v = op.v;
        bool ok = (rp_bit(a.alive, u) || (a.vstate[u] & VS_ADDING)) &&
                  (rp_bit(a.alive, v) || (a.vstate[v] & VS_ADDING));
        uint32_t st = 0;
        int po = -1, pi = -1;
        if (ok) {
            uint2 mo = a.out_meta[u], mi = a.in_meta[v];
            if (op.kind == RIPPLE_EDGE_ADD) {
                int p = (mo.y <= mi.y) ? rp_wave_find(a.out_pool + mo.x, mo.y, v)
                                       : rp_wave_find(a.in_pool + mi.x, mi.y, u);
                st = (p < 0) ? 1u : 0u;
            } else {
                po = rp_wave_find(a.out_pool + mo.x, mo.y, v);
                if (po >= 0) {
                    pi = rp_wave_find(a.in_pool + mi.x, mi.y, u);
                    if (pi >= 0) st = 1;
                    else if (lane == 0) a.ctr->error = 3;     // the two adjacencies disagree
                }
            }
        }
        if (lane == 0) {
            a.status[i] = st;
            uint32_t flags = 0;
            if (st) {
                const bool is_add = op.kind == RIPPLE_EDGE_ADD;
                if (is_add) {
                    atomicAdd(&a.pend_out[u], 1u);
                    atomicAdd(&a.pend_in[v], 1u);
                } else {
                    a.pos_out[i] = (uint32_t)po;
                    a.pos_in[i] = (uint32_t)pi;
                    atomicAdd(&a.dead_out[u], 1u);
                    atomicAdd(&a.dead_in[v], 1u);
                }
                if (a.defer_touch) {
                    // thousands of wavefronts bumping the same few counters would queue up behind one
                    // another: only the per-row bits are set here, k_touch_lists builds lists and counts
                    flags = 1u | (is_add ? 2u : 0u);
                    if (!(atomicOr(&a.vstate[u], VS_TOUCH_OUT) & VS_TOUCH_OUT)) flags |= 4u;
                    if (!(atomicOr(&a.vstate[v], VS_TOUCH_IN) & VS_TOUCH_IN)) flags |= 8u;
                } else {
                    atomicAdd(is_add ? &a.ctr->n_add : &a.ctr->n_del, 1u);
                    touch_row(a, u, VS_TOUCH_OUT);
                    touch_row(a, v, VS_TOUCH_IN);
                }
            }
            if (a.defer_touch) a.op_touch[i] = flags;
        }
    }
}

// Touched-row lists and accepted add / delete counts of the edge operations, from the flags that
// k_edge_validate left per operation: one workgroup, block-wide ranks instead of one atomic per row.
__global__ __launch_bounds__(1024) void k_touch_lists(MutArgs a) {
    __shared__ uint32_t s_o[16], s_i[16], s_a[16], s_d[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t base_o = a.ctr->n_touch_out, base_i = a.ctr->n_touch_in;     // nothing else runs meanwhile
    uint32_t adds = 0, dels = 0;                                            // per wavefront (lane 0 keeps them)
    for (uint32_t start = 0; start < a.n_ops; start += 1024) {
        const uint32_t i = start + tid;
        const uint32_t f = (i < a.n_ops) ? a.op_touch[i] : 0u;
        const unsigned long long mo = __ballot((f & 4u) != 0), mi = __ballot((f & 8u) != 0);
        adds += (uint32_t)__popcll(__ballot((f & 3u) == 3u));
        dels += (uint32_t)__popcll(__ballot((f & 3u) == 1u));
        if (lane == 0) {
            s_o[wave] = (uint32_t)__popcll(mo);
            s_i[wave] = (uint32_t)__popcll(mi);
        }
        __syncthreads();
        uint32_t off_o = 0, off_i = 0, tot_o = 0, tot_i = 0;
        for (int k = 0; k < 16; ++k) {
            if (k < wave) {
                off_o += s_o[k];
                off_i += s_i[k];
            }
            tot_o += s_o[k];
            tot_i += s_i[k];
        }
        const unsigned long long below = (1ull << lane) - 1ull;
        if (f & 4u) {
            const uint32_t p = base_o + off_o + (uint32_t)__popcll(mo & below);
            if (p < a.touch_cap) a.touch_out[p] = a.ops[i].u;
            else a.ctr->error = 2;
        }
        if (f & 8u) {
            const uint32_t p = base_i + off_i + (uint32_t)__popcll(mi & below);
            if (p < a.touch_cap) a.touch_in[p] = a.ops[i].v;
            else a.ctr->error = 2;
        }
        base_o += tot_o;
        base_i += tot_i;
        __syncthreads();                                    // s_o / s_i are rewritten by the next round
    }
    if (lane == 0) {
        s_a[wave] = adds;
        s_d[wave] = dels;
    }
    __syncthreads();
    if (tid == 0) {
        uint32_t ta = 0, td = 0;
        for (int k = 0; k < 16; ++k) {
            ta += s_a[k];
            td += s_d[k];
        }
        a.ctr->n_add += ta;
        a.ctr->n_del += td;
        a.ctr->n_touch_out = base_o;
        a.ctr->n_touch_in = base_i;
    }
}

// How much pool space relocation will take, then (by the last workgroup to finish) the decision
// whether the batch may be committed at all.
__global__ void k_capacity(MutArgs a) {
    uint32_t j = blockIdx.x * blockDim.x + threadIdx.x;
    uint32_t no = min(a.ctr->n_touch_out, a.touch_cap), ni = min(a.ctr->n_touch_in, a.touch_cap);
    if (j < no) {
        uint32_t x = a.touch_out[j], pend = a.pend_out[x];
        uint32_t need = a.out_meta[x].y - a.dead_out[x] + pend;
        if (pend && need > a.out_capv[x]) atomicAdd(&a.ctr->need_out, rp_row_cap(need));
    } else if (j < no + ni) {
        uint32_t x = a.touch_in[j - no], pend = a.pend_in[x];
        uint32_t need = a.in_meta[x].y - a.dead_in[x] + pend;
        if (pend && need > a.in_capv[x]) atomicAdd(&a.ctr->need_in, rp_row_cap(need));
    }
    __shared__ bool last;
    __syncthreads();
    if (threadIdx.x == 0) {
        __threadfence();
        last = atomicAdd(&a.ctr->blocks_done, 1u) == gridDim.x - 1;
    }
    __syncthreads();
    if (!last || threadIdx.x != 0) return;
    __threadfence();
    DevCtr *c = a.ctr;
    const uint32_t need_out = atomicAdd(&c->need_out, 0u), need_in = atomicAdd(&c->need_in, 0u);
    uint32_t flag = 0;
    if ((unsigned long long)c->out_top + need_out > a.pool_cap || (unsigned long long)c->in_top + need_in > a.pool_cap)
        flag |= 1u;
    if (c->n_edges + c->n_add > a.e_cap + c->n_del) flag |= 2u;
    if (c->need_exp > a.exp_cap || (unsigned long long)c->n_add + c->n_del + c->need_exp > a.struct_cap ||
        (unsigned long long)c->n_add + c->n_del + c->need_exp > a.touch_cap)
        flag |= 4u;
    if (c->error) flag |= 8u;
    c->abort_flag = flag;
    c->blocks_done = 0;
}

// slot in a global list for every lane with pred, one atomic per wavefront
__device__ __forceinline__ uint32_t wave_reserve(uint32_t *counter, bool pred) {
    unsigned long long m = __ballot(pred);
    if (!m) return 0;
    const int lane = rp_lane();
    int leader = __ffsll((long long)m) - 1;
    uint32_t base = 0;
    if (lane == leader) base = atomicAdd(counter, (uint32_t)__popcll(m));
    base = __shfl(base, leader);
    return base + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
}

__global__ __launch_bounds__(256) void k_expand_vdel(MutArgs a) {
    if (a.ctr->abort_flag) return;
    const int lane = rp_lane();
    uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    for (uint32_t i = gw; i < a.n_ops; i += nw) {
        ripple_update op = a.ops[i];
        if (op.kind != RIPPLE_VERTEX_DEL || !a.status[i]) continue;
        uint32_t w = op.u;
        uint2 mo = a.out_meta[w], mi = a.in_meta[w];
        uint32_t base = 0;
        if (lane == 0) base = atomicAdd(&a.ctr->n_exp, mo.y + mi.y);
        base = __shfl(base, 0);
        uint32_t gone = mo.y;                               // every out-edge disappears
        for (uint32_t j0 = 0; j0 < mo.y; j0 += 64) {
            uint32_t j = j0 + lane;
            bool valid = j < mo.y;
            uint32_t y = valid ? a.out_pool[mo.x + j] : 0u;
            bool keep = valid && !(a.vstate[y] & VS_DYING);
            if (valid) {
                a.exp_kind[base + j] = keep ? EXP_OUT : EXP_NONE;
                a.exp_a[base + j] = w;
                a.exp_b[base + j] = y;
            }
            uint32_t s = wave_reserve(&a.ctr->n_struct, keep);
            if (keep) {
                if (s < a.struct_cap) {
                    a.st_src[s] = w;
                    a.st_dst[s] = y;
                    a.st_sign[s] = -1.0f;                   // times the edge weight: k_expand_apply, which finds the edge in y's in-row
                    a.st_unit[s] = -1.0f;
                }
                if (a.in_w) a.exp_s[base + j] = s;
                rp_set_bit(a.bm_sink, y);
            }
        }
        uint32_t cnt_in = 0;
        for (uint32_t j0 = 0; j0 < mi.y; j0 += 64) {
            uint32_t j = j0 + lane;
            bool valid = j < mi.y;
            uint32_t x = valid ? a.in_pool[mi.x + j] : 0u;
            bool keep = valid && !(a.vstate[x] & VS_DYING);   // edges between two dying vertices count once
            if (valid) {
                a.exp_kind[base + mo.y + j] = keep ? EXP_IN : EXP_NONE;
                a.exp_a[base + mo.y + j] = x;
                a.exp_b[base + mo.y + j] = w;
            }
            cnt_in += (uint32_t)__popcll(__ballot(keep));
        }
        gone += cnt_in;
        if (lane == 0) atomicAdd(&a.ctr->n_edges, (unsigned long long)(-(long long)gone));
    }
}

__global__ __launch_bounds__(256) void k_expand_apply(MutArgs a) {
    if (a.ctr->abort_flag) return;
    const int lane = rp_lane();
    uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    uint32_t n = min(a.ctr->n_exp, a.exp_cap);
    for (uint32_t e = gw; e < n; e += nw) {
        uint32_t kind = a.exp_kind[e];
        if (kind == EXP_NONE) continue;
        uint32_t x = a.exp_a[e], y = a.exp_b[e];
        if (kind == EXP_OUT) {                               // x -> y with x dying: erase x from y's in-row
            uint2 mi = a.in_meta[y];
            int p = rp_wave_find(a.in_pool + mi.x, mi.y, x);
            if (lane == 0) {
                if (p >= 0) {
                    if (a.in_w) {
                        const uint32_t slot = a.exp_s[e];
                        if (slot < a.struct_cap) a.st_sign[slot] = -a.in_w[mi.x + p];
                    }
                    a.in_pool[mi.x + p] = RP_TOMB;
                    a.hole_in[y] = (uint32_t)p;
                    atomicAdd(&a.dead_in[y], 1u);
                    touch_row(a, y, VS_TOUCH_IN);
                } else a.ctr->error = 4;
            }
        } else {                                             // x -> y with y dying: erase y from x's out-row
            uint2 mo = a.out_meta[x];
            int p = rp_wave_find(a.out_pool + mo.x, mo.y, y);
            if (lane == 0) {
                if (p >= 0) {
                    a.out_pool[mo.x + p] = RP_TOMB;
                    a.hole_out[x] = (uint32_t)p;
                    atomicAdd(&a.dead_out[x], 1u);
                    touch_row(a, x, VS_TOUCH_OUT);
                } else a.ctr->error = 5;
            }
        }
    }
}

// tombstone deleted edges, list every changed edge as a structural term, count results
__global__ __launch_bounds__(256) void k_apply_edges(MutArgs a) {
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    bool in_range = i < a.n_ops;
    bool aborted = a.ctr->abort_flag != 0;
    ripple_update op = in_range ? a.ops[i] : ripple_update{99u, 0u, 0u, 0u};
    bool acc = in_range && a.status[i] != 0;
    unsigned long long ma = __ballot(acc), mr = __ballot(in_range && !acc);
    if (rp_lane() == 0 && !aborted) {
        if (ma) atomicAdd(&a.ctr->n_applied, (uint32_t)__popcll(ma));
        if (mr) atomicAdd(&a.ctr->n_rejected, (uint32_t)__popcll(mr));
    }
    if (aborted) return;
    bool edge = acc && (op.kind == RIPPLE_EDGE_ADD || op.kind == RIPPLE_EDGE_DEL || op.kind == RIPPLE_EDGE_REWEIGHT);
    uint32_t s = wave_reserve(&a.ctr->n_struct, edge);
    if (!edge) return;
    if (op.kind == RIPPLE_EDGE_REWEIGHT) {           // the weighted sums of the sink gain (alpha_new - alpha_old) h_u
        float *w = a.in_w + a.in_meta[op.v].x + a.pos_in[i];
        const float alpha_new = __uint_as_float(op.feat_row);
        if (s < a.struct_cap) {
            a.st_src[s] = op.u;
            a.st_dst[s] = op.v;
            a.st_sign[s] = alpha_new - *w;
            a.st_unit[s] = 0.0f;
        }
        *w = alpha_new;
        rp_set_bit(a.bm_sink, op.v);
        return;
    }
    float alpha = 1.0f;                              // the edge's weight (1 on unweighted graphs)
    if (op.kind == RIPPLE_EDGE_DEL) {
        if (a.in_w) alpha = a.in_w[a.in_meta[op.v].x + a.pos_in[i]];
        a.out_pool[a.out_meta[op.u].x + a.pos_out[i]] = RP_TOMB;
        a.in_pool[a.in_meta[op.v].x + a.pos_in[i]] = RP_TOMB;
        a.hole_out[op.u] = a.pos_out[i];
        a.hole_in[op.v] = a.pos_in[i];
    } else if (a.in_w) {
        alpha = __uint_as_float(op.feat_row);       // weighted graphs: EDGE_ADD carries the weight's bits there
    }
    if (s < a.struct_cap) {
        a.st_src[s] = op.u;
        a.st_dst[s] = op.v;
        a.st_sign[s] = (op.kind == RIPPLE_EDGE_ADD) ? alpha : -alpha;
        a.st_unit[s] = (op.kind == RIPPLE_EDGE_ADD) ? 1.0f : -1.0f;
    }
    rp_set_bit(a.bm_sink, op.v);
}

// feature writes (with the hop-0 delta), vertex creation, vertex removal
__global__ __launch_bounds__(256) void k_apply_vertices(MutArgs a) {
    if (a.ctr->abort_flag) return;
    const int lane = rp_lane();
    uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    const uint32_t d0 = a.d[0];
    for (uint32_t i = gw; i < a.n_ops; i += nw) {
        ripple_update op = a.ops[i];
        if (!a.status[i]) continue;
        uint32_t w = op.u;
        if (op.kind == RIPPLE_FEAT_UPDATE || op.kind == RIPPLE_VERTEX_ADD) {
            uint32_t slot = 0;
            if (lane == 0) slot = atomicAdd(&a.ctr->a[0], 1u);
            slot = __shfl(slot, 0);
            const float *row = a.payload + (size_t)op.feat_row * d0;
            for (uint32_t c = lane; c < d0; c += 64) {
                float nv = row[c];
                size_t idx = (size_t)w * d0 + c;
                float old;
                if (a.store) {
                    __hip_bfloat16 *h = (__hip_bfloat16 *)a.H[0];
                    old = __bfloat162float(h[idx]);
                    __hip_bfloat16 r = __float2bfloat16(nv);
                    nv = __bfloat162float(r);
                    h[idx] = r;
                } else {
                    float *h = (float *)a.H[0];
                    old = h[idx];
                    h[idx] = nv;
                }
                a.D0[idx] = a.d0_old ? old : nv - old;
            }
            if (lane == 0) {
                a.list0[slot] = w;
                rp_set_bit(a.bm0, w);
                if (op.kind == RIPPLE_VERTEX_ADD) {
                    atomicOr(&a.alive[w >> 5], 1u << (w & 31));
                    rp_set_bit(a.bm_vadd, w);
                    atomicAdd(&a.ctr->n_alive, 1u);
                    atomicAdd(&a.ctr->n_vadd, 1u);
                }
            }
        } else if (op.kind == RIPPLE_VERTEX_DEL) {
            for (uint32_t l = 0; l <= a.L; ++l) {
                uint32_t dl = a.d[l];
                for (uint32_t c = lane; c < dl; c += 64) {
                    size_t idx = (size_t)w * dl + c;
                    if (a.store) ((__hip_bfloat16 *)a.H[l])[idx] = __float2bfloat16(0.0f);
                    else ((float *)a.H[l])[idx] = 0.0f;
                }
                if (l >= 1) {
                    uint32_t dp = a.xw[l];
                    for (uint32_t c = lane; c < dp; c += 64) a.X[l][(size_t)w * dp + c] = 0.0f;
                    if (a.T[l])                            // a vertex created under this id later has sent nothing yet
                        for (uint32_t c = lane; c < dp; c += 64) a.T[l][(size_t)w * dp + c] = 0.0f;
                }
            }
            if (lane == 0) {
                atomicAnd(&a.alive[w >> 5], ~(1u << (w & 31)));
                a.out_meta[w].y = 0;
                a.in_meta[w].y = 0;
                atomicSub(&a.ctr->n_alive, 1u);
            }
        }
    }
}

// one wavefront per touched row: squeeze tombstones out, move the row if the
// pending appends do not fit, reset the row's scratch counters
__global__ __launch_bounds__(256) void k_cleanup_rows(MutArgs a) {
    const int lane = rp_lane();
    const bool aborted = a.ctr->abort_flag != 0;
    uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    uint32_t no = min(a.ctr->n_touch_out, a.touch_cap), ni = min(a.ctr->n_touch_in, a.touch_cap);
    for (uint32_t j = gw; j < no + ni; j += nw) {
        const bool is_out = j < no;
        const uint32_t x = is_out ? a.touch_out[j] : a.touch_in[j - no];
        uint2 *meta = is_out ? a.out_meta : a.in_meta;
        uint32_t *capv = is_out ? a.out_capv : a.in_capv;
        uint32_t *pool = is_out ? a.out_pool : a.in_pool;
        float *wp = is_out ? nullptr : a.in_w;             // weights travel with the in-row's entries
        uint32_t *deadv = is_out ? a.dead_out : a.dead_in;
        uint32_t *pendv = is_out ? a.pend_out : a.pend_in;
        uint32_t *top = is_out ? &a.ctr->out_top : &a.ctr->in_top;
        if (!aborted) {
            uint2 m = meta[x];
            uint32_t dead = deadv[x], pend = pendv[x];
            uint32_t len = m.y;
            const uint32_t hole = is_out ? a.hole_out[x] : a.hole_in[x];
            if (dead == 1 && len && hole < len && pool[m.x + hole] == RP_TOMB) {
                // the usual case, one deletion in the row: its position is known, the last entry fills it
                if (hole != len - 1 && lane == 0) {
                    pool[m.x + hole] = pool[m.x + len - 1];
                    if (wp) wp[m.x + hole] = wp[m.x + len - 1];
                }
                len -= 1;
            } else if (dead && len) {
                // Rows are unordered, so holes in the part that stays (the first len - dead entries) are
                // filled from the part that goes. First the live entries of that tail are packed to its
                // front (it is at most `dead` long), then the head is read sixteen blocks per round and
                // its k-th hole takes the tail's k-th live entry.
                const uint32_t keep_len = len - min(dead, len);
                uint32_t n_tail = 0;                               // live entries packed at keep_len ..
                for (uint32_t base = keep_len; base < len; base += 64) {
                    const uint32_t i = base + lane;
                    const uint32_t val = (i < len) ? pool[m.x + i] : RP_TOMB;
                    const float wv = (wp && i < len) ? wp[m.x + i] : 0.0f;
                    const bool keep = val != RP_TOMB;
                    const unsigned long long mask = __ballot(keep);
                    const uint32_t off = (uint32_t)__popcll(mask & ((1ull << lane) - 1ull));
                    if (keep) {
                        pool[m.x + keep_len + n_tail + off] = val;
                        if (wp) wp[m.x + keep_len + n_tail + off] = wv;
                    }
                    n_tail += (uint32_t)__popcll(mask);
                }
                uint32_t filled = 0;                               // holes of the head filled so far
                for (uint32_t base = 0; base < keep_len && filled < n_tail; base += 1024) {
                    uint32_t v[16];
#pragma unroll
                    for (int t = 0; t < 16; ++t) {
                        const uint32_t i = base + 64 * t + lane;
                        v[t] = (i < keep_len) ? pool[m.x + i] : 0u;
                    }
#pragma unroll
                    for (int t = 0; t < 16; ++t) {
                        const uint32_t i = base + 64 * t + lane;
                        const bool hole = i < keep_len && v[t] == RP_TOMB;
                        const unsigned long long mask = __ballot(hole);
                        const uint32_t k = filled + (uint32_t)__popcll(mask & ((1ull << lane) - 1ull));
                        if (hole && k < n_tail) {
                            pool[m.x + i] = pool[m.x + keep_len + k];
                            if (wp) wp[m.x + i] = wp[m.x + keep_len + k];
                        }
                        filled += (uint32_t)__popcll(mask);
                    }
                }
                len = keep_len;
            }
            uint32_t need = len + pend;
            if (pend && need > capv[x]) {
                uint32_t ncap = rp_row_cap(need);
                uint32_t ns = 0;
                if (lane == 0) ns = atomicAdd(top, ncap);
                ns = __shfl(ns, 0);
                if ((unsigned long long)ns + ncap <= a.pool_cap) {
                    for (uint32_t base = 0; base < len; base += 512) {      // eight blocks in flight per round
                        uint32_t v[8];
#pragma unroll
                        for (int t = 0; t < 8; ++t) {
                            const uint32_t i = base + 64 * t + lane;
                            v[t] = (i < len) ? pool[m.x + i] : 0u;
                        }
#pragma unroll
                        for (int t = 0; t < 8; ++t) {
                            const uint32_t i = base + 64 * t + lane;
                            if (i < len) pool[ns + i] = v[t];
                        }
                    }
                    if (wp)
                        for (uint32_t i = lane; i < len; i += 64) wp[ns + i] = wp[m.x + i];
                    m.x = ns;
                    if (lane == 0) capv[x] = ncap;
                } else if (lane == 0) {
                    a.ctr->error = 6;                        // cannot happen: space was checked before commit
                }
            }
            if (lane == 0) {
                meta[x] = make_uint2(m.x, len);
                if (a.det && !is_out) a.hole_in[x] = len;    // where this batch's appends start (the hole is filled)
            }
        }
        if (lane == 0) {
            deadv[x] = 0;
            pendv[x] = 0;
            atomicAnd(&a.vstate[x], ~(is_out ? VS_TOUCH_OUT : VS_TOUCH_IN));
        }
    }
}

__global__ void k_apply_adds(MutArgs a) {
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    const bool aborted = a.ctr->abort_flag != 0;
    if (i == 0 && !aborted) {
        atomicAdd(&a.ctr->n_edges, (unsigned long long)a.ctr->n_add);
        atomicAdd(&a.ctr->n_edges, (unsigned long long)(-(long long)a.ctr->n_del));
    }
    if (i >= a.n_ops) return;
    ripple_update op = a.ops[i];
    if (op.kind == RIPPLE_VERTEX_ADD || op.kind == RIPPLE_VERTEX_DEL) {
        atomicAnd(&a.vstate[op.u], ~(VS_ADDING | VS_DYING));
        return;
    }
    if (aborted || op.kind != RIPPLE_EDGE_ADD || !a.status[i]) return;
    uint32_t p = atomicAdd(&((uint32_t *)a.out_meta)[2 * (size_t)op.u + 1], 1u);
    if (p < a.out_capv[op.u]) a.out_pool[a.out_meta[op.u].x + p] = op.v;
    else a.ctr->error = 7;
    p = atomicAdd(&((uint32_t *)a.in_meta)[2 * (size_t)op.v + 1], 1u);
    if (p < a.in_capv[op.v]) {
        a.in_pool[a.in_meta[op.v].x + p] = op.u;
        if (a.in_w) a.in_w[a.in_meta[op.v].x + p] = __uint_as_float(op.feat_row);
    } else a.ctr->error = 7;
}

// Deterministic mode. The entries appended above land in the order their atomics were served. A sum that
// walks a row in storage order is only a function of the graph if that order is one, so the appended part
// of every touched in-row (it starts where k_cleanup_rows left the row's end) is put in ascending id order;
// ids are distinct within a row. With the rows built in the order the edges were given, and the fills of
// k_cleanup_rows being functions of the row and the deleted positions alone, an in-row's order then depends
// on the batches that were applied and on nothing else. Up to 64 appended entries are ranked in registers by
// the row's wavefront; longer runs are queued for k_sort_long_tails.
__global__ __launch_bounds__(256) void k_sort_tails(MutArgs a) {
    if (a.ctr->abort_flag) return;
    const int lane = rp_lane();
    uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    const uint32_t ni = min(a.ctr->n_touch_in, a.touch_cap);
    for (uint32_t j = gw; j < ni; j += nw) {
        const uint32_t x = a.touch_in[j];
        const uint2 m = a.in_meta[x];
        const uint32_t start = a.hole_in[x];
        if (start >= m.y || m.y - start < 2u) continue;
        const uint32_t t = m.y - start;
        if (t > 64u) {
            if (lane == 0) a.tail_q[atomicAdd(&a.ctr->n_tail_q, 1u)] = x;
            continue;
        }
        uint32_t *row = a.in_pool + m.x + start;
        float *wr = a.in_w ? a.in_w + m.x + start : nullptr;
        const bool mine = (uint32_t)lane < t;
        const uint32_t id = mine ? row[lane] : 0xFFFFFFFFu;
        const float wv = (mine && wr) ? wr[lane] : 0.0f;
        uint32_t rank = 0;
        for (uint32_t k = 0; k < t; ++k) rank += (__shfl(id, (int)k) < id) ? 1u : 0u;
        if (mine) {
            row[rank] = id;
            if (wr) wr[rank] = wv;
        }
    }
}

// one workgroup per queued row: the appended entries are copied aside, every one counts the smaller ids
// (the copy is read through LDS, 4096 at a time) and goes to that position
__global__ __launch_bounds__(1024) void k_sort_long_tails(MutArgs a) {
    __shared__ uint32_t s_ids[4096];
    __shared__ uint32_t s_base;
    if (a.ctr->abort_flag) return;
    const uint32_t tid = threadIdx.x;
    const uint32_t n = min(a.ctr->n_tail_q, a.touch_cap);
    for (uint32_t q = blockIdx.x; q < n; q += gridDim.x) {
        const uint32_t x = a.tail_q[q];
        const uint2 m = a.in_meta[x];
        const uint32_t start = a.hole_in[x];
        const uint32_t t = m.y - start;
        __syncthreads();
        if (tid == 0) s_base = atomicAdd(&a.ctr->tail_top, t);
        __syncthreads();
        const uint32_t base = s_base;
        if ((unsigned long long)base + t > a.tail_cap) {     // cannot happen: a batch appends at most n_ops entries
            if (tid == 0) a.ctr->error = 10;
            continue;
        }
        uint32_t *row = a.in_pool + m.x + start;
        float *wr = a.in_w ? a.in_w + m.x + start : nullptr;
        for (uint32_t i = tid; i < t; i += 1024) {
            a.tail_ids[base + i] = row[i];
            if (wr) a.tail_w[base + i] = wr[i];
        }
        __syncthreads();
        for (uint32_t eb = 0; eb < t; eb += 1024) {
            const uint32_t i = eb + tid;
            const uint32_t my = (i < t) ? a.tail_ids[base + i] : 0u;
            uint32_t rank = 0;
            for (uint32_t tb = 0; tb < t; tb += 4096) {
                const uint32_t cnt = min(4096u, t - tb);
                __syncthreads();
                for (uint32_t k = tid; k < cnt; k += 1024) s_ids[k] = a.tail_ids[base + tb + k];
                __syncthreads();
                if (i < t)
                    for (uint32_t k = 0; k < cnt; ++k) rank += (s_ids[k] < my) ? 1u : 0u;
            }
            if (i < t) {
                row[rank] = my;
                if (wr) wr[rank] = a.tail_w[base + i];
            }
        }
    }
}

// X^l[v] += sign * H^{l-1}[u] for every changed edge and every layer, taken
// while all H still hold their pre-batch values (Sec. 3.3.3: an added edge
// uses 0 as the source's old embedding, a deleted edge 0 as its new one).
__global__ __launch_bounds__(256) void k_struct_scatter(MutArgs a) {
    if (a.ctr->abort_flag) return;
    const int lane = rp_lane();
    uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    uint32_t n = min(a.ctr->n_struct, a.struct_cap);
    // one task per changed edge and layer. A project-first layer's aggregate is the sum of what its in-neighbours
    // have sent (T), so a changed edge adds or removes T[u] itself
    const uint32_t per = a.L;
    unsigned long long total = (unsigned long long)n * per;
    for (unsigned long long t = gw; t < total; t += nw) {
        const uint32_t e = (uint32_t)(t / per), l = (uint32_t)(t % per) + 1;
        if ((a.mono_mask >> l) & 1u) continue;               // rows with a changed in-edge are recomputed instead
        uint32_t u = a.st_src[e], v = a.st_dst[e];
        const float sg = ((a.wsum_mask >> l) & 1u) ? a.st_sign[e] : a.st_unit[e];
        if (sg == 0.0f) continue;                            // a new weight means nothing to a layer that ignores weights
        if (a.T[l] == nullptr) {
            const uint32_t dp = a.d[l - 1];
            for (uint32_t c = lane; c < dp; c += 64) {
                float val = rp_load_h(a.H[l - 1], a.store, (size_t)u * dp + c);
                if (val != 0.0f) unsafeAtomicAdd(&a.X[l][(size_t)v * dp + c], sg * val);
            }
        } else {
            const uint32_t dn = a.xw[l];
            for (uint32_t c = lane; c < dn; c += 64) {
                const float val = a.T[l][(size_t)u * dn + c];
                if (val != 0.0f) unsafeAtomicAdd(&a.X[l][(size_t)v * dn + c], sg * val);
            }
        }
    }
}

// Deterministic mode: the same terms without atomics. The changed edges are sorted by (sink, source) - a piece of a
// batch holds at most one operation per edge, so the keys are distinct and the order is a function of the piece -
// and the wavefront that finds the first entry of a sink adds that sink's terms one after the other, for every
// layer, with plain loads and stores; eight source rows are in flight at a time.
__global__ void k_struct_keys(MutArgs a) {
    const uint32_t e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= a.n_sort) return;
    const uint32_t n = a.ctr->abort_flag ? 0u : min(a.ctr->n_struct, a.struct_cap);
    a.sk_in[e] = (e < n) ? (((unsigned long long)a.st_dst[e] << 32) | a.st_src[e]) : ~0ull;
    a.sv_in[e] = (e < n) ? a.st_unit[e] : 0.0f;
}

__global__ __launch_bounds__(256) void k_struct_ordered(MutArgs a) {
    if (a.ctr->abort_flag) return;
    constexpr int G = 8;
    const int lane = rp_lane();
    const uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    const uint32_t n = min(min(a.ctr->n_struct, a.struct_cap), a.n_sort);
    for (uint32_t e0 = gw; e0 < n; e0 += nw) {
        const uint32_t v = (uint32_t)(a.sk_out[e0] >> 32);
        if (e0 > 0 && (uint32_t)(a.sk_out[e0 - 1] >> 32) == v) continue;   // not the sink's first entry
        uint32_t len = 1;                                                  // entries of this sink
        for (bool more = true; more;) {
            const uint32_t f = e0 + len + (uint32_t)lane;
            const unsigned long long other = __ballot(f >= n || (uint32_t)(a.sk_out[f] >> 32) != v);
            if (other) {
                len += (uint32_t)__ffsll((long long)other) - 1u;
                more = false;
            } else len += 64u;
        }
        for (uint32_t l = 1; l <= a.L; ++l) {
            if ((a.mono_mask >> l) & 1u) continue;
            const float *Tl = a.T[l];
            const uint32_t w = Tl ? a.xw[l] : a.d[l - 1];
            for (uint32_t c0 = 0; c0 < w; c0 += 64) {
                const uint32_t col = c0 + (uint32_t)lane;
                float *xp = a.X[l] + (size_t)v * w + col;
                float x = (col < w) ? *xp : 0.0f;
                for (uint32_t j0 = 0; j0 < len; j0 += G) {
                    float val[G], sg[G];
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        const uint32_t e = e0 + min(j0 + (uint32_t)g, len - 1u);
                        const uint32_t u = (uint32_t)a.sk_out[e];
                        sg[g] = (j0 + (uint32_t)g < len) ? a.sv_out[e] : 0.0f;
                        val[g] = 0.0f;
                        if (col < w && sg[g] != 0.0f)
                            val[g] = Tl ? Tl[(size_t)u * w + col] : rp_load_h(a.H[l - 1], a.store, (size_t)u * w + col);
                    }
#pragma unroll
                    for (int g = 0; g < G; ++g)
                        if (sg[g] != 0.0f) x += sg[g] * val[g];
                }
                if (col < w) *xp = x;
            }
        }
    }
}

__global__ void k_batch_reset(DevCtr *ctr, uint32_t *bitmaps, size_t n_bitmap_words) {
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_bitmap_words; i += stride) bitmaps[i] = 0;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        for (int l = 0; l <= RIPPLE_MAX_LAYERS; ++l) {
            ctr->a[l] = 0;
            ctr->m[l] = 0;
            ctr->touched[l] = 0;
            ctr->isum[l] = 0;
            ctr->n_long[l] = 0;
            ctr->cand[l] = 0;
            ctr->n_big[l] = 0;
            ctr->n_seg[l] = 0;
            ctr->hop_mode[l] = 0;
            ctr->pull_next[l] = 0;
        }
        ctr->n_struct = 0;
        ctr->n_touch_out = ctr->n_touch_in = 0;
        ctr->n_exp = ctr->need_exp = 0;
        ctr->n_applied = ctr->n_rejected = 0;
        ctr->n_add = ctr->n_del = 0;
        ctr->need_out = ctr->need_in = 0;
        ctr->n_vadd = 0;
        ctr->abort_flag = 0;
        ctr->range_rows = 0;
        ctr->n_tail_q = ctr->tail_top = 0;
        for (int k = 0; k < 3; ++k)
            for (int l = 0; l <= RIPPLE_MAX_LAYERS; ++l) ctr->mono[k][l] = 0;
    }
}

static MutArgs make_args(ripple_ctx *c, uint32_t n_ops) {
    MutArgs a;
    a.ops = c->ops_d;
    a.n_ops = n_ops;
    a.payload = c->payload_d;
    a.status = c->op_status;
    a.hole_out = c->hole_out;
    a.hole_in = c->hole_in;
    a.op_touch = c->op_touch;
    a.defer_touch = n_ops > 512 ? 1 : 0;
    a.pos_out = c->op_pos_out;
    a.pos_in = c->op_pos_in;
    a.out_meta = c->out_meta;
    a.in_meta = c->in_meta;
    a.out_capv = c->out_capv;
    a.in_capv = c->in_capv;
    a.out_pool = c->out_pool;
    a.in_pool = c->in_pool;
    a.in_w = c->in_w;
    a.alive = c->alive;
    a.vstate = c->vstate;
    a.pend_out = c->pend_out;
    a.pend_in = c->pend_in;
    a.dead_out = c->dead_out;
    a.dead_in = c->dead_in;
    a.touch_out = c->touch_out;
    a.touch_in = c->touch_in;
    a.touch_cap = c->touch_cap;
    a.exp_kind = c->exp_kind;
    a.exp_s = c->exp_s;
    a.exp_a = c->exp_a;
    a.exp_b = c->exp_b;
    a.exp_cap = c->exp_cap;
    a.st_src = c->st_src;
    a.st_dst = c->st_dst;
    a.st_sign = c->st_sign;
    a.st_unit = c->st_unit;
    a.struct_cap = c->struct_cap;
    a.bm0 = c->bm[0];
    a.bm_sink = c->bm_sink;
    a.bm_vadd = c->bm_vadd;
    a.list0 = c->list[0];
    a.D0 = c->D[0];
    a.ctr = c->ctr;
    a.n_cap = c->n_cap;
    a.e_cap = c->e_cap;
    a.pool_cap = c->pool_cap;
    a.store = c->store;
    a.L = c->L;
    for (uint32_t l = 0; l <= RIPPLE_MAX_LAYERS; ++l) {
        a.d[l] = c->d[l];
        a.xw[l] = c->xw[l];
        a.H[l] = c->H[l];
        a.X[l] = c->X[l];
        a.T[l] = (l >= 1 && l <= c->L && c->layers[l - 1].proj) ? c->layers[l - 1].T : nullptr;
    }
    a.mono_mask = 0;
    a.wsum_mask = 0;
    for (uint32_t l = 1; l <= c->L; ++l) {
        if (rp_layer_mono(c, l) || rp_layer_attn(c, l)) a.mono_mask |= 1u << l;
        if (c->layers[l - 1].agg == RIPPLE_AGG_WSUM) a.wsum_mask |= 1u << l;
    }
    a.d0_old = rp_layer_mono(c, 1) ? 1 : 0;
    a.det = c->opt_deterministic;
    a.tail_ids = c->tail_ids;
    a.tail_q = c->tail_q;
    a.tail_w = c->tail_w;
    a.tail_cap = c->ops_cap;
    a.sk_in = c->sk_in;
    a.sk_out = c->sk_out;
    a.sv_in = c->sv_in;
    a.sv_out = c->sv_out;
    a.n_sort = 0;
    return a;
}

void rp_launch_batch_reset(ripple_ctx *c) {
    // the per-layer bitmaps, S and V_added are one allocation starting at bm[0]
    size_t words = (size_t)c->n_words * (c->L + 3);
    uint32_t gb = std::min<uint32_t>(rp_div_up(words, 256), c->n_cu * 4);
    hipLaunchKernelGGL(k_batch_reset, dim3(gb), dim3(256), 0, c->stream, c->ctr, c->bm[0], words);
}

// Enqueue the whole Apply step for the n_ops operations staged in ops_d / payload_d.
void rp_launch_mutate(ripple_ctx *c, uint32_t n_ops, bool has_vertex_add, bool has_vertex_del, bool has_vertex_or_feat) {
    if (n_ops == 0) return;
    hipStream_t s = c->stream;
    MutArgs a = make_args(c, n_ops);
    uint32_t tb = rp_div_up(n_ops, 256);                              // thread per op
    uint32_t wb = std::min<uint32_t>(rp_div_up(n_ops, 4), c->n_cu * 8);  // wavefront per op
    uint32_t big = c->n_cu * 8;
    if (has_vertex_add || has_vertex_del) hipLaunchKernelGGL(k_vertex_validate, dim3(tb), dim3(256), 0, s, a);
    hipLaunchKernelGGL(k_edge_validate, dim3(wb), dim3(256), 0, s, a);
    if (a.defer_touch) hipLaunchKernelGGL(k_touch_lists, dim3(1), dim3(1024), 0, s, a);
    uint32_t touch_threads = 2 * n_ops;                               // validation touches <= n_ops rows per side
    hipLaunchKernelGGL(k_capacity, dim3(rp_div_up(touch_threads, 256)), dim3(256), 0, s, a);
    if (has_vertex_del) {
        hipLaunchKernelGGL(k_expand_vdel, dim3(wb), dim3(256), 0, s, a);
        hipLaunchKernelGGL(k_expand_apply, dim3(big), dim3(256), 0, s, a);
    }
    hipLaunchKernelGGL(k_apply_edges, dim3(tb), dim3(256), 0, s, a);
    int t = rp_timer_begin(c);
    if (c->opt_deterministic) {
        // without vertex deletions a piece changes at most one edge per operation; with them, any number up to the lists' size
        a.n_sort = has_vertex_del ? c->struct_cap : std::min<uint32_t>(n_ops, c->struct_cap);
        hipLaunchKernelGGL(k_struct_keys, dim3(rp_div_up(a.n_sort, 256)), dim3(256), 0, s, a);
        rp_sort_pairs_u64(c, c->sk_in, c->sk_out, c->sv_in, c->sv_out, a.n_sort, c->sort_tmp, c->sort_tmp_bytes);
        hipLaunchKernelGGL(k_struct_ordered, dim3(std::min<uint32_t>(big, rp_div_up(a.n_sort, 4))), dim3(256), 0, s, a);
    } else {
        hipLaunchKernelGGL(k_struct_scatter, dim3(has_vertex_del ? big : std::min<uint32_t>(big, rp_div_up((uint64_t)n_ops * c->L, 4))),
                           dim3(256), 0, s, a);
    }
    rp_timer_end(c, t, RIPPLE_PH_STRUCT, 0);
    if (has_vertex_or_feat) hipLaunchKernelGGL(k_apply_vertices, dim3(wb), dim3(256), 0, s, a);
    hipLaunchKernelGGL(k_cleanup_rows, dim3(has_vertex_del ? big : std::min<uint32_t>(big, rp_div_up(2 * (uint64_t)n_ops, 4))),
                       dim3(256), 0, s, a);
    hipLaunchKernelGGL(k_apply_adds, dim3(tb), dim3(256), 0, s, a);
    if (c->opt_deterministic) {
        hipLaunchKernelGGL(k_sort_tails, dim3(has_vertex_del ? big : std::min<uint32_t>(big, rp_div_up((uint64_t)n_ops, 4))),
                           dim3(256), 0, s, a);
        hipLaunchKernelGGL(k_sort_long_tails, dim3(c->n_cu), dim3(1024), 0, s, a);
    }
}

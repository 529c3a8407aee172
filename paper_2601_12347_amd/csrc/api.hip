// C ABI of the library: context lifetime, model upload, bootstrap inference,
// the per-batch driver (host-side validation and conflict splitting, then the
// device pipeline Apply -> per layer {frontier, scatter, transform}), and the
// read-back calls the tests use.
#include "common.h"
#include "kernels.h"

#include <cstring>
#include <new>

// ---------------------------------------------------------------------------------
// timing
// ---------------------------------------------------------------------------------
struct PhaseTimer {
    struct Rec {
        int phase, layer, e0, e1, counted;
    };
    std::vector<hipEvent_t> ev;
    std::vector<Rec> recs;
    int used = 0;
    int get(ripple_ctx *c) {
        if (used == (int)ev.size()) {
            hipEvent_t e;
            if (hipEventCreate(&e) != hipSuccess) return -1;
            ev.push_back(e);
        }
        return used++;
    }
};

int rp_timer_begin(ripple_ctx *c) {
    if (!c->opt_timing) return -1;
    int e = c->timer->get(c);
    if (e >= 0) hipEventRecord(c->timer->ev[e], c->stream);
    return e;
}

// counted = false: a second stretch of a phase already recorded for this hop (adds time, not a launch)
void rp_timer_end(ripple_ctx *c, int token, int phase, int layer, bool counted) {
    if (token < 0) return;
    int e = c->timer->get(c);
    if (e < 0) return;
    hipEventRecord(c->timer->ev[e], c->stream);
    c->timer->recs.push_back({phase, layer, token, e, counted ? 1 : 0});
}

static void timer_collect(ripple_ctx *c) {       // after the stream has been synchronised
    PhaseTimer *t = c->timer;
    for (const auto &r : t->recs) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, t->ev[r.e0], t->ev[r.e1]) == hipSuccess) {
            c->stats.ms[r.phase][r.layer] += ms;
            c->stats.launches[r.phase][r.layer] += r.counted;
        }
    }
    t->recs.clear();
    t->used = 0;
}

// ---------------------------------------------------------------------------------
// small kernels
// ---------------------------------------------------------------------------------
__global__ void k_store_rows(const float *src, void *dst, size_t n, int store) {
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        if (store) ((__hip_bfloat16 *)dst)[i] = __float2bfloat16(src[i]);
        else ((float *)dst)[i] = src[i];
    }
}

__global__ void k_gather_rows(const void *M, int store, uint32_t d, const uint32_t *ids, uint32_t first,
                              size_t n_rows, uint32_t n_cap, float *out) {
    size_t total = n_rows * d, stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        size_t r = i / d;
        uint32_t col = (uint32_t)(i % d);
        uint32_t id = ids ? ids[r] : (uint32_t)(first + r);
        float v = 0.0f;
        if (id < n_cap) v = rp_load_h(M, store, (size_t)id * d + col);
        out[i] = v;
    }
}

__global__ void k_or_words(uint32_t *dst, const uint32_t *src, uint32_t n) {
    uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n && src[i]) dst[i] |= src[i];
}

__global__ void k_meta_len2(const uint2 *meta, uint32_t n_cap, uint32_t *len) {
    uint32_t v = blockIdx.x * blockDim.x + threadIdx.x;
    if (v < n_cap) len[v] = meta[v].y;
}

__global__ __launch_bounds__(256) void k_export_rows(const uint2 *meta, const uint32_t *pool, const uint32_t *off,
                                                     uint32_t n_cap, int direction, uint32_t *src_out,
                                                     uint32_t *dst_out) {
    const int lane = rp_lane();
    uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    for (uint32_t v = gw; v < n_cap; v += nw) {
        uint2 m = meta[v];
        uint32_t o = off[v];
        for (uint32_t i = lane; i < m.y; i += 64) {
            uint32_t nb = pool[m.x + i];
            src_out[o + i] = direction ? nb : v;
            dst_out[o + i] = direction ? v : nb;
        }
    }
}

// ---------------------------------------------------------------------------------
// helpers
// ---------------------------------------------------------------------------------
static bool is_device_ptr(const void *p) {
    hipPointerAttribute_t at;
    hipError_t e = hipPointerGetAttributes(&at, p);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return at.type == hipMemoryTypeDevice || at.type == hipMemoryTypeManaged;
}

template <typename T>
static ripple_status dev_alloc(ripple_ctx *c, T **p, size_t count, bool zero) {
    size_t bytes = (count ? count : 1) * sizeof(T);
    hipError_t e = hipMalloc((void **)p, bytes);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        c->err = "device allocation of " + std::to_string(bytes) + " bytes failed";
        *p = nullptr;
        return RIPPLE_ENOMEM;
    }
    if (zero) RP_HIP(c, hipMemsetAsync(*p, 0, bytes, c->stream));
    return RIPPLE_OK;
}

#define RP_TRY(expr)                         \
    do {                                     \
        ripple_status rc__ = (expr);         \
        if (rc__ != RIPPLE_OK) return rc__;  \
    } while (0)

static size_t elem_size(const ripple_ctx *c) { return c->store ? 2 : 4; }

static ripple_status fail(ripple_ctx *c, ripple_status rc, const char *msg) {
    c->err = msg;
    return rc;
}

// ---------------------------------------------------------------------------------
// init / destroy
// ---------------------------------------------------------------------------------
static ripple_status init_graph(ripple_ctx **out, uint32_t n_vertices, uint32_t vertex_capacity, uint64_t n_edges,
                                uint64_t edge_capacity, const uint32_t *src, const uint32_t *dst, const float *weights,
                                const float *features, uint32_t d0, int store, void *hip_stream) {
    if (!out) return RIPPLE_EINVAL;
    *out = nullptr;
    if (vertex_capacity == 0 || n_vertices > vertex_capacity || vertex_capacity > (1u << 31) || d0 == 0 ||
        d0 > 1024 || n_edges > edge_capacity || (store != RIPPLE_STORE_F32 && store != RIPPLE_STORE_BF16) ||
        (n_edges && (!src || !dst)) || (n_vertices && !features))
        return RIPPLE_EINVAL;
    uint64_t pool_cap = edge_capacity + edge_capacity / 4 + 8ull * vertex_capacity + 1024;
    if (pool_cap >= (1ull << 32)) return RIPPLE_EINVAL;
    ripple_ctx *c = new (std::nothrow) ripple_ctx();
    if (!c) return RIPPLE_ENOMEM;
    *out = c;                                   // returned even on failure so that the error text can be read
    c->timer = new (std::nothrow) PhaseTimer();
    memset(&c->stats, 0, sizeof(c->stats));
    c->stream = (hipStream_t)hip_stream;
    RP_HIP(c, hipGetDevice(&c->device));
    RP_TRY(rp_static_scratch_init(c));
    int cu = 0;
    RP_HIP(c, hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, c->device));
    c->n_cu = cu > 0 ? (uint32_t)cu : 256u;
    c->n_cap = vertex_capacity;
    c->n_words = rp_div_up(vertex_capacity, 32);
    c->e_cap = edge_capacity;
    c->pool_cap = pool_cap;
    c->store = store;
    c->d[0] = d0;
    const size_t n = c->n_cap;
    RP_TRY(dev_alloc(c, &c->out_meta, n, true));
    RP_TRY(dev_alloc(c, &c->in_meta, n, true));
    RP_TRY(dev_alloc(c, &c->out_capv, n, true));
    RP_TRY(dev_alloc(c, &c->in_capv, n, true));
    RP_TRY(dev_alloc(c, &c->vstate, n, true));
    RP_TRY(dev_alloc(c, &c->pend_out, n, true));
    RP_TRY(dev_alloc(c, &c->pend_in, n, true));
    RP_TRY(dev_alloc(c, &c->dead_out, n, true));
    RP_TRY(dev_alloc(c, &c->dead_in, n, true));
    RP_TRY(dev_alloc(c, &c->hole_out, n, true));
    RP_TRY(dev_alloc(c, &c->hole_in, n, true));
    RP_TRY(dev_alloc(c, &c->out_pool, (size_t)pool_cap, false));
    RP_TRY(dev_alloc(c, &c->in_pool, (size_t)pool_cap, false));
    if (weights) RP_TRY(dev_alloc(c, &c->in_w, (size_t)pool_cap, false));
    RP_TRY(dev_alloc(c, &c->alive, (size_t)c->n_words, true));
    c->n_part = std::max(rp_div_up(n, 1024), rp_div_up(c->n_words, 256)) + 1;
    RP_TRY(dev_alloc(c, &c->part_cnt, (size_t)c->n_part, true));
    RP_TRY(dev_alloc(c, &c->part_deg, (size_t)c->n_part, true));
    RP_TRY(dev_alloc(c, &c->part_ideg, (size_t)c->n_part, true));
    RP_TRY(dev_alloc(c, &c->ctr, 1, true));
    RP_HIP(c, hipHostMalloc((void **)&c->ctr_host, sizeof(DevCtr), hipHostMallocDefault));
    memset(c->ctr_host, 0, sizeof(DevCtr));
    {   // features
        void *h0 = nullptr;
        size_t bytes = n * d0 * elem_size(c);
        hipError_t e = hipMalloc(&h0, bytes ? bytes : 4);
        if (e != hipSuccess) return fail(c, RIPPLE_ENOMEM, "device allocation of the feature matrix failed");
        c->H[0] = h0;
        RP_HIP(c, hipMemsetAsync(h0, 0, bytes, c->stream));
        if (n_vertices) {
            size_t cnt = (size_t)n_vertices * d0;
            if (store == RIPPLE_STORE_F32) {
                RP_HIP(c, hipMemcpyAsync(h0, features, cnt * 4, hipMemcpyHostToDevice, c->stream));
            } else {
                float *tmp = nullptr;
                RP_TRY(dev_alloc(c, &tmp, cnt, false));
                RP_HIP(c, hipMemcpyAsync(tmp, features, cnt * 4, hipMemcpyHostToDevice, c->stream));
                hipLaunchKernelGGL(k_store_rows, dim3(c->n_cu * 8), dim3(256), 0, c->stream, tmp, h0, cnt, 1);
                RP_HIP(c, hipStreamSynchronize(c->stream));
                hipFree(tmp);
            }
        }
    }
    RP_TRY(rp_build_graph(c, n_vertices, n_edges, src, dst, weights));
    // counters that persist across batches
    c->ctr_host->n_alive = n_vertices;
    c->ctr_host->n_edges = n_edges;
    RP_HIP(c, hipMemcpyAsync(&c->ctr->n_alive, &c->ctr_host->n_alive, 4, hipMemcpyHostToDevice, c->stream));
    RP_HIP(c, hipMemcpyAsync(&c->ctr->n_edges, &c->ctr_host->n_edges, 8, hipMemcpyHostToDevice, c->stream));
    RP_HIP(c, hipStreamSynchronize(c->stream));
    c->state = 1;
    return RIPPLE_OK;
}

extern "C" ripple_status ripple_init_graph(ripple_ctx **out, uint32_t n_vertices, uint32_t vertex_capacity,
                                           uint64_t n_edges, uint64_t edge_capacity, const uint32_t *src,
                                           const uint32_t *dst, const float *features, uint32_t d0, int store,
                                           void *hip_stream) {
    return init_graph(out, n_vertices, vertex_capacity, n_edges, edge_capacity, src, dst, nullptr, features, d0, store,
                      hip_stream);
}

extern "C" ripple_status ripple_init_graph_weighted(ripple_ctx **out, uint32_t n_vertices, uint32_t vertex_capacity,
                                                    uint64_t n_edges, uint64_t edge_capacity, const uint32_t *src,
                                                    const uint32_t *dst, const float *edge_weights,
                                                    const float *features, uint32_t d0, int store, void *hip_stream) {
    if (!edge_weights) return RIPPLE_EINVAL;
    return init_graph(out, n_vertices, vertex_capacity, n_edges, edge_capacity, src, dst, edge_weights, features, d0,
                      store, hip_stream);
}

extern "C" void ripple_destroy(ripple_ctx *c) {
    if (!c) return;
    hipStreamSynchronize(c->stream);
    void *ptrs[] = {c->out_meta, c->in_meta, c->out_capv, c->in_capv, c->vstate, c->pend_out, c->pend_in, c->dead_out,
                    c->dead_in, c->hole_out, c->hole_in, c->out_pool, c->in_pool, c->in_w, c->alive, c->part_cnt, c->part_deg, c->part_ideg, c->ioff[0], c->ctr, c->D[0], c->D[1],
                    c->tmp, c->PD, c->MSG, c->side_v, c->side_acc, c->Pold, c->sold, c->seg_v, c->seg_done, c->seg_base, c->seg_r, c->seg_part, c->bm[0], c->rep[0], c->list[0], c->eoff[0], c->all_list, c->ioff_all, c->mk, c->ops_d, c->payload_d,
                    c->op_status, c->op_pos_out, c->op_pos_in, c->op_touch, c->touch_out, c->touch_in, c->exp_kind, c->exp_s, c->exp_a,
                    c->exp_b, c->st_src, c->st_dst, c->st_sign, c->st_unit, c->tail_ids, c->tail_q, c->tail_w, c->sk_in, c->sk_out, c->sv_in, c->sv_out, c->sort_tmp, c->gather_d, c->gather_ids, c->pk_a, c->pk_b, c->pv_a, c->pv_b, c->pair_tmp};
    for (void *p : ptrs)
        if (p) hipFree(p);
    for (uint32_t l = 0; l <= RIPPLE_MAX_LAYERS; ++l) {
        if (c->H[l]) hipFree(c->H[l]);
        if (c->X[l]) hipFree(c->X[l]);
    }
    for (uint32_t l = 0; l < c->L; ++l) {
        LayerDev &ly = c->layers[l];
        void *w[] = {ly.W0, ly.b0, ly.W1, ly.b1, ly.W0h, ly.W1h, ly.bzero, (ly.Wn != ly.W0) ? ly.Wn : nullptr, ly.PS,
                     ly.W0s, ly.W1s, (ly.Wns != ly.W0s) ? ly.Wns : nullptr,
                     ly.att, ly.P, ly.ssrc, ly.sdst, ly.den, ly.T, ly.Wc, ly.bzero_c, ly.Wc96, ly.Wc96p};
        for (void *p : w)
            if (p) hipFree(p);
    }
    if (c->ctr_host) hipHostFree(c->ctr_host);
    if (c->ops_pin) hipHostFree(c->ops_pin);
    if (c->payload_pin) hipHostFree(c->payload_pin);
    if (c->timer) {
        for (hipEvent_t e : c->timer->ev) hipEventDestroy(e);
        delete c->timer;
    }
    delete c;
}

extern "C" const char *ripple_last_error(const ripple_ctx *c) { return c ? c->err.c_str() : ""; }

// ---------------------------------------------------------------------------------
// model
// ---------------------------------------------------------------------------------
static uint32_t pad_n(uint32_t n) { return n <= 64 ? 64u : (n <= 128 ? 128u : rp_round_up(n, 256)); }

// planes (optional): the padded matrix as three transposed bf16 matrices [Npad x Kpad] whose sum is W exactly
// (leading, middle and last 8 significant bits of every weight), for the split products on the bf16 matrix cores
static ripple_status upload_padded(ripple_ctx *c, const float *w, const float *b, uint32_t K, uint32_t N,
                                   uint32_t Kpad, uint32_t Npad, float **W_d, float **b_d,
                                   unsigned short **planes = nullptr) {
    std::vector<float> wp((size_t)Kpad * Npad, 0.0f), bp(Npad, 0.0f);
    for (uint32_t k = 0; k < K; ++k) memcpy(&wp[(size_t)k * Npad], &w[(size_t)k * N], (size_t)N * 4);
    memcpy(bp.data(), b, (size_t)N * 4);
    if (planes) {
        const size_t plane = (size_t)Npad * Kpad;
        std::vector<uint16_t> pl(3 * plane, 0);
        for (uint32_t k = 0; k < K; ++k)
            for (uint32_t j = 0; j < N; ++j) {
                float x = wp[(size_t)k * Npad + j];
                for (int p = 0; p < 3; ++p) {
                    uint32_t bits;
                    memcpy(&bits, &x, 4);
                    bits &= 0xFFFF0000u;
                    float head;
                    memcpy(&head, &bits, 4);
                    pl[p * plane + (size_t)j * Kpad + k] = (uint16_t)(bits >> 16);
                    x -= head;                         // exact
                }
            }
        RP_TRY(dev_alloc(c, planes, pl.size(), false));
        RP_HIP(c, hipMemcpy(*planes, pl.data(), pl.size() * 2, hipMemcpyHostToDevice));
    }
    RP_TRY(dev_alloc(c, W_d, wp.size(), false));
    RP_TRY(dev_alloc(c, b_d, bp.size(), false));
    RP_HIP(c, hipMemcpy(*W_d, wp.data(), wp.size() * 4, hipMemcpyHostToDevice));
    RP_HIP(c, hipMemcpy(*b_d, bp.data(), bp.size() * 4, hipMemcpyHostToDevice));
    return RIPPLE_OK;
}

extern "C" ripple_status ripple_load_model(ripple_ctx *c, uint32_t n_layers, const ripple_layer_desc *layers) {
    if (!c) return RIPPLE_EINVAL;
    if (c->state != 1) return fail(c, RIPPLE_ESTATE, "load_model needs a context fresh from init_graph");
    if (!layers || n_layers == 0 || n_layers > RIPPLE_MAX_LAYERS) return fail(c, RIPPLE_EINVAL, "bad layer count");
    uint32_t prev = c->d[0];
    for (uint32_t l = 0; l < n_layers; ++l) {
        const ripple_layer_desc &s = layers[l];
        if (s.d_in != prev || s.d_out == 0 || s.d_out > 1024 || s.d_hidden > 1024 || s.agg > RIPPLE_AGG_ATTN ||
            s.self_mode > RIPPLE_SELF_ADD || s.act_inner > RIPPLE_ACT_RELU || s.act_out > RIPPLE_ACT_RELU || !s.W0 ||
            !s.b0 || (s.d_hidden && (!s.W1 || !s.b1)))
            return fail(c, RIPPLE_EINVAL, "bad layer descriptor (widths must chain, dims <= 1024, pointers set)");
        if (s.agg == RIPPLE_AGG_WSUM && !c->in_w)
            return fail(c, RIPPLE_EINVAL, "weighted-sum layer on a graph that was built without edge weights");
        if (s.agg == RIPPLE_AGG_ATTN && (!s.att || s.self_mode != RIPPLE_SELF_NONE || s.d_hidden))
            return fail(c, RIPPLE_EINVAL, "attention layer: att must be set, self_mode none, d_hidden 0");
        if ((s.agg == RIPPLE_AGG_WSUM || s.agg >= RIPPLE_AGG_MAX) && c->opt_deterministic)
            return fail(c, RIPPLE_EINVAL, "the deterministic mode takes sum and mean layers only");
        prev = s.d_out;
    }
    c->L = n_layers;
    c->dmax = c->d[0];
    c->hmax = 0;
    for (uint32_t l = 0; l < n_layers; ++l) {
        const ripple_layer_desc &s = layers[l];
        LayerDev &ly = c->layers[l];
        memset(&ly, 0, sizeof(ly));
        ly.d_in = s.d_in;
        ly.d_hidden = s.d_hidden;
        ly.d_out = s.d_out;
        ly.K = (s.self_mode == RIPPLE_SELF_CONCAT) ? 2 * s.d_in : s.d_in;
        ly.agg = s.agg;
        ly.self_mode = s.self_mode;
        ly.act_inner = s.act_inner;
        ly.act_out = s.act_out;
        ly.eps = s.eps;
        uint32_t n0 = s.d_hidden ? s.d_hidden : s.d_out;
        ly.K0pad = rp_round_up(ly.K, 32);
        ly.N0pad = pad_n(n0);
        const bool split = c->store == RIPPLE_STORE_F32 && c->opt_split;
        RP_TRY(upload_padded(c, s.W0, s.b0, ly.K, n0, ly.K0pad, ly.N0pad, &ly.W0, &ly.b0, split ? &ly.W0s : nullptr));
        if (c->store == RIPPLE_STORE_BF16) {               // transposed bf16 copy for the bf16 matrix cores
            std::vector<uint16_t> wt((size_t)ly.N0pad * ly.K0pad, 0);
            for (uint32_t k = 0; k < ly.K; ++k)
                for (uint32_t j = 0; j < n0; ++j) {
                    uint32_t bits;
                    memcpy(&bits, &s.W0[(size_t)k * n0 + j], 4);
                    bits += 0x7FFFu + ((bits >> 16) & 1u);      // round to nearest even
                    wt[(size_t)j * ly.K0pad + k] = (uint16_t)(bits >> 16);
                }
            RP_TRY(dev_alloc(c, &ly.W0h, wt.size(), false));
            RP_HIP(c, hipMemcpy(ly.W0h, wt.data(), wt.size() * 2, hipMemcpyHostToDevice));
        }
        // project first where the single linear map shrinks the row at least by half
        ly.proj = (c->opt_project && s.agg < RIPPLE_AGG_MAX && s.d_hidden == 0 && s.self_mode != RIPPLE_SELF_ADD && 2 * s.d_out <= s.d_in) ? 1u : 0u;
        ly.selfc = (c->opt_selfcache && s.d_hidden == 0 && s.self_mode == RIPPLE_SELF_CONCAT) ? 1u : 0u;
        if (s.agg == RIPPLE_AGG_ATTN) {
            RP_TRY(dev_alloc(c, &ly.att, (size_t)2 * s.d_out, false));
            RP_HIP(c, hipMemcpy(ly.att, s.att, (size_t)2 * s.d_out * 4, hipMemcpyHostToDevice));
            RP_TRY(dev_alloc(c, &ly.bzero, (size_t)ly.N0pad, true));
            RP_TRY(dev_alloc(c, &ly.P, (size_t)c->n_cap * s.d_out, true));
            RP_TRY(dev_alloc(c, &ly.ssrc, (size_t)c->n_cap, true));
            RP_TRY(dev_alloc(c, &ly.sdst, (size_t)c->n_cap, true));
            RP_TRY(dev_alloc(c, &ly.den, (size_t)c->n_cap, true));
        }
        if (ly.proj || ly.selfc) {
            std::vector<float> zeros(ly.N0pad, 0.0f);
            if (s.self_mode == RIPPLE_SELF_CONCAT) {           // rows d_in .. 2 d_in - 1 of W0
                RP_TRY(upload_padded(c, s.W0 + (size_t)s.d_in * s.d_out, zeros.data(), s.d_in, s.d_out,
                                     rp_round_up(s.d_in, 32), ly.N0pad, &ly.Wn, &ly.bzero, split ? &ly.Wns : nullptr));
                ly.Wns_ld = rp_round_up(s.d_in, 32);
            } else {
                ly.Wn = ly.W0;
                ly.Wns = ly.W0s;
                ly.Wns_ld = ly.K0pad;
                RP_TRY(dev_alloc(c, &ly.bzero, (size_t)ly.N0pad, true));
            }
        }
        if (ly.proj && ly.selfc && s.d_out <= 64 && s.d_in % 4 == 0 && !split) {
            const uint32_t kp = rp_round_up(s.d_in, 32);
            std::vector<float> wc((size_t)kp * 128, 0.0f);
            for (uint32_t k = 0; k < s.d_in; ++k)
                for (uint32_t j = 0; j < s.d_out; ++j) {
                    wc[(size_t)k * 128 + j] = s.W0[(size_t)k * s.d_out + j];                       // W_self
                    wc[(size_t)k * 128 + 64 + j] = s.W0[(size_t)(s.d_in + k) * s.d_out + j];       // W_neigh
                }
            RP_TRY(dev_alloc(c, &ly.Wc, wc.size(), false));
            RP_HIP(c, hipMemcpy(ly.Wc, wc.data(), wc.size() * 4, hipMemcpyHostToDevice));
            RP_TRY(dev_alloc(c, &ly.bzero_c, (size_t)128, true));
            if (s.d_out <= 48) {
                std::vector<float> w96((size_t)kp * 96, 0.0f);
                for (uint32_t k = 0; k < s.d_in; ++k)
                    for (uint32_t j = 0; j < s.d_out; ++j) {
                        w96[(size_t)k * 96 + j] = s.W0[(size_t)k * s.d_out + j];
                        w96[(size_t)k * 96 + 48 + j] = s.W0[(size_t)(s.d_in + k) * s.d_out + j];
                    }
                RP_TRY(dev_alloc(c, &ly.Wc96, w96.size(), false));
                RP_HIP(c, hipMemcpy(ly.Wc96, w96.data(), w96.size() * 4, hipMemcpyHostToDevice));
                if (s.d_in == 256 && s.d_out > 16) {           // [k][n][j]: n < 16 column 16 j + n of W_self, else 16 j + n - 16 of W_neigh
                    std::vector<float> wp((size_t)256 * 96, 0.0f);
                    for (uint32_t k = 0; k < 256; ++k)
                        for (uint32_t n = 0; n < 32; ++n)
                            for (uint32_t j = 0; j < 3; ++j) {
                                const uint32_t col = 16 * j + (n & 15u);
                                if (col >= s.d_out) continue;
                                wp[((size_t)k * 32 + n) * 3 + j] = s.W0[(size_t)((n < 16 ? 0 : s.d_in) + k) * s.d_out + col];
                            }
                    RP_TRY(dev_alloc(c, &ly.Wc96p, wp.size(), false));
                    RP_HIP(c, hipMemcpy(ly.Wc96p, wp.data(), wp.size() * 4, hipMemcpyHostToDevice));
                }
            }
        }
        if (s.d_hidden) {
            ly.K1pad = rp_round_up(s.d_hidden, 32);
            ly.N1pad = pad_n(s.d_out);
            RP_TRY(upload_padded(c, s.W1, s.b1, s.d_hidden, s.d_out, ly.K1pad, ly.N1pad, &ly.W1, &ly.b1, split ? &ly.W1s : nullptr));
        }
        c->d[l + 1] = s.d_out;
        c->dmax = std::max(c->dmax, s.d_out);
        c->hmax = std::max(c->hmax, s.d_hidden);
    }
    const size_t n = c->n_cap;
    for (uint32_t l = 1; l <= c->L; ++l) {
        void *h = nullptr;
        size_t bytes = n * c->d[l] * elem_size(c);
        if (hipMalloc(&h, bytes) != hipSuccess) return fail(c, RIPPLE_ENOMEM, "device allocation of H failed");
        c->H[l] = h;
        RP_HIP(c, hipMemsetAsync(h, 0, bytes, c->stream));
        c->xw[l] = (c->layers[l - 1].proj || rp_layer_attn(c, l)) ? c->d[l] : c->d[l - 1];
        RP_TRY(dev_alloc(c, &c->X[l], n * c->xw[l], true));
        if (c->layers[l - 1].selfc) RP_TRY(dev_alloc(c, &c->layers[l - 1].PS, n * c->d[l], true));
        if (c->layers[l - 1].proj) {
            RP_TRY(dev_alloc(c, &c->layers[l - 1].T, n * c->d[l], true));
            // packed rows are addressed with 32-bit byte offsets (vertex id * 128): below 2^25 vertices
            c->layers[l - 1].packed = (c->opt_pack && n < (1u << 25)) ? rp_msg_packed(c->d[l]) : 0u;
        }
    }
    {
        uint32_t aw = 0;                                 // widest attention layer
        for (uint32_t l = 1; l <= c->L; ++l)
            if (rp_layer_attn(c, l)) aw = std::max(aw, c->d[l]);
        if (aw) {
            RP_TRY(dev_alloc(c, &c->Pold, n * aw, true));
            RP_TRY(dev_alloc(c, &c->sold, n, true));
        }
    }
    {
        uint32_t mw = 0;                                 // widest max / min aggregate, widest attention numerator and its denominator
        for (uint32_t l = 1; l <= c->L; ++l) {
            if (rp_layer_mono(c, l)) mw = std::max(mw, c->xw[l]);
            if (rp_layer_attn(c, l)) mw = std::max(mw, c->d[l] + 1);
        }
        if (mw) {                                        // in-rows sum to at most the pool: that bounds rows and segments
            c->big_cap = (uint32_t)std::min<uint64_t>(c->pool_cap / ROW_SPLIT_MIN + 1, ROW_SEG_MAX);
            c->seg_cap = (uint32_t)std::min<uint64_t>(c->pool_cap / ROW_SEG + c->big_cap, ROW_SEG_MAX);
            c->seg_ld = rp_round_up(mw, 32);             // partial rows share no 128-byte line
            RP_TRY(dev_alloc(c, &c->seg_v, c->big_cap, false));
            RP_TRY(dev_alloc(c, &c->seg_done, c->big_cap, false));
            RP_TRY(dev_alloc(c, &c->seg_base, c->big_cap, false));
            RP_TRY(dev_alloc(c, &c->seg_r, c->seg_cap, false));
            RP_TRY(dev_alloc(c, &c->seg_part, (size_t)c->seg_cap * c->seg_ld, false));
        }
    }
    RP_TRY(dev_alloc(c, &c->D[0], n * c->dmax, false));
    RP_TRY(dev_alloc(c, &c->D[1], n * c->dmax, false));
    if (c->hmax) RP_TRY(dev_alloc(c, &c->tmp, n * c->hmax, false));
    {
        uint32_t pw = 0;
        for (uint32_t l = 1; l <= c->L; ++l)
            if (c->layers[l - 1].proj) pw = std::max(pw, c->d[l]);
        c->pd_ld = pw <= 32 ? 32 : rp_round_up(pw, 16);  // up to 32 columns: one 128-byte line per row; else 64-byte multiples
        if (pw) RP_TRY(dev_alloc(c, &c->PD, n * c->pd_ld, true));
        bool packed = false;
        for (uint32_t l = 1; l <= c->L; ++l) packed |= c->layers[l - 1].proj && c->layers[l - 1].packed;
        if (packed) RP_TRY(dev_alloc(c, &c->MSG, n * RP_MSG_WORDS, true));
    }
    if (c->opt_deterministic) {                          // two side entries per run of chunks of the pull kernels
        uint32_t xmax = 1;
        for (uint32_t l = 1; l <= c->L; ++l) xmax = std::max(xmax, c->xw[l]);
        // runs: up to four per wavefront of the grid while a run is shorter than eight chunks, else an eighth of the chunks
        // (256 in-row entries each) that the in-row pool can hold
        const size_t nw = (size_t)c->n_cu * 8 * 4;
        c->side_runs = (uint32_t)std::max<size_t>(4 * nw, c->pool_cap / (256 * 8) + 2);
        const size_t entries = 2 * (size_t)c->side_runs;
        RP_TRY(dev_alloc(c, &c->side_v, entries, false));
        RP_TRY(dev_alloc(c, &c->side_acc, entries * xmax, false));
    }
    if (!c->opt_deterministic) {
        // (destination, source) pairs of a hop's messages, before and after the sort by destination: room for a quarter
        // of the edge capacity (a hop with more messages than that is pulled or discovers), at most 2^25
        c->pair_cap = (uint32_t)std::min<uint64_t>(std::max<uint64_t>(c->pool_cap / 4, 1u << 14), 1u << 25);
        c->pair_bits = 1;
        while (c->pair_bits < 32 && (1ull << c->pair_bits) <= n) ++c->pair_bits;   // 2^bits > every vertex id; the filler key has all of them set
        c->pair_tmp_bytes = rp_sort_u32_tmp_bytes(c->pair_cap);
        if (c->pair_tmp_bytes) {
            uint8_t *tmp = nullptr;
            RP_TRY(dev_alloc(c, &c->pk_a, c->pair_cap, false));
            RP_TRY(dev_alloc(c, &c->pk_b, c->pair_cap, false));
            RP_TRY(dev_alloc(c, &c->pv_a, c->pair_cap, false));
            RP_TRY(dev_alloc(c, &c->pv_b, c->pair_cap, false));
            RP_TRY(dev_alloc(c, &tmp, c->pair_tmp_bytes, false));
            c->pair_tmp = tmp;
        } else {
            c->pair_cap = 0;
        }
    }
    // bitmaps: layers 0..L, then S, then V_added, contiguous; reporting copies separately
    uint32_t *bmall = nullptr, *repall = nullptr, *lists = nullptr, *eoffs = nullptr, *ioffs = nullptr;
    RP_TRY(dev_alloc(c, &bmall, (size_t)c->n_words * (c->L + 3), true));
    RP_TRY(dev_alloc(c, &repall, (size_t)c->n_words * (c->L + 1), true));
    RP_TRY(dev_alloc(c, &lists, (n + 1) * (c->L + 1), true));
    RP_TRY(dev_alloc(c, &eoffs, (n + 1) * (c->L + 1), true));
    RP_TRY(dev_alloc(c, &ioffs, (n + 1) * (c->L + 1), true));
    for (uint32_t l = 0; l <= c->L; ++l) {
        c->bm[l] = bmall + (size_t)l * c->n_words;
        c->rep[l] = repall + (size_t)l * c->n_words;
        c->list[l] = lists + (size_t)l * (n + 1);
        c->eoff[l] = eoffs + (size_t)l * (n + 1);
        c->ioff[l] = ioffs + (size_t)l * (n + 1);
    }
    c->bm_sink = bmall + (size_t)(c->L + 1) * c->n_words;
    c->bm_vadd = bmall + (size_t)(c->L + 2) * c->n_words;
    RP_TRY(dev_alloc(c, &c->all_list, n + 1, true));
    {
        uint32_t *mkw = nullptr;                         // n_words * 32 bytes
        RP_TRY(dev_alloc(c, &mkw, (size_t)c->n_words * 8, true));
        c->mk = (uint8_t *)mkw;
    }
    RP_TRY(dev_alloc(c, &c->ioff_all, n + 1, true));
    RP_HIP(c, hipStreamSynchronize(c->stream));
    c->state = 2;
    return RIPPLE_OK;
}

static ripple_status range_error(ripple_ctx *c, uint32_t rows) {
    c->err = "attention exponentials overflowed the float range: " + std::to_string(rows) +
             " row updates used sums that were not finite (scores must stay below about 88)";
    return RIPPLE_ERANGE;
}

// ---------------------------------------------------------------------------------
// bootstrap inference
// ---------------------------------------------------------------------------------
extern "C" ripple_status ripple_full_infer(ripple_ctx *c) {
    if (!c) return RIPPLE_EINVAL;
    if (c->state < 2) return fail(c, RIPPLE_ESTATE, "full_infer needs init_graph and load_model first");
    // all live vertices as one list (the alive bitmap itself is the source)
    hipLaunchKernelGGL(k_or_words, dim3(rp_div_up(c->n_words, 256)), dim3(256), 0, c->stream, c->bm[0], c->alive,
                       c->n_words);
    rp_launch_bitmap_to_list(c, c->bm[0], c->all_list, &c->ctr->a[0]);
    if (c->opt_deterministic) rp_launch_alive_list(c);     // the same list once more, with its in-degree prefix
    for (uint32_t l = 1; l <= c->L; ++l) {
        if (rp_layer_attn(c, l)) {
            rp_launch_gat_project(c, l, c->all_list, &c->ctr->a[0]);
            rp_launch_gat_scores(c, l, c->all_list, &c->ctr->a[0]);
            rp_launch_gat_scatter(c, l, true);
            rp_launch_transform(c, l, c->all_list, &c->ctr->a[0], false);
            continue;
        }
        if (rp_has_project_both(c, l)) {
            rp_launch_project_both(c, l, c->all_list, &c->ctr->a[0], true);
        } else {
            if (c->layers[l - 1].proj) rp_launch_project(c, l, c->all_list, &c->ctr->a[0], true);
            if (c->layers[l - 1].selfc) rp_launch_self_project(c, l, c->all_list, &c->ctr->a[0]);
        }
        if (c->opt_deterministic) rp_launch_scatter_pull_det(c, l, true);  // same summation order as the batches use
        else rp_launch_pull_all(c, l);
        rp_launch_transform(c, l, c->all_list, &c->ctr->a[0], false);
    }
    RP_HIP(c, hipMemcpyAsync(c->ctr_host, c->ctr, sizeof(DevCtr), hipMemcpyDeviceToHost, c->stream));
    rp_launch_batch_reset(c);
    RP_HIP(c, hipStreamSynchronize(c->stream));
    RP_HIP(c, hipGetLastError());
    const uint32_t range_rows = c->ctr_host->range_rows;
    for (uint32_t l = 0; l <= c->L; ++l) c->last_a[l] = 0;
    c->hints_valid = false;
    c->last_n_ops = 0;
    c->last_from_rep = false;
    c->state = 3;
    if (range_rows) return range_error(c, range_rows);
    return RIPPLE_OK;
}

// ---------------------------------------------------------------------------------
// per-batch driver
// ---------------------------------------------------------------------------------
// Flat hash over the keys a sub-batch has touched: edge (u,v) -> present,
// vertex w -> flags. Entries are valid only for the current generation.
struct TouchTable {
    std::vector<uint64_t> keys;
    std::vector<uint32_t> gen;
    std::vector<uint8_t> val;
    uint32_t cur = 1;
    size_t mask = 0;
    void reserve(size_t n_keys) {
        size_t want = 64;
        while (want < n_keys * 4) want <<= 1;
        if (want > keys.size()) {
            keys.assign(want, 0);
            gen.assign(want, 0);
            val.assign(want, 0);
            cur = 1;
        }
        mask = keys.size() - 1;
    }
    void next_generation() {
        if (++cur == 0) {
            std::fill(gen.begin(), gen.end(), 0);
            cur = 1;
        }
    }
    uint8_t *find(uint64_t key, bool insert) {
        size_t h = (size_t)((key * 0x9E3779B97F4A7C15ull) >> 20) & mask;
        for (;;) {
            if (gen[h] != cur) {
                if (!insert) return nullptr;
                gen[h] = cur;
                keys[h] = key;
                val[h] = 0;
                return &val[h];
            }
            if (keys[h] == key) return &val[h];
            h = (h + 1) & mask;
        }
    }
};

#define TF_EDGE_REF 1
#define TF_FEAT 2
#define TF_VADD 4
#define TF_VDEL 8

struct SubBatch {
    uint32_t begin, end;
    bool has_vadd, has_vdel, has_vertex_or_feat;
};

// Cut the batch where an operation depends on an earlier one of the same piece, so that every
// piece can be applied in parallel with the same result as applying it in array order.
static void split_batch(const ripple_update *ops, uint32_t n, TouchTable &tt, std::vector<SubBatch> &out) {
    out.clear();
    tt.reserve((size_t)n * 3 + 16);
    tt.next_generation();
    SubBatch cur{0, 0, false, false, false};
    const uint64_t VKEY = 0x8000000000000000ull;
    for (uint32_t i = 0; i < n; ++i) {
        const ripple_update &op = ops[i];
        for (int attempt = 0; attempt < 2; ++attempt) {
            bool conflict = false;
            if (op.kind == RIPPLE_EDGE_ADD || op.kind == RIPPLE_EDGE_DEL || op.kind == RIPPLE_EDGE_REWEIGHT) {
                uint64_t ek = ((uint64_t)op.u << 32) | op.v;
                uint8_t *fu = tt.find(VKEY | op.u, false), *fv = tt.find(VKEY | op.v, false);
                if (tt.find(ek, false) || (fu && (*fu & TF_VDEL)) || (fv && (*fv & TF_VDEL))) conflict = true;
                else {
                    *tt.find(ek, true) = 1;
                    *tt.find(VKEY | op.u, true) |= TF_EDGE_REF;
                    *tt.find(VKEY | op.v, true) |= TF_EDGE_REF;
                }
            } else {
                uint8_t *f = tt.find(VKEY | op.u, false);
                uint8_t flags = f ? *f : 0;
                if (op.kind == RIPPLE_FEAT_UPDATE) {
                    if (flags & (TF_FEAT | TF_VADD | TF_VDEL)) conflict = true;
                    else *tt.find(VKEY | op.u, true) |= TF_FEAT;
                } else {
                    if (flags) conflict = true;
                    else *tt.find(VKEY | op.u, true) |= (op.kind == RIPPLE_VERTEX_ADD ? TF_VADD : TF_VDEL);
                }
            }
            if (!conflict) break;
            cur.end = i;                       // close the piece before this operation and start afresh
            out.push_back(cur);
            cur = SubBatch{i, i, false, false, false};
            tt.next_generation();
        }
        if (op.kind == RIPPLE_VERTEX_DEL) cur.has_vdel = true;
        if (op.kind == RIPPLE_VERTEX_ADD) cur.has_vadd = true;
        if (op.kind >= RIPPLE_VERTEX_ADD && op.kind <= RIPPLE_FEAT_UPDATE) cur.has_vertex_or_feat = true;
    }
    cur.end = n;
    if (cur.end > cur.begin || out.empty()) out.push_back(cur);
}

static bool ops_in_range(const ripple_update *ops, uint32_t n_ops, uint32_t n_cap, uint32_t n_feat_rows) {
    for (uint32_t i = 0; i < n_ops; ++i) {
        const ripple_update &op = ops[i];
        bool bad = op.kind > RIPPLE_EDGE_REWEIGHT || op.u >= n_cap;
        if (!bad && (op.kind <= RIPPLE_EDGE_DEL || op.kind == RIPPLE_EDGE_REWEIGHT)) bad = op.v >= n_cap;
        if (!bad && (op.kind == RIPPLE_VERTEX_ADD || op.kind == RIPPLE_FEAT_UPDATE)) bad = op.feat_row >= n_feat_rows;
        if (bad) return false;
    }
    return true;
}

extern "C" ripple_status ripple_plan_batch(const ripple_update *ops, uint32_t n_ops, uint32_t vertex_capacity,
                                           uint32_t n_feat_rows, uint32_t *piece_end, uint32_t cap, uint32_t *n_pieces) {
    if ((n_ops && !ops) || !n_pieces || (cap && !piece_end)) return RIPPLE_EINVAL;
    if (!ops_in_range(ops, n_ops, vertex_capacity, n_feat_rows)) return RIPPLE_EINVAL;
    *n_pieces = 0;
    if (n_ops == 0) return RIPPLE_OK;
    TouchTable tt;
    std::vector<SubBatch> pieces;
    split_batch(ops, n_ops, tt, pieces);
    for (size_t p = 0; p < pieces.size(); ++p)
        if (p < cap) piece_end[p] = pieces[p].end;
    *n_pieces = (uint32_t)pieces.size();
    return RIPPLE_OK;
}

static ripple_status ensure_batch_buffers(ripple_ctx *c, uint32_t n_ops, uint32_t n_feat, uint32_t want_exp) {
    if (n_ops > c->ops_cap || want_exp > c->exp_cap) {
        RP_HIP(c, hipStreamSynchronize(c->stream));
        uint32_t cap = std::max<uint32_t>(std::max<uint32_t>(n_ops, c->ops_cap), 4096);
        cap = rp_round_up(cap + cap / 2, 1024);
        uint32_t exp = std::max<uint32_t>(std::max<uint32_t>(want_exp, c->exp_cap), 1u << 20);
        void *old[] = {c->ops_d, c->op_status, c->op_pos_out, c->op_pos_in, c->op_touch, c->touch_out, c->touch_in, c->exp_kind, c->exp_s,
                       c->exp_a, c->exp_b, c->st_src, c->st_dst, c->st_sign, c->st_unit, c->tail_ids, c->tail_q, c->tail_w, c->sk_in, c->sk_out, c->sv_in, c->sv_out, c->sort_tmp};
        for (void *p : old)
            if (p) hipFree(p);
        c->tail_ids = c->tail_q = nullptr;
        c->tail_w = nullptr;
        c->sk_in = c->sk_out = nullptr;
        c->sv_in = c->sv_out = nullptr;
        c->sort_tmp = nullptr;
        c->ops_cap = c->exp_cap = c->touch_cap = c->struct_cap = 0;
        RP_TRY(dev_alloc(c, &c->ops_d, cap, false));
        RP_TRY(dev_alloc(c, &c->op_status, cap, true));
        RP_TRY(dev_alloc(c, &c->op_pos_out, cap, true));
        RP_TRY(dev_alloc(c, &c->op_pos_in, cap, true));
        RP_TRY(dev_alloc(c, &c->op_touch, cap, true));
        RP_TRY(dev_alloc(c, &c->touch_out, (size_t)cap + exp, false));
        RP_TRY(dev_alloc(c, &c->touch_in, (size_t)cap + exp, false));
        RP_TRY(dev_alloc(c, &c->exp_kind, exp, false));
        RP_TRY(dev_alloc(c, &c->exp_s, exp, false));
        RP_TRY(dev_alloc(c, &c->exp_a, exp, false));
        RP_TRY(dev_alloc(c, &c->exp_b, exp, false));
        RP_TRY(dev_alloc(c, &c->st_src, (size_t)cap + exp, false));
        RP_TRY(dev_alloc(c, &c->st_dst, (size_t)cap + exp, false));
        RP_TRY(dev_alloc(c, &c->st_sign, (size_t)cap + exp, false));
        RP_TRY(dev_alloc(c, &c->st_unit, (size_t)cap + exp, false));
        if (c->opt_deterministic) {
            RP_TRY(dev_alloc(c, &c->tail_ids, cap, false));
            RP_TRY(dev_alloc(c, &c->tail_w, cap, false));
            RP_TRY(dev_alloc(c, &c->tail_q, (size_t)cap + exp, false));
            RP_TRY(dev_alloc(c, &c->sk_in, (size_t)cap + exp, false));
            RP_TRY(dev_alloc(c, &c->sk_out, (size_t)cap + exp, false));
            RP_TRY(dev_alloc(c, &c->sv_in, (size_t)cap + exp, false));
            RP_TRY(dev_alloc(c, &c->sv_out, (size_t)cap + exp, false));
            c->sort_tmp_bytes = rp_sort_u64_tmp_bytes((size_t)cap + exp);
            if (!c->sort_tmp_bytes) return fail(c, RIPPLE_EDEVICE, "the sort's temporary storage could not be sized");
            unsigned char *tmp = nullptr;
            RP_TRY(dev_alloc(c, &tmp, c->sort_tmp_bytes, false));
            c->sort_tmp = tmp;
        }
        c->ops_cap = cap;
        c->exp_cap = exp;
        c->touch_cap = cap + exp;
        c->struct_cap = cap + exp;
    }
    if (n_ops > c->pin_ops_cap) {
        if (c->ops_pin) hipHostFree(c->ops_pin);
        c->ops_pin = nullptr;
        c->pin_ops_cap = 0;
        RP_HIP(c, hipHostMalloc((void **)&c->ops_pin, (size_t)c->ops_cap * sizeof(ripple_update), hipHostMallocDefault));
        c->pin_ops_cap = c->ops_cap;
    }
    if (n_feat > c->feat_cap) {
        RP_HIP(c, hipStreamSynchronize(c->stream));
        uint32_t cap = rp_round_up(std::max<uint32_t>(n_feat + n_feat / 2, 1024), 256);
        if (c->payload_d) hipFree(c->payload_d);
        if (c->payload_pin) hipHostFree(c->payload_pin);
        c->payload_d = nullptr;
        c->payload_pin = nullptr;
        c->feat_cap = 0;
        RP_TRY(dev_alloc(c, &c->payload_d, (size_t)cap * c->d[0], false));
        RP_HIP(c, hipHostMalloc((void **)&c->payload_pin, (size_t)cap * c->d[0] * 4, hipHostMallocDefault));
        c->feat_cap = cap;
    }
    return RIPPLE_OK;
}

// A_{l-1} is part of A_l: the layer reads the vertex's own row (a self term, or its attention score)
#define SPARSE_MAX_ROWS 4096u
#define SPARSE_MAX_EDGES 65536u

// Hop l + 1 forwards D^l = new - old rows of layer l, unless its layer is handled project-first: that one
// sends H^l W_neigh minus what it has sent before and never looks at the difference.
static bool next_reads_delta(const ripple_ctx *c, uint32_t l) { return l < c->L && !c->layers[l].proj; }

static bool layer_self(const ripple_ctx *c, uint32_t l) {
    return c->layers[l - 1].self_mode != RIPPLE_SELF_NONE || rp_layer_attn(c, l);
}

// Hop l's set (and the previous hop's) was small in the previous batch, which was of about this size: the
// hop lists its vertices while marking them instead of scanning the bitmap. Only a choice between two
// correct paths.
static bool small_frontier(const ripple_ctx *c, uint32_t l, uint32_t n_ops, bool multi) {
    return c->opt_sparse && !multi && c->last_a[l] <= SPARSE_MAX_ROWS && c->last_a[l - 1] <= SPARSE_MAX_ROWS &&
           c->last_m[l] <= SPARSE_MAX_EDGES && c->last_n_ops && n_ops <= 2 * c->last_n_ops;
}

// Enqueue one conflict-free piece: Apply, then hop by hop frontier / scatter / transform.
static void enqueue_piece(ripple_ctx *c, const SubBatch &sb, bool multi) {
    const uint32_t n = sb.end - sb.begin;
    int t = rp_timer_begin(c);
    rp_launch_batch_reset(c);
    rp_launch_mutate(c, n, sb.has_vadd, sb.has_vdel, sb.has_vertex_or_feat);
    rp_launch_list_eoff(c, 0);
    rp_timer_end(c, t, RIPPLE_PH_INGEST, 0);
    if (multi)
        hipLaunchKernelGGL(k_or_words, dim3(rp_div_up(c->n_words, 256)), dim3(256), 0, c->stream, c->rep[0], c->bm[0],
                           c->n_words);
    bool have_all = false;                              // live-vertex list of this piece exists
    if (c->opt_deterministic) {                         // one owner per aggregate row, fixed summation order
        for (uint32_t l = 1; l <= c->L; ++l) {
            t = rp_timer_begin(c);
            rp_launch_frontier_mark(c, l, false);
            rp_timer_end(c, t, RIPPLE_PH_FRONTIER, (int)l);
            t = rp_timer_begin(c);
            rp_launch_frontier_compact(c, l, layer_self(c, l), l < c->L, true, multi);
            rp_timer_end(c, t, RIPPLE_PH_COMPACT, (int)l);
            if (c->layers[l - 1].proj || c->layers[l - 1].selfc) {
                t = rp_timer_begin(c);
                if (rp_has_project_both(c, l)) {
                    rp_launch_project_both(c, l, c->list[l - 1], &c->ctr->a[l - 1], false);
                } else {
                    if (c->layers[l - 1].proj) rp_launch_project(c, l, c->list[l - 1], &c->ctr->a[l - 1], false);
                    if (c->layers[l - 1].selfc) rp_launch_self_project(c, l, c->list[l - 1], &c->ctr->a[l - 1]);
                }
                if (c->layers[l - 1].proj) rp_launch_messages(c, l);
                rp_timer_end(c, t, RIPPLE_PH_OTHER, (int)l);
            }
            t = rp_timer_begin(c);
            rp_launch_scatter_pull_det(c, l, false);
            rp_timer_end(c, t, RIPPLE_PH_SCATTER, (int)l);
            t = rp_timer_begin(c);
            rp_launch_transform(c, l, c->list[l], &c->ctr->a[l], next_reads_delta(c, l));
            rp_timer_end(c, t, RIPPLE_PH_TRANSFORM, (int)l);
        }
        return;
    }
    for (uint32_t l = 1; l <= c->L; ++l) {
        if (rp_layer_mono(c, l)) {                     // max / min: keep, raise or recompute, then prune (Sec. 3.4.2)
            const bool listed = small_frontier(c, l, n, multi) && c->last_cand[l] <= SPARSE_MAX_ROWS;
            t = rp_timer_begin(c);
            if (listed) rp_launch_candidates_sparse(c, l, layer_self(c, l), RP_MONO_LISTED_LONG);
            else rp_launch_frontier_mark(c, l, false);
            rp_timer_end(c, t, RIPPLE_PH_FRONTIER, (int)l);
            if (!listed) {
                t = rp_timer_begin(c);
                rp_launch_candidates(c, l);
                rp_timer_end(c, t, RIPPLE_PH_COMPACT, (int)l, false);
            }
            if (c->layers[l - 1].selfc) {
                t = rp_timer_begin(c);
                rp_launch_self_project(c, l, c->list[l - 1], &c->ctr->a[l - 1]);
                rp_timer_end(c, t, RIPPLE_PH_OTHER, (int)l);
            }
            t = rp_timer_begin(c);
            rp_launch_scatter_mono(c, l, listed ? &c->ctr->cand[l] : &c->ctr->n_all, listed);
            rp_timer_end(c, t, RIPPLE_PH_SCATTER, (int)l);
            t = rp_timer_begin(c);
            if (listed) rp_launch_list_offsets(c, l, l < c->L);  // the aggregation kernels listed what stays
            else rp_launch_frontier_compact(c, l, layer_self(c, l), l < c->L, false, multi, true);
            rp_timer_end(c, t, RIPPLE_PH_COMPACT, (int)l);
            t = rp_timer_begin(c);
            rp_launch_transform(c, l, c->list[l], &c->ctr->a[l], next_reads_delta(c, l));
            rp_timer_end(c, t, RIPPLE_PH_TRANSFORM, (int)l);
            have_all = false;                          // the candidates went through the live-vertex list's buffer
            continue;
        }
        if (rp_layer_attn(c, l)) {                     // attention: recompute or numerator / denominator deltas (Sec. 3.4.1)
            t = rp_timer_begin(c);
            rp_launch_gat_save(c, l, c->list[l - 1], &c->ctr->a[l - 1]);
            rp_launch_gat_project(c, l, c->list[l - 1], &c->ctr->a[l - 1]);
            rp_launch_gat_scores(c, l, c->list[l - 1], &c->ctr->a[l - 1]);
            rp_timer_end(c, t, RIPPLE_PH_OTHER, (int)l);
            const bool listed = small_frontier(c, l, n, multi);
            if (listed) {
                t = rp_timer_begin(c);
                rp_launch_frontier_sparse(c, l, true, l < c->L, RP_MONO_LISTED_LONG);
                rp_timer_end(c, t, RIPPLE_PH_FRONTIER, (int)l);
            } else {
                t = rp_timer_begin(c);
                rp_launch_frontier_mark(c, l, false);
                rp_timer_end(c, t, RIPPLE_PH_FRONTIER, (int)l);
                t = rp_timer_begin(c);
                rp_launch_frontier_compact(c, l, true, l < c->L, false, multi);
                rp_timer_end(c, t, RIPPLE_PH_COMPACT, (int)l);
            }
            t = rp_timer_begin(c);
            rp_launch_gat_scatter(c, l, false, listed);
            rp_timer_end(c, t, RIPPLE_PH_SCATTER, (int)l);
            t = rp_timer_begin(c);
            rp_launch_transform(c, l, c->list[l], &c->ctr->a[l], next_reads_delta(c, l));
            rp_timer_end(c, t, RIPPLE_PH_TRANSFORM, (int)l);
            have_all = false;                          // the long-row queue went through the live-vertex list's buffer
            continue;
        }
        // hop 1 always pushes: hop-0 rows are in operation order, not ranked by vertex id. Where the
        // previous batch pushed with a wide margin the pull kernel is not even enqueued (pushing is
        // always correct; the prediction only saves a launch). The same goes for the discovering
        // mode: its kernels are enqueued only where the previous batch came near its threshold.
        // Weighted-sum layers gather along in-edges at every hop (the weights are stored with the in-rows only).
        const bool wsum = c->layers[l - 1].agg == RIPPLE_AGG_WSUM;
        const bool may_pull = wsum || (l >= 2 && c->opt_scatter != 1 && !(c->opt_scatter == 0 && c->push_margin[l]));
        const bool may_disc = l >= 2 && may_pull && (c->opt_scatter == 3 || ((c->opt_scatter == 0 || wsum) && c->disc_near[l]));
        // a frontier that was small last time (and a batch of about the same size) is listed as it is marked
        const bool sparse = !may_disc && small_frontier(c, l, n, multi);
        t = rp_timer_begin(c);
        if (may_disc && !have_all) {
            rp_launch_alive_list(c);
            have_all = true;
        }
        // A hop that the last batch pulled (or took from the list already) through in-rows holding enough entries for the
        // sort to pay (rp_sorted_pays) is taken from the sorted list of its messages (k_scatter_sorted): the out-edge
        // walk writes the list, and as many entries are sorted as the last batch had messages, and a quarter more. The
        // kernels make sure on the device that the list is only used if this batch's messages fit and the sort
        // still pays; else the hop is pulled.
        uint32_t pair_cap = 0;
        if (may_pull && !wsum && !sparse && c->pair_cap && c->opt_sorted && !(c->layers[l - 1].proj && c->layers[l - 1].packed)) {
            if (c->opt_sorted == 2) pair_cap = c->pair_cap;
            else if (c->hints_valid && c->last_m[l] && rp_sorted_pays(c->last_m[l], c->last_isum[l]) &&
                     (c->last_hop_mode[l] == 1u + RP_HOP_PULL || c->last_hop_mode[l] == 1u + RP_HOP_SORTED)) {
                const uint64_t want = ((uint64_t)c->last_m[l] + c->last_m[l] / 4 + 4096) & ~4095ull;
                if (want <= c->pair_cap) pair_cap = (uint32_t)want;
            }
        }
        if (sparse) rp_launch_frontier_sparse(c, l, layer_self(c, l), l < c->L);
        else rp_launch_frontier_mark(c, l, may_disc, pair_cap);
        rp_timer_end(c, t, RIPPLE_PH_FRONTIER, (int)l);
        const bool both = rp_has_project_both(c, l);
        if (c->layers[l - 1].proj) {                   // what travels is already multiplied by W_neigh
            t = rp_timer_begin(c);
            if (both) rp_launch_project_both(c, l, c->list[l - 1], &c->ctr->a[l - 1], false);   // and the self terms in the same pass
            else rp_launch_project(c, l, c->list[l - 1], &c->ctr->a[l - 1], false);
            rp_launch_messages(c, l);
            rp_timer_end(c, t, RIPPLE_PH_OTHER, (int)l);
        }
        if (c->layers[l - 1].selfc && !both) {         // H^{l-1} changed exactly on A_{l-1}
            t = rp_timer_begin(c);
            rp_launch_self_project(c, l, c->list[l - 1], &c->ctr->a[l - 1]);
            rp_timer_end(c, t, RIPPLE_PH_OTHER, (int)l, !c->layers[l - 1].proj);
        }
        if (may_disc) {                                // scatters and marks A_l in one scan of all in-rows
            t = rp_timer_begin(c);
            rp_launch_scatter_pull(c, l, true, true);
            rp_timer_end(c, t, RIPPLE_PH_SCATTER, (int)l, false);
        }
        if (!sparse) {
            t = rp_timer_begin(c);
            rp_launch_frontier_compact(c, l, layer_self(c, l), l < c->L, true, multi);
            rp_timer_end(c, t, RIPPLE_PH_COMPACT, (int)l);
        }
        t = rp_timer_begin(c);
        if (!wsum && (c->opt_scatter < 2 || !may_pull)) rp_launch_scatter_push(c, l, may_pull, may_disc);
        if (pair_cap && !rp_launch_scatter_sorted(c, l, may_disc, pair_cap)) pair_cap = 0;
        if (may_pull) rp_launch_scatter_pull(c, l, false, may_disc, pair_cap);
        rp_timer_end(c, t, RIPPLE_PH_SCATTER, (int)l);
        t = rp_timer_begin(c);
        rp_launch_transform(c, l, c->list[l], &c->ctr->a[l], next_reads_delta(c, l));
        rp_timer_end(c, t, RIPPLE_PH_TRANSFORM, (int)l);
    }
}

// Stage, enqueue and wait for one piece; on a full adjacency pool or a full scratch buffer the piece (which
// aborts on the device before it changes anything) is retried after compaction / growth. On return with
// RIPPLE_OK the pinned mirror of the counters describes the piece.
static ripple_status run_piece(ripple_ctx *c, const SubBatch &sb, bool multi, uint32_t *compactions) {
    hipStream_t s = c->stream;
    const uint32_t n = sb.end - sb.begin;
    for (int attempt = 0;; ++attempt) {
        RP_HIP(c, hipMemcpyAsync(c->ops_d, c->ops_pin + sb.begin, (size_t)n * sizeof(ripple_update),
                                 hipMemcpyHostToDevice, s));
        enqueue_piece(c, sb, multi);
        RP_HIP(c, hipMemcpyAsync(c->ctr_host, c->ctr, sizeof(DevCtr), hipMemcpyDeviceToHost, s));
        RP_HIP(c, hipStreamSynchronize(s));
        const DevCtr &h = *c->ctr_host;
        if (!h.abort_flag) return RIPPLE_OK;
        if (h.abort_flag & 8u) {
            c->err = "graph store consistency error " + std::to_string(h.error);
            return RIPPLE_EDEVICE;
        }
        if (h.abort_flag & 2u) return fail(c, RIPPLE_ECAPACITY, "edge capacity exceeded");
        if (attempt >= 2) return fail(c, RIPPLE_ECAPACITY, "adjacency pool exhausted even after compaction");
        if (h.abort_flag & 4u) {
            uint32_t want = h.need_exp + h.need_exp / 2 + 1024;
            // the caller's payload pointer may sit in payload_d: only the operation-side buffers grow here
            RP_TRY(ensure_batch_buffers(c, c->ops_cap, 0, want));
        }
        if (h.abort_flag & 1u) {
            ++*compactions;
            RP_TRY(rp_compact(c));
        }
    }
}

extern "C" ripple_status ripple_apply_updates(ripple_ctx *c, const ripple_update *ops, uint32_t n_ops,
                                              const float *feat_payload, uint32_t n_feat_rows,
                                              ripple_batch_result *res) {
    if (!c) return RIPPLE_EINVAL;
    if (c->state != 3) return fail(c, RIPPLE_ESTATE, "apply_updates needs full_infer first");
    if ((n_ops && !ops) || (n_feat_rows && !feat_payload)) return fail(c, RIPPLE_EINVAL, "null batch pointer");
    if (res) memset(res, 0, sizeof(*res));
    static thread_local TouchTable tt;
    static thread_local std::vector<SubBatch> pieces;
    hipStream_t s = c->stream;
    int t_total = rp_timer_begin(c);

    RP_TRY(ensure_batch_buffers(c, n_ops, n_feat_rows, 0));
    // operations are needed on the host (validation, conflict analysis)
    const ripple_update *hops = ops;
    if (n_ops && is_device_ptr(ops)) {
        RP_HIP(c, hipMemcpyAsync(c->ops_pin, ops, (size_t)n_ops * sizeof(ripple_update), hipMemcpyDeviceToHost, s));
        RP_HIP(c, hipStreamSynchronize(s));
        hops = c->ops_pin;
    }
    if (!ops_in_range(hops, n_ops, c->n_cap, n_feat_rows))
        return fail(c, RIPPLE_EINVAL, "operation with unknown kind, vertex id or payload row out of range");
    if (n_ops == 0) {                              // nothing to do: the affected sets become empty
        rp_launch_batch_reset(c);
        RP_HIP(c, hipMemcpyAsync(c->ctr_host, c->ctr, sizeof(DevCtr), hipMemcpyDeviceToHost, s));
        RP_HIP(c, hipStreamSynchronize(s));
        for (uint32_t l = 0; l <= c->L; ++l) c->last_a[l] = 0;
        c->last_from_rep = false;
        if (res) {
            res->n_sub_batches = 0;
            res->n_alive = c->ctr_host->n_alive;
            res->n_edges = c->ctr_host->n_edges;
        }
        return RIPPLE_OK;
    }
    split_batch(hops, n_ops, tt, pieces);
    const bool multi = pieces.size() > 1;
    if (hops != c->ops_pin) memcpy(c->ops_pin, hops, (size_t)n_ops * sizeof(ripple_update));

    if (multi)
        RP_HIP(c, hipMemsetAsync(c->rep[0], 0, (size_t)c->n_words * (c->L + 1) * 4, s));
    // payload: used in place when it already lives on the device
    float *payload_saved = c->payload_d;
    if (n_feat_rows) {
        size_t bytes = (size_t)n_feat_rows * c->d[0] * 4;
        if (is_device_ptr(feat_payload)) {
            c->payload_d = const_cast<float *>(feat_payload);
        } else {
            memcpy(c->payload_pin, feat_payload, bytes);
            RP_HIP(c, hipMemcpyAsync(c->payload_d, c->payload_pin, bytes, hipMemcpyHostToDevice, s));
        }
    }

    ripple_status rc = RIPPLE_OK;
    uint32_t applied = 0, rejected = 0, n_struct = 0, compactions = 0, ops_done = 0, range_rows = 0;
    uint64_t msgs[RIPPLE_MAX_LAYERS + 1] = {0}, tchd[RIPPLE_MAX_LAYERS + 1] = {0};
    uint32_t mono[3][RIPPLE_MAX_LAYERS + 1] = {{0}};
    uint32_t hop_mode[RIPPLE_MAX_LAYERS + 1] = {0};
    for (size_t p = 0; p < pieces.size() && rc == RIPPLE_OK; ++p) {
        const SubBatch &sb = pieces[p];
        const uint32_t n = sb.end - sb.begin;
        rc = run_piece(c, sb, multi, &compactions);
        if (rc != RIPPLE_OK) break;
        ops_done = sb.end;
        const DevCtr &h = *c->ctr_host;
        applied += h.n_applied;
        rejected += h.n_rejected;
        n_struct += h.n_struct;
        range_rows += h.range_rows;
        for (uint32_t l = 1; l <= c->L; ++l) {
            msgs[l] += h.m[l];
            tchd[l] += h.touched[l];
            c->last_m[l] = h.m[l];
            c->last_isum[l] = h.isum[l];
            c->last_hop_mode[l] = h.hop_mode[l];
            hop_mode[l] = h.hop_mode[l];
            for (int k = 0; k < 3; ++k) mono[k][l] += h.mono[k][l];
            c->last_cand[l] = h.mono[0][l] + h.mono[1][l] + h.mono[2][l];
            // pull wins when m * row_bytes * ratio >= 8 * in-edges; remember if push won by a factor of 16
            const unsigned long long lhs = (unsigned long long)h.m[l] * c->xw[l] * 4ull * (unsigned)c->opt_pull_ratio * 16ull;
            c->push_margin[l] = lhs < 8ull * h.isum[l];
            c->disc_near[l] = (unsigned long long)h.m[l] * 64ull >= h.n_edges;     // threshold: m * 8 >= edges
        }
        if (!multi)
            for (uint32_t l = 0; l <= c->L; ++l) c->last_a[l] = h.a[l];
        c->last_n_ops = multi ? 0u : n;
        c->hints_valid = !multi;
    }
    c->payload_d = payload_saved;                  // never leave the caller's buffer in the context
    if (rc != RIPPLE_OK) {
        // Pieces before the failing one stay applied and fully propagated (the state is that of the batch's
        // first ops_done operations); the failing piece changed nothing. Say how far the batch got.
        (void)hipStreamSynchronize(s);
        c->timer->recs.clear();
        c->timer->used = 0;
        c->hints_valid = false;
        if (res) {
            res->n_ops = n_ops;
            res->n_ops_done = ops_done;
            res->n_applied = applied;
            res->n_rejected = rejected;
            res->n_sub_batches = (uint32_t)pieces.size();
            res->n_compactions = compactions;
            res->n_structural = n_struct;
            if (ops_done) {                        // counters of the last piece that went through
                res->n_alive = c->ctr_host->n_alive;
                res->n_edges = c->ctr_host->n_edges;
            }
        }
        if (multi && ops_done) {                   // the sets reported are those of the applied pieces
            for (uint32_t l = 0; l <= c->L; ++l) rp_launch_bitmap_to_list(c, c->rep[l], c->all_list, &c->ctr->a[l]);
            if (hipMemcpyAsync(c->ctr_host, c->ctr, sizeof(DevCtr), hipMemcpyDeviceToHost, s) == hipSuccess &&
                hipStreamSynchronize(s) == hipSuccess)
                for (uint32_t l = 0; l <= c->L; ++l) {
                    c->last_a[l] = c->ctr_host->a[l];
                    if (res) res->affected[l] = c->last_a[l];
                }
            c->last_from_rep = true;
        }
        return rc;
    }
    RP_HIP(c, hipGetLastError());
    if (multi) {                                   // sizes of the united sets
        for (uint32_t l = 0; l <= c->L; ++l) rp_launch_bitmap_to_list(c, c->rep[l], c->all_list, &c->ctr->a[l]);
        RP_HIP(c, hipMemcpyAsync(c->ctr_host, c->ctr, sizeof(DevCtr), hipMemcpyDeviceToHost, s));
        RP_HIP(c, hipStreamSynchronize(s));
        for (uint32_t l = 0; l <= c->L; ++l) c->last_a[l] = c->ctr_host->a[l];
    }
    c->last_from_rep = multi;
    rp_timer_end(c, t_total, RIPPLE_PH_TOTAL, 0);
    if (c->opt_timing) {
        RP_HIP(c, hipStreamSynchronize(s));
        timer_collect(c);
        c->stats.batches += 1;
        for (uint32_t l = 0; l <= c->L; ++l) {
            c->stats.rows[l] += c->last_a[l];
            c->stats.msgs[l] += msgs[l];
            c->stats.touched[l] += tchd[l];
        }
    }
    if (res) {
        res->n_ops = n_ops;
        res->n_ops_done = n_ops;
        res->n_applied = applied;
        res->n_rejected = rejected;
        res->n_sub_batches = (uint32_t)pieces.size();
        res->n_compactions = compactions;
        res->n_alive = c->ctr_host->n_alive;
        res->n_edges = c->ctr_host->n_edges;
        res->n_structural = n_struct;
        for (uint32_t l = 0; l <= c->L; ++l) {
            res->affected[l] = c->last_a[l];
            res->messages[l] = msgs[l];
            res->mono_unchanged[l] = mono[0][l];
            res->mono_incremental[l] = mono[1][l];
            res->mono_recomputed[l] = mono[2][l];
            res->hop_mode[l] = hop_mode[l];
        }
    }
    if (range_rows) return range_error(c, range_rows);      // the batch is applied; res describes it
    return RIPPLE_OK;
}

// ---------------------------------------------------------------------------------
// read-back
// ---------------------------------------------------------------------------------
static ripple_status gather_rows(ripple_ctx *c, const void *M, int store, uint32_t d, const uint32_t *ids,
                                 uint32_t n_ids, float *out) {
    if (n_ids == 0) return RIPPLE_OK;
    if (!out) return fail(c, RIPPLE_EINVAL, "null output pointer");
    hipStream_t s = c->stream;
    const uint32_t *ids_d = nullptr;
    if (ids) {
        if (is_device_ptr(ids)) {
            ids_d = ids;
        } else {
            for (uint32_t i = 0; i < n_ids; ++i)
                if (ids[i] >= c->n_cap) return fail(c, RIPPLE_EINVAL, "vertex id out of range");
            if (n_ids > c->gather_ids_cap) {
                if (c->gather_ids) hipFree(c->gather_ids);
                c->gather_ids = nullptr;
                c->gather_ids_cap = 0;
                RP_TRY(dev_alloc(c, &c->gather_ids, (size_t)n_ids, false));
                c->gather_ids_cap = n_ids;
            }
            RP_HIP(c, hipMemcpyAsync(c->gather_ids, ids, (size_t)n_ids * 4, hipMemcpyHostToDevice, s));
            ids_d = c->gather_ids;
        }
    } else if (n_ids > c->n_cap) {
        return fail(c, RIPPLE_EINVAL, "more rows requested than vertex_capacity");
    }
    if (!ids && !store) {                           // contiguous float32 rows: plain copy
        RP_HIP(c, hipMemcpyAsync(out, M, (size_t)n_ids * d * 4, hipMemcpyDefault, s));
        RP_HIP(c, hipStreamSynchronize(s));
        return RIPPLE_OK;
    }
    const size_t chunk_rows = std::max<size_t>(1, ((size_t)64 << 20) / d);
    const size_t need = std::min<size_t>(chunk_rows, n_ids) * d;
    if (need > c->gather_cap) {
        if (c->gather_d) hipFree(c->gather_d);
        c->gather_d = nullptr;
        c->gather_cap = 0;
        RP_TRY(dev_alloc(c, &c->gather_d, need, false));
        c->gather_cap = need;
    }
    for (size_t r0 = 0; r0 < n_ids; r0 += chunk_rows) {
        size_t rows = std::min<size_t>(chunk_rows, n_ids - r0);
        uint32_t gb = std::min<uint32_t>(rp_div_up(rows * d, 256), c->n_cu * 16);
        hipLaunchKernelGGL(k_gather_rows, dim3(gb), dim3(256), 0, s, M, store, d, ids_d ? ids_d + r0 : nullptr,
                           (uint32_t)r0, rows, c->n_cap, c->gather_d);
        RP_HIP(c, hipMemcpyAsync(out + r0 * d, c->gather_d, rows * d * 4, hipMemcpyDefault, s));
        RP_HIP(c, hipStreamSynchronize(s));
    }
    return RIPPLE_OK;
}

extern "C" ripple_status ripple_get_embeddings(ripple_ctx *c, uint32_t layer, const uint32_t *ids, uint32_t n_ids,
                                               float *out) {
    if (!c) return RIPPLE_EINVAL;
    if (c->state < 1 || (layer > 0 && c->state < 3)) return fail(c, RIPPLE_ESTATE, "embeddings not computed yet");
    if (layer > c->L) return fail(c, RIPPLE_EINVAL, "layer out of range");
    return gather_rows(c, c->H[layer], c->store, c->d[layer], ids, n_ids, out);
}

extern "C" ripple_status ripple_get_aggregates(ripple_ctx *c, uint32_t layer, const uint32_t *ids, uint32_t n_ids,
                                               float *out) {
    if (!c) return RIPPLE_EINVAL;
    if (c->state < 3) return fail(c, RIPPLE_ESTATE, "aggregates not computed yet");
    if (layer == 0 || layer > c->L) return fail(c, RIPPLE_EINVAL, "layer out of range");
    return gather_rows(c, c->X[layer], 0, c->xw[layer], ids, n_ids, out);
}

extern "C" ripple_status ripple_get_layer_info(ripple_ctx *c, uint32_t layer, uint32_t *aggregate_width,
                                                int *projected) {
    if (!c) return RIPPLE_EINVAL;
    if (c->state < 2) return fail(c, RIPPLE_ESTATE, "no model loaded");
    if (layer == 0 || layer > c->L) return fail(c, RIPPLE_EINVAL, "layer out of range");
    if (aggregate_width) *aggregate_width = c->xw[layer];
    if (projected)
        *projected = (int)(c->layers[layer - 1].proj | (c->layers[layer - 1].selfc << 1) |
                           ((c->layers[layer - 1].proj && c->layers[layer - 1].packed) ? 4u : 0u));
    return RIPPLE_OK;
}

extern "C" ripple_status ripple_get_affected(ripple_ctx *c, uint32_t layer, uint32_t *ids_out, uint32_t cap,
                                             uint32_t *n_out) {
    if (!c) return RIPPLE_EINVAL;
    if (c->state != 3) return fail(c, RIPPLE_ESTATE, "no batch has been applied");
    if (layer > c->L || !n_out || (cap && !ids_out)) return fail(c, RIPPLE_EINVAL, "bad argument");
    hipStream_t s = c->stream;
    uint32_t *bitmap = c->last_from_rep ? c->rep[layer] : c->bm[layer];
    uint32_t *cnt_d = &c->ctr->n_all;              // free between batches
    rp_launch_bitmap_to_list(c, bitmap, c->all_list, cnt_d);
    uint32_t n = 0;
    RP_HIP(c, hipMemcpyAsync(&n, cnt_d, 4, hipMemcpyDeviceToHost, s));
    RP_HIP(c, hipStreamSynchronize(s));
    *n_out = n;
    uint32_t m = std::min(n, cap);
    if (m) RP_HIP(c, hipMemcpy(ids_out, c->all_list, (size_t)m * 4, hipMemcpyDeviceToHost));
    return RIPPLE_OK;
}

extern "C" ripple_status ripple_get_affected_static(ripple_ctx *c, uint32_t layer, uint32_t *ids_out, uint32_t cap,
                                                    uint32_t *n_out) {
    if (!c) return RIPPLE_EINVAL;
    if (c->state != 3) return fail(c, RIPPLE_ESTATE, "no batch has been applied");
    if (layer > c->L || !n_out || (cap && !ids_out)) return fail(c, RIPPLE_EINVAL, "bad argument");
    if (!is_device_ptr(n_out) || (cap && !is_device_ptr(ids_out)))
        return fail(c, RIPPLE_EINVAL, "ids_out and n_out must be device memory");
    return rp_launch_affected_static(c, c->last_from_rep ? c->rep[layer] : c->bm[layer], ids_out, cap, n_out);
}

extern "C" ripple_status ripple_export_edges(ripple_ctx *c, int direction, uint32_t *src_out, uint32_t *dst_out,
                                             uint64_t cap, uint64_t *n_out) {
    if (!c) return RIPPLE_EINVAL;
    if (c->state < 1) return fail(c, RIPPLE_ESTATE, "no graph");
    if (!n_out || (direction != 0 && direction != 1)) return fail(c, RIPPLE_EINVAL, "bad argument");
    hipStream_t s = c->stream;
    const uint2 *meta = direction ? c->in_meta : c->out_meta;
    const uint32_t *pool = direction ? c->in_pool : c->out_pool;
    uint32_t *len = nullptr, *off = nullptr, *total_d = nullptr, *sd = nullptr, *dd = nullptr;
    RP_TRY(dev_alloc(c, &len, (size_t)c->n_cap, false));
    RP_TRY(dev_alloc(c, &off, (size_t)c->n_cap, false));
    RP_TRY(dev_alloc(c, &total_d, 16, true));
    uint32_t vb = rp_div_up(c->n_cap, 256);
    hipLaunchKernelGGL(k_meta_len2, dim3(vb), dim3(256), 0, s, meta, c->n_cap, len);
    rp_exclusive_scan(s, len, off, c->n_cap, c->part_cnt, total_d);
    uint32_t total = 0;
    RP_HIP(c, hipMemcpyAsync(&total, total_d, 4, hipMemcpyDeviceToHost, s));
    RP_HIP(c, hipStreamSynchronize(s));
    *n_out = total;
    ripple_status rc = RIPPLE_OK;
    if (total && total <= cap) {
        if (!src_out || !dst_out) rc = fail(c, RIPPLE_EINVAL, "null output pointer");
        else {
            rc = dev_alloc(c, &sd, (size_t)total, false);
            if (rc == RIPPLE_OK) rc = dev_alloc(c, &dd, (size_t)total, false);
            if (rc == RIPPLE_OK) {
                hipLaunchKernelGGL(k_export_rows, dim3(c->n_cu * 8), dim3(256), 0, s, meta, pool, off, c->n_cap,
                                   direction, sd, dd);
                hipMemcpyAsync(src_out, sd, (size_t)total * 4, hipMemcpyDeviceToHost, s);
                hipMemcpyAsync(dst_out, dd, (size_t)total * 4, hipMemcpyDeviceToHost, s);
                if (hipStreamSynchronize(s) != hipSuccess) rc = fail(c, RIPPLE_EDEVICE, "export failed");
            }
        }
    }
    hipFree(len);
    hipFree(off);
    hipFree(total_d);
    if (sd) hipFree(sd);
    if (dd) hipFree(dd);
    return rc;
}

extern "C" ripple_status ripple_get_degrees(ripple_ctx *c, int direction, uint32_t *deg_out, uint8_t *alive_out) {
    if (!c) return RIPPLE_EINVAL;
    if (c->state < 1) return fail(c, RIPPLE_ESTATE, "no graph");
    if (direction != 0 && direction != 1) return fail(c, RIPPLE_EINVAL, "bad direction");
    hipStream_t s = c->stream;
    if (deg_out) {
        uint32_t *len = nullptr;
        RP_TRY(dev_alloc(c, &len, (size_t)c->n_cap, false));
        hipLaunchKernelGGL(k_meta_len2, dim3(rp_div_up(c->n_cap, 256)), dim3(256), 0, s,
                           direction ? c->in_meta : c->out_meta, c->n_cap, len);
        hipMemcpyAsync(deg_out, len, (size_t)c->n_cap * 4, hipMemcpyDeviceToHost, s);
        hipError_t e = hipStreamSynchronize(s);
        hipFree(len);
        if (e != hipSuccess) return fail(c, RIPPLE_EDEVICE, "degree read-back failed");
    }
    if (alive_out) {
        std::vector<uint32_t> bm(c->n_words);
        RP_HIP(c, hipMemcpy(bm.data(), c->alive, (size_t)c->n_words * 4, hipMemcpyDeviceToHost));
        for (uint32_t v = 0; v < c->n_cap; ++v) alive_out[v] = (bm[v >> 5] >> (v & 31)) & 1u;
    }
    return RIPPLE_OK;
}

extern "C" ripple_status ripple_compact(ripple_ctx *c) {
    if (!c) return RIPPLE_EINVAL;
    if (c->state < 1) return fail(c, RIPPLE_ESTATE, "no graph");
    return rp_compact(c);
}

extern "C" ripple_status ripple_set_option(ripple_ctx *c, int option, int64_t value) {
    if (!c) return RIPPLE_EINVAL;
    switch (option) {
    case RIPPLE_OPT_TIMING: c->opt_timing = value ? 1 : 0; return RIPPLE_OK;
    case RIPPLE_OPT_SCATTER_MODE:
        if (value < 0 || value > 3) return fail(c, RIPPLE_EINVAL, "scatter mode must be 0, 1, 2 or 3");
        c->opt_scatter = (int)value;
        return RIPPLE_OK;
    case RIPPLE_OPT_DETERMINISTIC:
        if (c->state != 1) return fail(c, RIPPLE_ESTATE, "the deterministic mode is chosen before load_model");
        c->opt_deterministic = value ? 1 : 0;
        return RIPPLE_OK;
    case RIPPLE_OPT_SELF_CACHE:
        if (c->state != 1) return fail(c, RIPPLE_ESTATE, "the self-projection cache is chosen before load_model");
        c->opt_selfcache = value ? 1 : 0;
        return RIPPLE_OK;
    case RIPPLE_OPT_SPLIT_MFMA:
        if (c->state != 1) return fail(c, RIPPLE_ESTATE, "RIPPLE_OPT_SPLIT_MFMA must be set before load_model");
        c->opt_split = value ? 1 : 0;
        return RIPPLE_OK;
    case RIPPLE_OPT_BF16_MFMA:
        c->opt_bf16_mfma = value ? 1 : 0;
        return RIPPLE_OK;
    case RIPPLE_OPT_SPARSE_FRONTIER:
        c->opt_sparse = value ? 1 : 0;
        return RIPPLE_OK;
    case RIPPLE_OPT_ROW_SEGMENTS:
        if (value < 0) return fail(c, RIPPLE_EINVAL, "the number of row segments cannot be negative");
        c->seg_limit = (uint32_t)std::min<long long>(value, 0xffffffffll);
        return RIPPLE_OK;
    case RIPPLE_OPT_PROJECT_FIRST:
        if (c->state != 1) return fail(c, RIPPLE_ESTATE, "project-first must be chosen before load_model");
        c->opt_project = value ? 1 : 0;
        return RIPPLE_OK;
    case RIPPLE_OPT_PACKED_MESSAGES:
        if (c->state != 1) return fail(c, RIPPLE_ESTATE, "packed messages must be chosen before load_model");
        c->opt_pack = value ? 1 : 0;
        return RIPPLE_OK;
    case RIPPLE_OPT_STREAM_TRANSFORM:
        if (value < 0 || value > 2) return fail(c, RIPPLE_EINVAL, "RIPPLE_OPT_STREAM_TRANSFORM must be 0, 1 or 2");
        c->opt_stream = (int)value;
        return RIPPLE_OK;
    case RIPPLE_OPT_SORTED_MESSAGES:
        if (value < 0 || value > 2) return fail(c, RIPPLE_EINVAL, "RIPPLE_OPT_SORTED_MESSAGES must be 0, 1 or 2");
        c->opt_sorted = (int)value;
        return RIPPLE_OK;
    case RIPPLE_OPT_PULL_RATIO:
        if (value < 1 || value > 1024) return fail(c, RIPPLE_EINVAL, "pull ratio must be in 1..1024");
        c->opt_pull_ratio = (int)value;
        return RIPPLE_OK;
    default: return fail(c, RIPPLE_EINVAL, "unknown option");
    }
}

extern "C" ripple_status ripple_get_stats(ripple_ctx *c, ripple_stats *out, int reset) {
    if (!c || !out) return RIPPLE_EINVAL;
    *out = c->stats;
    if (reset) memset(&c->stats, 0, sizeof(c->stats));
    return RIPPLE_OK;
}

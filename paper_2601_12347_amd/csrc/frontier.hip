// Frontier construction (the per-hop slice of the propagation tree, Sec. 3.3):
//   A_l = (S  u  Out(A_{l-1})  u  [A_{l-1} if the layer reads the vertex's own
//          embedding]  u  V_added)  n  Alive
// as a bitmap and as an ascending list, plus the exclusive scan of out-degrees
// over that list, which lets the next hop's edge walk be split evenly over
// wavefronts regardless of degree skew.
#include "common.h"
#include "kernels.h"
#include <cstring>

#define MARK_CHUNK 256

// mark the out-neighbours of every vertex of A_{l-1}. Every wavefront walks a contiguous run of
// 256-edge chunks of the flattened out-edge space, so only its first chunk needs a search over the
// whole list; the 64 rows after the chunk's first one are described in registers (one per lane:
// where the row's edges start in the pool, and the first edge of the next row) and an edge finds its
// row with shuffles. Nothing to do on a discovering hop (the in-row scan finds A_l).
// Small frontiers (SparseArgs given): a marked vertex is entered into the hop's bitmap at once and the
// first wavefront to do so appends it to the hop's list, so no scan of the whole bitmap is needed
// afterwards; the list is then in no particular order.
struct SparseArgs {
    uint32_t *bm;                  // the hop's bitmap (zero on entry)
    const uint32_t *alive;
    uint32_t *list, *count;        // the hop's list and its length (zero on entry)
    uint32_t *touched;             // += vertices first entered by an out-edge (statistics)
    // roots merged in by the same kernel: sinks of changed edges, created vertices, the previous hop's set (self term)
    const uint32_t *st_dst, *n_struct;
    uint32_t struct_cap;
    const uint32_t *list0, *count0, *bm_vadd;
    int self_term;
    // optional second list: vertices with more than long_min in-neighbours are appended there instead
    const uint2 *in_meta;
    uint32_t long_min;
    uint32_t *long_list, *long_count;
    int long_dup;                  // those vertices are appended to the hop's list as well
};

// T vertices per lane (0xFFFFFFFF: none): the T marks go out together and one reservation covers all of
// them (two round trips instead of 2 T). To be called by all 64 lanes together.
template <int T>
__device__ __forceinline__ void sparse_enter_many(const SparseArgs &s, const uint32_t *v, bool from_edge) {
    bool live[T], fresh[T], lng[T];
#pragma unroll
    for (int t = 0; t < T; ++t) live[t] = v[t] != 0xFFFFFFFFu && rp_bit(s.alive, v[t]);
#pragma unroll
    for (int t = 0; t < T; ++t) {
        fresh[t] = false;
        if (live[t]) {
            const uint32_t m = 1u << (v[t] & 31);
            fresh[t] = !(atomicOr(&s.bm[v[t] >> 5], m) & m);
        }
    }
#pragma unroll
    for (int t = 0; t < T; ++t) lng[t] = fresh[t] && s.long_list && s.in_meta[v[t]].y > s.long_min;
    unsigned long long mask[T], lmask[T];
    uint32_t total = 0, ltotal = 0;
#pragma unroll
    for (int t = 0; t < T; ++t) {
        mask[t] = __ballot(fresh[t] && (!lng[t] || s.long_dup));
        lmask[t] = __ballot(lng[t]);
        total += (uint32_t)__popcll(mask[t]);
        ltotal += (uint32_t)__popcll(lmask[t]);
    }
    if (!(total + ltotal)) return;
    const int lane = rp_lane();
    uint32_t base = 0, lbase = 0;
    if (lane == 0) {
        if (total) base = atomicAdd(s.count, total);
        if (ltotal) lbase = atomicAdd(s.long_count, ltotal);
        if (from_edge && s.touched) atomicAdd(s.touched, total + ltotal);
    }
    base = __shfl(base, 0);
    lbase = __shfl(lbase, 0);
    const unsigned long long below = (1ull << lane) - 1ull;
#pragma unroll
    for (int t = 0; t < T; ++t) {
        if (fresh[t] && (!lng[t] || s.long_dup)) s.list[base + (uint32_t)__popcll(mask[t] & below)] = v[t];
        if (lng[t]) s.long_list[lbase + (uint32_t)__popcll(lmask[t] & below)] = v[t];
        base += (uint32_t)__popcll(mask[t]);
        lbase += (uint32_t)__popcll(lmask[t]);
    }
}

// one vertex per valid lane; to be called by all 64 lanes together
__device__ __forceinline__ void sparse_enter(const SparseArgs &s, uint32_t v, bool valid, bool from_edge) {
    const uint32_t one[1] = {valid ? v : 0xFFFFFFFFu};
    sparse_enter_many<1>(s, one, from_edge);
}

// EMIT: edge e of the flattened out-edge space is also written down as the pair (destination, source) in pk[e], pv[e]
template <bool SPARSE, bool EMIT = false>
__device__ __forceinline__ void frontier_walk(const uint32_t *list, const uint32_t *count_ptr, const uint32_t *eoff,
                                              const uint2 *out_meta, const uint32_t *out_pool, uint8_t *mk,
                                              const SparseArgs &sp, uint32_t *pk = nullptr, uint32_t *pv = nullptr) {
    const uint32_t count = *count_ptr;
    if (count == 0) return;
    constexpr int T = MARK_CHUNK / 64;
    const int lane = rp_lane();
    const uint32_t M = eoff[count];
    // few out-edges: 64-edge chunks (only the first of a lane's T slots is used) so that more wavefronts share them
    const uint32_t chunk = (SPARSE && M <= 16384u) ? 64u : (uint32_t)MARK_CHUNK;
    const uint32_t n_chunks = (M + chunk - 1) / chunk;
    const uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    const uint32_t per = (n_chunks + nw - 1) / nw;
    const uint32_t c_begin = min(n_chunks, gw * per), c_end = min(n_chunks, c_begin + per);
    if (c_begin >= c_end) return;
    const uint32_t last = count - 1;
    uint32_t i_lo = rp_seg_search_wave(eoff, 0, last, c_begin * chunk);
    uint32_t rbase, bnd, rsrc = 0;                          // lane j: row i_lo + j
    {
        const uint32_t ri = min(last, i_lo + lane);
        rsrc = list[ri];
        rbase = out_meta[rsrc].x - eoff[ri];                // pool position of edge e: rbase + e (mod 2^32)
        bnd = eoff[min(count, i_lo + 1 + lane)];
    }
    for (uint32_t c = c_begin; c < c_end; ++c) {
        const uint32_t e0 = c * chunk, e1 = min(M, e0 + chunk);
        const bool fits = __shfl(bnd, 63) > e1 - 1;         // every row of the chunk is among the 64 held
        uint32_t v[T];
        uint32_t i_nx;
        if (fits) {
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const uint32_t e = e0 + lane + 64 * t;
                const int r = (int)min(63u, rp_count_le(bnd, e));
                const uint32_t base = __shfl(rbase, r);
                v[t] = (e < e1) ? out_pool[base + e] : 0xFFFFFFFFu;
                if (EMIT) {
                    const uint32_t u = __shfl(rsrc, r);
                    if (e < e1) {
                        pk[e] = v[t];
                        pv[e] = u;
                    }
                }
            }
            i_nx = min(last, i_lo + rp_count_le(bnd, e1));
        } else {
            const uint32_t i_hi = rp_seg_forward(eoff, i_lo, last, e1 - 1);
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const uint32_t e = e0 + lane + 64 * t;
                v[t] = 0xFFFFFFFFu;
                if (e < e1) {
                    const uint32_t i = rp_seg_search(eoff, i_lo, i_hi, e);
                    const uint32_t u = list[i];
                    v[t] = out_pool[out_meta[u].x + (e - eoff[i])];
                    if (EMIT) {
                        pk[e] = v[t];
                        pv[e] = u;
                    }
                }
            }
            i_nx = rp_seg_forward(eoff, i_hi, last, e1);
        }
        uint32_t rbase_n, bnd_n, rsrc_n;                    // next chunk's rows, requested before the marks
        {
            const uint32_t ri = min(last, i_nx + lane);
            rsrc_n = list[ri];
            rbase_n = out_meta[rsrc_n].x - eoff[ri];
            bnd_n = eoff[min(count, i_nx + 1 + lane)];
        }
        if (SPARSE) {
            sparse_enter_many<T>(sp, v, true);
        } else {
#pragma unroll
            for (int t = 0; t < T; ++t)
                if (v[t] != 0xFFFFFFFFu) mk[v[t]] = 1;       // plain byte stores: idempotent, no atomics
        }
        i_lo = i_nx;
        rbase = rbase_n;
        bnd = bnd_n;
        rsrc = rsrc_n;
    }
}

// The walk that also lists the hop's messages as (destination, source) pairs for the sorted scatter: pair_cap entries
// will be sorted, so the list is written only if the hop's out-edges fit, and the entries behind them get the key
// that sorts last.
__global__ __launch_bounds__(256) void k_frontier_mark_pairs(const uint32_t *list, const uint32_t *count_ptr,
                                                             const uint32_t *eoff, const uint2 *out_meta,
                                                             const uint32_t *out_pool, uint8_t *mk, const DevCtr *ctr,
                                                             uint32_t l, uint32_t d, int mode, int ratio, int allow_disc,
                                                             uint32_t *pk, uint32_t *pv, uint32_t pair_cap) {
    if (allow_disc && rp_hop_mode(ctr, l, d, mode, ratio, allow_disc) == RP_HOP_DISCOVER) return;
    const uint32_t count = *count_ptr;
    const uint32_t M = count ? eoff[count] : 0u;
    if (M == 0 || M > pair_cap) {
        frontier_walk<false>(list, count_ptr, eoff, out_meta, out_pool, mk, SparseArgs());
        return;
    }
    frontier_walk<false, true>(list, count_ptr, eoff, out_meta, out_pool, mk, SparseArgs(), pk, pv);
    for (uint32_t i = M + blockIdx.x * blockDim.x + threadIdx.x; i < pair_cap; i += gridDim.x * blockDim.x) pk[i] = 0xFFFFFFFFu;
}

__global__ __launch_bounds__(256) void k_frontier_mark(const uint32_t *list, const uint32_t *count_ptr,
                                                       const uint32_t *eoff, const uint2 *out_meta,
                                                       const uint32_t *out_pool, uint8_t *mk, const DevCtr *ctr,
                                                       uint32_t l, uint32_t d, int mode, int ratio, int allow_disc) {
    if (allow_disc && rp_hop_mode(ctr, l, d, mode, ratio, allow_disc) == RP_HOP_DISCOVER) return;
    frontier_walk<false>(list, count_ptr, eoff, out_meta, out_pool, mk, SparseArgs());
}

// the out-edge walk and the roots in one kernel, straight into the hop's bitmap and (unordered) list
__global__ __launch_bounds__(256) void k_frontier_sparse(const uint32_t *list, const uint32_t *count_ptr,
                                                         const uint32_t *eoff, const uint2 *out_meta,
                                                         const uint32_t *out_pool, SparseArgs sp) {
    frontier_walk<true>(list, count_ptr, eoff, out_meta, out_pool, nullptr, sp);
    const int lane = rp_lane();
    const uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    const uint32_t n_s = min(*sp.n_struct, sp.struct_cap), n_0 = *sp.count0, n_p = sp.self_term ? *count_ptr : 0u;
    const uint32_t total = n_s + n_0 + n_p;
    for (uint32_t base = gw * 64; base < total; base += nw * 64) {
        const uint32_t i = base + lane;
        uint32_t v = 0;
        bool valid = i < total;
        if (valid) {
            if (i < n_s) v = sp.st_dst[i];
            else if (i < n_s + n_0) {
                v = sp.list0[i - n_s];
                valid = rp_bit(sp.bm_vadd, v);
            } else v = list[i - n_s - n_0];
        }
        sparse_enter(sp, v, valid, false);
    }
}

struct CompactArgs {
    uint32_t *bm;                  // the layer's bitmap: marks in (a discovering hop sets them here), final set out
    uint8_t *mk;                   // more marks, one byte per vertex (set by the out-edge walk, cleared here), or null
    const uint32_t *bm_prev;       // previous hop's set (layers with a self term) or null
    const uint32_t *bm_sink;       // S or null
    const uint32_t *bm_vadd;       // V_added (read only when bm_sink is set)
    const uint32_t *alive;
    uint32_t n_words;
    const uint2 *out_meta, *in_meta;
    int want_out, want_in;         // emit out-degree / in-degree prefixes over the list
    uint32_t *part_cnt, *part_out, *part_in;
    uint32_t *rep;                 // reporting union or null
    uint32_t *touched_out;         // += vertices that received a message, or null
    uint32_t *list, *eoff, *ioff;  // outputs
    uint32_t *count_out, *msgs_out, *isum_out;
    uint32_t list_cap;             // entries the list has room for (positions beyond are counted, not written)
};

// bitmap word of 32 mark bytes (each 0 or 1); the bytes are cleared again when any was set
__device__ __forceinline__ uint32_t take_marks(uint8_t *mk, uint32_t idx) {
    uint4 *p = (uint4 *)(mk + (size_t)idx * 32);
    const uint4 lo = p[0], hi = p[1];
    const uint32_t d[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    uint32_t w = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) w |= (((d[k] * 0x00204081u) >> 21) & 0xFu) << (4 * k);   // bytes 0/1 -> four bits
    if (w) {
        p[0] = make_uint4(0, 0, 0, 0);
        p[1] = make_uint4(0, 0, 0, 0);
    }
    return w;
}

__device__ __forceinline__ void word_degrees(const CompactArgs &a, uint32_t idx, uint32_t w, uint32_t &dout,
                                             uint32_t &din) {
    dout = din = 0;
    if (!(a.want_out | a.want_in)) return;
    while (w) {
        uint32_t v = idx * 32 + (__ffs(w) - 1);
        w &= w - 1;
        if (a.want_out) dout += a.out_meta[v].y;
        if (a.want_in) din += a.in_meta[v].y;
    }
}

// Degrees of the vertices of one bitmap word, all requested before any is used (the loads are
// unconditional: a vertex that is not in the word reads entry 0 and counts as zero).
struct WordDeg {
    uint32_t o[32], i[32];
    __device__ __forceinline__ void gather(const CompactArgs &a, uint32_t idx, uint32_t w, uint32_t &dout, uint32_t &din) {
        dout = din = 0;
#pragma unroll
        for (int b = 0; b < 32; ++b) {
            const bool on = (w >> b) & 1u;
            const uint32_t v = on ? idx * 32 + b : 0u;
            const uint32_t x = a.out_meta[v].y, y = a.in_meta[v].y;
            o[b] = (on && a.want_out) ? x : 0u;
            i[b] = (on && a.want_in) ? y : 0u;
            dout += o[b];
            din += i[b];
        }
    }
    // list entries and prefixes of the word's vertices, starting at position oc with running sums oo, oi
    __device__ __forceinline__ void emit(const CompactArgs &a, uint32_t idx, uint32_t w, uint32_t &oc, uint32_t &oo,
                                         uint32_t &oi) const {
#pragma unroll
        for (int b = 0; b < 32; ++b) {
            if (!((w >> b) & 1u)) continue;
            if (oc < a.list_cap) {
                a.list[oc] = idx * 32 + b;
                if (a.want_out) a.eoff[oc] = oo;
                if (a.want_in) a.ioff[oc] = oi;
            }
            oo += o[b];
            oi += i[b];
            ++oc;
        }
    }
};

// pass 1: merge the root sets (S, V_added, and the previous hop's set when the layer has a
// self term) into the layer's bitmap, restrict to live vertices, count vertices and
// (optionally) their degrees per block of 256 words
__global__ __launch_bounds__(256) void k_frontier_count(CompactArgs a) {
    __shared__ uint32_t sh[16];
    const int tid = threadIdx.x;
    uint32_t idx = blockIdx.x * 256 + tid;
    uint32_t w = 0, tch = 0;
    if (idx < a.n_words) {
        const uint32_t live = a.alive[idx];
        w = a.bm[idx];
        if (a.mk) w |= take_marks(a.mk, idx);
        w &= live;
        tch = __popc(w);                         // vertices that received at least one message
        if (a.bm_sink) w |= (a.bm_sink[idx] | a.bm_vadd[idx]) & live;
        if (a.bm_prev) w |= a.bm_prev[idx] & live;
        a.bm[idx] = w;
        if (a.rep && w) a.rep[idx] |= w;
    }
    uint32_t cnt = __popc(w), dout, din;
    word_degrees(a, idx, w, dout, din);
    for (int o = 32; o > 0; o >>= 1) {
        cnt += __shfl_down(cnt, o);
        dout += __shfl_down(dout, o);
        din += __shfl_down(din, o);
        tch += __shfl_down(tch, o);
    }
    if ((tid & 63) == 0) {
        sh[tid >> 6] = cnt;
        sh[4 + (tid >> 6)] = dout;
        sh[8 + (tid >> 6)] = din;
        sh[12 + (tid >> 6)] = tch;
    }
    __syncthreads();
    if (tid == 0) {
        a.part_cnt[blockIdx.x] = sh[0] + sh[1] + sh[2] + sh[3];
        a.part_out[blockIdx.x] = sh[4] + sh[5] + sh[6] + sh[7];
        a.part_in[blockIdx.x] = sh[8] + sh[9] + sh[10] + sh[11];
        const uint32_t t = sh[12] + sh[13] + sh[14] + sh[15];
        if (a.touched_out && t) atomicAdd(a.touched_out, t);
    }
}

// pass 2: write the ascending list, the degree prefixes and the per-word ranks
__global__ __launch_bounds__(256) void k_frontier_emit(CompactArgs a) {
    __shared__ uint32_t sh[12];
    __shared__ uint32_t wc[4], wo[4], wi[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t pc = 0, po = 0, pi = 0;
    for (uint32_t b = tid; b < blockIdx.x; b += 256) {
        pc += a.part_cnt[b];
        po += a.part_out[b];
        pi += a.part_in[b];
    }
    for (int o = 32; o > 0; o >>= 1) {
        pc += __shfl_down(pc, o);
        po += __shfl_down(po, o);
        pi += __shfl_down(pi, o);
    }
    if (lane == 0) {
        sh[wave] = pc;
        sh[4 + wave] = po;
        sh[8 + wave] = pi;
    }
    __syncthreads();
    pc = sh[0] + sh[1] + sh[2] + sh[3];
    po = sh[4] + sh[5] + sh[6] + sh[7];
    pi = sh[8] + sh[9] + sh[10] + sh[11];
    uint32_t idx = blockIdx.x * 256 + tid;
    uint32_t w = (idx < a.n_words) ? a.bm[idx] : 0u;
    uint32_t cnt = __popc(w), dout = 0, din = 0;
    WordDeg wd;
    if (w) wd.gather(a, idx, w, dout, din);
    uint32_t ic = cnt, io = dout, ii = din;
    for (int o = 1; o < 64; o <<= 1) {
        uint32_t tc = __shfl_up(ic, o), to = __shfl_up(io, o), ti = __shfl_up(ii, o);
        if (lane >= o) {
            ic += tc;
            io += to;
            ii += ti;
        }
    }
    if (lane == 63) {
        wc[wave] = ic;
        wo[wave] = io;
        wi[wave] = ii;
    }
    __syncthreads();
    uint32_t oc = pc + ic - cnt, oo = po + io - dout, oi = pi + ii - din;
    for (int k = 0; k < wave; ++k) {
        oc += wc[k];
        oo += wo[k];
        oi += wi[k];
    }
    if (w) wd.emit(a, idx, w, oc, oo, oi);
    if (blockIdx.x == gridDim.x - 1 && tid == 255) {     // the running values now hold the grand totals
        *a.count_out = oc;
        if (a.want_out) {
            a.eoff[oc] = oo;
            if (a.msgs_out) *a.msgs_out = oo;
        }
        if (a.want_in) {
            a.ioff[oc] = oi;
            if (a.isum_out) *a.isum_out = oi;
        }
    }
}

// Both passes in one workgroup, for bitmaps of at most SMALL_WORDS words (small graphs: saves
// two launches per hop, which is most of the hop's time when batches are small).
#define SMALL_WPT 8
#define SMALL_WORDS (1024 * SMALL_WPT)
__global__ __launch_bounds__(1024) void k_frontier_compact_small(CompactArgs a) {
    __shared__ uint32_t wc[16], wo[16], wi[16], wt[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t wpt = (a.n_words + 1023u) / 1024u;      // consecutive words per thread (<= SMALL_WPT)
    const uint32_t w0 = tid * wpt;
    uint32_t words[SMALL_WPT];
    uint32_t cnt = 0, dout = 0, din = 0, tch = 0;
#pragma unroll
    for (int k = 0; k < SMALL_WPT; ++k) {
        words[k] = 0;
        const uint32_t idx = w0 + k;
        if ((uint32_t)k < wpt && idx < a.n_words) {
            const uint32_t live = a.alive[idx];
            uint32_t w = a.bm[idx];
            if (a.mk) w |= take_marks(a.mk, idx);
            w &= live;
            tch += __popc(w);
            if (a.bm_sink) w |= (a.bm_sink[idx] | a.bm_vadd[idx]) & live;
            if (a.bm_prev) w |= a.bm_prev[idx] & live;
            a.bm[idx] = w;
            if (a.rep && w) a.rep[idx] |= w;
            words[k] = w;
            cnt += __popc(w);
            uint32_t d_o, d_i;
            word_degrees(a, idx, w, d_o, d_i);
            dout += d_o;
            din += d_i;
        }
    }
    uint32_t ic = cnt, io = dout, ii = din, it = tch;
    for (int o = 1; o < 64; o <<= 1) {
        uint32_t tc = __shfl_up(ic, o), to = __shfl_up(io, o), ti = __shfl_up(ii, o);
        if (lane >= o) {
            ic += tc;
            io += to;
            ii += ti;
        }
    }
    for (int o = 32; o > 0; o >>= 1) it += __shfl_down(it, o);
    if (lane == 63) {
        wc[wave] = ic;
        wo[wave] = io;
        wi[wave] = ii;
    }
    if (lane == 0) wt[wave] = it;
    __syncthreads();
    uint32_t oc = ic - cnt, oo = io - dout, oi = ii - din;
    for (int k = 0; k < wave; ++k) {
        oc += wc[k];
        oo += wo[k];
        oi += wi[k];
    }
#pragma unroll 1
    for (uint32_t k = 0; k < wpt; ++k) {                   // one copy of the (long, unrolled) word code
        const uint32_t idx = w0 + k;
        if (idx >= a.n_words) break;
        const uint32_t w = a.bm[idx];                      // this thread's own store of the first loop
        if (!w) continue;
        WordDeg wd;
        uint32_t d_o, d_i;
        wd.gather(a, idx, w, d_o, d_i);
        wd.emit(a, idx, w, oc, oo, oi);
    }
    if (tid == 1023) {                                     // the last thread ends on the grand totals
        *a.count_out = oc;
        if (a.want_out) {
            a.eoff[oc] = oo;
            if (a.msgs_out) *a.msgs_out = oo;
        }
        if (a.want_in) {
            a.ioff[oc] = oi;
            if (a.isum_out) *a.isum_out = oi;
        }
    }
    if (tid == 0 && a.touched_out) {
        uint32_t t = 0;
        for (int k = 0; k < 16; ++k) t += wt[k];
        if (t) atomicAdd(a.touched_out, t);
    }
}

// expect: how many vertices the list will probably hold. One workgroup writes a long list slowly
// (its scattered stores all leave through one CU), so the single-launch kernel is kept for short ones.
static void launch_compact(ripple_ctx *c, const CompactArgs &a, uint32_t expect) {
    if (a.n_words <= SMALL_WORDS && expect <= 4096) {
        hipLaunchKernelGGL(k_frontier_compact_small, dim3(1), dim3(1024), 0, c->stream, a);
        return;
    }
    const uint32_t nb = rp_div_up(a.n_words, 256);
    hipLaunchKernelGGL(k_frontier_count, dim3(nb), dim3(256), 0, c->stream, a);
    hipLaunchKernelGGL(k_frontier_emit, dim3(nb), dim3(256), 0, c->stream, a);
}

// degree prefixes over an arbitrary (unsorted) list, one workgroup: out-degrees into eoff (hop 0, and the
// lists of small frontiers) and, with in_meta and ioff given, in-degrees into ioff in the same sweep.
// Every thread takes four consecutive entries per round, so that a list that turns out long (the
// small-frontier path is chosen on the previous batch's sizes) costs a quarter of the round trips.
#define EOFF_PER 4
__global__ __launch_bounds__(1024) void k_list_eoff(const uint32_t *list, const uint32_t *count_ptr,
                                                    const uint2 *out_meta, uint32_t *eoff, uint32_t *msgs_out,
                                                    const uint2 *in_meta, uint32_t *ioff, uint32_t *isum_out) {
    __shared__ uint32_t wo[16], wi[16];
    __shared__ uint32_t carry_o, carry_i;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t count = *count_ptr;
    const bool want_o = eoff != nullptr, want_i = in_meta != nullptr && ioff != nullptr;   // kernel arguments: uniform
    if (tid == 0) {
        carry_o = 0;
        carry_i = 0;
    }
    __syncthreads();
    for (uint32_t base = 0; base < count; base += 1024 * EOFF_PER) {
        const uint32_t i0 = base + tid * EOFF_PER;
        uint32_t v[EOFF_PER], dgo[EOFF_PER], dgi[EOFF_PER];
#pragma unroll
        for (int k = 0; k < EOFF_PER; ++k) v[k] = (i0 + k < count) ? list[i0 + k] : 0u;
        uint32_t so = 0, si = 0;
#pragma unroll
        for (int k = 0; k < EOFF_PER; ++k) {
            const bool on = i0 + k < count;
            dgo[k] = (on && want_o) ? out_meta[v[k]].y : 0u;
            dgi[k] = (on && want_i) ? in_meta[v[k]].y : 0u;
            so += dgo[k];
            si += dgi[k];
        }
        uint32_t inc_o = so, inc_i = si;
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t to = __shfl_up(inc_o, o), ti = __shfl_up(inc_i, o);
            if (lane >= o) {
                inc_o += to;
                inc_i += ti;
            }
        }
        if (lane == 63) {
            wo[wave] = inc_o;
            wi[wave] = inc_i;
        }
        __syncthreads();
        uint32_t off_o = carry_o, off_i = carry_i;
        for (int k = 0; k < wave; ++k) {
            off_o += wo[k];
            off_i += wi[k];
        }
        uint32_t run_o = off_o + inc_o - so, run_i = off_i + inc_i - si;
#pragma unroll
        for (int k = 0; k < EOFF_PER; ++k) {
            if (i0 + k < count) {
                if (want_o) eoff[i0 + k] = run_o;
                if (want_i) ioff[i0 + k] = run_i;
            }
            run_o += dgo[k];
            run_i += dgi[k];
        }
        __syncthreads();
        if (tid == 1023) {
            carry_o = off_o + inc_o;
            carry_i = off_i + inc_i;
        }
        __syncthreads();
    }
    if (tid == 0) {
        if (want_o) {
            eoff[count] = carry_o;
            if (msgs_out) *msgs_out = carry_o;
        }
        if (want_i) {
            ioff[count] = carry_i;
            if (isum_out) *isum_out = carry_i;
        }
    }
}

void rp_launch_frontier_mark(ripple_ctx *c, uint32_t l, bool allow_disc, uint32_t pair_cap) {
    if (pair_cap) {
        hipLaunchKernelGGL(k_frontier_mark_pairs, dim3(c->n_cu * 8), dim3(256), 0, c->stream, c->list[l - 1],
                           &c->ctr->a[l - 1], c->eoff[l - 1], c->out_meta, c->out_pool, c->mk, c->ctr, l, c->xw[l],
                           rp_layer_mode(c, l), c->opt_pull_ratio, allow_disc ? 1 : 0, c->pk_a, c->pv_a, pair_cap);
        return;
    }
    hipLaunchKernelGGL(k_frontier_mark, dim3(c->n_cu * 8), dim3(256), 0, c->stream, c->list[l - 1], &c->ctr->a[l - 1],
                       c->eoff[l - 1], c->out_meta, c->out_pool, c->mk, c->ctr, l, c->xw[l], rp_layer_mode(c, l),
                       c->opt_pull_ratio, allow_disc ? 1 : 0);
}

// all live vertices, ascending, in c->all_list (count in ctr->n_all) with the exclusive scan of
// their in-degrees in c->ioff_all: the work list of a discovering hop
void rp_launch_alive_list(ripple_ctx *c) {
    CompactArgs a;
    memset(&a, 0, sizeof(a));
    a.list_cap = 0xFFFFFFFFu;
    a.bm = c->alive;                               // rewritten with the same bits
    a.alive = c->alive;
    a.n_words = c->n_words;
    a.out_meta = c->out_meta;
    a.in_meta = c->in_meta;
    a.want_in = 1;
    a.part_cnt = c->part_cnt;
    a.part_out = c->part_deg;
    a.part_in = c->part_ideg;
    a.list = c->all_list;
    a.ioff = c->ioff_all;
    a.count_out = &c->ctr->n_all;
    launch_compact(c, a, c->n_cap);
}

// bitmap of layer l, merged with S, V_added (and A_{l-1} when self_term) -> list[l], ctr->a[l];
// want_out: eoff[l] and ctr->m[l+1] (the next hop's edge walk); want_in: ioff[l], ctr->isum[l]
// pruned: bm[l] already is the hop's final set (max / min layers: candidates whose aggregate did not
// change have been taken out again), so neither marks nor S are merged into it
void rp_launch_frontier_compact(ripple_ctx *c, uint32_t l, bool self_term, bool want_out, bool want_in,
                                bool accumulate_rep, bool pruned) {
    CompactArgs a;
    a.bm = c->bm[l];
    a.mk = pruned ? nullptr : c->mk;
    a.bm_prev = self_term ? c->bm[l - 1] : nullptr;
    a.bm_sink = pruned ? nullptr : c->bm_sink;
    a.bm_vadd = c->bm_vadd;
    a.alive = c->alive;
    a.n_words = c->n_words;
    a.out_meta = c->out_meta;
    a.in_meta = c->in_meta;
    a.want_out = want_out ? 1 : 0;
    a.want_in = want_in ? 1 : 0;
    a.part_cnt = c->part_cnt;
    a.part_out = c->part_deg;
    a.part_in = c->part_ideg;
    a.rep = accumulate_rep ? c->rep[l] : nullptr;
    a.touched_out = pruned ? nullptr : &c->ctr->touched[l];
    a.list = c->list[l];
    a.eoff = c->eoff[l];
    a.ioff = c->ioff[l];
    a.count_out = &c->ctr->a[l];
    a.msgs_out = (l < RIPPLE_MAX_LAYERS) ? &c->ctr->m[l + 1] : nullptr;
    a.isum_out = &c->ctr->isum[l];
    a.list_cap = 0xFFFFFFFFu;
    launch_compact(c, a, rp_rows_hint(c, l));
}

// Candidates of a max / min hop: the vertices marked by the out-edge walk from A_{l-1}, S and V_added,
// into bm[l] and, ascending, into c->all_list (count in ctr->n_all). The aggregation kernel then
// clears the bits of those whose aggregate stays as it is.
void rp_launch_candidates(ripple_ctx *c, uint32_t l) {
    CompactArgs a;
    memset(&a, 0, sizeof(a));
    a.list_cap = 0xFFFFFFFFu;
    a.bm = c->bm[l];
    a.mk = c->mk;
    a.bm_sink = c->bm_sink;
    a.bm_vadd = c->bm_vadd;
    a.alive = c->alive;
    a.n_words = c->n_words;
    a.out_meta = c->out_meta;
    a.in_meta = c->in_meta;
    a.part_cnt = c->part_cnt;
    a.part_out = c->part_deg;
    a.part_in = c->part_ideg;
    a.touched_out = &c->ctr->touched[l];
    a.list = c->all_list;
    a.count_out = &c->ctr->n_all;
    launch_compact(c, a, c->hints_valid ? c->last_cand[l] : c->n_cap);
}

// any bitmap & alive -> ascending list in `out_list`, count in *count_d (device)
void rp_launch_bitmap_to_list(ripple_ctx *c, uint32_t *bitmap, uint32_t *out_list, uint32_t *count_d) {
    CompactArgs a;
    memset(&a, 0, sizeof(a));
    a.list_cap = 0xFFFFFFFFu;
    a.bm = bitmap;
    a.alive = c->alive;
    a.n_words = c->n_words;
    a.out_meta = c->out_meta;
    a.in_meta = c->in_meta;
    a.part_cnt = c->part_cnt;
    a.part_out = c->part_deg;
    a.part_in = c->part_ideg;
    a.list = out_list;
    a.count_out = count_d;
    launch_compact(c, a, c->n_cap);
}

// ---------------------------------------------------------------------------------
// the same compaction without any allocation: block sums in a static device array
// ---------------------------------------------------------------------------------
// Per-block partial sums of the two-pass compaction (three arrays of RP_STATIC_BLOCKS entries: vertex
// counts, and the out- and in-degree sums the first pass writes alongside). One copy per GPU, shared by
// every context on that GPU and kept until the process ends; every launch writes the entries it reads,
// so nothing has to be cleared between calls, and calls that overlap on one GPU race on it.
#define RP_STATIC_BLOCKS 16384u                  // 256 bitmap words = 8192 vertices per block
static __device__ __align__(256) uint32_t scratch[3 * RP_STATIC_BLOCKS];
#define RP_MAX_DEVICES 64
static uint32_t *g_scratch_ptr[RP_MAX_DEVICES] = {nullptr};    // the array's address on each GPU

uint32_t rp_static_max_vertices() { return RP_STATIC_BLOCKS * 256u * 32u; }

// Called by init_graph with the context's device current: looks the array's address up once per GPU.
ripple_status rp_static_scratch_init(ripple_ctx *c) {
    if (c->device < 0 || c->device >= RP_MAX_DEVICES) return RIPPLE_OK;      // such a GPU has no no-allocation path
    if (g_scratch_ptr[c->device]) return RIPPLE_OK;
    uint32_t *ptr = nullptr;
    RP_HIP(c, hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)));
    g_scratch_ptr[c->device] = ptr;
    return RIPPLE_OK;
}

// bitmap & alive -> ascending ids in ids_out (device, room for cap), set size in *n_out (device). Allocates nothing.
ripple_status rp_launch_affected_static(ripple_ctx *c, uint32_t *bitmap, uint32_t *ids_out, uint32_t cap,
                                        uint32_t *n_out) {
    uint32_t *ptr = (c->device >= 0 && c->device < RP_MAX_DEVICES) ? g_scratch_ptr[c->device] : nullptr;
    if (!ptr) {
        c->err = "the static scratch array was not set up for this GPU";
        return RIPPLE_ESTATE;
    }
    const uint32_t nb = rp_div_up(c->n_words, 256);
    if (nb > RP_STATIC_BLOCKS) {
        c->err = "vertex capacity " + std::to_string(c->n_cap) + " exceeds what the no-allocation call supports (" +
                 std::to_string(rp_static_max_vertices()) + ")";
        return RIPPLE_EINVAL;
    }
    CompactArgs a;
    memset(&a, 0, sizeof(a));
    a.bm = bitmap;
    a.alive = c->alive;
    a.n_words = c->n_words;
    a.out_meta = c->out_meta;
    a.in_meta = c->in_meta;
    a.part_cnt = ptr;
    a.part_out = ptr + RP_STATIC_BLOCKS;
    a.part_in = ptr + 2 * RP_STATIC_BLOCKS;
    a.list = ids_out;
    a.list_cap = cap;
    a.count_out = n_out;
    hipLaunchKernelGGL(k_frontier_count, dim3(nb), dim3(256), 0, c->stream, a);
    hipLaunchKernelGGL(k_frontier_emit, dim3(nb), dim3(256), 0, c->stream, a);
    RP_HIP(c, hipGetLastError());
    RP_HIP(c, hipStreamSynchronize(c->stream));
    return RIPPLE_OK;
}

void rp_launch_list_eoff(ripple_ctx *c, uint32_t l) {
    hipLaunchKernelGGL(k_list_eoff, dim3(1), dim3(1024), 0, c->stream, c->list[l], &c->ctr->a[l], c->out_meta,
                       c->eoff[l], l < RIPPLE_MAX_LAYERS ? &c->ctr->m[l + 1] : (uint32_t *)nullptr,
                       (const uint2 *)nullptr, (uint32_t *)nullptr, (uint32_t *)nullptr);
}

static SparseArgs sparse_args(ripple_ctx *c, uint32_t l, uint32_t *list, uint32_t *count, bool self_term) {
    SparseArgs sp;
    sp.bm = c->bm[l];
    sp.alive = c->alive;
    sp.list = list;
    sp.count = count;
    sp.touched = &c->ctr->touched[l];
    sp.st_dst = c->st_dst;
    sp.n_struct = &c->ctr->n_struct;
    sp.struct_cap = c->struct_cap;
    sp.list0 = c->list[0];
    sp.count0 = &c->ctr->a[0];
    sp.bm_vadd = c->bm_vadd;
    sp.self_term = self_term ? 1 : 0;
    sp.in_meta = c->in_meta;
    sp.long_min = 0;
    sp.long_list = nullptr;
    sp.long_count = nullptr;
    sp.long_dup = 0;
    return sp;
}

// Candidates of a small max / min hop, listed while they are marked: the set of rp_launch_candidates
// (with A_{l-1} when the layer has a self term) in bm[l] and, unordered, in c->all_list, count in
// ctr->cand[l] (zero since the batch began).
void rp_launch_candidates_sparse(ripple_ctx *c, uint32_t l, bool self_term, uint32_t long_min) {
    SparseArgs sp = sparse_args(c, l, c->all_list, &c->ctr->cand[l], self_term);
    sp.long_min = long_min;                              // candidates with longer in-rows: straight into the queue of the
    sp.long_list = c->eoff[l];                           // workgroup role (free until the hop's set is final), count in
    sp.long_count = &c->ctr->n_long[l];                  // ctr->n_long[l] (zero since the batch began)
    hipLaunchKernelGGL(k_frontier_sparse, dim3(c->n_cu), dim3(256), 0, c->stream, c->list[l - 1], &c->ctr->a[l - 1],
                       c->eoff[l - 1], c->out_meta, c->out_pool, sp);
}

// Hop l for a small frontier: out-edge walk from A_{l-1} and the roots (S, V_added, A_{l-1} when self_term)
// straight into bm[l] and list[l] (unordered), then the degree prefixes over that list. Two launches
// instead of the walk plus a scan of the whole bitmap.
// long_min > 0 (attention hops): vertices with more in-neighbours than that are also queued in c->all_list
// (count in ctr->n_long[l], zero since the batch began) for the workgroup role of the aggregation kernel.
void rp_launch_frontier_sparse(ripple_ctx *c, uint32_t l, bool self_term, bool want_out, uint32_t long_min) {
    SparseArgs sp = sparse_args(c, l, c->list[l], &c->ctr->a[l], self_term);
    if (long_min) {
        sp.long_min = long_min;
        sp.long_list = c->all_list;
        sp.long_count = &c->ctr->n_long[l];
        sp.long_dup = 1;
    }
    hipLaunchKernelGGL(k_frontier_sparse, dim3(c->n_cu), dim3(256), 0, c->stream, c->list[l - 1], &c->ctr->a[l - 1],
                       c->eoff[l - 1], c->out_meta, c->out_pool, sp);
    rp_launch_list_offsets(c, l, want_out);
}

// degree prefixes over the (unordered) list of hop l
void rp_launch_list_offsets(ripple_ctx *c, uint32_t l, bool want_out) {
    hipLaunchKernelGGL(k_list_eoff, dim3(1), dim3(1024), 0, c->stream, c->list[l], &c->ctr->a[l], c->out_meta,
                       want_out ? c->eoff[l] : (uint32_t *)nullptr,
                       (want_out && l < RIPPLE_MAX_LAYERS) ? &c->ctr->m[l + 1] : (uint32_t *)nullptr, c->in_meta, c->ioff[l],
                       &c->ctr->isum[l]);
}

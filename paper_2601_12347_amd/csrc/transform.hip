// Dirty-row transform (the Compute step of Sec. 3.3 in re-apply form): for every
// vertex v of A_l gather the layer's input row
//     GraphConv  x            GraphSAGE  [h_self | x]        GIN  (1+eps) h_self + x
// (x = X^l[v], divided by the in-degree for mean), multiply by the weight
// matrix on the matrix cores, add the bias, apply the activation, and emit
//     D^l[v] = h_new - H^l[v],   H^l[v] = h_new
// so that the next hop can forward the delta (Sec. 3.3.3).
//
// Tiling: a workgroup of four wavefronts computes a (WAVES_M*TM*32) x (WAVES_N*TN*32)
// output tile; each wavefront owns TM x TN MFMA 32x32x2 (fp32) accumulators. K is
// consumed in slices of 32 staged through LDS. Later slices are already on their
// way from memory into registers while the matrix cores work on the current one:
// the weight slice (an L2 hit) one step ahead, the gathered rows (HBM latency)
// STAGES steps ahead. The fetch is branch-free (addresses are clamped, the row
// mode is a template parameter) and touches no loaded value, so nothing waits on
// memory until the registers are written to LDS; scaling, the SAGE/GIN combination
// and zero padding are applied at that point.
//
// Layers whose output is much narrower than their input (the classifier layer) are
// handled "project first": aggregation and the linear map commute, so the deltas are
// multiplied by the neighbour weights before they are scattered, the cached aggregate
// holds sum_u H[u] W_neigh (d_out wide), and the row transform only adds it
// (scaled for mean) to h_self W_self + b in the epilogue.
#include "common.h"
#include "kernels.h"
#include <algorithm>

#include "transform_args.h"

__device__ __forceinline__ float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {     // round to nearest even
    const __hip_bfloat16 a = __float2bfloat16(lo), b = __float2bfloat16(hi);
    return (uint32_t)__builtin_bit_cast(unsigned short, a) | ((uint32_t)__builtin_bit_cast(unsigned short, b) << 16);
}

// Raw 16 (or 8) bytes for four consecutive k of one gathered row; no arithmetic on the data.
// MODE 1 with bf16 embeddings and MODE 2 need two sources (p: own embedding, q: aggregate).
template <int MODE, int STORE>
__device__ __forceinline__ void fetch_raw(const TArgs &a, uint32_t v, uint32_t slot, uint32_t k, floatx4 &p, floatx4 &q) {
    const uint32_t kc = min(k, a.K - 4u);                     // stay inside the row; padding is zeroed later
    const size_t row = (size_t)v * a.d_in;
    if (MODE == 0) {
        p = *(const floatx4 *)(a.X + row + kc);
    } else if (MODE == 3) {
        p = *(const floatx4 *)(a.tmp_in + (size_t)slot * a.tmp_ld + kc);
    } else if (MODE == 4) {
        if (STORE) {
            const uint2 r = *(const uint2 *)((const __hip_bfloat16 *)a.Hprev + row + kc);
            p.x = __uint_as_float(r.x);
            p.y = __uint_as_float(r.y);
        } else {
            p = *(const floatx4 *)((const float *)a.Hprev + row + kc);
        }
    } else if (MODE == 2) {
        q = *(const floatx4 *)(a.X + row + kc);
        if (STORE) {
            const uint2 r = *(const uint2 *)((const __hip_bfloat16 *)a.Hprev + row + kc);
            p.x = __uint_as_float(r.x);
            p.y = __uint_as_float(r.y);
        } else {
            p = *(const floatx4 *)((const float *)a.Hprev + row + kc);
        }
    } else {                                                  // MODE 1: k < d_in own embedding, else aggregate
        if (STORE) {
            const uint32_t kh = min(kc, a.d_in - 4u), kx = kc >= a.d_in ? kc - a.d_in : 0u;
            const uint2 r = *(const uint2 *)((const __hip_bfloat16 *)a.Hprev + row + kh);
            p.x = __uint_as_float(r.x);
            p.y = __uint_as_float(r.y);
            q = *(const floatx4 *)(a.X + row + kx);
        } else {
            const float *src = (kc < a.d_in) ? (const float *)a.Hprev + row + kc : a.X + row + (kc - a.d_in);
            p = *(const floatx4 *)src;
        }
    }
}

template <int MODE, int STORE>
__device__ __forceinline__ floatx4 finish_raw(const TArgs &a, floatx4 p, floatx4 q, uint32_t k, float scale) {
    floatx4 h = p;
    if (STORE && (MODE == 1 || MODE == 2 || MODE == 4)) {
        const uint32_t w0 = __float_as_uint(p.x), w1 = __float_as_uint(p.y);
        h.x = bf_lo(w0);
        h.y = bf_hi(w0);
        h.z = bf_lo(w1);
        h.w = bf_hi(w1);
    }
    floatx4 r;
    if (MODE == 0) {
        r = p * scale;
    } else if (MODE == 3) {
        r = p;
    } else if (MODE == 4) {
        r = h;
    } else if (MODE == 2) {
        r = h * a.one_plus_eps + q * scale;
    } else {
        const floatx4 x = STORE ? q : p;
        r = (k < a.d_in) ? h : x * scale;
    }
    if (k >= a.K) r = (floatx4)(0.0f);
    return r;
}

// Bias, (projected aggregate,) activation, delta against the stored row, store. Everything that
// is read (old rows, aggregate rows) is read in batches of TN*16 loads before anything is written:
// a load may not move above an earlier store to the same array, so interleaving them would pay one
// memory round trip per element.
template <int TM, int TN>
__device__ __forceinline__ void epilogue(const TArgs &a, floatx16 (&acc)[TM][TN], const uint32_t *s_vtx,
                                         const float *s_scale, uint32_t row0, uint32_t count, uint32_t n0, int wm, int wn,
                                         int lane) {
#pragma unroll
    for (int sm = 0; sm < TM; ++sm) {
        float old[TN][16], add[TN][16];
#pragma unroll
        for (int sn = 0; sn < TN; ++sn) {
            const uint32_t col = n0 + (wn * TN + sn) * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int lr = (wm * TM + sm) * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                float o = 0.0f, ad = 0.0f;
                if (col < a.N && row0 + lr < count) {
                    const size_t hidx = (size_t)s_vtx[lr] * a.N + col;
                    if (a.out_mode == 1)
                        o = a.store ? __bfloat162float(((const __hip_bfloat16 *)a.Hout)[hidx]) : ((const float *)a.Hout)[hidx];
                    if (a.addend) ad = a.addend[hidx] * (a.addend_scaled ? s_scale[lr] : 1.0f);
                }
                old[sn][r] = o;
                add[sn][r] = ad;
            }
        }
#pragma unroll
        for (int sn = 0; sn < TN; ++sn) {
            const uint32_t col = n0 + (wn * TN + sn) * 32 + (lane & 31);
            if (col >= a.N) continue;
            const float bias = a.bias[col];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int lr = (wm * TM + sm) * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                const uint32_t slot = row0 + lr;
                if (slot >= count) continue;
                float z = acc[sm][sn][r] + bias + add[sn][r];
                if (a.act == RIPPLE_ACT_RELU) z = z > 0.0f ? z : 0.0f;
                if (a.out_mode == 0) {
                    a.tmp_out[(size_t)slot * a.tmp_out_ld + col] = z;
                } else if (a.out_mode == 2) {
                    a.tmp_out[(size_t)s_vtx[lr] * a.tmp_out_ld + col] = z;
                } else {
                    const size_t hidx = (size_t)s_vtx[lr] * a.N + col;
                    if (a.store) {
                        const __hip_bfloat16 zr = __float2bfloat16(z);
                        z = __bfloat162float(zr);
                        ((__hip_bfloat16 *)a.Hout)[hidx] = zr;
                    } else {
                        ((float *)a.Hout)[hidx] = z;
                    }
                    if (a.D) a.D[hidx] = a.d_old ? old[sn][r] : z - old[sn][r];
                }
            }
        }
    }
}

// 16-byte (or element-wise, for rows whose width is not a multiple of four) accesses of the epilogues
__device__ __forceinline__ floatx4 ld4(const float *p, bool vec, uint32_t n_valid) {
    if (vec) return *(const floatx4 *)p;
    floatx4 r = (floatx4)(0.0f);
    if (n_valid > 0) r.x = p[0];
    if (n_valid > 1) r.y = p[1];
    if (n_valid > 2) r.z = p[2];
    if (n_valid > 3) r.w = p[3];
    return r;
}
__device__ __forceinline__ void st4(float *p, floatx4 v, bool vec, uint32_t n_valid) {
    if (vec) {
        *(floatx4 *)p = v;
        return;
    }
    if (n_valid > 0) p[0] = v.x;
    if (n_valid > 1) p[1] = v.y;
    if (n_valid > 2) p[2] = v.z;
    if (n_valid > 3) p[3] = v.w;
}
__device__ __forceinline__ floatx4 ld4_bf16(const __hip_bfloat16 *p, bool vec, uint32_t n_valid) {
    floatx4 r = (floatx4)(0.0f);
    if (vec) {
        const uint2 w = *(const uint2 *)p;
        r.x = bf_lo(w.x);
        r.y = bf_hi(w.x);
        r.z = bf_lo(w.y);
        r.w = bf_hi(w.y);
        return r;
    }
    if (n_valid > 0) r.x = __bfloat162float(p[0]);
    if (n_valid > 1) r.y = __bfloat162float(p[1]);
    if (n_valid > 2) r.z = __bfloat162float(p[2]);
    if (n_valid > 3) r.w = __bfloat162float(p[3]);
    return r;
}

// One round of the staged epilogue: U groups of four consecutive columns per thread. What the round
// reads and writes is fixed at compile time, so that its loads form one branch-free batch (a branch
// between two loads makes the second wait for the first):
//   EPI 0: act(z) goes to tmp_out (by slot or by vertex); nothing is read
//   EPI 1: H is updated;  EPI 2: H is updated and the delta row written
//   VEC: 16-byte accesses (row widths that are multiples of four); BF: bf16 embeddings
template <int BN, int U, bool VEC, int EPI, bool BF>
struct EpiRound {
    floatx4 old[U], add[U];
    uint32_t nv[U];                                        // valid columns of the group (0: nothing to do)

    // request the old row and the addend of round it0 (no stores in here). With VEC, groups that will
    // not be stored read a valid address all the same (the row of vertex 0 for slots past the end, the
    // row's last four columns for padded columns), and a missing addend reads the bias instead.
    __device__ __forceinline__ void load(const TArgs &a, const uint32_t *s_vtx, const float *s_scale, uint32_t row0,
                                         uint32_t count, uint32_t n0, int tid, int it0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int idx = tid + (it0 + u) * 256;
            const int r = idx / (BN / 4), c4 = (idx % (BN / 4)) * 4;
            const uint32_t col = n0 + c4;
            const uint32_t lim = (a.split_col && col < a.split_col) ? a.N1 : a.N;   // end of the block of columns `col` lies in
            nv[u] = (row0 + r < count && col < lim) ? min(4u, lim - col) : 0u;
            old[u] = (floatx4)(0.0f);
            add[u] = (floatx4)(0.0f);
            if (EPI == 0) continue;
            if (VEC) {
                const uint32_t lcol = min(col, a.N - 4u);
                const size_t hidx = (size_t)s_vtx[r] * a.N + lcol;
                old[u] = BF ? ld4_bf16((const __hip_bfloat16 *)a.Hout + hidx, true, 4) : ld4((const float *)a.Hout + hidx, true, 4);
                const float *ap = a.addend ? a.addend + hidx : a.bias + lcol;
                const floatx4 t = ld4(ap, true, 4);
                const float sc = a.addend ? (a.addend_scaled ? s_scale[r] : 1.0f) : 0.0f;
                add[u] = a.addend ? t * sc : (floatx4)(0.0f);
            } else if (nv[u]) {
                const size_t hidx = (size_t)s_vtx[r] * a.N + col;
                old[u] = BF ? ld4_bf16((const __hip_bfloat16 *)a.Hout + hidx, false, nv[u])
                            : ld4((const float *)a.Hout + hidx, false, nv[u]);
                if (a.addend) add[u] = ld4(a.addend + hidx, false, nv[u]) * (a.addend_scaled ? s_scale[r] : 1.0f);
            }
        }
    }

    // bias, addend, activation, delta, stores
    __device__ __forceinline__ void finish(const TArgs &a, const float *Cs, const uint32_t *s_vtx, uint32_t row0,
                                           uint32_t n0, int tid, int it0) const {
        constexpr int C_LD = BN + 4;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (!nv[u]) continue;
            const int idx = tid + (it0 + u) * 256;
            const int r = idx / (BN / 4), c4 = (idx % (BN / 4)) * 4;
            const uint32_t col = n0 + c4, slot = row0 + r;
            floatx4 v = *(const floatx4 *)&Cs[r * C_LD + c4] + *(const floatx4 *)(a.bias + col) + add[u];   // bias is padded
            if (a.act == RIPPLE_ACT_RELU) {
                v.x = v.x > 0.0f ? v.x : 0.0f;
                v.y = v.y > 0.0f ? v.y : 0.0f;
                v.z = v.z > 0.0f ? v.z : 0.0f;
                v.w = v.w > 0.0f ? v.w : 0.0f;
            }
            if (EPI == 0) {
                const size_t orow = (a.out_mode == 0) ? slot : s_vtx[r];
                if (a.split_col && col >= a.split_col) st4(a.tmp_out2 + orow * a.tmp_out2_ld + (col - a.split_col), v, VEC, nv[u]);
                else st4(a.tmp_out + orow * a.tmp_out_ld + col, v, VEC, nv[u]);
                continue;
            }
            const size_t hidx = (size_t)s_vtx[r] * a.N + col;
            if (BF) {
                uint2 w;
                w.x = pack_bf16x2(v.x, v.y);
                w.y = pack_bf16x2(v.z, v.w);
                unsigned short *hp = (unsigned short *)a.Hout + hidx;
                if (VEC) {
                    *(uint2 *)hp = w;
                } else {
                    if (nv[u] > 0) hp[0] = (unsigned short)(w.x & 0xFFFFu);
                    if (nv[u] > 1) hp[1] = (unsigned short)(w.x >> 16);
                    if (nv[u] > 2) hp[2] = (unsigned short)(w.y & 0xFFFFu);
                    if (nv[u] > 3) hp[3] = (unsigned short)(w.y >> 16);
                }
                v.x = bf_lo(w.x);
                v.y = bf_hi(w.x);
                v.z = bf_lo(w.y);
                v.w = bf_hi(w.y);
            } else {
                st4((float *)a.Hout + hidx, v, VEC, nv[u]);
            }
            if (EPI == 2) st4(a.D + hidx, a.d_old ? old[u] : v - old[u], VEC, nv[u]);
        }
    }
};

// The global reads (old row, addend) run one round ahead of the stores: the first round is requested
// while the accumulators settle in LDS, each later one before the previous round is finished, so that
// only one memory round trip per tile is exposed.
template <int BN, int ITER, int U, bool VEC, int EPI, bool BF>
__device__ __forceinline__ void epilogue_rounds(const TArgs &a, const float *Cs, const uint32_t *s_vtx, const float *s_scale,
                                                uint32_t row0, uint32_t count, uint32_t n0, int tid) {
    EpiRound<BN, U, VEC, EPI, BF> ra, rb;
    ra.load(a, s_vtx, s_scale, row0, count, n0, tid, 0);
    __syncthreads();                                       // the tile is in LDS
#pragma unroll 1
    for (int it0 = 0; it0 < ITER; it0 += 2 * U) {
        rb.load(a, s_vtx, s_scale, row0, count, n0, tid, it0 + U);
        ra.finish(a, Cs, s_vtx, row0, n0, tid, it0);
        if (it0 + 2 * U < ITER) ra.load(a, s_vtx, s_scale, row0, count, n0, tid, it0 + 2 * U);
        rb.finish(a, Cs, s_vtx, row0, n0, tid, it0 + U);
    }
}

template <int BN, int ITER, int U, bool VEC, bool BF>
__device__ __forceinline__ void epilogue_pick(const TArgs &a, const float *Cs, const uint32_t *s_vtx, const float *s_scale,
                                              uint32_t row0, uint32_t count, uint32_t n0, int tid) {
    if (a.out_mode != 1) epilogue_rounds<BN, ITER, U, VEC, 0, BF>(a, Cs, s_vtx, s_scale, row0, count, n0, tid);
    else if (a.D) epilogue_rounds<BN, ITER, U, VEC, 2, BF>(a, Cs, s_vtx, s_scale, row0, count, n0, tid);
    else epilogue_rounds<BN, ITER, U, VEC, 1, BF>(a, Cs, s_vtx, s_scale, row0, count, n0, tid);
}

// Epilogue of the pipelined kernels: the accumulators are laid out row-major in LDS (over the A/B
// staging area, which is free by then), so that every thread handles four consecutive columns of a
// row. An addend is only read when H is updated (out_mode 1).
template <int TM, int TN, int BM, int BN, bool BF>
__device__ __forceinline__ void epilogue_staged(const TArgs &a, floatx16 (&acc)[TM][TN], float *Cs, const uint32_t *s_vtx,
                                                const float *s_scale, uint32_t row0, uint32_t count, uint32_t n0, int wm,
                                                int wn, int tid) {
    constexpr int C_LD = BN + 4;
    constexpr int ITER = BM * BN / 4 / 256, U = (ITER % 8 == 0) ? 4 : (ITER % 6 == 0) ? 3 : ITER / 2;
    static_assert(U >= 1 && ITER % (2 * U) == 0, "tile size");
    const int lane = tid & 63;
    const bool vec = (a.N & 3u) == 0 && (a.out_mode == 1 || (a.tmp_out_ld & 3u) == 0) &&
                     (a.split_col == 0 || ((a.N1 & 3u) == 0 && (a.tmp_out2_ld & 3u) == 0));
    __syncthreads();                                       // every wavefront is done with the A/B slices
#pragma unroll
    for (int sm = 0; sm < TM; ++sm)
#pragma unroll
        for (int sn = 0; sn < TN; ++sn)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int lr = (wm * TM + sm) * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                Cs[lr * C_LD + (wn * TN + sn) * 32 + (lane & 31)] = acc[sm][sn][r];
            }
    if (vec) epilogue_pick<BN, ITER, U, true, BF>(a, Cs, s_vtx, s_scale, row0, count, n0, tid);
    else epilogue_pick<BN, ITER, U, false, BF>(a, Cs, s_vtx, s_scale, row0, count, n0, tid);
}

// Project-first layers have no matrix product left per row: h = act(Y[v] * scale + PS[v] + b), with
// Y the projected aggregate and PS the cached self term (absent for GraphConv).
template <bool BF>
__device__ __forceinline__ void addend_only_rows(const TArgs &a) {
    constexpr int R = 8;                                   // rows per wavefront and round: their loads overlap
    const uint32_t count = *a.count_ptr;
    const int lane = threadIdx.x & 63;
    const uint32_t gw = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, nw = (gridDim.x * blockDim.x) >> 6;
    for (uint32_t s0 = gw * R; s0 < count; s0 += nw * R) {
        uint32_t v[R];
        float sc[R];
#pragma unroll
        for (int u = 0; u < R; ++u) v[u] = a.list[min(s0 + u, count - 1u)];
#pragma unroll
        for (int u = 0; u < R; ++u) {
            const uint32_t deg = a.in_meta[v[u]].y;        // read in any case: no branch between the loads
            sc[u] = a.mean ? 1.0f / (float)(deg > 1u ? deg : 1u) : 1.0f;
        }
        bool bad[R];
#pragma unroll
        for (int u = 0; u < R; ++u) bad[u] = false;
        if (a.den) {                                       // attention: numerator / denominator, 0 without in-neighbours
#pragma unroll
            for (int u = 0; u < R; ++u) {
                const float dn = a.den[v[u]];
                bad[u] = !isfinite(dn) && s0 + u < count;
                sc[u] = (a.in_meta[v[u]].y > 0u && dn > 0.0f) ? 1.0f / dn : 0.0f;
            }
        }
        const float *p2 = a.addend2 ? a.addend2 : a.addend;
        const float w2 = a.addend2 ? 1.0f : 0.0f;
        for (uint32_t col = lane; col < a.N; col += 64) {
            float y[R], p[R], old[R];
#pragma unroll
            for (int u = 0; u < R; ++u) {                  // rows past the end repeat the last one and are not stored
                const size_t hidx = (size_t)v[u] * a.N + col;
                y[u] = a.addend[hidx];
                p[u] = p2[hidx];                           // unconditional: a branch here would serialise the loads
                old[u] = BF ? __bfloat162float(((const __hip_bfloat16 *)a.Hout)[hidx]) : ((const float *)a.Hout)[hidx];
            }
            const float b = a.bias[col];
#pragma unroll
            for (int u = 0; u < R; ++u) {
                if (s0 + u >= count) continue;
                const size_t hidx = (size_t)v[u] * a.N + col;
                float z = y[u] * sc[u] + b + (w2 != 0.0f ? p[u] : 0.0f);
                if (a.den && !isfinite(z)) bad[u] = true;      // an overflowed exponential: inf / inf, or inf itself
                if (a.act == RIPPLE_ACT_RELU) z = z > 0.0f ? z : 0.0f;
                if (BF) {
                    const __hip_bfloat16 zr = __float2bfloat16(z);
                    z = __bfloat162float(zr);
                    ((__hip_bfloat16 *)a.Hout)[hidx] = zr;
                } else {
                    ((float *)a.Hout)[hidx] = z;
                }
                if (a.D) a.D[hidx] = a.d_old ? old[u] : z - old[u];
            }
        }
        if (a.den) {
            uint32_t n_bad = 0;
#pragma unroll
            for (int u = 0; u < R; ++u) n_bad += __ballot(bad[u]) != 0ull ? 1u : 0u;
            if (n_bad && lane == 0) atomicAdd(a.range_rows, n_bad);
        }
    }
}

// The same for sum / mean layers (no denominators), element by element over the flattened (slot, column) space: rows
// of a narrow layer (47 columns) leave a quarter of a wavefront idle when a lane is a column, and consecutive slots are
// mostly consecutive vertices, so consecutive lanes read consecutive addresses across row ends. OLD: the stored row is
// read (a delta row is written); ADD2: there is a cached self term.
template <bool BF, bool OLD, bool ADD2>
__global__ __launch_bounds__(256) void k_transform_addend_flat(TArgs a) {
    constexpr int U = 4;                                   // elements per thread and round: their loads overlap
    const uint32_t count = *a.count_ptr;
    const uint32_t total = count * a.N;                    // < 2^32 (checked by the launch)
    const uint32_t stride = gridDim.x * blockDim.x;
    for (uint64_t e0 = blockIdx.x * blockDim.x + threadIdx.x; e0 < total; e0 += (uint64_t)stride * U) {
        uint32_t col[U];
        size_t hidx[U];
        float sc[U], y[U], p[U], old[U];
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint64_t e = e0 + (uint64_t)u * stride;
            ok[u] = e < total;
            const uint32_t ec = ok[u] ? (uint32_t)e : total - 1u;   // past the end: the last element again, not stored
            const uint32_t slot = ec / a.N;
            col[u] = ec - slot * a.N;
            const uint32_t v = a.list[slot];
            hidx[u] = (size_t)v * a.N + col[u];
            const uint32_t deg = a.in_meta[v].y;
            sc[u] = a.mean ? 1.0f / (float)(deg > 1u ? deg : 1u) : 1.0f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            y[u] = a.addend[hidx[u]];
            p[u] = ADD2 ? a.addend2[hidx[u]] : 0.0f;
            old[u] = !OLD ? 0.0f : BF ? __bfloat162float(((const __hip_bfloat16 *)a.Hout)[hidx[u]]) : ((const float *)a.Hout)[hidx[u]];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (!ok[u]) continue;
            float z = y[u] * sc[u] + a.bias[col[u]] + p[u];
            if (a.act == RIPPLE_ACT_RELU) z = z > 0.0f ? z : 0.0f;
            if (BF) {
                const __hip_bfloat16 zr = __float2bfloat16(z);
                z = __bfloat162float(zr);
                ((__hip_bfloat16 *)a.Hout)[hidx[u]] = zr;
            } else {
                ((float *)a.Hout)[hidx[u]] = z;
            }
            if (OLD) a.D[hidx[u]] = a.d_old ? old[u] : z - old[u];
        }
    }
}

static void launch_addend_flat(ripple_ctx *c, const TArgs &a) {
    const dim3 grid(c->n_cu * 16), block(256);
#define RP_FLAT(BF, OLD, ADD2) hipLaunchKernelGGL((k_transform_addend_flat<BF, OLD, ADD2>), grid, block, 0, c->stream, a)
    const bool old = a.D != nullptr, add2 = a.addend2 != nullptr;
    if (a.store) {
        if (old) { if (add2) RP_FLAT(true, true, true); else RP_FLAT(true, true, false); }
        else { if (add2) RP_FLAT(true, false, true); else RP_FLAT(true, false, false); }
    } else {
        if (old) { if (add2) RP_FLAT(false, true, true); else RP_FLAT(false, true, false); }
        else { if (add2) RP_FLAT(false, false, true); else RP_FLAT(false, false, false); }
    }
#undef RP_FLAT
}

__global__ __launch_bounds__(256) void k_transform_addend_only(TArgs a) {
    if (a.store) addend_only_rows<true>(a);
    else addend_only_rows<false>(a);
}

template <int WAVES_M, int WAVES_N, int TM, int TN, int STAGES, int MODE, int STORE, int MINB = 2>
__global__ __launch_bounds__(256, MINB) void k_transform_f32(TArgs a) {
    constexpr int BM = WAVES_M * TM * 32, BN = WAVES_N * TN * 32;
    constexpr int NA = BM / 32, NB = BN / 32;              // float4 per thread per slice (A, B)
    constexpr bool TWO = (MODE == 2) || (MODE == 1 && STORE == 1);
    constexpr int A_BYTES = BM * (T_BK + 1) * 4, B_BYTES = T_BK * BN * 4, C_BYTES = BM * (BN + 4) * 4;
    constexpr int S_BYTES = (A_BYTES + B_BYTES > C_BYTES) ? A_BYTES + B_BYTES : C_BYTES;
    static_assert(A_BYTES % 16 == 0, "alignment of the weight slice");
    __shared__ __attribute__((aligned(16))) char smem[S_BYTES];   // A and B slices; reused by the staged epilogue
    float (*As)[T_BK + 1] = (float (*)[T_BK + 1]) smem;
    float (*Bs)[BN] = (float (*)[BN])(smem + A_BYTES);
    __shared__ uint32_t s_vtx[BM];
    __shared__ float s_scale[BM];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const uint32_t count = *a.count_ptr;
    const uint32_t n_tiles = (count + BM - 1) / BM;
    const uint32_t n0 = blockIdx.y * BN;

    for (uint32_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const uint32_t row0 = tile * BM;
        __syncthreads();                                   // previous tile's epilogue has read s_vtx
        for (int r = tid; r < BM; r += 256) {
            uint32_t slot = row0 + r;
            uint32_t v = 0;                                // rows past the end read vertex 0; never stored
            float sc = 1.0f;
            if (slot < count) {
                v = a.list[slot];
                if (a.mean) {
                    uint32_t deg = a.in_meta[v].y;
                    sc = 1.0f / (float)(deg > 1u ? deg : 1u);
                }
            }
            s_vtx[r] = v;
            s_scale[r] = sc;
        }
        __syncthreads();

        floatx16 acc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

        // per-thread row coordinates of its NA float4 of every slice
        uint32_t my_v[NA], my_slot[NA];
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int r = (tid + i * 256) / (T_BK / 4);
            my_v[i] = s_vtx[r];
            my_slot[i] = min(row0 + r, count - 1u);
        }
        const uint32_t c4a = (tid % (T_BK / 4)) * 4;       // (tid + i*256) % 8 is the same for every i

        floatx4 ra[STAGES][NA], rq[TWO ? STAGES : 1][TWO ? NA : 1], rb[NB];
        // weights first, as in every step of the loop, so that one wait count fits both ways into it
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int idx = tid + i * 256;
            const int kr = idx / (BN / 4), c4 = (idx % (BN / 4)) * 4;
            rb[i] = *(const floatx4 *)(a.W + (size_t)kr * a.Npad + n0 + c4);
        }
#pragma unroll
        for (int st = 0; st < STAGES; ++st)
#pragma unroll
            for (int i = 0; i < NA; ++i) {
                floatx4 q = (floatx4)(0.0f);
                fetch_raw<MODE, STORE>(a, my_v[i], my_slot[i], (uint32_t)st * T_BK + c4a, ra[st][i], q);
                if constexpr (TWO) rq[st][i] = q;
            }
        __builtin_amdgcn_sched_barrier(0);

        // The staging registers rotate by unrolling (slot s of step s mod STAGES), not by moves: a move
        // would have to wait for the load it copies.
        for (uint32_t kbase = 0; kbase < a.Kpad; kbase += STAGES * T_BK) {
#pragma unroll
          for (int s = 0; s < STAGES; ++s) {
            const uint32_t k0 = kbase + s * T_BK;
            if (k0 >= a.Kpad) break;
            __syncthreads();                               // the matrix cores are done with the previous slice
#pragma unroll
            for (int i = 0; i < NA; ++i) {
                const int r = (tid + i * 256) / (T_BK / 4);
                floatx4 q = (floatx4)(0.0f);
                if constexpr (TWO) q = rq[s][i];
                const floatx4 val = finish_raw<MODE, STORE>(a, ra[s][i], q, k0 + c4a, s_scale[r]);
                As[r][c4a + 0] = val.x;
                As[r][c4a + 1] = val.y;
                As[r][c4a + 2] = val.z;
                As[r][c4a + 3] = val.w;
            }
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                const int idx = tid + i * 256;
                const int kr = idx / (BN / 4), c4 = (idx % (BN / 4)) * 4;
                *(floatx4 *)&Bs[kr][c4] = rb[i];
            }
            __syncthreads();
            // memory returns loads in order: the weights (needed one step from now) are requested
            // before the rows (needed STAGES steps from now), so waiting for them leaves the rows in flight
            {                                              // weights of the next slice (last step re-reads its own: in bounds)
                const uint32_t kb = min(k0 + T_BK, a.Kpad - T_BK);
#pragma unroll
                for (int i = 0; i < NB; ++i) {
                    const int idx = tid + i * 256;
                    const int kr = idx / (BN / 4), c4 = (idx % (BN / 4)) * 4;
                    rb[i] = *(const floatx4 *)(a.W + (size_t)(kb + kr) * a.Npad + n0 + c4);
                }
            }
            {                                              // rows of the slice STAGES steps ahead (clamped: harmless past the end)
                const uint32_t kn = k0 + STAGES * T_BK + c4a;
#pragma unroll
                for (int i = 0; i < NA; ++i) {
                    floatx4 q = (floatx4)(0.0f);
                    fetch_raw<MODE, STORE>(a, my_v[i], my_slot[i], kn, ra[s][i], q);
                    if constexpr (TWO) rq[s][i] = q;
                }
            }
            // keep the requests above the matrix-core work: the scheduler would otherwise sink them to
            // the end of the step, where nothing is left to hide their latency behind
            __builtin_amdgcn_sched_barrier(0);
            // operands of the next pair of k are read from LDS before the matrix cores take the
            // current pair, so that no LDS round trip separates two groups of products
            float av[2][TM], bv[2][TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) av[0][i] = As[(wm * TM + i) * 32 + (lane & 31)][lane >> 5];
#pragma unroll
            for (int j = 0; j < TN; ++j) bv[0][j] = Bs[lane >> 5][(wn * TN + j) * 32 + (lane & 31)];
#pragma unroll
            for (int kk = 0; kk < T_BK; kk += 2) {
                const int cur = (kk >> 1) & 1, nxt = cur ^ 1;
                if (kk + 2 < T_BK) {
                    const int kq = kk + 2 + (lane >> 5);
#pragma unroll
                    for (int i = 0; i < TM; ++i) av[nxt][i] = As[(wm * TM + i) * 32 + (lane & 31)][kq];
#pragma unroll
                    for (int j = 0; j < TN; ++j) bv[nxt][j] = Bs[kq][(wn * TN + j) * 32 + (lane & 31)];
                }
                __builtin_amdgcn_sched_barrier(0);         // the scheduler would move the reads back next to their use
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[cur][i], bv[cur][j], acc[i][j], 0, 0, 0);
            }
          }
        }
        epilogue_staged<TM, TN, BM, BN, STORE != 0>(a, acc, (float *)smem, s_vtx, s_scale, row0, count, n0, wm, wn, tid);
    }
}

// Fallback for row widths that are not multiples of 4 (no 16-byte loads): same tiling, scalar
// gathers, no prefetch.
__device__ __forceinline__ float load_a1(const TArgs &a, uint32_t v, uint32_t slot, float scale, uint32_t k) {
    if (k >= a.K) return 0.0f;
    switch (a.a_mode) {
    case 0: return a.X[(size_t)v * a.d_in + k] * scale;
    case 1:
        return (k < a.d_in) ? rp_load_h(a.Hprev, a.store, (size_t)v * a.d_in + k)
                            : a.X[(size_t)v * a.d_in + (k - a.d_in)] * scale;
    case 2:
        return a.one_plus_eps * rp_load_h(a.Hprev, a.store, (size_t)v * a.d_in + k) + a.X[(size_t)v * a.d_in + k] * scale;
    case 4: return rp_load_h(a.Hprev, a.store, (size_t)v * a.d_in + k);
    default: return a.tmp_in[(size_t)slot * a.tmp_ld + k];
    }
}

template <int WAVES_M, int WAVES_N>
__global__ __launch_bounds__(256) void k_transform_generic(TArgs a) {
    constexpr int TM = 2, TN = 2;
    constexpr int BM = WAVES_M * 64, BN = WAVES_N * 64;
    __shared__ float As[BM][T_BK + 1];
    __shared__ float Bs[T_BK][BN];
    __shared__ uint32_t s_vtx[BM];
    __shared__ float s_scale[BM];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const uint32_t count = *a.count_ptr;
    const uint32_t n_tiles = (count + BM - 1) / BM;
    const uint32_t n0 = blockIdx.y * BN;
    for (uint32_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const uint32_t row0 = tile * BM;
        __syncthreads();
        for (int r = tid; r < BM; r += 256) {
            uint32_t slot = row0 + r;
            uint32_t v = 0;
            float sc = 1.0f;
            if (slot < count) {
                v = a.list[slot];
                if (a.mean) {
                    uint32_t deg = a.in_meta[v].y;
                    sc = 1.0f / (float)(deg > 1u ? deg : 1u);
                }
            }
            s_vtx[r] = v;
            s_scale[r] = sc;
        }
        __syncthreads();
        floatx16 acc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
        for (uint32_t k0 = 0; k0 < a.Kpad; k0 += T_BK) {
            for (int idx = tid; idx < BM * T_BK; idx += 256) {
                const int r = idx / T_BK, k = idx % T_BK;
                const uint32_t slot = row0 + r;
                As[r][k] = (slot < count) ? load_a1(a, s_vtx[r], slot, s_scale[r], k0 + k) : 0.0f;
            }
            for (int idx = tid; idx < T_BK * (BN / 4); idx += 256) {
                const int kr = idx / (BN / 4), c4 = (idx % (BN / 4)) * 4;
                *(float4 *)&Bs[kr][c4] = *(const float4 *)(a.W + (size_t)(k0 + kr) * a.Npad + n0 + c4);
            }
            __syncthreads();
#pragma unroll
            for (int kk = 0; kk < T_BK; kk += 2) {
                const int kq = kk + (lane >> 5);
                float av[TM], bv[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i) av[i] = As[(wm * TM + i) * 32 + (lane & 31)][kq];
#pragma unroll
                for (int j = 0; j < TN; ++j) bv[j] = Bs[kq][(wn * TN + j) * 32 + (lane & 31)];
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], bv[j], acc[i][j], 0, 0, 0);
            }
            __syncthreads();
        }
        epilogue<TM, TN>(a, acc, s_vtx, s_scale, row0, count, n0, wm, wn, lane);
    }
}

// ---------------------------------------------------------------------------------
// bf16 matrix-core variant (embeddings stored in bfloat16): MFMA 32x32x16 bf16 with fp32
// accumulation. Same tiling, prefetch and epilogue; the gathered rows are rounded to bf16 when
// they are written to LDS, the weights come from a transposed bf16 copy so that the eight
// consecutive k a lane feeds into one MFMA are one 16-byte LDS read for both operands.
// ---------------------------------------------------------------------------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));
#define TB_LD 40                                            // LDS row stride in bf16 (80 bytes)

template <int WAVES_M, int WAVES_N, int TM, int TN, int STAGES, int MODE>
__global__ __launch_bounds__(256, 2) void k_transform_bf16(TArgs a) {
    constexpr int STORE = 1;
    constexpr int BM = WAVES_M * TM * 32, BN = WAVES_N * TN * 32;
    constexpr int NA = BM / 32, NB = BN / 64;              // per thread per slice: float4 of A, 16-byte chunks of B
    constexpr bool TWO = (MODE == 2) || (MODE == 1);
    constexpr int A_BYTES = BM * TB_LD * 2, B_BYTES = BN * TB_LD * 2, C_BYTES = BM * (BN + 4) * 4;
    constexpr int S_BYTES = (A_BYTES + B_BYTES > C_BYTES) ? A_BYTES + B_BYTES : C_BYTES;
    static_assert(A_BYTES % 16 == 0, "alignment of the weight slice");
    __shared__ __attribute__((aligned(16))) char smem[S_BYTES];   // A and B slices; reused by the staged epilogue
    unsigned short (*As)[TB_LD] = (unsigned short (*)[TB_LD]) smem;
    unsigned short (*Bs)[TB_LD] = (unsigned short (*)[TB_LD])(smem + A_BYTES);
    __shared__ uint32_t s_vtx[BM];
    __shared__ float s_scale[BM];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const uint32_t count = *a.count_ptr;
    const uint32_t n_tiles = (count + BM - 1) / BM;
    const uint32_t n0 = blockIdx.y * BN;

    for (uint32_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const uint32_t row0 = tile * BM;
        __syncthreads();
        for (int r = tid; r < BM; r += 256) {
            uint32_t slot = row0 + r;
            uint32_t v = 0;
            float sc = 1.0f;
            if (slot < count) {
                v = a.list[slot];
                if (a.mean) {
                    uint32_t deg = a.in_meta[v].y;
                    sc = 1.0f / (float)(deg > 1u ? deg : 1u);
                }
            }
            s_vtx[r] = v;
            s_scale[r] = sc;
        }
        __syncthreads();

        floatx16 acc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

        uint32_t my_v[NA], my_slot[NA];
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int r = (tid + i * 256) / (T_BK / 4);
            my_v[i] = s_vtx[r];
            my_slot[i] = min(row0 + r, count - 1u);
        }
        const uint32_t c4a = (tid % (T_BK / 4)) * 4;

        floatx4 ra[STAGES][NA], rq[TWO ? STAGES : 1][TWO ? NA : 1];
        uintx4 rb[NB];
#pragma unroll
        for (int i = 0; i < NB; ++i) {                     // weights first, as in every step of the loop
            const int idx = tid + i * 256;
            const int n = idx / 4, kc = (idx % 4) * 8;
            rb[i] = *(const uintx4 *)(a.Wt + (size_t)(n0 + n) * a.wt_ld + kc);
        }
#pragma unroll
        for (int st = 0; st < STAGES; ++st)
#pragma unroll
            for (int i = 0; i < NA; ++i) {
                floatx4 q = (floatx4)(0.0f);
                fetch_raw<MODE, STORE>(a, my_v[i], my_slot[i], (uint32_t)st * T_BK + c4a, ra[st][i], q);
                if constexpr (TWO) rq[st][i] = q;
            }
        __builtin_amdgcn_sched_barrier(0);

        for (uint32_t kbase = 0; kbase < a.Kpad; kbase += STAGES * T_BK) {    // staging registers rotate by unrolling
#pragma unroll
          for (int s = 0; s < STAGES; ++s) {
            const uint32_t k0 = kbase + s * T_BK;
            if (k0 >= a.Kpad) break;
            __syncthreads();
#pragma unroll
            for (int i = 0; i < NA; ++i) {
                const int r = (tid + i * 256) / (T_BK / 4);
                floatx4 q = (floatx4)(0.0f);
                if constexpr (TWO) q = rq[s][i];
                const floatx4 val = finish_raw<MODE, STORE>(a, ra[s][i], q, k0 + c4a, s_scale[r]);
                uint2 pk;
                pk.x = pack_bf16x2(val.x, val.y);
                pk.y = pack_bf16x2(val.z, val.w);
                *(uint2 *)&As[r][c4a] = pk;
            }
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                const int idx = tid + i * 256;
                const int n = idx / 4, kc = (idx % 4) * 8;
                *(uintx4 *)&Bs[n][kc] = rb[i];
            }
            __syncthreads();
            {
                const uint32_t kb = min(k0 + T_BK, a.Kpad - T_BK);
#pragma unroll
                for (int i = 0; i < NB; ++i) {
                    const int idx = tid + i * 256;
                    const int n = idx / 4, kc = (idx % 4) * 8;
                    rb[i] = *(const uintx4 *)(a.Wt + (size_t)(n0 + n) * a.wt_ld + kb + kc);
                }
            }
            {
                const uint32_t kn = k0 + STAGES * T_BK + c4a;
#pragma unroll
                for (int i = 0; i < NA; ++i) {
                    floatx4 q = (floatx4)(0.0f);
                    fetch_raw<MODE, STORE>(a, my_v[i], my_slot[i], kn, ra[s][i], q);
                    if constexpr (TWO) rq[s][i] = q;
                }
            }
            __builtin_amdgcn_sched_barrier(0);             // requests stay above the matrix-core work
#pragma unroll
            for (int kh = 0; kh < 2; ++kh) {
                const int ko = kh * 16 + (lane >> 5) * 8;
                bf16x8 av[TM], bv[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    av[i] = __builtin_bit_cast(bf16x8, *(const uintx4 *)&As[(wm * TM + i) * 32 + (lane & 31)][ko]);
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    bv[j] = __builtin_bit_cast(bf16x8, *(const uintx4 *)&Bs[(wn * TN + j) * 32 + (lane & 31)][ko]);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i], bv[j], acc[i][j], 0, 0, 0);
            }
          }
        }
        epilogue_staged<TM, TN, BM, BN, true>(a, acc, (float *)smem, s_vtx, s_scale, row0, count, n0, wm, wn, tid);
    }
}

// narrow: few rows expected. One workgroup then covers 128 rows x 64 columns and the columns are
// spread over blockIdx.y, which shortens the serial chain of matrix-core work per tile fourfold.
// The grid holds about one workgroup per expected tile (a grid-stride loop covers any excess):
// workgroups that start at different times do not all sit in their memory phase at once, which a
// grid of resident, persistent workgroups does.
static uint32_t tile_grid(const ripple_ctx *c, uint32_t rows_hint, uint32_t bm, uint32_t floor_wg) {
    const uint64_t want = ((uint64_t)rows_hint + rows_hint / 4) / bm + 1;
    const uint64_t cap = (uint64_t)c->n_cap / bm + 1;
    return (uint32_t)std::max<uint64_t>(floor_wg, std::min(want, cap));
}

template <int MODE>
static void launch_bf16(ripple_ctx *c, const TArgs &a, bool narrow, uint32_t rows_hint) {
    if (a.Npad >= 256 && !narrow) {
        hipLaunchKernelGGL((k_transform_bf16<1, 4, 2, 2, 3, MODE>), dim3(tile_grid(c, rows_hint, 64, c->n_cu * 2), a.Npad / 256),
                           dim3(256), 0, c->stream, a);
    } else if (a.Npad == 128 && !narrow) {
        hipLaunchKernelGGL((k_transform_bf16<2, 2, 2, 2, 3, MODE>), dim3(tile_grid(c, rows_hint, 128, c->n_cu * 2), 1), dim3(256), 0,
                           c->stream, a);
    } else {
        hipLaunchKernelGGL((k_transform_bf16<4, 1, 1, 2, 3, MODE>),
                           dim3(tile_grid(c, rows_hint, 128, narrow ? c->n_cu : c->n_cu * 2), a.Npad / 64), dim3(256), 0, c->stream, a);
    }
}

// fp32 embeddings on the bf16 matrix cores: every fp32 number is the exact sum of three bf16 numbers
// (its leading 8 significant bits, the next 8, the last 8), so a product a b is the sum of nine bf16
// products; the six largest (a1 b1, a1 b2, a2 b1, a2 b2, a1 b3, a3 b1) are kept, each exact in the
// fp32 accumulator, and what is dropped is below 2^-24 |a b|. Six bf16 products cost 3/8 of one fp32
// product on this chip (the bf16 rate is sixteen times the fp32 rate), which leaves the kernel bound by
// the gathered rows rather than by the matrix cores. Rows are split as they enter LDS, the weights
// come from three transposed bf16 planes made when the model is loaded.
__device__ __forceinline__ void split3(float a, float &a1, float &a2, float &a3) {
    a1 = __uint_as_float(__float_as_uint(a) & 0xFFFF0000u);
    const float r = a - a1;                                   // exact: the low 16 bits of the significand
    a2 = __uint_as_float(__float_as_uint(r) & 0xFFFF0000u);
    a3 = r - a2;                                              // exact, at most 8 significant bits
}
__device__ __forceinline__ uint32_t pack_hi16(float lo, float hi) {       // the two values are bf16-representable
    return (__float_as_uint(lo) >> 16) | (__float_as_uint(hi) & 0xFFFF0000u);
}

template <int WAVES_M, int WAVES_N, int TM, int TN, int STAGES, int MODE>
__global__ __launch_bounds__(256, 2) void k_transform_split(TArgs a) {
    constexpr int STORE = 0;
    constexpr int BM = WAVES_M * TM * 32, BN = WAVES_N * TN * 32;
    constexpr int NA = BM / 32, NB = BN / 64;              // per thread per slice: float4 of A, 16-byte chunks of B per plane
    constexpr bool TWO = (MODE == 2);
    constexpr int A_BYTES = BM * TB_LD * 2, B_BYTES = BN * TB_LD * 2, C_BYTES = BM * (BN + 4) * 4;
    constexpr int PB = 3;                                  // weight planes
    constexpr int S_BYTES = (3 * A_BYTES + PB * B_BYTES > C_BYTES) ? 3 * A_BYTES + PB * B_BYTES : C_BYTES;
    static_assert(A_BYTES % 16 == 0 && B_BYTES % 16 == 0, "alignment of the planes");
    __shared__ __attribute__((aligned(16))) char smem[S_BYTES];   // three A and three B planes; reused by the staged epilogue
    typedef unsigned short (*plane_t)[TB_LD];
    plane_t As[3], Bs[PB];
#pragma unroll
    for (int p = 0; p < 3; ++p) As[p] = (plane_t)(smem + p * A_BYTES);
#pragma unroll
    for (int p = 0; p < PB; ++p) Bs[p] = (plane_t)(smem + 3 * A_BYTES + p * B_BYTES);
    __shared__ uint32_t s_vtx[BM];
    __shared__ float s_scale[BM];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const uint32_t count = *a.count_ptr;
    const uint32_t n_tiles = (count + BM - 1) / BM;
    const uint32_t n0 = blockIdx.y * BN;

    for (uint32_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const uint32_t row0 = tile * BM;
        __syncthreads();
        for (int r = tid; r < BM; r += 256) {
            uint32_t slot = row0 + r;
            uint32_t v = 0;
            float sc = 1.0f;
            if (slot < count) {
                v = a.list[slot];
                if (a.mean) {
                    uint32_t deg = a.in_meta[v].y;
                    sc = 1.0f / (float)(deg > 1u ? deg : 1u);
                }
            }
            s_vtx[r] = v;
            s_scale[r] = sc;
        }
        __syncthreads();

        floatx16 acc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

        uint32_t my_v[NA], my_slot[NA];
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int r = (tid + i * 256) / (T_BK / 4);
            my_v[i] = s_vtx[r];
            my_slot[i] = min(row0 + r, count - 1u);
        }
        const uint32_t c4a = (tid % (T_BK / 4)) * 4;

        floatx4 ra[STAGES][NA], rq[TWO ? STAGES : 1][TWO ? NA : 1];
        uintx4 rb[PB][NB];
#pragma unroll
        for (int p = 0; p < PB; ++p)
#pragma unroll
            for (int i = 0; i < NB; ++i) {                 // weights first, as in every step of the loop
                const int idx = tid + i * 256;
                const int n = idx / 4, kc = (idx % 4) * 8;
                rb[p][i] = *(const uintx4 *)(a.Ws + p * a.ws_plane + (size_t)(n0 + n) * a.wt_ld + kc);
            }
#pragma unroll
        for (int st = 0; st < STAGES; ++st)
#pragma unroll
            for (int i = 0; i < NA; ++i) {
                floatx4 q = (floatx4)(0.0f);
                fetch_raw<MODE, STORE>(a, my_v[i], my_slot[i], (uint32_t)st * T_BK + c4a, ra[st][i], q);
                if constexpr (TWO) rq[st][i] = q;
            }
        __builtin_amdgcn_sched_barrier(0);

        for (uint32_t kbase = 0; kbase < a.Kpad; kbase += STAGES * T_BK) {    // staging registers rotate by unrolling
#pragma unroll
          for (int s = 0; s < STAGES; ++s) {
            const uint32_t k0 = kbase + s * T_BK;
            if (k0 >= a.Kpad) break;
            __syncthreads();
#pragma unroll
            for (int i = 0; i < NA; ++i) {
                const int r = (tid + i * 256) / (T_BK / 4);
                floatx4 q = (floatx4)(0.0f);
                if constexpr (TWO) q = rq[s][i];
                const floatx4 val = finish_raw<MODE, STORE>(a, ra[s][i], q, k0 + c4a, s_scale[r]);
                float x1[4], x2[4], x3[4];
                split3(val.x, x1[0], x2[0], x3[0]);
                split3(val.y, x1[1], x2[1], x3[1]);
                split3(val.z, x1[2], x2[2], x3[2]);
                split3(val.w, x1[3], x2[3], x3[3]);
                *(uint2 *)&As[0][r][c4a] = make_uint2(pack_hi16(x1[0], x1[1]), pack_hi16(x1[2], x1[3]));
                *(uint2 *)&As[1][r][c4a] = make_uint2(pack_hi16(x2[0], x2[1]), pack_hi16(x2[2], x2[3]));
                *(uint2 *)&As[2][r][c4a] = make_uint2(pack_hi16(x3[0], x3[1]), pack_hi16(x3[2], x3[3]));
            }
#pragma unroll
            for (int p = 0; p < PB; ++p)
#pragma unroll
                for (int i = 0; i < NB; ++i) {
                    const int idx = tid + i * 256;
                    const int n = idx / 4, kc = (idx % 4) * 8;
                    *(uintx4 *)&Bs[p][n][kc] = rb[p][i];
                }
            __syncthreads();
            {
                const uint32_t kb = min(k0 + T_BK, a.Kpad - T_BK);
#pragma unroll
                for (int p = 0; p < PB; ++p)
#pragma unroll
                    for (int i = 0; i < NB; ++i) {
                        const int idx = tid + i * 256;
                        const int n = idx / 4, kc = (idx % 4) * 8;
                        rb[p][i] = *(const uintx4 *)(a.Ws + p * a.ws_plane + (size_t)(n0 + n) * a.wt_ld + kb + kc);
                    }
            }
            {
                const uint32_t kn = k0 + STAGES * T_BK + c4a;
#pragma unroll
                for (int i = 0; i < NA; ++i) {
                    floatx4 q = (floatx4)(0.0f);
                    fetch_raw<MODE, STORE>(a, my_v[i], my_slot[i], kn, ra[s][i], q);
                    if constexpr (TWO) rq[s][i] = q;
                }
            }
            __builtin_amdgcn_sched_barrier(0);             // requests stay above the matrix-core work
#pragma unroll
            for (int kh = 0; kh < 2; ++kh) {
                const int ko = kh * 16 + (lane >> 5) * 8;
                bf16x8 av[3][TM];
#pragma unroll
                for (int p = 0; p < 3; ++p)
#pragma unroll
                    for (int i = 0; i < TM; ++i)
                        av[p][i] = __builtin_bit_cast(bf16x8, *(const uintx4 *)&As[p][(wm * TM + i) * 32 + (lane & 31)][ko]);
#pragma unroll
                for (int j = 0; j < TN; ++j) {               // one column block's three planes at a time (registers)
                    bf16x8 bv[PB];
#pragma unroll
                    for (int p = 0; p < PB; ++p)
                        bv[p] = __builtin_bit_cast(bf16x8, *(const uintx4 *)&Bs[p][(wn * TN + j) * 32 + (lane & 31)][ko]);
#pragma unroll
                    for (int i = 0; i < TM; ++i) {           // smallest terms first
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[2][i], bv[0], acc[i][j], 0, 0, 0);
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[0][i], bv[2], acc[i][j], 0, 0, 0);
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[1][i], bv[1], acc[i][j], 0, 0, 0);
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[1][i], bv[0], acc[i][j], 0, 0, 0);
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[0][i], bv[1], acc[i][j], 0, 0, 0);
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[0][i], bv[0], acc[i][j], 0, 0, 0);
                    }
                }
            }
          }
        }
        epilogue_staged<TM, TN, BM, BN, false>(a, acc, (float *)smem, s_vtx, s_scale, row0, count, n0, wm, wn, tid);
    }
}

template <int MODE>
static void launch_split(ripple_ctx *c, const TArgs &a, bool narrow, uint32_t rows_hint) {
    if (a.Npad >= 256 && !narrow) {
        hipLaunchKernelGGL((k_transform_split<1, 4, 2, 2, 3, MODE>), dim3(tile_grid(c, rows_hint, 64, c->n_cu * 2), a.Npad / 256),
                           dim3(256), 0, c->stream, a);
    } else if (a.Npad == 128 && !narrow) {
        hipLaunchKernelGGL((k_transform_split<2, 2, 2, 2, 3, MODE>), dim3(tile_grid(c, rows_hint, 128, c->n_cu * 2), 1), dim3(256), 0,
                           c->stream, a);
    } else {
        hipLaunchKernelGGL((k_transform_split<4, 1, 1, 2, 3, MODE>),
                           dim3(tile_grid(c, rows_hint, 128, narrow ? c->n_cu : c->n_cu * 2), a.Npad / 64), dim3(256), 0, c->stream, a);
    }
}

template <int MODE, int STORE>
static void launch_fast(ripple_ctx *c, const TArgs &a, bool narrow, uint32_t rows_hint) {
    if (rows_hint <= 32 && a.Npad % 128 == 0) {
        // a handful of rows: one 32-row tile, four wavefronts side by side on 32 columns each, so that the
        // chain of dependent matrix-core operations per K step is a quarter of the 128 x 64 tile's
        // (the grid does not follow the hint: workgroups without a tile leave at once, and a set that turns out
        // large still finds the whole chip)
        hipLaunchKernelGGL((k_transform_f32<1, 4, 1, 1, 3, MODE, STORE>), dim3(c->n_cu / 4, a.Npad / 128), dim3(256), 0, c->stream, a);
        return;
    }
    if (rows_hint <= 2048) {                               // few rows: 64 x 64 tiles, one 32 x 32 block per wavefront
        hipLaunchKernelGGL((k_transform_f32<2, 2, 1, 1, 3, MODE, STORE>), dim3(c->n_cu / 4, a.Npad / 64),
                           dim3(256), 0, c->stream, a);
        return;
    }
    if (a.Npad == 96) {                                    // [W_self | W_neigh] of a narrow layer: three 32-column blocks per wavefront
        hipLaunchKernelGGL((k_transform_f32<4, 1, 1, 3, 3, MODE, STORE>), dim3(tile_grid(c, rows_hint, 128, c->n_cu * 2), 1), dim3(256),
                           0, c->stream, a);
    } else if (a.Npad >= 256 && !narrow) {
        hipLaunchKernelGGL((k_transform_f32<1, 4, 2, 2, 3, MODE, STORE>), dim3(tile_grid(c, rows_hint, 64, c->n_cu * 2), a.Npad / 256),
                           dim3(256), 0, c->stream, a);
    } else if (a.Npad == 128 && !narrow) {
        hipLaunchKernelGGL((k_transform_f32<2, 2, 2, 2, 3, MODE, STORE>), dim3(tile_grid(c, rows_hint, 128, c->n_cu * 2), 1), dim3(256),
                           0, c->stream, a);
    } else {
        hipLaunchKernelGGL((k_transform_f32<4, 1, 1, 2, 3, MODE, STORE>),
                           dim3(tile_grid(c, rows_hint, 128, narrow ? c->n_cu : c->n_cu * 2), a.Npad / 64), dim3(256), 0, c->stream, a);
    }
}

static void launch_t(ripple_ctx *c, const TArgs &a, bool vec_ok, uint32_t rows_hint) {
    const bool narrow = rows_hint < 64u * c->n_cu;
    if (rp_launch_stream(c, a, rows_hint)) return;
    const uint32_t gx = c->n_cu * 2;
    if (!vec_ok || a.K < 4) {
        if (a.Npad >= 256) hipLaunchKernelGGL((k_transform_generic<1, 4>), dim3(gx, a.Npad / 256), dim3(256), 0, c->stream, a);
        else if (a.Npad == 128) hipLaunchKernelGGL((k_transform_generic<2, 2>), dim3(gx, 1), dim3(256), 0, c->stream, a);
        else hipLaunchKernelGGL((k_transform_generic<4, 1>), dim3(gx, 1), dim3(256), 0, c->stream, a);
        return;
    }
#define T_CASE(M)                                            \
    case M:                                                  \
        if (a.store && a.Wt) launch_bf16<M>(c, a, narrow, rows_hint);   \
        else if (a.store) launch_fast<M, 1>(c, a, narrow, rows_hint);   \
        else if (a.Ws) launch_split<M>(c, a, narrow, rows_hint);        \
        else launch_fast<M, 0>(c, a, narrow, rows_hint);                \
        break;
    switch (a.a_mode) {
        T_CASE(0)
        T_CASE(1)
        T_CASE(2)
        T_CASE(4)
    default:
        if (a.store) launch_fast<3, 1>(c, a, narrow, rows_hint);   // compact fp32 rows; the storage type only shapes the epilogue
        else if (a.Ws) launch_split<3>(c, a, narrow, rows_hint);
        else launch_fast<3, 0>(c, a, narrow, rows_hint);
        break;
    }
#undef T_CASE
}

static TArgs base_args(ripple_ctx *c, uint32_t l, const uint32_t *list, const uint32_t *count_d) {
    const LayerDev &ly = c->layers[l - 1];
    TArgs a;
    a.list = list;
    a.count_ptr = count_d;
    a.Hprev = c->H[l - 1];
    a.X = c->X[l];
    a.in_meta = c->in_meta;
    a.mean = (ly.agg == RIPPLE_AGG_MEAN) ? 1 : 0;
    a.one_plus_eps = 1.0f + ly.eps;
    a.d_in = ly.d_in;
    a.tmp_in = nullptr;
    a.tmp_ld = 0;
    a.store = c->store;
    a.Hout = c->H[l];
    a.D = nullptr;
    a.d_old = 0;
    a.tmp_out = nullptr;
    a.tmp_out_ld = 0;
    a.split_col = 0;
    a.N1 = ly.d_out;
    a.tmp_out2 = nullptr;
    a.tmp_out2_ld = 0;
    a.addend = nullptr;
    a.addend_scaled = 1;
    a.addend2 = nullptr;
    a.den = nullptr;
    a.range_rows = &c->ctr->range_rows;
    a.a_mode = 0;
    a.out_mode = 1;
    a.act = 0;
    a.W = ly.W0;
    a.Wt = (c->store && c->opt_bf16_mfma) ? ly.W0h : nullptr;   // bf16 storage: bf16 matrix cores
    a.wt_ld = ly.K0pad;
    a.Ws = ly.W0s;                                 // fp32 storage with split products, else null
    a.ws_plane = (size_t)ly.N0pad * ly.K0pad;
    a.bias = ly.b0;
    a.K = ly.K;
    a.Kpad = ly.K0pad;
    a.N = ly.d_out;
    a.Npad = ly.N0pad;
    return a;
}

// Project-first layers: P[v] = H^{l-1}[v] W_neigh for the listed vertices, no bias, no activation.
//   bootstrap: into the layer's T (what every vertex has sent: the aggregates are then summed from it)
//   otherwise: into c->PD, from where rp_launch_messages turns the rows into this hop's messages
void rp_launch_project(ripple_ctx *c, uint32_t l, const uint32_t *list, const uint32_t *count_d, bool bootstrap) {
    const LayerDev &ly = c->layers[l - 1];
    TArgs a = base_args(c, l, list, count_d);
    a.mean = 0;
    a.W = ly.Wn;
    a.Wt = nullptr;                                // messages are differences of such products: fp32 path also for bf16 rows
    a.Ws = ly.Wns;
    a.wt_ld = ly.Wns_ld;
    a.ws_plane = (size_t)ly.N0pad * ly.Wns_ld;
    a.bias = ly.bzero;
    a.K = ly.d_in;
    a.Kpad = rp_round_up(ly.d_in, 32);
    a.act = RIPPLE_ACT_NONE;
    a.tmp_out = bootstrap ? ly.T : c->PD;
    a.tmp_out_ld = bootstrap ? ly.d_out : c->pd_ld;
    a.Hout = nullptr;
    a.out_mode = 2;
    a.a_mode = 4;
    launch_t(c, a, ly.d_in % 4 == 0, bootstrap ? c->n_cap : rp_rows_hint(c, l - 1));
}

// Layers handled project-first that also cache their self term: both products of H^{l-1}[v], with W_self (into PS)
// and with W_neigh (into T at the bootstrap, else into c->PD), from one pass over the rows, against the
// layer's combined weight matrix [W_self | W_neigh] (second block from column 64 on).
bool rp_has_project_both(const ripple_ctx *c, uint32_t l) { return c->layers[l - 1].Wc != nullptr; }

void rp_launch_project_both(ripple_ctx *c, uint32_t l, const uint32_t *list, const uint32_t *count_d, bool bootstrap) {
    const LayerDev &ly = c->layers[l - 1];
    TArgs a = base_args(c, l, list, count_d);
    a.mean = 0;
    a.W = ly.Wc;
    a.Wt = nullptr;
    a.Ws = nullptr;
    a.bias = ly.bzero_c;
    a.K = ly.d_in;
    a.Kpad = rp_round_up(ly.d_in, 32);
    a.N = 64 + ly.d_out;
    a.Npad = 128;
    a.act = RIPPLE_ACT_NONE;
    a.a_mode = 4;
    a.out_mode = 2;
    a.Hout = nullptr;
    a.tmp_out = ly.PS;
    a.tmp_out_ld = ly.d_out;
    a.split_col = 64;
    a.N1 = ly.d_out;
    a.tmp_out2 = bootstrap ? ly.T : c->PD;
    a.tmp_out2_ld = bootstrap ? ly.d_out : c->pd_ld;
    const uint32_t hint = bootstrap ? c->n_cap : rp_rows_hint(c, l - 1);
    if (rp_launch_project_both_stream(c, l, list, count_d, a.tmp_out2, a.tmp_out2_ld, hint)) return;
    if (ly.Wc96 && hint > 2048) {                  // many rows: the products are bound by the matrix cores, 96 columns instead of 128
        a.W = ly.Wc96;
        a.N = 48 + ly.d_out;
        a.Npad = 96;
        a.split_col = 48;
    }
    launch_t(c, a, true, hint);
}

// Attention layer l: P[v] = H^{l-1}[v] W0 for the listed vertices (fp32, no bias, no activation).
void rp_launch_gat_project(ripple_ctx *c, uint32_t l, const uint32_t *list, const uint32_t *count_d) {
    const LayerDev &ly = c->layers[l - 1];
    TArgs a = base_args(c, l, list, count_d);
    a.mean = 0;
    a.Wt = nullptr;
    a.bias = ly.bzero;
    a.act = RIPPLE_ACT_NONE;
    a.a_mode = 4;
    a.out_mode = 2;
    a.tmp_out = ly.P;
    a.tmp_out_ld = ly.d_out;
    a.Hout = nullptr;
    launch_t(c, a, ly.d_in % 4 == 0, (list == c->all_list) ? c->n_cap : rp_rows_hint(c, l - 1));
}

// Cached self term of layer l: PS[v] = H^{l-1}[v] W_self for the listed vertices (fp32, no bias).
void rp_launch_self_project(ripple_ctx *c, uint32_t l, const uint32_t *list, const uint32_t *count_d) {
    const LayerDev &ly = c->layers[l - 1];
    TArgs a = base_args(c, l, list, count_d);
    a.mean = 0;
    a.W = ly.W0;                                   // W_self: the first d_in rows (the kernel zeroes k >= K)
    a.Wt = nullptr;
    a.bias = ly.bzero;
    a.K = ly.d_in;
    a.Kpad = rp_round_up(ly.d_in, 32);
    a.act = RIPPLE_ACT_NONE;
    a.a_mode = 4;
    a.out_mode = 2;
    a.tmp_out = ly.PS;
    a.tmp_out_ld = ly.d_out;
    a.Hout = nullptr;
    launch_t(c, a, ly.d_in % 4 == 0, (list == c->all_list) ? c->n_cap : rp_rows_hint(c, l - 1));
}

// Re-apply layer l (1-based) to the vertices in `list` (count on the device).
// emit_delta: write D^l (into the ping-pong buffer of parity l) for the next hop.
void rp_launch_transform(ripple_ctx *c, uint32_t l, const uint32_t *list, const uint32_t *count_d, bool emit_delta) {
    const LayerDev &ly = c->layers[l - 1];
    TArgs a = base_args(c, l, list, count_d);
    a.D = emit_delta ? c->D[l & 1] : nullptr;
    a.d_old = rp_layer_mono(c, l + 1) ? 1 : 0;
    a.a_mode = (ly.self_mode == RIPPLE_SELF_NONE) ? 0 : (ly.self_mode == RIPPLE_SELF_CONCAT ? 1 : 2);
    const bool vec_in = (ly.d_in % 4 == 0);
    // expected row count: the previous batch's (bootstrap passes the list of all live vertices)
    const uint32_t hint = (list == c->all_list) ? c->n_cap : rp_rows_hint(c, l);
    if (ly.agg == RIPPLE_AGG_ATTN) {             // h = act(numerator / denominator + b): no product left per row
        a.addend = c->X[l];
        a.den = ly.den;
        a.act = (int)ly.act_out;
        hipLaunchKernelGGL(k_transform_addend_only, dim3(c->n_cu * 8), dim3(256), 0, c->stream, a);
        return;
    }
    if (ly.proj) {                               // aggregate already multiplied by W_neigh: add it in the epilogue
        a.addend = c->X[l];
        a.act = (int)ly.act_out;
        if (ly.self_mode == RIPPLE_SELF_NONE || ly.selfc) {
            a.addend2 = ly.selfc ? ly.PS : nullptr;
            if (hint >= 65536u && (uint64_t)c->n_cap * a.N < (1ull << 32)) launch_addend_flat(c, a);  // many rows: every lane busy, whatever the row width
            else hipLaunchKernelGGL(k_transform_addend_only, dim3(c->n_cu * 8), dim3(256), 0, c->stream, a);
            return;
        }
        a.a_mode = 4;                            // h_self * W_self: the first d_in rows of W0
        a.K = ly.d_in;
        a.Kpad = rp_round_up(ly.d_in, 32);
        launch_t(c, a, vec_in, hint);
        return;
    }
    if (ly.selfc) {                              // act((x * scale) W_neigh + PS[v] + b)
        a.a_mode = 0;
        a.W = ly.Wn;
        a.Wt = nullptr;
        a.Ws = ly.Wns;
        a.wt_ld = ly.Wns_ld;
        a.ws_plane = (size_t)ly.N0pad * ly.Wns_ld;
        a.K = ly.d_in;
        a.Kpad = rp_round_up(ly.d_in, 32);
        a.addend = ly.PS;
        a.addend_scaled = 0;
        a.act = (int)ly.act_out;
        launch_t(c, a, vec_in, hint);
        return;
    }
    if (ly.d_hidden == 0) {
        a.act = (int)ly.act_out;
        launch_t(c, a, vec_in, hint);
        return;
    }
    // two-stage update: hidden = act_inner(row W0 + b0) -> tmp, then h = act_out(hidden W1 + b1)
    TArgs s1 = a;
    s1.N = ly.d_hidden;
    s1.act = (int)ly.act_inner;
    s1.out_mode = 0;
    s1.tmp_out = c->tmp;
    s1.tmp_out_ld = ly.d_hidden;
    s1.Hout = nullptr;
    s1.D = nullptr;
    launch_t(c, s1, vec_in, hint);
    TArgs s2 = a;
    s2.a_mode = 3;
    s2.tmp_in = c->tmp;
    s2.tmp_ld = ly.d_hidden;
    s2.mean = 0;
    s2.W = ly.W1;
    s2.Wt = nullptr;
    s2.Ws = ly.W1s;
    s2.wt_ld = ly.K1pad;
    s2.ws_plane = (size_t)ly.N1pad * ly.K1pad;
    s2.bias = ly.b1;
    s2.K = ly.d_hidden;
    s2.Kpad = ly.K1pad;
    s2.N = ly.d_out;
    s2.Npad = ly.N1pad;
    s2.act = (int)ly.act_out;
    s2.out_mode = 1;
    launch_t(c, s2, ly.d_hidden % 4 == 0, hint);
}

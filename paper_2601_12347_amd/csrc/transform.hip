// Dirty-row transform (the Compute step of Sec. 3.3 in re-apply form): for every
// vertex v of A_l gather the layer's input row
//     GraphConv  x            GraphSAGE  [h_self | x]        GIN  (1+eps) h_self + x
// (x = X^l[v], divided by the in-degree for mean), multiply by the weight
// matrix on the matrix cores, add the bias, apply the activation, and emit
//     D^l[slot] = h_new - H^l[v],   H^l[v] = h_new
// so that the next hop can forward the delta (Sec. 3.3.3).
//
// Tiling: a workgroup of four wavefronts computes a (WM*64) x (WN*64) output
// tile; each wavefront owns a 64 x 64 block as 2 x 2 MFMA 32x32x2 (fp32)
// accumulators. K is consumed in slices of 32 staged through LDS: the gathered
// rows (A) once per slice, the weight slice (B) from the L2-resident padded
// weight matrix.
#include "common.h"
#include "kernels.h"

typedef float floatx16 __attribute__((ext_vector_type(16)));

struct TArgs {
    const uint32_t *list;          // slot -> vertex id
    const uint32_t *count_ptr;     // number of slots (device)
    int a_mode;                    // 0 x | 1 [h_self | x] | 2 (1+eps) h_self + x | 3 compact rows of tmp_in
    const void *Hprev;
    const float *X;
    const uint2 *in_meta;
    int mean;
    float one_plus_eps;
    uint32_t d_in;
    const float *tmp_in;
    uint32_t tmp_ld;
    const float *W;                // [Kpad x Npad], zero padded
    const float *bias;             // [Npad]
    uint32_t K, Kpad, N, Npad;
    int act;
    int out_mode;                  // 0 write act(z) to tmp_out[slot] | 1 update H, emit delta
    float *tmp_out;
    uint32_t tmp_out_ld;
    void *Hout;
    float *D;                      // compact delta rows [slot x N] or null
    int store;                     // 0 fp32, 1 bf16 embeddings
};

__device__ __forceinline__ float ld_h(const void *H, int store, size_t idx) {
    return store ? __bfloat162float(((const __hip_bfloat16 *)H)[idx]) : ((const float *)H)[idx];
}

__device__ __forceinline__ float load_a1(const TArgs &a, uint32_t v, uint32_t slot, float scale, uint32_t k) {
    if (k >= a.K) return 0.0f;
    switch (a.a_mode) {
    case 0: return a.X[(size_t)v * a.d_in + k] * scale;
    case 1:
        return (k < a.d_in) ? ld_h(a.Hprev, a.store, (size_t)v * a.d_in + k)
                            : a.X[(size_t)v * a.d_in + (k - a.d_in)] * scale;
    case 2: return a.one_plus_eps * ld_h(a.Hprev, a.store, (size_t)v * a.d_in + k) + a.X[(size_t)v * a.d_in + k] * scale;
    default: return a.tmp_in[(size_t)slot * a.tmp_ld + k];
    }
}

__device__ __forceinline__ float4 ld_h4(const void *H, int store, size_t idx) {
    if (store) {
        const ushort4 r = *(const ushort4 *)((const __hip_bfloat16 *)H + idx);
        return make_float4(__uint_as_float((uint32_t)r.x << 16), __uint_as_float((uint32_t)r.y << 16),
                           __uint_as_float((uint32_t)r.z << 16), __uint_as_float((uint32_t)r.w << 16));
    }
    return *(const float4 *)((const float *)H + idx);
}

// four consecutive k (k % 4 == 0); requires d_in % 4 == 0 and tmp_ld % 4 == 0
__device__ __forceinline__ float4 load_a4(const TArgs &a, uint32_t v, uint32_t slot, float scale, uint32_t k) {
    if (k >= a.K) return make_float4(0.f, 0.f, 0.f, 0.f);
    switch (a.a_mode) {
    case 0: {
        float4 x = *(const float4 *)(a.X + (size_t)v * a.d_in + k);
        return make_float4(x.x * scale, x.y * scale, x.z * scale, x.w * scale);
    }
    case 1: {
        if (k < a.d_in) return ld_h4(a.Hprev, a.store, (size_t)v * a.d_in + k);
        float4 x = *(const float4 *)(a.X + (size_t)v * a.d_in + (k - a.d_in));
        return make_float4(x.x * scale, x.y * scale, x.z * scale, x.w * scale);
    }
    case 2: {
        float4 h = ld_h4(a.Hprev, a.store, (size_t)v * a.d_in + k);
        float4 x = *(const float4 *)(a.X + (size_t)v * a.d_in + k);
        const float e = a.one_plus_eps;
        return make_float4(e * h.x + x.x * scale, e * h.y + x.y * scale, e * h.z + x.z * scale, e * h.w + x.w * scale);
    }
    default: return *(const float4 *)(a.tmp_in + (size_t)slot * a.tmp_ld + k);
    }
}

#define T_BK 32

template <int WM, int WN, bool VEC>
__global__ __launch_bounds__(256) void k_transform_f32(TArgs a) {
    constexpr int BM = WM * 64, BN = WN * 64;
    __shared__ float As[BM][T_BK + 1];
    __shared__ float Bs[T_BK][BN];
    __shared__ uint32_t s_vtx[BM];
    __shared__ float s_scale[BM];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const uint32_t count = *a.count_ptr;
    const uint32_t n_tiles = (count + BM - 1) / BM;
    const uint32_t n0 = blockIdx.y * BN;

    for (uint32_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const uint32_t row0 = tile * BM;
        __syncthreads();                                   // previous tile's epilogue has read s_vtx
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

        floatx16 acc[2][2];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

        for (uint32_t k0 = 0; k0 < a.Kpad; k0 += T_BK) {
            // stage A: BM rows x 32 k
            for (int idx = tid; idx < BM * (T_BK / 4); idx += 256) {
                const int r = idx / (T_BK / 4), c4 = (idx % (T_BK / 4)) * 4;
                const uint32_t slot = row0 + r;
                float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
                if (slot < count) {
                    if (VEC) {
                        val = load_a4(a, s_vtx[r], slot, s_scale[r], k0 + c4);
                    } else {
                        val.x = load_a1(a, s_vtx[r], slot, s_scale[r], k0 + c4 + 0);
                        val.y = load_a1(a, s_vtx[r], slot, s_scale[r], k0 + c4 + 1);
                        val.z = load_a1(a, s_vtx[r], slot, s_scale[r], k0 + c4 + 2);
                        val.w = load_a1(a, s_vtx[r], slot, s_scale[r], k0 + c4 + 3);
                    }
                }
                As[r][c4 + 0] = val.x;
                As[r][c4 + 1] = val.y;
                As[r][c4 + 2] = val.z;
                As[r][c4 + 3] = val.w;
            }
            // stage B: 32 k x BN columns of the padded weights
            for (int idx = tid; idx < T_BK * (BN / 4); idx += 256) {
                const int kr = idx / (BN / 4), c4 = (idx % (BN / 4)) * 4;
                const float4 w = *(const float4 *)(a.W + (size_t)(k0 + kr) * a.Npad + n0 + c4);
                *(float4 *)&Bs[kr][c4] = w;
            }
            __syncthreads();
#pragma unroll
            for (int kk = 0; kk < T_BK; kk += 2) {
                const int kq = kk + (lane >> 5);
                const float a0 = As[wm * 64 + (lane & 31)][kq];
                const float a1 = As[wm * 64 + 32 + (lane & 31)][kq];
                const float b0 = Bs[kq][wn * 64 + (lane & 31)];
                const float b1 = Bs[kq][wn * 64 + 32 + (lane & 31)];
                acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
                acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
                acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
                acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
            }
            __syncthreads();
        }

        // epilogue: bias, activation, delta against the stored row, store
#pragma unroll
        for (int sm = 0; sm < 2; ++sm)
#pragma unroll
            for (int sn = 0; sn < 2; ++sn) {
                const uint32_t col = n0 + wn * 64 + sn * 32 + (lane & 31);
                if (col >= a.N) continue;
                const float bias = a.bias[col];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int lr = wm * 64 + sm * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                    const uint32_t slot = row0 + lr;
                    if (slot >= count) continue;
                    float z = acc[sm][sn][r] + bias;
                    if (a.act == RIPPLE_ACT_RELU) z = z > 0.0f ? z : 0.0f;
                    if (a.out_mode == 0) {
                        a.tmp_out[(size_t)slot * a.tmp_out_ld + col] = z;
                    } else {
                        const size_t hidx = (size_t)s_vtx[lr] * a.N + col;
                        float old;
                        if (a.store) {
                            __hip_bfloat16 *h = (__hip_bfloat16 *)a.Hout;
                            old = __bfloat162float(h[hidx]);
                            const __hip_bfloat16 zr = __float2bfloat16(z);
                            z = __bfloat162float(zr);
                            h[hidx] = zr;
                        } else {
                            float *h = (float *)a.Hout;
                            old = h[hidx];
                            h[hidx] = z;
                        }
                        if (a.D) a.D[(size_t)slot * a.N + col] = z - old;
                    }
                }
            }
    }
}

template <bool VEC>
static void launch_t(ripple_ctx *c, const TArgs &a) {
    const uint32_t gx = c->n_cu * 2;
    if (a.Npad >= 256 || a.Npad == 192) {
        dim3 grid(gx, rp_div_up(a.Npad, 256));
        hipLaunchKernelGGL((k_transform_f32<1, 4, VEC>), grid, dim3(256), 0, c->stream, a);
    } else if (a.Npad == 128) {
        dim3 grid(gx, 1);
        hipLaunchKernelGGL((k_transform_f32<2, 2, VEC>), grid, dim3(256), 0, c->stream, a);
    } else {
        dim3 grid(gx, 1);
        hipLaunchKernelGGL((k_transform_f32<4, 1, VEC>), grid, dim3(256), 0, c->stream, a);
    }
}

// Re-apply layer l (1-based) to the vertices in `list` (count on the device).
// emit_delta: write D^l (into the ping-pong buffer of parity l) for the next hop.
void rp_launch_transform(ripple_ctx *c, uint32_t l, const uint32_t *list, const uint32_t *count_d, bool emit_delta) {
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
    a.D = emit_delta ? c->D[l & 1] : nullptr;
    a.tmp_out = nullptr;
    a.tmp_out_ld = 0;
    a.a_mode = (ly.self_mode == RIPPLE_SELF_NONE) ? 0 : (ly.self_mode == RIPPLE_SELF_CONCAT ? 1 : 2);
    const bool vec_in = (ly.d_in % 4 == 0);
    if (ly.d_hidden == 0) {
        a.W = ly.W0;
        a.bias = ly.b0;
        a.K = ly.K;
        a.Kpad = ly.K0pad;
        a.N = ly.d_out;
        a.Npad = ly.N0pad;
        a.act = (int)ly.act_out;
        a.out_mode = 1;
        if (vec_in) launch_t<true>(c, a);
        else launch_t<false>(c, a);
        return;
    }
    // two-stage update: hidden = act_inner(row W0 + b0) -> tmp, then h = act_out(hidden W1 + b1)
    TArgs s1 = a;
    s1.W = ly.W0;
    s1.bias = ly.b0;
    s1.K = ly.K;
    s1.Kpad = ly.K0pad;
    s1.N = ly.d_hidden;
    s1.Npad = ly.N0pad;
    s1.act = (int)ly.act_inner;
    s1.out_mode = 0;
    s1.tmp_out = c->tmp;
    s1.tmp_out_ld = ly.d_hidden;
    s1.Hout = nullptr;
    s1.D = nullptr;
    if (vec_in) launch_t<true>(c, s1);
    else launch_t<false>(c, s1);
    TArgs s2 = a;
    s2.a_mode = 3;
    s2.tmp_in = c->tmp;
    s2.tmp_ld = ly.d_hidden;
    s2.mean = 0;
    s2.W = ly.W1;
    s2.bias = ly.b1;
    s2.K = ly.d_hidden;
    s2.Kpad = ly.K1pad;
    s2.N = ly.d_out;
    s2.Npad = ly.N1pad;
    s2.act = (int)ly.act_out;
    s2.out_mode = 1;
    if (ly.d_hidden % 4 == 0) launch_t<true>(c, s2);
    else launch_t<false>(c, s2);
}

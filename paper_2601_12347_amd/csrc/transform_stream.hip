#include "transform_args.h"
#include "kernels.h"

typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));

// Streaming variant for the shape that dominates large batches: x W with K = N = 256 (x = X^l[v], scaled for mean), fp32
// rows, H updated in place (ADD: plus an unscaled cached row; DELTA: the delta row is written too). Workgroups are
// persistent and nothing of a tile waits for memory on its own: the finished tile's accumulators are parked in a second
// set of registers and leave for memory chunk by chunk during the K steps of the next tile (the rows they are added to
// are requested one step before they are used, and each lane stores straight from its accumulator layout: 32 lanes
// cover one 128-byte line of a row), and the first slices of the next tile's rows are requested during the last steps
// of the current one. The matrix cores then only ever wait for the barriers around the LDS slices.
template <bool ADD, bool DELTA>
__global__ __launch_bounds__(256, 2) void k_transform_stream(TArgs a) {
    constexpr int BM = 64, BN = 256, KS = 8, STAGES = 2, NA = 2, NB = 8;
    __shared__ __attribute__((aligned(16))) float As[BM][T_BK + 1];
    __shared__ __attribute__((aligned(16))) float Bs[T_BK][BN];
    __shared__ uint32_t s_vtx[2][BM];

    const int tid = threadIdx.x, lane = tid & 63, wn = tid >> 6;
    const uint32_t count = *a.count_ptr;
    const uint32_t n_tiles = (count + BM - 1) / BM;
    uint32_t tile = blockIdx.x;
    if (tile >= n_tiles) return;

    const uint32_t c4a = (tid % (T_BK / 4)) * 4;
    const int r_own = tid / (T_BK / 4);                    // this thread stages rows r_own and r_own + 32 of every slice
    const float *Xc = a.X + c4a;
    float bias[2];
#pragma unroll
    for (int sn = 0; sn < 2; ++sn) bias[sn] = a.bias[wn * 64 + sn * 32 + (lane & 31)];

    uint32_t v_cur[NA], v_nxt[NA];
    float sc_cur[NA], sc_nxt[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        v_cur[i] = a.list[min(tile * BM + r_own + i * 32, count - 1u)];   // rows past the end repeat the last one; never stored
        v_nxt[i] = v_cur[i];
    }
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const uint32_t deg = a.in_meta[v_cur[i]].y;
        sc_cur[i] = a.mean ? 1.0f / (float)(deg > 1u ? deg : 1u) : 1.0f;
        sc_nxt[i] = sc_cur[i];
    }

    if (c4a == 0) {                                        // nothing is parked yet: its row ids only have to be valid
#pragma unroll
        for (int i = 0; i < NA; ++i) s_vtx[1][r_own + i * 32] = v_cur[i];
    }

    floatx4 ra[STAGES][NA], rb[NB];
    // The weights are read through a buffer descriptor: a thread's eight 16-byte pieces of a slice lie 4 KB apart and
    // the slices 32 KB, all of it constants beside one offset register (as flat addresses the compiler keeps
    // sixty-four 64-bit pointers alive, which no register file holds).
    const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc((void *)a.W, 0, 256 * 256 * 4, 0x00020000);
    const uint32_t wo = (uint32_t)tid * 16u;
#pragma unroll
    for (int i = 0; i < NB; ++i) rb[i] = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(wres, wo, i * 4096, 0));
#pragma unroll
    for (int st = 0; st < STAGES; ++st)
#pragma unroll
        for (int i = 0; i < NA; ++i) ra[st][i] = *(const floatx4 *)(Xc + (size_t)v_cur[i] * 256 + st * T_BK);

    floatx16 acc[2][2], accp[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                acc[i][j][r] = 0.0f;
                accp[i][j][r] = 0.0f;
            }
    uint32_t prev_rows = 0;                                // valid rows of the parked tile (0: nothing parked)
    int par = 0;
    float pa[8], po[8];                                    // addend and old values of the chunk in flight
    uint32_t pv[4];                                        // the vertices of its four rows
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        pa[e] = 0.0f;
        po[e] = 0.0f;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) pv[j] = 0;
    const uint32_t col0 = wn * 64 + (lane & 31);

    // chunk c of a parked tile: accumulator elements 4 (c & 3) .. + 3 of blocks [c >> 2][0] and [c >> 2][1]
    auto chunk_request = [&](int c, const uint32_t *vtx) {
#pragma unroll
        for (int j = 0; j < 4; ++j) pv[j] = vtx[(c >> 2) * 32 + (c & 3) * 8 + (lane >> 5) * 4 + j];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const size_t h = (size_t)pv[e & 3] * 256 + col0 + (e >> 2) * 32;
            if (ADD) pa[e] = a.addend[h];
            if (DELTA) po[e] = ((const float *)a.Hout)[h];
        }
    };
    auto chunk_finish = [&](int c, uint32_t rows) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int sn = e >> 2, j = e & 3;
            const int lr = (c >> 2) * 32 + (c & 3) * 8 + (lane >> 5) * 4 + j;
            float z = accp[c >> 2][sn][(c & 3) * 4 + j] + bias[sn] + (ADD ? pa[e] : 0.0f);
            if (a.act == RIPPLE_ACT_RELU) z = z > 0.0f ? z : 0.0f;
            if ((uint32_t)lr < rows) {
                const size_t h = (size_t)pv[j] * 256 + col0 + sn * 32;
                ((float *)a.Hout)[h] = z;
                if (DELTA) a.D[h] = a.d_old ? po[e] : z - po[e];
            }
        }
    };

    for (;;) {
        const uint32_t tile_n = tile + gridDim.x;
#pragma unroll
        for (int i = 0; i < NA; ++i) v_nxt[i] = a.list[min(tile_n * BM + r_own + i * 32, count - 1u)];
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            __syncthreads();                               // the matrix cores are done with the previous slice
#pragma unroll
            for (int i = 0; i < NA; ++i) {
                const floatx4 val = ra[s % STAGES][i] * sc_cur[i];
                float *dst = &As[r_own + i * 32][c4a];
                dst[0] = val.x;
                dst[1] = val.y;
                dst[2] = val.z;
                dst[3] = val.w;
            }
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                const int idx = tid + i * 256;
                *(floatx4 *)&Bs[idx / (BN / 4)][(idx % (BN / 4)) * 4] = rb[i];
            }
            if (s == 0 && c4a == 0) {
#pragma unroll
                for (int i = 0; i < NA; ++i) s_vtx[par][r_own + i * 32] = v_cur[i];
            }
            __syncthreads();
            {                                              // weights of the next slice (after the last: slice 0 again, for the next tile)
#pragma unroll
                for (int i = 0; i < NB; ++i)
                    rb[i] = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(wres, wo, ((s + 1) % KS) * T_BK * BN * 4 + i * 4096, 0));
            }
            if (s == 2) {                                  // the next tile's scale factors
#pragma unroll
                for (int i = 0; i < NA; ++i) {
                    const uint32_t deg = a.in_meta[v_nxt[i]].y;
                    sc_nxt[i] = a.mean ? 1.0f / (float)(deg > 1u ? deg : 1u) : 1.0f;
                }
            }
#pragma unroll
            for (int i = 0; i < NA; ++i) {                 // rows of the slice STAGES steps ahead: this tile's, then the next tile's
                const uint32_t v = (s + STAGES < KS) ? v_cur[i] : v_nxt[i];
                ra[s % STAGES][i] = *(const floatx4 *)(Xc + (size_t)v * 256 + ((s + STAGES) % KS) * T_BK);
            }
            // the parked tile: finish the chunk requested one step ago, request the next one
            if (s > 0) chunk_finish(s - 1, prev_rows);
            chunk_request(s, s_vtx[par ^ 1]);
            __builtin_amdgcn_sched_barrier(0);
            float av[2][2], bv[2][2];
#pragma unroll
            for (int i = 0; i < 2; ++i) av[0][i] = As[i * 32 + (lane & 31)][lane >> 5];
#pragma unroll
            for (int j = 0; j < 2; ++j) bv[0][j] = Bs[lane >> 5][(wn * 2 + j) * 32 + (lane & 31)];
#pragma unroll
            for (int kk = 0; kk < T_BK; kk += 2) {
                const int cur = (kk >> 1) & 1, nxt = cur ^ 1;
                if (kk + 2 < T_BK) {
                    const int kq = kk + 2 + (lane >> 5);
#pragma unroll
                    for (int i = 0; i < 2; ++i) av[nxt][i] = As[i * 32 + (lane & 31)][kq];
#pragma unroll
                    for (int j = 0; j < 2; ++j) bv[nxt][j] = Bs[kq][(wn * 2 + j) * 32 + (lane & 31)];
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[cur][i], bv[cur][j], acc[i][j], 0, 0, 0);
            }
            if (s == KS - 1) chunk_finish(KS - 1, prev_rows);
        }
        // park the tile, move on
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                accp[i][j] = acc[i][j];
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
            }
        prev_rows = min((uint32_t)BM, count - tile * BM);
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            v_cur[i] = v_nxt[i];
            sc_cur[i] = sc_nxt[i];
        }
        par ^= 1;
        tile = tile_n;
        if (tile >= n_tiles) break;
    }
    __syncthreads();                                       // s_vtx[par ^ 1] of the last tile is complete since its first step
#pragma unroll
    for (int c = 0; c < KS; ++c) {
        chunk_request(c, s_vtx[par ^ 1]);
        chunk_finish(c, prev_rows);
    }
}

// x W with K = N = 256 on fp32 rows, H updated in place, and enough rows for every persistent workgroup to see several tiles
bool rp_launch_stream(ripple_ctx *c, const TArgs &a, uint32_t rows_hint) {
    if (!c->opt_stream || a.a_mode != 0 || a.store || a.Ws || a.out_mode != 1) return false;
    if (a.K != 256 || a.Kpad != 256 || a.N != 256 || a.Npad != 256 || a.d_in != 256) return false;
    if (a.addend && a.addend_scaled) return false;
    if (rows_hint < 64u * 4u * 2u * c->n_cu) return false;   // at least four tiles per persistent workgroup
    const dim3 grid(2 * c->n_cu), block(256);
    if (a.addend && a.D) hipLaunchKernelGGL((k_transform_stream<true, true>), grid, block, 0, c->stream, a);
    else if (a.addend) hipLaunchKernelGGL((k_transform_stream<true, false>), grid, block, 0, c->stream, a);
    else if (a.D) hipLaunchKernelGGL((k_transform_stream<false, true>), grid, block, 0, c->stream, a);
    else hipLaunchKernelGGL((k_transform_stream<false, false>), grid, block, 0, c->stream, a);
    return true;
}


#include "transform_args.h"
#include "kernels.h"

typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

// Streaming variant of the row transform (the Compute step of Sec. 3.3 in re-apply form) for the shape that dominates
// large batches: x W with K = N = 256 (x = X^l[v], divided by the in-degree for mean), fp32 rows, H updated in place
// (ADD: plus an unscaled cached row; DELTA: the delta row is written too).
//
// A workgroup of four wavefronts owns 64-row tiles; wavefront w owns 64 output columns, as two 32-column blocks of
// interleaved columns (block j holds columns 64 w + 2 n + j), so that everything a lane reads or writes per row is
// eight adjacent bytes. Workgroups are persistent and no part of a tile waits for memory on its own:
//  * the weights never pass through LDS: a wavefront only needs its own 64 columns, so each lane loads the two
//    numbers it feeds into the matrix cores for a pair of k straight from the (L2-resident) matrix, eight pairs
//    (half a step) ahead, into the register an earlier pair has just freed;
//  * the gathered rows pass through a double-buffered LDS slice (one barrier per step): slice s + 1 is written while
//    slice s is multiplied, from registers requested two steps earlier, also across the tile boundary;
//  * the finished tile's accumulators are parked in a second set of registers and leave for memory in eight chunks
//    during the K steps of the next tile; the cached / old values a chunk is combined with are requested two steps
//    before the chunk is finished (the first two chunks of a tile during its own last steps);
//  * all of this is issued between the matrix-core operations of a step, where the wavefront has issue slots to spare;
//  * the mean's 1/deg is applied to the finished row instead of the gathered one, so staging is a plain copy.
// Every array is addressed through a buffer descriptor with 32-bit offsets (row id * 1 KB + constants): as flat
// addresses the compiler keeps dozens of 64-bit pointers alive across the unrolled steps, which no register file holds.
// The launch therefore requires vertex_capacity * 1 KB < 4 GB - 4 KB.
template <bool ADD, bool DELTA>
__global__ __launch_bounds__(256, 2) void k_transform_stream(TArgs a, uint32_t n_cap) {
    constexpr int BM = 64, KS = 8, NA = 2, LEAD = 2, KP = T_BK / 2, WLEAD = 8;
    __shared__ __attribute__((aligned(16))) float As[2][BM][T_BK + 1];
    __shared__ uint32_t s_vtx[2][BM];
    __shared__ float s_scale[2][BM];

    const int tid = threadIdx.x, lane = tid & 63, wn = tid >> 6;
    const uint32_t count = *a.count_ptr;
    const uint32_t n_tiles = (count + BM - 1) / BM;
    uint32_t tile = blockIdx.x;
    if (tile >= n_tiles) return;

    constexpr uint32_t RSRC3 = 0x00020000u;                // raw buffer, 32-bit elements
    const uint32_t row_bytes_total = n_cap * 1024u;        // < 4 GB - 4 KB (checked by the launch)
    const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc((void *)a.W, 0, 256 * 256 * 4, RSRC3);
    const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc((void *)a.X, 0, row_bytes_total, RSRC3);
    const __amdgpu_buffer_rsrc_t hres = __builtin_amdgcn_make_buffer_rsrc(a.Hout, 0, row_bytes_total, RSRC3);
    const __amdgpu_buffer_rsrc_t pres = __builtin_amdgcn_make_buffer_rsrc((void *)(ADD ? a.addend : a.X), 0, row_bytes_total, RSRC3);
    const __amdgpu_buffer_rsrc_t dres = __builtin_amdgcn_make_buffer_rsrc((void *)(DELTA ? a.D : (float *)a.Hout), 0, row_bytes_total, RSRC3);

    const uint32_t c4a = (tid % (T_BK / 4)) * 4;
    const int r_own = tid / (T_BK / 4);                    // this thread stages rows r_own and r_own + 32 of every slice
    const uint32_t colb = (wn * 64 + 2 * (lane & 31)) * 4u;    // byte offset of its two adjacent output columns in a row
    const uint32_t wvo = (lane >> 5) * 1024u + colb;       // weights: row (lane >> 5) of a pair of k, those two columns
    const floatx2 bias = *(const floatx2 *)(a.bias + wn * 64 + 2 * (lane & 31));

    // byte offsets of the two rows this thread stages, for the current and the next tile; rows past the end repeat
    // the last one and are never stored
    uint32_t xo_cur[NA], xo_nxt[NA];
    float sc_cur[NA], sc_nxt[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const uint32_t v = a.list[min(tile * BM + r_own + i * 32, count - 1u)];
        xo_cur[i] = v * 1024u + c4a * 4u;
        xo_nxt[i] = xo_cur[i];
        const uint32_t deg = a.in_meta[v].y;
        sc_cur[i] = a.mean ? 1.0f / (float)(deg > 1u ? deg : 1u) : 1.0f;
        sc_nxt[i] = sc_cur[i];
        if (c4a == 0) {                                    // nothing is parked yet: its row ids only have to be valid
            s_vtx[1][r_own + i * 32] = v;
            s_scale[1][r_own + i * 32] = 1.0f;
        }
    }

    auto load_x = [&](uint32_t xo, int slice) {
        return __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(xres, xo + slice * T_BK * 4, 0, 0));
    };
    auto load_w = [&](int slice, int q) {                  // pair q of k of a slice: the lane's operand for both column blocks
        return __builtin_bit_cast(floatx2, __builtin_amdgcn_raw_buffer_load_b64(wres, wvo, slice * T_BK * 1024 + q * 2048, 0));
    };
    auto stage_x = [&](int buf, const floatx4 (&r)[NA]) {
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            float *dst = &As[buf][r_own + i * 32][c4a];
            dst[0] = r[i].x;
            dst[1] = r[i].y;
            dst[2] = r[i].z;
            dst[3] = r[i].w;
        }
    };

    floatx4 ra[2][NA];                                     // ra[p]: the slice that goes to As[p] next
    floatx2 bq[WLEAD];                                     // bq[q % WLEAD]: pair q of k, requested WLEAD pairs before its use
#pragma unroll
    for (int i = 0; i < NA; ++i) ra[0][i] = load_x(xo_cur[i], 0);
#pragma unroll
    for (int i = 0; i < NA; ++i) ra[1][i] = load_x(xo_cur[i], 1);
#pragma unroll
    for (int q = 0; q < WLEAD; ++q) bq[q] = load_w(0, q);
    stage_x(0, ra[0]);
#pragma unroll
    for (int i = 0; i < NA; ++i) ra[0][i] = load_x(xo_cur[i], 2);

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
    int par = 0;                                           // s_vtx / s_scale [par]: the current tile, [par ^ 1]: the parked one
    floatx2 pa[LEAD][4], po[LEAD][4];                      // cached-row and old values of the chunks in flight
#pragma unroll
    for (int q = 0; q < LEAD; ++q)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            pa[q][j] = (floatx2)(0.0f);
            po[q][j] = (floatx2)(0.0f);
        }

    // Chunk c of a tile: accumulator elements 4 (c & 3) .. + 3 of blocks [c >> 2][0] and [c >> 2][1], i.e. for this lane
    // four rows (j) with its two columns each. `buf` names the tile's entry in s_vtx / s_scale.
    uint32_t rowoff[4];                                    // byte offsets of the chunk being finished (rows past the end of the
    float rsc[4];                                          // list: beyond the buffer, so that the hardware drops their stores)
    auto finish_rows = [&](int c, int buf, uint32_t rows) {
        const int lr0 = (c >> 2) * 32 + (c & 3) * 8 + (lane >> 5) * 4;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            rowoff[j] = s_vtx[buf][lr0 + j] * 1024u;
            rsc[j] = s_scale[buf][lr0 + j];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) rowoff[j] = (((uint32_t)(lr0 + j) < rows) ? rowoff[j] : 0xFFFFF000u) + colb;
    };
    auto finish_row = [&](int c, int j) {
        floatx2 z;
        z.x = accp[c >> 2][0][(c & 3) * 4 + j] * rsc[j] + bias.x + (ADD ? pa[c % LEAD][j].x : 0.0f);
        z.y = accp[c >> 2][1][(c & 3) * 4 + j] * rsc[j] + bias.y + (ADD ? pa[c % LEAD][j].y : 0.0f);
        if (a.act == RIPPLE_ACT_RELU) {
            z.x = z.x > 0.0f ? z.x : 0.0f;
            z.y = z.y > 0.0f ? z.y : 0.0f;
        }
        __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(uintx2, z), hres, rowoff[j], 0, 0);
        if (DELTA) {
            const floatx2 d = a.d_old ? po[c % LEAD][j] : z - po[c % LEAD][j];
            __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(uintx2, d), dres, rowoff[j], 0, 0);
        }
    };
    auto request_row = [&](int c, int buf, int j) {
        const uint32_t off = s_vtx[buf][(c >> 2) * 32 + (c & 3) * 8 + (lane >> 5) * 4 + j] * 1024u + colb;
        if (ADD) pa[c % LEAD][j] = __builtin_bit_cast(floatx2, __builtin_amdgcn_raw_buffer_load_b64(pres, off, 0, 0));
        if (DELTA) po[c % LEAD][j] = __builtin_bit_cast(floatx2, __builtin_amdgcn_raw_buffer_load_b64(hres, off, 0, 0));
    };

    for (;;) {
        const uint32_t tile_n = tile + gridDim.x;
        uint32_t v_nxt[NA];
#pragma unroll
        for (int i = 0; i < NA; ++i) v_nxt[i] = a.list[min(tile_n * BM + r_own + i * 32, count - 1u)];
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            // every wavefront is done with slice s - 1 (As[(s + 1) & 1] may be overwritten) and has written its part of slice s
            __syncthreads();
            if (s == 0 && c4a == 0) {                      // this tile's row ids and scale factors, for when it is written out
#pragma unroll
                for (int i = 0; i < NA; ++i) {
                    s_vtx[par][r_own + i * 32] = xo_cur[i] >> 10;
                    s_scale[par][r_own + i * 32] = sc_cur[i];
                }
            }
            if (s == 1) {                                  // the next tile's rows: offsets and scale factors
#pragma unroll
                for (int i = 0; i < NA; ++i) {
                    xo_nxt[i] = v_nxt[i] * 1024u + c4a * 4u;
                    const uint32_t deg = a.in_meta[v_nxt[i]].y;
                    sc_nxt[i] = a.mean ? 1.0f / (float)(deg > 1u ? deg : 1u) : 1.0f;
                }
            }
            float av[2][2];
#pragma unroll
            for (int i = 0; i < 2; ++i) av[0][i] = As[s & 1][i * 32 + (lane & 31)][lane >> 5];
#pragma unroll
            for (int q = 0; q < KP; ++q) {
                const int cur = q & 1, nxt = cur ^ 1;
                if (q + 1 < KP) {
#pragma unroll
                    for (int i = 0; i < 2; ++i) av[nxt][i] = As[s & 1][i * 32 + (lane & 31)][2 * (q + 1) + (lane >> 5)];
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[cur][i], bq[q % WLEAD].x, acc[i][0], 0, 0, 0);
                    acc[i][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[cur][i], bq[q % WLEAD].y, acc[i][1], 0, 0, 0);
                }
                // between the products: the pair WLEAD on (past the slice's end: of the next slice; after the last
                // slice: slice 0, for the next tile) ...
                bq[q % WLEAD] = (q + WLEAD < KP) ? load_w(s, q + WLEAD) : load_w((s + 1) % KS, q + WLEAD - KP);
                // ... and one piece of the parked tile's traffic or of the row staging. Chunk s of the parked tile,
                // requested LEAD steps ago, is finished; the chunk LEAD on is requested (the first LEAD chunks of the
                // tile being multiplied, once the parked one has none left).
                if (q == 0) {
                    finish_rows(s, par ^ 1, prev_rows);
                } else if (q <= 4) {
                    finish_row(s, q - 1);
                } else if (q >= 8 && q < 12) {
                    if (s + LEAD < KS) request_row(s + LEAD, par ^ 1, q - 8);
                    else request_row(s + LEAD - KS, par, q - 8);
                } else if (q == 12) {                      // slice s + 1 into the other LDS buffer
                    stage_x((s + 1) & 1, ra[(s + 1) & 1]);
                } else if (q == 13) {                      // and slice s + 3 into the registers it came from
#pragma unroll
                    for (int i = 0; i < NA; ++i)
                        ra[(s + 1) & 1][i] = load_x((s + 3 < KS) ? xo_cur[i] : xo_nxt[i], (s + 3) % KS);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
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
            xo_cur[i] = xo_nxt[i];
            sc_cur[i] = sc_nxt[i];
        }
        par ^= 1;
        tile = tile_n;
        if (tile >= n_tiles) break;
    }
    // the last tile: its first LEAD chunks are on their way already
#pragma unroll
    for (int c = 0; c < KS; ++c) {
        finish_rows(c, par ^ 1, prev_rows);
#pragma unroll
        for (int j = 0; j < 4; ++j) finish_row(c, j);
        if (c + LEAD < KS) {
#pragma unroll
            for (int j = 0; j < 4; ++j) request_row(c + LEAD, par ^ 1, j);
        }
    }
}

// x W with K = N = 256 on fp32 rows, H updated in place, and enough rows for every persistent workgroup to see several
// tiles (RIPPLE_OPT_STREAM_TRANSFORM = 2: whatever the number of rows)
bool rp_launch_stream(ripple_ctx *c, const TArgs &a, uint32_t rows_hint) {
    if (!c->opt_stream || a.a_mode != 0 || a.store || a.Ws || a.out_mode != 1) return false;
    if (a.K != 256 || a.Kpad != 256 || a.N != 256 || a.Npad != 256 || a.d_in != 256) return false;
    if (a.addend && a.addend_scaled) return false;
    if ((uint64_t)c->n_cap * 1024u > 0xFFFFF000ull) return false;   // 32-bit byte offsets into the row arrays, the top 4 KB kept free
    if (rows_hint < 64u * 4u * 2u * c->n_cu) return false;          // at least four tiles per persistent workgroup
    const dim3 grid(2 * c->n_cu), block(256);
    if (a.addend && a.D) hipLaunchKernelGGL((k_transform_stream<true, true>), grid, block, 0, c->stream, a, c->n_cap);
    else if (a.addend) hipLaunchKernelGGL((k_transform_stream<true, false>), grid, block, 0, c->stream, a, c->n_cap);
    else if (a.D) hipLaunchKernelGGL((k_transform_stream<false, true>), grid, block, 0, c->stream, a, c->n_cap);
    else hipLaunchKernelGGL((k_transform_stream<false, false>), grid, block, 0, c->stream, a, c->n_cap);
    return true;
}

// ---------------------------------------------------------------------------------
// Both products of a narrow project-first layer, H^{l-1}[v] W_self (into PS) and H^{l-1}[v] W_neigh (into PD, or T at
// the bootstrap), for d_in = 256 and d_out <= 48 on fp32 rows. Every wavefront is on its own: it owns 32-row tiles and
// all 96 columns (three matrix-core blocks), stages its rows through a private, double-buffered LDS slice and reads the
// weights straight from L2 into the operand registers half a step ahead, so there is no barrier anywhere and three
// wavefronts per SIMD cover one another's waits. The weight matrix comes permuted, [k][n][j] with three adjacent
// floats per lane: position n < 16 of block j is column 16 j + n of W_self, n >= 16 column 16 j + n - 16 of W_neigh,
// so a lane ends up with columns (c, 16 + c, 32 + c) of one of the two products.
// ---------------------------------------------------------------------------------
struct PArgs {
    const uint32_t *list;
    const uint32_t *count_ptr;
    const float *H;                // [n_cap x 256]
    const float *Wp;               // [256][32][3]
    float *out1, *out2;            // PS [n_cap x ld1], PD or T [n_cap x ld2]
    uint32_t ld1, ld2, d_out, n_cap;
};

typedef uint32_t uintx3 __attribute__((ext_vector_type(3)));
typedef float floatx3 __attribute__((ext_vector_type(3)));

__global__ __launch_bounds__(256, 3) void k_project_both_stream(PArgs a) {
    constexpr int BM = 32, KS = 8, NA = 4, KP = T_BK / 2, WLEAD = 8;
    __shared__ __attribute__((aligned(16))) float As_all[4][2][BM][T_BK + 1];
    __shared__ uint32_t s_vtx_all[4][BM];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float (*As)[BM][T_BK + 1] = As_all[wave];
    uint32_t *s_vtx = s_vtx_all[wave];
    const uint32_t count = *a.count_ptr;
    const uint32_t n_tiles = (count + BM - 1) / BM;
    const uint32_t n_waves = gridDim.x * 4u;
    uint32_t tile = blockIdx.x * 4u + wave;
    if (tile >= n_tiles) return;

    constexpr uint32_t RSRC3 = 0x00020000u;
    const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc((void *)a.Wp, 0, 256 * 96 * 4, RSRC3);
    const __amdgpu_buffer_rsrc_t hres = __builtin_amdgcn_make_buffer_rsrc((void *)a.H, 0, a.n_cap * 1024u, RSRC3);

    const uint32_t c4a = (lane & 7) * 4;                   // the lane stages rows (lane >> 3) + 8 i, i = 0..3, of every slice
    const int r_own = lane >> 3;
    const uint32_t wvo = (lane >> 5) * 384u + (lane & 31) * 12u;   // weights: row (lane >> 5) of a pair of k, its three numbers

    auto load_h = [&](uint32_t ho, int slice) {
        return __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(hres, ho + slice * T_BK * 4, 0, 0));
    };
    auto load_w = [&](int slice, int q) {
        return __builtin_bit_cast(floatx3, __builtin_amdgcn_raw_buffer_load_b96(wres, wvo, slice * T_BK * 384 + q * 768, 0));
    };
    auto stage = [&](int buf, const floatx4 (&r)[NA]) {
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            float *dst = &As[buf][r_own + 8 * i][c4a];
            dst[0] = r[i].x;
            dst[1] = r[i].y;
            dst[2] = r[i].z;
            dst[3] = r[i].w;
        }
    };

    uint32_t ho_cur[NA], ho_nxt[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        ho_cur[i] = a.list[min(tile * BM + r_own + 8 * i, count - 1u)] * 1024u + c4a * 4u;   // rows past the end repeat the last one
        ho_nxt[i] = ho_cur[i];
    }
    floatx4 ra[2][NA];
    floatx3 bq[WLEAD];                                     // bq[q % WLEAD]: pair q of k, requested WLEAD pairs before its use
#pragma unroll
    for (int i = 0; i < NA; ++i) ra[0][i] = load_h(ho_cur[i], 0);
#pragma unroll
    for (int i = 0; i < NA; ++i) ra[1][i] = load_h(ho_cur[i], 1);
#pragma unroll
    for (int q = 0; q < WLEAD; ++q) bq[q] = load_w(0, q);
    stage(0, ra[0]);
#pragma unroll
    for (int i = 0; i < NA; ++i) ra[0][i] = load_h(ho_cur[i], 2);

    floatx16 acc[3];
#pragma unroll
    for (int j = 0; j < 3; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;

    // where this lane's three columns go
    const uint32_t sub = lane & 15u;
    const bool second = (lane & 16) != 0;
    float *const obase = (second ? a.out2 : a.out1) + sub;
    const uint32_t old = second ? a.ld2 : a.ld1;

    for (;;) {
        const uint32_t tile_n = tile + n_waves;
        uint32_t v_nxt[NA];
#pragma unroll
        for (int i = 0; i < NA; ++i) v_nxt[i] = a.list[min(tile_n * BM + r_own + 8 * i, count - 1u)];
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            // the wavefront's LDS accesses are served in order: slice s (written during step s - 1) is complete
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            if (s == 0 && c4a == 0) {
#pragma unroll
                for (int i = 0; i < NA; ++i) s_vtx[r_own + 8 * i] = ho_cur[i] >> 10;
            }
            if (s == 1) {
#pragma unroll
                for (int i = 0; i < NA; ++i) ho_nxt[i] = v_nxt[i] * 1024u + c4a * 4u;
            }
            float av[2];
            av[0] = As[s & 1][lane & 31][lane >> 5];
#pragma unroll
            for (int q = 0; q < KP; ++q) {
                const int cur = q & 1, nxt = cur ^ 1;
                if (q + 1 < KP) av[nxt] = As[s & 1][lane & 31][2 * (q + 1) + (lane >> 5)];
                __builtin_amdgcn_sched_barrier(0);
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[cur], bq[q % WLEAD].x, acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[cur], bq[q % WLEAD].y, acc[1], 0, 0, 0);
                acc[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[cur], bq[q % WLEAD].z, acc[2], 0, 0, 0);
                // the pair WLEAD on (past the slice's end: of the next slice; after the last slice: slice 0, for the next tile)
                bq[q % WLEAD] = (q + WLEAD < KP) ? load_w(s, q + WLEAD) : load_w((s + 1) % KS, q + WLEAD - KP);
                if (q == 10) {                             // slice s + 1 into the other LDS buffer
                    stage((s + 1) & 1, ra[(s + 1) & 1]);
                } else if (q == 11) {                      // and slice s + 3 into the registers it came from
#pragma unroll
                    for (int i = 0; i < NA; ++i)
                        ra[(s + 1) & 1][i] = load_h((s + 3 < KS) ? ho_cur[i] : ho_nxt[i], (s + 3) % KS);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // the tile's 32 x 96 results leave straight from the accumulators: element r of block j is row
        // 8 (r >> 2) + 4 (lane >> 5) + (r & 3), column 16 j + sub of this lane's product
        const uint32_t rows = min((uint32_t)BM, count - tile * BM);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const uint32_t lr = (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
            if (lr < rows) {
                float *o = obase + (size_t)s_vtx[lr] * old;
                o[0] = acc[0][r];
                if (16u + sub < a.d_out) o[16] = acc[1][r];
                if (32u + sub < a.d_out) o[32] = acc[2][r];
            }
        }
#pragma unroll
        for (int j = 0; j < 3; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;
#pragma unroll
        for (int i = 0; i < NA; ++i) ho_cur[i] = ho_nxt[i];
        tile = tile_n;
        if (tile >= n_tiles) break;
    }
}

bool rp_launch_project_both_stream(ripple_ctx *c, uint32_t l, const uint32_t *list, const uint32_t *count_d, float *out2,
                                   uint32_t ld2, uint32_t rows_hint) {
    const LayerDev &ly = c->layers[l - 1];
    if (!c->opt_stream || !ly.Wc96p || c->store || ly.d_in != 256 || ly.d_out > 48 || ly.d_out < 17) return false;
    if ((uint64_t)c->n_cap * 1024u > 0xFFFFF000ull) return false;
    if (rows_hint < 131072u && c->opt_stream != 2) return false;   // enough 32-row tiles for every wavefront of the chip (2: any number, for tests)
    PArgs a;
    a.list = list;
    a.count_ptr = count_d;
    a.H = (const float *)c->H[l - 1];
    a.Wp = ly.Wc96p;
    a.out1 = ly.PS;
    a.ld1 = ly.d_out;
    a.out2 = out2;
    a.ld2 = ld2;
    a.d_out = ly.d_out;
    a.n_cap = c->n_cap;
    hipLaunchKernelGGL(k_project_both_stream, dim3(3 * c->n_cu), dim3(256), 0, c->stream, a);
    return true;
}

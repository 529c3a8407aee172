// Arguments of the row-transform kernels (shared by the tiled kernels and the streaming variant).
#pragma once
#include "common.h"

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));   // native vector: stays in registers

struct TArgs {
    const uint32_t *list;          // slot -> vertex id
    const uint32_t *count_ptr;     // number of slots (device)
    int a_mode;                    // 0 x | 1 [h_self | x] | 2 (1+eps) h_self + x | 3 compact rows of tmp_in | 4 h_self
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
    const __hip_bfloat16 *Wt;      // bf16 copy of W, transposed [Npad x Kpad] (k contiguous), or null
    const unsigned short *Ws;      // fp32 storage: W as three transposed bf16 planes (W = plane 0 + plane 1 + plane 2), or null
    size_t ws_plane;               // elements per plane
    uint32_t wt_ld;                // its row stride
    uint32_t K, Kpad, N, Npad;
    int act;
    int out_mode;                  // 0 write act(z) to tmp_out[slot] | 1 update H, emit delta | 2 write to tmp_out[vertex]
    const float *addend;           // [vertex x N] rows added before the activation (projected aggregate or cached self term), or null
    int addend_scaled;             // 1: the addend is an aggregate and takes the mean scale
    const float *addend2;          // second, unscaled addend (k_transform_addend_only), or null
    const float *den;              // attention layers (k_transform_addend_only): the addend is divided by den[vertex], or null
    uint32_t *range_rows;          // with den: += rows whose numerator or denominator was not finite
    float *tmp_out;
    uint32_t tmp_out_ld;
    // two products from one pass over the rows (out_mode 2 only): the weight matrix holds a second block of
    // columns from split_col on (a multiple of 4); columns [0, N1) go to tmp_out, columns [split_col, N) to
    // tmp_out2 as its columns 0 .. N - split_col - 1. split_col = 0: one block, N1 = N.
    uint32_t split_col, N1;
    float *tmp_out2;
    uint32_t tmp_out2_ld;
    void *Hout;
    float *D;                      // delta rows [vertex x N] or null
    int d_old;                     // D receives the row's old value instead of new - old (the next layer takes max / min)
    int store;                     // 0 fp32, 1 bf16 embeddings
};

#define T_BK 32

// transform_stream.hip: launches the streaming kernel if the arguments have its shape and enough rows are expected
bool rp_launch_stream(ripple_ctx *c, const TArgs &a, uint32_t rows_hint);
// the same for both products of a narrow project-first layer with a cached self term (second product into out2)
bool rp_launch_project_both_stream(ripple_ctx *c, uint32_t l, const uint32_t *list, const uint32_t *count_d, float *out2,
                                   uint32_t ld2, uint32_t rows_hint);

// Host-side launchers implemented next to their kernels.
#pragma once
#include "common.h"
#include <algorithm>

// graph_store.hip
void rp_exclusive_scan(hipStream_t s, const uint32_t *in, uint32_t *out, uint32_t n, uint32_t *part,
                       uint32_t *total_out);
ripple_status rp_build_graph(ripple_ctx *c, uint32_t n_vertices, uint64_t n_edges, const uint32_t *src_h,
                             const uint32_t *dst_h, const float *w_h);
ripple_status rp_compact(ripple_ctx *c);
void rp_launch_batch_reset(ripple_ctx *c);
void rp_launch_mutate(ripple_ctx *c, uint32_t n_ops, bool has_vertex_add, bool has_vertex_del, bool has_vertex_or_feat);

// order.hip
ripple_status rp_stable_sort_pairs(ripple_ctx *c, const uint32_t *keys_in, uint32_t *keys_out, const uint32_t *vals_in,
                                   uint32_t *vals_out, size_t n, unsigned key_bits);
size_t rp_sort_u64_tmp_bytes(size_t n_max);
size_t rp_sort_u32_tmp_bytes(size_t n_max);
bool rp_sort_pairs_u32(ripple_ctx *c, const uint32_t *keys_in, uint32_t *keys_out, const uint32_t *vals_in, uint32_t *vals_out,
                       size_t n, unsigned key_bits, void *tmp, size_t tmp_bytes);
void rp_sort_pairs_u64(ripple_ctx *c, const unsigned long long *keys_in, unsigned long long *keys_out, const float *vals_in,
                       float *vals_out, size_t n, void *tmp, size_t tmp_bytes);

// frontier.hip
void rp_launch_frontier_mark(ripple_ctx *c, uint32_t l, bool allow_disc, uint32_t pair_cap = 0);
void rp_launch_alive_list(ripple_ctx *c);
void rp_launch_frontier_compact(ripple_ctx *c, uint32_t l, bool self_term, bool want_out, bool want_in,
                                bool accumulate_rep, bool pruned = false);
void rp_launch_candidates(ripple_ctx *c, uint32_t l);
void rp_launch_candidates_sparse(ripple_ctx *c, uint32_t l, bool self_term, uint32_t long_min);
void rp_launch_list_offsets(ripple_ctx *c, uint32_t l, bool want_out);
void rp_launch_bitmap_to_list(ripple_ctx *c, uint32_t *bitmap, uint32_t *out_list, uint32_t *count_d);
void rp_launch_list_eoff(ripple_ctx *c, uint32_t l);
ripple_status rp_static_scratch_init(ripple_ctx *c);
uint32_t rp_static_max_vertices();
ripple_status rp_launch_affected_static(ripple_ctx *c, uint32_t *bitmap, uint32_t *ids_out, uint32_t cap, uint32_t *n_out);
void rp_launch_frontier_sparse(ripple_ctx *c, uint32_t l, bool self_term, bool want_out, uint32_t long_min = 0);

// scatter.hip
void rp_launch_scatter_push(ripple_ctx *c, uint32_t l, bool may_pull, bool allow_disc);
void rp_launch_scatter_pull_det(ripple_ctx *c, uint32_t l, bool bootstrap);
void rp_launch_scatter_pull(ripple_ctx *c, uint32_t l, bool discover, bool allow_disc, uint32_t pair_cap = 0);
bool rp_launch_scatter_sorted(ripple_ctx *c, uint32_t l, bool allow_disc, uint32_t pair_cap);
void rp_launch_pull_all(ripple_ctx *c, uint32_t l);
void rp_launch_messages(ripple_ctx *c, uint32_t l);
void rp_launch_scatter_mono(ripple_ctx *c, uint32_t l, const uint32_t *count_ptr, bool listed);

// attention.hip
void rp_launch_gat_scatter(ripple_ctx *c, uint32_t l, bool bootstrap, bool prequeued = false);
void rp_launch_gat_save(ripple_ctx *c, uint32_t l, const uint32_t *list, const uint32_t *count_d);
void rp_launch_gat_scores(ripple_ctx *c, uint32_t l, const uint32_t *list, const uint32_t *count_d);

// transform.hip
void rp_launch_gat_project(ripple_ctx *c, uint32_t l, const uint32_t *list, const uint32_t *count_d);
void rp_launch_transform(ripple_ctx *c, uint32_t l, const uint32_t *list, const uint32_t *count_d, bool emit_delta);
void rp_launch_self_project(ripple_ctx *c, uint32_t l, const uint32_t *list, const uint32_t *count_d);
void rp_launch_project(ripple_ctx *c, uint32_t l, const uint32_t *list, const uint32_t *count_d, bool bootstrap);
bool rp_has_project_both(const ripple_ctx *c, uint32_t l);
void rp_launch_project_both(ripple_ctx *c, uint32_t l, const uint32_t *list, const uint32_t *count_d, bool bootstrap);

// api.hip: HIP-event timing of kernel classes (no-ops unless RIPPLE_OPT_TIMING is on)
int rp_timer_begin(ripple_ctx *c);
void rp_timer_end(ripple_ctx *c, int token, int phase, int layer, bool counted = true);

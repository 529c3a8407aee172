// Stable device-wide sort of (key, value) pairs of 32-bit words, used once when the graph store is built.
// The sort itself is rocPRIM's radix sort (a library primitive); everything around it is in graph_store.hip.
#include "kernels.h"
#include <cstring>
#include <rocprim/device/device_radix_sort.hpp>

ripple_status rp_stable_sort_pairs(ripple_ctx *c, const uint32_t *keys_in, uint32_t *keys_out, const uint32_t *vals_in,
                                   uint32_t *vals_out, size_t n, unsigned key_bits) {
    size_t tmp_bytes = 0;
    void *tmp = nullptr;
    RP_HIP(c, rocprim::radix_sort_pairs(nullptr, tmp_bytes, keys_in, keys_out, vals_in, vals_out, n, 0u, key_bits, c->stream));
    RP_HIP(c, hipMalloc(&tmp, tmp_bytes ? tmp_bytes : 1));
    hipError_t e = rocprim::radix_sort_pairs(tmp, tmp_bytes, keys_in, keys_out, vals_in, vals_out, n, 0u, key_bits, c->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    hipFree(tmp);
    RP_HIP(c, e);
    return RIPPLE_OK;
}

// The same for 64-bit keys with float values, all 64 bits, in memory the caller holds: `tmp` of at least
// rp_sort_u64_tmp_bytes(n_max) bytes serves any n <= n_max. Nothing is allocated and the stream is not waited for.
size_t rp_sort_u64_tmp_bytes(size_t n_max) {
    size_t bytes = 0;
    const unsigned long long *k = nullptr;
    unsigned long long *ko = nullptr;
    const float *v = nullptr;
    float *vo = nullptr;
    if (rocprim::radix_sort_pairs(nullptr, bytes, k, ko, v, vo, n_max, 0u, 64u, (hipStream_t)0) != hipSuccess) return 0;
    return bytes ? bytes : 1;
}

void rp_sort_pairs_u64(ripple_ctx *c, const unsigned long long *keys_in, unsigned long long *keys_out, const float *vals_in,
                       float *vals_out, size_t n, void *tmp, size_t tmp_bytes) {
    (void)rocprim::radix_sort_pairs(tmp, tmp_bytes, keys_in, keys_out, vals_in, vals_out, n, 0u, 64u, c->stream);
}

// The same for 32-bit keys and values on the low `key_bits` bits (a hop's messages by destination).
size_t rp_sort_u32_tmp_bytes(size_t n_max) {
    size_t bytes = 0;
    const uint32_t *k = nullptr;
    uint32_t *ko = nullptr;
    if (rocprim::radix_sort_pairs(nullptr, bytes, k, ko, k, ko, n_max, 0u, 32u, (hipStream_t)0) != hipSuccess) return 0;
    return bytes ? bytes : 1;
}

// false (nothing enqueued) if `tmp` is too small for this n after all
bool rp_sort_pairs_u32(ripple_ctx *c, const uint32_t *keys_in, uint32_t *keys_out, const uint32_t *vals_in, uint32_t *vals_out,
                       size_t n, unsigned key_bits, void *tmp, size_t tmp_bytes) {
    size_t need = 0;
    if (rocprim::radix_sort_pairs(nullptr, need, keys_in, keys_out, vals_in, vals_out, n, 0u, key_bits, c->stream) != hipSuccess) return false;
    if (need > tmp_bytes) return false;
    return rocprim::radix_sort_pairs(tmp, need, keys_in, keys_out, vals_in, vals_out, n, 0u, key_bits, c->stream) == hipSuccess;
}

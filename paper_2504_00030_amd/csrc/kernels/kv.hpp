// Addressing of the paged KV cache.
// K pages are [kv head][token][hd]; V pages are stored transposed, [kv head][hd][token], so that the
// attention kernels read consecutive tokens of one channel with a single vector load.
#pragma once

#include "common.hpp"
#include "params.hpp"

namespace sd {

__device__ __forceinline__ int kv_page(const KVCache &kv, int seq, int pos) {
    return kv.block_table[seq * kv.pages_per_seq + (pos >> kv.page_shift)];
}
__device__ __forceinline__ size_t kv_head_base(const KVCache &kv, int page, int kvh) {
    return ((size_t)page * kv.n_kv + kvh) * kv.page_tokens * kv.hd;
}
__device__ __forceinline__ size_t kv_index_k(const KVCache &kv, int seq, int pos, int kvh, int j) {
    return kv_head_base(kv, kv_page(kv, seq, pos), kvh) + (size_t)(pos & (kv.page_tokens - 1)) * kv.hd + j;
}
__device__ __forceinline__ size_t kv_index_v(const KVCache &kv, int seq, int pos, int kvh, int j) {
    return kv_head_base(kv, kv_page(kv, seq, pos), kvh) + (size_t)j * kv.page_tokens + (pos & (kv.page_tokens - 1));
}
__device__ __forceinline__ void kv_store(const KVCache &kv, int kv_dtype, bool is_k, int seq, int pos, int kvh, int j,
                                         float v) {
    const size_t e = is_k ? kv_index_k(kv, seq, pos, kvh, j) : kv_index_v(kv, seq, pos, kvh, j);
    void *pool = is_k ? kv.k : kv.v;
    if (kv_dtype == DT_BF16) reinterpret_cast<bf16_t *>(pool)[e] = f32_to_bf16(v);
    else reinterpret_cast<float *>(pool)[e] = v;
}
__device__ __forceinline__ float kv_load(const void *pool, int kv_dtype, size_t e) {
    return kv_dtype == DT_BF16 ? bf16_to_f32(reinterpret_cast<const bf16_t *>(pool)[e])
                               : reinterpret_cast<const float *>(pool)[e];
}

}  // namespace sd

// Addressing of the paged KV cache.
// A page holds, per kv head, a block of page_tokens x hd elements.  Two arrangements of that block:
//  * plain (kv.frag == 0): K is [token][hd]; V is stored transposed, [hd][token].
//  * fragment order (kv.frag == 1; head dimensions that are multiples of 32, pages of at least 16 tokens): the block
//    is a sequence of 16-token slabs, and inside a slab the elements sit in the order in which the lanes of the
//    matrix instructions of the attention kernels hold them.  K: [channel group of 8][token of the slab][8 channels]
//    (lane = 16 * (group mod 4) + token reads 16 bytes; the 64 lanes of one load read 1 KiB end to end).  V: [channel
//    tile of 16][token quad][channel of the tile][4 tokens] (lane = 16 * quad + channel reads 8 bytes; 512 bytes end
//    to end).  With the plain arrangement neighbouring lanes read from different cache lines (a token's row, a
//    channel's row), and the number of lines a load touches, not its bytes, bounds the attention kernels.
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
// element offset of (token t of the page, channel j) inside a head's block
__device__ __forceinline__ size_t kv_in_k(const KVCache &kv, int t, int j) {
    return kv.frag ? (size_t)(t >> 4) * 16 * kv.hd + (size_t)(((j >> 3) * 16 + (t & 15)) * 8 + (j & 7))
                   : (size_t)t * kv.hd + j;
}
__device__ __forceinline__ size_t kv_in_v(const KVCache &kv, int t, int j) {
    return kv.frag ? (size_t)(t >> 4) * 16 * kv.hd +
                         (size_t)((((j >> 4) * 4 + ((t & 15) >> 2)) * 16 + (j & 15)) * 4 + (t & 3))
                   : (size_t)j * kv.page_tokens + t;
}
// distance between the fragments of consecutive 32-channel steps of K / 16-channel tiles of V of one lane
__device__ __forceinline__ int kv_step_k(const KVCache &kv) { return kv.frag ? 512 : 32; }
__device__ __forceinline__ int kv_step_v(const KVCache &kv) { return kv.frag ? 256 : 16 * kv.page_tokens; }
__device__ __forceinline__ size_t kv_index_k(const KVCache &kv, int seq, int pos, int kvh, int j) {
    return kv_head_base(kv, kv_page(kv, seq, pos), kvh) + kv_in_k(kv, pos & (kv.page_tokens - 1), j);
}
__device__ __forceinline__ size_t kv_index_v(const KVCache &kv, int seq, int pos, int kvh, int j) {
    return kv_head_base(kv, kv_page(kv, seq, pos), kvh) + kv_in_v(kv, pos & (kv.page_tokens - 1), j);
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

// KV-cache write: scatters the keys and values of new tokens into the paged cache by slot mapping
// (the step in front of paged attention; layout as in the PagedAttention work the paper cites).
// A copy bound by HBM: each lane moves 16 bytes, a token row of K and of V is covered by
// consecutive lanes, and the slot of a token is read once per lane through the vector cache.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/attn.h"

namespace attn {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct KvWriteParams {
    const unsigned char *k_new, *v_new;
    unsigned char *k_cache, *v_cache;
    const int32_t *slot_mapping;
    int64_t new_tok_bytes, new_head_bytes, blk_bytes, tok_bytes, head_bytes;
    int32_t num_tokens, num_kv_heads, vec_per_head, block_size;
};

__global__ __launch_bounds__(256) void kv_cache_write_kernel(const KvWriteParams p)
{
    // one item = one 16-byte vector of one (token, tensor, head); K and V interleave at head granularity
    const int per_tok = 2 * p.num_kv_heads * p.vec_per_head;
    const int64_t total = (int64_t)p.num_tokens * per_tok;
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int t = (int)(i / per_tok);
        int r = (int)(i % per_tok);
        const int is_v = r >= p.num_kv_heads * p.vec_per_head;
        if (is_v) r -= p.num_kv_heads * p.vec_per_head;
        const int h = r / p.vec_per_head, c = r % p.vec_per_head;
        const int slot = p.slot_mapping[t];
        if (slot < 0) continue;
        const int blk = slot / p.block_size, off = slot % p.block_size;
        const unsigned char *src = (is_v ? p.v_new : p.k_new) + t * p.new_tok_bytes + h * p.new_head_bytes + 16 * c;
        unsigned char *dst = (is_v ? p.v_cache : p.k_cache) + blk * p.blk_bytes + off * p.tok_bytes + h * p.head_bytes + 16 * c;
        *(u32x4 *)dst = *(const u32x4 *)src;
    }
}

}  // namespace
}  // namespace attn

extern "C" int attn_kv_cache_write(const attn_kv_write_args *a, void *hip_stream)
{
    using namespace attn;
    if (!a) return ATTN_ERR_NULL;
    if (a->struct_bytes != sizeof(attn_kv_write_args)) return ATTN_ERR_SHAPE;
    if (a->dtype != ATTN_BF16 && a->dtype != ATTN_F32 && a->dtype != ATTN_F16) return ATTN_ERR_DTYPE;
    const int esz = a->dtype == ATTN_F32 ? 4 : 2;
    if (a->num_tokens < 0 || a->num_kv_heads <= 0 || a->head_dim <= 0 || a->block_size <= 0 || a->num_blocks <= 0) return ATTN_ERR_SHAPE;
    if ((a->head_dim * esz) % 16 != 0) return ATTN_ERR_UNSUPPORTED;
    if (a->num_tokens == 0) return ATTN_OK;
    if (!a->k_new || !a->v_new || !a->k_cache || !a->v_cache || !a->slot_mapping) return ATTN_ERR_NULL;
    const int64_t strides[5] = {a->new_stride_tok, a->new_stride_head, a->kv_stride_block, a->kv_stride_tok, a->kv_stride_head};
    for (int64_t st : strides)
        if (st < a->head_dim || (st * esz) % 16 != 0) return ATTN_ERR_SHAPE;
    if (((uintptr_t)a->k_new | (uintptr_t)a->v_new | (uintptr_t)a->k_cache | (uintptr_t)a->v_cache) & 15) return ATTN_ERR_SHAPE;
    KvWriteParams p;
    p.k_new = (const unsigned char *)a->k_new;
    p.v_new = (const unsigned char *)a->v_new;
    p.k_cache = (unsigned char *)a->k_cache;
    p.v_cache = (unsigned char *)a->v_cache;
    p.slot_mapping = a->slot_mapping;
    p.new_tok_bytes = a->new_stride_tok * esz;
    p.new_head_bytes = a->new_stride_head * esz;
    p.blk_bytes = a->kv_stride_block * esz;
    p.tok_bytes = a->kv_stride_tok * esz;
    p.head_bytes = a->kv_stride_head * esz;
    p.num_tokens = a->num_tokens;
    p.num_kv_heads = a->num_kv_heads;
    p.vec_per_head = a->head_dim * esz / 16;
    p.block_size = a->block_size;
    const int64_t total = (int64_t)a->num_tokens * 2 * a->num_kv_heads * p.vec_per_head;
    if (total > ((int64_t)1 << 40)) return ATTN_ERR_SHAPE;
    const int64_t want = (total + 255) / 256;
    const unsigned blocks = (unsigned)(want < 16384 ? want : 16384);  // grid-stride beyond that
    hipLaunchKernelGGL(kv_cache_write_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)hip_stream, p);
    return hipGetLastError() == hipSuccess ? ATTN_OK : ATTN_ERR_HIP;
}

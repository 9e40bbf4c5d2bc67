// fp32 attention on plain FMA: one wavefront per (query token, query head).
//
// Same operation as the bf16 MFMA kernels (tiled online-softmax attention, the
// FlashAttention-2 formulation the paper's kernel follows, section "Method and
// Investigated Kernels"), kept in true fp32 for inputs that are fp32.  It serves
// small latency-bound calls; no matrix cores are involved.
#include "kernel_params.hpp"

namespace attn {
namespace {

__device__ __forceinline__ float wave_max(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    return x;
}
__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

// HD is 64 or 128: lane owns output channels lane, lane + 64.
template <int HD>
__global__ __launch_bounds__(64) void prefill_f32_kernel(const KParams p)
{
    constexpr int CPL = HD / 64;
    __shared__ float q_s[HD];
    __shared__ float p_s[64];
    __shared__ long long off_s[64];

    const int head = blockIdx.y;
    const int kvh = head / p.group;
    const int lane = threadIdx.x;
    // blockIdx.x enumerates (sequence, token slot); slots past n_q exit
    const int s = blockIdx.x / p.max_q_len;
    const int i = blockIdx.x % p.max_q_len;
    const int q0 = p.query_start_loc[s];
    const int n_q = p.query_start_loc[s + 1] - q0;
    if (i >= n_q) return;
    const int n_kv = p.seq_lens[s];
    int limit = p.causal ? (n_kv - n_q) + i + 1 : n_kv;
    limit = limit < n_kv ? limit : n_kv;

    const float *qrow = (const float *)p.q + (int64_t)(q0 + i) * p.q_stride_tok + (int64_t)head * p.q_stride_head;
#pragma unroll
    for (int c = 0; c < CPL; ++c) q_s[lane + 64 * c] = qrow[lane + 64 * c];
    __syncthreads();

    const float *kbase = (const float *)p.k;
    const float *vbase = (const float *)p.v;
    const int kv0 = p.block_table ? 0 : p.kv_start_loc[s];
    const int32_t *bt_row = p.block_table ? p.block_table + (int64_t)s * p.block_table_stride : nullptr;

    float m = -INFINITY, l = 0.f;
    float acc[CPL];
#pragma unroll
    for (int c = 0; c < CPL; ++c) acc[c] = 0.f;

    for (int j0 = 0; j0 < limit; j0 += 64) {
        const int j = j0 + lane;
        float x = -INFINITY;
        long long ro = 0;
        if (j < limit) {
            if (bt_row) {
                const int blk = bt_row[j >> p.block_shift];
                ro = (long long)blk * p.kv_stride_block + (long long)(j & (p.block_size - 1)) * p.kv_stride_tok;
            } else {
                ro = (long long)(kv0 + j) * p.kv_stride_tok;
            }
            ro += (long long)kvh * p.kv_stride_head;
            const float *kr = kbase + ro;
            float dot = 0.f;
#pragma unroll 8
            for (int d = 0; d < HD; ++d) dot = fmaf(q_s[d], kr[d], dot);
            x = dot * p.scale;
        }
        const float m_new = fmaxf(m, wave_max(x));  // finite: key j0 is always visible
        const float alpha = expf(m - m_new);
        const float e = j < limit ? expf(x - m_new) : 0.f;
        l = l * alpha + wave_sum(e);
        m = m_new;
        __syncthreads();  // previous chunk's readers are done
        p_s[lane] = e;
        off_s[lane] = ro;
        __syncthreads();
        const int cnt = limit - j0 < 64 ? limit - j0 : 64;
#pragma unroll
        for (int c = 0; c < CPL; ++c) acc[c] *= alpha;
        for (int jj = 0; jj < cnt; ++jj) {
            const float pj = p_s[jj];
            const float *vr = vbase + off_s[jj];
#pragma unroll
            for (int c = 0; c < CPL; ++c) acc[c] = fmaf(pj, vr[lane + 64 * c], acc[c]);
        }
    }
    float *orow = (float *)p.out + (int64_t)(q0 + i) * p.o_stride_tok + (int64_t)head * p.o_stride_head;
    const float inv = l > 0.f ? 1.f / l : 0.f;
#pragma unroll
    for (int c = 0; c < CPL; ++c) orow[lane + 64 * c] = acc[c] * inv;
}

}  // namespace

hipError_t launch_prefill_f32(const KParams &p, hipStream_t stream)
{
    const int64_t slots = (int64_t)p.num_seqs * p.max_q_len;
    if (slots <= 0) return hipSuccess;
    if (slots > 0x7fffffff || p.num_q_heads > 65535) return hipErrorInvalidConfiguration;
    dim3 grid((unsigned)slots, (unsigned)p.num_q_heads);
    if (p.head_dim == 64)
        hipLaunchKernelGGL(prefill_f32_kernel<64>, grid, dim3(64), 0, stream, p);
    else if (p.head_dim == 128)
        hipLaunchKernelGGL(prefill_f32_kernel<128>, grid, dim3(64), 0, stream, p);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace attn

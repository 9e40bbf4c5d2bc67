// Paged-KV decode with split-K on bf16 MFMA (gfx950), plus the wavefront combine.
//
// One query token per sequence attends to its whole paged context (the
// PagedAttention setting the paper cites; Llama3 head shapes from its section
// "Method and Investigated Kernels").  The work is bound by streaming K and V
// from HBM once, so the design is about bytes in flight, not about flops:
//
//  * A workgroup owns (sequence, KV head, one part of the key axis); its
//    wavefronts take interleaved 32-key chunks of that part and never
//    synchronise with each other until the end.
//  * All G query heads of the KV head ride in the 16 columns of
//    v_mfma_f32_16x16x32_bf16 (S^T = K Q^T), so every K/V byte is fetched once
//    for the whole group.
//  * K rows go from HBM straight into MFMA A-operand registers (64 contiguous
//    bytes per row and instruction, whole 256-byte rows per chunk); V rows are
//    fetched with fully coalesced 128-bit loads, parked in a wave-private LDS
//    tile and read back transposed (ds_read_b64_tr_b16).  The next chunk's loads
//    are issued before the current chunk is consumed.
//  * Each part leaves an fp32 (partial output, max, sum) triple per query head;
//    a second kernel merges the parts, one wavefront per (sequence, head).
#include "kernel_params.hpp"

namespace attn {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

constexpr int kChunk = 32;  // keys per wavefront step

template <int HD, int WAVES>
struct DecodeCfg {
    static constexpr int kThreads = WAVES * 64;
    static constexpr int kVPitch = HD * 2 + 64;             // bytes per staged V row
    static constexpr int kVBytes = kChunk * kVPitch;        // per wave
    static constexpr int kRedStride = HD + 2;               // floats per (wave, head) in the final reduction
    static constexpr int kRedBytes = WAVES * 16 * kRedStride * 4;
    static constexpr int kLdsBytes = WAVES * kVBytes > kRedBytes ? WAVES * kVBytes : kRedBytes;
};

template <int HD, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void decode_bf16_kernel(const KParams p)
{
    using C = DecodeCfg<HD, WAVES>;
    constexpr int KS = HD / 32;   // MFMA steps along the head dimension for S^T
    constexpr int DB = HD / 16;   // 16-channel blocks of the output
    constexpr int VLD = kChunk * (HD / 8) / 64;  // 16-byte V loads per lane and chunk
    constexpr int VROWS = 64 / (HD / 8);         // V rows covered by one wave-wide load
    __shared__ __attribute__((aligned(16))) unsigned char lds[C::kLdsBytes];

    // ---- which (KV head, sequence, part) -----------------------------------------------------
    int bid = blockIdx.x;
    const int kvh = bid % p.num_kv_heads;  // fastest: one KV head per XCD when Hkv == 8
    bid /= p.num_kv_heads;
    const int s = bid % p.num_seqs;
    const int part = bid / p.num_seqs;
    const int n_kv = p.seq_lens[s];
    const int k_lo = part * p.split_len;
    if (k_lo >= n_kv && !(part == 0)) return;  // parts past the end write nothing
    const int k_hi = k_lo + p.split_len < n_kv ? k_lo + p.split_len : n_kv;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int l16 = lane & 15;
    const int lg = lane >> 4;  // k-group of the MFMA operands
    const int G = p.group;

    // ---- Q fragment (B operand): lane holds head column l16, channels 32*ks + 8*lg .. +7 ----
    bf16x8 qf[KS];
    {
        const __bf16 *qrow = (const __bf16 *)p.q + (int64_t)s * p.q_stride_tok +
                             (int64_t)(kvh * G + (l16 < G ? l16 : 0)) * p.q_stride_head + 8 * lg;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            bf16x8 t = *(const bf16x8 *)(qrow + 32 * ks);
            if (l16 >= G) {
#pragma unroll
                for (int e = 0; e < 8; ++e) t[e] = (__bf16)0.f;
            }
            qf[ks] = t;
        }
    }

    const __bf16 *kbase = (const __bf16 *)p.k + (int64_t)kvh * p.kv_stride_head;
    const __bf16 *vbase = (const __bf16 *)p.v + (int64_t)kvh * p.kv_stride_head;
    const int32_t *bt_row = p.block_table + (int64_t)s * p.block_table_stride;
    unsigned char *vst = lds + wave * C::kVBytes;

    // element offset of the first row of the 16-key group that starts at key `key` (16 | block_size)
    auto group_offset = [&](int key) -> int64_t {
        key = key < n_kv ? key : (n_kv - 1) & ~15;
        const int blk = bt_row[key >> p.block_shift];
        return (int64_t)blk * p.kv_stride_block + (int64_t)(key & (p.block_size - 1)) * p.kv_stride_tok;
    };

    u32x4 kreg[2][KS], vreg[VLD];
    auto load_chunk = [&](int c0) {
        const int64_t g0 = group_offset(c0), g1 = group_offset(c0 + 16);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const __bf16 *kr = kbase + (t ? g1 : g0) + (int64_t)l16 * p.kv_stride_tok + 8 * lg;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) kreg[t][ks] = *(const u32x4 *)(kr + 32 * ks);
        }
#pragma unroll
        for (int i = 0; i < VLD; ++i) {
            const int row = lane / (HD / 8) + VROWS * i;  // 0..31
            const __bf16 *vr = vbase + (row < 16 ? g0 : g1) + (int64_t)(row & 15) * p.kv_stride_tok + 8 * (lane % (HD / 8));
            vreg[i] = *(const u32x4 *)vr;
        }
    };

    f32x4 oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) oacc[db] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY, l_run = 0.f;

    // transposing V read: lane supplies row 4*lg + (l16/4) [+16] and channels 4*(l16%4) of a 16-channel block
    const int v_rd = (4 * lg + (l16 >> 2)) * C::kVPitch + 8 * (l16 & 3);

    int c0 = k_lo + wave * kChunk;
    if (c0 < k_hi) load_chunk(c0);
    for (; c0 < k_hi; c0 += WAVES * kChunk) {
        // consume the registers of this chunk: K feeds the MFMA directly, V is parked in LDS
        f32x4 sacc[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            sacc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                sacc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kreg[t][ks]), qf[ks], sacc[t], 0, 0, 0);
        }
        const bool tail = c0 + kChunk > k_hi;
#pragma unroll
        for (int i = 0; i < VLD; ++i) {
            const int row = lane / (HD / 8) + VROWS * i;
            // rows past the end may hold anything (even NaN): their weight is 0, so store zeros
            const u32x4 val = (tail && c0 + row >= k_hi) ? u32x4{0u, 0u, 0u, 0u} : vreg[i];
            *(u32x4 *)(vst + row * C::kVPitch + 16 * (lane % (HD / 8))) = val;
        }
        const int next = c0 + WAVES * kChunk;
        if (next < k_hi) load_chunk(next);

        // ---- online softmax over the 32 keys of the chunk -----------------------------------
        float x[8];
        float mloc = -INFINITY;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float y = sacc[t][v] * p.scale_log2e;
                if (tail && c0 + 16 * t + 4 * lg + v >= k_hi) y = -INFINITY;
                x[4 * t + v] = y;
                mloc = fmaxf(mloc, y);
            }
        mloc = fmaxf(mloc, __shfl_xor(mloc, 16));
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
        const float m_new = fmaxf(m_run, mloc);  // finite: key c0 < k_hi is unmasked
        const float alpha = fast_exp2(m_run - m_new);
        m_run = m_new;
        bf16x8 pf;
        float rowsum = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float w = fast_exp2(x[e] - m_new);
            rowsum += w;
            pf[e] = (__bf16)w;
        }
        l_run = l_run * alpha + rowsum;
#pragma unroll
        for (int db = 0; db < DB; ++db) oacc[db] *= alpha;

        // ---- O^T += V^T P^T (wave-private LDS: no barrier, the wave's own writes are ordered) ----
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const unsigned char *a = vst + v_rd + db * 32;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)a);
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(a + 16 * C::kVPitch));
            const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            oacc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, both), pf, oacc[db], 0, 0, 0);
        }
    }

    // ---- merge the wavefronts of this workgroup ----------------------------------------------
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    __syncthreads();  // all waves are done with their V tiles; LDS is reused for the reduction
    float *red = (float *)lds;  // [WAVES][16 heads][HD + 2]
    {
        float *mine = red + (wave * 16 + l16) * C::kRedStride;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int v = 0; v < 4; ++v) mine[db * 16 + 4 * lg + v] = oacc[db][v];
        if (lg == 0) {
            mine[HD] = m_run;
            mine[HD + 1] = l_run;
        }
    }
    __syncthreads();
    // thread -> (head column, channel): G * HD outputs spread over the workgroup
    for (int idx = tid; idx < G * HD; idx += C::kThreads) {
        const int hq = idx / HD, d = idx % HD;
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) M = fmaxf(M, red[(w * 16 + hq) * C::kRedStride + HD]);
        float L = 0.f, O = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) {
            const float *r = red + (w * 16 + hq) * C::kRedStride;
            const float mw = r[HD];
            const float sc = mw == -INFINITY ? 0.f : fast_exp2(mw - M);
            L += r[HD + 1] * sc;
            O += r[d] * sc;
        }
        const int head = kvh * G + hq;
        if (p.num_splits == 1) {
            __bf16 *o = (__bf16 *)p.out + (int64_t)s * p.o_stride_tok + (int64_t)head * p.o_stride_head;
            o[d] = (__bf16)(L > 0.f ? O / L : 0.f);
        } else {
            float *w = p.workspace + (((int64_t)s * p.num_q_heads + head) * p.num_splits + part) * (HD + 2);
            w[d] = O;
            if (d == 0) {
                w[HD] = M;
                w[HD + 1] = L;
            }
        }
    }
}

// One wavefront per (sequence, query head): merges the split-K parts.
//   M = max_s m_s,  L = sum_s l_s 2^(m_s - M),  out = sum_s O_s 2^(m_s - M) / L
// Parts that hold no key were never written and are not read.
template <int HD>
__global__ __launch_bounds__(64) void decode_combine_kernel(const KParams p)
{
    const int head = blockIdx.x % p.num_q_heads;
    const int s = blockIdx.x / p.num_q_heads;
    const int lane = threadIdx.x;
    const int n_kv = p.seq_lens[s];
    int parts = (n_kv + p.split_len - 1) / p.split_len;
    parts = parts < 1 ? 1 : parts;
    const float *w = p.workspace + ((int64_t)s * p.num_q_heads + head) * p.num_splits * (HD + 2);
    float M = -INFINITY;
    for (int i = lane; i < parts; i += 64) M = fmaxf(M, w[i * (HD + 2) + HD]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) M = fmaxf(M, __shfl_xor(M, o));
    float L = 0.f;
    for (int i = lane; i < parts; i += 64) {
        const float mi = w[i * (HD + 2) + HD];
        L += mi == -INFINITY ? 0.f : w[i * (HD + 2) + HD + 1] * fast_exp2(mi - M);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) L += __shfl_xor(L, o);
    constexpr int CPL = HD / 64;
    float acc[CPL];
#pragma unroll
    for (int c = 0; c < CPL; ++c) acc[c] = 0.f;
    for (int i = 0; i < parts; ++i) {
        const float mi = w[i * (HD + 2) + HD];
        const float sc = mi == -INFINITY ? 0.f : fast_exp2(mi - M);
#pragma unroll
        for (int c = 0; c < CPL; ++c) acc[c] += w[i * (HD + 2) + CPL * lane + c] * sc;
    }
    __bf16 *o = (__bf16 *)p.out + (int64_t)s * p.o_stride_tok + (int64_t)head * p.o_stride_head;
    const float inv = L > 0.f ? 1.f / L : 0.f;
#pragma unroll
    for (int c = 0; c < CPL; ++c) o[CPL * lane + c] = (__bf16)(acc[c] * inv);
}

template <int HD, int WAVES>
bool decode_valid(const KParams &p)
{
    return p.head_dim == HD && p.group <= 16 && p.block_table != nullptr && p.block_size >= 16;
}

template <int HD, int WAVES>
hipError_t decode_launch(const KParams &p, hipStream_t stream)
{
    using C = DecodeCfg<HD, WAVES>;
    const int64_t blocks = (int64_t)p.num_kv_heads * p.num_seqs * p.num_splits;
    if (blocks <= 0) return hipSuccess;
    if (blocks > 0x7fffffff) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((decode_bf16_kernel<HD, WAVES>), dim3((unsigned)blocks), dim3(C::kThreads), 0, stream, p);
    return hipGetLastError();
}

#define DECODE_INSTANCE(HD, WAVES, SPLIT)                                                                     \
    {                                                                                                         \
        "decode_bf16 d" #HD " w" #WAVES " split" #SPLIT, 16, kChunk, WAVES, 16, 2, SPLIT, decode_valid<HD, WAVES>, \
            decode_launch<HD, WAVES>                                                                          \
    }

}  // namespace

hipError_t launch_decode_combine(const KParams &p, hipStream_t stream)
{
    const int64_t blocks = (int64_t)p.num_seqs * p.num_q_heads;
    if (blocks <= 0) return hipSuccess;
    if (blocks > 0x7fffffff) return hipErrorInvalidConfiguration;
    if (p.head_dim == 128)
        hipLaunchKernelGGL(decode_combine_kernel<128>, dim3((unsigned)blocks), dim3(64), 0, stream, p);
    else if (p.head_dim == 64)
        hipLaunchKernelGGL(decode_combine_kernel<64>, dim3((unsigned)blocks), dim3(64), 0, stream, p);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

const Instance *decode_instances(int *count)
{
    static const Instance table[] = {
        DECODE_INSTANCE(128, 4, 0),    DECODE_INSTANCE(128, 4, 256),  DECODE_INSTANCE(128, 4, 512),
        DECODE_INSTANCE(128, 4, 1024), DECODE_INSTANCE(128, 4, 2048), DECODE_INSTANCE(128, 4, 4096),
        DECODE_INSTANCE(128, 8, 0),    DECODE_INSTANCE(128, 8, 512),  DECODE_INSTANCE(128, 8, 1024),
        DECODE_INSTANCE(128, 8, 2048), DECODE_INSTANCE(128, 8, 4096), DECODE_INSTANCE(128, 2, 256),
        DECODE_INSTANCE(128, 2, 512),  DECODE_INSTANCE(128, 2, 1024), DECODE_INSTANCE(64, 4, 0),
        DECODE_INSTANCE(64, 4, 512),   DECODE_INSTANCE(64, 4, 2048),
    };
    *count = (int)(sizeof(table) / sizeof(table[0]));
    return table;
}

}  // namespace attn

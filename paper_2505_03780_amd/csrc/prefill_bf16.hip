// Causal variable-length prefill on bf16 MFMA (gfx950), contiguous or paged K/V.
//
// The method is the tiled online-softmax attention (FlashAttention-2) that the
// paper's kernel implements (section "Method and Investigated Kernels"; Fig. 2:
// causal, variable-length batches, Llama3-8B head shapes).  The layout below is
// this library's own design for CDNA4:
//
//  * A workgroup owns a tile of query rows that all read the same keys: HPW
//    query heads of one KV head (grouped-query attention) times TSUB token
//    sub-tiles; each wavefront owns 32*QB tokens of one head.
//  * Scores are computed transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16:
//    a lane then holds 16 keys of ONE query column, so row max / row sum are
//    lane-local plus one exchange with lane^32, and the fp32 result, packed to
//    bf16, already is the B operand of the second product O^T += V^T P^T.
//  * K/V tiles are staged in LDS (double buffered, one barrier per tile); K is
//    read back with 128-bit reads in A-operand order, V with the gfx950
//    transposing read (ds_read_b64_tr_b16), so V is never transposed in memory.
//  * Keys are addressed through the block table when one is given; rows past
//    the end of a sequence are clamped to its last key and masked.
#include "kernel_params.hpp"

namespace attn {
namespace {

// This file is compiled twice: as it stands for bf16, and included by prefill_f16.hip with
// ATTN_PREFILL_ELEM_F16 defined for fp16 (the element type only changes the MFMA opcode and the
// conversions of weights and outputs; a smaller set of instances is built).
#ifdef ATTN_PREFILL_ELEM_F16
typedef _Float16 elem_t;
#define PREFILL_MFMA __builtin_amdgcn_mfma_f32_32x32x16_f16
#define PREFILL_NAME "prefill_f16"
constexpr int kElemDtype = kDtypeF16;
#else
typedef __bf16 elem_t;
#define PREFILL_MFMA __builtin_amdgcn_mfma_f32_32x32x16_bf16
#define PREFILL_NAME "prefill_bf16"
constexpr int kElemDtype = kDtypeBf16;
#endif
typedef elem_t ex8 __attribute__((ext_vector_type(8)));
typedef elem_t ex4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int HD, int BN, int QB, int WAVES, int HPW>
struct PrefillCfg {
    static constexpr int kTSub = WAVES / HPW;    // token sub-tiles per workgroup
    static constexpr int kWaveTok = 32 * QB;     // tokens per wavefront
    static constexpr int kTok = kTSub * kWaveTok;  // tokens per workgroup
    static constexpr int kThreads = WAVES * 64;
    static constexpr int kKPitch = HD * 2 + 16;  // bytes; 16 consecutive rows hit 16 distinct 4-bank groups
    static constexpr int kVPitch = HD * 2 + 64;  // bytes; 4 consecutive rows hit 4 distinct 16-bank groups
    static constexpr int kChunksPerRow = HD / 8;  // 16-byte chunks
    static constexpr int kLoadIters = BN * kChunksPerRow / kThreads;
    static constexpr int kRowsPerIter = kThreads / kChunksPerRow;
    static constexpr size_t kLdsBytes = 2 * (size_t)BN * (kKPitch + kVPitch);
    static_assert(WAVES % HPW == 0, "waves must split evenly over heads");
    static_assert(BN * kChunksPerRow % kThreads == 0, "tile must split evenly over threads");
    static_assert(BN % 32 == 0 && HD % 32 == 0, "MFMA tile sizes");
};

template <int HD, int BN, int QB, int WAVES, int HPW>
__global__ __launch_bounds__(WAVES * 64) void prefill_bf16_kernel(const KParams p)
{
    using C = PrefillCfg<HD, BN, QB, WAVES, HPW>;
    constexpr int KSTEPS = HD / 16;
    constexpr int DB = HD / 32;
    constexpr int KB = BN / 32;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    unsigned char *lds_k = lds;                              // [2][BN][kKPitch]
    unsigned char *lds_v = lds + 2 * BN * C::kKPitch;        // [2][BN][kVPitch]

    // ---- which (head group, sequence, query tile) is this workgroup -----------------------
    const int groups_per_kvh = p.group / HPW;
    const int nhg = p.num_kv_heads * groups_per_kvh;
    int bid = blockIdx.x;
    const int hg = bid % nhg;  // fastest: workgroups of one KV head land on one XCD when Hkv == 8
    bid /= nhg;
    // Tile level outermost, counted down from the longest sequence's last tile (costly tiles first, in
    // every sequence at the same time); the sequence index rotates with the level, because inside an
    // XCD workgroups are dealt to the four shader engines round-robin by index and a fixed map would
    // give one engine all tiles of a long sequence.
    const int q_tiles = (p.max_q_len + C::kTok - 1) / C::kTok;  // the grid's tile dimension
    const int r = bid / p.num_seqs;
    const int s = (bid % p.num_seqs + r) % p.num_seqs;
    const int kvh = hg % p.num_kv_heads;
    const int hsub = hg / p.num_kv_heads;

    const int q0 = p.query_start_loc[s];
    const int n_q = p.query_start_loc[s + 1] - q0;
    const int n_kv = p.seq_lens[s];
    const int off = n_kv - n_q;
    const int n_tiles_q = (n_q + C::kTok - 1) / C::kTok;
    const int qtile = q_tiles - 1 - r;
    if (qtile < 0 || qtile >= n_tiles_q) return;
    const int t0 = qtile * C::kTok;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int lhalf = lane >> 5;  // which half-wave: selects the k-group of MFMA operands
    const int l32 = lane & 31;
    const int head = kvh * p.group + hsub * HPW + (wave % HPW);
    const int t0w = t0 + (wave / HPW) * C::kWaveTok;

    // ---- Q fragments (B operand of S^T = K Q^T): lane holds query column l32, 8 channels ----
    const elem_t *qbase = (const elem_t *)p.q;
    ex8 qf[QB][KSTEPS];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        int t = t0w + qb * 32 + l32;
        t = t < n_q ? t : n_q - 1;
        const elem_t *src = qbase + (int64_t)(q0 + t) * p.q_stride_tok + (int64_t)head * p.q_stride_head + 8 * lhalf;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) qf[qb][ks] = *(const ex8 *)(src + 16 * ks);
    }

    // ---- key range of this workgroup ---------------------------------------------------------
    int kv_end = n_kv;
    if (p.causal) {
        int last_tok = t0 + C::kTok < n_q ? t0 + C::kTok : n_q;
        kv_end = off + last_tok < n_kv ? off + last_tok : n_kv;
    }
    const int n_tiles = (kv_end + BN - 1) / BN;
    // positions of this wave's queries on the key axis (bottom-right aligned causal mask)
    const int qpos_lo = p.causal ? off + t0w : 0x7fffffff - 64;
    int qpos[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) qpos[qb] = p.causal ? off + t0w + qb * 32 + l32 : 0x7fffffff;

    // ---- K/V tile loader: thread -> (row, 16-byte chunk) ------------------------------------
    const int ld_chunk = tid % C::kChunksPerRow;
    const int ld_row = tid / C::kChunksPerRow;
    const elem_t *kbase = (const elem_t *)p.k;
    const elem_t *vbase = (const elem_t *)p.v;
    const int kv0 = p.block_table ? 0 : p.kv_start_loc[s];
    const int32_t *bt_row = p.block_table ? p.block_table + (int64_t)s * p.block_table_stride : nullptr;
    auto row_offset = [&](int row) -> int64_t {
        row = row < n_kv ? row : n_kv - 1;
        int64_t o;
        if (bt_row) {
            const int blk = bt_row[row >> p.block_shift];
            o = (int64_t)blk * p.kv_stride_block + (int64_t)(row & (p.block_size - 1)) * p.kv_stride_tok;
        } else {
            o = (int64_t)(kv0 + row) * p.kv_stride_tok;
        }
        return o + (int64_t)kvh * p.kv_stride_head + 8 * ld_chunk;
    };
    u32x4 kreg[C::kLoadIters], vreg[C::kLoadIters];
    auto load_tile = [&](int tile) {
#pragma unroll
        for (int i = 0; i < C::kLoadIters; ++i) {
            const int64_t o = row_offset(tile * BN + ld_row + i * C::kRowsPerIter);
            kreg[i] = *(const u32x4 *)(kbase + o);
            vreg[i] = *(const u32x4 *)(vbase + o);
        }
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int i = 0; i < C::kLoadIters; ++i) {
            const int row = ld_row + i * C::kRowsPerIter;
            *(u32x4 *)(lds_k + (buf * BN + row) * C::kKPitch + 16 * ld_chunk) = kreg[i];
            *(u32x4 *)(lds_v + (buf * BN + row) * C::kVPitch + 16 * ld_chunk) = vreg[i];
        }
    };

    // ---- accumulators ------------------------------------------------------------------------
    f32x16 oacc[QB][DB];
    float m_run[QB], l_run[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        m_run[qb] = -INFINITY;
        l_run[qb] = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) oacc[qb][db][v] = 0.f;
    }

    if (n_tiles > 0) {
        load_tile(0);
        store_tile(0);
    }
    __syncthreads();

    // per-lane LDS read offsets
    const int k_rd = l32 * C::kKPitch + 16 * lhalf;  // + kb*32*pitch + 32*ks bytes
    // transposing V read: lane supplies row (lane%16)/4 (+4*lhalf) and 4 channels at 4*(lane%4) + 16*((lane/16)%2)
    const int v_rd = (((lane & 15) >> 2) + 4 * lhalf) * C::kVPitch + (4 * (lane & 3) + 16 * ((lane >> 4) & 1)) * 2;

    for (int j = 0; j < n_tiles; ++j) {
        const int buf = j & 1;
        const int tile0 = j * BN;
        if (j + 1 < n_tiles) load_tile(j + 1);

        // a wave whose queries all precede this tile has nothing to do in it (token-packed mode)
        const bool active = tile0 <= qpos_lo + C::kWaveTok - 1;
        if (active) {
            // ---- S^T = K Q^T -----------------------------------------------------------------
            f32x16 sacc[QB][KB];
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) sacc[qb][kb][v] = 0.f;
            const unsigned char *kt = lds_k + buf * BN * C::kKPitch + k_rd;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
                for (int ks = 0; ks < KSTEPS; ++ks) {
                    const ex8 kf = *(const ex8 *)(kt + kb * 32 * C::kKPitch + 32 * ks);
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb)
                        sacc[qb][kb] = PREFILL_MFMA(kf, qf[qb][ks], sacc[qb][kb], 0, 0, 0);
                }
            }

            // ---- mask + online softmax ---------------------------------------------------------
            const bool need_mask = (tile0 + BN - 1 > qpos_lo) || (tile0 + BN > n_kv);
            ex8 pf[QB][KB][2];
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                float mloc = -INFINITY;
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        float x = sacc[qb][kb][v] * p.scale_log2e;
                        if (need_mask) {
                            const int kvi = tile0 + kb * 32 + 8 * (v >> 2) + 4 * lhalf + (v & 3);
                            if (kvi > qpos[qb] || kvi >= n_kv) x = -INFINITY;
                        }
                        sacc[qb][kb][v] = x;
                        mloc = fmaxf(mloc, x);
                    }
                }
                mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
                const float m_new = fmaxf(m_run[qb], mloc);
                const float m_use = m_new == -INFINITY ? 0.f : m_new;
                const float alpha = fast_exp2(m_run[qb] - m_use);
                m_run[qb] = m_new;
                float rowsum = 0.f;
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const float e = fast_exp2(sacc[qb][kb][v] - m_use);
                        rowsum += e;
                        pf[qb][kb][v >> 3][v & 7] = (elem_t)e;
                    }
                }
                l_run[qb] = l_run[qb] * alpha + rowsum;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int v = 0; v < 16; ++v) oacc[qb][db][v] *= alpha;
            }

            // ---- O^T += V^T P^T ----------------------------------------------------------------
            const unsigned char *vt = lds_v + buf * BN * C::kVPitch + v_rd;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
                    for (int db = 0; db < DB; ++db) {
                        const unsigned char *a = vt + (kb * 32 + 16 * ks) * C::kVPitch + db * 64;
                        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)a);
                        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(a + 8 * C::kVPitch));
                        const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                        const ex8 vf = __builtin_bit_cast(ex8, both);
#pragma unroll
                        for (int qb = 0; qb < QB; ++qb)
                            oacc[qb][db] = PREFILL_MFMA(vf, pf[qb][kb][ks], oacc[qb][db], 0, 0, 0);
                    }
                }
            }
        }

        if (j + 1 < n_tiles) store_tile(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: O / l -> bf16 -------------------------------------------------------------
    elem_t *obase = (elem_t *)p.out;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float l = l_run[qb] + __shfl_xor(l_run[qb], 32);
        const float inv = l > 0.f ? 1.f / l : 0.f;
        const int t = t0w + qb * 32 + l32;
        if (t < n_q) {
            elem_t *dst = obase + (int64_t)(q0 + t) * p.o_stride_tok + (int64_t)head * p.o_stride_head + 4 * lhalf;
#pragma unroll
            for (int db = 0; db < DB; ++db) {
#pragma unroll
                for (int vq = 0; vq < 4; ++vq) {
                    ex4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = (elem_t)(oacc[qb][db][4 * vq + e] * inv);
                    *(ex4 *)(dst + db * 32 + 8 * vq) = o;
                }
            }
        }
    }
}

template <int HD, int BN, int QB, int WAVES, int HPW>
bool prefill_valid(const KParams &p)
{
    return p.dtype == kElemDtype && p.head_dim == HD && p.group % HPW == 0;
}

template <int HD, int BN, int QB, int WAVES, int HPW>
hipError_t prefill_launch(const KParams &p, hipStream_t stream)
{
    using C = PrefillCfg<HD, BN, QB, WAVES, HPW>;
    auto kern = prefill_bf16_kernel<HD, BN, QB, WAVES, HPW>;
    static hipError_t attr = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::kLdsBytes);
    if (attr != hipSuccess) return attr;
    const int64_t q_tiles = (p.max_q_len + C::kTok - 1) / C::kTok;
    const int64_t nhg = (int64_t)p.num_kv_heads * (p.group / HPW);
    const int64_t blocks = q_tiles * p.num_seqs * nhg;
    if (blocks <= 0) return hipSuccess;
    if (blocks > 0x7fffffff) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(C::kThreads), C::kLdsBytes, stream, p);
    return hipGetLastError();
}

#define PREFILL_INSTANCE(HD, BN, QB, WAVES, HPW)                                                              \
    {                                                                                                         \
        PREFILL_NAME " d" #HD " bn" #BN " qb" #QB " w" #WAVES " hpw" #HPW, (WAVES / HPW) * 32 * QB * HPW, BN,  \
            WAVES, HPW, 2, 0, prefill_valid<HD, BN, QB, WAVES, HPW>, prefill_launch<HD, BN, QB, WAVES, HPW>     \
    }

}  // namespace

#ifdef ATTN_PREFILL_ELEM_F16
const Instance *prefill_staged_f16_instances(int *count)
{
    static const Instance table[] = {
        PREFILL_INSTANCE(128, 64, 1, 4, 4), PREFILL_INSTANCE(128, 64, 1, 4, 1), PREFILL_INSTANCE(128, 64, 1, 8, 8),
        PREFILL_INSTANCE(64, 64, 2, 4, 4),  PREFILL_INSTANCE(64, 64, 2, 4, 2),  PREFILL_INSTANCE(64, 64, 2, 4, 1),
        PREFILL_INSTANCE(64, 128, 2, 4, 1),
    };
    *count = (int)(sizeof(table) / sizeof(table[0]));
    return table;
}
#else
const Instance *prefill_staged_instances(int *count)
{
    // Built inside a host function so that the table of host function pointers is not
    // emitted for the device.
    static const Instance table[] = {
        PREFILL_INSTANCE(128, 64, 2, 4, 4),
        PREFILL_INSTANCE(128, 64, 2, 4, 2),
        PREFILL_INSTANCE(128, 64, 2, 4, 1),
        PREFILL_INSTANCE(128, 64, 1, 4, 4),
        PREFILL_INSTANCE(128, 64, 1, 4, 2),
        PREFILL_INSTANCE(128, 64, 1, 4, 1),
        PREFILL_INSTANCE(128, 64, 1, 8, 8),
        PREFILL_INSTANCE(128, 64, 1, 8, 4),
        PREFILL_INSTANCE(128, 64, 1, 8, 1),
        PREFILL_INSTANCE(128, 128, 1, 4, 4),
        PREFILL_INSTANCE(128, 128, 1, 4, 1),
        PREFILL_INSTANCE(64, 64, 2, 4, 4),
        PREFILL_INSTANCE(64, 64, 2, 4, 2),
        PREFILL_INSTANCE(64, 64, 2, 4, 1),
        PREFILL_INSTANCE(64, 128, 2, 4, 1),
    };
    *count = (int)(sizeof(table) / sizeof(table[0]));
    return table;
}

#endif

}  // namespace attn

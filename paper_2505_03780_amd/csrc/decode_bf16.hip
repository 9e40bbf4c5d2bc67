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
//  * K and V rows are fetched as whole head slices (four rows x 256 contiguous
//    bytes per wave-wide 128-bit load at D = 128) with the non-temporal hint:
//    every byte is read once, and a load that covers only half of a 128-byte
//    line (as MFMA operand order would) pays for the line twice under that hint.
//    A wave-private LDS tile turns K into A-operand order (plain 128-bit reads)
//    and then V into key-contiguous operands (ds_read_b64_tr_b16).  The next
//    chunk's loads are issued before the current chunk is consumed.
//  * Each part leaves an fp32 (partial output, max, sum) triple per query head;
//    a second kernel merges the parts, one wavefront per (sequence, head).
//
// Three kernels share these pieces (each is described where it is defined):
// decode_bf16_kernel, the one sketched above; decode_seq_kernel, one wavefront
// per KV head so that a workgroup fetches whole cache blocks; and
// decode_balanced_kernel, which deals the batch's 32-key chunks out evenly over
// one workgroup per compute unit whatever the mix of lengths.  The last two
// stream through decode_stream_run.
#include "kernel_params.hpp"

namespace attn {
namespace {

// This file is compiled twice: as it stands for bf16, and included by decode_f16.hip with
// ATTN_DECODE_ELEM_F16 defined for fp16 caches (the element type only changes the MFMA opcode and the
// conversions of weights and outputs; a smaller set of instances is built).
#ifdef ATTN_DECODE_ELEM_F16
typedef _Float16 elem_t;
#define DECODE_MFMA __builtin_amdgcn_mfma_f32_16x16x32_f16
#define DECODE_NAME "decode_f16"
constexpr int kElemDtype = kDtypeF16;
#else
typedef __bf16 elem_t;
#define DECODE_MFMA __builtin_amdgcn_mfma_f32_16x16x32_bf16
#define DECODE_NAME "decode_bf16"
constexpr int kElemDtype = kDtypeBf16;
#endif
typedef elem_t ex8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// K and V are read exactly once per call: the loads carry the non-temporal hint so that the stream
// does not displace the caches' contents (measured on a 2 GiB read: 7.1 TB/s with the hint, 6.2 without)
__device__ __forceinline__ u32x4 kv_load(const void *src)
{
    return __builtin_nontemporal_load((const u32x4 *)src);
}

constexpr int kChunk = 32;  // keys per wavefront step

template <int HD, int WAVES>
struct DecodeCfg {
    static constexpr int kThreads = WAVES * 64;
    static constexpr int kVPitch = HD * 2 + 64;             // bytes per staged V row
    static constexpr int kVBytes = kChunk * kVPitch;        // per wave
    static constexpr int kKPitch = HD * 2 + 16;             // bytes per staged K row (same tile, before V)
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
    // The sequence index rotates with the part index: workgroups are dealt to XCDs, and inside an XCD to
    // its shader engines, round-robin by index, so a fixed map would pin every part of a long sequence
    // to one engine.
    const int part = bid / p.num_seqs;
    const int s = (bid % p.num_seqs + part) % p.num_seqs;
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
    ex8 qf[KS];
    {
        const elem_t *qrow = (const elem_t *)p.q + (int64_t)s * p.q_stride_tok +
                             (int64_t)(kvh * G + (l16 < G ? l16 : 0)) * p.q_stride_head + 8 * lg;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            ex8 t = *(const ex8 *)(qrow + 32 * ks);
            if (l16 >= G) {
#pragma unroll
                for (int e = 0; e < 8; ++e) t[e] = (elem_t)0.f;
            }
            qf[ks] = t;
        }
    }

    const elem_t *kbase = (const elem_t *)p.k + (int64_t)kvh * p.kv_stride_head;
    const elem_t *vbase = (const elem_t *)p.v + (int64_t)kvh * p.kv_stride_head;
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
            // whole head slices (four rows x 256 bytes per wave-wide load at D = 128), like V
#pragma unroll
            for (int i = 0; i < KS; ++i) {
                const int row = lane / (HD / 8) + VROWS * i;  // 0..15
                kreg[t][i] = kv_load(kbase + (t ? g1 : g0) + (int64_t)row * p.kv_stride_tok + 8 * (lane % (HD / 8)));
            }
        }
#pragma unroll
        for (int i = 0; i < VLD; ++i) {
            const int row = lane / (HD / 8) + VROWS * i;  // 0..31
            const elem_t *vr = vbase + (row < 16 ? g0 : g1) + (int64_t)(row & 15) * p.kv_stride_tok + 8 * (lane % (HD / 8));
            vreg[i] = kv_load(vr);
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
        // consume the registers of this chunk: K, then V, pass through the wave's LDS tile
        f32x4 sacc[2];
        // the wave's LDS tile turns the K rows into MFMA operand order; V takes the tile over below
        // (LDS instructions of one wave execute in order, so no wait is needed between the two uses)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int i = 0; i < KS; ++i) {
                const int row = 16 * t + lane / (HD / 8) + VROWS * i;
                *(u32x4 *)(vst + row * C::kKPitch + 16 * (lane % (HD / 8))) = kreg[t][i];
            }
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            sacc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const ex8 kf = *(const ex8 *)(vst + (16 * t + l16) * C::kKPitch + 16 * lg + 64 * ks);
                sacc[t] = DECODE_MFMA(kf, qf[ks], sacc[t], 0, 0, 0);
            }
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
        ex8 pf;
        float rowsum = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float w = fast_exp2(x[e] - m_new);
            rowsum += w;
            pf[e] = (elem_t)w;
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
            oacc[db] = DECODE_MFMA(__builtin_bit_cast(ex8, both), pf, oacc[db], 0, 0, 0);
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
            elem_t *o = (elem_t *)p.out + (int64_t)s * p.o_stride_tok + (int64_t)head * p.o_stride_head;
            o[d] = (elem_t)(L > 0.f ? O / L : 0.f);
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

// Streams a run of `nrun` 32-key chunks for KV head kvh through one wavefront.  The run starts `off0`
// chunks into sequence s0 and may go on through any number of following sequences (the token-balanced
// kernel's unit of work; the wave-per-head kernel passes one part of one sequence).  The chunks a run
// takes from one sequence are a piece; a piece ends with the sequence or with the run.
// Each piece leaves either fp32 (partial output, max, sum) records, the one of query head h at
// record(s, whole) + h * head_stride, or, where record(s, whole) returns null, the final output row
// (`whole` says that the piece holds every key of sequence s).
// The load pipeline does not stop where one sequence ends and the next begins: the chunks of the next
// piece are requested two steps ahead like any others, so all a wavefront waits for at a boundary is
// the next sequence's query row.  Sequences without keys inside the run are skipped.
template <int HD, int WAVES, class Record>
__device__ __forceinline__ void decode_stream_run(const KParams &p, unsigned char *vst, int lane, int kvh, int s0, int off0, int nrun,
                                                  Record record, int64_t head_stride)
{
    using C = DecodeCfg<HD, WAVES>;
    constexpr int KS = HD / 32;
    constexpr int DB = HD / 16;
    constexpr int VLD = kChunk * (HD / 8) / 64;
    constexpr int VROWS = 64 / (HD / 8);
    typedef const __attribute__((address_space(4))) int32_t *table_ptr;  // read-only, scalar loads
    const int l16 = lane & 15;
    const int lg = lane >> 4;
    const int G = p.group;
    const int B = p.num_seqs;
    const unsigned char *kbase = (const unsigned char *)p.k + (int64_t)kvh * p.kv_stride_head * 2;
    const unsigned char *vbase = (const unsigned char *)p.v + (int64_t)kvh * p.kv_stride_head * 2;
    const uint32_t tok_bytes = (uint32_t)p.kv_stride_tok * 2;
    table_ptr lens = (table_ptr)p.seq_lens;

    // per-lane byte offsets inside a 16-key group, the same for K and V: whole head slices, fully coalesced
    uint32_t v_lane[VLD];
#pragma unroll
    for (int i = 0; i < VLD; ++i) {
        const int row = lane / (HD / 8) + VROWS * i;
        v_lane[i] = (uint32_t)(row & 15) * tok_bytes + 16 * (lane % (HD / 8));
    }

    // ---- load cursor: the chunk whose addresses are worked out next ---------------------------------
    int ld_s = s0, ld_key = off0 * kChunk, ld_left = nrun;  // sequence, first key of the chunk, chunks still to address
    int ld_nkv = lens[s0];
    table_ptr ld_row = (table_ptr)(p.block_table + (int64_t)s0 * p.block_table_stride);
    struct Bases {
        int64_t g0, g1;
    };
    // byte offsets (wave-uniform) of the two 16-key groups of the next chunk of the run; groups past the
    // end of their sequence fall back to its last real group, whose rows are allocated (and masked)
    auto next_bases = [&]() -> Bases {
        if (ld_left <= 0) return Bases{0, 0};
        const int last_group = (ld_nkv - 1) & ~15;
        auto base = [&](int key) -> int64_t {
            key = key < last_group ? key : last_group;
            const int blk = ld_row[key >> p.block_shift];
            return (int64_t)blk * p.kv_stride_block * 2 + (int64_t)(key & (p.block_size - 1)) * tok_bytes;
        };
        const Bases b{base(ld_key), base(ld_key + 16)};
        ld_key += kChunk;
        --ld_left;
        if (ld_key >= ld_nkv && ld_left > 0) {  // on to the next sequence that has keys
            do {
                ++ld_s;
                ld_nkv = lens[ld_s < B ? ld_s : B - 1];
            } while (ld_nkv <= 0 && ld_s < B - 1);
            if (ld_nkv <= 0) ld_left = 0;  // (lengths that changed under the kernel: stop rather than run on)
            ld_row = (table_ptr)(p.block_table + (int64_t)ld_s * p.block_table_stride);
            ld_key = 0;
        }
        return b;
    };

    struct Regs {
        u32x4 k[2][KS];
        u32x4 v[VLD];
    };
    auto load = [&](Regs &r, const Bases &b) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
#pragma unroll
            for (int i = 0; i < KS; ++i) r.k[t][i] = kv_load(kbase + (t ? b.g1 : b.g0) + v_lane[i]);
        }
#pragma unroll
        for (int i = 0; i < VLD; ++i) {
            const int row = lane / (HD / 8) + VROWS * i;
            r.v[i] = kv_load(vbase + (row < 16 ? b.g0 : b.g1) + v_lane[i]);
        }
    };

    // ---- consume cursor: the piece whose chunks are being multiplied --------------------------------
    int cs = s0 - 1, c_key = 0, c_hi = 0, c_left = nrun;  // sequence, next key, end of the piece, chunks still to consume
    bool c_whole = false;
    int c_off = off0;
    ex8 qf[KS];
    f32x4 oacc[DB];
    float m_run = -INFINITY, l_run = 0.f;
    auto begin_piece = [&]() {
        int n_kv;
        do {
            ++cs;
            n_kv = lens[cs < B ? cs : B - 1];
        } while (n_kv <= 0 && cs < B - 1);
        const int nc = (n_kv + kChunk - 1) / kChunk;
        const int n = c_left < nc - c_off ? c_left : nc - c_off;
        c_key = c_off * kChunk;
        c_hi = (c_off + n) * kChunk < n_kv ? (c_off + n) * kChunk : n_kv;
        c_whole = n == nc;
        c_off = 0;
        const elem_t *qrow = (const elem_t *)p.q + (int64_t)cs * p.q_stride_tok + (int64_t)(kvh * G + (l16 < G ? l16 : 0)) * p.q_stride_head + 8 * lg;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            ex8 t = *(const ex8 *)(qrow + 32 * ks);
            if (l16 >= G) {
#pragma unroll
                for (int e = 0; e < 8; ++e) t[e] = (elem_t)0.f;
            }
            qf[ks] = t;
        }
#pragma unroll
        for (int db = 0; db < DB; ++db) oacc[db] = f32x4{0.f, 0.f, 0.f, 0.f};
        m_run = -INFINITY;
        l_run = 0.f;
    };
    // this wave's result for the piece: G heads x HD channels, no other wave involved
    auto end_piece = [&]() {
        float l_all = l_run + __shfl_xor(l_run, 16);
        l_all += __shfl_xor(l_all, 32);
        float *rec_base = record(cs, c_whole);
        if (l16 < G) {
            const int head = kvh * G + l16;
            if (rec_base == nullptr) {
                elem_t *o = (elem_t *)p.out + (int64_t)cs * p.o_stride_tok + (int64_t)head * p.o_stride_head;
                const float inv = l_all > 0.f ? 1.f / l_all : 0.f;
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    typedef elem_t ex4 __attribute__((ext_vector_type(4)));
                    ex4 o4;
#pragma unroll
                    for (int v = 0; v < 4; ++v) o4[v] = (elem_t)(oacc[db][v] * inv);
                    *(ex4 *)(o + db * 16 + 4 * lg) = o4;
                }
            } else {
                float *rec = rec_base + (int64_t)head * head_stride;
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    // (HD + 2) floats per record: 8-byte aligned, so two 8-byte stores per block of 4
                    *(float2 *)(rec + db * 16 + 4 * lg) = float2{oacc[db][0], oacc[db][1]};
                    *(float2 *)(rec + db * 16 + 4 * lg + 2) = float2{oacc[db][2], oacc[db][3]};
                }
                if (lg == 0) *(float2 *)(rec + HD) = float2{m_run, l_all};
            }
        }
    };

    const int v_rd = (4 * lg + (l16 >> 2)) * C::kVPitch + 8 * (l16 & 3);
    f32x4 sacc[2];
    // consume: the chunk leaves its registers (K through the wave's LDS tile into the score MFMAs, V into
    // the tile), so the same registers can take the loads of the chunk after next right away
    auto consume = [&](Regs &r, int c0) {
        // K rows arrive as whole head slices (V's wave-wide shape); the wave's LDS tile turns them into
        // MFMA operand order.  The tile is shared with V: LDS instructions of a wave execute in order,
        // so these writes follow the previous chunk's V reads and the V writes below follow the K reads.
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int i = 0; i < KS; ++i) {
                const int row = 16 * t + lane / (HD / 8) + VROWS * i;
                *(u32x4 *)(vst + row * C::kKPitch + 16 * (lane % (HD / 8))) = r.k[t][i];
            }
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            sacc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const ex8 kf = *(const ex8 *)(vst + (16 * t + l16) * C::kKPitch + 16 * lg + 64 * ks);
                sacc[t] = DECODE_MFMA(kf, qf[ks], sacc[t], 0, 0, 0);
            }
        }
        const bool tail = c0 + kChunk > c_hi;
#pragma unroll
        for (int i = 0; i < VLD; ++i) {
            const int row = lane / (HD / 8) + VROWS * i;
            // rows past the end may hold anything (even NaN): their weight is 0, so store zeros
            const u32x4 val = (tail && c0 + row >= c_hi) ? u32x4{0u, 0u, 0u, 0u} : r.v[i];
            *(u32x4 *)(vst + row * C::kVPitch + 16 * (lane % (HD / 8))) = val;
        }
    };
    auto finish = [&](int c0) {
        const bool tail = c0 + kChunk > c_hi;
        float x[8];
        float mloc = -INFINITY;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float y = sacc[t][v] * p.scale_log2e;
                if (tail && c0 + 16 * t + 4 * lg + v >= c_hi) y = -INFINITY;
                x[4 * t + v] = y;
                mloc = fmaxf(mloc, y);
            }
        mloc = fmaxf(mloc, __shfl_xor(mloc, 16));
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
        const float m_new = fmaxf(m_run, mloc);  // finite: key c0 < c_hi is unmasked
        const float alpha = fast_exp2(m_run - m_new);
        m_run = m_new;
        ex8 pf;
        float rowsum = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float wgt = fast_exp2(x[e] - m_new);
            rowsum += wgt;
            pf[e] = (elem_t)wgt;
        }
        l_run = l_run * alpha + rowsum;
#pragma unroll
        for (int db = 0; db < DB; ++db) oacc[db] *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const unsigned char *a = vst + v_rd + db * 32;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)a);
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(a + 16 * C::kVPitch));
            const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            oacc[db] = DECODE_MFMA(__builtin_bit_cast(ex8, both), pf, oacc[db], 0, 0, 0);
        }
    };
    // One chunk of the run: multiply, reload the freed registers with the chunk after next, and close
    // the piece if this was its last chunk.  Two register sets alternate, so about two chunks (32 KB
    // per wave) are in flight; the addresses of the chunk that is loaded next are worked out (scalar
    // loads of table entries) one step before they are needed.
    Bases gn;
    auto step = [&](Regs &r, bool reload) {
        const Bases t = next_bases();
        const int c0 = c_key;
        consume(r, c0);
        if (reload) load(r, gn);
        gn = t;
        finish(c0);
        c_key += kChunk;
        --c_left;
        if (c_key >= c_hi) {
            end_piece();
            if (c_left > 0) begin_piece();
        }
    };

    Regs ra, rb;
    {
        const Bases a = next_bases(), b = next_bases();
        if (nrun > 0) load(ra, a);
        if (nrun > 1) load(rb, b);
        gn = next_bases();
    }
    begin_piece();
    for (int g = 0; g < nrun; g += 2) {
        step(ra, g + 2 < nrun);
        if (g + 1 < nrun) step(rb, g + 3 < nrun);
    }
}

// The result of a part that holds no key (an empty context): zeros as output, or a record with
// m = -inf and l = 0.  No table entry is touched.
template <int HD>
__device__ __forceinline__ void decode_write_empty(const KParams &p, int lane, int s, int kvh, float *partial_base, int64_t head_stride)
{
    const int l16 = lane & 15;
    const int lg = lane >> 4;
    if (l16 >= p.group) return;
    const int head = kvh * p.group + l16;
    if (partial_base == nullptr) {
        elem_t *o = (elem_t *)p.out + (int64_t)s * p.o_stride_tok + (int64_t)head * p.o_stride_head;
        for (int d = 4 * lg; d < HD; d += 16) *(uint2 *)(o + d) = uint2{0u, 0u};
    } else {
        float *w = partial_base + (int64_t)head * head_stride;
        for (int d = 4 * lg; d < HD; d += 16) {
            *(float2 *)(w + d) = float2{0.f, 0.f};
            *(float2 *)(w + d + 2) = float2{0.f, 0.f};
        }
        if (lg == 0) *(float2 *)(w + HD) = float2{-INFINITY, 0.f};
    }
}

// Variant that keeps a whole KV-cache block together: a workgroup owns (sequence, part) and its
// wavefront w owns KV head w, so the eight 256-byte head slices of a token row are fetched by one
// workgroup at about the same time (whole 32 KB blocks per 16 keys instead of scattered slices), and
// no wavefront ever waits for another: there is no barrier and no cross-wave reduction.  A part is a
// run of chunks inside one sequence (decode_stream_run).
template <int HD, int WAVES>
__global__ __launch_bounds__(WAVES * 64, 8 / WAVES) void decode_seq_kernel(const KParams p)
{
    using C = DecodeCfg<HD, WAVES>;
    __shared__ __attribute__((aligned(16))) unsigned char lds[WAVES * C::kVBytes];
    const int head_blocks = (p.num_kv_heads + WAVES - 1) / WAVES;
    int bid = blockIdx.x;
    const int hb = bid % head_blocks;
    bid /= head_blocks;
    const int part = bid / p.num_seqs;
    const int s = (bid % p.num_seqs + part) % p.num_seqs;  // rotated: the parts of a sequence spread over XCDs and engines
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int kvh = hb * WAVES + wave;
    if (kvh >= p.num_kv_heads) return;
    const int n_kv = p.seq_lens[s];
    const int k_lo = part * p.split_len;
    if (k_lo >= n_kv && part != 0) return;
    const int k_hi = k_lo + p.split_len < n_kv ? k_lo + p.split_len : n_kv;
    float *partial = p.num_splits == 1 ? nullptr
                                       : p.workspace + ((int64_t)s * p.num_q_heads * p.num_splits + part) * (HD + 2);
    // records of one sequence are laid out [head][part]
    const int64_t head_stride = (int64_t)p.num_splits * (HD + 2);
    if (k_hi <= k_lo) {
        decode_write_empty<HD>(p, lane, s, kvh, partial, head_stride);
        return;
    }
    decode_stream_run<HD, WAVES>(
        p, lds + wave * C::kVBytes, lane, kvh, s, k_lo / kChunk, (k_hi - k_lo + kChunk - 1) / kChunk, [&](int, bool) { return partial; },
        head_stride);
}

// Merge of the `parts` records of one query head by half a wavefront (32 lanes, all active; `sub` =
// lane within the half); the record of part i starts at r + i * stride.  Lane `sub` owns channels
// [HD/32 * sub, + HD/32) of the result, written as bf16 to o (already offset to those channels).
//   M = max_i m_i,  L = sum_i l_i 2^(m_i - M),  out = sum_i O_i 2^(m_i - M) / L
// Parts go in blocks of 32: each lane fetches one (m, l) pair and its channels of all 32 partial
// outputs at once, and the block's scales come from one 32-lane reduction, so the merge costs one
// memory round trip per block instead of several per part.  A part that was never written must not
// be passed; m = -inf (a part without keys) gets weight zero.
template <int HD>
__device__ __forceinline__ void merge_head(const float *r, int parts, int64_t stride, int lane, elem_t *o)
{
    constexpr int CPL = HD / 32;  // 4 or 2 channels per lane
    const int sub = lane & 31;
    auto load2 = [](const float *src) -> float2 { return *(const float2 *)src; };
    auto half_max = [](float x) {
#pragma unroll
        for (int sh = 1; sh < 32; sh <<= 1) x = fmaxf(x, __shfl_xor(x, sh));
        return x;
    };
    auto half_sum = [](float x) {
#pragma unroll
        for (int sh = 1; sh < 32; sh <<= 1) x += __shfl_xor(x, sh);
        return x;
    };
    float acc[CPL];
#pragma unroll
    for (int c = 0; c < CPL; ++c) acc[c] = 0.f;
    float M = -INFINITY, L = 0.f;
    for (int b0 = 0; b0 < parts; b0 += 32) {
        const int nb = parts - b0 < 32 ? parts - b0 : 32;
        // every load of the block is issued before the first result is needed: one round trip per block
        const float2 ml = sub < nb ? load2(r + (int64_t)(b0 + sub) * stride + HD) : float2{-INFINITY, 0.f};
        float2 d[32][CPL / 2];
#pragma unroll
        for (int j = 0; j < 32; ++j) {
            const float *rj = r + (int64_t)(b0 + j) * stride + CPL * sub;
#pragma unroll
            for (int c = 0; c < CPL / 2; ++c) d[j][c] = j < nb ? load2(rj + 2 * c) : float2{0.f, 0.f};
        }
        const float m_new = fmaxf(M, half_max(ml.x));
        if (m_new == -INFINITY) continue;  // nothing but empty parts so far (uniform over the half)
        const float keep = fast_exp2(M - m_new);  // 0 for the first block
        const float sc = fast_exp2(ml.x - m_new);  // 0 for lanes past the block and for empty parts
        L = L * keep + half_sum(ml.y * sc);
        M = m_new;
#pragma unroll
        for (int c = 0; c < CPL; ++c) acc[c] *= keep;
#pragma unroll
        for (int j = 0; j < 32; ++j) {
            const float wj = __shfl(sc, (lane & 32) | j);
#pragma unroll
            for (int c = 0; c < CPL / 2; ++c) {
                acc[2 * c] += d[j][c].x * wj;
                acc[2 * c + 1] += d[j][c].y * wj;
            }
        }
    }
    const float inv = L > 0.f ? 1.f / L : 0.f;
    typedef elem_t exC __attribute__((ext_vector_type(CPL)));
    exC w;
#pragma unroll
    for (int c = 0; c < CPL; ++c) w[c] = (elem_t)(acc[c] * inv);
    *(exC *)o = w;
}

// One wavefront merges query heads 2*pair and 2*pair + 1 of the G heads of (sequence s, KV head kvh).
// rec = record of part 0 at this KV head's first query head; head_stride / part_stride in floats.
template <int HD>
__device__ __forceinline__ void merge_pair(const KParams &p, int lane, int s, int kvh, int pair, const float *rec, int parts,
                                           int64_t head_stride, int64_t part_stride)
{
    const int G = p.group;
    const int hl = 2 * pair + (lane >> 5);
    const int hc = hl < G ? hl : G - 1;  // an idle half repeats the last head (same values, same address)
    elem_t *o = (elem_t *)p.out + (int64_t)s * p.o_stride_tok + (int64_t)(kvh * G + hc) * p.o_stride_head + (HD / 32) * (lane & 31);
    merge_head<HD>(rec + (int64_t)hc * head_stride, parts, part_stride, lane, o);
}

// Where a workgroup's run of chunks starts, for the token-balanced kernels: the batch's 32-key chunks
// laid end to end are cut into num_wgs runs of equal length (to within one chunk); run w is [x0, x1) and starts `off` chunks into
// sequence `s`.  Every wavefront works this out on its own (no barrier): lane l sums the chunk counts
// of a contiguous block of ceil(B / 64) sequences (independent loads, no cross-lane step inside the
// loop), one 64-wide scan gives the block prefix sums, and a second 64-wide scan over the one block
// that holds x0 finds the sequence.  Batches beyond 4096 sequences take a loop of 64-wide scans.
// The writer wavefront also stores the per-sequence chunk prefix sums for the merge kernel.
struct RunStart {
    int total, x0, x1, s, off;
};
// [0, total) cut into n runs whose lengths differ by at most one chunk (the first total % n runs are the
// longer ones): where run w begins, and which run holds chunk c.  (Runs of ceil(total / n) chunks would
// leave the last workgroups idle and make all others up to one chunk in total / n longer: 5 % at 19.008
// chunks per workgroup.)
__device__ __forceinline__ int run_begin(int total, int n, int w)
{
    const int q = total / n, rem = total - q * n;
    return w * q + (w < rem ? w : rem);
}
__device__ __forceinline__ int run_of(int total, int n, int c)
{
    const int q = total / n, rem = total - q * n, big = rem * (q + 1);
    return c < big ? c / (q + 1) : rem + (c - big) / (q > 0 ? q : 1);
}
__device__ __forceinline__ RunStart locate_run(const KParams &p, int lane, int w, int num_wgs, bool writer, int32_t *prefix_out)
{
    const int B = p.num_seqs;
    RunStart r{0, 0, 0, 0, 0};
    auto scan64 = [&](int v) {
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(v, o);
            if (lane >= o) v += t;
        }
        return v;
    };
    if (B <= 4096) {
        const int R = (B + 63) / 64;  // sequences per lane
        int mine = 0;
#pragma unroll 8
        for (int k = 0; k < R; ++k) {  // unrolled, and every load unconditional (index clamped, value masked), so
            const int i = lane * R + k;  // that the loads of a batch of eight are in flight together
            const int len = p.seq_lens[i < B ? i : B - 1];
            mine += ((len + kChunk - 1) / kChunk) & -(int)(i < B);  // masked by arithmetic: a select would become a branch around the load
        }
        const int incl = scan64(mine);
        r.total = __builtin_amdgcn_readlane(incl, 63);
        if (writer) {
            int run = incl - mine;
#pragma unroll 8
            for (int k = 0; k < R; ++k) {
                const int i = lane * R + k;
                const int len = p.seq_lens[i < B ? i : B - 1];
                if (i < B) {
                    prefix_out[i] = run;
                    run += (len + kChunk - 1) / kChunk;
                }
            }
            if (lane == 0) prefix_out[B] = r.total;
        }
        r.x0 = run_begin(r.total, num_wgs, w);
        r.x1 = run_begin(r.total, num_wgs, w + 1);
        if (r.x0 >= r.x1) return r;
        // the block (lane) that holds chunk x0, then the sequence inside the block
        const int blk = __builtin_ctzll(__builtin_amdgcn_ballot_w64(incl > r.x0));
        const int base = __builtin_amdgcn_readlane(incl - mine, blk);
        const int i2 = blk * R + lane;
        const int len2 = p.seq_lens[i2 < B ? i2 : B - 1];
        const int c2 = (lane < R && i2 < B) ? (len2 + kChunk - 1) / kChunk : 0;
        const int incl2 = scan64(c2);
        const int j = __builtin_ctzll(__builtin_amdgcn_ballot_w64(base + incl2 > r.x0));
        r.s = blk * R + j;
        r.off = r.x0 - (base + __builtin_amdgcn_readlane(incl2 - c2, j));
        return r;
    }
    for (int g0 = 0; g0 < B; g0 += 64) {
        const int i = g0 + lane;
        const int c = i < B ? (p.seq_lens[i] + kChunk - 1) / kChunk : 0;
        const int incl = scan64(c);
        if (writer && i < B) prefix_out[i] = r.total + incl - c;
        r.total += __builtin_amdgcn_readlane(incl, 63);
    }
    if (writer && lane == 0) prefix_out[B] = r.total;
    r.x0 = run_begin(r.total, num_wgs, w);
    r.x1 = run_begin(r.total, num_wgs, w + 1);
    if (r.x0 >= r.x1) return r;
    int base = 0;
    for (int g0 = 0; g0 < B; g0 += 64) {
        const int i = g0 + lane;
        const int c = i < B ? (p.seq_lens[i] + kChunk - 1) / kChunk : 0;
        const int incl = scan64(c);
        const int grp = __builtin_amdgcn_readlane(incl, 63);
        if (r.x0 < base + grp) {
            const int idx = __builtin_ctzll(__builtin_amdgcn_ballot_w64(base + incl > r.x0));
            r.s = g0 + idx;
            r.off = r.x0 - (base + __builtin_amdgcn_readlane(incl - c, idx));
            break;
        }
        base += grp;
    }
    return r;
}

// Token-balanced variant: the key axis of the whole batch, cut into 32-key chunks and laid end to
// end, is divided evenly over the workgroups (one per compute unit and KV-head block), whatever the
// mix of sequence lengths.  A workgroup therefore walks a run of chunks that may start in the middle
// of one sequence and end in the middle of another; every (workgroup, sequence) piece leaves one
// partial record with the unique index  workgroup + sequence  (both only grow along the walk).  The
// chunk prefix sums of the batch are recomputed by every wavefront (locate_run) and written once for
// the combine kernel.
//   workspace: [num_wgs + num_seqs][Hq][HD + 2] floats, then int32 chunk prefix sums [num_seqs + 1].
template <int HD, int WAVES>
__global__ __launch_bounds__(WAVES * 64, 8 / WAVES) void decode_balanced_kernel(const KParams p)
{
    using C = DecodeCfg<HD, WAVES>;
    __shared__ __attribute__((aligned(16))) unsigned char lds[WAVES * C::kVBytes];
    const int head_blocks = (p.num_kv_heads + WAVES - 1) / WAVES;
    const int hb = blockIdx.x % head_blocks;
    const int w = blockIdx.x / head_blocks;
    const int num_wgs = p.num_splits;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int kvh = hb * WAVES + wave;
    const int B = p.num_seqs;
    int32_t *prefix_out = (int32_t *)(p.workspace + (int64_t)(num_wgs + B) * p.num_q_heads * (HD + 2));
    const bool writer = blockIdx.x == 0 && wave == 0;

    const RunStart run = locate_run(p, lane, w, num_wgs, writer, prefix_out);
    if (kvh >= p.num_kv_heads || run.x0 >= run.x1) return;
    // a sequence that lies inside the run is finished there; a piece of a sequence shared with other
    // workgroups leaves a record for the merge kernel
    decode_stream_run<HD, WAVES>(
        p, lds + wave * C::kVBytes, lane, kvh, run.s, run.off, run.x1 - run.x0,
        [&](int s, bool whole) { return whole ? nullptr : p.workspace + (int64_t)(w + s) * p.num_q_heads * (HD + 2); }, HD + 2);
}

// Combine for the token-balanced variant: the pieces of sequence s are the workgroups that overlap its
// chunk range, at record indices workgroup + s.  One wavefront per (sequence, KV head, pair of query heads).
constexpr int kMergeWaves = 4;  // (sequence, KV head, head pair) units per merge workgroup

template <int HD>
__global__ __launch_bounds__(64 * kMergeWaves) void decode_balanced_combine_kernel(const KParams p)
{
    const int pairs = (p.group + 1) / 2;
    const int lane = threadIdx.x & 63;
    int bid = blockIdx.x * kMergeWaves + (threadIdx.x >> 6);
    if (bid >= p.num_seqs * p.num_kv_heads * pairs) return;
    const int pair = bid % pairs;
    bid /= pairs;
    const int kvh = bid % p.num_kv_heads;
    const int s = bid / p.num_kv_heads;
    const int num_wgs = p.num_splits;
    const int B = p.num_seqs;
    const int32_t *prefix = (const int32_t *)(p.workspace + (int64_t)(num_wgs + B) * p.num_q_heads * (HD + 2));
    const int c0 = prefix[s], c1 = prefix[s + 1], total = prefix[B];
    // an empty context has no piece: parts = 0 makes the merge write zeros
    const int w0 = c1 > c0 ? run_of(total, num_wgs, c0) : 0;
    const int parts = c1 > c0 ? run_of(total, num_wgs, c1 - 1) - w0 + 1 : 0;
    if (parts == 1) return;  // the main kernel wrote this sequence itself
    const int64_t stride = (int64_t)p.num_q_heads * (HD + 2);
    merge_pair<HD>(p, lane, s, kvh, pair, p.workspace + (int64_t)(w0 + s) * stride + (int64_t)kvh * p.group * (HD + 2), parts, HD + 2, stride);
}

// Combine for the fixed-split kernels, one wavefront per (sequence, KV head, pair of query heads): records are laid out
// [sequence][head][part].  Parts that hold no key were never written and are not read.
template <int HD>
__global__ __launch_bounds__(64 * kMergeWaves) void decode_combine_kernel(const KParams p)
{
    const int pairs = (p.group + 1) / 2;
    const int lane = threadIdx.x & 63;
    int bid = blockIdx.x * kMergeWaves + (threadIdx.x >> 6);
    if (bid >= p.num_seqs * p.num_kv_heads * pairs) return;
    const int pair = bid % pairs;
    bid /= pairs;
    const int kvh = bid % p.num_kv_heads;
    const int s = bid / p.num_kv_heads;
    const int n_kv = p.seq_lens[s];
    int parts = (n_kv + p.split_len - 1) / p.split_len;
    parts = parts < 1 ? 1 : parts;  // part 0 is always written (m = -inf, l = 0 for an empty context)
    const int64_t head_stride = (int64_t)p.num_splits * (HD + 2);
    merge_pair<HD>(p, lane, s, kvh, pair, p.workspace + ((int64_t)s * p.num_q_heads + (int64_t)kvh * p.group) * head_stride, parts,
                          head_stride, HD + 2);
}

template <int HD, int WAVES>
bool decode_valid(const KParams &p)
{
    return p.dtype == kElemDtype && p.head_dim == HD && p.group <= 16 && p.block_table != nullptr && p.block_size >= 16;
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

template <int HD, int WAVES>
hipError_t decode_seq_launch(const KParams &p, hipStream_t stream)
{
    const int64_t head_blocks = (p.num_kv_heads + WAVES - 1) / WAVES;
    const int64_t blocks = head_blocks * p.num_seqs * p.num_splits;
    if (blocks <= 0) return hipSuccess;
    if (blocks > 0x7fffffff) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((decode_seq_kernel<HD, WAVES>), dim3((unsigned)blocks), dim3(WAVES * 64), 0, stream, p);
    return hipGetLastError();
}

// Token-balanced launch: p.num_splits carries the number of workgroups per KV-head block (set by the
// dispatcher from the compute-unit count); the combine kernel follows on the same stream.
template <int HD, int WAVES>
hipError_t decode_balanced_launch(const KParams &p, hipStream_t stream)
{
    const int64_t head_blocks = (p.num_kv_heads + WAVES - 1) / WAVES;
    const int64_t blocks = head_blocks * p.num_splits;
    if (blocks <= 0 || p.num_seqs <= 0) return hipSuccess;
    if (blocks > 0x7fffffff) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((decode_balanced_kernel<HD, WAVES>), dim3((unsigned)blocks), dim3(WAVES * 64), 0, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int64_t units = (int64_t)p.num_seqs * p.num_kv_heads * ((p.group + 1) / 2);
    hipLaunchKernelGGL(decode_balanced_combine_kernel<HD>, dim3((unsigned)((units + kMergeWaves - 1) / kMergeWaves)), dim3(64 * kMergeWaves), 0,
                       stream, p);
    return hipGetLastError();
}

// SPLIT < 0 marks the token-balanced variant with -SPLIT workgroups per compute unit
#define DECODE_BAL_INSTANCE(HD, WAVES, PER_CU)                                                                  \
    {                                                                                                          \
        DECODE_NAME "_balanced d" #HD " w" #WAVES " percu" #PER_CU, 16, kChunk, WAVES, 16, 2, -PER_CU,           \
            decode_valid<HD, WAVES>, decode_balanced_launch<HD, WAVES>                                  \
    }
#define DECODE_SEQ_INSTANCE(HD, WAVES, SPLIT)                                                                  \
    {                                                                                                          \
        DECODE_NAME "_seq d" #HD " w" #WAVES " split" #SPLIT, 16, kChunk, WAVES, 16, 2, SPLIT, decode_valid<HD, WAVES>, \
            decode_seq_launch<HD, WAVES>                                                                       \
    }

#define DECODE_INSTANCE(HD, WAVES, SPLIT)                                                                     \
    {                                                                                                         \
        DECODE_NAME " d" #HD " w" #WAVES " split" #SPLIT, 16, kChunk, WAVES, 16, 2, SPLIT, decode_valid<HD, WAVES>, \
            decode_launch<HD, WAVES>                                                                          \
    }

}  // namespace

#ifdef ATTN_DECODE_ELEM_F16
hipError_t launch_decode_combine_f16(const KParams &p, hipStream_t stream)
{
    const int64_t blocks = ((int64_t)p.num_seqs * p.num_kv_heads * ((p.group + 1) / 2) + kMergeWaves - 1) / kMergeWaves;
    if (blocks <= 0) return hipSuccess;
    if (blocks > 0x7fffffff) return hipErrorInvalidConfiguration;
    if (p.head_dim == 128)
        hipLaunchKernelGGL(decode_combine_kernel<128>, dim3((unsigned)blocks), dim3(64 * kMergeWaves), 0, stream, p);
    else if (p.head_dim == 64)
        hipLaunchKernelGGL(decode_combine_kernel<64>, dim3((unsigned)blocks), dim3(64 * kMergeWaves), 0, stream, p);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

const Instance *decode_f16_instances(int *count)
{
    static const Instance table[] = {
        DECODE_SEQ_INSTANCE(128, 8, 0),    DECODE_SEQ_INSTANCE(128, 8, 256),  DECODE_SEQ_INSTANCE(128, 8, 512),
        DECODE_SEQ_INSTANCE(128, 8, 1024), DECODE_SEQ_INSTANCE(128, 8, 2048), DECODE_SEQ_INSTANCE(128, 4, 256),
        DECODE_SEQ_INSTANCE(128, 4, 512),  DECODE_SEQ_INSTANCE(128, 4, 1024), DECODE_SEQ_INSTANCE(64, 8, 256),
        DECODE_SEQ_INSTANCE(64, 4, 512),   DECODE_BAL_INSTANCE(128, 8, 1),    DECODE_BAL_INSTANCE(128, 4, 1),
        DECODE_BAL_INSTANCE(128, 8, 2),    DECODE_BAL_INSTANCE(64, 8, 1),
    };
    *count = (int)(sizeof(table) / sizeof(table[0]));
    return table;
}

#else
hipError_t launch_decode_combine(const KParams &p, hipStream_t stream)
{
    const int64_t blocks = ((int64_t)p.num_seqs * p.num_kv_heads * ((p.group + 1) / 2) + kMergeWaves - 1) / kMergeWaves;
    if (blocks <= 0) return hipSuccess;
    if (blocks > 0x7fffffff) return hipErrorInvalidConfiguration;
    if (p.head_dim == 128)
        hipLaunchKernelGGL(decode_combine_kernel<128>, dim3((unsigned)blocks), dim3(64 * kMergeWaves), 0, stream, p);
    else if (p.head_dim == 64)
        hipLaunchKernelGGL(decode_combine_kernel<64>, dim3((unsigned)blocks), dim3(64 * kMergeWaves), 0, stream, p);
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
        DECODE_SEQ_INSTANCE(128, 8, 0),    DECODE_SEQ_INSTANCE(128, 8, 128),  DECODE_SEQ_INSTANCE(128, 8, 256),
        DECODE_SEQ_INSTANCE(128, 8, 512),  DECODE_SEQ_INSTANCE(128, 8, 1024), DECODE_SEQ_INSTANCE(128, 8, 2048),
        DECODE_SEQ_INSTANCE(128, 4, 256),  DECODE_SEQ_INSTANCE(128, 4, 512),  DECODE_SEQ_INSTANCE(128, 4, 1024),
        DECODE_SEQ_INSTANCE(64, 8, 256),   DECODE_SEQ_INSTANCE(64, 4, 512),
        DECODE_BAL_INSTANCE(128, 8, 1),    DECODE_BAL_INSTANCE(128, 8, 2),    DECODE_BAL_INSTANCE(128, 4, 1),
        DECODE_BAL_INSTANCE(128, 4, 2),    DECODE_BAL_INSTANCE(64, 8, 1),     DECODE_BAL_INSTANCE(64, 4, 2),
    };
    *count = (int)(sizeof(table) / sizeof(table[0]));
    return table;
}

#endif

}  // namespace attn

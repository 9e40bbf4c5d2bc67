// Kernel-side view of one attention call and the launcher table shared by the
// host dispatcher, the tuner and the kernel translation units.
//
// Notation follows the problem statement of the paper's study (section "Method
// and Investigated Kernels"): Q/K/V, query heads Hq, KV heads Hkv, head size D,
// a batch of sequences of different lengths, a causal mask; the paged KV cache
// with its block table is the PagedAttention layout the paper cites.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace attn {

// element types of q, k, v, out (the values of attn_dtype in the C ABI)
constexpr int kDtypeF32 = 0, kDtypeBf16 = 1, kDtypeF16 = 2;

struct KParams {
    const void *q;
    void *out;
    const void *k;
    const void *v;
    const int32_t *block_table;  // nullptr -> contiguous K/V
    const int32_t *query_start_loc;  // nullptr in decode (one token per sequence)
    const int32_t *kv_start_loc;
    const int32_t *seq_lens;
    int64_t q_stride_tok, q_stride_head;
    int64_t o_stride_tok, o_stride_head;
    int64_t kv_stride_block, kv_stride_tok, kv_stride_head;
    int32_t dtype;  // kDtype*
    int32_t num_seqs, num_q_heads, num_kv_heads, head_dim;
    int32_t group;  // Hq / Hkv
    int32_t block_table_stride;
    int32_t block_size, block_shift;  // block_size == 1 << block_shift when block_shift >= 0
    int32_t max_q_len, max_kv_len;
    float scale;        // softmax scale
    float scale_log2e;  // scale * log2(e): scores are exponentiated with exp2
    int32_t causal;
    // split-K decode
    float *workspace;
    int32_t num_splits;  // parts the key axis is cut into (grid dimension)
    int32_t split_len;   // keys per part, a multiple of the kernel's key tile
    // prefill grid order: 0 = query tiles outermost (the longest tiles of all sequences start first),
    // 1 = sequences outermost (all tiles of a sequence run together and share its K/V in one L2)
    int32_t tile_order;
};

// One ahead-of-time compiled template instance: the unit the autotuner sweeps
// (the paper's "kernel configuration"; its requirement list asks for a way to
// declare the parameter space together with the dependencies between
// parameters -- here `valid` is that predicate).
struct Instance {
    const char *name;
    int block_m;  // query rows (token x head) per workgroup
    int block_n;  // keys per tile
    int waves;    // wavefronts per workgroup
    int heads_per_wg;  // query heads of one KV head packed into a workgroup
    int stages;   // K/V tiles in flight (pipeline depth)
    int split_len;  // decode: keys per split-K part (0 = never split); prefill: 0
    bool (*valid)(const KParams &);
    hipError_t (*launch)(const KParams &, hipStream_t);
    int variant;  // prefill: KParams::tile_order this instance launches with; decode: 0
};

const Instance *prefill_instances(int *count);         // all prefill instances, ring variants first
const Instance *prefill_ring_instances(int *count);    // LDS-ring, software-pipelined (D = 128), bf16
const Instance *prefill_ring_f16_instances(int *count);  // the same kernel for fp16
const Instance *prefill_staged_instances(int *count);  // register-staged double buffer (D = 64, 128)
const Instance *prefill_staged_f16_instances(int *count);  // the same kernel for fp16
const Instance *decode_instances(int *count);       // bf16
const Instance *decode_f16_instances(int *count);   // fp16: the wave-per-head and token-balanced kernels

hipError_t launch_prefill_f32(const KParams &, hipStream_t);
hipError_t launch_decode_combine(const KParams &, hipStream_t);
hipError_t launch_decode_combine_f16(const KParams &, hipStream_t);

// Floats per (sequence, query head, split) in the split-K workspace: D partial
// outputs followed by the running max and the running sum.
inline int partial_stride(int head_dim) { return head_dim + 2; }

}  // namespace attn

/*
 * attn.h -- C ABI of the MI355X (gfx950) fused-attention library.
 *
 * The library computes exact scaled-dot-product attention for LLM inference,
 * the kernel the paper uses as its main vehicle (section "Method and
 * Investigated Kernels": flash attention, Llama3-8B shapes -- head size 128,
 * 32 query heads, 8 KV heads -- with sequences of different lengths in one
 * batch; Fig. 2: causal).  For every sequence s, query head h and new-token
 * index i it returns
 *
 *     out[i,h,:] = sum_j softmax_j( scale * q[i,h,:] . k[j,h/G,:] ) * v[j,h/G,:]
 *
 * over the keys j visible to query i, with G = num_q_heads / num_kv_heads
 * (consecutive query heads share a KV head).  The paper states no interface;
 * the argument names follow its problem statement (Q, K, V, block table,
 * sequence lengths, query start offsets, softmax scale).
 *
 * Conventions
 *  - Every pointer in attn_args is a DEVICE pointer owned by the caller and must
 *    stay valid until the work queued on the stream has finished.  The host
 *    never dereferences them.  Strides are in ELEMENTS; head_dim is contiguous.
 *  - attn_prefill_varlen and attn_decode_paged only validate host-visible
 *    fields, look up a kernel instance and enqueue kernels on `hip_stream`
 *    (a hipStream_t passed as void*; NULL = the default stream).  They do not
 *    allocate, free, synchronise or copy, so they may be captured in a HIP graph
 *    (the paper times its kernels under CUDA/HIP graphs, same section).
 *  - Errors that the host can see are returned as a negative attn_status and
 *    nothing is enqueued.  Out-of-range block_table entries, or seq_lens /
 *    query_start_loc that disagree with total_q, max_q_len, max_kv_len, are
 *    undefined behaviour -- unless ATTN_DEBUG_VALIDATE=1 is set in the environment:
 *    then every hot call first drains the stream, copies these integers to the
 *    host and returns ATTN_ERR_SHAPE if they are inconsistent (a debugging mode:
 *    synchronous, not capturable).
 *  - Hot calls are re-entrant; the winner cache is guarded by a mutex.
 *  - Environment, each read once per process: ATTN_TUNE_CACHE=<file> (winner cache loaded on the
 *    first hot call), ATTN_FORCE_INSTANCE=<exact instance name> (that instance wherever it is valid
 *    for the shape, the usual choice elsewhere), ATTN_LOG=1 (one line on stderr whenever the
 *    instance for a new shape is resolved: kind, bucket key, instance, reason),
 *    ATTN_DEBUG_VALIDATE=1 (above).
 */
#ifndef ATTN_H_
#define ATTN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum attn_status {
    ATTN_OK = 0,
    ATTN_ERR_NULL = -1,        /* a required pointer is NULL */
    ATTN_ERR_SHAPE = -2,       /* inconsistent sizes, strides or head counts */
    ATTN_ERR_DTYPE = -3,       /* dtype not supported by this entry point */
    ATTN_ERR_UNSUPPORTED = -4, /* head_dim / block_size / group size without a kernel instance */
    ATTN_ERR_WORKSPACE = -5,   /* workspace missing or smaller than attn_workspace_bytes() */
    ATTN_ERR_HIP = -6,         /* the HIP runtime refused a launch or an allocation */
    ATTN_ERR_CACHE_IO = -7     /* the tuning cache file could not be read or written */
} attn_status;

typedef enum attn_dtype {
    ATTN_F32 = 0, /* q, k, v, out are IEEE fp32; arithmetic is fp32 FMA */
    ATTN_BF16 = 1, /* q, k, v, out are bfloat16; products on bf16 MFMA, fp32 accumulation and softmax */
    ATTN_F16 = 2   /* q, k, v, out are IEEE fp16; products on fp16 MFMA, fp32 accumulation and softmax */
} attn_dtype;

typedef struct attn_args {
    uint32_t struct_bytes; /* = sizeof(attn_args); calls with another value are rejected */
    int32_t dtype;         /* attn_dtype of q, k, v and out */
    int32_t num_seqs;      /* B */
    int32_t num_q_heads;   /* Hq */
    int32_t num_kv_heads;  /* Hkv, divides Hq */
    int32_t head_dim;      /* D: 64 or 128 */
    int32_t total_q;       /* host copy of query_start_loc[B]; decode: = B */
    int32_t max_q_len;     /* host upper bound of n_q(s); sizes the grid, no device sync needed */
    int32_t max_kv_len;    /* host upper bound of seq_lens[s] */

    const void *q; /* [total_q, Hq, D] */
    int64_t q_stride_tok, q_stride_head;
    void *out; /* [total_q, Hq, D], same dtype as q */
    int64_t o_stride_tok, o_stride_head;

    /* contiguous mode (block_table == NULL): k, v are [total_kv, Hkv, D] and key j of sequence s
     * is row kv_start_loc[s] + j.  paged mode: k, v are [num_blocks, block_size, Hkv, D] and key j
     * of sequence s is slot j % block_size of block block_table[s][j / block_size]. */
    const void *k;
    const void *v;
    int64_t kv_stride_block, kv_stride_tok, kv_stride_head;

    const int32_t *block_table; /* int32 [B, block_table_stride]; entries past ceil(seq_len/block_size) are never read */
    int32_t block_table_stride;
    int32_t block_size; /* paged: a power of two, at least 16 */
    int32_t num_blocks; /* pool size, used only for validation */

    const int32_t *query_start_loc; /* int32 [B+1], exclusive prefix sum of n_q; decode: ignored (n_q = 1) */
    const int32_t *kv_start_loc;    /* int32 [B+1], contiguous mode only; NULL -> query_start_loc */
    const int32_t *seq_lens;        /* int32 [B]: keys of sequence s = cached prefix + new tokens, already stored */

    float scale;    /* softmax scale applied to q.k (1/sqrt(D) for standard attention) */
    int32_t causal; /* 1: query i sees keys j <= (seq_lens[s] - n_q(s)) + i (bottom-right aligned); 0: all keys.
                     * Requires seq_lens[s] >= n_q(s); a query that would sit before key 0 gets zeros. */

    void *workspace; /* device scratch for split-K partials; may be NULL if attn_workspace_bytes() == 0 */
    uint64_t workspace_bytes;
} attn_args;

/*
 * Causal variable-length prefill, also over a paged prefix (chunked prefill).
 * Tiled online-softmax attention in the FlashAttention-2 formulation the paper
 * builds on (same section; Fig. 2 "causal flash attention"): the score matrix
 * is never materialised.  Sequences with n_q = 0 write nothing.  A query with
 * no visible key (possible only when causal == 0 and seq_len == 0) gets zeros.
 * dtype ATTN_BF16 (D = 128 or 64), ATTN_F16 (D = 128 or 64) or ATTN_F32 (D = 64 or 128).
 * Returns ATTN_OK after enqueueing, or a negative attn_status.
 */
int attn_prefill_varlen(const attn_args *args, void *hip_stream);

/*
 * Paged-KV decode: one query token per sequence (q is [B, Hq, D]) attending to
 * all seq_lens[s] keys held in the paged cache addressed by block_table (the
 * paper cites PagedAttention for this setting; layout above).  Long contexts
 * are split along the key axis; each part writes an fp32 (max, sum, partial
 * output) triple into `workspace` and a second kernel merges them.  The caller
 * provides at least attn_workspace_bytes(args, 1) bytes, 8-byte aligned.  dtype ATTN_BF16 or ATTN_F16.
 */
int attn_decode_paged(const attn_args *args, void *hip_stream);

/*
 * attn_decode_paged for callers that cannot provide or allocate device memory beyond the inputs and
 * outputs: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * same kernels and the same instance choice as attn_decode_paged, but the split-K records go to a
 * device array that the library owns (attn_static_scratch_bytes() bytes, 16 MiB, held on every GPU the
 * library runs on until the process ends); args->workspace and args->workspace_bytes are ignored.
 * The call allocates and frees nothing; the array's address is looked up once per device, on the
 * first call made with that device current.  A call whose instance needs more than the array holds
 * (very large batches: one record of (D + 2) floats per query head for every sequence and for up to
 * four workgroups per compute unit) returns ATTN_ERR_WORKSPACE and enqueues nothing.  All calls on
 * one GPU share the array, which needs no clearing between calls (every record a call reads it has
 * written itself): calls that overlap in time on one GPU, on whatever streams, race -- serialise them.
 */
int attn_decode_paged_static(const attn_args *args, void *hip_stream);
/* Size of that array in bytes (pure host function). */
size_t attn_static_scratch_bytes(void);

/*
 * The step in front of paged attention: stores the keys and values of new tokens into the paged
 * cache (the PagedAttention layout the paper cites; the paper itself is silent on this step).
 * Token t goes to slot slot_mapping[t] = block * block_size + offset of both caches; a negative slot
 * marks a padding token and stores nothing.  A pure copy (bit-exact), any element type of 2 or 4
 * bytes.  Two tokens mapped to the same slot race.
 */
typedef struct attn_kv_write_args {
    uint32_t struct_bytes; /* = sizeof(attn_kv_write_args) */
    int32_t dtype;         /* attn_dtype: only the element size matters */
    int32_t num_tokens;    /* T */
    int32_t num_kv_heads;  /* Hkv */
    int32_t head_dim;      /* D; D * element size is a multiple of 16 bytes */
    int32_t block_size;    /* slots per cache block, > 0 */
    int32_t num_blocks;    /* pool size, used only for validation */
    int32_t reserved;
    const void *k_new; /* [T, Hkv, D] */
    const void *v_new;
    int64_t new_stride_tok, new_stride_head; /* elements; rows 16-byte aligned */
    void *k_cache; /* [num_blocks, block_size, Hkv, D] */
    void *v_cache;
    int64_t kv_stride_block, kv_stride_tok, kv_stride_head;
    const int32_t *slot_mapping; /* int32 [T], device; slots >= num_blocks * block_size are undefined behaviour */
} attn_kv_write_args;

/* Enqueues the copy on `hip_stream`; allocates nothing, capturable.  ATTN_OK or a negative attn_status. */
int attn_kv_cache_write(const attn_kv_write_args *args, void *hip_stream);

/*
 * Bytes of workspace the call described by `args` may use (pure host function apart from one
 * device-property query; pointer fields are ignored): the largest need of any kernel instance that
 * may be chosen for it, whatever the winner cache holds.  Fixed-split instances cut a context into at
 * most 64 parts and a batch into at most two parts per compute unit; the token-balanced ones use one
 * record per workgroup (at most four per compute unit) and per sequence.  is_decode = 1 for
 * attn_decode_paged.  Returns 0 when args is NULL or malformed.
 */
size_t attn_workspace_bytes(const attn_args *args, int is_decode);

/*
 * Ahead-of-time autotuning (the paper's requirements list: tune off the
 * critical path, keep results in a reusable cache that records its
 * environment).  Times every valid compiled kernel instance for the shape
 * bucket of `shape_like` on synthetic device buffers that this call allocates
 * and frees itself.  Of the pointer fields of shape_like only seq_lens and (for
 * prefill) query_start_loc are used, if not NULL: the tuning batch then has the
 * caller's own lengths (copied to the host; they must respect max_q_len and
 * max_kv_len).  Otherwise lengths are spread evenly between half of and the full
 * max_q_len / max_kv_len.  Paged tuning batches use a random permutation of the
 * block pool.  The search is a successive halving: three timed launches of every
 * valid instance, iters/2 of the best third (the built-in choice and the winners
 * already known for neighbouring buckets always stay in); an instance three times
 * slower than the best so far is dropped after one launch.  The best three and the
 * built-in choice are then measured `iters` (<= 0: a default) more times each,
 * taking turns launch by launch, and the medians decide; the built-in choice wins
 * ties within 3 % (launch-to-launch noise).  The call records the
 * fastest instance and, if cache_path is not NULL, merges it into that file:
 * read, change and replace (write to a temporary file, fsync, rename) under an
 * exclusive flock on "<cache_path>.lock", so concurrent tuners keep each other's
 * lines; damaged lines are dropped, other environments' lines kept.  Synchronous;
 * not capturable.
 * flags: bit 0 = print one line per measurement to stderr; bit 1 = exhaustive
 * sweep (`iters` launches of every valid instance) instead of the halving.
 */
int attn_tune(const attn_args *shape_like, int is_decode, const char *cache_path, int iters, int flags);

/* Writes the NUL-terminated environment key that attn_tune stores with every cache line (device
 * architecture, compute units, HIP runtime and driver versions, a hash of the compiled instance set)
 * and returns its length.  Pure host function apart from a device-property query. */
int attn_environment_key(char *buf, size_t buf_bytes);

/* Load winners from a cache file written by attn_tune.  Entries recorded for a different device,
 * CU count, runtime or library build are skipped, and so is a line that does not parse (the lines
 * around it still count).  Also done lazily from $ATTN_TUNE_CACHE on the first hot call.  A file that
 * is missing, does not start with the format's first line, or holds nothing but damaged lines returns
 * ATTN_ERR_CACHE_IO and leaves the built-in heuristic in force; hot calls never fail because of the cache. */
int attn_load_cache(const char *cache_path);

/* Forget all cached winners (hot calls fall back to the built-in heuristic). */
void attn_clear_cache(void);

/* Introspection for the tuner and the tests (pure host functions). */
int attn_num_instances(int is_decode);
/* Writes the NUL-terminated name of instance `id` (kernel family and template parameters, e.g.
 * "prefill_bf16_ring d128 qb1 w8 hpw4 slots8 pf5 seqmajor" or "decode_bf16_balanced d128 w4 percu1"),
 * truncated to buf_bytes - 1 characters; returns the length written, or a negative attn_status for a bad id. */
int attn_instance_name(int is_decode, int id, char *buf, size_t buf_bytes);
/* Instance the next hot call with these args would launch (cache winner, else heuristic), or <0. */
int attn_selected_instance(const attn_args *args, int is_decode);
/* Force an instance id for all later hot calls of that kind (-1 = back to automatic).  Invalid
 * combinations are rejected by the hot call with ATTN_ERR_UNSUPPORTED. */
void attn_force_instance(int is_decode, int id);

const char *attn_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* ATTN_H_ */

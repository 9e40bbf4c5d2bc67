// Causal variable-length prefill on bf16 (or fp16) MFMA (gfx950): LDS-ring, software-pipelined variant.
//
// Same operation and same operand layout as prefill_bf16.hip (tiled online-softmax
// attention, the FlashAttention-2 formulation of the paper's kernel, section
// "Method and Investigated Kernels"; causal, variable-length, grouped-query heads),
// restructured so that the matrix cores and the vector ALU work at the same time:
//
//  * K and V travel HBM -> LDS with global_load_lds (no registers, no ds_write) into a
//    ring of NSLOT slots of 32 keys; PF units are in flight, counted with s_waitcnt
//    vmcnt, one workgroup barrier per 32-key unit.  The 16-byte chunks of a row are
//    XOR-swizzled (by choosing which global chunk each lane fetches) so that both the
//    128-bit K reads and the transposing 64-bit V reads are free of bank conflicts
//    without padding.
//  * The unit loop is software pipelined: while the MFMAs of S(u+1) = K(u+1) Q^T run,
//    the ALU exponentiates S(u); while the MFMAs of O += V(u) P(u) run, it takes the
//    row maxima of S(u+1) and applies the masks.
//  * The running maximum is only moved when it would grow by more than 2^kSlack
//    (then O and l are rescaled); otherwise exponentials are taken against the stale
//    reference.  The result is unchanged, because numerator and denominator
//    carry the same reference, and the rescale of the accumulators becomes rare.
//  * The output tile is transposed through LDS and written as whole 256-byte rows.
#include "kernel_params.hpp"

namespace attn {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// The two 16-bit element types the kernel is instantiated for: how a 32x32x16 product and the packing
// of two weights are spelled.  Everything else (transfers, swizzles,
// transposing reads, masks, the fp32 softmax) is the same code.
struct ElemBf16 {
    typedef __bf16 elem;
    typedef bf16x8 x8;
    typedef bf16x2 x2;
    static constexpr int kDtype = kDtypeBf16;
    static __device__ __forceinline__ f32x16 mfma(x8 a, x8 b, f32x16 c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0); }
};
struct ElemF16 {
    typedef _Float16 elem;
    typedef f16x8 x8;
    typedef f16x2 x2;
    static constexpr int kDtype = kDtypeF16;
    static __device__ __forceinline__ f32x16 mfma(x8 a, x8 b, f32x16 c) { return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0); }
};
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void gbl_void;

constexpr int kHD = 128;
constexpr int kUnit = 32;          // keys per pipeline unit
constexpr int kSlotBytes = 16384;  // 32 K rows + 32 V rows of 256 bytes
constexpr int kVOff = 8192;
constexpr float kSlack = 8.f;      // log2 of the largest weight tolerated before the reference moves

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// value of the same register in lane ^ 32
__device__ __forceinline__ float swap32_max(float x)
{
    const uint32_t u = __float_as_uint(x);
    const u32x2 r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float swap32_sum(float x)
{
    const uint32_t u = __float_as_uint(x);
    const u32x2 r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// LDS traffic of the unit loop is issued behind the compiler's back, as inline assembly, and waited
// for by count.  Two reasons.  The compiler cannot tell that a transposing read never touches a ring
// slot with a transfer in flight and would drain the whole prefetch queue (s_waitcnt vmcnt(0)) in
// front of the builtin.  And once any of the loop's LDS operations is hidden from it, it waits for
// the ones it still sees with lgkmcnt(0), i.e. for the read it issued a moment ago, several times per
// unit.  LDS operations of a wave complete in order, so "at most N operations outstanding" means
// that everything but the N youngest has returned: every consumer below waits with the number of LDS
// operations issued after the one it needs (lds_wait), counted at compile time along the unrolled code.
__device__ __forceinline__ s16x4 lds_read_tr16_b64_untracked(const unsigned char *p)
{
    s16x4 r;
    const unsigned addr = (unsigned)(uintptr_t)(__attribute__((address_space(3))) const unsigned char *)p;
    asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(r) : "v"(addr) : "memory");
    return r;
}
__device__ __forceinline__ unsigned lds_addr(const unsigned char *p)
{
    return (unsigned)(uintptr_t)(__attribute__((address_space(3))) const unsigned char *)p;
}
template <int OFFSET>
__device__ __forceinline__ u32x4 lds_read_b128_untracked(unsigned addr)
{
    u32x4 r;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFFSET) : "memory");
    return r;
}
__device__ __forceinline__ void lds_write_b128_untracked(unsigned addr, s16x8 v)
{
    asm volatile("ds_write_b128 %0, %1" : : "v"(addr), "v"(v) : "memory");
}
// all LDS operations of this wave have returned; ties the registers so that their uses stay below
__device__ __forceinline__ void lds_wait(s16x4 &a, s16x4 &b) { asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a), "+v"(b)::"memory"); }
// at most n LDS operations of this wave are still outstanding (n is a constant once the loops around
// the call are unrolled, so the switch folds to one instruction); `r` is tied so that its use stays below
template <typename T>
__device__ __forceinline__ void lds_wait_upto(int n, T &r)
{
#define LDS_WAIT_CASE(N) case N: asm volatile("s_waitcnt lgkmcnt(" #N ")" : "+v"(r)::"memory"); break;
    switch (n < 0 ? 0 : n) {
        LDS_WAIT_CASE(0) LDS_WAIT_CASE(1) LDS_WAIT_CASE(2) LDS_WAIT_CASE(3) LDS_WAIT_CASE(4) LDS_WAIT_CASE(5) LDS_WAIT_CASE(6)
        LDS_WAIT_CASE(7) LDS_WAIT_CASE(8) LDS_WAIT_CASE(9) LDS_WAIT_CASE(10) LDS_WAIT_CASE(11) LDS_WAIT_CASE(12) LDS_WAIT_CASE(13)
        LDS_WAIT_CASE(14)
        default: asm volatile("s_waitcnt lgkmcnt(15)" : "+v"(r)::"memory"); break;  // the counter's largest value
    }
#undef LDS_WAIT_CASE
}

// s_waitcnt with only vmcnt constrained (gfx9 encoding: vmcnt in bits 3:0 and 15:14)
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);
}

// chunk swizzle of a row inside a unit: rows r..r+15 get 16 distinct values (128-bit K reads),
// rows r..r+3 differ in the upper two bits (64-bit transposing V reads)
__device__ __forceinline__ int swz(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

template <int QB, int HPW, int NSLOT, int PF, int WAVES>
struct RingCfg {
    static constexpr int kWaves = WAVES;
    static constexpr int kRowsPerWave = kUnit / WAVES;   // rows of a unit that one wave transfers
    static constexpr int kDmaPerWave = kRowsPerWave / 4;  // 1 KB transfers per wave, for K and again for V
    static constexpr int kTSub = kWaves / HPW;
    static constexpr int kWaveTok = 32 * QB;
    static constexpr int kTok = kTSub * kWaveTok;
    static constexpr int kThreads = WAVES * 64;
    static constexpr int kImgBytes = 8192;               // V^T fragments of one unit, in MFMA operand order
    static constexpr int kFragsPerWave = 8 / WAVES;      // fragments each wave transposes per unit
    static constexpr size_t kLdsBytes = (size_t)NSLOT * kSlotBytes + 2 * kImgBytes;
    static_assert(WAVES == 4 || WAVES == 8, "4 or 8 wavefronts");
    // during iteration u the slots of units u+1 (V, transposed for the next iteration) and u+2 (K) are
    // read and units u+3..u+PF are in flight; unit u+PF reuses the slot of unit u+PF-NSLOT <= u
    static_assert(NSLOT >= PF, "ring too small for the prefetch distance");
    static_assert(PF >= 3, "K of unit u+2 is read one iteration ahead, so three units must be resident");
    static_assert(kWaves % HPW == 0, "waves must split evenly over heads");
    static_assert(kLdsBytes >= (size_t)kWaves * kWaveTok * kHD * 2, "epilogue staging must fit in the ring");
};

template <typename E, int QB, int HPW, int NSLOT, int PF, int WAVES, bool PAGED>
__global__ __launch_bounds__(WAVES * 64, (QB == 1 && WAVES == 4) ? 2 : 1) void prefill_ring_kernel(const KParams p)
{
    using C = RingCfg<QB, HPW, NSLOT, PF, WAVES>;
    using elem = typename E::elem;
    using x8 = typename E::x8;
    using x2 = typename E::x2;
    constexpr int KSTEPS = kHD / 16;
    constexpr int DB = kHD / 32;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    // ---- which (head group, sequence, query tile) ---------------------------------------------
    // Workgroups go to the eight XCDs round-robin, so with the KV head innermost every XCD (and its
    // own L2) serves one KV head when Hkv is a multiple or a divisor of eight.
    const int groups_per_kvh = p.group / HPW;
    int bid = blockIdx.x;
    const int kvh = bid % p.num_kv_heads;
    bid /= p.num_kv_heads;
    const int hsub = bid % groups_per_kvh;
    bid /= groups_per_kvh;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int q_tiles = (p.max_q_len + C::kTok - 1) / C::kTok;  // the grid's tile dimension
    // Workgroups start in block-index order as slots come free, so the order is the schedule: work that
    // costs most (most keys to visit) goes first, and small tiles are left to fill the end.
    int s, r;
    if (p.tile_order == 0) {
        // tile index outermost, counted down from the longest sequence's last tile: the tiles in flight
        // cost about the same in every sequence, and every sequence keeps its cheap first tiles for the end.
        // The sequence index rotates with the tile index: inside an XCD the dispatcher deals workgroups
        // to its four shader engines round-robin by index and waits for the engine whose turn it is,
        // so with a fixed sequence-to-index map (say 8 sequences) a long sequence would load one
        // engine with all of its tiles and the other three would wait for it (measured: 20 % imbalance
        // on 8 sequences of 400-1800 tokens).
        r = bid / p.num_seqs;
        s = (bid % p.num_seqs + r) % p.num_seqs;
    } else {
        // sequences outermost (all tiles of a sequence run side by side on the XCD of their KV head and
        // stream its K/V together), heaviest tile first.  For the same reason as above the tiles swap
        // places inside each group of four, differently from one sequence to the next (with a tile
        // count that is a multiple of four every engine would otherwise get the same tile of each
        // group from all sequences, the first engine always the heaviest); the order stays heaviest
        // first to within three places, which matters for the last sequence.
        s = bid / q_tiles;
        r = bid % q_tiles;
        if (r < (q_tiles & ~3)) r ^= s & 3;
    }

    const int q0 = p.query_start_loc[s];
    const int n_q = p.query_start_loc[s + 1] - q0;
    const int n_kv = p.seq_lens[s];
    const int off = n_kv - n_q;
    const int n_tiles_q = (n_q + C::kTok - 1) / C::kTok;
    const int qtile = p.tile_order == 0 ? q_tiles - 1 - r : n_tiles_q - 1 - r;
    if (qtile < 0 || qtile >= n_tiles_q) return;
    const int t0 = qtile * C::kTok;

    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lhalf = lane >> 5;
    const int l32 = lane & 31;
    const int l16 = lane & 15;
    const int head = kvh * p.group + hsub * HPW + (wave % HPW);
    const int t0w = t0 + (wave / HPW) * C::kWaveTok;

    // scores are exponentiated as 2^(c*s - ref); a negative scale is moved into Q (sign flips are exact)
    const float c = fabsf(p.scale_log2e);
    const bool negate_q = p.scale_log2e < 0.f;

    // ---- Q fragments ---------------------------------------------------------------------------
    const elem *qbase = (const elem *)p.q;
    x8 qf[QB][KSTEPS];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        int t = t0w + qb * 32 + l32;
        t = t < n_q ? t : n_q - 1;
        const elem *src = qbase + (int64_t)(q0 + t) * p.q_stride_tok + (int64_t)head * p.q_stride_head + 8 * lhalf;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            u32x4 raw = *(const u32x4 *)(src + 16 * ks);
            if (negate_q) raw ^= 0x80008000u;
            qf[qb][ks] = __builtin_bit_cast(x8, raw);
        }
    }

    // ---- key range -------------------------------------------------------------------------------
    int kv_end = n_kv;
    if (p.causal) {
        const int last_tok = t0 + C::kTok < n_q ? t0 + C::kTok : n_q;
        kv_end = off + last_tok < n_kv ? off + last_tok : n_kv;
    }
    const int n_units = (kv_end + kUnit - 1) / kUnit;

    elem *obase = (elem *)p.out;
    if (n_units <= 0) {  // no visible key at all (an empty context; also lengths that break seq_lens >= n_q): zeros
        for (int i = lane; i < C::kWaveTok * (kHD / 8); i += 64) {
            const int t = t0w + i / (kHD / 8);
            if (t < n_q)
                *(u32x4 *)(obase + (int64_t)(q0 + t) * p.o_stride_tok + (int64_t)head * p.o_stride_head + 8 * (i % (kHD / 8))) =
                    u32x4{0u, 0u, 0u, 0u};
        }
        return;
    }

    // first key position of this wave's rows, and the first unit that needs masking for this wave
    const int qpos_lo = p.causal ? off + t0w : 0x7fffff00;
    int first_masked = (qpos_lo + 1) / kUnit;             // units below lie entirely at or before qpos_lo
    first_masked = first_masked < n_kv / kUnit ? first_masked : n_kv / kUnit;  // and entirely inside the sequence
    int qrel[QB];  // key index (relative to the lane's first key of a unit) up to which a row sees keys
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int qp = p.causal ? off + t0w + qb * 32 + l32 : 0x7fffff00;
        const int lim = qp < n_kv - 1 ? qp : n_kv - 1;  // last visible key
        qrel[qb] = lim - 4 * lhalf;
    }

    // ---- DMA of one unit: wave w moves rows 8w..8w+7 of K and of V (2 x 1 KB each) -------------
    // The address of a transfer is a wave-uniform 64-bit base (SGPRs: pool block or packed row of the
    // unit, KV head) plus a 32-bit per-lane offset (row inside the block, swizzled 16-byte chunk).
    // The rows of a wave never straddle a 16-key block, so the table entry is wave-uniform.
    const unsigned char *kbase = (const unsigned char *)p.k + (int64_t)kvh * p.kv_stride_head * 2;
    const unsigned char *vbase = (const unsigned char *)p.v + (int64_t)kvh * p.kv_stride_head * 2;
    const int kv0 = PAGED ? 0 : p.kv_start_loc[s];
    // The block table is read through the scalar cache (constant address space): a vector load would
    // share the counter of the LDS transfers, and waiting for it would drain the whole transfer queue
    // once per unit.
    typedef const __attribute__((address_space(4))) int32_t *table_ptr;
    const table_ptr bt_row = PAGED ? (table_ptr)(p.block_table + (int64_t)s * p.block_table_stride) : (table_ptr) nullptr;
    constexpr int RPW = C::kRowsPerWave, NDMA = C::kDmaPerWave;
    const int dma_row = RPW * wave + (lane >> 4);  // + 4*i, row inside the unit
    const uint32_t tok_bytes = (uint32_t)p.kv_stride_tok * 2;
    const int last_unit0 = (n_kv - 1) & ~(kUnit - 1);  // first key of the last unit that holds a real key
    // Per-lane byte offset of a transfer from the first row of this wave's share of a unit: the lane's
    // row and its swizzled 16-byte chunk.  It is the same in every unit whose rows all exist; in a
    // ragged last unit (and in the repeats of it past the end) the rows past the end re-read the last
    // key (finite, masked), which gives a second set of offsets.  Everything else about a transfer's
    // address is wave-uniform: scalar arithmetic.
    uint32_t dma_off[NDMA], dma_off_last[NDMA];
    const uint32_t block_bytes = (uint32_t)(p.kv_stride_block * 2);  // (ring_valid checks that it fits)
    {
        const int wrow_last = last_unit0 + RPW * wave < n_kv ? last_unit0 + RPW * wave : n_kv - 1;
#pragma unroll
        for (int i = 0; i < NDMA; ++i) {
            const uint32_t chunk = 16 * ((lane & 15) ^ swz(dma_row + 4 * i));
            dma_off[i] = (uint32_t)((lane >> 4) + 4 * i) * tok_bytes + chunk;
            int row = last_unit0 + dma_row + 4 * i;
            row = row < n_kv ? row : n_kv - 1;
            dma_off_last[i] = (uint32_t)(row - wrow_last) * tok_bytes + chunk;
        }
    }
    // wave-uniform table entry of the block that holds this wave's rows of `unit` (clamped to the sequence)
    auto table_entry = [&](int unit) -> int {
        if (!PAGED) return 0;
        int u0 = unit * kUnit < last_unit0 ? unit * kUnit : last_unit0;
        int row = u0 + RPW * wave;
        row = row < n_kv ? row : n_kv - 1;
        return bt_row[__builtin_amdgcn_readfirstlane(row) >> p.block_shift];
    };
    // The same entry, requested with an untracked scalar load (inline assembly): the value may only be
    // used after an s_waitcnt lgkmcnt(0) that follows the request (scalar loads return out of order).
    auto table_entry_request = [&](int unit) -> int {
        if (!PAGED) return 0;
        int u0 = unit * kUnit < last_unit0 ? unit * kUnit : last_unit0;
        int row = u0 + RPW * wave;
        row = row < n_kv ? row : n_kv - 1;
        const unsigned byte_off = (unsigned)(__builtin_amdgcn_readfirstlane(row) >> p.block_shift) * 4u;
        int r;
        asm volatile("s_load_dword %0, %1, %2" : "=s"(r) : "s"(bt_row), "s"(byte_off) : "memory");
        return r;
    };
    auto issue_unit = [&](int unit, int entry) {
        unsigned char *slot = lds + (unit % NSLOT) * kSlotBytes + RPW * wave * 256;
        const int u0 = unit * kUnit < last_unit0 ? unit * kUnit : last_unit0;  // units past the end repeat the last one
        const bool ragged = u0 + kUnit > n_kv;
        int wrow = u0 + RPW * wave;  // first row of this wave's share
        wrow = wrow < n_kv ? wrow : n_kv - 1;
        // the rows of a wave never straddle a 16-key block: one table entry (PAGED) or one packed run of rows
        const uint64_t base = PAGED ? (uint64_t)(uint32_t)entry * block_bytes + (uint32_t)(wrow & (p.block_size - 1)) * tok_bytes
                                    : (uint64_t)(kv0 + wrow) * tok_bytes;
        const unsigned char *kb = kbase + base, *vb = vbase + base;
#pragma unroll
        for (int i = 0; i < NDMA; ++i) {
            uint32_t o = ragged ? dma_off_last[i] : dma_off[i];
            // (kept opaque: a loop-invariant offset would be widened and added to the array bases once, and
            // the transfers would then carry 64-bit per-lane addresses instead of scalar base + 32-bit offset)
            asm volatile("" : "+v"(o));
            __builtin_amdgcn_global_load_lds((gbl_void *)(kb + o), (lds_void *)(slot + 4 * i * 256), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((gbl_void *)(vb + o), (lds_void *)(slot + kVOff + 4 * i * 256), 16, 0, 0);
        }
    };

    // Publish the ring.  Each wave issues 2*NDMA transfers per unit and memory operations complete in order,
    // so once at most 2*NDMA*(PF-3) are outstanding, this wave's transfers of every unit but the newest PF-3
    // have landed (a table load that sits between them only makes the wait stricter).  All LDS reads of
    // the slot about to be refilled have returned, because their values fed MFMAs issued earlier.  A
    // bare s_barrier is used: the fence of __syncthreads would drain vmcnt to zero and with it the
    // whole prefetch queue.
    auto ring_barrier = [&]() {
        wait_vmcnt<2 * NDMA * (PF - 3)>();
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): this wave's LDS write of transposed V has been performed
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    };
    // V^T fragment images: a wave transposes its share of the V fragments of a unit once
    // (ds_read_b64_tr_b16, the slow path) and stores them in MFMA A-operand order; every wave then
    // fetches all eight fragments with plain 128-bit reads.  Two images alternate.
    unsigned char *img_base = lds + NSLOT * kSlotBytes;
    // where inside a slot each of this lane's transposing reads goes (the same in every unit)
    int tr_off[C::kFragsPerWave][2];
#pragma unroll
    for (int i = 0; i < C::kFragsPerWave; ++i) {
        const int f = wave * C::kFragsPerWave + i;  // f = ks2 * DB + db
        const int db = f % DB, ks2 = f / DB;
        const int a = l16 >> 2, h1 = (lane >> 4) & 1, h0 = (lane & 3) >> 1;
#pragma unroll
        for (int rd = 0; rd < 2; ++rd)
            tr_off[i][rd] = kVOff + (8 * rd + 4 * lhalf + a) * 256 + 16 * (((db ^ a) << 2) | (2 * (h1 ^ rd)) | (h0 ^ lhalf)) + 8 * (lane & 1) +
                            ks2 * 16 * 256;
    }
    auto transpose_load = [&](int unit, s16x4 (&raw)[C::kFragsPerWave][2]) {
        const unsigned char *vt = lds + (unit % NSLOT) * kSlotBytes;
#pragma unroll
        for (int i = 0; i < C::kFragsPerWave; ++i) {
#pragma unroll
            for (int rd = 0; rd < 2; ++rd) raw[i][rd] = lds_read_tr16_b64_untracked(vt + tr_off[i][rd]);
        }
    };
    auto transpose_store = [&](int unit, s16x4 (&raw)[C::kFragsPerWave][2]) {
        unsigned char *img = img_base + (unit & 1) * C::kImgBytes;
#pragma unroll
        for (int i = 0; i < C::kFragsPerWave; ++i) {
            lds_wait(raw[i][0], raw[i][1]);
            const int f = wave * C::kFragsPerWave + i;
            const s16x8 both = __builtin_shufflevector(raw[i][0], raw[i][1], 0, 1, 2, 3, 4, 5, 6, 7);
            *(s16x8 *)(img + f * 1024 + lane * 16) = both;
        }
    };

    // ---- per-lane LDS read offsets ----------------------------------------------------------------
    int koff[KSTEPS];
    {
        const int kx = swz(l32);
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) koff[ks] = l32 * 256 + 16 * ((2 * ks + lhalf) ^ kx);
    }
    // ---- state ---------------------------------------------------------------------------------------
    f32x16 oacc[QB][DB];
    f32x16 s_cur[QB], s_nxt[QB];
    float m_ref[QB], l_run[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        m_ref[qb] = -INFINITY;
        l_run[qb] = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) oacc[qb][db][v] = 0.f;
    }

    // S(u) = K(u) Q^T for both query blocks
    auto qk = [&](int unit, f32x16 (&sacc)[QB]) {
        const unsigned char *kt = lds + (unit % NSLOT) * kSlotBytes;
        x8 kf[KSTEPS];
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) kf[ks] = *(const x8 *)(kt + koff[ks]);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int v = 0; v < 16; ++v) sacc[qb][v] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) sacc[qb] = E::mfma(kf[ks], qf[qb][ks], sacc[qb]);
        }
    };
    // Move the reference of the rows whose new maximum outgrew it by more than the slack; rare, and
    // wave-uniform, so the accumulators are only touched when needed.
    auto reference_outgrown = [&](const float (&bm)[QB]) -> bool {
        bool grow = false;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) grow |= bm[qb] > m_ref[qb] + kSlack;
        return __builtin_amdgcn_ballot_w64(grow) != 0;
    };
    auto rescale_to = [&](const float (&bm)[QB]) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            float m_new = fmaxf(m_ref[qb], bm[qb]);
            m_new = m_new == -INFINITY ? 0.f : m_new;
            const float alpha = fast_exp2(m_ref[qb] - m_new);
            m_ref[qb] = m_new;
            l_run[qb] *= alpha;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) oacc[qb][db][v] *= alpha;
        }
    };
    auto move_reference = [&](const float (&bm)[QB]) {
        if (reference_outgrown(bm)) rescale_to(bm);
    };
    // Row maxima of a fresh score tile (masked if MASK), then move the reference if a row outgrew it.
    // With MASK the tile is left scaled (x = c*s, masked entries -inf); without, it stays raw.
    auto settle = [&](int unit, f32x16 (&sacc)[QB], auto mask_tag) {
        constexpr bool MASK = decltype(mask_tag)::value;
        float bm[QB];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            if (MASK) {
                const int rel = qrel[qb] - unit * kUnit;  // entries with 8*(v/4) + (v%4) > rel are hidden
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float x = sacc[qb][v] * c;
                    sacc[qb][v] = (8 * (v >> 2) + (v & 3)) > rel ? -INFINITY : x;
                }
            }
            float mx = fmaxf(fmaxf(sacc[qb][0], sacc[qb][1]), sacc[qb][2]);
#pragma unroll
            for (int v = 3; v < 15; v += 2) mx = fmaxf(fmaxf(mx, sacc[qb][v]), sacc[qb][v + 1]);
            mx = fmaxf(mx, sacc[qb][15]);
            mx = swap32_max(mx);
            bm[qb] = MASK ? mx : mx * c;
        }
        move_reference(bm);
    };
    // ---- prologue: PF units in flight, S(0) ready ------------------------------------------------
#pragma unroll
    for (int u = 0; u < PF; ++u) issue_unit(u, table_entry(u));
    ring_barrier();
    qk(0, s_cur);
    using Masked = std::integral_constant<bool, true>;
    using Plain = std::integral_constant<bool, false>;
    bool cur_masked = first_masked <= 0;
    if (cur_masked)
        settle(0, s_cur, Masked{});
    else
        settle(0, s_cur, Plain{});
    u32x4 kf[KSTEPS];  // K fragments of the next unit, fetched one iteration ahead
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) kf[ks] = *(const u32x4 *)(lds + (1 % NSLOT) * kSlotBytes + koff[ks]);
    int entry_cur = table_entry(PF);  // (a tracked scalar load: the wait below covers it)
    {
        s16x4 raw[C::kFragsPerWave][2];
        transpose_load(0, raw);
        transpose_store(0, raw);
        asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(entry_cur)::"memory");
        __builtin_amdgcn_s_waitcnt(0xC07F);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    }

    // ---- main loop ------------------------------------------------------------------------------------
    // Invariant at the top of iteration u: S(u) settled in `cur`; units u and u+1 resident; units up to
    // u+PF-1 issued.  S(u+1) is always computed, also past the last unit (the ring slot then holds
    // the clamped rows of a dummy transfer): that keeps every iteration one straight-line block.
    // One iteration is written as groups of "one MFMA plus the vector and LDS work that hides under
    // it", fenced by scheduling barriers, because a wavefront issues in order: the matrix pipe only
    // stays busy if independent ALU work sits between consecutive MFMAs in program order.
    //   phase X: S(u+1) += K(u+1) Q^T, one MFMA per group, with the exponentials of one pair of
    //            scores of S(u) and one or two transposing V(u) reads per group;
    //   phase Y: O += V(u) P(u), one MFMA per group, with the row maxima (and masks) of S(u+1), the
    //            K(u+2) fragment reads for the next iteration and the transfers of unit u+PF.
    // Invariant at the top of iteration u: S(u) settled in `cur`; kf = K(u+1); units <= u+2 resident;
    // units <= u+PF-1 issued.  S(u+1) is computed even past the last unit (its ring slot then holds the
    // re-read rows of a dummy transfer and every entry is masked): no branch inside the iteration.
    // LDS operations of one iteration, in issue order (the same in every iteration, so the position of
    // an operation of the previous iteration is known too):
    //   phase X: V^T image fragments f = 0..7 (one per 1/8 of the phase), after fragment 1 the wave's
    //            transposing reads of V(u+1) (2 per fragment it owns), after fragment kWriteAfter the
    //            wave's image stores of V(u+1);
    //   phase Y: K(u+2) fragments ks = 0..7, kKPerGroup per group from the first group on.
    // A consumer waits until at most as many operations are outstanding as were issued after the one it
    // needs.  Nothing in the loop waits for "all": the image stores are older than the last image
    // fragments the same wave waits for in phase Y, so they have been performed when the wave reaches
    // the barrier; the K reads stay in flight across the barrier.
    constexpr int kWriteAfter = 5;
    constexpr int kXOps = 8 + 3 * C::kFragsPerWave;  // LDS operations of phase X
    constexpr int kKPerGroup = 2;
    // Block-table entry of the unit that the next iteration transfers (entry_cur, set up in the prologue):
    // requested (scalar cache) at the top of an iteration, awaited at its barrier -- the one place where
    // this wave waits for everything it has in flight, because scalar loads share the LDS counter and
    // return out of order.
    // LDS addresses of this lane's K fragment reads inside slot 0, and the same 64 KiB further on: with
    // the slot known at compile time (the plain units' loop below is unrolled over the ring) the slot
    // becomes the read's 16-bit immediate offset instead of an addition per read.
    unsigned kaddr[KSTEPS], kaddr_far[KSTEPS];
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
        kaddr[ks] = lds_addr(lds + koff[ks]);
        kaddr_far[ks] = kaddr[ks] + 65536u;
        if (NSLOT > 4) asm volatile("" : "+v"(kaddr_far[ks]));  // a register of its own, not an addition at every use
    }
    // SLOT2 >= 0: the ring slot of unit u+2, known at compile time
    auto iteration = [&](int u, f32x16 (&cur)[QB], f32x16 (&nxt)[QB], auto cur_tag, auto nxt_tag, auto slot_tag) {
        constexpr bool CUR_MASK = decltype(cur_tag)::value;
        constexpr bool NXT_MASK = decltype(nxt_tag)::value;
        constexpr int SLOT2 = decltype(slot_tag)::value;
        constexpr int G = 8 * QB;  // MFMAs per product
        const unsigned img_rd = lds_addr(img_base + (u & 1) * C::kImgBytes + lane * 16);
        const unsigned img_wr = lds_addr(img_base + ((u + 1) & 1) * C::kImgBytes + lane * 16);
        const unsigned char *kt2 = lds + ((u + 2) % NSLOT) * kSlotBytes;

        x8 pf[QB][2];
        u32x4 vfrag[2 * DB];
        s16x4 raw[C::kFragsPerWave][2];
        float sum[QB][2];
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        int seq = 0;        // LDS operations issued so far in this iteration
        int vpos[2 * DB];   // position of image fragment f in this iteration's sequence
        int tr_last = 0;    // position of the last transposing read
        int entry_nxt = table_entry_request(u + 1 + PF);
        // weights 2p, 2p+1 of row block qb: exponentials, rounding, row sum.  The exponentials are spread over
        // both phases (half under the score MFMAs, half under the first PV MFMAs, which only need the
        // first half), so that neither phase has more vector work than matrix work to hide it under.
        // Two steps, a group apart: the exponentials are issued under one MFMA and their results are
        // rounded and summed under the next, so that nothing waits for the transcendental unit's
        // latency (a wavefront issues in order: a use right behind the exponential stalls it).
        float e_pending[QB][2];
        auto exp_issue = [&](int qb, int pair) {
            const int v = 2 * pair;
            e_pending[qb][0] = fast_exp2(CUR_MASK ? cur[qb][v] - m_ref[qb] : __builtin_fmaf(cur[qb][v], c, -m_ref[qb]));
            e_pending[qb][1] = fast_exp2(CUR_MASK ? cur[qb][v + 1] - m_ref[qb] : __builtin_fmaf(cur[qb][v + 1], c, -m_ref[qb]));
            asm volatile("" : "+v"(e_pending[qb][0]), "+v"(e_pending[qb][1]));  // issued here, not where they are used
        };
        auto exp_finish = [&](int qb, int pair) {
            const int v = 2 * pair;
            const float e0 = e_pending[qb][0], e1 = e_pending[qb][1];
            x2 pr;
            pr[0] = (elem)e0;
            pr[1] = (elem)e1;
            // Row sums with plain adds, two chains per row block (even and odd pairs).  The dot-product
            // instruction that would sum the rounded pair in one go occupies the matrix pipe for about
            // half an MFMA (measured), so it is not free under the MFMAs; the sum of the unrounded
            // weights differs from the sum of the rounded ones by rounding errors that average out.
            sum[qb][pair & 1] = pair < 2 ? e0 + e1 : sum[qb][pair & 1] + (e0 + e1);  // pairs come in order: 0 and 1 start the chains
            pf[qb][v >> 3][v & 7] = pr[0];
            pf[qb][v >> 3][(v & 7) + 1] = pr[1];
        };
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const int ks = g / QB, qb = g % QB;
            // K(u+1) fragment ks was read in phase Y of the previous iteration, at position kXOps + ks of
            // kXOps + 8; since then the rest of that iteration and `seq` operations of this one were issued
            if (qb == 0) lds_wait_upto((KSTEPS - 1 - ks) + seq, kf[ks]);
            nxt[qb] = E::mfma(__builtin_bit_cast(x8, kf[ks]), qf[qb][ks], ks == 0 ? zero : nxt[qb]);
            // weights of keys 0..15 (the B operand of the first four PV MFMAs): issued under the even steps,
            // finished under the odd ones
            if (ks % 2 == 0)
                exp_issue(qb, ks / 2);
            else
                exp_finish(qb, ks / 2);
            if (g * 8 / G != (g + 1) * 8 / G) {
                const int f = g * 8 / G;
                switch (f) {  // the fragment index becomes the instruction's immediate offset
                    case 0: vfrag[0] = lds_read_b128_untracked<0 * 1024>(img_rd); break;
                    case 1: vfrag[1] = lds_read_b128_untracked<1 * 1024>(img_rd); break;
                    case 2: vfrag[2] = lds_read_b128_untracked<2 * 1024>(img_rd); break;
                    case 3: vfrag[3] = lds_read_b128_untracked<3 * 1024>(img_rd); break;
                    case 4: vfrag[4] = lds_read_b128_untracked<4 * 1024>(img_rd); break;
                    case 5: vfrag[5] = lds_read_b128_untracked<5 * 1024>(img_rd); break;
                    case 6: vfrag[6] = lds_read_b128_untracked<6 * 1024>(img_rd); break;
                    default: vfrag[7] = lds_read_b128_untracked<7 * 1024>(img_rd); break;
                }
                vpos[f] = seq++;
                if (f == 1) {  // this wave's share of V(u+1): transposed here, stored a few groups later
                    transpose_load(u + 1, raw);
                    seq += 2 * C::kFragsPerWave;
                    tr_last = seq - 1;
                }
                if (f == kWriteAfter) {  // image (u+1)&1 was last read in iteration u-1, before the barrier
#pragma unroll
                    for (int i = 0; i < C::kFragsPerWave; ++i) {
                        lds_wait_upto(seq - 1 - tr_last, raw[i][0]);
                        lds_wait_upto(15, raw[i][1]);  // already there: only ties the register below the wait
                        const s16x8 both = __builtin_shufflevector(raw[i][0], raw[i][1], 0, 1, 2, 3, 4, 5, 6, 7);
                        lds_write_b128_untracked(img_wr + (wave * C::kFragsPerWave + i) * 1024, both);
                        ++seq;
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }

        float mx[QB], bm[QB];
        bool outgrown = false;
        int rel[QB];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) rel[qb] = qrel[qb] - (u + 1) * kUnit;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const int f = g / QB, qb = g % QB;  // f = ks2 * DB + db
            // weights of keys 16..31, needed from the fifth PV MFMA on: each pair is finished a group after
            // it was issued (the last one just ahead of the MFMA that needs it)
            if (f >= 1 && f <= DB) exp_finish(qb, 3 + f);
            if (qb == 0) lds_wait_upto(seq - 1 - vpos[f], vfrag[f]);
            oacc[qb][f % DB] = E::mfma(__builtin_bit_cast(x8, vfrag[f]), pf[qb][f / DB], oacc[qb][f % DB]);
            if (f < DB) exp_issue(qb, 4 + f);
            // The second half of the phase (the last S MFMAs have drained) has vector slots to spare: the row
            // maxima of S(u+1), eight scores per group, and right behind them the test whether a reference
            // has to move, so that the answer is there when the last MFMA of the iteration has been issued.
            const int sl = g - 4 * QB;
            if (sl >= 0 && sl < 2 * QB) {
                const int q2 = sl / 2, v0 = 8 * (sl % 2);
                if (NXT_MASK) {
#pragma unroll
                    for (int v = v0; v < v0 + 8; ++v) {
                        const float x = nxt[q2][v] * c;
                        nxt[q2][v] = (8 * (v >> 2) + (v & 3)) > rel[q2] ? -INFINITY : x;
                    }
                }
                float m3 = fmaxf(fmaxf(nxt[q2][v0], nxt[q2][v0 + 1]), nxt[q2][v0 + 2]);
                m3 = fmaxf(fmaxf(m3, nxt[q2][v0 + 3]), nxt[q2][v0 + 4]);
                m3 = fmaxf(fmaxf(m3, nxt[q2][v0 + 5]), nxt[q2][v0 + 6]);
                mx[q2] = v0 == 0 ? fmaxf(m3, nxt[q2][v0 + 7]) : fmaxf(fmaxf(mx[q2], m3), nxt[q2][v0 + 7]);
            }
            if (sl == 2 * QB) {
#pragma unroll
                for (int q2 = 0; q2 < QB; ++q2) {
                    const float m = swap32_max(mx[q2]);
                    bm[q2] = NXT_MASK ? m : m * c;
                }
                outgrown = reference_outgrown(bm);
            }
            // K fragments of unit u+2 (the fragments of u+1 were consumed in phase X), in order, early in
            // the phase: they are a few groups old when the next iteration asks for them
#pragma unroll
            for (int j = 0; j < kKPerGroup; ++j) {
                const int ks = g * kKPerGroup + j;
                if (ks < KSTEPS) {
                    if (SLOT2 < 0)
                        kf[ks] = lds_read_b128_untracked<0>(lds_addr(kt2 + koff[ks]));
                    else
                        kf[ks] = lds_read_b128_untracked<(SLOT2 < 0 ? 0 : SLOT2 % 4) * kSlotBytes>(SLOT2 >= 4 ? kaddr_far[ks] : kaddr[ks]);
                    ++seq;
                }
            }
            if (g == G - 3) issue_unit(u + PF, entry_cur);  // refill: unit u+PF replaces unit u+PF-NSLOT <= u
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) l_run[qb] += sum[qb][0] + sum[qb][1];
        if (outgrown) rescale_to(bm);
        // Publish.  This wave's transfers of every unit but the newest PF-3 have landed (see ring_barrier);
        // its image stores have been performed (phase Y waited for younger reads); its K reads may still
        // be in flight, they target a slot that no transfer touches before the barrier after next.
        wait_vmcnt<2 * NDMA * (PF - 3)>();
        if (PAGED) asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(entry_nxt)::"memory");
        entry_cur = entry_nxt;
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    };
    auto copy_back = [&]() {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) s_cur[qb] = s_nxt[qb];
    };
    int u = 0;
    using AnySlot = std::integral_constant<int, -1>;
    // plain units whose successors are plain too, one trip round the ring per pass (u is a multiple of
    // NSLOT here, so unit u+2+i sits in slot (2+i) % NSLOT)
    for (; u + NSLOT < first_masked; u += NSLOT) {
        iteration(u, s_cur, s_nxt, Plain{}, Plain{}, std::integral_constant<int, 2 % NSLOT>{});
        iteration(u + 1, s_nxt, s_cur, Plain{}, Plain{}, std::integral_constant<int, 3 % NSLOT>{});
        iteration(u + 2, s_cur, s_nxt, Plain{}, Plain{}, std::integral_constant<int, 4 % NSLOT>{});
        iteration(u + 3, s_nxt, s_cur, Plain{}, Plain{}, std::integral_constant<int, 5 % NSLOT>{});
        if (NSLOT == 8) {
            iteration(u + 4, s_cur, s_nxt, Plain{}, Plain{}, std::integral_constant<int, 6 % NSLOT>{});
            iteration(u + 5, s_nxt, s_cur, Plain{}, Plain{}, std::integral_constant<int, 7 % NSLOT>{});
            iteration(u + 6, s_cur, s_nxt, Plain{}, Plain{}, std::integral_constant<int, 8 % NSLOT>{});
            iteration(u + 7, s_nxt, s_cur, Plain{}, Plain{}, std::integral_constant<int, 9 % NSLOT>{});
        }
    }
    static_assert(NSLOT == 4 || NSLOT == 8, "the loop above is written out for rings of four and eight slots");
    // the rest of them, two per trip so that the two score tiles swap roles
    for (; u + 2 < first_masked; u += 2) {
        iteration(u, s_cur, s_nxt, Plain{}, Plain{}, AnySlot{});
        iteration(u + 1, s_nxt, s_cur, Plain{}, Plain{}, AnySlot{});
    }
    if (u + 1 < first_masked) {
        iteration(u, s_cur, s_nxt, Plain{}, Plain{}, AnySlot{});
        copy_back();
        ++u;
    }
    if (!cur_masked) {  // the last plain unit: its successor (if any) is masked
        iteration(u, s_cur, s_nxt, Plain{}, Masked{}, AnySlot{});
        copy_back();
        ++u;
    }
    for (; u + 1 < n_units; u += 2) {
        iteration(u, s_cur, s_nxt, Masked{}, Masked{}, AnySlot{});
        iteration(u + 1, s_nxt, s_cur, Masked{}, Masked{}, AnySlot{});
    }
    if (u < n_units) iteration(u, s_cur, s_nxt, Masked{}, Masked{}, AnySlot{});
    // The last iteration's K reads are still in flight and nobody will use them: wait for them here,
    // with their registers tied, so that the compiler cannot hand those registers to anything else
    // while a read may still land in them.
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(kf[0]), "+v"(kf[1]), "+v"(kf[2]), "+v"(kf[3]), "+v"(kf[4]), "+v"(kf[5]), "+v"(kf[6]), "+v"(kf[7])::"memory");
    static_assert(KSTEPS == 8, "the drain above names eight fragments");

    // ---- epilogue: O / l, transposed through LDS, whole rows to HBM ------------------------------
    wait_vmcnt<0>();
    __syncthreads();  // the ring is free: every wave is past its last V read and no DMA is in flight
    unsigned char *stage = lds + wave * (C::kWaveTok * kHD * 2);  // [token][128] bf16, chunk-swizzled by token
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float l = swap32_sum(l_run[qb]);
        const float inv = l > 0.f ? 1.f / l : 0.f;
        const int tl = qb * 32 + l32;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                x2 a, b;
                a[0] = (elem)(oacc[qb][db][4 * vq + 0] * inv);
                a[1] = (elem)(oacc[qb][db][4 * vq + 1] * inv);
                b[0] = (elem)(oacc[qb][db][4 * vq + 2] * inv);
                b[1] = (elem)(oacc[qb][db][4 * vq + 3] * inv);
                const int chunk = 4 * db + vq;  // 16-byte chunk of the row; lhalf selects its 8-byte half
                u32x2 w;
                w[0] = __builtin_bit_cast(uint32_t, a);
                w[1] = __builtin_bit_cast(uint32_t, b);
                *(u32x2 *)(stage + tl * 256 + 16 * (chunk ^ (tl & 15)) + 8 * lhalf) = w;
            }
        }
    }
    // wave-private staging: the wave's own LDS writes are ordered before its reads
#pragma unroll
    for (int i = 0; i < C::kWaveTok / 4; ++i) {
        const int tl = 4 * i + (lane >> 4);
        const int chunk = lane & 15;
        const u32x4 row = *(const u32x4 *)(stage + tl * 256 + 16 * (chunk ^ (tl & 15)));
        const int t = t0w + tl;
        if (t < n_q)
            *(u32x4 *)(obase + (int64_t)(q0 + t) * p.o_stride_tok + (int64_t)head * p.o_stride_head + 8 * chunk) = row;
    }
}

template <typename E, int QB, int HPW, int NSLOT, int PF, int WAVES>
bool ring_valid(const KParams &p)
{
    // (a cache block of 4 GiB or more would need 64-bit block arithmetic in the transfers)
    return p.dtype == E::kDtype && p.head_dim == kHD && p.group % HPW == 0 && (!p.block_table || (uint64_t)p.kv_stride_block * 2 < (1ull << 32));
}

template <typename E, int QB, int HPW, int NSLOT, int PF, int WAVES, bool PAGED>
hipError_t ring_launch_impl(const KParams &p, hipStream_t stream, int64_t blocks)
{
    using C = RingCfg<QB, HPW, NSLOT, PF, WAVES>;
    auto kern = prefill_ring_kernel<E, QB, HPW, NSLOT, PF, WAVES, PAGED>;
    static hipError_t attr = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::kLdsBytes);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(C::kThreads), C::kLdsBytes, stream, p);
    return hipGetLastError();
}

template <typename E, int QB, int HPW, int NSLOT, int PF, int WAVES, int ORDER>
hipError_t ring_launch(const KParams &p_in, hipStream_t stream)
{
    KParams p = p_in;
    p.tile_order = ORDER;
    using C = RingCfg<QB, HPW, NSLOT, PF, WAVES>;
    const int64_t q_tiles = (p.max_q_len + C::kTok - 1) / C::kTok;
    const int64_t nhg = (int64_t)p.num_kv_heads * (p.group / HPW);
    const int64_t blocks = q_tiles * p.num_seqs * nhg;
    if (blocks <= 0) return hipSuccess;
    if (blocks > 0x7fffffff) return hipErrorInvalidConfiguration;
    return p.block_table ? ring_launch_impl<E, QB, HPW, NSLOT, PF, WAVES, true>(p, stream, blocks)
                         : ring_launch_impl<E, QB, HPW, NSLOT, PF, WAVES, false>(p, stream, blocks);
}

// This file is compiled twice: as it stands for bf16, and included by prefill_f16_ring.hip with
// ATTN_RING_ELEM_F16 defined for fp16 inputs (a smaller set of instances).
#ifdef ATTN_RING_ELEM_F16
#define RING_ELEM ElemF16
#define RING_NAME "prefill_f16_ring"
#else
#define RING_ELEM ElemBf16
#define RING_NAME "prefill_bf16_ring"
#endif

#define RING_ONE(QB, HPW, NSLOT, PF, WAVES, ORDER, TAG)                                                            \
    {                                                                                                              \
        RING_NAME " d128 qb" #QB " w" #WAVES " hpw" #HPW " slots" #NSLOT " pf" #PF TAG, WAVES * 32 * QB, kUnit, WAVES, \
            HPW, PF, 0, ring_valid<RING_ELEM, QB, HPW, NSLOT, PF, WAVES>,                                          \
            ring_launch<RING_ELEM, QB, HPW, NSLOT, PF, WAVES, ORDER>, ORDER                                        \
    }
// both grid orders of one compiled kernel
#define RING_INSTANCE(QB, HPW, NSLOT, PF, WAVES) \
    RING_ONE(QB, HPW, NSLOT, PF, WAVES, 0, ""), RING_ONE(QB, HPW, NSLOT, PF, WAVES, 1, " seqmajor")

}  // namespace

#ifdef ATTN_RING_ELEM_F16
const Instance *prefill_ring_f16_instances(int *count)
{
    static const Instance table[] = {
        RING_INSTANCE(1, 4, 8, 5, 8), RING_INSTANCE(1, 2, 8, 5, 8), RING_INSTANCE(1, 1, 8, 5, 8),
        RING_INSTANCE(1, 4, 8, 6, 8), RING_INSTANCE(1, 4, 4, 4, 4), RING_INSTANCE(1, 2, 4, 4, 4),
        RING_INSTANCE(1, 1, 4, 4, 4),
    };
    *count = (int)(sizeof(table) / sizeof(table[0]));
    return table;
}
#else
const Instance *prefill_ring_instances(int *count)
{
    static const Instance table[] = {
        RING_INSTANCE(1, 4, 8, 5, 8), RING_INSTANCE(1, 8, 8, 5, 8),
        RING_INSTANCE(1, 2, 8, 5, 8), RING_INSTANCE(1, 1, 8, 5, 8), RING_INSTANCE(1, 4, 8, 6, 8),
        RING_INSTANCE(1, 4, 8, 8, 8), RING_INSTANCE(1, 1, 8, 8, 8), RING_INSTANCE(1, 4, 4, 4, 4),
        RING_INSTANCE(1, 1, 4, 4, 4), RING_INSTANCE(1, 2, 4, 4, 4),
    };
    *count = (int)(sizeof(table) / sizeof(table[0]));
    return table;
}
#endif

}  // namespace attn

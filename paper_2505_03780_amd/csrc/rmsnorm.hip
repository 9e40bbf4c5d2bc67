// Fused residual add + RMS layer norm for gfx950: kernels, instance table, host entry points and
// the tuner hook-up.  The operation is the paper's second kernel (section "Method and Investigated
// Kernels"; Table I; Fig. 3).  The path is bound by HBM: 2 H bytes are read per row for x, 2 H for
// the residual, and as many written for each of the two outputs; the weight stays in cache.
//
// Every row is read once into registers, as 16-byte vectors spread over the TPR lanes that share the
// row, so the square sum, the scale and both stores need no second pass over memory.  The template
// parameters are the tunable configuration (the paper's requirement list: a declared parameter space
// with validity predicates): TPR lanes per row, VPT vectors per lane, ROWS rows per workgroup.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <string>
#include <vector>

#include "../../include/attn.h"
#include "../../include/rmsnorm.h"
#include "tuner_cache.hpp"

namespace attn {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
// Activations pass through once: non-temporal loads and stores keep the stream from displacing the
// caches' contents (measured on 8192 x 4096: 5.8 TB/s with the hint on both sides, 5.3 without).
#define RMS_LD(p) __builtin_nontemporal_load(p)
#define RMS_ST(v, p) __builtin_nontemporal_store(v, p)

struct RmsParams {
    const void *x;
    void *residual;
    const void *weight;
    void *out;
    int64_t x_stride, residual_stride, out_stride;
    int32_t num_tokens, hidden;
    float eps, inv_hidden;
    int32_t f16;  // element type: 0 = bf16, 1 = IEEE fp16
};

// two packed elements <-> fp32; the stores round to nearest even
template <bool F16>
__device__ __forceinline__ float elem_lo(uint32_t w)
{
    typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
    if (F16) return (float)__builtin_bit_cast(f16x2, w)[0];
    return __uint_as_float(w << 16);
}
template <bool F16>
__device__ __forceinline__ float elem_hi(uint32_t w)
{
    typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
    if (F16) return (float)__builtin_bit_cast(f16x2, w)[1];
    return __uint_as_float(w & 0xffff0000u);
}
template <bool F16>
__device__ __forceinline__ uint32_t pack_elems(float a, float b)
{
    if (F16) {
        typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
        f16x2 v;
        v[0] = (_Float16)a;
        v[1] = (_Float16)b;
        return __builtin_bit_cast(uint32_t, v);
    }
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 v;
    v[0] = (__bf16)a;
    v[1] = (__bf16)b;
    return __builtin_bit_cast(uint32_t, v);
}

template <bool F16, int TPR, int VPT, int ROWS>
__global__ __launch_bounds__(TPR *ROWS) void rmsnorm_kernel(const RmsParams p)
{
    constexpr int WAVES_PER_ROW = TPR > 64 ? TPR / 64 : 1;
    __shared__ float partial[ROWS * WAVES_PER_ROW];
    const int t = threadIdx.x % TPR;
    const int r_local = threadIdx.x / TPR;
    const int row_raw = blockIdx.x * ROWS + r_local;
    const bool live = row_raw < p.num_tokens;
    const int row = live ? row_raw : p.num_tokens - 1;  // idle rows shadow the last one and store nothing
    const int nvec = p.hidden >> 3;

    const unsigned char *xr = (const unsigned char *)p.x + (int64_t)row * p.x_stride * 2;
    unsigned char *rr = p.residual ? (unsigned char *)p.residual + (int64_t)row * p.residual_stride * 2 : nullptr;
    unsigned char *orow = (unsigned char *)p.out + (int64_t)row * p.out_stride * 2;

    float z[VPT][8];
    float ss = 0.f;
#pragma unroll
    for (int k = 0; k < VPT; ++k) {
        const int i = t + k * TPR;
        u32x4 a = {0u, 0u, 0u, 0u}, b = {0u, 0u, 0u, 0u};
        if (i < nvec) {
            a = RMS_LD((const u32x4 *)(xr + 16 * i));
            if (rr) b = RMS_LD((const u32x4 *)(rr + 16 * i));
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            z[k][2 * e] = elem_lo<F16>(a[e]) + elem_lo<F16>(b[e]);
            z[k][2 * e + 1] = elem_hi<F16>(a[e]) + elem_hi<F16>(b[e]);
            ss = __builtin_fmaf(z[k][2 * e], z[k][2 * e], ss);
            ss = __builtin_fmaf(z[k][2 * e + 1], z[k][2 * e + 1], ss);
        }
    }
    // the new residual can go out before the reduction
    if (rr && live) {
#pragma unroll
        for (int k = 0; k < VPT; ++k) {
            const int i = t + k * TPR;
            if (i < nvec) {
                u32x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = pack_elems<F16>(z[k][2 * e], z[k][2 * e + 1]);
                RMS_ST(o, (u32x4 *)(rr + 16 * i));
            }
        }
    }
    // square sum over the lanes of the row: inside the wavefront, then (rows wider than a wavefront) through LDS
    constexpr int SHUF = TPR < 64 ? TPR : 64;
#pragma unroll
    for (int sh = 1; sh < SHUF; sh <<= 1) ss += __shfl_xor(ss, sh);
    if (WAVES_PER_ROW > 1) {
        const int w = t >> 6;
        if ((t & 63) == 0) partial[r_local * WAVES_PER_ROW + w] = ss;
        __syncthreads();
        ss = 0.f;
#pragma unroll
        for (int i = 0; i < WAVES_PER_ROW; ++i) ss += partial[r_local * WAVES_PER_ROW + i];
    }
    const float inv = 1.0f / sqrtf(__builtin_fmaf(ss, p.inv_hidden, p.eps));
    if (!live) return;
    const unsigned char *wr = (const unsigned char *)p.weight;
#pragma unroll
    for (int k = 0; k < VPT; ++k) {
        const int i = t + k * TPR;
        if (i < nvec) {
            const u32x4 w4 = *(const u32x4 *)(wr + 16 * i);
            u32x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                o[e] = pack_elems<F16>(z[k][2 * e] * inv * elem_lo<F16>(w4[e]), z[k][2 * e + 1] * inv * elem_hi<F16>(w4[e]));
            RMS_ST(o, (u32x4 *)(orow + 16 * i));
        }
    }
}

struct RmsInstance {
    const char *name;
    int tpr, vpt, rows;
    hipError_t (*launch)(const RmsParams &, hipStream_t);
};

template <int TPR, int VPT, int ROWS>
hipError_t rms_launch(const RmsParams &p, hipStream_t stream)
{
    const unsigned blocks = (unsigned)((p.num_tokens + ROWS - 1) / ROWS);
    if (blocks == 0) return hipSuccess;
    if (p.f16)
        hipLaunchKernelGGL((rmsnorm_kernel<true, TPR, VPT, ROWS>), dim3(blocks), dim3(TPR * ROWS), 0, stream, p);
    else
        hipLaunchKernelGGL((rmsnorm_kernel<false, TPR, VPT, ROWS>), dim3(blocks), dim3(TPR * ROWS), 0, stream, p);
    return hipGetLastError();
}

#define RMS_INSTANCE(TPR, VPT, ROWS)                                                                   \
    {                                                                                                  \
        "rmsnorm tpr" #TPR " vpt" #VPT " rows" #ROWS, TPR, VPT, ROWS, rms_launch<TPR, VPT, ROWS>      \
    }

const RmsInstance kInstances[] = {
    RMS_INSTANCE(32, 4, 8),   RMS_INSTANCE(32, 8, 8),   RMS_INSTANCE(64, 2, 4),   RMS_INSTANCE(64, 4, 4),
    RMS_INSTANCE(64, 8, 4),   RMS_INSTANCE(64, 16, 4),  RMS_INSTANCE(64, 8, 1),   RMS_INSTANCE(128, 2, 2),
    RMS_INSTANCE(128, 4, 2),  RMS_INSTANCE(128, 8, 2),  RMS_INSTANCE(128, 4, 1),  RMS_INSTANCE(256, 1, 1),
    RMS_INSTANCE(256, 2, 1),  RMS_INSTANCE(256, 4, 1),  RMS_INSTANCE(256, 8, 1),  RMS_INSTANCE(256, 2, 2),
    RMS_INSTANCE(512, 1, 1),  RMS_INSTANCE(512, 2, 1),  RMS_INSTANCE(512, 4, 1),  RMS_INSTANCE(1024, 1, 1),
    RMS_INSTANCE(1024, 2, 1),
};
constexpr int kNumInstances = (int)(sizeof(kInstances) / sizeof(kInstances[0]));

// An instance fits when its lanes cover the row, and is not dominated by one with half the registers.
bool rms_valid(const RmsInstance &in, int hidden)
{
    const int nvec = hidden / 8;
    const int cap = in.tpr * in.vpt;
    return nvec <= cap && (in.vpt == 1 || nvec > in.tpr * (in.vpt / 2));
}

std::atomic<int> g_forced{-1};

int validate(const rmsnorm_args *a)
{
    if (!a) return ATTN_ERR_NULL;
    if (a->struct_bytes != sizeof(rmsnorm_args)) return ATTN_ERR_SHAPE;
    if (a->dtype != ATTN_BF16 && a->dtype != ATTN_F16) return ATTN_ERR_DTYPE;
    if (a->num_tokens < 0 || a->hidden <= 0) return ATTN_ERR_SHAPE;
    if (a->hidden % 8 != 0 || a->hidden > 16384) return ATTN_ERR_UNSUPPORTED;
    if (a->num_tokens == 0) return ATTN_OK;
    if (!a->x || !a->weight || !a->out) return ATTN_ERR_NULL;
    if (a->x_stride < a->hidden || a->out_stride < a->hidden || a->x_stride % 8 || a->out_stride % 8) return ATTN_ERR_SHAPE;
    if (a->residual && (a->residual_stride < a->hidden || a->residual_stride % 8)) return ATTN_ERR_SHAPE;
    if (((uintptr_t)a->x | (uintptr_t)a->weight | (uintptr_t)a->out | (uintptr_t)a->residual) & 15) return ATTN_ERR_SHAPE;
    return ATTN_OK;
}

RmsParams to_params(const rmsnorm_args *a)
{
    RmsParams p{};
    p.x = a->x;
    p.residual = a->residual;
    p.weight = a->weight;
    p.out = a->out;
    p.x_stride = a->x_stride;
    p.residual_stride = a->residual_stride;
    p.out_stride = a->out_stride;
    p.num_tokens = a->num_tokens;
    p.hidden = a->hidden;
    p.eps = a->eps;
    p.inv_hidden = 1.0f / (float)a->hidden;
    p.f16 = a->dtype == ATTN_F16;
    return p;
}

int ilog2_ceil(int x)
{
    int e = 0;
    while ((1 << e) < x) ++e;
    return e;
}

std::string bucket_key(const rmsnorm_args *a)
{
    char buf[96];
    snprintf(buf, sizeof buf, "rmsnorm|%s|h%d|res%d|T%d", a->dtype == ATTN_F16 ? "f16" : "bf16", a->hidden, a->residual ? 1 : 0, ilog2_ceil(std::max(1, a->num_tokens)));
    return buf;
}

// Built-in choice, from a sweep over hidden sizes 1024..8192 and 16..32768 rows: the fewest vectors
// per lane (the row spread over as many lanes as it has 16-byte vectors, up to 1024) wins or ties
// everywhere; among those the narrowest workgroup that covers the row, with the most rows.
int heuristic(const rmsnorm_args *a)
{
    // Exception, from the same sweep after the loads and stores became non-temporal: calls that move
    // about 24-160 MB over rows of at most 4096 elements run 15-30 % faster with four vectors per lane
    // in workgroups of 256 lanes (several rows each), i.e. with a quarter of the workgroups.
    const double traffic = 8.0 * (double)a->num_tokens * (double)a->hidden;
    if (a->hidden <= 4096 && traffic >= 24e6 && traffic <= 160e6)
        for (int i = 0; i < kNumInstances; ++i)
            if (kInstances[i].vpt == 4 && kInstances[i].tpr * kInstances[i].rows == 256 && rms_valid(kInstances[i], a->hidden)) return i;
    int best = -1;
    for (int i = 0; i < kNumInstances; ++i) {
        if (!rms_valid(kInstances[i], a->hidden)) continue;
        if (best < 0) {
            best = i;
            continue;
        }
        const RmsInstance &c = kInstances[i], &b = kInstances[best];
        if (c.vpt < b.vpt || (c.vpt == b.vpt && (c.tpr < b.tpr || (c.tpr == b.tpr && c.rows > b.rows)))) best = i;
    }
    return best;
}

int select(const rmsnorm_args *a)
{
    const int forced = g_forced.load();
    if (forced >= 0) return forced < kNumInstances && rms_valid(kInstances[forced], a->hidden) ? forced : ATTN_ERR_UNSUPPORTED;
    load_env_cache_once();
    std::string name;
    if (lookup_named_winner(bucket_key(a), &name))
        for (int i = 0; i < kNumInstances; ++i)
            if (name == kInstances[i].name && rms_valid(kInstances[i], a->hidden)) return i;
    const int id = heuristic(a);
    return id >= 0 ? id : ATTN_ERR_UNSUPPORTED;
}

int run(const rmsnorm_args *a, hipStream_t stream, int override_id)
{
    int rc = validate(a);
    if (rc != ATTN_OK) return rc;
    if (a->num_tokens == 0) return ATTN_OK;
    const int id = override_id >= 0 ? override_id : select(a);
    if (id < 0) return id;
    if (id >= kNumInstances || !rms_valid(kInstances[id], a->hidden)) return ATTN_ERR_UNSUPPORTED;
    return kInstances[id].launch(to_params(a), stream) == hipSuccess ? ATTN_OK : ATTN_ERR_HIP;
}

// pseudo-random values in [-2, 2), truncated to bf16 or rounded to fp16
__global__ void fill_elems_kernel(uint16_t *dst, size_t n, uint32_t seed, int f16)
{
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        uint32_t h = (uint32_t)i * 2654435761u ^ seed;
        h ^= h >> 15;
        h *= 2246822519u;
        h ^= h >> 13;
        const float f = ((int)(h & 0xffff) - 32768) * (1.f / 16384.f);
        const _Float16 hf = (_Float16)f;
        dst[i] = f16 ? __builtin_bit_cast(uint16_t, hf) : (uint16_t)(__float_as_uint(f) >> 16);
    }
}

int tune(const rmsnorm_args *shape, const char *cache_path, int iters, int flags)
{
    if (!shape) return ATTN_ERR_NULL;
    if (shape->struct_bytes != sizeof(rmsnorm_args)) return ATTN_ERR_SHAPE;
    if (shape->dtype != ATTN_BF16 && shape->dtype != ATTN_F16) return ATTN_ERR_DTYPE;
    if (shape->num_tokens <= 0 || shape->hidden <= 0) return ATTN_ERR_SHAPE;
    if (shape->hidden % 8 != 0 || shape->hidden > 16384) return ATTN_ERR_UNSUPPORTED;
    if (iters <= 0) iters = 20;
    const size_t n = (size_t)shape->num_tokens * shape->hidden;
    void *bufs[4] = {nullptr, nullptr, nullptr, nullptr};  // x, residual, out, weight
    auto release = [&]() {
        for (void *b : bufs)
            if (b) (void)hipFree(b);
    };
    for (int i = 0; i < 4; ++i)
        if (hipMalloc(&bufs[i], (i == 3 ? (size_t)shape->hidden : n) * 2) != hipSuccess) {
            (void)hipGetLastError();
            release();
            return ATTN_ERR_HIP;
        }
    const int f16 = shape->dtype == ATTN_F16;
    hipLaunchKernelGGL(fill_elems_kernel, dim3(2048), dim3(256), 0, 0, (uint16_t *)bufs[0], n, 11u, f16);
    hipLaunchKernelGGL(fill_elems_kernel, dim3(2048), dim3(256), 0, 0, (uint16_t *)bufs[1], n, 12u, f16);
    hipLaunchKernelGGL(fill_elems_kernel, dim3(64), dim3(256), 0, 0, (uint16_t *)bufs[3], (size_t)shape->hidden, 13u, f16);
    rmsnorm_args a = *shape;
    a.x = bufs[0];
    a.residual = shape->residual ? bufs[1] : nullptr;
    a.out = bufs[2];
    a.weight = bufs[3];
    a.x_stride = a.residual_stride = a.out_stride = shape->hidden;
    if (a.eps == 0.f) a.eps = 1e-6f;
    const std::string key = bucket_key(&a);
    hipEvent_t e0, e1;
    if (hipDeviceSynchronize() != hipSuccess || hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
        (void)hipGetLastError();
        release();
        return ATTN_ERR_HIP;
    }
    // one timed call; negative on failure
    auto time_once = [&](int id) -> double {
        float ms = 0.f;
        (void)hipEventRecord(e0, 0);
        const bool ok = run(&a, 0, id) == ATTN_OK;
        (void)hipEventRecord(e1, 0);
        if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess || !ok) {
            (void)hipGetLastError();
            return -1.0;
        }
        return 1000.0 * ms;
    };
    auto median = [](std::vector<double> &v) {
        std::sort(v.begin(), v.end());
        return v[v.size() / 2];
    };
    // First pass: every valid instance on its own, median of `iters` calls.
    std::vector<std::pair<double, int>> ranked;
    for (int id = 0; id < kNumInstances; ++id) {
        if (!rms_valid(kInstances[id], a.hidden)) continue;
        bool fail = false;
        for (int w = 0; w < 2 && !fail; ++w) fail = run(&a, 0, id) != ATTN_OK;
        if (fail || hipDeviceSynchronize() != hipSuccess) {
            (void)hipGetLastError();
            continue;
        }
        std::vector<double> us(iters);
        for (int i = 0; i < iters && !fail; ++i) fail = (us[i] = time_once(id)) < 0.0;
        if (fail) continue;
        const double m = median(us);
        if (flags & 1) fprintf(stderr, "[rmsnorm_tune] %s :: %-36s %10.2f us\n", key.c_str(), kInstances[id].name, m);
        ranked.push_back({m, id});
    }
    // Final: the three fastest and the built-in choice are measured again taking turns call by call
    // (instances measured minutes apart see different clocks); the built-in choice keeps ties within 3 %.
    int best = -1;
    double best_us = 0.0;
    if (!ranked.empty()) {
        std::sort(ranked.begin(), ranked.end());
        std::vector<int> finalists;
        for (size_t i = 0; i < ranked.size() && i < 3; ++i) finalists.push_back(ranked[i].second);
        const int builtin = heuristic(&a);
        if (builtin >= 0 && rms_valid(kInstances[builtin], a.hidden) && std::find(finalists.begin(), finalists.end(), builtin) == finalists.end())
            finalists.push_back(builtin);
        std::vector<std::vector<double>> turns(finalists.size());
        bool fail = false;
        for (int i = 0; i < iters && !fail; ++i)
            for (size_t f = 0; f < finalists.size() && !fail; ++f) {
                const double t = time_once(finalists[f]);
                fail = t < 0.0;
                turns[f].push_back(t);
            }
        if (fail) {  // keep the first pass's answer
            best = ranked[0].second;
            best_us = ranked[0].first;
        } else {
            double builtin_us = -1.0;
            for (size_t f = 0; f < finalists.size(); ++f) {
                const double m = median(turns[f]);
                if (flags & 1) fprintf(stderr, "[rmsnorm_tune] %s :: final %-30s %10.2f us\n", key.c_str(), kInstances[finalists[f]].name, m);
                if (finalists[f] == builtin) builtin_us = m;
                if (best < 0 || m < best_us) {
                    best = finalists[f];
                    best_us = m;
                }
            }
            if (builtin_us > 0.0 && best != builtin && best_us > 0.97 * builtin_us) {
                best = builtin;
                best_us = builtin_us;
            }
        }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    release();
    if (best < 0) return ATTN_ERR_UNSUPPORTED;
    store_named_winner(key, kInstances[best].name);
    if (flags & 1) fprintf(stderr, "[rmsnorm_tune] winner %s -> %s (%.2f us)\n", key.c_str(), kInstances[best].name, best_us);
    return cache_path ? merge_cache_line(cache_path, key, kInstances[best].name, best_us) : ATTN_OK;
}

}  // namespace
}  // namespace attn

extern "C" {

int rmsnorm_fused_add(const rmsnorm_args *args, void *hip_stream) { return attn::run(args, (hipStream_t)hip_stream, -1); }

int rmsnorm_tune(const rmsnorm_args *shape_like, const char *cache_path, int iters, int flags)
{
    return attn::tune(shape_like, cache_path, iters, flags);
}

int rmsnorm_num_instances(void) { return attn::kNumInstances; }

int rmsnorm_instance_name(int id, char *buf, size_t buf_bytes)
{
    if (id < 0 || id >= attn::kNumInstances) return ATTN_ERR_SHAPE;
    if (buf && buf_bytes) snprintf(buf, buf_bytes, "%s", attn::kInstances[id].name);
    return (int)strlen(attn::kInstances[id].name);
}

int rmsnorm_selected_instance(const rmsnorm_args *args)
{
    const int rc = attn::validate(args);
    return rc != ATTN_OK ? rc : attn::select(args);
}

void rmsnorm_force_instance(int id) { attn::g_forced.store(id); }

}  // extern "C"

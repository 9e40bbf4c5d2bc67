// C ABI of the attention library: argument validation, shape buckets, instance
// selection (winner cache, else heuristic), the in-library autotuner and its
// persistent cache.
//
// The tuner is the paper's thesis applied natively: instead of JIT-compiling
// configurations at first call, every configuration is a template instance
// compiled ahead of time; attn_tune times the valid ones for a shape bucket off
// the critical path and stores the winner, together with the environment it was
// measured in, in a file that later processes load (the paper's list of gaps
// towards practical autotuning: configuration spaces with parameter
// dependencies, reusable caches that record their environment, tuning moved off
// the critical path).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <fstream>
#include <mutex>
#include <sstream>
#include <string>
#include <unordered_map>
#include <vector>

#include <fcntl.h>
#include <sys/file.h>
#include <unistd.h>

#include "../../include/attn.h"
#include "kernel_params.hpp"
#include "tuner_cache.hpp"

namespace attn {
namespace {

constexpr const char *kCacheMagic = "attn-tune-cache-v1";
// Changes whenever the kernels change in a way that invalidates old timings.
// Identifies the set of compiled instances: a cache line tuned against another set must not be
// trusted (the paper asks that cached results record the environment they were measured in).
std::string build_id();
// Bounds on the split-K records of the fixed-split decode kernels: a context is cut into at most
// kMaxPartsPerSeq parts, and a batch into at most two parts per compute unit in all (more parts add
// workspace traffic and merge work, never parallelism: every part already is Hkv workgroups).
constexpr int kMaxPartsPerSeq = 64;

std::mutex g_mu;
std::unordered_map<std::string, int> g_winner[2];  // [is_decode]: bucket key -> instance id
std::unordered_map<std::string, std::string> g_named;  // other kernel kinds: bucket key -> instance name
std::atomic<int> g_forced[2] = {{-1}, {-1}};
bool g_env_cache_tried = false;
// bumped whenever the winner table may have changed (tune, load, clear): invalidates the per-thread memo
std::atomic<uint64_t> g_generation{1};

const Instance *all_decode_instances(int *count);
const Instance *instances(int is_decode, int *n) { return is_decode ? all_decode_instances(n) : prefill_instances(n); }
bool is16(int dtype) { return dtype == ATTN_BF16 || dtype == ATTN_F16; }

int ilog2_ceil(int64_t x)
{
    int r = 0;
    while (((int64_t)1 << r) < x) ++r;
    return r;
}

// ---- validation --------------------------------------------------------------------------------

int validate(const attn_args *a, int is_decode)
{
    if (!a) return ATTN_ERR_NULL;
    if (a->struct_bytes != sizeof(attn_args)) return ATTN_ERR_SHAPE;
    if (a->dtype != ATTN_F32 && !is16(a->dtype)) return ATTN_ERR_DTYPE;
    if (is_decode && !is16(a->dtype)) return ATTN_ERR_DTYPE;
    if (a->num_seqs < 0 || a->num_q_heads <= 0 || a->num_kv_heads <= 0 || a->total_q < 0 || a->max_q_len < 0 ||
        a->max_kv_len < 0)
        return ATTN_ERR_SHAPE;
    if (a->num_q_heads % a->num_kv_heads != 0) return ATTN_ERR_SHAPE;
    if (a->head_dim != 64 && a->head_dim != 128) return ATTN_ERR_UNSUPPORTED;
    if (is_decode && a->total_q != a->num_seqs) return ATTN_ERR_SHAPE;
    if (is_decode && a->max_q_len > 1) return ATTN_ERR_SHAPE;
    const int vec = is16(a->dtype) ? 8 : 1;  // elements per 16-byte vector access
    if (a->q_stride_head < a->head_dim || a->o_stride_head < a->head_dim || a->kv_stride_head < a->head_dim ||
        a->q_stride_tok <= 0 || a->o_stride_tok <= 0 || a->kv_stride_tok <= 0)
        return ATTN_ERR_SHAPE;
    if (a->q_stride_tok % vec || a->q_stride_head % vec || a->o_stride_tok % vec || a->o_stride_head % vec ||
        a->kv_stride_tok % vec || a->kv_stride_head % vec)
        return ATTN_ERR_SHAPE;
    if (a->block_table) {
        if (a->block_size < 16 || (a->block_size & (a->block_size - 1)) != 0) return ATTN_ERR_UNSUPPORTED;
        if (a->block_table_stride <= 0 || a->num_blocks <= 0 || a->kv_stride_block <= 0 || a->kv_stride_block % vec)
            return ATTN_ERR_SHAPE;
        if ((int64_t)a->block_table_stride * a->block_size < a->max_kv_len) return ATTN_ERR_SHAPE;
    } else if (is_decode) {
        return ATTN_ERR_NULL;  // decode is paged only
    }
    if (a->num_seqs == 0 || a->total_q == 0) return ATTN_OK;  // nothing to do; pointers may be NULL
    if (!a->q || !a->out || !a->seq_lens) return ATTN_ERR_NULL;
    if (a->max_kv_len > 0 && (!a->k || !a->v)) return ATTN_ERR_NULL;
    if (!is_decode && !a->query_start_loc) return ATTN_ERR_NULL;
    if (is16(a->dtype)) {
        const uintptr_t bits = (uintptr_t)a->q | (uintptr_t)a->out | (uintptr_t)a->k | (uintptr_t)a->v;
        if (bits & 15) return ATTN_ERR_SHAPE;  // 128-bit accesses
    }
    return ATTN_OK;
}

KParams to_kparams(const attn_args *a, int is_decode)
{
    KParams p{};
    p.dtype = a->dtype;
    p.q = a->q;
    p.out = a->out;
    p.k = a->k;
    p.v = a->v;
    p.block_table = a->block_table;
    p.query_start_loc = is_decode ? nullptr : a->query_start_loc;
    p.kv_start_loc = a->kv_start_loc ? a->kv_start_loc : a->query_start_loc;
    p.seq_lens = a->seq_lens;
    p.q_stride_tok = a->q_stride_tok;
    p.q_stride_head = a->q_stride_head;
    p.o_stride_tok = a->o_stride_tok;
    p.o_stride_head = a->o_stride_head;
    p.kv_stride_block = a->kv_stride_block;
    p.kv_stride_tok = a->kv_stride_tok;
    p.kv_stride_head = a->kv_stride_head;
    p.num_seqs = a->num_seqs;
    p.num_q_heads = a->num_q_heads;
    p.num_kv_heads = a->num_kv_heads;
    p.head_dim = a->head_dim;
    p.group = a->num_q_heads / a->num_kv_heads;
    p.block_table_stride = a->block_table_stride;
    p.block_size = a->block_table ? a->block_size : 0;
    p.block_shift = a->block_table ? ilog2_ceil(a->block_size) : 0;
    p.max_q_len = is_decode ? 1 : a->max_q_len;
    p.max_kv_len = a->max_kv_len;
    p.scale = a->scale;
    p.scale_log2e = a->scale * 1.4426950408889634f;
    p.causal = a->causal ? 1 : 0;
    p.workspace = (float *)a->workspace;
    p.num_splits = 1;
    p.split_len = 0;
    return p;
}

// ---- shape buckets ------------------------------------------------------------------------------
// A bucket fixes everything a kernel instance is specialised on and rounds the three extents
// (sequences, longest query, longest context) up to powers of two.
std::string bucket_key(const KParams &p, int dtype, int is_decode)
{
    char buf[192];
    snprintf(buf, sizeof buf, "%s|%s|d%d|hq%d|hkv%d|%s|bs%d|c%d|B%d|q%d|kv%d", is_decode ? "decode" : "prefill",
             dtype == ATTN_BF16 ? "bf16" : dtype == ATTN_F16 ? "f16" : "f32", p.head_dim, p.num_q_heads, p.num_kv_heads,
             p.block_table ? "paged" : "contig", p.block_size, p.causal, ilog2_ceil(std::max(1, p.num_seqs)),
             ilog2_ceil(std::max(1, p.max_q_len)), ilog2_ceil(std::max(1, p.max_kv_len)));
    return buf;
}

// Keys of the buckets next to the one of `p`: one step up or down in each of the three extents.
std::vector<std::string> neighbour_keys(const KParams &p, int dtype, int is_decode)
{
    std::vector<std::string> out;
    for (int axis = 0; axis < 3; ++axis)
        for (int dir = -1; dir <= 1; dir += 2) {
            KParams q = p;
            int *ext = axis == 0 ? &q.num_seqs : axis == 1 ? &q.max_q_len : &q.max_kv_len;
            const int e = ilog2_ceil(std::max(1, *ext)) + dir;
            if (e < 0 || e > 30 || (axis == 1 && is_decode)) continue;
            *ext = 1 << e;
            out.push_back(bucket_key(q, dtype, is_decode));
        }
    return out;
}

constexpr int kMaxBalancedWgs = 2048;  // launch bound of the token-balanced decode

int compute_units()
{
    static std::atomic<int> cached{0};
    int cu = cached.load();
    if (cu > 0) return cu;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
        (void)hipGetLastError();
        return 256;
    }
    cached.store(prop.multiProcessorCount);
    return prop.multiProcessorCount;
}

// Parts per sequence a fixed-split decode instance cuts the longest context into (1: no split).
int fixed_parts(const KParams &p, const Instance &inst)
{
    const int sl = inst.split_len;
    return (sl <= 0 || sl >= p.max_kv_len) ? 1 : (p.max_kv_len + sl - 1) / sl;
}

// The parameter-dependency predicate of an instance (the paper's requirement list asks for
// configuration spaces that carry the dependencies between parameters): the kernel's own conditions,
// and for a fixed-split decode instance the bound on the split-K records.
bool usable(const Instance &inst, const KParams &p, int is_decode)
{
    if (!inst.valid(p)) return false;
    if (!is_decode || inst.split_len <= 0) return true;
    const int parts = fixed_parts(p, inst);
    if (parts == 1) return true;
    return parts <= kMaxPartsPerSeq && (int64_t)p.num_seqs * parts <= std::max<int64_t>(2 * compute_units(), 2);
}

void apply_split(KParams &p, const Instance &inst)
{
    int sl = inst.split_len;
    if (sl < 0) {  // token-balanced: a fixed number of workgroups, each with an equal share of the chunks
        const int waves = inst.waves;
        const int head_blocks = (p.num_kv_heads + waves - 1) / waves;
        int wgs = compute_units() * (-sl) * (8 / waves) / head_blocks;
        wgs = std::max(1, std::min(wgs, kMaxBalancedWgs));
        p.num_splits = wgs;
        p.split_len = 0;
        return;
    }
    if (sl <= 0 || sl >= p.max_kv_len) {
        p.split_len = std::max(p.max_kv_len, 1);
        p.num_splits = 1;
    } else {
        p.split_len = sl;
        p.num_splits = (p.max_kv_len + sl - 1) / sl;
    }
}

// ---- built-in heuristic (used until a bucket has been tuned) -----------------------------------
int find_instance(int is_decode, const KParams &p, int waves, int hpw, int bn, int bm, int split_len, int variant = 0, int stages = 0)
{
    int n;
    const Instance *t = instances(is_decode, &n);
    for (int i = 0; i < n; ++i) {
        if (!usable(t[i], p, is_decode)) continue;
        if (t[i].waves == waves && t[i].heads_per_wg == hpw && t[i].block_n == bn && (bm <= 0 || t[i].block_m == bm) &&
            t[i].split_len == split_len && t[i].variant == variant && (stages <= 0 || t[i].stages == stages))
            return i;
    }
    return -1;
}

int heuristic(const KParams &p, int is_decode)
{
    int n;
    const Instance *t = instances(is_decode, &n);
    int id = -1;
    if (!is_decode) {
        // pack as many heads of a KV head as divide the group: they share every K/V tile
        int hpw = p.group % 4 == 0 ? 4 : (p.group % 2 == 0 ? 2 : 1);
        // The rules below come from tuning a batch x length grid (profiles: configuration portability).
        // Sequences of many query tiles, many sequences, or a cached prefix that dominates the key
        // range: run the tiles of a sequence side by side so that they share its K/V in one L2.
        const bool prefix = p.block_table && p.max_kv_len >= 2 * p.max_q_len;
        const int order = (prefix || p.max_kv_len >= 4096 || p.num_seqs >= 32) ? 1 : 0;
        // Short sequences: two small workgroups per compute unit hide each other's prologue and
        // epilogue; long ones: one large workgroup with the deeper ring.
        const bool small_wg = p.max_kv_len <= 2048;
        // a paged context adds the table entry to every transfer's address chain: the deepest prefetch
        // (8 units) measured up to 10 % ahead of 5 on the slower machines there, level elsewhere
        if (!small_wg && p.block_table) id = find_instance(0, p, 8, hpw, 32, 256, 0, order, 8);
        if (id < 0) id = find_instance(0, p, small_wg ? 4 : 8, hpw, 32, small_wg ? 128 : 256, 0, order);  // LDS-ring kernel (D = 128)
        if (id < 0) id = find_instance(0, p, 8, hpw, 32, 256, 0, order);
        if (id < 0) id = find_instance(0, p, 4, hpw, 32, 256, 0, order);
        if (id < 0) id = find_instance(0, p, 4, hpw, 64, 64 * 4, 0);  // register-staged kernel
    } else {
        // With four or more KV heads and enough keys to give every compute unit a long run, a workgroup
        // owns whole cache blocks (one wavefront per head): the token-balanced kernel, one workgroup
        // per compute unit.  Small batches of short contexts start and finish faster with one KV head
        // per workgroup and fixed parts: enough workgroups to fill the chip several times over, parts
        // no shorter than 256 keys.
        const int64_t key_bound = (int64_t)p.num_seqs * p.max_kv_len;
        if (p.num_kv_heads >= 4 && key_bound >= 100000) {
            // two workgroups of four heads per compute unit measured 0.5-2 % ahead of one of eight from
            // eight KV heads on, 1-2 % behind at four
            if (p.num_kv_heads >= 8) id = find_instance(1, p, 4, 16, 32, 0, -1);
            if (id < 0) id = find_instance(1, p, 8, 16, 32, 0, -1);
        }
        if (id < 0) {
            const int64_t units = (int64_t)p.num_seqs * p.num_kv_heads;
            int64_t want = units * (int64_t)p.max_kv_len / 2048;
            int sl = 256;
            while (sl * 2 <= want && sl < 4096) sl *= 2;
            if (sl >= p.max_kv_len) sl = 0;
            // the merge takes 32 parts per round trip: a long context in few units gets longer parts and
            // eight waves per workgroup rather than more parts
            bool wide = false;
            while (sl > 0 && sl < 4096 && (p.max_kv_len + sl - 1) / sl > 32) {
                sl *= 2;
                wide = true;
            }
            // and the batch at most two parts per compute unit in all (the bound `usable` enforces)
            while (sl > 0 && sl < 4096 && (int64_t)p.num_seqs * ((p.max_kv_len + sl - 1) / sl) > 2 * compute_units()) sl *= 2;
            if (sl >= p.max_kv_len || (sl > 0 && (int64_t)p.num_seqs * ((p.max_kv_len + sl - 1) / sl) > 2 * compute_units())) sl = 0;
            if (wide) id = find_instance(1, p, 8, 16, 32, 0, sl);
            if (id < 0) id = find_instance(1, p, 4, 16, 32, 0, sl);
            if (id < 0) id = find_instance(1, p, 4, 16, 32, 0, 0);
            if (id < 0) id = find_instance(1, p, 8, 16, 32, 0, sl);  // fp16 has the wave-per-head family only
            if (id < 0) id = find_instance(1, p, 8, 16, 32, 0, 0);
        }
    }
    if (id >= 0) return id;
    for (int i = 0; i < n; ++i)
        if (usable(t[i], p, is_decode)) return i;
    return -1;
}

// ---- environment key and cache file ------------------------------------------------------------
std::string env_key_impl()
{
    hipDeviceProp_t prop;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
        (void)hipGetLastError();
        return std::string("nodevice|cu0|") + build_id();
    }
    int rt = 0, drv = 0;
    (void)hipRuntimeGetVersion(&rt);
    (void)hipDriverGetVersion(&drv);
    std::ostringstream os;
    os << prop.gcnArchName << "|cu" << prop.multiProcessorCount << "|hip" << rt << "|drv" << drv << "|" << build_id();
    return os.str();
}

std::string build_id()
{
    // FNV-1a over the names of all instances, in table order
    uint64_t h = 1469598103934665603ull;
    for (int is_decode = 0; is_decode < 2; ++is_decode) {
        int n;
        const Instance *t = instances(is_decode, &n);
        for (int i = 0; i < n; ++i)
            for (const char *c = t[i].name; *c; ++c) h = (h ^ (unsigned char)*c) * 1099511628211ull;
    }
    char buf[24];
    snprintf(buf, sizeof buf, "k%016llx", (unsigned long long)h);
    return buf;
}

int instance_by_name(int is_decode, const std::string &name)
{
    int n;
    const Instance *t = instances(is_decode, &n);
    for (int i = 0; i < n; ++i)
        if (name == t[i].name) return i;
    return -1;
}

struct CacheLine {
    std::string env, key, inst;
    double us;
};

bool parse_line(const std::string &line, CacheLine *out)
{
    // fields separated by tabs: env, bucket key, instance name, microseconds
    std::vector<std::string> f;
    size_t pos = 0;
    while (true) {
        size_t t = line.find('\t', pos);
        f.push_back(line.substr(pos, t == std::string::npos ? std::string::npos : t - pos));
        if (t == std::string::npos) break;
        pos = t + 1;
    }
    if (f.size() != 4) return false;
    char *end = nullptr;
    double us = strtod(f[3].c_str(), &end);
    if (end == f[3].c_str() || !(us >= 0)) return false;
    *out = CacheLine{f[0], f[1], f[2], us};
    return true;
}

// Reads the lines of a cache file.  A line that does not parse is skipped and counted, never a reason
// to drop the lines after it (they may be other environments' winners).  ATTN_ERR_CACHE_IO for a file
// that is missing or does not start with the magic line.
int read_cache_file(const char *path, std::vector<CacheLine> *lines, int *damaged)
{
    *damaged = 0;
    std::ifstream in(path);
    if (!in) return ATTN_ERR_CACHE_IO;
    std::string line;
    if (!std::getline(in, line) || line != kCacheMagic) return ATTN_ERR_CACHE_IO;
    while (std::getline(in, line)) {
        if (line.empty() || line[0] == '#') continue;
        CacheLine cl;
        if (!parse_line(line, &cl)) {
            ++*damaged;
            continue;
        }
        lines->push_back(cl);
    }
    return ATTN_OK;
}

int load_cache_locked(const char *path)
{
    std::vector<CacheLine> lines;
    int damaged = 0;
    int rc = read_cache_file(path, &lines, &damaged);
    if (rc != ATTN_OK) return rc;
    if (lines.empty() && damaged > 0) return ATTN_ERR_CACHE_IO;  // nothing but damage
    const std::string env = env_key_impl();
    for (const CacheLine &cl : lines) {
        if (cl.env != env) continue;  // measured on another device or library build
        const int is_decode = cl.key.compare(0, 6, "decode") == 0;
        if (!is_decode && cl.key.compare(0, 7, "prefill") != 0) {
            g_named[cl.key] = cl.inst;
            continue;
        }
        const int id = instance_by_name(is_decode, cl.inst);
        if (id < 0) continue;
        g_winner[is_decode][cl.key] = id;
    }
    g_generation.fetch_add(1, std::memory_order_release);
    return ATTN_OK;
}

void maybe_load_env_cache()
{
    std::lock_guard<std::mutex> lk(g_mu);
    if (g_env_cache_tried) return;
    g_env_cache_tried = true;
    const char *path = getenv("ATTN_TUNE_CACHE");
    if (path && *path) (void)load_cache_locked(path);
}

// Everything the choice depends on.  A serving loop calls with the same shape over and over: the
// last answer per thread and call kind is kept, so a hot call pays one comparison of this key
// instead of building the bucket string, taking the lock and walking the instance table.
struct SelectKey {
    int32_t dtype, head_dim, num_q_heads, num_kv_heads, paged, block_size, causal, num_seqs, max_q_len, max_kv_len;
    bool operator==(const SelectKey &o) const
    {
        return dtype == o.dtype && head_dim == o.head_dim && num_q_heads == o.num_q_heads && num_kv_heads == o.num_kv_heads &&
               paged == o.paged && block_size == o.block_size && causal == o.causal && num_seqs == o.num_seqs &&
               max_q_len == o.max_q_len && max_kv_len == o.max_kv_len;
    }
};
struct SelectMemo {
    uint64_t generation = 0;
    SelectKey key{};
    int id = -1;
};

// ATTN_FORCE_INSTANCE=<exact instance name>: calls of the kind that has an instance of that name use
// it whenever it is valid for the shape (and fall back to the usual choice when it is not), as if
// it were every bucket's winner.  ATTN_LOG=1: one line on stderr whenever a shape is resolved.
// ATTN_DEBUG_VALIDATE=1: hot calls check the device-side integers first.  All are read once.
struct EnvKnobs {
    int forced[2] = {-1, -1};
    bool log = false;
    bool debug_validate = false;
};

const EnvKnobs &env_knobs()
{
    static const EnvKnobs k = [] {
        EnvKnobs e;
        const char *lg = getenv("ATTN_LOG");
        e.log = lg && lg[0] == '1';
        const char *dbg = getenv("ATTN_DEBUG_VALIDATE");
        e.debug_validate = dbg && dbg[0] == '1';
        if (const char *name = getenv("ATTN_FORCE_INSTANCE"))
            for (int d = 0; d < 2; ++d) e.forced[d] = instance_by_name(d, name);
        return e;
    }();
    return k;
}

int select_instance_slow(const KParams &p, int dtype, int is_decode)
{
    int n;
    const Instance *t = instances(is_decode, &n);
    maybe_load_env_cache();
    const EnvKnobs &env = env_knobs();
    const std::string key = bucket_key(p, dtype, is_decode);
    int id = -1;
    const char *why = "heuristic";
    if (env.forced[is_decode] >= 0 && usable(t[env.forced[is_decode]], p, is_decode)) {
        id = env.forced[is_decode];
        why = "ATTN_FORCE_INSTANCE";
    }
    if (id < 0) {
        std::lock_guard<std::mutex> lk(g_mu);
        auto it = g_winner[is_decode].find(key);
        if (it != g_winner[is_decode].end() && it->second < n && usable(t[it->second], p, is_decode)) {
            id = it->second;
            why = "tuned";
        }
    }
    if (id < 0) id = heuristic(p, is_decode);
    if (env.log) {
        if (id >= 0)
            fprintf(stderr, "[attn] %s %s -> %s (%s)\n", is_decode ? "decode" : "prefill", key.c_str(), t[id].name, why);
        else
            fprintf(stderr, "[attn] %s %s -> no valid instance\n", is_decode ? "decode" : "prefill", key.c_str());
    }
    return id >= 0 ? id : ATTN_ERR_UNSUPPORTED;
}

int select_instance(const KParams &p, int dtype, int is_decode)
{
    const int forced = g_forced[is_decode].load();
    if (forced >= 0) {
        int n;
        const Instance *t = instances(is_decode, &n);
        return forced < n && usable(t[forced], p, is_decode) ? forced : ATTN_ERR_UNSUPPORTED;
    }
    static thread_local SelectMemo memo[2];
    SelectMemo &m = memo[is_decode];
    const SelectKey key{dtype, p.head_dim, p.num_q_heads, p.num_kv_heads, p.block_table ? 1 : 0, p.block_size, p.causal,
                        p.num_seqs, p.max_q_len, p.max_kv_len};
    const uint64_t gen = g_generation.load(std::memory_order_acquire);
    if (m.generation == gen && m.key == key) return m.id;
    const int id = select_instance_slow(p, dtype, is_decode);
    // the generation is read again: a table change that raced with the slow path must not be memoised
    if (g_generation.load(std::memory_order_acquire) == gen) {
        m.generation = gen;
        m.key = key;
        m.id = id;
    }
    return id;
}

size_t balanced_workspace_bytes(int num_seqs, int num_q_heads, int head_dim, int wgs)
{
    return (size_t)(wgs + num_seqs) * num_q_heads * partial_stride(head_dim) * sizeof(float) + (size_t)(num_seqs + 1) * sizeof(int32_t);
}

// Workspace bytes instance `inst` needs for the call `p` (0: it writes the output directly).
size_t instance_workspace_bytes(const Instance &inst, const KParams &p_in)
{
    KParams p = p_in;
    apply_split(p, inst);
    if (inst.split_len < 0) return balanced_workspace_bytes(p.num_seqs, p.num_q_heads, p.head_dim, p.num_splits);
    if (p.num_splits <= 1) return 0;
    return (size_t)p.num_seqs * p.num_q_heads * p.num_splits * partial_stride(p.head_dim) * sizeof(float);
}

// The largest need of any instance that may be chosen for this call (cache winner, forced or built-in),
// so the answer does not depend on the state of the winner cache.
size_t decode_workspace_bytes(const KParams &p)
{
    int n;
    const Instance *t = instances(1, &n);
    size_t need = 0;
    for (int i = 0; i < n; ++i)
        if (usable(t[i], p, 1)) need = std::max(need, instance_workspace_bytes(t[i], p));
    return need;
}

// Debug aid, switched on by ATTN_DEBUG_VALIDATE=1 in the environment: the device-side integers that
// the hot call otherwise trusts are copied to the host (the stream is drained first, so the call
// is neither asynchronous nor capturable in this mode) and checked against the host-side bounds.
int debug_validate_device_side(const attn_args *a, int is_decode, hipStream_t stream)
{
    const int B = a->num_seqs;
    if (hipStreamSynchronize(stream) != hipSuccess) return ATTN_ERR_HIP;
    std::vector<int32_t> lens(B), qsl(B + 1, 0), kvsl;
    if (hipMemcpy(lens.data(), a->seq_lens, B * sizeof(int32_t), hipMemcpyDeviceToHost) != hipSuccess) return ATTN_ERR_HIP;
    if (!is_decode && hipMemcpy(qsl.data(), a->query_start_loc, (B + 1) * sizeof(int32_t), hipMemcpyDeviceToHost) != hipSuccess)
        return ATTN_ERR_HIP;
    if (is_decode)
        for (int s = 0; s <= B; ++s) qsl[s] = s;
    if (qsl[0] != 0 || qsl[B] != a->total_q) return ATTN_ERR_SHAPE;
    for (int s = 0; s < B; ++s) {
        const int nq = qsl[s + 1] - qsl[s];
        if (nq < 0 || nq > a->max_q_len || lens[s] < 0 || lens[s] > a->max_kv_len) return ATTN_ERR_SHAPE;
        if (a->causal && nq > lens[s]) return ATTN_ERR_SHAPE;  // a query positioned before key 0
    }
    if (a->block_table) {
        std::vector<int32_t> row(a->block_table_stride);
        for (int s = 0; s < B; ++s) {
            const int need = (lens[s] + a->block_size - 1) / a->block_size;
            if (need > a->block_table_stride) return ATTN_ERR_SHAPE;
            if (hipMemcpy(row.data(), a->block_table + (size_t)s * a->block_table_stride, (size_t)need * sizeof(int32_t),
                          hipMemcpyDeviceToHost) != hipSuccess)
                return ATTN_ERR_HIP;
            for (int b = 0; b < need; ++b)
                if (row[b] < 0 || row[b] >= a->num_blocks) return ATTN_ERR_SHAPE;
        }
    } else {
        const int32_t *src = a->kv_start_loc ? a->kv_start_loc : a->query_start_loc;
        kvsl.resize(B + 1);
        if (hipMemcpy(kvsl.data(), src, (B + 1) * sizeof(int32_t), hipMemcpyDeviceToHost) != hipSuccess) return ATTN_ERR_HIP;
        for (int s = 0; s < B; ++s)
            if (kvsl[s] < 0 || kvsl[s + 1] < kvsl[s] || kvsl[s] + lens[s] > kvsl[s + 1]) return ATTN_ERR_SHAPE;
    }
    return ATTN_OK;
}

int run(const attn_args *a, int is_decode, hipStream_t stream, int instance_override)
{
    int rc = validate(a, is_decode);
    if (rc != ATTN_OK) return rc;
    if (a->num_seqs == 0 || a->total_q == 0) return ATTN_OK;
    if (env_knobs().debug_validate) {
        rc = debug_validate_device_side(a, is_decode, stream);
        if (rc != ATTN_OK) {
            (void)hipGetLastError();
            return rc;
        }
    }
    KParams p = to_kparams(a, is_decode);
    if (a->dtype == ATTN_F32) {
        return launch_prefill_f32(p, stream) == hipSuccess ? ATTN_OK : ATTN_ERR_HIP;
    }
    int n;
    const Instance *t = instances(is_decode, &n);
    int id = instance_override >= 0 ? instance_override : select_instance(p, a->dtype, is_decode);
    if (id < 0) return id;
    if (id >= n || !usable(t[id], p, is_decode)) return ATTN_ERR_UNSUPPORTED;
    if (is_decode) {
        const size_t need = instance_workspace_bytes(t[id], p);
        apply_split(p, t[id]);
        if (need > 0) {
            if (!a->workspace || a->workspace_bytes < need) return ATTN_ERR_WORKSPACE;
            if ((uintptr_t)a->workspace & 7) return ATTN_ERR_WORKSPACE;  // records are accessed as 8-byte pairs
        }
    }
    if (t[id].launch(p, stream) != hipSuccess) return ATTN_ERR_HIP;
    // fixed-split decode merges its parts with a second kernel (the token-balanced launcher brings its own)
    if (is_decode && t[id].split_len >= 0 && p.num_splits > 1 &&
        (p.dtype == kDtypeF16 ? launch_decode_combine_f16(p, stream) : launch_decode_combine(p, stream)) != hipSuccess)
        return ATTN_ERR_HIP;
    return ATTN_OK;
}

// ---- tuner ----------------------------------------------------------------------------------------

// same values as fill_bf16_kernel, stored as fp16
__global__ void fill_f16_kernel(_Float16 *dst, size_t n, uint32_t seed)
{
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        uint32_t h = (uint32_t)i * 2654435761u ^ seed;
        h ^= h >> 15;
        h *= 2246822519u;
        h ^= h >> 13;
        dst[i] = (_Float16)(((int)(h & 0xffff) - 32768) * (1.f / 16384.f));
    }
}

__global__ void fill_bf16_kernel(uint16_t *dst, size_t n, uint32_t seed)
{
    // cheap counter hash -> bf16 in roughly [-2, 2); values only need to be finite and varied
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        uint32_t h = (uint32_t)i * 2654435761u ^ seed;
        h ^= h >> 15;
        h *= 2246822519u;
        h ^= h >> 13;
        const float f = ((int)(h & 0xffff) - 32768) * (1.f / 16384.f);
        dst[i] = (uint16_t)(__float_as_uint(f) >> 16);
    }
}

struct DeviceBuf {
    void *p = nullptr;
    hipError_t alloc(size_t bytes) { return hipMalloc(&p, bytes ? bytes : 16); }
    ~DeviceBuf()
    {
        if (p) (void)hipFree(p);
    }
};

int tune(const attn_args *shape, int is_decode, const char *cache_path, int iters, int flags)
{
    if (!shape) return ATTN_ERR_NULL;
    if (shape->struct_bytes != sizeof(attn_args)) return ATTN_ERR_SHAPE;
    if (!is16(shape->dtype)) return ATTN_ERR_DTYPE;  // the fp32 path has a single kernel
    if (shape->num_seqs <= 0 || shape->num_q_heads <= 0 || shape->num_kv_heads <= 0 ||
        shape->num_q_heads % shape->num_kv_heads || shape->max_kv_len <= 0)
        return ATTN_ERR_SHAPE;
    if (shape->head_dim != 64 && shape->head_dim != 128) return ATTN_ERR_UNSUPPORTED;
    if (iters <= 0) iters = 20;
    const int B = shape->num_seqs, Hq = shape->num_q_heads, Hkv = shape->num_kv_heads, D = shape->head_dim;
    const bool paged = is_decode || shape->block_size > 0;
    const int bs = paged ? (shape->block_size > 0 ? shape->block_size : 16) : 0;
    if (paged && (bs < 16 || (bs & (bs - 1)))) return ATTN_ERR_UNSUPPORTED;
    const int max_q = is_decode ? 1 : std::max(1, shape->max_q_len);
    const int max_kv = std::max(shape->max_kv_len, max_q);

    // lengths: the caller's own batch if it passes seq_lens (and query_start_loc for prefill), else
    // spread evenly between half of the maximum and the maximum
    std::vector<int32_t> qsl(B + 1, 0), kvsl(B + 1, 0), lens(B);
    bool have_lens = false;
    if (shape->seq_lens && (is_decode || shape->query_start_loc)) {
        std::vector<int32_t> hl(B), hq(B + 1, 0);
        have_lens = hipMemcpy(hl.data(), shape->seq_lens, B * sizeof(int32_t), hipMemcpyDeviceToHost) == hipSuccess;
        if (have_lens && !is_decode)
            have_lens = hipMemcpy(hq.data(), shape->query_start_loc, (B + 1) * sizeof(int32_t), hipMemcpyDeviceToHost) == hipSuccess;
        if (!have_lens) (void)hipGetLastError();
        for (int s = 0; s < B && have_lens; ++s) {
            const int nq = is_decode ? 1 : hq[s + 1] - hq[s];
            if (nq < 0 || nq > max_q || hl[s] < nq || hl[s] > max_kv) have_lens = false;  // disagrees with the bounds: ignore
            qsl[s + 1] = qsl[s] + nq;
            kvsl[s + 1] = kvsl[s] + hl[s];
            lens[s] = hl[s];
        }
    }
    for (int s = 0; s < B && !have_lens; ++s) {
        const double f = B > 1 ? 0.5 + 0.5 * (double)((s * 7) % B) / (B - 1) : 1.0;
        int nq = is_decode ? 1 : std::max(1, (int)(max_q * f));
        int nkv = std::max(nq, (int)(max_kv * f));
        if (s == 0) {
            nq = max_q;
            nkv = max_kv;
        }
        qsl[s + 1] = qsl[s] + nq;
        kvsl[s + 1] = kvsl[s] + nkv;
        lens[s] = nkv;
    }
    const int total_q = qsl[B];
    const int64_t total_kv = kvsl[B];
    int width = 0;
    int64_t nblocks = 0;
    std::vector<int32_t> table;
    if (paged) {
        width = (max_kv + bs - 1) / bs;
        for (int s = 0; s < B; ++s) nblocks += (lens[s] + bs - 1) / bs;
        table.assign((size_t)B * width, -1);
        // a random permutation of the pool (Fisher-Yates over a fixed-seed xorshift generator): the
        // block order of a cache that has served for a while.  A regular scatter (a fixed stride) gives
        // the memory channels a regular pattern, and a kernel family can look better on it than it is.
        std::vector<int32_t> perm((size_t)nblocks);
        for (int64_t i = 0; i < nblocks; ++i) perm[(size_t)i] = (int32_t)i;
        uint64_t rng = 0x9e3779b97f4a7c15ull;
        for (int64_t i = nblocks - 1; i > 0; --i) {
            rng ^= rng << 13;
            rng ^= rng >> 7;
            rng ^= rng << 17;
            std::swap(perm[(size_t)i], perm[(size_t)(rng % (uint64_t)(i + 1))]);
        }
        int64_t next = 0;
        for (int s = 0; s < B; ++s)
            for (int b = 0; b < (lens[s] + bs - 1) / bs; ++b) table[(size_t)s * width + b] = perm[(size_t)next++];
    }

    const size_t q_elems = (size_t)total_q * Hq * D;
    const size_t kv_elems = paged ? (size_t)nblocks * bs * Hkv * D : (size_t)total_kv * Hkv * D;
    DeviceBuf dq, dout, dk, dv, dtab, dqsl, dkvsl, dlens, dws;
    if (dq.alloc(q_elems * 2) != hipSuccess || dout.alloc(q_elems * 2) != hipSuccess || dk.alloc(kv_elems * 2) != hipSuccess ||
        dv.alloc(kv_elems * 2) != hipSuccess || dtab.alloc(table.size() * 4) != hipSuccess ||
        dqsl.alloc((B + 1) * 4) != hipSuccess || dkvsl.alloc((B + 1) * 4) != hipSuccess || dlens.alloc(B * 4) != hipSuccess ||
        false) {
        (void)hipGetLastError();
        return ATTN_ERR_HIP;
    }
    if (shape->dtype == ATTN_F16) {
        hipLaunchKernelGGL(fill_f16_kernel, dim3(1024), dim3(256), 0, 0, (_Float16 *)dq.p, q_elems, 1u);
        hipLaunchKernelGGL(fill_f16_kernel, dim3(4096), dim3(256), 0, 0, (_Float16 *)dk.p, kv_elems, 2u);
        hipLaunchKernelGGL(fill_f16_kernel, dim3(4096), dim3(256), 0, 0, (_Float16 *)dv.p, kv_elems, 3u);
    } else {
        hipLaunchKernelGGL(fill_bf16_kernel, dim3(1024), dim3(256), 0, 0, (uint16_t *)dq.p, q_elems, 1u);
        hipLaunchKernelGGL(fill_bf16_kernel, dim3(4096), dim3(256), 0, 0, (uint16_t *)dk.p, kv_elems, 2u);
        hipLaunchKernelGGL(fill_bf16_kernel, dim3(4096), dim3(256), 0, 0, (uint16_t *)dv.p, kv_elems, 3u);
    }
    bool ok = hipMemcpy(dqsl.p, qsl.data(), (B + 1) * 4, hipMemcpyHostToDevice) == hipSuccess &&
              hipMemcpy(dkvsl.p, kvsl.data(), (B + 1) * 4, hipMemcpyHostToDevice) == hipSuccess &&
              hipMemcpy(dlens.p, lens.data(), B * 4, hipMemcpyHostToDevice) == hipSuccess;
    if (paged && ok) ok = hipMemcpy(dtab.p, table.data(), table.size() * 4, hipMemcpyHostToDevice) == hipSuccess;
    if (!ok || hipDeviceSynchronize() != hipSuccess) return ATTN_ERR_HIP;

    attn_args a = *shape;
    a.total_q = total_q;
    a.max_q_len = max_q;
    a.max_kv_len = max_kv;
    a.q = dq.p;
    a.out = dout.p;
    a.k = dk.p;
    a.v = dv.p;
    a.q_stride_tok = a.o_stride_tok = (int64_t)Hq * D;
    a.q_stride_head = a.o_stride_head = D;
    a.kv_stride_head = D;
    a.kv_stride_tok = (int64_t)Hkv * D;
    a.kv_stride_block = paged ? (int64_t)bs * Hkv * D : 0;
    a.block_table = paged ? (const int32_t *)dtab.p : nullptr;
    a.block_table_stride = width;
    a.block_size = bs;
    a.num_blocks = (int32_t)nblocks;
    a.query_start_loc = (const int32_t *)dqsl.p;
    a.kv_start_loc = paged ? nullptr : (const int32_t *)dkvsl.p;
    a.seq_lens = (const int32_t *)dlens.p;
    if (a.scale == 0.f) a.scale = 1.f / std::sqrt((float)D);

    int rc = validate(&a, is_decode);
    if (rc != ATTN_OK) return rc;
    const size_t ws_bytes = is_decode ? decode_workspace_bytes(to_kparams(&a, is_decode)) : 0;
    if (dws.alloc(ws_bytes) != hipSuccess) {
        (void)hipGetLastError();
        return ATTN_ERR_HIP;
    }
    a.workspace = dws.p;
    a.workspace_bytes = ws_bytes;
    const KParams p = to_kparams(&a, is_decode);
    const std::string key = bucket_key(p, a.dtype, is_decode);

    int n;
    const Instance *t = instances(is_decode, &n);
    struct Events {  // destroyed on every way out of this function
        hipEvent_t e0 = nullptr, e1 = nullptr;
        ~Events()
        {
            if (e0) (void)hipEventDestroy(e0);
            if (e1) (void)hipEventDestroy(e1);
        }
    } ev;
    if (hipEventCreate(&ev.e0) != hipSuccess || hipEventCreate(&ev.e1) != hipSuccess) {
        (void)hipGetLastError();
        return ATTN_ERR_HIP;
    }
    const hipEvent_t e0 = ev.e0, e1 = ev.e1;
    // median of `count` timed launches after `warm` untimed ones; < 0 if the instance fails.  A launch
    // slower than `give_up_us` ends the measurement early (the instance cannot win any more).
    auto time_instance = [&](int id, int warm, int count, double give_up_us) -> double {
        for (int w = 0; w < warm; ++w)
            if (run(&a, is_decode, 0, id) != ATTN_OK) return -1.0;
        if (hipDeviceSynchronize() != hipSuccess) {
            (void)hipGetLastError();
            return -1.0;
        }
        std::vector<float> ms;
        for (int i = 0; i < count; ++i) {
            (void)hipEventRecord(e0, 0);
            if (run(&a, is_decode, 0, id) != ATTN_OK) return -1.0;
            (void)hipEventRecord(e1, 0);
            float t = 0.f;
            if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&t, e0, e1) != hipSuccess) {
                (void)hipGetLastError();
                return -1.0;
            }
            ms.push_back(t);
            if (1000.0 * t > give_up_us) break;
        }
        std::sort(ms.begin(), ms.end());
        return 1000.0 * ms[ms.size() / 2];
    };
    struct Cand {
        int id;
        double us;
        bool seed;
    };
    std::vector<Cand> cand;
    for (int id = 0; id < n; ++id)
        if (usable(t[id], p, is_decode)) cand.push_back(Cand{id, 0.0, false});
    if (cand.empty()) return ATTN_ERR_UNSUPPORTED;
    // seeds always survive the first cut: the built-in choice and the winners of the neighbouring buckets
    {
        std::vector<int> seeds;
        const int h = heuristic(p, is_decode);
        if (h >= 0) seeds.push_back(h);
        std::lock_guard<std::mutex> lk(g_mu);
        for (const std::string &nk : neighbour_keys(p, a.dtype, is_decode)) {
            auto it = g_winner[is_decode].find(nk);
            if (it != g_winner[is_decode].end()) seeds.push_back(it->second);
        }
        for (Cand &c : cand)
            for (int sd : seeds) c.seed |= c.id == sd;
    }
    const bool exhaustive = (flags & 2) != 0;
    // Successive halving: a cheap look at every valid instance, a closer one at the best third, the
    // full count only for the last three.  (Exhaustive sweeps are what the paper names as the cost
    // that keeps autotuning out of practice: its requirement list asks for an efficient search.)
    const int plan[2][2] = {{3, 0}, {std::max(5, iters / 2), 0}};
    const int rounds = exhaustive ? 1 : 2;
    int launches = 0;
    for (int r = 0; r < rounds; ++r) {
        const int count = exhaustive ? iters : plan[r][0];
        double best_so_far = 1e30;
        for (Cand &c : cand) {
            c.us = time_instance(c.id, r == 0 ? 2 : 1, count, exhaustive ? 1e30 : 3.0 * best_so_far);
            launches += count + (r == 0 ? 2 : 1);
            if (c.us >= 0 && c.us < best_so_far) best_so_far = c.us;
            if ((flags & 1) && c.us >= 0)
                fprintf(stderr, "[attn_tune] %s :: round %d %-48s %10.2f us\n", key.c_str(), r, t[c.id].name, c.us);
        }
        cand.erase(std::remove_if(cand.begin(), cand.end(), [](const Cand &c) { return c.us < 0; }), cand.end());
        if (cand.empty()) break;
        std::stable_sort(cand.begin(), cand.end(), [](const Cand &x, const Cand &y) { return x.us < y.us; });
        if (r + 1 < rounds) {
            const size_t keep = std::max<size_t>(4, (cand.size() + 2) / 3);
            std::vector<Cand> next;
            for (size_t i = 0; i < cand.size(); ++i)
                if (i < keep || (r == 0 && cand[i].seed)) next.push_back(cand[i]);
            cand.swap(next);
        }
    }
    // The finalists (and the built-in choice, whatever its rank) are measured once more, taking turns
    // launch by launch, so that a drift of the clocks during the measurement hits all of them alike;
    // the median of each decides.  Launch-to-launch noise is a few percent: the built-in choice keeps
    // its place unless a finalist beats it by more than 3 %.
    const int h = heuristic(p, is_decode);
    if (!exhaustive && !cand.empty()) {
        if (cand.size() > 3) cand.resize(3);
        bool has_h = false;
        for (const Cand &c : cand) has_h |= c.id == h;
        if (!has_h && h >= 0 && usable(t[h], p, is_decode)) cand.push_back(Cand{h, 0.0, true});
        std::vector<std::vector<double>> samples(cand.size());
        for (int i = 0; i < iters; ++i)
            for (size_t k = 0; k < cand.size(); ++k) {
                const double us = time_instance(cand[k].id, 0, 1, 1e30);
                ++launches;
                if (us >= 0) samples[k].push_back(us);
            }
        for (size_t k = 0; k < cand.size(); ++k) {
            std::sort(samples[k].begin(), samples[k].end());
            cand[k].us = samples[k].empty() ? -1.0 : samples[k][samples[k].size() / 2];
            if ((flags & 1) && cand[k].us >= 0)
                fprintf(stderr, "[attn_tune] %s :: final   %-48s %10.2f us\n", key.c_str(), t[cand[k].id].name, cand[k].us);
        }
        cand.erase(std::remove_if(cand.begin(), cand.end(), [](const Cand &c) { return c.us < 0; }), cand.end());
        std::stable_sort(cand.begin(), cand.end(), [](const Cand &x, const Cand &y) { return x.us < y.us; });
    }
    int best = cand.empty() ? -1 : cand[0].id;
    double best_us = cand.empty() ? 0.0 : cand[0].us;
    for (const Cand &c : cand)
        if (c.id == h && c.id != best && best_us > 0.97 * c.us) {
            best = c.id;
            best_us = c.us;
        }
    if (flags & 1) fprintf(stderr, "[attn_tune] %s :: %d launches in all\n", key.c_str(), launches);
    if (best < 0) return ATTN_ERR_UNSUPPORTED;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        g_winner[is_decode][key] = best;
        g_generation.fetch_add(1, std::memory_order_release);
    }
    if (flags & 1) fprintf(stderr, "[attn_tune] winner %s -> %s (%.2f us)\n", key.c_str(), t[best].name, best_us);
    if (!cache_path) return ATTN_OK;

    return merge_cache_line(cache_path, key, t[best].name, best_us);
}

}  // namespace

std::string environment_key() { return env_key_impl(); }

int merge_cache_line(const char *path, const std::string &key, const std::string &instance_name, double us)
{
    // Read, change and replace under an exclusive lock on a side file, so that two processes tuning into
    // one cache file do not lose each other's lines (the data file itself is replaced by rename and
    // cannot carry the lock).
    struct Lock {
        int fd = -1;
        explicit Lock(const std::string &p)
        {
            fd = open(p.c_str(), O_CREAT | O_RDWR | O_CLOEXEC, 0644);
            if (fd >= 0 && flock(fd, LOCK_EX) != 0) {
                close(fd);
                fd = -1;
            }
        }
        ~Lock()
        {
            if (fd >= 0) {
                (void)flock(fd, LOCK_UN);
                close(fd);
            }
        }
    } lock(std::string(path) + ".lock");
    if (lock.fd < 0) return ATTN_ERR_CACHE_IO;

    // keep every other line, replace this (environment, bucket) pair; damaged lines are dropped, a
    // missing file or one without the magic line starts afresh
    std::vector<CacheLine> lines;
    int damaged = 0;
    (void)read_cache_file(path, &lines, &damaged);
    const std::string env = env_key_impl();
    std::ostringstream text;
    text << kCacheMagic << "\n";
    for (const CacheLine &cl : lines)
        if (!(cl.env == env && cl.key == key)) text << cl.env << "\t" << cl.key << "\t" << cl.inst << "\t" << cl.us << "\n";
    text << env << "\t" << key << "\t" << instance_name << "\t" << us << "\n";
    const std::string body = text.str();

    const std::string tmp = std::string(path) + ".tmp." + std::to_string((long)getpid());
    const int fd = open(tmp.c_str(), O_CREAT | O_TRUNC | O_WRONLY | O_CLOEXEC, 0644);
    if (fd < 0) return ATTN_ERR_CACHE_IO;
    bool ok = true;
    for (size_t done = 0; ok && done < body.size();) {
        const ssize_t w = write(fd, body.data() + done, body.size() - done);
        if (w <= 0)
            ok = false;
        else
            done += (size_t)w;
    }
    ok = ok && fsync(fd) == 0;  // the new contents are on disk before the name points at them
    ok = (close(fd) == 0) && ok;
    if (!ok || rename(tmp.c_str(), path) != 0) {
        (void)remove(tmp.c_str());
        return ATTN_ERR_CACHE_IO;
    }
    return ATTN_OK;
}

void store_named_winner(const std::string &key, const std::string &instance_name)
{
    std::lock_guard<std::mutex> lk(g_mu);
    g_named[key] = instance_name;
}

bool lookup_named_winner(const std::string &key, std::string *instance_name)
{
    std::lock_guard<std::mutex> lk(g_mu);
    auto it = g_named.find(key);
    if (it == g_named.end()) return false;
    *instance_name = it->second;
    return true;
}

void load_env_cache_once() { maybe_load_env_cache(); }

namespace {
const Instance *all_decode_instances(int *count)
{
    static const std::vector<Instance> all = [] {
        std::vector<Instance> v;
        int n;
        const Instance *t = decode_instances(&n);
        v.insert(v.end(), t, t + n);
        t = decode_f16_instances(&n);
        v.insert(v.end(), t, t + n);
        return v;
    }();
    *count = (int)all.size();
    return all.data();
}
}  // namespace

const Instance *prefill_instances(int *count)
{
    static const std::vector<Instance> all = [] {
        std::vector<Instance> v;
        int n;
        const Instance *t = prefill_ring_instances(&n);
        v.insert(v.end(), t, t + n);
        t = prefill_staged_instances(&n);
        v.insert(v.end(), t, t + n);
        t = prefill_ring_f16_instances(&n);
        v.insert(v.end(), t, t + n);
        t = prefill_staged_f16_instances(&n);
        v.insert(v.end(), t, t + n);
        return v;
    }();
    *count = (int)all.size();
    return all.data();
}

}  // namespace attn

using namespace attn;

// ---- the entry point that allocates nothing ------------------------------------------------------
// Split-K records of attn_decode_paged_static live in this array instead of a caller workspace.  Every
// GPU the library runs on holds its own copy, at its own address, until the process ends.  In host
// code the name `scratch` is only a handle for hipGetSymbolAddress, never a device address.
constexpr size_t kScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device, resolved once per device (with that device
// current); nullptr if the runtime refuses.
void *scratch_on_current_device()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return nullptr;
    }
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

extern "C" {

int attn_decode_paged_static(const attn_args *args, void *hip_stream)
{
    int rc = validate(args, 1);
    if (rc != ATTN_OK) return rc;
    if (args->num_seqs == 0 || args->total_q == 0) return ATTN_OK;
    // the need of the instance this call will take, against the fixed size of the array
    const KParams p = to_kparams(args, 1);
    int n;
    const Instance *t = instances(1, &n);
    const int id = select_instance(p, args->dtype, 1);
    if (id < 0) return id;
    if (id >= n || !usable(t[id], p, 1)) return ATTN_ERR_UNSUPPORTED;
    if (instance_workspace_bytes(t[id], p) > kScratchBytes) return ATTN_ERR_WORKSPACE;
    void *ptr = scratch_on_current_device();
    if (!ptr) return ATTN_ERR_HIP;
    attn_args a = *args;
    a.workspace = ptr;
    a.workspace_bytes = kScratchBytes;
    return run(&a, 1, (hipStream_t)hip_stream, id);
}

size_t attn_static_scratch_bytes(void) { return kScratchBytes; }

int attn_prefill_varlen(const attn_args *args, void *hip_stream) { return run(args, 0, (hipStream_t)hip_stream, -1); }

int attn_decode_paged(const attn_args *args, void *hip_stream) { return run(args, 1, (hipStream_t)hip_stream, -1); }

size_t attn_workspace_bytes(const attn_args *a, int is_decode)
{
    if (!a || a->struct_bytes != sizeof(attn_args) || !is_decode) return 0;
    if (a->num_seqs <= 0 || a->num_q_heads <= 0 || a->num_kv_heads <= 0 || a->num_q_heads % a->num_kv_heads || a->max_kv_len < 0 ||
        (a->head_dim != 64 && a->head_dim != 128) || !is16(a->dtype))
        return 0;
    KParams p = to_kparams(a, 1);
    // pointer fields are ignored: decode is always paged, whatever block_table holds at this point
    static const int32_t dummy_table = 0;
    p.block_table = &dummy_table;
    if (p.block_size <= 0) {
        p.block_size = a->block_size > 0 ? a->block_size : 16;
        p.block_shift = ilog2_ceil(p.block_size);
    }
    return decode_workspace_bytes(p);
}

int attn_tune(const attn_args *shape_like, int is_decode, const char *cache_path, int iters, int flags)
{
    return tune(shape_like, is_decode ? 1 : 0, cache_path, iters, flags);
}

int attn_environment_key(char *buf, size_t buf_bytes)
{
    const std::string k = env_key_impl();
    if (buf && buf_bytes) snprintf(buf, buf_bytes, "%s", k.c_str());
    return (int)k.size();
}

int attn_load_cache(const char *cache_path)
{
    if (!cache_path) return ATTN_ERR_NULL;
    std::lock_guard<std::mutex> lk(g_mu);
    return load_cache_locked(cache_path);
}

void attn_clear_cache(void)
{
    std::lock_guard<std::mutex> lk(g_mu);
    g_winner[0].clear();
    g_winner[1].clear();
    g_named.clear();
    g_generation.fetch_add(1, std::memory_order_release);
}

int attn_num_instances(int is_decode)
{
    int n;
    (void)instances(is_decode ? 1 : 0, &n);
    return n;
}

int attn_instance_name(int is_decode, int id, char *buf, size_t buf_bytes)
{
    int n;
    const Instance *t = instances(is_decode ? 1 : 0, &n);
    if (id < 0 || id >= n) return ATTN_ERR_SHAPE;
    if (!buf || buf_bytes == 0) return ATTN_ERR_NULL;
    snprintf(buf, buf_bytes, "%s", t[id].name);
    return (int)strlen(buf);
}

int attn_selected_instance(const attn_args *a, int is_decode)
{
    is_decode = is_decode ? 1 : 0;
    if (!a || a->struct_bytes != sizeof(attn_args)) return ATTN_ERR_NULL;
    if (!is16(a->dtype)) return ATTN_ERR_DTYPE;
    if (a->num_q_heads <= 0 || a->num_kv_heads <= 0 || a->num_q_heads % a->num_kv_heads) return ATTN_ERR_SHAPE;
    const KParams p = to_kparams(a, is_decode);
    return select_instance(p, a->dtype, is_decode);
}

void attn_force_instance(int is_decode, int id) { g_forced[is_decode ? 1 : 0].store(id); }

const char *attn_status_string(int status)
{
    switch (status) {
        case ATTN_OK: return "ok";
        case ATTN_ERR_NULL: return "a required pointer is NULL";
        case ATTN_ERR_SHAPE: return "inconsistent sizes, strides or head counts";
        case ATTN_ERR_DTYPE: return "dtype not supported by this entry point";
        case ATTN_ERR_UNSUPPORTED: return "no kernel instance for this head_dim / block_size / group size";
        case ATTN_ERR_WORKSPACE: return "workspace missing or too small";
        case ATTN_ERR_HIP: return "HIP runtime error";
        case ATTN_ERR_CACHE_IO: return "tuning cache file could not be read or written";
        default: return "unknown status";
    }
}

}  // extern "C"

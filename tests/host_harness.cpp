// Host-side driver of the attention library for the CPU tests: it is linked against a build of the
// dispatcher (csrc/attn_api.hip) whose host code carries AddressSanitizer and
// UndefinedBehaviorSanitizer, and exercises everything that needs no GPU: validation, workspace
// arithmetic, shape buckets and the built-in choice over a sweep of shapes, the per-thread selection
// memo from several threads, the cache parser on good, stale and damaged files, and the
// read-modify-replace of the cache file.  No kernel is launched.
//
//   host_harness selftest <dir>             everything above; prints "selftest ok"
//   host_harness merge <file> <prefix> <n>  n merges of keys <prefix>0..<prefix>n-1 into <file>
//                                           (run from several processes at once by the test)
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <fstream>
#include <string>
#include <thread>
#include <vector>

#include "../include/attn.h"
#include "../paper_2505_03780_amd/csrc/tuner_cache.hpp"

#define CHECK(cond)                                                            \
    do {                                                                       \
        if (!(cond)) {                                                         \
            fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
            exit(1);                                                           \
        }                                                                      \
    } while (0)

static attn_args base_args()
{
    attn_args a;
    memset(&a, 0, sizeof a);
    a.struct_bytes = sizeof a;
    a.dtype = ATTN_BF16;
    a.num_seqs = 4;
    a.num_q_heads = 32;
    a.num_kv_heads = 8;
    a.head_dim = 128;
    a.total_q = 400;
    a.max_q_len = 100;
    a.max_kv_len = 100;
    a.q = a.out = (void *)0x1000;
    a.k = a.v = (void *)0x1000;
    a.q_stride_tok = a.o_stride_tok = 32 * 128;
    a.q_stride_head = a.o_stride_head = 128;
    a.kv_stride_tok = 8 * 128;
    a.kv_stride_head = 128;
    a.kv_stride_block = 16 * 8 * 128;
    a.query_start_loc = a.seq_lens = (const int32_t *)0x2000;
    a.scale = 0.088f;
    a.causal = 1;
    return a;
}

static attn_args paged_args(int B, int max_kv)
{
    attn_args a = base_args();
    a.num_seqs = a.total_q = B;
    a.max_q_len = 1;
    a.max_kv_len = max_kv;
    a.block_table = (const int32_t *)0x3000;
    a.block_size = 16;
    a.block_table_stride = (max_kv + 15) / 16 + 1;
    a.num_blocks = 1 << 20;
    return a;
}

static std::string name_of(int is_decode, int id)
{
    char buf[160];
    CHECK(attn_instance_name(is_decode, id, buf, sizeof buf) > 0);
    return buf;
}

static void write_file(const std::string &path, const std::string &text)
{
    std::ofstream f(path, std::ios::binary | std::ios::trunc);
    f << text;
}

static int count_lines_with(const std::string &path, const std::string &needle)
{
    std::ifstream f(path);
    std::string l;
    int n = 0;
    while (std::getline(f, l))
        if (l.find(needle) != std::string::npos) ++n;
    return n;
}

static void selftest(const std::string &dir)
{
    // ---- validation: every error is found on the host, nothing is enqueued ----
    CHECK(attn_prefill_varlen(nullptr, nullptr) == ATTN_ERR_NULL);
    {
        attn_args a = base_args();
        a.struct_bytes = 8;
        CHECK(attn_prefill_varlen(&a, nullptr) == ATTN_ERR_SHAPE);
        a = base_args();
        a.num_kv_heads = 5;
        CHECK(attn_prefill_varlen(&a, nullptr) == ATTN_ERR_SHAPE);
        a = base_args();
        a.head_dim = 96;
        CHECK(attn_prefill_varlen(&a, nullptr) == ATTN_ERR_UNSUPPORTED);
        a = base_args();
        a.q = nullptr;
        CHECK(attn_prefill_varlen(&a, nullptr) == ATTN_ERR_NULL);
        a = base_args();
        a.dtype = 9;
        CHECK(attn_prefill_varlen(&a, nullptr) == ATTN_ERR_DTYPE);
        a = base_args();
        a.num_seqs = 0;
        a.total_q = 0;
        a.q = a.out = nullptr;
        CHECK(attn_prefill_varlen(&a, nullptr) == ATTN_OK);
        a = paged_args(4, 4096);
        a.workspace = nullptr;  // every decode instance that splits needs a workspace
        const int rc = attn_decode_paged(&a, nullptr);
        CHECK(rc == ATTN_ERR_WORKSPACE || rc == ATTN_ERR_HIP);  // (no device: a launch without split would fail in HIP)
        a.workspace = (void *)0x100004;  // misaligned for the 8-byte record accesses
        a.workspace_bytes = 1u << 30;
        CHECK(attn_decode_paged(&a, nullptr) == ATTN_ERR_WORKSPACE);
    }

    // ---- instance tables, buckets and the built-in choice over a sweep of shapes ----
    const int np = attn_num_instances(0), nd = attn_num_instances(1);
    CHECK(np > 0 && nd > 0);
    for (int i = 0; i < np; ++i) (void)name_of(0, i);
    for (int i = 0; i < nd; ++i) (void)name_of(1, i);
    char tiny[4];
    CHECK(attn_instance_name(0, 0, tiny, sizeof tiny) == 3);  // truncated, still terminated
    CHECK(attn_instance_name(0, np, tiny, sizeof tiny) < 0);
    attn_clear_cache();
    const int dtypes[2] = {ATTN_BF16, ATTN_F16};
    for (int dt = 0; dt < 2; ++dt)
        for (int hd = 64; hd <= 128; hd += 64)
            for (int hkv = 1; hkv <= 8; hkv *= 2)
                for (int g = 1; g <= 8; g *= 2)
                    for (int B = 1; B <= 4096; B *= 8)
                        for (int kv = 1; kv <= (1 << 20); kv *= 16) {
                            attn_args a = base_args();
                            a.dtype = dtypes[dt];
                            a.head_dim = hd;
                            a.num_kv_heads = hkv;
                            a.num_q_heads = hkv * g;
                            a.num_seqs = B;
                            a.max_kv_len = kv;
                            a.max_q_len = kv < 512 ? kv : 512;
                            const int id = attn_selected_instance(&a, 0);
                            CHECK(id >= 0 && id < np);
                            attn_args d = paged_args(B, kv);
                            d.dtype = dtypes[dt];
                            d.head_dim = hd;
                            d.num_kv_heads = hkv;
                            d.num_q_heads = hkv * g;
                            const int idd = attn_selected_instance(&d, 1);
                            CHECK(idd >= 0 && idd < nd);
                            // the workspace the caller is told to provide is bounded and covers the choice
                            const size_t ws = attn_workspace_bytes(&d, 1);
                            // (at most four records per compute unit, 256 without a device, and one per sequence)
                            CHECK(ws <= (size_t)(1024 + B) * d.num_q_heads * (hd + 2) * 4 + (size_t)(B + 1) * 4);
                            for (int f = 0; f < nd; ++f) {  // forcing any instance: valid or refused, never out of bounds
                                attn_force_instance(1, f);
                                const int got = attn_selected_instance(&d, 1);
                                CHECK(got == f || got == ATTN_ERR_UNSUPPORTED);
                            }
                            attn_force_instance(1, -1);
                        }

    // ---- cache files: good, stale, damaged in the middle, hostile ----
    char envbuf[256];
    CHECK(attn_environment_key(envbuf, sizeof envbuf) > 0);
    const std::string env = envbuf;
    attn_args a = base_args();
    const int dflt = attn_selected_instance(&a, 0);
    int other = -1;
    for (int i = 0; i < np; ++i)
        if (i != dflt && name_of(0, i).find("bf16_ring") != std::string::npos && name_of(0, i).find("hpw1") != std::string::npos) other = i;
    CHECK(other >= 0);
    const std::string key = "prefill|bf16|d128|hq32|hkv8|contig|bs0|c1|B2|q7|kv7";
    const std::string good = dir + "/good.txt";
    write_file(good, "attn-tune-cache-v1\n" + env + "\t" + key + "\t" + name_of(0, other) + "\t12.5\n");
    CHECK(attn_load_cache(good.c_str()) == ATTN_OK);
    CHECK(attn_selected_instance(&a, 0) == other);
    attn_clear_cache();
    CHECK(attn_selected_instance(&a, 0) == dflt);
    const std::string mixed = dir + "/mixed.txt";
    write_file(mixed, "attn-tune-cache-v1\ngfx000|cu1|hip0|drv0|k0\tsome|key\tsome kernel\t1.5\n\x01\x02 no tabs here\n\t\t\t\n" + env + "\t" + key +
                          "\t" + name_of(0, other) + "\tnot-a-number\n" + env + "\t" + key + "\t" + name_of(0, other) + "\t3\n" +
                          std::string(5000, 'x') + "\n");
    CHECK(attn_load_cache(mixed.c_str()) == ATTN_OK);
    CHECK(attn_selected_instance(&a, 0) == other);
    attn_clear_cache();
    write_file(dir + "/bad.txt", "garbage\n");
    CHECK(attn_load_cache((dir + "/bad.txt").c_str()) == ATTN_ERR_CACHE_IO);
    write_file(dir + "/empty.txt", "");
    CHECK(attn_load_cache((dir + "/empty.txt").c_str()) == ATTN_ERR_CACHE_IO);
    write_file(dir + "/onlybad.txt", "attn-tune-cache-v1\nonly\ttwo\n");
    CHECK(attn_load_cache((dir + "/onlybad.txt").c_str()) == ATTN_ERR_CACHE_IO);
    CHECK(attn_load_cache((dir + "/missing.txt").c_str()) == ATTN_ERR_CACHE_IO);
    CHECK(attn_load_cache(nullptr) == ATTN_ERR_NULL);
    CHECK(attn_selected_instance(&a, 0) == dflt);

    // ---- merging into a file with a damaged middle line keeps the other lines ----
    CHECK(attn::merge_cache_line(mixed.c_str(), "prefill|new|bucket", name_of(0, dflt), 9.0) == ATTN_OK);
    CHECK(count_lines_with(mixed, "gfx000|cu1|hip0|drv0|k0\tsome|key") == 1);  // another environment's winner survives
    CHECK(count_lines_with(mixed, key) == 1);
    CHECK(count_lines_with(mixed, "prefill|new|bucket") == 1);
    CHECK(count_lines_with(mixed, "no tabs here") == 0);
    CHECK(attn::merge_cache_line(mixed.c_str(), "prefill|new|bucket", name_of(0, other), 8.0) == ATTN_OK);  // replaced, not added
    CHECK(count_lines_with(mixed, "prefill|new|bucket") == 1);
    CHECK(attn_load_cache(mixed.c_str()) == ATTN_OK);
    CHECK(attn::merge_cache_line((dir + "/no/such/dir/cache.txt").c_str(), "k", "i", 1.0) == ATTN_ERR_CACHE_IO);
    attn_clear_cache();

    // ---- the per-thread selection memo under concurrent table changes ----
    {
        std::vector<std::thread> th;
        for (int t = 0; t < 4; ++t)
            th.emplace_back([&, t] {
                attn_args x = base_args();
                for (int i = 0; i < 2000; ++i) {
                    x.max_kv_len = 100 + (i % 7) * 1000;
                    x.max_q_len = x.max_kv_len;
                    const int id = attn_selected_instance(&x, 0);
                    if (id < 0 || id >= np) abort();
                    if (t == 0 && i % 50 == 0) (void)attn_load_cache(good.c_str());
                    if (t == 1 && i % 70 == 0) attn_clear_cache();
                }
            });
        for (auto &t : th) t.join();
    }
    attn_clear_cache();
    for (int s = -9; s <= 1; ++s) CHECK(attn_status_string(s) != nullptr);
    printf("selftest ok\n");
}

int main(int argc, char **argv)
{
    if (argc == 3 && !strcmp(argv[1], "selftest")) {
        selftest(argv[2]);
        return 0;
    }
    if (argc == 5 && !strcmp(argv[1], "merge")) {
        const int n = atoi(argv[4]);
        for (int i = 0; i < n; ++i)
            if (attn::merge_cache_line(argv[2], std::string(argv[3]) + std::to_string(i), "some instance", 1.0 + i) != ATTN_OK) return 2;
        return 0;
    }
    fprintf(stderr, "usage: host_harness selftest <dir> | merge <file> <prefix> <n>\n");
    return 64;
}

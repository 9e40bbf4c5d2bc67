"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer: a small C driver includes the
oracle's source, runs ragged contiguous and paged problems on buffers of exactly the needed size
(unused block-table entries hold -1 and INT_MAX, so any read of them would leave the pool), and its
output must equal what the normal build returns through Python for the same inputs."""
import os
import subprocess

import numpy as np

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

DRIVER = r'''
#include "%(src)s"
#include <stdio.h>
#include <limits.h>

static uint32_t state = 12345u;
static uint16_t next_bf16(void)
{   /* pseudo-random value in [-2, 2) on a grid of 2^-5, exactly representable in bf16 */
    state = state * 1664525u + 1013904223u;
    float f = (float)((int)((state >> 16) & 127) - 64) / 32.0f;
    uint32_t bits;
    memcpy(&bits, &f, 4);
    return (uint16_t)(bits >> 16);
}

int main(void)
{
    enum { B = 3, HQ = 4, HKV = 2, D = 16, BS = 4 };
    const int n_q[B] = {5, 1, 3}, n_kv[B] = {5, 9, 6};
    int32_t qsl[B + 1] = {0}, kvsl[B + 1] = {0}, seq_lens[B];
    for (int s = 0; s < B; ++s) { qsl[s + 1] = qsl[s] + n_q[s]; kvsl[s + 1] = kvsl[s] + n_kv[s]; seq_lens[s] = n_kv[s]; }
    const int total_q = qsl[B], total_kv = kvsl[B];
    uint16_t *q = malloc(sizeof(uint16_t) * total_q * HQ * D);
    uint16_t *k = malloc(sizeof(uint16_t) * total_kv * HKV * D);
    uint16_t *v = malloc(sizeof(uint16_t) * total_kv * HKV * D);
    for (int i = 0; i < total_q * HQ * D; ++i) q[i] = next_bf16();
    for (int i = 0; i < total_kv * HKV * D; ++i) k[i] = next_bf16();
    for (int i = 0; i < total_kv * HKV * D; ++i) v[i] = next_bf16();
    double *out = malloc(sizeof(double) * total_q * HQ * D);

    oracle_problem p;
    memset(&p, 0, sizeof p);
    p.dtype = ORACLE_BF16; p.num_seqs = B; p.num_q_heads = HQ; p.num_kv_heads = HKV; p.head_dim = D;
    p.q = q; p.q_stride_tok = HQ * D; p.q_stride_head = D;
    p.k = k; p.v = v; p.kv_stride_tok = HKV * D; p.kv_stride_head = D;
    p.query_start_loc = qsl; p.kv_start_loc = kvsl; p.seq_lens = seq_lens; p.scale = 0.25f; p.causal = 1;
    if (oracle_attention(&p, out) != 0) return 2;
    for (int i = 0; i < total_q * HQ * D; ++i) printf("%%.17g\n", out[i]);

    /* the same tokens scattered into a pool: blocks handed out in reverse order, exactly as many as needed */
    int nblk = 0, width = 0;
    for (int s = 0; s < B; ++s) { int nb = (n_kv[s] + BS - 1) / BS; nblk += nb; if (nb > width) width = nb; }
    uint16_t *kp = malloc(sizeof(uint16_t) * nblk * BS * HKV * D), *vp = malloc(sizeof(uint16_t) * nblk * BS * HKV * D);
    for (int i = 0; i < nblk * BS * HKV * D; ++i) { kp[i] = 0x7fc0; vp[i] = 0x7fc0; } /* NaN in every slot no key owns */
    int32_t *table = malloc(sizeof(int32_t) * B * width);
    int next = nblk - 1;
    for (int s = 0; s < B; ++s)
        for (int b = 0; b < width; ++b) {
            const int nb = (n_kv[s] + BS - 1) / BS;
            table[s * width + b] = b < nb ? next-- : (b %% 2 ? -1 : INT_MAX);
        }
    for (int s = 0; s < B; ++s)
        for (int j = 0; j < n_kv[s]; ++j) {
            const int blk = table[s * width + j / BS];
            memcpy(kp + ((int64_t)blk * BS + j %% BS) * HKV * D, k + (int64_t)(kvsl[s] + j) * HKV * D, sizeof(uint16_t) * HKV * D);
            memcpy(vp + ((int64_t)blk * BS + j %% BS) * HKV * D, v + (int64_t)(kvsl[s] + j) * HKV * D, sizeof(uint16_t) * HKV * D);
        }
    p.k = kp; p.v = vp; p.kv_stride_block = BS * HKV * D; p.block_table = table; p.block_table_stride = width; p.block_size = BS;
    p.kv_start_loc = NULL;
    double *out2 = malloc(sizeof(double) * total_q * HQ * D);
    if (oracle_attention(&p, out2) != 0) return 3;
    for (int i = 0; i < total_q * HQ * D; ++i)
        if (out2[i] != out[i]) { fprintf(stderr, "paged differs at %%d\n", i); return 4; }
    /* sampled rows: the last token of every sequence, head 3 */
    int32_t ss[B] = {0, 1, 2}, st[B] = {4, 0, 2}, sh[B] = {3, 3, 3};
    double rows[B * D];
    if (oracle_attention_rows(&p, B, ss, st, sh, rows) != 0) return 5;
    for (int r = 0; r < B; ++r)
        for (int d = 0; d < D; ++d)
            if (rows[r * D + d] != out[((int64_t)(qsl[ss[r]] + st[r]) * HQ + sh[r]) * D + d]) return 6;
    free(q); free(k); free(v); free(out); free(kp); free(vp); free(table); free(out2);
    return 0;
}
'''


def _lcg_bf16(n, state):
    out = np.empty(n, np.float32)
    for i in range(n):
        state = (state * 1664525 + 1013904223) & 0xFFFFFFFF
        out[i] = (((state >> 16) & 127) - 64) / 32.0
    return out, state


def test_oracle_is_clean_under_asan_and_ubsan_and_matches_the_normal_build(tmp_path):
    src = os.path.join(tmp_path, "driver.c")
    exe = os.path.join(tmp_path, "driver")
    with open(src, "w") as f:
        f.write(DRIVER % {"src": os.path.join(ROOT, "oracle", "attn_oracle.c")})
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-static-libasan", "-o", exe, src, "-lm"])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, r.stderr[-2000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-2000:]
    got = np.array([float(x) for x in r.stdout.split()])

    B, HQ, HKV, D = 3, 4, 2, 16
    n_q, n_kv = [5, 1, 3], [5, 9, 6]
    st = 12345
    q, st = _lcg_bf16(sum(n_q) * HQ * D, st)
    k, st = _lcg_bf16(sum(n_kv) * HKV * D, st)
    v, st = _lcg_bf16(sum(n_kv) * HKV * D, st)
    qsl = np.concatenate([[0], np.cumsum(n_q)]).astype(np.int32)
    kvsl = np.concatenate([[0], np.cumsum(n_kv)]).astype(np.int32)
    # the values are exact in bf16, so the float32 reader sees the same numbers as the driver's bf16 arrays
    prob = oracle.OracleProblem(q.reshape(-1, HQ, D), k.reshape(-1, HKV, D), v.reshape(-1, HKV, D), qsl, np.asarray(n_kv, np.int32),
                                0.25, True, kv_start_loc=kvsl)
    ref = oracle.attention(prob).reshape(-1)
    assert got.shape == ref.shape
    assert np.array_equal(got, ref), float(np.max(np.abs(got - ref)))

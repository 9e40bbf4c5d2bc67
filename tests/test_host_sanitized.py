"""The host side of the library (validation, buckets, built-in choice, selection memo, cache parser and
cache-file merging in csrc/attn_api.hip) under AddressSanitizer and UndefinedBehaviorSanitizer, on the
CPU: tests/host_harness.cpp is linked against a build of the dispatcher whose host code is
instrumented (the kernels' translation units come from the normal library) and drives every entry
point that needs no GPU.  The same program, started several times at once, shows that concurrent
tuner processes merging into one cache file do not lose each other's lines."""
import os
import subprocess

import pytest

import paper_2505_03780_amd as A

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2505_03780_amd")
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all"]


@pytest.fixture(scope="module")
def harness(tmp_path_factory):
    A.load_library()  # the kernels' side of the link; raises if the library has not been built
    d = tmp_path_factory.mktemp("host_sanitized")
    obj, exe = str(d / "attn_api_san.o"), str(d / "host_harness")
    flags = ["--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
    subprocess.check_call(["hipcc", *flags, *SAN, "-c", os.path.join(PKG, "csrc", "attn_api.hip"), "-o", obj], stderr=subprocess.DEVNULL)
    hobj = str(d / "host_harness.o")
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", *SAN, "-c", os.path.join(ROOT, "tests", "host_harness.cpp"),
                           "-o", hobj], stderr=subprocess.DEVNULL)
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", *SAN, hobj, obj, "-L" + PKG, "-lattn_gfx950", "-Wl,-rpath," + PKG, "-lpthread",
                           "-o", exe], stderr=subprocess.DEVNULL)
    return exe


def _env():
    # the HIP runtime keeps allocations of its own until exit: leaks are not what this test looks for
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")
    for k in ("LD_PRELOAD", "ATTN_TUNE_CACHE", "ATTN_FORCE_INSTANCE", "ATTN_LOG", "ATTN_DEBUG_VALIDATE"):
        env.pop(k, None)
    return env


def test_host_dispatcher_tuner_cache_and_parser_are_clean_under_asan_and_ubsan(harness, tmp_path):
    r = subprocess.run([harness, "selftest", str(tmp_path)], capture_output=True, text=True, env=_env(), timeout=600)
    assert r.returncode == 0, (r.stdout[-1000:], r.stderr[-3000:])
    assert "selftest ok" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-3000:]


def test_concurrent_merges_into_one_cache_file_all_survive(harness, tmp_path):
    """Four processes merge 25 buckets each into one file at the same time; a pre-existing line of
    another environment and a damaged line sit in the file from the start."""
    path = tmp_path / "cache.txt"
    path.write_text("attn-tune-cache-v1\nother-env|cu1\tdecode|x\tsome kernel\t2.5\n\x00damaged line\n")
    procs = [subprocess.Popen([harness, "merge", str(path), "prefill|proc%d|b" % i, "25"], env=_env(), stderr=subprocess.PIPE, text=True)
             for i in range(4)]
    for p in procs:
        _, err = p.communicate(timeout=300)
        assert p.returncode == 0, err[-2000:]
        assert "runtime error" not in err and "AddressSanitizer" not in err, err[-2000:]
    lines = path.read_text().splitlines()
    assert lines[0] == "attn-tune-cache-v1"
    body = [l.split("\t") for l in lines[1:]]
    assert all(len(f) == 4 for f in body), "a damaged line survived or a line was torn"
    keys = [f[1] for f in body]
    assert len(keys) == len(set(keys)) == 101
    assert "decode|x" in keys
    for i in range(4):
        for j in range(25):
            assert "prefill|proc%d|b%d" % (i, j) in keys
    assert not [f for f in os.listdir(tmp_path) if ".tmp." in f], "a temporary file was left behind"

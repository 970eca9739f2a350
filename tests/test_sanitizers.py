"""The CPU oracle, the input generator and the HIP library's host code under AddressSanitizer and UndefinedBehaviorSanitizer.

The first two are plain C; a stray index in either would silently bend every parity claim built on them.  They are compiled
here with -fsanitize=address,undefined into a scratch directory and driven, in a child process that preloads the
sanitizer runtime, through the same Python bindings the tests use: the tiny workload's prompt pass, masked and
multi-row passes, plain, speculative, adaptive and sampled generation, Algorithm 1, and the generator's entry points.
Any report from either sanitizer fails the test.  The library's host code (second test) is compiled by hipcc with the
sanitizers on the host side only and driven through the entry points that need no device."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

DRIVER = r"""
import sys
sys.path.insert(0, {root!r})
import numpy as np
import asd_inputs as si
import oracle
si._LIB_PATH = {synth!r}
oracle._LIB = {orc!r}
si.build = lambda force=False: si._LIB_PATH
oracle.build = lambda force=False: oracle._LIB
s = si.SHAPES["tiny"]
for shape in (s, s.with_(dtype=si.DT_BF16, n_kv_heads=2, d_ffn=208)):
    W = list(si.all_tensors(shape, 3, gain_std=0.1))
    orc = oracle.Oracle(shape, 96, kv_storage=True).load(W)
    p = si.prompt(1, 40, shape.vocab)
    r = orc.forward(p[:33], 0)
    mask = oracle.admg(r["cos"][0::2], 0.985, 2, 1)
    orc.forward(p[33:36], 33, mask, commit=False)
    orc.forward(p[33:34], 33)
    orc.truncate(20)
    plain = orc.generate_plain(p[:12], 12)
    spec, st, m, C = orc.generate_spec(p[:12], 12, 4, alpha=0.985, m=2, n=1)
    assert np.array_equal(plain, spec)
    orc.generate_adaptive(p[:12], 10, 5, alpha=0.9, m=2, n=1, exit_mode=1, gamma0=0.01, refresh=True)
    orc.generate_sampled(p[:12], 10, 3, 0.7, 5, mask=m)
    orc.close()
oracle.admg2(np.linspace(0.9, 1.0, 16), 0.95, 3, 2, True, 0.97, True)
oracle.sample_logits(np.linspace(-1, 1, 50), 0.6, 0.3)
si.sublayer_scales(1, 5); si.prompt(2, 9, 100); si.sampling_uniform(1, 2, 1)
print("sanitized run complete")
"""


@pytest.mark.slow
def test_oracle_and_input_generator_under_asan_and_ubsan(tmp_path):
    libasan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(libasan) or not os.path.exists(libasan):
        pytest.skip("no AddressSanitizer runtime with this gcc")
    flags = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-shared", "-fPIC"]
    orc = str(tmp_path / "liborc_san.so")
    synth = str(tmp_path / "libsynth_san.so")
    subprocess.check_call(["gcc", "-std=c11", "-fopenmp", *flags, "-o", orc, os.path.join(ROOT, "oracle", "asd_oracle.c"), "-lm"])
    subprocess.check_call(["gcc", "-fopenmp", *flags, "-o", synth, os.path.join(ROOT, "asd_inputs", "synth.c"), "-lm"])
    env = dict(os.environ)
    env["LD_PRELOAD"] = libasan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # CPython itself is not instrumented: its deliberate leaks at exit are not this test's business
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=97"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1:exitcode=98"
    env["OMP_NUM_THREADS"] = "4"
    r = subprocess.run([sys.executable, "-c", DRIVER.format(root=ROOT, synth=synth, orc=orc)], env=env, capture_output=True, text=True, timeout=600)
    report = r.stdout + r.stderr
    assert "AddressSanitizer" not in report and "runtime error" not in report, report[-4000:]
    assert r.returncode == 0 and "sanitized run complete" in r.stdout, report[-4000:]


HOST_DRIVER = r"""
import sys, ctypes
sys.path.insert(0, {root!r})
import numpy as np
import asd_inputs as si
import paper_2410_01028_amd as asd
asd.LIB_PATH = {lib!r}
L = asd.lib()
rng = np.random.default_rng(0)
for n_layers in (1, 4, 7, 32, 80):
    for _ in range(40):
        c = rng.uniform(0.9, 1.0, n_layers).astype(np.float32)
        mask = asd.admg(c, 0.95, int(rng.integers(0, 6)), int(rng.integers(0, n_layers + 2)), bool(rng.integers(0, 2)))
        assert mask.size == 2 * n_layers
        asd.admg2(rng.uniform(0.9, 1, 2 * n_layers).astype(np.float32), 0.95, 3, 1, True, 0.97, True)
for name in ("tiny", "7b", "13b", "7b-long", "70b"):
    s = si.SHAPES[name]
    for tune in (None, "qkv=1,8,1,1;o=1,16,0,0", "qkv_rows=2;pf_gu=4,1,2", "garbage", "qkv=,,,", ";;=;", "lm=2,8,1,1" * 40):
        assert asd.arena_bytes(asd.make_config(s, 4096, 64, debug_tune=tune)) > 0
assert asd.arena_bytes(asd.make_config(si.SHAPES["tiny"], asd.MAX_SEQ + 64, 64)) == 0
assert asd.arena_bytes(asd.make_config(si.SHAPES["tiny"], 64, 48)) == 0
h = ctypes.c_void_p()
cfg = asd.make_config(si.SHAPES["tiny"], 64, 64)
assert L.asd_create(ctypes.byref(cfg), 0, 0, None, ctypes.byref(h)) != 0 and L.asd_last_error(None)
for fn, args in ((L.asd_reset, (None,)), (L.asd_kv_len, (None,)), (L.asd_check, (None,)), (L.asd_truncate, (None, 0)),
                 (L.asd_get_kv, (None, 0, 0, 0, None, None))):
    assert fn(*args) != 0
print("sanitized run complete")
"""


@pytest.mark.slow
def test_host_code_of_the_library_under_asan_and_ubsan(tmp_path):
    """The HIP library's host code (argument checks, Algorithm 1, the arena plan, the launch-shape parser) compiled with
    -Xarch_host -fsanitize=address,undefined and driven on the CPU through every entry point that needs no device."""
    import shutil
    hipcc = shutil.which("hipcc")
    if not hipcc:
        pytest.skip("no hipcc")
    rt = subprocess.run([hipcc, "--offload-arch=gfx950", "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(rt) or not os.path.exists(rt):
        cand = [os.path.join(d, f) for d, _, fs in os.walk("/opt/rocm/lib/llvm/lib/clang") for f in fs if f == "libclang_rt.asan-x86_64.so"]
        if not cand:
            pytest.skip("no AddressSanitizer runtime with this hipcc")
        rt = cand[0]
    lib = str(tmp_path / "libasd_san.so")
    host = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"]
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-shared", "-shared-libsan"]
    for f in host:
        cmd += ["-Xarch_host", f]
    cmd += ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-result", "-Wno-unused-value", "-mllvm",
            "-amdgpu-kernarg-preload-count=16", os.path.join(ROOT, "paper_2410_01028_amd", "csrc", "asd_engine.hip"), "-o", lib]
    subprocess.run(cmd, check=True, capture_output=True, timeout=900)
    env = dict(os.environ)
    env["LD_PRELOAD"] = rt + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=97"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1:exitcode=98"
    r = subprocess.run([sys.executable, "-c", HOST_DRIVER.format(root=ROOT, lib=lib)], env=env, capture_output=True, text=True, timeout=600)
    report = r.stdout + r.stderr
    assert "AddressSanitizer" not in report and "runtime error" not in report, report[-4000:]
    assert r.returncode == 0 and "sanitized run complete" in r.stdout, report[-4000:]

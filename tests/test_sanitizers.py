"""The CPU oracle and the input generator under AddressSanitizer and UndefinedBehaviorSanitizer.

Both are plain C; a stray index in either would silently bend every parity claim built on them.  They are compiled
here with -fsanitize=address,undefined into a scratch directory and driven, in a child process that preloads the
sanitizer runtime, through the same Python bindings the tests use: the tiny workload's prompt pass, masked and
multi-row passes, plain, speculative, adaptive and sampled generation, Algorithm 1, and the generator's entry points.
Any report from either sanitizer fails the test."""
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

"""Hygiene of the CPU oracle, on the CPU: (1) the debug build that checks every integer sum and
difference of two samples for overflow, run over all five benchmark configurations at reduced
size -- the precondition of the whole algebra (no candidate leaves the element type) holds on the
generated inputs, and the debug build returns what the normal build returns; (2) the oracle's
source under AddressSanitizer and UndefinedBehaviorSanitizer, every entry point on every curve
length from 1 to 70."""
import os
import subprocess
import sys

import numpy as np
import pytest

from oracle import oracle
from paper_1912_04050_amd import workloads as wl

HERE = os.path.dirname(os.path.abspath(__file__))
ORACLE_DIR = os.path.join(os.path.dirname(HERE), "oracle")


def run_all_configs():
    """Every oracle operator the configurations use, at reduced size; returns the results."""
    out = []
    c = wl.config1(wl.DEFAULT_SEED)
    f, g = c["f"][:, :700], c["g"][:, :700]
    out += [oracle.minplus_conv(f, g), oracle.maxplus_deconv(f, g)]
    c = wl.config2(wl.DEFAULT_SEED, 6, 900)
    out += [oracle.minplus_conv(c["alpha_u"], c["beta_l"]), oracle.maxplus_deconv(c["alpha_u"], c["beta_l"]),
            oracle.max_hdev(c["alpha_u"], c["beta_l"])[0], oracle.max_vdev(c["alpha_u"], c["beta_l"]),
            oracle.closure(c["alpha_u"][:2, :120])[0]]
    c = wl.config3(wl.DEFAULT_SEED, 3, 1500)
    out += [oracle.minplus_conv(c["f"], c["g"]), oracle.maxplus_deconv(c["f"], c["g"]),
            oracle.maxplus_conv(c["f"], c["g"]), oracle.minplus_deconv(c["f"], c["g"])]
    c = wl.config4(wl.DEFAULT_SEED, chains=3, components=3, n=1200)
    a, _ = oracle.compose(c["gamma_u"], c["alpha_bar_u"])
    out.append(a)
    for i in range(3):
        au, bl = oracle.gpc_step(a, c["beta_u"][i], c["beta_l"][i])
        out += [au, bl, oracle.pseudo_inverse(c["gamma_u"], bl, 0), oracle.pseudo_inverse(c["gamma_u"], bl, 1)]
        a = au
    al = (a // 3).astype(a.dtype)
    out += list(oracle.gpc_step_lower(al, c["beta_u"][0], c["beta_l"][0]))
    out.append(oracle.conv_chain(np.ascontiguousarray(c["beta_l"])))
    c = wl.config5(wl.DEFAULT_SEED, 1500)
    out += [oracle.minplus_conv(c["f"], c["g"]), oracle.maxplus_deconv(c["f"], c["g"]),
            oracle.pseudo_inverse(c["f"], c["x"], 0), oracle.pseudo_inverse(c["f"], c["x"], 1)]
    return out


def test_overflow_checking_build_on_all_five_configurations():
    assert oracle.overflow_count() == -1            # the normal build does not count
    plain = run_all_configs()
    oracle.use_checked_build(True)
    try:
        oracle.overflow_count(reset=True)
        checked = run_all_configs()
        assert oracle.overflow_count() == 0          # the precondition holds on every configuration
        assert len(plain) == len(checked)
        for p, q in zip(plain, checked):
            assert p.dtype == q.dtype and np.array_equal(p, q)
        # and the check does see a violation: sums beyond int32, differences beyond int64
        f = np.array([[2**31 - 10, 2**31 - 5]], np.int32)
        oracle.minplus_conv(f, f)
        assert oracle.overflow_count() == 3          # three candidates, all of them overflow
        g = np.array([[-2**62, -2**62 + 1]], np.int64)
        h = np.array([[2**62, 2**62 + 5]], np.int64)
        oracle.maxplus_deconv(g, h)
        assert oracle.overflow_count() >= 1
        assert oracle.overflow_count() == 0          # reading resets
    finally:
        oracle.use_checked_build(False)


def test_oracle_source_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-fopenmp", "-DORACLE_CHECK_OVERFLOW", "-o", exe,
           os.path.join(ORACLE_DIR, "sanitize_main.cpp")]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0 and "asan" in (built.stderr or "").lower():
        pytest.skip("this toolchain has no static AddressSanitizer runtime: " + built.stderr.strip().splitlines()[-1])
    assert built.returncode == 0, built.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    sys.stdout.write(run.stdout)
    assert run.returncode == 0, run.stderr[-4000:]
    assert "oracle sanitizer run ok" in run.stdout and "overflow counter 0" in run.stdout

"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the CPU-side code: the fp64 oracle (plain C) and the host
checker of the kernels' staging addresses (C++). Each is linked with a small driver (tests/sanitize/) into an
executable of its own, so no sanitizer runtime has to be loaded into the Python process; a bad access or an
undefined operation aborts the run with a non-zero status. The oracle's results under the sanitizers are also
compared with those of the ordinary build, function by function."""
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import reference as ref

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
           OMP_NUM_THREADS="4")
ENV.pop("LD_PRELOAD", None)      # the sanitizer runtime must come first in the executable's own link order


def _build(compiler, sources, out, extra=()):
    if shutil.which(compiler) is None:
        pytest.skip(f"{compiler} not available")
    cmd = [compiler, *SAN, *extra, *sources, "-o", out, "-lm"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    return out


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = _build("gcc", [os.path.join(ROOT, "oracle", "dash_oracle.c"),
                         os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c")], str(tmp_path / "oracle_san"),
                 extra=["-std=c11", "-fopenmp", "-Wall"])
    rng = np.random.default_rng(77)
    n, Hq, Hkv, dh, d, m, N = 37, 4, 2, 8, 24, 16, 90
    k_keep, n_first, n_last = 15, 2, 1
    x = rng.standard_normal((n, d)) * np.exp(rng.standard_normal((n, 1)))
    q, k, v = rng.standard_normal((n, Hq, dh)), rng.standard_normal((n, Hkv, dh)), rng.standard_normal((n, Hkv, dh))
    w_o = rng.standard_normal((Hq * dh, d)) / np.sqrt(d)
    w_gate, w_up = rng.standard_normal((d, m)) / np.sqrt(d), rng.standard_normal((d, m)) / np.sqrt(d)
    w_down = rng.standard_normal((m, d)) / np.sqrt(m)
    pos = np.sort(rng.choice(N, size=n, replace=False)).astype(np.int32)
    rows = np.array([0, 5, 17, 36], dtype=np.int64)
    tau, theta = 0.35, 1.0e4
    inp, outp = tmp_path / "in.bin", tmp_path / "out.bin"
    with open(inp, "wb") as f:
        np.array([n, Hq, Hkv, dh, d, m, N, k_keep, n_first, n_last, len(rows)], dtype=np.int64).tofile(f)
        for a in (x, q, k, v, w_o, w_gate, w_up, w_down, np.array([tau]), np.array([theta])):
            np.ascontiguousarray(a, dtype=np.float64).tofile(f)
        pos.tofile(f)
        rows.tofile(f)
    r = subprocess.run([exe, str(inp), str(outp)], capture_output=True, text=True, env=ENV, timeout=120)
    assert r.returncode == 0, (r.returncode, r.stderr[-3000:])
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-3000:]
    got = np.fromfile(outp, dtype=np.float64)

    # the same calls through the ordinary build
    O = ref.attention_rows(q, k, v, pos, causal=True, scale=0.3)
    Osub = ref.attention_rows(q, k, v, pos, rows=rows, causal=False, scale=0.3)
    delta = ref.project(O, w_o)
    xn = ref.residual(x, delta)
    s_rel, s_abs = ref.scores(delta, x, ref.SCORE_REL), ref.scores(delta, None, ref.SCORE_ABS)
    h_thr = ref.decide_threshold(s_rel, tau, n_first, n_last)
    h_low = ref.decide_topk(s_rel, k_keep, n_first, n_last, keep_low=True)
    h_top = ref.decide_topk(s_rel, k_keep, n_first, n_last)
    new_idx, xc, n_out = ref.compact(h_top, pos, xn)
    full = ref.scatter_rows(xn, pos, np.full((N, d), -1.0), sel=h_top, sel_value=1)
    red = ref.flops_reduction_and_speedup(8192, 2792, 3584, 18944, 28, 11)
    full_cost = 28 * ref.flops_A(8192, 3584, 18944)
    want = np.concatenate([a.ravel().astype(np.float64) for a in (
        O, Osub, delta, xn, s_rel, s_abs, h_thr, h_low, h_top, np.array([n_out]), new_idx, xc, ref.rmsnorm(x),
        ref.rope(q, pos, theta), ref.ffn_swiglu(x, w_gate, w_up, w_down), full,
        np.array([ref.keep_count(n, 0.667), ref.keep_count(32768, 0.667, 64, 32, True), -1,
                  ref.flops_A(8192, 3584, 18944), full_cost, full_cost / red[1]]))])
    assert got.shape == want.shape
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)
    assert n_out == k_keep and int(h_low.sum()) == n - k_keep


def test_staging_checker_runs_clean_under_asan_and_ubsan(tmp_path):
    from test_staging_addresses import GEMM_SHAPES
    csrc = os.path.join(ROOT, "paper_2604_18103_amd", "csrc")
    exe = _build("g++", [os.path.join(csrc, "staging_check.cpp"),
                         os.path.join(ROOT, "tests", "sanitize", "staging_driver.cpp")], str(tmp_path / "staging_san"),
                 extra=["-std=c++17", "-Wall", f"-I{csrc}"])
    lines, kinds = [], []
    for M, K, N in GEMM_SHAPES:
        if M * N > 6e7:          # the largest launches take too long under the sanitizers; their addressing is the same
            continue
        for split in (0, 1 << 30):
            lines.append(f"g {M} {K} {N} 256 {split}")
            kinds.append("g")
    for n in (1, 63, 64, 65, 255, 257, 333, 1000, 10976):
        for Hkv, DH in ((4, 128), (2, 64)):
            lines.append(f"f {n} {Hkv} {DH} 1")
            kinds.append("f")
    r = subprocess.run([exe], input="\n".join(lines) + "\n", capture_output=True, text=True, env=ENV, timeout=600)
    assert r.returncode == 0, (r.returncode, r.stderr[-3000:])
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-3000:]
    out = r.stdout.strip().splitlines()
    assert len(out) == len(lines)
    for line, res in zip(lines, out):
        fields = res.split()
        assert fields[0] == "0" and int(fields[1]) > 0, (line, res)

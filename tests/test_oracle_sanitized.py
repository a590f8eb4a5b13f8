"""The oracle's C++ under AddressSanitizer + UBSan on the host: a subset of the pins through a sanitized build.

Runs as a child process (the sanitizer runtime has to be loaded first); skipped if the toolchain cannot build it."""
import os
import subprocess
import sys
import textwrap

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_under_asan_ubsan(tmp_path):
    lib = tmp_path / "liboracle_san.so"
    src = os.path.join(ROOT, "oracle", "srigl_oracle.cpp")
    r = subprocess.run(["g++", "-O1", "-g", "-std=c++17", "-fPIC", "-shared", "-fsanitize=address,undefined",
                        "-fno-sanitize-recover=undefined", "-o", str(lib), src], capture_output=True, text=True)
    if r.returncode != 0:
        pytest.skip("cannot build a sanitized oracle: " + r.stderr[-200:])
    asan = subprocess.run(["g++", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(asan):
        pytest.skip("libasan.so not found")
    code = textwrap.dedent("""
        import ctypes, sys
        sys.path.insert(0, %r)
        import numpy as np
        import oracle, synth_inputs as si
        oracle._lib = ctypes.CDLL(%r)          # route the front end to the sanitized build
        for (d_in, d_out, K, B, abl, dt) in ((16, 8, 3, 3, 0.25, "f32"), (50, 7, 1, 5, 0.0, "f32"), (257, 5, 257, 2, 0.0, "f32"),
                                             (130, 9, 7, 5, 0.2, "bf16"), (64, 4, 5, 0, 0.0, "f32"), (64, 6, 5, 2, 1.0, "f32")):
            L = si.make_layer(d_in, d_out, K, B, ablate_frac=abl, dtype=dt, seed=5)
            Wsrc = L.W_bf16 if dt == "bf16" else L.W
            xsrc = L.x_bf16 if dt == "bf16" else L.x
            assert oracle.check_fanin_mask(L.mask)["status"] == 0
            W_c, idx, active = oracle.condense(Wsrc, L.mask, K)
            assert oracle.check_fanin_idx(idx, d_in)["status"] == 0
            y, S = oracle.fwd(xsrc, W_c, idx, active, L.bias, d_out, want_scale=True)
            if dt == "f32":
                yd = oracle.dense_masked_fwd(L.x, L.W, L.mask, L.bias)
                assert np.array_equal(y, yd)
        print("sanitized oracle ok")
    """) % (ROOT, str(lib))
    preload = asan + (":" + os.environ["LD_PRELOAD"] if os.environ.get("LD_PRELOAD") else "")   # keep what is already preloaded
    env = dict(os.environ, LD_PRELOAD=preload, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0")
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0 and "sanitized oracle ok" in r.stdout, (r.stdout[-500:], r.stderr[-1500:])

"""The library driven by a caller written in C (tests/c_abi/decode_from_c.c: HIP runtime C API + include/vatt.h,
no Python or torch in that process), checked against the oracle and against the Python binding's call."""
import os
import struct
import subprocess

import numpy as np
import pytest

import workloads
from parity import check_all, alternatives_used, say
from util import plan_params

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_decode_from_a_c_program(tmp_path):
    say("vatt_decode called from a C program")
    from paper_2510_05688_amd import binding as vb
    from paper_2510_05688_amd.session import DecodeSession
    libdir = os.path.dirname(vb.LIB_PATH)
    exe = str(tmp_path / "decode_from_c")
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                        "-I", "/opt/rocm/include", os.path.join(ROOT, "tests", "c_abi", "decode_from_c.c"), "-o", exe,
                        "-L", libdir, "-l:libvatt.so", "-L", "/opt/rocm/lib", "-lamdhip64",
                        "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib"], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr

    wl = workloads.small_gqa(seed=71, batch=2, n=3008, seq_lens=[3008, 2963], epsilon=0.02)
    p = wl.params
    fin, fout = str(tmp_path / "in.bin"), str(tmp_path / "out.bin")
    with open(fin, "wb") as f:
        f.write(struct.pack("<9i", wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.n_max, int(p["sink"]),
                            int(p["window"]), int(p["topk_abs"]), int(p["base_abs"])))
        f.write(struct.pack("<4f", p["topk_frac"], p["base_frac"], p["epsilon"], p["delta"]))
        for a, dt in ((wl.q_bits, np.uint16), (wl.k_bits, np.uint16), (wl.v_bits, np.uint16),
                      (wl.seq_lens, np.int32), (wl.seeds, np.uint64)):
            f.write(np.ascontiguousarray(a, dtype=dt).tobytes())
    out = subprocess.run([exe, fin, fout], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "short workspace: workspace too small" in out.stdout and "vatt_decode: ok" in out.stdout

    raw = open(fout, "rb").read()
    head = np.frombuffer(raw, dtype=np.int64, count=6)
    idx_cap, seg = int(head[0]), [int(x) for x in head[1:]]
    B, Hq, d = wl.batch, wl.n_q_heads, wl.head_dim
    off = 48

    def take(dtype, shape):
        nonlocal off
        n = int(np.prod(shape))
        a = np.frombuffer(raw, dtype=dtype, count=n, offset=off).reshape(shape)
        off += n * np.dtype(dtype).itemsize
        return a
    res = dict(O=take(np.float32, (B, Hq, d)), lse=take(np.float32, (B, Hq)), idx=take(np.int32, (B, Hq, idx_cap)),
               counts=take(np.int32, (B, Hq, 8)), b_star=take(np.float64, (B, Hq)), stats=take(np.float32, (B, Hq, 4)),
               seg=seg)
    assert off == len(raw)
    reports = check_all(wl, res, label="from C")
    assert alternatives_used(reports) == (0, 0)
    assert any(r["b"] > r["b0"] for r in reports)

    # the same call through the Python binding gives the same bits
    sess = DecodeSession(plan_params(wl))
    sess.upload(wl.q_bits, wl.k_bits, wl.v_bits, wl.seq_lens, wl.seeds)
    sess.decode()
    py = sess.results_host()
    assert py["seg"] == seg
    for key in ("O", "lse", "counts", "b_star", "stats"):
        assert np.array_equal(py[key], res[key], equal_nan=True), key
    for b in range(B):
        for h in range(Hq):
            c = res["counts"][b, h]
            for s_, cnt in ((0, c[0]), (1, c[1]), (2, c[2]), (3, c[3]), (4, c[4])):
                assert np.array_equal(py["idx"][b, h, seg[s_]:seg[s_] + cnt], res["idx"][b, h, seg[s_]:seg[s_] + cnt])
    sess.close()

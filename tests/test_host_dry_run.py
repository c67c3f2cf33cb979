"""Host logic of the C ABI on the CPU: the library is compiled once more with kernel launches
stubbed out (tests/host_dry_run/dry_launch.h) and the host compiler's undefined-behaviour checks
in trap mode, then every entry point is called with thousands of valid and invalid shapes and
fake, never dereferenced device pointers.  A division by zero, an overflowing shift or a wild
index in the planning code ends the subprocess with a signal; a valid call must return CIRC_OK."""
import os
import shutil
import subprocess
import sys
import textwrap

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_1708_08917_amd", "csrc", "circ_api.hip")
DRY = os.path.join(ROOT, "tests", "host_dry_run", "dry_launch.h")
HIPCC = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"

DRIVER = textwrap.dedent(r'''
    import ctypes, random, sys
    L = ctypes.CDLL(sys.argv[1])
    c_int, c_size, c_ptr, c_ll, c_f = ctypes.c_int, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_longlong, ctypes.c_float
    for n in ["circ_spectra_bytes", "circ_fc_workspace_bytes", "circ_conv_workspace_bytes",
              "circ_conv_backward_workspace_bytes", "circ_spectra_bytes_f16", "circ_fc_workspace_bytes_f16",
              "circ_fc_backward_workspace_bytes_f16"]:
        getattr(L, n).restype = c_size
    A, big = 0x10000, 1 << 36
    P = [c_ptr(A + i * big) for i in range(6)]
    ws = c_size(1 << 62)
    # valid calls run to the end of the host code
    assert L.circ_precompute_spectra(P[0], 1, 64, 64, 64, P[1], None) == 0
    assert L.circ_precompute_spectra(P[0], 9, 4, 4, 64, P[1], None) == 0
    assert L.circ_precompute_spectra(P[0], 1, 3, 5, 12, P[1], None) == 0
    for (p, q, k, b) in [(64, 64, 16, 1), (64, 64, 64, 64), (32, 72, 128, 256), (32, 72, 128, 1), (64, 64, 256, 1024),
                         (3, 5, 12, 7), (40, 40, 100, 64), (2, 3, 1, 4), (125, 512, 8, 1), (2, 3, 512, 2)]:
        assert L.circ_fc_forward(P[0], P[1], None, P[2], p, q, k, b, 0, P[3], ws, None) == 0, (p, q, k, b)
        fits = L.circ_fc_workspace_bytes(p, q, k, b, 0) <= (32 << 20)
        assert L.circ_fc_forward_static(P[0], P[1], None, P[2], p, q, k, b, 0, None) == (0 if fits else -3), (p, q, k, b)
        assert L.circ_fc_backward(P[0], P[1], P[2], P[3], P[4], p, q, k, b, P[5], ws, None) == 0, (p, q, k, b)
        assert L.circ_fc_sgd_step(P[0], P[1], P[2], P[3], c_f(0.1), p, q, k, b, P[5], ws, None) == 0, (p, q, k, b)
        assert L.circ_export_weights(P[0], 1, p, q, k, P[1], None) == 0
        if k >= 8 and k & (k - 1) == 0:
            assert L.circ_precompute_spectra_f16(P[0], p, q, k, P[1], None) == 0
            assert L.circ_fc_forward_f16(P[0], P[1], None, P[2], p, q, k, b, 0, P[3], ws, None) == 0
            assert L.circ_precompute_spectra_bf16(P[0], p, q, k, P[1], None) == 0
            assert L.circ_fc_forward_bf16(P[0], P[1], None, P[2], p, q, k, b, 0, P[3], ws, None) == 0
            assert L.circ_fc_backward_f16(P[0], P[1], P[2], P[3], P[4], p, q, k, b, P[5], ws, None) == 0
            assert L.circ_fc_backward_bf16(P[0], P[1], P[2], P[3], P[4], p, q, k, b, P[5], ws, None) == 0
    for (N, Ci, Co, H, W, r, pad, k) in [(32, 256, 256, 28, 28, 3, 1, 64), (2, 384, 384, 13, 13, 3, 1, 96), (1, 8, 8, 5, 5, 3, 0, 4),
                                         (3, 16, 32, 9, 4, 1, 0, 16), (2, 128, 64, 7, 32, 5, 2, 64), (2, 64, 64, 224, 224, 3, 1, 64),
                                         (1, 64, 64, 6, 2000, 3, 1, 64), (2, 6, 9, 8, 1, 3, 1, 3)]:
        assert L.circ_conv_forward(P[0], P[1], None, P[2], N, Ci, Co, H, W, r, 1, pad, k, 0, P[3], ws, None) == 0
        assert L.circ_conv_backward(P[0], P[1], P[2], P[3], P[4], N, Ci, Co, H, W, r, 1, pad, k, P[5], ws, None) == 0
        if k >= 8 and k & (k - 1) == 0:
            assert L.circ_conv_forward_f16(P[0], P[1], None, P[2], N, Ci, Co, H, W, r, 1, pad, k, 0, P[3], ws, None) == 0
            assert L.circ_conv_forward_bf16(P[0], P[1], None, P[2], N, Ci, Co, H, W, r, 2, pad, k, 0, P[3], ws, None) == 0
            assert L.circ_conv_backward_f16(P[0], P[1], P[2], P[3], P[4], N, Ci, Co, H, W, r, 1, pad, k, P[5], ws, None) == 0
            assert L.circ_conv_backward_bf16(P[0], P[1], P[2], P[3], P[4], N, Ci, Co, H, W, r, 2, pad, k, P[5], ws, None) == 0
        assert L.circ_conv_sgd_step(P[0], P[1], P[2], None, c_f(0.1), N, Ci, Co, H, W, r, 1, pad, k, P[5], ws, None) == 0
        for st in (2, 3):
            assert L.circ_conv_forward(P[0], P[1], None, P[2], N, Ci, Co, H, W, r, st, pad, k, 0, P[3], ws, None) == 0
            assert L.circ_conv_backward(P[0], P[1], P[2], P[3], P[4], N, Ci, Co, H, W, r, st, pad, k, P[5], ws, None) == 0
    assert L.circ_bias_grad(P[0], P[1], c_ll(32), 256, c_ll(784), None) == 0
    # max-pooling and chains of layers
    class Layer(ctypes.Structure):
        _fields_ = [("kind", c_int), ("epilogue", c_int), ("w_hat", c_ptr), ("bias", c_ptr), ("k", c_int), ("p", c_int), ("q", c_int),
                    ("C_in", c_int), ("C_out", c_int), ("H", c_int), ("W", c_int), ("r", c_int), ("stride", c_int), ("pad", c_int)]
    L.circ_chain_workspace_bytes.restype = c_size
    for (N, C, H, W, win, st) in [(32, 256, 28, 28, 2, 2), (1, 1, 1, 1, 1, 1), (2, 70000, 3, 3, 2, 1), (1, 3, 1000, 1000, 3, 2)]:
        assert L.circ_maxpool_forward(P[0], P[1], N, C, H, W, win, st, None) == 0, (N, C, H, W, win, st)
    assert L.circ_maxpool_forward(P[0], P[1], 1, 1, 2, 2, 3, 1, None) == -1
    assert L.circ_maxpool_forward(P[0], P[1], 1, 3, 60000, 60000, 3, 2, None) == -1      # in-plane index beyond 32 bits
    head = (Layer * 3)(Layer(kind=0, epilogue=3, w_hat=P[2], bias=P[3], k=128, p=32, q=72),
                       Layer(kind=0, epilogue=3, w_hat=P[2], bias=P[3], k=128, p=32, q=32),
                       Layer(kind=0, epilogue=1, w_hat=P[2], bias=P[3], k=8, p=125, q=512))
    net = (Layer * 4)(Layer(kind=1, epilogue=3, w_hat=P[2], bias=P[3], k=64, C_in=64, C_out=128, H=14, W=14, r=3, stride=1, pad=1),
                      Layer(kind=2, C_in=128, H=14, W=14, r=2, stride=2),
                      Layer(kind=0, epilogue=3, w_hat=P[2], bias=P[3], k=64, p=4, q=98),
                      Layer(kind=0, epilogue=0, w_hat=P[2], bias=None, k=2, p=5, q=128))
    for chain, n in ((head, 3), (net, 4)):
        for b in (1, 2, 64):
            need = L.circ_chain_workspace_bytes(chain, n, b)
            assert need > 0
            assert L.circ_chain_forward(chain, n, P[0], P[1], b, P[5], ws, None) == 0
            assert L.circ_chain_forward(chain, n, P[0], P[1], b, P[5], c_size(need - 1), None) == -3
    net[2].q = 97
    assert L.circ_chain_workspace_bytes(net, 4, 1) == 0 and L.circ_chain_forward(net, 4, P[0], P[1], 1, P[5], ws, None) == -1
    assert L.circ_chain_forward(head, 0, P[0], P[1], 1, P[5], ws, None) == -1
    head[1].kind = 7
    assert L.circ_chain_forward(head, 3, P[0], P[1], 1, P[5], ws, None) == -1
    # random shapes, valid or not: only the absence of a trap counts
    rng = random.Random(1708)
    ks = [1, 2, 3, 4, 5, 6, 7, 8, 12, 16, 24, 32, 48, 64, 96, 100, 128, 192, 256, 384, 500, 511, 512, 0, -1, 513, 1024]
    dims = [1, 2, 3, 4, 5, 7, 8, 9, 15, 16, 17, 31, 32, 33, 63, 64, 65, 72, 100, 128, 129, 255, 256, 1000, 4096, 65535, 70000, 0, -3]
    bat = [1, 2, 3, 4, 5, 8, 16, 17, 31, 32, 33, 64, 100, 128, 129, 255, 256, 257, 1000, 1024, 5000, 100000, 1 << 20, 0, -1]
    for _ in range(6000):
        p, q, k, b = rng.choice(dims), rng.choice(dims), rng.choice(ks), rng.choice(bat)
        L.circ_spectra_bytes(1, p, q, k); L.circ_spectra_bytes(9, p, q, k)
        L.circ_fc_workspace_bytes(p, q, k, b, 0); L.circ_fc_workspace_bytes(p, q, k, b, 1)
        L.circ_spectra_bytes_f16(p, q, k); L.circ_fc_workspace_bytes_f16(p, q, k, b)
        L.circ_precompute_spectra(P[0], rng.choice([1, 9, 25]), p, q, k, P[1], None)
        L.circ_precompute_spectra_f16(P[0], p, q, k, P[1], None)
        L.circ_fc_forward(P[0], P[1], None, P[2], p, q, k, b, 0, P[3], ws, None)
        L.circ_fc_forward_static(P[0], P[1], None, P[2], p, q, k, b, 0, None)
        L.circ_fc_forward_f16(P[0], P[1], None, P[2], p, q, k, b, 0, P[3], ws, None)
        L.circ_fc_forward_bf16(P[0], P[1], None, P[2], p, q, k, b, 0, P[3], ws, None)
        L.circ_fc_backward_workspace_bytes_f16(p, q, k, b)
        L.circ_fc_backward_f16(P[0], P[1], P[2], P[3], P[4], p, q, k, b, P[5], ws, None)
        L.circ_fc_backward_bf16(P[0], P[1], P[2], None, P[4], p, q, k, b, P[5], ws, None)
        L.circ_fc_backward(P[0], P[1], P[2], P[3], P[4], p, q, k, b, P[5], ws, None)
        L.circ_fc_backward(P[0], P[1], P[2], None, P[4], p, q, k, b, P[5], ws, None)
        L.circ_fc_sgd_step(P[0], P[1], P[2], None, c_f(0.1), p, q, k, b, P[5], ws, None)
        L.circ_export_weights(P[0], rng.choice([1, 9, 25]), p, q, k, P[1], None)
        N, H, W = rng.choice([1, 2, 3, 32, 33, 256, 0]), rng.choice([1, 2, 5, 13, 14, 28, 56, 224, 1024, 0]), rng.choice([1, 2, 4, 5, 13, 14, 28, 56, 224, 1024, 4000])
        r, pad, st = rng.choice([1, 3, 5, 7, 9, 2, 4, 0]), rng.choice([0, 1, 2, 3, 4]), rng.choice([1, 1, 2, 3, 0])
        Ci = min(max(q, 1) * max(k, 1), 1 << 20); Co = min(max(p, 1) * max(k, 1), 1 << 20)
        L.circ_conv_workspace_bytes(N, Ci, Co, H, W, r, st, pad, k); L.circ_conv_backward_workspace_bytes(N, Ci, Co, H, W, r, st, pad, k)
        L.circ_conv_forward(P[0], P[1], None, P[2], N, Ci, Co, H, W, r, st, pad, k, 0, P[3], ws, None)
        L.circ_conv_forward_f16(P[0], P[1], None, P[2], N, Ci, Co, H, W, r, st, pad, k, 0, P[3], ws, None)
        L.circ_conv_backward_bf16(P[0], P[1], P[2], P[3], P[4], N, Ci, Co, H, W, r, st, pad, k, P[5], ws, None)
        L.circ_conv_backward(P[0], P[1], P[2], P[3], P[4], N, Ci, Co, H, W, r, st, pad, k, P[5], ws, None)
        L.circ_conv_backward(P[0], P[1], P[2], None, P[4], N, Ci, Co, H, W, r, st, pad, k, P[5], ws, None)
        L.circ_conv_sgd_step(P[0], P[1], P[2], None, c_f(0.1), N, Ci, Co, H, W, r, st, pad, k, P[5], ws, None)
        L.circ_bias_grad(P[0], P[1], c_ll(rng.choice([1, 32, 0, 1 << 40])), rng.choice([1, 256, 0]), c_ll(rng.choice([1, 784, 0])), None)
    print("dry run ok")
''')


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not found")
def test_host_code_dry_run_under_ub_checks(tmp_path):
    lib = str(tmp_path / "libcirc_dry.so")
    cmd = [HIPCC, "-O0", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-Wno-pass-failed", "-Wno-unused-value", "-w", "-include", DRY, "-Xarch_host",
           "-fsanitize=undefined", "-Xarch_host", "-fsanitize-trap=undefined", "-o", lib, SRC]
    subprocess.run(cmd, check=True, capture_output=True, timeout=600)
    drv = tmp_path / "driver.py"
    drv.write_text(DRIVER)
    out = subprocess.run([sys.executable, str(drv), lib], capture_output=True, text=True, timeout=600)
    assert out.returncode == 0, (out.returncode, out.stdout[-2000:], out.stderr[-2000:])
    assert "dry run ok" in out.stdout

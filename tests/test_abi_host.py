"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, sizes are as documented, and argument errors come back as status codes
before anything is launched."""
import ctypes
import os
import re

import pytest

from paper_1708_08917_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "circ.h")

pytestmark = pytest.mark.skipif(not os.path.exists(B.LIB_PATH), reason="libcirc.so not built (run __graft_entry__.build())")


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(circ_[a-z0-9_]+)\s*\(", src)))


def test_exports_every_declared_symbol():
    L = ctypes.CDLL(B.LIB_PATH)
    names = declared_functions()
    assert {"circ_precompute_spectra", "circ_fc_forward", "circ_conv_forward", "circ_fc_backward"} <= set(names)
    for n in names:
        assert hasattr(L, n), n
    assert set(names) == set(B.SIGNATURES), "binding and header list different entry points"


def test_status_strings():
    for s in (0, -1, -2, -3, -4):
        assert B.status_string(s).startswith("CIRC_")
    assert "unknown" in B.status_string(-99)


def test_spectra_bytes():
    # FC blob: unfused forward + backward operands ((k/2+1) bins per block), then for each of the two
    # directions (forward grid p x q, backward-data grid q x p) the k/2-slot operands of the fused
    # kernel (k >= 32) and of the batch <= 2 kernel (k >= 4); every section 256 B aligned
    assert B.circ_spectra_bytes(1, 64, 64, 64) == 2 * 64 * 64 * 33 * 8 + 4 * 64 * 64 * 32 * 8
    assert B.circ_spectra_bytes(1, 3, 5, 2) == 2 * 256          # k = 2: only the two unfused sections
    # CONV blob (9 grids of 4 x 4 blocks, k = 64): unfused sections + fused CONV operands (9*4*2*64 float2)
    # for the forward pass and the same again for backward-data (transposed grids, reflected filter)
    assert B.circ_spectra_bytes(9, 4, 4, 64) == 2 * ((9 * 16 * 33 * 8 + 255) // 256 * 256) + 2 * 9 * 4 * 2 * 64 * 8
    # block sizes that are not powers of two (and k = 1) hold only the two unfused sections
    assert B.circ_spectra_bytes(1, 3, 5, 3) == 2 * 256          # 3*5 blocks x 2 bins x 8 B = 240 -> 256
    assert B.circ_spectra_bytes(1, 64, 64, 96) == 2 * 64 * 64 * 49 * 8
    assert B.circ_spectra_bytes(1, 2, 2, 1) == 2 * 256
    for bad in [(0, 1, 1, 8), (1, 0, 1, 8), (1, 1, 0, 8), (1, 1, 1, 513), (1, 1, 1, -2), (1, 1, 1, 1024), (1, 1, 1, 0)]:
        assert B.circ_spectra_bytes(*bad) == 0


def test_workspace_bytes():
    F = 33
    assert B.circ_fc_workspace_bytes(64, 64, 64, 64) == 2 * F * 64 * 64 * 8
    assert B.circ_fc_workspace_bytes(64, 64, 64, 64, True) == 3 * F * 64 * 64 * 8
    assert B.circ_fc_workspace_bytes(64, 64, 48, 64) == 2 * 25 * 64 * 64 * 8      # any 1 <= k <= 512
    assert B.circ_fc_workspace_bytes(64, 64, 600, 64) == 0
    assert B.circ_conv_workspace_bytes(32, 256, 256, 28, 28, 3, 1, 1, 64) == 2 * F * 4 * 32 * 784 * 8
    assert B.circ_conv_workspace_bytes(32, 256, 256, 28, 28, 3, 2, 1, 64) == F * 4 * 32 * (784 + 196) * 8    # stride 2: 14 x 14 outputs
    assert B.circ_conv_workspace_bytes(32, 256, 256, 28, 28, 3, 0, 1, 64) == 0
    assert B.circ_conv_workspace_bytes(32, 250, 256, 28, 28, 3, 1, 1, 64) == 0


A = 0x1000  # fake, aligned, never dereferenced: the calls below must fail before any launch


def test_fc_forward_argument_errors():
    f = B.lib().circ_fc_forward
    ws = 1 << 30
    ok_args = dict(w_hat=A, x=A, bias=None, y=A + (1 << 28), p=2, q=2, k=8, batch=2, epi=0, wsp=A + (2 << 28), wsb=ws)

    def call(**kw):
        a = dict(ok_args); a.update(kw)
        return f(a["w_hat"], a["x"], a["bias"], a["y"], a["p"], a["q"], a["k"], a["batch"], a["epi"], a["wsp"], a["wsb"], None)

    assert call(k=0) == B.CIRC_EINVAL
    assert call(k=513) == B.CIRC_EINVAL
    assert call(k=1024) == B.CIRC_EINVAL
    assert call(p=0) == B.CIRC_EINVAL
    assert call(batch=-1) == B.CIRC_EINVAL
    assert call(x=None) == B.CIRC_EINVAL
    assert call(y=None) == B.CIRC_EINVAL
    assert call(w_hat=None) == B.CIRC_EINVAL
    assert call(x=A + 4) == B.CIRC_EINVAL                     # misaligned
    assert call(epi=B.EPI_BIAS) == B.CIRC_EINVAL              # bias flag without bias pointer
    assert call(epi=8) == B.CIRC_EINVAL
    assert call(y=A) == B.CIRC_EINVAL                         # in place
    assert call(wsb=16) == B.CIRC_EWORKSPACE
    assert call(wsp=None) == B.CIRC_EWORKSPACE


def test_fc_backward_argument_errors():
    f = B.lib().circ_fc_backward
    big = 1 << 28

    def call(w_hat=A, x=A + big, dy=A + 2 * big, dx=A + 3 * big, dw=A + 4 * big, p=2, q=2, k=8, batch=2,
             wsp=A + 5 * big, wsb=1 << 30):
        return f(w_hat, x, dy, dx, dw, p, q, k, batch, wsp, wsb, None)

    assert call(k=0) == B.CIRC_EINVAL
    assert call(dy=None) == B.CIRC_EINVAL
    assert call(dx=None, dw=None) == B.CIRC_EINVAL
    assert call(x=None) == B.CIRC_EINVAL                      # dw needs x
    assert call(dx=A + 2 * big) == B.CIRC_EINVAL              # dx aliases dy
    assert call(wsb=0) == B.CIRC_EWORKSPACE


def test_conv_argument_errors():
    f = B.lib().circ_conv_forward
    big = 1 << 28

    def call(w_hat=A, x=A + big, bias=None, y=A + 2 * big, N=1, C_in=8, C_out=8, H=4, W=4, r=3, stride=1, pad=1, k=4,
             epi=0, wsp=A + 3 * big, wsb=1 << 30):
        return f(w_hat, x, bias, y, N, C_in, C_out, H, W, r, stride, pad, k, epi, wsp, wsb, None)

    assert call(C_in=6) == B.CIRC_EINVAL                      # k does not divide C_in
    assert call(k=1024, C_in=1024, C_out=1024) == B.CIRC_EINVAL
    assert call(stride=0) == B.CIRC_EINVAL
    assert call(stride=-2) == B.CIRC_EINVAL
    assert call(r=0) == B.CIRC_EINVAL
    assert call(r=7) == B.CIRC_EINVAL                         # filter larger than the padded image
    assert call(pad=3) == B.CIRC_EINVAL
    assert call(x=None) == B.CIRC_EINVAL
    assert call(wsb=8) == B.CIRC_EWORKSPACE


def test_conv_backward_argument_errors():
    f = B.lib().circ_conv_backward
    big = 1 << 28

    def call(w_hat=A, x=A + big, dy=A + 2 * big, dx=A + 3 * big, dw=A + 4 * big, N=1, C_in=8, C_out=8, H=4, W=4, r=3,
             stride=1, pad=1, k=4, wsp=A + 5 * big, wsb=1 << 30):
        return f(w_hat, x, dy, dx, dw, N, C_in, C_out, H, W, r, stride, pad, k, wsp, wsb, None)

    assert call(C_out=6) == B.CIRC_EINVAL                     # k does not divide C_out
    assert call(stride=0) == B.CIRC_EINVAL
    assert call(r=0) == B.CIRC_EINVAL
    assert call(pad=3) == B.CIRC_EINVAL
    assert call(N=0) == B.CIRC_EINVAL                         # empty batch
    assert call(dy=None) == B.CIRC_EINVAL
    assert call(dx=None, dw=None) == B.CIRC_EINVAL
    assert call(x=None) == B.CIRC_EINVAL                      # dw needs x
    assert call(dx=A + 2 * big) == B.CIRC_EINVAL              # dx aliases dy
    assert call(dw=A + big) == B.CIRC_EINVAL                  # dw aliases x
    assert call(dy=A + 2 * big + 8) == B.CIRC_EINVAL          # misaligned
    assert call(wsb=64) == B.CIRC_EWORKSPACE
    assert call(wsp=None) == B.CIRC_EWORKSPACE
    wb = B.circ_conv_backward_workspace_bytes
    assert wb(1, 8, 8, 4, 4, 3, 1, 1, 4) > B.circ_conv_workspace_bytes(1, 8, 8, 4, 4, 3, 1, 1, 4)
    assert wb(1, 8, 8, 4, 4, 3, 0, 1, 4) == 0 and wb(1, 6, 8, 4, 4, 3, 1, 1, 4) == 0
    assert 0 < wb(1, 8, 8, 4, 4, 3, 2, 1, 4) < wb(1, 8, 8, 4, 4, 3, 1, 1, 4)    # stride 2: fewer output pixels


def test_sgd_step_and_export_argument_errors():
    import ctypes
    big = 1 << 28
    f = B.lib().circ_fc_sgd_step

    def call(w_hat=A, x=A + big, dy=A + 2 * big, dx=A + 3 * big, lr=0.1, p=2, q=2, k=8, batch=2, wsp=A + 5 * big,
             wsb=1 << 30):
        return f(w_hat, x, dy, dx, ctypes.c_float(lr), p, q, k, batch, wsp, wsb, None)

    assert call(w_hat=None) == B.CIRC_EINVAL
    assert call(lr=float("nan")) == B.CIRC_EINVAL
    assert call(x=None) == B.CIRC_EINVAL                      # the step needs x
    assert call(k=0) == B.CIRC_EINVAL
    assert call(batch=0) == B.CIRC_EINVAL
    assert call(x=A + 256) == B.CIRC_EINVAL                   # x lies inside the blob that is rewritten
    assert call(dx=A) == B.CIRC_EINVAL
    assert call(wsb=0) == B.CIRC_EWORKSPACE
    g = B.lib().circ_conv_sgd_step

    def callc(w_hat=A, x=A + big, dy=A + 2 * big, dx=None, lr=0.1, N=1, C_in=8, C_out=8, H=4, W=4, r=3, stride=1, pad=1,
              k=4, wsp=A + 5 * big, wsb=1 << 30):
        return g(w_hat, x, dy, dx, ctypes.c_float(lr), N, C_in, C_out, H, W, r, stride, pad, k, wsp, wsb, None)

    assert callc(w_hat=None) == B.CIRC_EINVAL
    assert callc(lr=float("nan")) == B.CIRC_EINVAL
    assert callc(stride=0) == B.CIRC_EINVAL
    assert callc(x=None) == B.CIRC_EINVAL
    assert callc(dy=A + 512) == B.CIRC_EINVAL                 # dy lies inside the blob
    assert callc(wsb=64) == B.CIRC_EWORKSPACE
    e = B.lib().circ_export_weights
    assert e(A, 1, 2, 2, 8, None, None) == B.CIRC_EINVAL
    assert e(None, 1, 2, 2, 8, A + big, None) == B.CIRC_EINVAL
    assert e(A, 0, 2, 2, 8, A + big, None) == B.CIRC_EINVAL
    assert e(A, 1, 2, 2, 513, A + big, None) == B.CIRC_EINVAL
    assert e(A, 1, 2, 2, 8, A + 64, None) == B.CIRC_EINVAL    # w lies inside the blob


def test_f16_argument_errors():
    big = 1 << 28
    # both orientations of the grid, each also in the fused kernel's operand order (32 slots per block)
    # ... and in the batch <= 2 kernel's (k/2 words per block)
    assert B.lib().circ_spectra_bytes_f16(64, 64, 64) == 2 * 33 * 64 * 64 * 4 + 2 * 32 * 64 * 64 * 4 + 2 * 32 * 64 * 64 * 4
    assert B.lib().circ_spectra_bytes_f16(64, 64, 512) == 2 * 257 * 64 * 64 * 4 + 2 * 256 * 64 * 64 * 4   # no fused kernel for k = 512
    assert B.lib().circ_spectra_bytes_f16(64, 64, 4) == 0          # k below 8
    assert B.lib().circ_spectra_bytes_f16(64, 64, 96) == 0         # not a power of two
    assert B.lib().circ_spectra_bytes_f16(0, 64, 64) == 0
    assert B.circ_fc_workspace_bytes_f16(64, 64, 64, 64) == 2 * 33 * 64 * 64 * 4
    assert B.circ_fc_workspace_bytes_f16(64, 64, 64, 0) == 0
    pre = B.lib().circ_precompute_spectra_f16
    assert pre(None, 2, 2, 8, A, None) == B.CIRC_EINVAL
    assert pre(A, 2, 2, 12, A + big, None) == B.CIRC_EINVAL
    assert pre(A, 2, 2, 8, A, None) == B.CIRC_EINVAL              # output aliases input
    assert B.lib().circ_spectra_bytes_bf16(64, 64, 64) == B.lib().circ_spectra_bytes_f16(64, 64, 64)
    assert B.lib().circ_fc_workspace_bytes_bf16(64, 64, 64, 64) == 2 * 33 * 64 * 64 * 4
    assert B.lib().circ_precompute_spectra_bf16(A, 2, 2, 12, A + big, None) == B.CIRC_EINVAL
    for f in (B.lib().circ_fc_forward_f16, B.lib().circ_fc_forward_bf16):

        def call(w_hat=A, x=A + big, bias=None, y=A + 2 * big, p=2, q=2, k=8, batch=2, epi=0, wsp=A + 3 * big, wsb=1 << 30):
            return f(w_hat, x, bias, y, p, q, k, batch, epi, wsp, wsb, None)

        assert call(k=4) == B.CIRC_EINVAL
        assert call(k=24) == B.CIRC_EINVAL
        assert call(x=None) == B.CIRC_EINVAL
        assert call(epi=B.EPI_BIAS) == B.CIRC_EINVAL                  # bias flag without a bias
        assert call(epi=8) == B.CIRC_EINVAL
        assert call(y=A + big) == B.CIRC_EINVAL                       # in place
        assert call(x=A + big + 2) == B.CIRC_EINVAL                   # misaligned
        assert call(wsb=16) == B.CIRC_EWORKSPACE


def test_f16_backward_argument_errors():
    big = 1 << 28
    spec = 33 * 64 * 64 * 4
    # two spectra each of x and dy, one fp32 partial spectrum of dw per slice of the batch
    assert B.circ_fc_backward_workspace_bytes_f16(64, 64, 64, 64) == 4 * spec + 2 * spec
    assert B.lib().circ_fc_backward_workspace_bytes_bf16(64, 64, 64, 64) == 6 * spec
    assert B.circ_fc_backward_workspace_bytes_f16(64, 64, 64, 1024) == 4 * 16 * spec + 8 * 2 * spec   # 8 slices of 128
    assert B.circ_fc_backward_workspace_bytes_f16(64, 64, 24, 64) == 0
    assert B.circ_fc_backward_workspace_bytes_f16(64, 0, 64, 64) == 0
    for f in (B.lib().circ_fc_backward_f16, B.lib().circ_fc_backward_bf16):

        def call(w_hat=A, x=A + big, dy=A + 2 * big, dx=A + 3 * big, dw=A + 4 * big, p=2, q=2, k=8, batch=2, wsp=A + 5 * big,
                 wsb=1 << 30):
            return f(w_hat, x, dy, dx, dw, p, q, k, batch, wsp, wsb, None)

        assert call(k=4) == B.CIRC_EINVAL
        assert call(k=48) == B.CIRC_EINVAL
        assert call(dy=None) == B.CIRC_EINVAL
        assert call(dx=None, dw=None) == B.CIRC_EINVAL               # nothing to compute
        assert call(x=None) == B.CIRC_EINVAL                         # dw needs x
        assert call(dx=A + 2 * big) == B.CIRC_EINVAL                 # dx aliases dy
        assert call(dw=A + 3 * big) == B.CIRC_EINVAL                 # dw aliases dx
        assert call(dy=A + 2 * big + 2) == B.CIRC_EINVAL             # misaligned
        assert call(batch=0) == B.CIRC_EINVAL
        assert call(wsb=16) == B.CIRC_EWORKSPACE


def test_conv_f16_argument_errors():
    big = 1 << 28
    for f in (B.lib().circ_conv_forward_f16, B.lib().circ_conv_forward_bf16):

        def call(w_hat=A, x=A + big, bias=None, y=A + 2 * big, N=2, Ci=16, Co=16, H=5, W=5, r=3, stride=1, pad=1, k=8, epi=0,
                 wsp=A + 3 * big, wsb=1 << 30):
            return f(w_hat, x, bias, y, N, Ci, Co, H, W, r, stride, pad, k, epi, wsp, wsb, None)

        assert call(k=4) == B.CIRC_EINVAL                             # below the 16-bit range of k
        assert call(Ci=12, Co=12, k=12) == B.CIRC_EINVAL              # not a power of two
        assert call(x=None) == B.CIRC_EINVAL
        assert call(Ci=20) == B.CIRC_EINVAL                           # channels not a multiple of k
        assert call(stride=0) == B.CIRC_EINVAL
        assert call(pad=3) == B.CIRC_EINVAL
        assert call(epi=B.EPI_BIAS) == B.CIRC_EINVAL
        assert call(y=A + big) == B.CIRC_EINVAL                       # in place
        assert call(wsb=16) == B.CIRC_EWORKSPACE


def test_conv_backward_f16_argument_errors():
    big = 1 << 28
    for f in (B.lib().circ_conv_backward_f16, B.lib().circ_conv_backward_bf16):

        def call(w_hat=A, x=A + big, dy=A + 2 * big, dx=A + 3 * big, dw=A + 4 * big, N=2, Ci=16, Co=16, H=5, W=5, r=3, stride=1,
                 pad=1, k=8, wsp=A + 5 * big, wsb=1 << 30):
            return f(w_hat, x, dy, dx, dw, N, Ci, Co, H, W, r, stride, pad, k, wsp, wsb, None)

        assert call(k=4) == B.CIRC_EINVAL
        assert call(Ci=12, Co=12, k=12) == B.CIRC_EINVAL              # not a power of two
        assert call(dy=None) == B.CIRC_EINVAL
        assert call(dx=None, dw=None) == B.CIRC_EINVAL
        assert call(x=None) == B.CIRC_EINVAL                          # dw needs x
        assert call(dx=A + 2 * big) == B.CIRC_EINVAL                  # dx aliases dy
        assert call(wsb=16) == B.CIRC_EWORKSPACE


def test_bias_grad_argument_errors():
    f = B.lib().circ_bias_grad
    assert f(None, A, 2, 8, 1, None) == B.CIRC_EINVAL
    assert f(A, None, 2, 8, 1, None) == B.CIRC_EINVAL
    assert f(A, A + (1 << 20), 0, 8, 1, None) == B.CIRC_EINVAL    # empty batch
    assert f(A, A + (1 << 20), 2, 0, 1, None) == B.CIRC_EINVAL
    assert f(A, A + (1 << 20), 2, 8, 0, None) == B.CIRC_EINVAL
    assert f(A, A + 16, 2, 8, 1, None) == B.CIRC_EINVAL           # db inside dy
    assert f(A + 4, A + (1 << 20), 2, 8, 1, None) == B.CIRC_EINVAL


def test_empty_and_degenerate_sizes_are_rejected():
    """Empty inputs (batch 0, no blocks) and block sizes outside 1..512 come back as
    CIRC_EINVAL / size 0, never as a launch."""
    assert B.circ_fc_workspace_bytes(2, 2, 8, 0) == 0
    assert B.circ_fc_workspace_bytes(0, 2, 8, 4) == 0
    assert B.circ_fc_workspace_bytes(2, 2, 0, 4) == 0
    assert B.circ_fc_workspace_bytes(2, 2, 3, 4) > 0
    f = B.lib().circ_fc_forward
    assert f(A, A + (1 << 28), None, A + (2 << 28), 2, 2, 8, 0, 0, A + (3 << 28), 1 << 30, None) == B.CIRC_EINVAL
    assert f(A, A + (1 << 28), None, A + (2 << 28), 2, 2, 0, 4, 0, A + (3 << 28), 1 << 30, None) == B.CIRC_EINVAL


def test_precompute_argument_errors():
    f = B.lib().circ_precompute_spectra
    assert f(None, 1, 2, 2, 8, A, None) == B.CIRC_EINVAL
    assert f(A, 1, 2, 2, 600, A + (1 << 20), None) == B.CIRC_EINVAL
    assert f(A, 0, 2, 2, 8, A + (1 << 20), None) == B.CIRC_EINVAL
    assert f(A, 1, 2, 2, 8, A, None) == B.CIRC_EINVAL         # output aliases input


def test_floor_helper_rejects_out_of_range_pieces():
    """The measurement helper library checks every piece index against the region sizes on the
    host and launches nothing when one does not fit."""
    path = os.path.join(os.path.dirname(B.LIB_PATH), "libcirc_floor.so")
    if not os.path.exists(path):
        pytest.skip("libcirc_floor.so not built")
    FL = ctypes.CDLL(path)
    FL.circ_floor_stream.restype = ctypes.c_int
    FL.circ_floor_stream.argtypes = [ctypes.c_void_p, ctypes.c_size_t] * 3 + [ctypes.c_int] * 2 + \
                                    [ctypes.c_size_t] * 3 + [ctypes.c_int] * 3 + [ctypes.c_void_p]
    a = 0x1000   # never dereferenced: every call below is rejected before a launch
    mb = 1 << 20
    assert FL.circ_floor_stream(a, 64 * mb, a, 64 * mb, a, 64 * mb, 1024, 512, 256 << 10, 16, 16, 0, 0, 0, None) == -1
    assert FL.circ_floor_stream(a, mb - 16, a, mb, a, mb, 256, 512, 131072, 32768, 4096, 4, 2, 16, None) == -1
    assert FL.circ_floor_stream(a, mb, a, mb - 16, a, mb, 256, 512, 131072, 32768, 4096, 4, 2, 16, None) == -1
    assert FL.circ_floor_stream(a, mb, a, mb, a, mb - 16, 256, 512, 131072, 32768, 4096, 4, 2, 16, None) == -1
    assert FL.circ_floor_stream(a, mb, a, mb, a, mb, 256, 512, 131072, 32768, 4100, 4, 2, 16, None) == -1   # not a multiple of 16
    assert FL.circ_floor_stream(None, mb, a, mb, a, mb, 256, 512, 16, 16, 16, 0, 0, 0, None) == -1
    assert FL.circ_floor_empty(0, 512, None) == -1 and FL.circ_floor_empty(256, 2048, None) == -1


"""GPU parity: the HIP path through the C ABI against the float64 dense oracle.

Gate: max_e |gpu_e - oracle_e| / max_e |oracle_e| <= 1e-4 per output tensor (fp32 path).
The value expected from fp32 rounding is ~1e-6, so a tighter bound TIGHT is asserted too:
an error between the two would pass the gate but point at a defect (e.g. twiddle precision).
"""
import numpy as np
import pytest
import torch

from oracle import circ_oracle as O
from paper_1708_08917_amd import binding as B
from paper_1708_08917_amd import synth
from tests import gpu_helpers as G

pytestmark = pytest.mark.gpu

GATE = 1e-4
TIGHT = 2e-5
RNG = np.random.default_rng(1708)


def check(got, ref, what=""):
    err = O.max_norm_rel_err(got, ref)
    print(f"[parity] {what} max-norm rel err = {err:.3e}", flush=True)
    assert np.all(np.isfinite(got)), what
    assert err <= GATE, (what, err)
    assert err <= TIGHT, (what, err, "passes the gate but is far above fp32 rounding")
    return err


def rand_fc(p, q, k, batch, bias=True):
    w = (RNG.standard_normal((p, q, k)) / np.sqrt(q * k)).astype(np.float32)
    x = RNG.uniform(-1, 1, (batch, q * k)).astype(np.float32)
    b = (0.1 * RNG.standard_normal(p * k)).astype(np.float32) if bias else None
    return w, x, b


# ---- every supported block size, ragged p / q / batch (tiles with tails) ------------------
@pytest.mark.parametrize("k", [2, 4, 8, 16, 32, 64, 128, 256, 512])
def test_fc_forward_all_block_sizes(k):
    p, q, batch = 3, 5, 7
    w, x, b = rand_fc(p, q, k, batch)
    check(G.gpu_fc_forward(w, x, b, relu=True), O.fc_forward(w, x, b, relu=True), f"fc fwd k={k}")
    check(G.gpu_fc_forward(w, x), O.fc_forward(w, x), f"fc fwd k={k} no epilogue")


@pytest.mark.parametrize("p,q,k,batch", [
    (1, 1, 8, 1), (1, 1, 64, 1), (2, 1, 16, 2), (1, 3, 16, 33), (37, 41, 16, 35), (33, 2, 64, 70),
    (5, 67, 32, 3), (64, 64, 16, 1), (40, 24, 64, 100), (3, 3, 128, 129), (2, 2, 256, 65),
    # more than 8 tiles of output block rows: the unfused FFT -> contraction -> IFFT route
    (72, 3, 64, 5), (70, 2, 128, 34), (130, 2, 32, 3), (66, 1, 256, 2), (65, 1, 512, 3),
    # fused route with ragged tiles: p not a multiple of 8, odd batch, q not a multiple of the chunk
    (9, 33, 64, 3), (7, 17, 128, 5), (5, 9, 256, 1), (3, 5, 512, 2), (17, 65, 32, 1), (64, 64, 64, 2),
    # fused route, two packed batch pairs per workgroup (taken when >= 256 such tiles exist)
    (64, 3, 64, 130), (33, 5, 128, 207), (17, 2, 256, 341), (60, 70, 64, 133),
])
def test_fc_forward_shapes(p, q, k, batch):
    w, x, b = rand_fc(p, q, k, batch)
    check(G.gpu_fc_forward(w, x, b, relu=False), O.fc_forward(w, x, b), f"fc fwd {p}x{q} k={k} B={batch}")


# ---- one or two input vectors: the streaming matrix-vector kernel, every block size, more
# input blocks than one chunk holds (chunk = min(4096/k, 128) blocks)
@pytest.mark.parametrize("k,q", [(4, 3), (4, 130), (8, 129), (16, 64), (16, 131), (32, 129), (64, 65), (128, 33), (256, 17), (512, 9)])
@pytest.mark.parametrize("batch", [1, 2])
def test_fc_forward_one_or_two_vectors(k, q, batch):
    p = 5
    w, x, b = rand_fc(p, q, k, batch)
    check(G.gpu_fc_forward(w, x, b, relu=True), O.fc_forward(w, x, b, relu=True), f"gemv k={k} q={q} B={batch}")
    check(G.gpu_fc_forward(w, x), O.fc_forward(w, x), f"gemv k={k} q={q} B={batch} no epilogue")


# ---- batch <= 2 on few block rows with long rows: two launches, the input blocks split over
# several workgroups per block row (split counts 2..16, ragged last split, several chunks per split)
@pytest.mark.parametrize("p,q,k", [(5, 72, 128), (3, 40, 256), (2, 130, 64), (3, 600, 16), (4, 17, 512), (32, 72, 128),
                                   (1, 300, 32), (7, 1100, 8)])
@pytest.mark.parametrize("batch", [1, 2])
def test_fc_one_or_two_vectors_split(p, q, k, batch):
    w, x, b = rand_fc(p, q, k, batch)
    check(G.gpu_fc_forward(w, x, b, relu=True), O.fc_forward(w, x, b, relu=True), f"split gemv {p}x{q} k={k} B={batch}")
    # backward-data of the transposed layer takes the same route
    wt, _, _ = rand_fc(q, p, k, batch, bias=False)
    dy = RNG.uniform(-1, 1, (batch, q * k)).astype(np.float32)
    xt = RNG.uniform(-1, 1, (batch, p * k)).astype(np.float32)
    dx, dw = G.gpu_fc_backward(wt, xt, dy)
    check(dx, O.fc_backward_dx(wt, dy), f"split gemv dx {q}x{p} k={k} B={batch}")
    check(dw, O.fc_backward_dw(xt, dy, k), f"split gemv dw {q}x{p} k={k} B={batch}")


def test_fc_forward_bias_only_and_relu_only():
    w, x, b = rand_fc(4, 4, 16, 9)
    check(G.gpu_fc_forward(w, x, None, relu=True), O.fc_forward(w, x, None, relu=True), "relu only")
    check(G.gpu_fc_forward(w, x, b, relu=False), O.fc_forward(w, x, b, relu=False), "bias only")


def test_shift_direction_on_gpu():
    k = 16
    w = np.zeros((1, 1, k), np.float32); w[0, 0, 1] = 1
    x = np.arange(1, k + 1, dtype=np.float32).reshape(1, k)
    y = G.gpu_fc_forward(w, x)
    np.testing.assert_allclose(y[0], np.roll(x[0], 1), atol=1e-5)


def test_exact_integers_on_gpu():
    p, q, k, batch = 5, 6, 32, 9
    w = synth.small_integers(3, 0, (p, q, k)); x = synth.small_integers(3, 1, (batch, q * k))
    ref = O.fc_forward(w, x)
    y = G.gpu_fc_forward(w, x)
    np.testing.assert_array_equal(np.round(y), ref)
    assert np.max(np.abs(y - ref)) < 1e-5 * np.max(np.abs(ref))


def test_deterministic():
    w, x, b = rand_fc(8, 8, 64, 40)
    y1 = G.gpu_fc_forward(w, x, b, True); y2 = G.gpu_fc_forward(w, x, b, True)
    np.testing.assert_array_equal(y1, y2)
    dy = RNG.uniform(-1, 1, (40, 8 * 64)).astype(np.float32)
    a = G.gpu_fc_backward(w, x, dy); c = G.gpu_fc_backward(w, x, dy)
    np.testing.assert_array_equal(a[0], c[0]); np.testing.assert_array_equal(a[1], c[1])


# ---- backward ------------------------------------------------------------------------------
# backward-data runs as a forward pass on the transposed grid: batch <= 2 -> streaming kernel,
# 32 <= k <= 256 and small -> fused kernel (one or two packed pairs per workgroup), else unfused
@pytest.mark.parametrize("p,q,k,batch", [(1, 1, 8, 1), (3, 5, 16, 7), (5, 3, 64, 33), (2, 2, 256, 10), (33, 34, 4, 70),
                                         (4, 6, 128, 67), (2, 3, 512, 5), (7, 9, 32, 2), (17, 64, 64, 130), (3, 70, 64, 5),
                                         (64, 64, 64, 64)])
def test_fc_backward_shapes(p, q, k, batch):
    w, x, _ = rand_fc(p, q, k, batch, bias=False)
    dy = RNG.uniform(-1, 1, (batch, p * k)).astype(np.float32)
    dx, dw = G.gpu_fc_backward(w, x, dy)
    check(dx, O.fc_backward_dx(w, dy), f"dx {p}x{q} k={k} B={batch}")
    check(dw, O.fc_backward_dw(x, dy, k), f"dw {p}x{q} k={k} B={batch}")
    dx_only, none = G.gpu_fc_backward(w, x, dy, need_dw=False)
    assert none is None
    np.testing.assert_array_equal(dx_only, dx)
    none, dw_only = G.gpu_fc_backward(w, x, dy, need_dx=False)
    np.testing.assert_array_equal(dw_only, dw)


# ---- unfused route with large batches (k too small or too large for the fused kernel): ragged
# tails of the 32x32 GEMM tiles in m, n and k; sampled block rows against the oracle
@pytest.mark.parametrize("p,q,k,batch", [(40, 3, 512, 200), (40, 3, 512, 100), (20, 2, 512, 150), (40, 5, 16, 8000),
                                         (70, 33, 16, 4100), (3, 2, 8, 9000)])
def test_fc_forward_unfused_large_batch(p, q, k, batch):
    w, x, b = rand_fc(p, q, k, batch)
    y = G.gpu_fc_forward(w, x, b, relu=True)
    rows = sorted(RNG.choice(p, min(p, 6), replace=False).tolist())
    y_s = np.concatenate([y[:, i * k:(i + 1) * k] for i in rows], axis=1)
    check(y_s, O.fc_forward(w, x, b, True, block_rows=rows), f"unfused fwd {p}x{q} k={k} B={batch}")


# ---- backward-weights on the LDS-tiled GEMM (taken when q <= 64, p > 32 and enough 64x64 tiles
# exist): ragged tails in m, n and k, a reduction slice shorter than one k-slab, split-K slices
# with a tail, the tile shared by the DC and Nyquist bins; the last two shapes take the
# one-wave-per-tile GEMM with split-K
@pytest.mark.parametrize("p,q,k,batch", [(40, 40, 512, 300), (40, 3, 512, 130), (70, 33, 16, 5000), (64, 64, 64, 700),
                                         (40, 70, 16, 5000), (70, 3, 8, 3000)])
def test_fc_backward_tiled_gemm(p, q, k, batch):
    w, x, _ = rand_fc(p, q, k, batch, bias=False)
    dy = RNG.uniform(-1, 1, (batch, p * k)).astype(np.float32)
    dx, dw = G.gpu_fc_backward(w, x, dy)
    cols = sorted(RNG.choice(q, min(q, 4), replace=False).tolist())
    pairs = [(int(i), int(j)) for i, j in zip(RNG.integers(0, p, 24), RNG.integers(0, q, 24))]
    dx_s = np.concatenate([dx[:, j * k:(j + 1) * k] for j in cols], axis=1)
    check(dx_s, O.fc_backward_dx(w, dy, block_cols=cols), f"tiled gemm dx {p}x{q} k={k} B={batch}")
    check(np.stack([dw[i, j] for (i, j) in pairs]), O.fc_backward_dw(x, dy, k, pairs=pairs), f"tiled gemm dw {p}x{q} k={k} B={batch}")
    # dw alone transforms dy itself (with dx it reuses the spectrum made for backward-data)
    none, dw_only = G.gpu_fc_backward(w, x, dy, need_dx=False)
    assert none is None
    np.testing.assert_array_equal(dw_only, dw)


# ---- CONV ----------------------------------------------------------------------------------
@pytest.mark.parametrize("N,p,q,k,H,W,r,pad", [(1, 1, 1, 4, 5, 5, 3, 1), (2, 2, 3, 8, 6, 7, 3, 1), (3, 5, 2, 16, 9, 4, 3, 0),
                                               (2, 1, 2, 64, 7, 7, 1, 0), (1, 2, 2, 32, 8, 8, 5, 2), (2, 4, 4, 64, 14, 14, 3, 1)])
def test_conv_forward_shapes(N, p, q, k, H, W, r, pad):
    _conv_case(N, p, q, k, H, W, r, pad)


# ---- fused CONV kernel (k = 64, 3x3, q in {1,2,3,4,6,8}, p <= 16): odd image counts, ragged tiles
# in both directions, every padding, every row-group count; rows that are a multiple of 4 input
# and 2 output pixels (aligned vector loads and paired stores) and rows that are not (13 x 13,
# 7 x 7, 14 x 14: element-wise loads and stores)
@pytest.mark.parametrize("N,p,q,H,W,pad", [(1, 1, 1, 5, 8, 1), (3, 4, 4, 9, 12, 1), (2, 5, 2, 13, 8, 0), (5, 9, 1, 7, 32, 2),
                                           (2, 16, 4, 8, 8, 1), (4, 3, 2, 28, 28, 1), (1, 2, 4, 3, 4, 0), (2, 4, 4, 33, 4, 2),
                                           (3, 2, 2, 10, 20, 1), (2, 4, 4, 16, 16, 0), (1, 1, 1, 5, 5, 1), (3, 4, 4, 9, 11, 1),
                                           (2, 5, 2, 13, 6, 0), (3, 6, 6, 13, 13, 1), (2, 3, 3, 8, 8, 1), (2, 2, 8, 7, 7, 1),
                                           (1, 8, 6, 14, 14, 1), (2, 4, 3, 13, 13, 2), (1, 1, 1, 4, 3, 1), (2, 2, 1, 5, 17, 0),
                                           (1, 3, 8, 6, 31, 1), (1, 1, 1, 3, 3, 0), (2, 2, 2, 20, 2, 1), (3, 1, 2, 1, 9, 1)])
def test_conv_forward_fused_shapes(N, p, q, H, W, pad):
    _conv_case(N, p, q, 64, H, W, 3, pad)


def _conv_case(N, p, q, k, H, W, r, pad):
    w = (RNG.standard_normal((r, r, p, q, k)) * np.sqrt(2.0 / (r * r * q * k))).astype(np.float32)
    x = RNG.uniform(-1, 1, (N, q * k, H, W)).astype(np.float32)
    b = (0.1 * RNG.standard_normal(p * k)).astype(np.float32)
    check(G.gpu_conv_forward(w, x, None, False, pad), O.conv_forward(w, x, pad=pad), f"conv {N},{p}x{q},k={k},{H}x{W},r={r}")
    check(G.gpu_conv_forward(w, x, b, True, pad), O.conv_forward(w, x, b, True, pad), "conv bias+relu")


# ---- CONV backward and the bias gradient ----------------------------------------------------
@pytest.mark.parametrize("N,p,q,k,H,W,r,pad", [(1, 1, 1, 4, 5, 5, 3, 1), (2, 2, 3, 8, 6, 7, 3, 1), (3, 5, 2, 16, 9, 4, 3, 0),
                                               (2, 1, 2, 64, 7, 7, 1, 0), (1, 2, 2, 32, 8, 8, 5, 2), (2, 4, 4, 64, 14, 14, 3, 1),
                                               (3, 3, 5, 2, 11, 6, 3, 2), (5, 2, 2, 8, 40, 40, 3, 1)])
def test_conv_backward_shapes(N, p, q, k, H, W, r, pad):
    w = (RNG.standard_normal((r, r, p, q, k)) * np.sqrt(2.0 / (r * r * q * k))).astype(np.float32)
    x = RNG.uniform(-1, 1, (N, q * k, H, W)).astype(np.float32)
    Ho, Wo = H + 2 * pad - r + 1, W + 2 * pad - r + 1
    dy = RNG.uniform(-1, 1, (N, p * k, Ho, Wo)).astype(np.float32)
    dx, dw = G.gpu_conv_backward(w, x, dy, pad)
    check(dx, O.conv_backward_dx(w, dy, H, W, pad), f"conv dx {N},{p}x{q},k={k},{H}x{W},r={r},pad={pad}")
    check(dw, O.conv_backward_dw(x, dy, k, r, pad), f"conv dw {N},{p}x{q},k={k},{H}x{W},r={r},pad={pad}")
    dx_only, none = G.gpu_conv_backward(w, x, dy, pad, need_dw=False)
    assert none is None
    np.testing.assert_array_equal(dx_only, dx)
    none, dw_only = G.gpu_conv_backward(w, x, dy, pad, need_dx=False)
    np.testing.assert_array_equal(dw_only, dw)
    a = G.gpu_conv_backward(w, x, dy, pad)                       # deterministic
    np.testing.assert_array_equal(a[0], dx); np.testing.assert_array_equal(a[1], dw)


# backward-data on the fused forward kernel (k = 64, 3x3; the p x q grid is transposed, so it needs
# p in {1, 2, 3, 4, 6, 8} and q <= 16): odd image counts, ragged tiles, every padding, aligned and
# unaligned row lengths; the shapes that do not qualify take the unfused route
@pytest.mark.parametrize("N,p,q,H,W,pad", [(1, 1, 1, 5, 8, 1), (3, 4, 4, 9, 12, 1), (2, 2, 5, 13, 8, 0), (5, 1, 9, 7, 32, 2),
                                           (2, 4, 16, 8, 8, 1), (4, 2, 3, 28, 28, 1), (1, 4, 2, 3, 6, 0), (2, 4, 4, 33, 4, 2),
                                           (3, 2, 2, 10, 20, 1), (2, 3, 4, 16, 16, 1), (1, 1, 1, 5, 5, 1), (2, 5, 2, 13, 6, 0),
                                           (3, 6, 6, 13, 13, 1), (2, 8, 2, 7, 7, 1), (1, 6, 8, 14, 14, 1), (2, 3, 4, 13, 13, 0),
                                           (1, 1, 1, 4, 3, 1), (2, 8, 3, 6, 31, 2), (1, 1, 1, 3, 3, 0), (2, 2, 2, 20, 2, 1), (3, 2, 1, 1, 9, 1)])
def test_conv_backward_fused_shapes(N, p, q, H, W, pad):
    k, r = 64, 3
    w = (RNG.standard_normal((r, r, p, q, k)) * np.sqrt(2.0 / (r * r * q * k))).astype(np.float32)
    x = RNG.uniform(-1, 1, (N, q * k, H, W)).astype(np.float32)
    Ho, Wo = H + 2 * pad - r + 1, W + 2 * pad - r + 1
    dy = RNG.uniform(-1, 1, (N, p * k, Ho, Wo)).astype(np.float32)
    dx, dw = G.gpu_conv_backward(w, x, dy, pad)
    check(dx, O.conv_backward_dx(w, dy, H, W, pad), f"conv dx fused {N},{p}x{q},{H}x{W},pad={pad}")
    check(dw, O.conv_backward_dw(x, dy, k, r, pad), f"conv dw {N},{p}x{q},{H}x{W},pad={pad}")
    dx_only, _ = G.gpu_conv_backward(w, x, dy, pad, need_dw=False)
    np.testing.assert_array_equal(dx_only, dx)


@pytest.mark.parametrize("seed", [0, 1])
def test_cfg4_conv_backward(seed):
    """Full size on the GPU; dx against the oracle on three images (images are independent),
    dw through the bilinear identity <dw, w> = <dy, y> = <dx, x> and the oracle on a reduced
    batch (first 4 images) run separately."""
    c = synth.CFG4
    w, x = synth.conv_inputs(c, seed)
    dy = synth.conv_upstream_grad(c, seed)
    dx, dw = G.gpu_conv_backward(w, x, dy, c.pad)
    for n in (0, c.N // 2, c.N - 1):
        check(dx[n:n + 1], O.conv_backward_dx(w, dy[n:n + 1], c.H, c.W, c.pad), f"cfg4 dx seed {seed} image {n}")
    y = G.gpu_conv_forward(w, x, None, False, c.pad)
    s = np.sum(dy.astype(np.float64) * y)
    assert abs(np.sum(dx.astype(np.float64) * x) - s) <= 1e-4 * abs(s) + 1e-2
    assert abs(np.sum(dw.astype(np.float64) * w) - s) <= 1e-4 * abs(s) + 1e-2
    _, dw4 = G.gpu_conv_backward(w, x[:4], dy[:4], c.pad, need_dx=False)
    check(dw4, O.conv_backward_dw(x[:4], dy[:4], c.k, c.r, c.pad), f"cfg4 dw seed {seed} (4 images)")


@pytest.mark.parametrize("shape", [(1, 8), (7, 130), (1024, 4096), (33, 65), (3, 4, 5, 6), (32, 256, 28, 28), (2, 3, 1, 1)])
def test_bias_grad(shape):
    dy = RNG.uniform(-1, 1, shape).astype(np.float32)
    db = G.gpu_bias_grad(dy)
    check(db, O.bias_grad(dy), f"bias grad {shape}")
    np.testing.assert_array_equal(G.gpu_bias_grad(dy), db)


# ---- seeded sweep over random valid shapes: every entry point, every dispatch path that small
# shapes reach (streaming kernel, fused kernels with one or several chunks, unfused route,
# fused and unfused CONV), ragged everywhere
# ---- gradient step on the cached spectra -------------------------------------------------------
def _step_size(w, dw):
    """A step that changes the weights by about half their size, so that both terms of
    w - lr*dw carry weight in the comparison."""
    return float(0.5 * np.max(np.abs(w)) / max(np.max(np.abs(dw)), 1e-30))


@pytest.mark.parametrize("k", [2, 4, 8, 16, 32, 64, 128, 256, 512])
def test_export_weights_roundtrip(k):
    for n_grids, p, q in ((1, 3, 5), (9, 2, 3)):
        w = RNG.standard_normal((n_grids, p, q, k)).astype(np.float32)
        wh = B.circ_precompute_spectra(G.dev(w))
        check(B.circ_export_weights(wh, n_grids, p, q, k).cpu().numpy(), w, f"export k={k} grids={n_grids}")


@pytest.mark.parametrize("p,q,k,batch", [(1, 1, 8, 1), (3, 5, 16, 7), (5, 3, 64, 33), (2, 2, 256, 10), (33, 34, 4, 70),
                                         (4, 6, 128, 2), (2, 3, 512, 5), (7, 9, 2, 3), (17, 64, 64, 130), (64, 64, 64, 64),
                                         (40, 33, 32, 700), (70, 33, 16, 5000), (3, 70, 64, 1)])
def test_fc_sgd_step_shapes(p, q, k, batch):
    """Two steps in a row on the blob against two oracle steps on the block vectors; then every
    operand order of the updated blob is exercised: backward-data (returned by the second step
    from the once-updated weights), forward at this batch and forward of a single vector."""
    w, x1, b = rand_fc(p, q, k, batch)
    x2 = RNG.uniform(-1, 1, (batch, q * k)).astype(np.float32)
    dy1 = RNG.uniform(-1, 1, (batch, p * k)).astype(np.float32)
    dy2 = RNG.uniform(-1, 1, (batch, p * k)).astype(np.float32)
    lr = _step_size(w, O.fc_backward_dw(x1, dy1, k))
    w1 = O.fc_sgd_step(w, x1, dy1, lr)
    w2 = O.fc_sgd_step(w1, x2, dy2, lr)
    got, wh, dxs = G.gpu_fc_sgd_steps(w, [(x1, dy1), (x2, dy2)], lr, need_dx=True)
    what = f"{p}x{q} k={k} B={batch}"
    check(got, w2, "sgd w " + what)
    check(dxs[0], O.fc_backward_dx(w, dy1), "sgd dx before the step " + what)
    check(dxs[1], O.fc_backward_dx(w1, dy2), "sgd dx after one step " + what)
    y = B.circ_fc_forward(wh, G.dev(x1), G.dev(b), None, p, q, k, epilogue=B.EPI_BIAS).cpu().numpy()
    check(y, O.fc_forward(w2, x1, b), "forward after two steps " + what)
    y1 = B.circ_fc_forward(wh, G.dev(x1[:1]), None, None, p, q, k).cpu().numpy()
    check(y1, O.fc_forward(w2, x1[:1]), "single-vector forward after two steps " + what)
    dx1, _ = B.circ_fc_backward(wh, None, G.dev(dy1[:1]), p, q, k, need_dw=False)
    check(dx1.cpu().numpy(), O.fc_backward_dx(w2, dy1[:1]), "single-vector dx after two steps " + what)


def test_fc_sgd_step_zero_step_and_agreement_with_time_domain():
    p, q, k, batch = 5, 7, 64, 40
    w, x, _ = rand_fc(p, q, k, batch, bias=False)
    dy = RNG.uniform(-1, 1, (batch, p * k)).astype(np.float32)
    wh = B.circ_precompute_spectra(G.dev(w))
    before = wh.clone()
    B.circ_fc_sgd_step(wh, G.dev(x), G.dev(dy), 0.0, p, q, k)
    # lr = 0: every stored value unchanged (the sign of a zero may flip; bytes between the
    # sections are never written and may hold anything)
    a, b = wh.view(torch.float32), before.view(torch.float32)
    assert bool(((a == b) | (a.isnan() & b.isnan())).all())
    # the step in the frequency domain against: gradient to the time domain, step there, precompute again
    lr = 0.01
    B.circ_fc_sgd_step(wh, G.dev(x), G.dev(dy), lr, p, q, k)
    _, dw = B.circ_fc_backward(before, G.dev(x), G.dev(dy), p, q, k, need_dx=False)
    wh_t = B.circ_precompute_spectra((G.dev(w) - lr * dw).contiguous())
    xt = G.dev(x)
    ya = B.circ_fc_forward(wh, xt, None, None, p, q, k).cpu().numpy()
    yb = B.circ_fc_forward(wh_t, xt, None, None, p, q, k).cpu().numpy()
    check(ya, yb, "frequency-domain step vs time-domain step")


@pytest.mark.parametrize("N,p,q,k,H,W,r,pad", [(1, 1, 1, 4, 5, 5, 3, 1), (2, 2, 3, 8, 6, 7, 3, 1), (3, 5, 2, 16, 9, 4, 3, 0),
                                               (2, 3, 2, 32, 5, 6, 1, 0), (3, 4, 4, 64, 9, 12, 3, 1), (2, 2, 5, 64, 13, 8, 3, 0),
                                               (2, 1, 2, 128, 6, 6, 5, 2), (40, 2, 2, 64, 14, 14, 3, 1)])
def test_conv_sgd_step_shapes(N, p, q, k, H, W, r, pad):
    w = (RNG.standard_normal((r, r, p, q, k)) / np.sqrt(r * r * q * k)).astype(np.float32)
    Ho, Wo = H + 2 * pad - r + 1, W + 2 * pad - r + 1
    mk = lambda: (RNG.uniform(-1, 1, (N, q * k, H, W)).astype(np.float32),
                  RNG.uniform(-1, 1, (N, p * k, Ho, Wo)).astype(np.float32))
    (x1, dy1), (x2, dy2) = mk(), mk()
    lr = _step_size(w, O.conv_backward_dw(x1, dy1, k, r, pad))
    w1 = O.conv_sgd_step(w, x1, dy1, lr, pad)
    w2 = O.conv_sgd_step(w1, x2, dy2, lr, pad)
    got, wh, dxs = G.gpu_conv_sgd_steps(w, [(x1, dy1), (x2, dy2)], lr, pad, need_dx=True)
    what = f"N={N} {p}x{q} k={k} {H}x{W} r={r} pad={pad}"
    check(got, w2, "conv sgd w " + what)
    check(dxs[1], O.conv_backward_dx(w1, dy2, H, W, pad), "conv sgd dx after one step " + what)
    y = B.circ_conv_forward(wh, G.dev(x1), None, None, p * k, r, 1, pad, k).cpu().numpy()
    check(y, O.conv_forward(w2, x1, None, False, pad), "conv forward after two steps " + what)


def test_conv_large_image():
    """A 224 x 224 image: many tiles of the fused kernel per image, and for the weight gradient
    many bands of rows per image (a band of 4 input blocks must fit the LDS budget) walked over by
    one workgroup.  Also with stride 2 (unfused route)."""
    N, p, q, k, H, W, r, pad = 2, 1, 1, 64, 224, 224, 3, 1
    w = (RNG.standard_normal((r, r, p, q, k)) / np.sqrt(r * r * q * k)).astype(np.float32)
    x = RNG.uniform(-1, 1, (N, q * k, H, W)).astype(np.float32)
    for stride in (1, 2):
        Ho = (H + 2 * pad - r) // stride + 1
        dy = RNG.uniform(-1, 1, (N, p * k, Ho, Ho)).astype(np.float32)
        check(G.gpu_conv_forward(w, x, None, False, pad, stride), O.conv_forward(w, x, None, False, pad, stride),
              f"224x224 fwd stride {stride}")
        dx, dw = G.gpu_conv_backward(w, x, dy, pad, stride=stride)
        check(dx, O.conv_backward_dx(w, dy, H, W, pad, stride), f"224x224 dx stride {stride}")
        check(dw, O.conv_backward_dw(x, dy, k, r, pad, stride), f"224x224 dw stride {stride}")


def test_fc_forward_largest_batch():
    """The largest batch the ABI accepts (65535 * 16 vectors): activations of 4.29 GB each (byte
    offsets up to 2^32), spectra of 5.4e8 elements and 4.31 GB each (byte offsets beyond 2^32).
    Inputs are made on the GPU; rows at the start, around the 2^31-byte mark, in the middle and at
    the end are checked against the oracle."""
    p, q, k, batch = 2, 2, 512, 65535 * 16
    w = (RNG.standard_normal((p, q, k)) / np.sqrt(q * k)).astype(np.float32)
    b = (0.1 * RNG.standard_normal(p * k)).astype(np.float32)
    gen = torch.Generator(device=G.DEV)
    gen.manual_seed(1708)
    x = torch.rand(batch, q * k, device=G.DEV, generator=gen) * 2 - 1
    wh = B.circ_precompute_spectra(G.dev(w))
    y = B.circ_fc_forward(wh, x, G.dev(b), None, p, q, k, epilogue=B.EPI_BIAS | B.EPI_RELU)
    torch.cuda.synchronize()
    row_bytes = q * k * 4
    marks = [0, (1 << 31) // row_bytes - 4, batch // 2 + 5, 3 * (batch // 4), batch - 8]
    for r0 in marks:
        xs = x[r0:r0 + 8].cpu().numpy()
        check(y[r0:r0 + 8].cpu().numpy(), O.fc_forward(w, xs, b, True), f"largest batch, rows {r0}..{r0 + 7}")
    # backward at the same size: dx on the same rows against the oracle; dw (a sum over all
    # 1,048,560 rows) through the bilinear identity <dw, w> = <dy, W x> with the forward result
    dy = torch.rand(batch, p * k, device=G.DEV, generator=gen) * 2 - 1
    dx, dw = B.circ_fc_backward(wh, x, dy, p, q, k)
    y_lin = B.circ_fc_forward(wh, x, None, y, p, q, k)
    torch.cuda.synchronize()
    for r0 in marks:
        check(dx[r0:r0 + 8].cpu().numpy(), O.fc_backward_dx(w, dy[r0:r0 + 8].cpu().numpy()), f"largest batch dx, rows {r0}..{r0 + 7}")
    lhs = float((dw.double() * torch.from_numpy(w).to(G.DEV).double()).sum())
    rhs = float((dy.double() * y_lin.double()).sum())
    print(f"[identity] <dw, w> = {lhs:.6e}, <dy, y> = {rhs:.6e}", flush=True)
    assert abs(lhs - rhs) <= 1e-4 * abs(rhs) + 1e-2
    del x, y, dy, dx
    torch.cuda.empty_cache()


# ---- half-width storage (16-bit values in memory, fp32 arithmetic) ---------------------------
# Four 16-bit roundings lie between the inputs and an output (spectra of the weights, spectra of
# the inputs, output spectra, the output itself), each at most 2^-11 (fp16) or 2^-8 (bfloat16)
# relative; the gate is their sum, the value expected from independent roundings about a quarter.
HALF_GATE = {torch.float16: 4 * 2.0 ** -11, torch.bfloat16: 4 * 2.0 ** -8}
HALF_DTYPES = [torch.float16, torch.bfloat16]


def check_half(got, ref, what, dtype):
    err = O.max_norm_rel_err(got, ref)
    print(f"[parity {dtype}] {what} max-norm rel err = {err:.3e}", flush=True)
    assert np.all(np.isfinite(got)), what
    assert err <= HALF_GATE[dtype], (what, err)
    return err


def to_half(x, dtype):
    """fp32 array -> (device tensor of `dtype`, the same values back in fp32): the inputs are
    16-bit values on both sides of the comparison."""
    t = torch.from_numpy(x).to(dtype)
    return t.to(G.DEV), t.float().numpy()


def gpu_fc_forward_half(w, xt, bias, relu):
    p, q, k = w.shape
    wh = B.circ_precompute_spectra_f16(G.dev(w), dtype=xt.dtype)
    y = B.circ_fc_forward_f16(wh, xt, G.dev(bias), None, p, q, k, G.epi_flags(bias, relu))
    assert y.dtype == xt.dtype
    return y.float().cpu().numpy()


@pytest.mark.parametrize("dtype", HALF_DTYPES)
@pytest.mark.parametrize("p,q,k,batch", [(1, 1, 8, 1), (3, 5, 16, 7), (5, 3, 64, 33), (2, 4, 256, 10), (33, 34, 8, 70),
                                         (4, 6, 128, 67), (2, 3, 512, 5), (7, 9, 32, 2), (17, 64, 64, 130), (70, 12, 64, 300),
                                         (64, 64, 64, 64), (65, 8, 32, 129), (3, 72, 128, 40), (2, 130, 16, 9),
                                         (4, 72, 128, 1), (32, 32, 128, 2), (125, 512, 8, 1), (3, 5, 16, 2), (2, 3, 512, 1),
                                         (64, 64, 16, 1), (5, 40, 256, 2)])
def test_fc_forward_half_shapes(p, q, k, batch, dtype):
    w, x, b = rand_fc(p, q, k, batch)
    xt, xr = to_half(x, dtype)
    what = f"{p}x{q} k={k} B={batch}"
    check_half(gpu_fc_forward_half(w, xt, b, True), O.fc_forward(w, xr, b, True), "bias+relu " + what, dtype)
    check_half(gpu_fc_forward_half(w, xt, None, False), O.fc_forward(w, xr), "plain " + what, dtype)


def test_fc_forward_bf16_large_inputs():
    """Inputs far outside the fp16 range (|x| k up to 4e7) are fine in bfloat16."""
    p, q, k, batch = 3, 4, 64, 9
    w, x, _ = rand_fc(p, q, k, batch, bias=False)
    xt, xr = to_half(x * 6.0e5, torch.bfloat16)
    check_half(gpu_fc_forward_half(w, xt, None, False), O.fc_forward(w, xr), "large inputs", torch.bfloat16)


@pytest.mark.parametrize("dtype", HALF_DTYPES)
@pytest.mark.parametrize("cfg", ["cfg2", "cfg3_l1", "cfg5"])
def test_fc_forward_half_configs(cfg, dtype):
    c = {"cfg2": synth.CFG2, "cfg3_l1": synth.CFG3_L1, "cfg5": synth.CFG5}[cfg]
    w, x, b = synth.fc_inputs(c, 0)
    xt, xr = to_half(x, dtype)
    got = gpu_fc_forward_half(w, xt, b, c.relu)
    rows = sorted(set(int(i) for i in np.linspace(0, c.p - 1, 4)))   # sampled output block rows, all batch elements
    ref = O.fc_forward(w, xr, b, c.relu, block_rows=rows)
    sel = np.concatenate([np.arange(i * c.k, (i + 1) * c.k) for i in rows])
    check_half(got[:, sel], ref, f"{cfg} block rows {rows}", dtype)


# Backward with 16-bit storage.  dx passes the same four roundings as y; dw (fp32 out, fp32
# spectrum) only the two of the operand spectra.  Batches that are not multiples of 4 take the
# element-wise staging of the contraction, long batches cut the reduction into slices.
@pytest.mark.parametrize("dtype", HALF_DTYPES)
@pytest.mark.parametrize("p,q,k,batch", [(1, 1, 8, 1), (3, 5, 16, 7), (5, 3, 64, 33), (2, 4, 256, 10), (33, 34, 8, 70),
                                         (4, 6, 128, 68), (2, 3, 512, 5), (7, 9, 32, 2), (2, 3, 16, 700), (3, 2, 8, 1025),
                                         (70, 130, 8, 260), (64, 64, 64, 64), (65, 8, 32, 129), (3, 72, 128, 40),
                                         (72, 4, 128, 1), (32, 32, 128, 2), (512, 125, 8, 1), (3, 5, 16, 2), (40, 5, 256, 2)])
def test_fc_backward_half_shapes(p, q, k, batch, dtype):
    w, x, _ = rand_fc(p, q, k, batch, bias=False)
    dy = RNG.uniform(-1, 1, (batch, p * k)).astype(np.float32)
    xt, xr = to_half(x, dtype)
    dyt, dyr = to_half(dy, dtype)
    wh = B.circ_precompute_spectra_f16(G.dev(w), dtype=dtype)
    what = f"{p}x{q} k={k} B={batch}"
    dx, dw = B.circ_fc_backward_f16(wh, xt, dyt, p, q, k)
    assert dx.dtype == dtype and dw.dtype == torch.float32
    check_half(dx.float().cpu().numpy(), O.fc_backward_dx(w, dyr), "dx " + what, dtype)
    check_half(dw.cpu().numpy(), O.fc_backward_dw(xr, dyr, k), "dw " + what, dtype)
    # one result at a time: dw is the same computation; dx then reads the spectra of dy in the
    # other order, in which a row shares its packed transform with a different partner row, so
    # the 16-bit spectra can differ in their last bit
    dx1, _ = B.circ_fc_backward_f16(wh, None, dyt, p, q, k, need_dw=False)
    _, dw1 = B.circ_fc_backward_f16(wh, xt, dyt, p, q, k, need_dx=False)
    assert torch.equal(dw1, dw)
    check_half(dx1.float().cpu().numpy(), O.fc_backward_dx(w, dyr), "dx alone " + what, dtype)


@pytest.mark.parametrize("dtype", HALF_DTYPES)
def test_cfg5_backward_half(dtype):
    c = synth.CFG5
    w, x, _ = synth.fc_inputs(c, 0)
    dy = synth.fc_upstream_grad(c, 0)
    xt, xr = to_half(x, dtype)
    dyt, dyr = to_half(dy, dtype)
    wh = B.circ_precompute_spectra_f16(G.dev(w), dtype=dtype)
    dx, dw = B.circ_fc_backward_f16(wh, xt, dyt, c.p, c.q, c.k)
    dx, dw = dx.float().cpu().numpy(), dw.cpu().numpy()
    pick = np.random.default_rng(5)
    cols = sorted(pick.choice(c.q, 4, replace=False).tolist())
    pairs = [(int(i), int(j)) for i, j in zip(pick.integers(0, c.p, 64), pick.integers(0, c.q, 64))]
    k = c.k
    dx_s = np.concatenate([dx[:, j * k:(j + 1) * k] for j in cols], axis=1)
    dw_s = np.stack([dw[i, j] for (i, j) in pairs])
    check_half(dx_s, O.fc_backward_dx(w, dyr, block_cols=cols), "cfg5 dx", dtype)
    check_half(dw_s, O.fc_backward_dw(xr, dyr, k, pairs=pairs), "cfg5 dw", dtype)


# CONV forward with 16-bit activations: the weight spectra stay fp32, so only x (rounded before the
# comparison, on both sides) and y are 16-bit: one rounding of the output, gated like the others.
@pytest.mark.parametrize("dtype", HALF_DTYPES)
@pytest.mark.parametrize("N,p,q,k,H,W,r,pad,stride", [
    (2, 4, 4, 64, 28, 28, 3, 1, 1), (3, 2, 1, 64, 14, 12, 3, 1, 1), (1, 1, 2, 64, 8, 8, 3, 0, 1), (5, 16, 4, 64, 6, 8, 3, 1, 1),
    (2, 2, 3, 8, 9, 8, 3, 1, 2), (3, 1, 2, 16, 7, 7, 3, 0, 1), (2, 2, 2, 32, 8, 8, 2, 0, 2), (2, 3, 1, 8, 9, 10, 5, 2, 1),
    (2, 1, 1, 128, 5, 7, 1, 0, 1), (2, 2, 2, 64, 13, 12, 3, 1, 3), (1, 1, 1, 512, 3, 4, 3, 1, 1), (2, 2, 2, 256, 6, 5, 3, 1, 1),
    (3, 6, 6, 64, 13, 13, 3, 1, 1), (2, 3, 8, 64, 7, 7, 3, 1, 1), (1, 2, 3, 64, 14, 14, 3, 0, 1)])
def test_conv_forward_half(N, p, q, k, H, W, r, pad, stride, dtype):
    w = (RNG.standard_normal((r, r, p, q, k)) / np.sqrt(r * r * q * k)).astype(np.float32)
    x = RNG.uniform(-1, 1, (N, q * k, H, W)).astype(np.float32)
    b = (0.1 * RNG.standard_normal(p * k)).astype(np.float32)
    xt, xr = to_half(x, dtype)
    wh = B.circ_precompute_spectra(G.dev(w))
    what = f"N={N} {p}x{q} k={k} {H}x{W} r={r} pad={pad} stride={stride}"
    y = B.circ_conv_forward_f16(wh, xt, G.dev(b), None, p * k, r, stride, pad, k, B.EPI_BIAS | B.EPI_RELU)
    assert y.dtype == dtype
    check_half(y.float().cpu().numpy(), O.conv_forward(w, xr, b, True, pad, stride), "conv fwd bias+relu " + what, dtype)
    y = B.circ_conv_forward_f16(wh, xt, None, None, p * k, r, stride, pad, k)
    check_half(y.float().cpu().numpy(), O.conv_forward(w, xr, None, False, pad, stride), "conv fwd " + what, dtype)
    # backward on the same 16-bit activations: dx rounded to 16 bits, dw in fp32
    Ho, Wo = (H + 2 * pad - r) // stride + 1, (W + 2 * pad - r) // stride + 1
    dy = RNG.uniform(-1, 1, (N, p * k, Ho, Wo)).astype(np.float32)
    dyt, dyr = to_half(dy, dtype)
    dx, dw = B.circ_conv_backward_f16(wh, xt, dyt, q * k, H, W, r, stride, pad, k)
    assert dx.dtype == dtype and dw.dtype == torch.float32
    check_half(dx.float().cpu().numpy(), O.conv_backward_dx(w, dyr, H, W, pad, stride), "conv dx " + what, dtype)
    check(dw.cpu().numpy(), O.conv_backward_dw(xr, dyr, k, r, pad, stride), "conv dw (fp32 from 16-bit inputs) " + what)


@pytest.mark.parametrize("dtype", HALF_DTYPES)
def test_cfg4_forward_half(dtype):
    c = synth.CFG4
    w, x = synth.conv_inputs(c)
    xt, xr = to_half(x, dtype)
    wh = B.circ_precompute_spectra(G.dev(w))
    y = B.circ_conv_forward_f16(wh, xt, None, None, c.C_out, c.r, 1, c.pad, c.k).float().cpu().numpy()
    for n in (0, c.N - 1):
        check_half(y[n:n + 1], O.conv_forward(w, xr[n:n + 1], pad=c.pad), f"cfg4 image {n}", dtype)


# ---- stride > 1 and even filter sizes (Eq. 6 is the stride-1 case) ---------------------------
@pytest.mark.parametrize("N,p,q,k,H,W,r,pad,stride", [
    (2, 2, 3, 8, 9, 8, 3, 1, 2), (3, 1, 2, 16, 7, 7, 3, 0, 2), (2, 4, 4, 64, 28, 28, 3, 1, 2), (2, 2, 2, 64, 13, 12, 3, 1, 3),
    (1, 3, 2, 4, 11, 9, 5, 2, 2), (2, 2, 2, 32, 8, 8, 2, 0, 2), (2, 3, 1, 8, 9, 10, 4, 1, 2), (3, 2, 2, 16, 6, 6, 2, 1, 1),
    (2, 2, 3, 12, 10, 7, 3, 1, 2), (33, 2, 2, 64, 14, 14, 3, 1, 2), (2, 2, 2, 8, 5, 300, 3, 1, 2), (2, 1, 1, 8, 6, 1, 1, 0, 1),
    (1, 1, 2, 8, 9, 9, 7, 3, 1), (2, 2, 1, 4, 10, 10, 7, 6, 3), (1, 1, 1, 2, 1, 1, 1, 0, 1), (2, 5, 6, 4, 3, 2000, 3, 1, 1)])
def test_conv_strided_and_even_filters(N, p, q, k, H, W, r, pad, stride):
    w = (RNG.standard_normal((r, r, p, q, k)) / np.sqrt(r * r * q * k)).astype(np.float32)
    x = RNG.uniform(-1, 1, (N, q * k, H, W)).astype(np.float32)
    b = (0.1 * RNG.standard_normal(p * k)).astype(np.float32)
    Ho, Wo = (H + 2 * pad - r) // stride + 1, (W + 2 * pad - r) // stride + 1
    dy = RNG.uniform(-1, 1, (N, p * k, Ho, Wo)).astype(np.float32)
    what = f"N={N} {p}x{q} k={k} {H}x{W} r={r} pad={pad} stride={stride}"
    y = G.gpu_conv_forward(w, x, b, True, pad, stride)
    assert y.shape == (N, p * k, Ho, Wo)
    check(y, O.conv_forward(w, x, b, True, pad, stride), "conv fwd " + what)
    dx, dw = G.gpu_conv_backward(w, x, dy, pad, stride=stride)
    check(dx, O.conv_backward_dx(w, dy, H, W, pad, stride), "conv dx " + what)
    check(dw, O.conv_backward_dw(x, dy, k, r, pad, stride), "conv dw " + what)
    lr = _step_size(w, O.conv_backward_dw(x, dy, k, r, pad, stride))
    got, _, _ = G.gpu_conv_sgd_steps(w, [(x, dy)], lr, pad, stride=stride)
    check(got, O.conv_sgd_step(w, x, dy, lr, pad, stride), "conv sgd w " + what)


# ---- block sizes that are not powers of two (direct transforms around the same contraction) ----
@pytest.mark.parametrize("k", [1, 3, 5, 6, 7, 9, 12, 15, 20, 24, 40, 48, 80, 96, 100, 125, 160, 192, 200, 225, 250, 320,
                               384, 400, 509, 511])
@pytest.mark.parametrize("batch", [1, 2, 33])
def test_fc_general_block_sizes(k, batch):
    """Sizes 3 * 2^a, 5 * 2^a and 25 * 2^a (multiples of 4) run the mixed-radix transforms, the rest
    the transforms by their definition."""
    p, q = (3, 5) if k < 200 else (2, 3)
    w, x, b = rand_fc(p, q, k, batch)
    what = f"{p}x{q} k={k} B={batch}"
    check(G.gpu_fc_forward(w, x, b, True), O.fc_forward(w, x, b, True), "fwd bias+relu " + what)
    dy = RNG.uniform(-1, 1, (batch, p * k)).astype(np.float32)
    dx, dw = G.gpu_fc_backward(w, x, dy)
    check(dx, O.fc_backward_dx(w, dy), "dx " + what)
    check(dw, O.fc_backward_dw(x, dy, k), "dw " + what)
    lr = _step_size(w, O.fc_backward_dw(x, dy, k))
    got, wh, _ = G.gpu_fc_sgd_steps(w, [(x, dy)], lr)
    w1 = O.fc_sgd_step(w, x, dy, lr)
    check(got, w1, "sgd w " + what)
    y = B.circ_fc_forward(wh, G.dev(x), None, None, p, q, k).cpu().numpy()
    check(y, O.fc_forward(w1, x), "forward after the step " + what)


@pytest.mark.parametrize("p,q,k,batch", [(40, 37, 96, 300), (70, 33, 24, 3000), (33, 70, 3, 600), (10, 10, 100, 64),
                                         (64, 64, 1, 50)])
def test_fc_general_block_sizes_larger(p, q, k, batch):
    """Several row tiles of the direct transforms, ragged GEMM tiles, split reduction for dw."""
    w, x, b = rand_fc(p, q, k, batch)
    what = f"{p}x{q} k={k} B={batch}"
    check(G.gpu_fc_forward(w, x, b, False), O.fc_forward(w, x, b, False), "fwd " + what)
    dy = RNG.uniform(-1, 1, (batch, p * k)).astype(np.float32)
    dx, dw = G.gpu_fc_backward(w, x, dy)
    check(dx, O.fc_backward_dx(w, dy), "dx " + what)
    check(dw, O.fc_backward_dw(x, dy, k), "dw " + what)


@pytest.mark.parametrize("N,p,q,k,H,W,r,pad", [(2, 2, 3, 3, 6, 7, 3, 1), (3, 1, 2, 6, 5, 5, 3, 0), (2, 3, 2, 24, 9, 4, 1, 0),
                                               (2, 4, 4, 96, 13, 13, 3, 1), (2, 2, 2, 192, 13, 13, 3, 1),
                                               (3, 2, 2, 1, 8, 8, 5, 2), (33, 2, 3, 12, 14, 14, 3, 1),
                                               (5, 2, 1, 80, 7, 9, 3, 1), (3, 1, 2, 100, 6, 6, 3, 1)])
def test_conv_general_block_sizes(N, p, q, k, H, W, r, pad):
    """Includes the 384-channel 13 x 13 layers of an AlexNet-style network as 4 x 4 blocks of 96
    and 2 x 2 blocks of 192."""
    w = (RNG.standard_normal((r, r, p, q, k)) / np.sqrt(r * r * q * k)).astype(np.float32)
    x = RNG.uniform(-1, 1, (N, q * k, H, W)).astype(np.float32)
    b = (0.1 * RNG.standard_normal(p * k)).astype(np.float32)
    Ho, Wo = H + 2 * pad - r + 1, W + 2 * pad - r + 1
    dy = RNG.uniform(-1, 1, (N, p * k, Ho, Wo)).astype(np.float32)
    what = f"N={N} {p}x{q} k={k} {H}x{W} r={r} pad={pad}"
    check(G.gpu_conv_forward(w, x, b, True, pad), O.conv_forward(w, x, b, True, pad), "conv fwd " + what)
    dx, dw = G.gpu_conv_backward(w, x, dy, pad)
    check(dx, O.conv_backward_dx(w, dy, H, W, pad), "conv dx " + what)
    check(dw, O.conv_backward_dw(x, dy, k, r, pad), "conv dw " + what)
    lr = _step_size(w, O.conv_backward_dw(x, dy, k, r, pad))
    got, _, _ = G.gpu_conv_sgd_steps(w, [(x, dy)], lr, pad)
    check(got, O.conv_sgd_step(w, x, dy, lr, pad), "conv sgd w " + what)


def test_fig1_example_on_gpu():
    """The 6 x 3 matrix of Fig. 1: p = 2, q = 1, k = 3, six stored parameters."""
    w = np.arange(1, 7, dtype=np.float32).reshape(2, 1, 3)
    x = np.array([[1.0, -2.0, 0.5]], dtype=np.float32)
    got = G.gpu_fc_forward(w, x)
    check(got, O.expand_block_circulant(w) @ x[0], "Fig. 1 shape")


@pytest.mark.parametrize("seed", [11, 12, 13, 14])
def test_random_shapes_sweep(seed):
    rng = np.random.default_rng(seed)
    for case in range(60):
        kind = rng.choice(["fc", "fcb", "conv", "convb"], p=[0.4, 0.25, 0.2, 0.15])
        if kind in ("fc", "fcb"):
            # seed 14 draws block sizes that are not powers of two
            k = int(rng.choice([2, 4, 8, 16, 32, 64, 128, 256, 512] if seed != 14 else [1, 3, 6, 10, 20, 48, 96, 120, 200, 500]))
            p, q = int(rng.integers(1, 80)), int(rng.integers(1, 80))
            batch = int(rng.choice([1, 2, 3, 5, 8, 17, 33, 64, 100, 130, 257]))
            while (p * k) * (q * k) * batch > 2e8 and (p > 1 or q > 1):     # keep the dense oracle quick
                p, q = max(1, p // 2), max(1, q // 2)
            while (p * k) * (q * k) * batch > 2e8 and batch > 1:
                batch = max(1, batch // 2)
            w = (rng.standard_normal((p, q, k)) / np.sqrt(q * k)).astype(np.float32)
            x = rng.uniform(-1, 1, (batch, q * k)).astype(np.float32)
            what = f"sweep {seed}/{case} {kind} {p}x{q} k={k} B={batch}"
            print(what, flush=True)
            if kind == "fc":
                b = (0.1 * rng.standard_normal(p * k)).astype(np.float32) if rng.integers(0, 2) else None
                relu = bool(rng.integers(0, 2))
                check(G.gpu_fc_forward(w, x, b, relu), O.fc_forward(w, x, b, relu), what)
            else:
                dy = rng.uniform(-1, 1, (batch, p * k)).astype(np.float32)
                dx, dw = G.gpu_fc_backward(w, x, dy)
                check(dx, O.fc_backward_dx(w, dy), what + " dx")
                check(dw, O.fc_backward_dw(x, dy, k), what + " dw")
        else:
            k = int(rng.choice([2, 4, 8, 16, 32, 64] if seed != 14 else [1, 3, 6, 10, 24, 48]))
            p, q = int(rng.integers(1, 6)), int(rng.integers(1, 6))
            r = int(rng.choice([1, 3, 3, 3, 5]))
            pad = int(rng.integers(0, r))
            H, W = int(rng.integers(1, 18)), int(rng.integers(1, 18))
            if rng.integers(0, 2):
                W = max(4, (W // 4) * 4)                 # rows that are a multiple of 4 pixels take the aligned loads of the fused kernel
            while W + 2 * pad < r:
                W += 4
            while H + 2 * pad < r:
                H += 1
            N = int(rng.integers(1, 6))
            w = (rng.standard_normal((r, r, p, q, k)) * np.sqrt(2.0 / (r * r * q * k))).astype(np.float32)
            x = rng.uniform(-1, 1, (N, q * k, H, W)).astype(np.float32)
            what = f"sweep {seed}/{case} {kind} N={N} {p}x{q} k={k} {H}x{W} r={r} pad={pad}"
            print(what, flush=True)
            if kind == "conv":
                b = (0.1 * rng.standard_normal(p * k)).astype(np.float32)
                check(G.gpu_conv_forward(w, x, b, True, pad), O.conv_forward(w, x, b, True, pad), what)
            else:
                Ho, Wo = H + 2 * pad - r + 1, W + 2 * pad - r + 1
                dy = rng.uniform(-1, 1, (N, p * k, Ho, Wo)).astype(np.float32)
                dx, dw = G.gpu_conv_backward(w, x, dy, pad)
                check(dx, O.conv_backward_dx(w, dy, H, W, pad), what + " dx")
                check(dw, O.conv_backward_dw(x, dy, k, r, pad), what + " dw")
                check(G.gpu_bias_grad(dy), O.bias_grad(dy), what + " db")


# ---- the five layer configurations ---------------------------------------------------------
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_cfg1(seed):
    w, x, b = synth.fc_inputs(synth.CFG1, seed)
    check(G.gpu_fc_forward(w, x), O.fc_forward(w, x), f"cfg1 seed {seed}")


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_cfg2(seed):
    w, x, b = synth.fc_inputs(synth.CFG2, seed)
    check(G.gpu_fc_forward(w, x, b, True), O.fc_forward(w, x, b, True), f"cfg2 seed {seed}")


def test_cfg2_graph_over_streams_matches_eager():
    """The launch configuration of the benchmark: independent cfg2 steps recorded into one HIP graph,
    round-robin over several streams, replayed several times with eager work in between.  Every
    output of every replay must equal the eager result bit for bit (and the oracle on one pair)."""
    import ctypes
    c = synth.CFG2
    w, x0, b = synth.fc_inputs(c)
    wh = B.circ_precompute_spectra(G.dev(w))
    bd = G.dev(b)
    nsteps, nstreams = 40, 16                    # the stream count the benchmark uses
    gen = torch.Generator(device=G.DEV); gen.manual_seed(7)
    xs = torch.empty(nsteps, c.batch, c.n_in, device=G.DEV).uniform_(-1, 1, generator=gen)
    xs[0].copy_(torch.from_numpy(x0))
    epi = B.EPI_BIAS | B.EPI_RELU
    eager = torch.stack([B.circ_fc_forward(wh, xs[i], bd, None, c.p, c.q, c.k, epi) for i in range(nsteps)])
    torch.cuda.synchronize()
    check(eager[0].cpu().numpy(), O.fc_forward(w, x0, b, True), "cfg2 eager pair 0")
    ys = torch.zeros_like(eager)
    main = torch.cuda.Stream()
    side = [torch.cuda.Stream() for _ in range(nstreams - 1)]
    lanes = [main] + side
    wss = [torch.empty(max(1, B.circ_fc_workspace_bytes(c.p, c.q, c.k, c.batch)), dtype=torch.uint8, device=G.DEV)
           for _ in lanes]
    fn = B.lib().circ_fc_forward
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=main):
        for s_ in side:
            s_.wait_stream(main)
        for i in range(nsteps):
            ln = i % nstreams
            st = fn(ctypes.c_void_p(wh.data_ptr()), ctypes.c_void_p(xs[i].data_ptr()), ctypes.c_void_p(bd.data_ptr()),
                    ctypes.c_void_p(ys[i].data_ptr()), c.p, c.q, c.k, c.batch, epi, ctypes.c_void_p(wss[ln].data_ptr()),
                    wss[ln].numel(), ctypes.c_void_p(lanes[ln].cuda_stream))
            assert st == 0
        for s_ in side:
            main.wait_stream(s_)
    for rep in range(3):
        ys.fill_(-1.0)                         # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(ys, eager), f"replay {rep} differs from the eager result"


@pytest.mark.parametrize("p,q,k,batch", [(70, 40, 256, 901), (70, 41, 256, 900), (9, 9, 256, 1001), (72, 33, 128, 1001), (130, 3, 64, 17000), (130, 70, 32, 1950),
                                           (70, 40, 100, 651), (70, 40, 81, 651)])
def test_fc_unfused_route_with_long_ragged_runs_of_rows(p, q, k, batch):
    """More than 8 tiles of output block rows keep these layers off the fused kernel: q * batch rows go
    through the streaming row transform (at least 256 tiles of 4096 / k column pairs, the last tile
    ragged), p * batch rows through the inverse transform (its streaming form when their number is
    even, the tile-per-workgroup form when it is odd: 9 * 1001).  The last two cases take the split
    contraction with a mixed-radix block size and with an odd one (no real last bin).  Forward on sampled
    block rows, backward on sampled block columns and (i, j) pairs."""
    w, x, b = rand_fc(p, q, k, batch)
    assert (q * batch) % (2 * (4096 // k)) != 0 and q * batch >= 256 * 2 * (4096 // k)
    what = f"{p}x{q} k={k} B={batch}"
    rows = [0, p // 2, p - 1]
    got = G.gpu_fc_forward(w, x, b, True)
    sel = np.concatenate([np.arange(i * k, (i + 1) * k) for i in rows])
    check(got[:, sel], O.fc_forward(w, x, b, True, block_rows=rows), "fwd " + what)
    dy = RNG.uniform(-1, 1, (batch, p * k)).astype(np.float32)
    dx, dw = G.gpu_fc_backward(w, x, dy)
    cols = [0, q - 1]
    csel = np.concatenate([np.arange(j * k, (j + 1) * k) for j in cols])
    check(dx[:, csel], O.fc_backward_dx(w, dy, block_cols=cols), "dx " + what)
    pairs = [(0, 0), (p - 1, q - 1), (p // 2, q // 3)]
    ref = O.fc_backward_dw(x, dy, k, pairs=pairs)
    check(np.stack([dw[i, j] for i, j in pairs]), ref, "dw " + what)


def test_fc_split_gemm_route_with_fewer_columns_than_a_wave():
    """257 frequency slices of a 40 x 16 grid of 512-point blocks are enough tiles for the split
    contraction even at batch 5: every wave of a tile then has columns past the batch (computed on
    copies of the last one, not stored), three of the four waves nothing but such columns."""
    p, q, k, batch = 40, 16, 512, 5
    w, x, b = rand_fc(p, q, k, batch)
    rows = [0, 17, p - 1]
    sel = np.concatenate([np.arange(i * k, (i + 1) * k) for i in rows])
    got = G.gpu_fc_forward(w, x, b, True)
    check(got[:, sel], O.fc_forward(w, x, b, True, block_rows=rows), "split contraction, batch 5, k=512")


def test_fc_split_gemm_route_keeps_fp32_accuracy_per_batch_row():
    """Layers with at least 256 tiles of 64 x 128 outputs per frequency take the contraction that
    splits every fp32 operand into three bfloat16 terms.  Each value is split on its own, so batch
    rows of small magnitude next to rows eight decades larger must come out with the same relative
    accuracy as any others: the error of every output row is measured against that row's own
    largest value (forward; backward-data takes the same kernel with the transposed weights).  Rows
    2i and 2i + 1 share a scale: the row transforms carry two rows as one complex sequence, and
    their separation is exact only relative to the larger of the two."""
    p, q, k, batch = 34, 20, 256, 260
    w, x, b = rand_fc(p, q, k, batch, bias=False)
    scale = np.repeat(10.0 ** RNG.uniform(-4, 4, batch // 2), 2).astype(np.float32)
    x = x * scale[:, None]
    w = w * (10.0 ** RNG.uniform(-2, 2, (p, q, 1))).astype(np.float32)
    rows = [0, p // 2, p - 1]
    sel = np.concatenate([np.arange(i * k, (i + 1) * k) for i in rows])
    got = G.gpu_fc_forward(w, x)[:, sel]
    ref = O.fc_forward(w, x, block_rows=rows)
    assert np.all(np.isfinite(got))
    err = np.max(np.abs(got - ref), axis=1) / np.max(np.abs(ref), axis=1)
    print(f"[parity] split contraction, per-row rel err: max {err.max():.3e} median {np.median(err):.3e}", flush=True)
    assert err.max() <= TIGHT, err.max()
    dy = (RNG.uniform(-1, 1, (batch, p * k)) * scale[:, None]).astype(np.float32)
    cols = [0, q - 1]
    csel = np.concatenate([np.arange(j * k, (j + 1) * k) for j in cols])
    dx = G.gpu_fc_backward(w, x, dy)[0][:, csel]
    dref = O.fc_backward_dx(w, dy, block_cols=cols)
    derr = np.max(np.abs(dx - dref), axis=1) / np.max(np.abs(dref), axis=1)
    print(f"[parity] split contraction, backward-data per-row rel err: max {derr.max():.3e}", flush=True)
    assert derr.max() <= TIGHT, derr.max()


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_cfg3_two_stacked_layers(seed):
    w1, x, b1 = synth.fc_inputs(synth.CFG3_L1, seed)
    w2, _, b2 = synth.fc_inputs(synth.CFG3_L2, seed, second_layer=True)
    h_ref = O.fc_forward(w1, x, b1, True)
    y_ref = O.fc_forward(w2, h_ref, b2, True)
    c1, c2 = synth.CFG3_L1, synth.CFG3_L2
    wh1 = B.circ_precompute_spectra(G.dev(w1)); wh2 = B.circ_precompute_spectra(G.dev(w2))
    h = B.circ_fc_forward(wh1, G.dev(x), G.dev(b1), None, c1.p, c1.q, c1.k, B.EPI_BIAS | B.EPI_RELU)
    y = B.circ_fc_forward(wh2, h, G.dev(b2), None, c2.p, c2.q, c2.k, B.EPI_BIAS | B.EPI_RELU)
    torch.cuda.synchronize()
    check(h.cpu().numpy(), h_ref, f"cfg3 layer 1 seed {seed}")
    check(y.cpu().numpy(), y_ref, f"cfg3 layer 2 seed {seed}")


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_cfg4_conv(seed):
    c = synth.CFG4
    w, x = synth.conv_inputs(c, seed)
    y = G.gpu_conv_forward(w, x, None, False, c.pad)
    # every image of the batch (the kernel packs images in pairs; each image is independent)
    check(y, O.conv_forward(w, x, pad=c.pad), f"cfg4 seed {seed}, all {c.N} images")


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_cfg5_forward_backward(seed):
    """Full size on the GPU; the oracle is evaluated on sampled block rows / columns / pairs
    (all batch elements), which the dense definition allows one by one."""
    c = synth.CFG5
    w, x, _ = synth.fc_inputs(c, seed)
    dy = synth.fc_upstream_grad(c, seed)
    wh = B.circ_precompute_spectra(G.dev(w))
    xd, dyd = G.dev(x), G.dev(dy)
    y = B.circ_fc_forward(wh, xd, None, None, c.p, c.q, c.k).cpu().numpy()
    dx, dw = B.circ_fc_backward(wh, xd, dyd, c.p, c.q, c.k)
    dx, dw = dx.cpu().numpy(), dw.cpu().numpy()
    pick = np.random.default_rng(seed)
    rows = sorted(pick.choice(c.p, 8, replace=False).tolist())
    cols = sorted(pick.choice(c.q, 8, replace=False).tolist())
    pairs = [(int(i), int(j)) for i, j in zip(pick.integers(0, c.p, 256), pick.integers(0, c.q, 256))]
    k = c.k
    y_s = np.concatenate([y[:, i * k:(i + 1) * k] for i in rows], axis=1)
    dx_s = np.concatenate([dx[:, j * k:(j + 1) * k] for j in cols], axis=1)
    dw_s = np.stack([dw[i, j] for (i, j) in pairs])
    check(y_s, O.fc_forward(w, x, block_rows=rows), f"cfg5 y seed {seed}")
    check(dx_s, O.fc_backward_dx(w, dy, block_cols=cols), f"cfg5 dx seed {seed}")
    check(dw_s, O.fc_backward_dw(x, dy, k, pairs=pairs), f"cfg5 dw seed {seed}")
    # bilinear identities hold at any size: <dy, y> = <dx, x> = <dw, w>
    s = np.sum(dy.astype(np.float64) * y)
    assert abs(np.sum(dx.astype(np.float64) * x) - s) <= 1e-4 * abs(s) + 1e-2
    assert abs(np.sum(dw.astype(np.float64) * w) - s) <= 1e-4 * abs(s) + 1e-2


# ---- max-pooling and chains of layers (single-image regime) ---------------------------------
@pytest.mark.parametrize("N,C,H,W,window,stride", [(1, 1, 4, 4, 2, 2), (2, 3, 7, 9, 2, 2), (1, 4, 8, 8, 3, 2), (3, 1, 5, 6, 3, 3),
                                                   (2, 2, 6, 6, 1, 1), (32, 256, 28, 28, 2, 2), (2, 96, 55, 55, 3, 2),
                                                   (1, 2, 300, 1, 1, 1), (1, 1, 1, 1, 1, 1), (2, 70000, 3, 3, 2, 1)])
def test_maxpool(N, C, H, W, window, stride):
    x = RNG.standard_normal((N, C, H, W)).astype(np.float32)
    y = B.circ_maxpool_forward(G.dev(x), window, stride)
    torch.cuda.synchronize()
    ref = O.maxpool_forward(x, window, stride)
    assert y.shape == ref.shape
    assert np.array_equal(y.cpu().numpy().astype(np.float64), ref)       # a maximum is exact


def _chain_inputs(rng, spec, batch):
    """spec: list of ("fc", p, q, k, bias, relu) / ("conv", C_in, C_out, H, W, r, stride, pad, k, bias, relu) /
    ("pool", C, H, W, window, stride).  Returns (oracle layers, device layers, keep-alive tensors, x)."""
    olayers, dlayers, keep = [], [], []
    for l in spec:
        if l[0] == "fc":
            _, p, q, k, bias, relu = l
            w = (rng.standard_normal((p, q, k)) / np.sqrt(q * k)).astype(np.float32)
            b = (0.1 * rng.standard_normal(p * k)).astype(np.float32) if bias else None
            wh = B.circ_precompute_spectra(G.dev(w)); bd = G.dev(b)
            keep += [wh, bd]
            olayers.append(dict(kind="fc", w=w, bias=b, relu=relu))
            dlayers.append(B.fc_layer(wh, bd, p, q, k, G.epi_flags(b, relu)))
        elif l[0] == "conv":
            _, Ci, Co, H, W, r, stride, pad, k, bias, relu = l
            w = (rng.standard_normal((r, r, Co // k, Ci // k, k)) * np.sqrt(2.0 / (r * r * Ci))).astype(np.float32)
            b = (0.1 * rng.standard_normal(Co)).astype(np.float32) if bias else None
            wh = B.circ_precompute_spectra(G.dev(w)); bd = G.dev(b)
            keep += [wh, bd]
            olayers.append(dict(kind="conv", w=w, bias=b, relu=relu, pad=pad, stride=stride))
            dlayers.append(B.conv_layer(wh, bd, Ci, Co, H, W, r, stride, pad, k, G.epi_flags(b, relu)))
        else:
            _, C, H, W, window, stride = l
            olayers.append(dict(kind="pool", window=window, stride=stride))
            dlayers.append(B.maxpool_layer(C, H, W, window, stride))
    first = spec[0]
    shape = (batch, first[2] * first[3]) if first[0] == "fc" else (batch, first[1], first[2], first[3]) if first[0] == "pool" \
        else (batch, first[1], first[3], first[4])
    x = rng.uniform(-1, 1, shape).astype(np.float32)
    return olayers, dlayers, keep, x


HEAD = [("fc", 32, 72, 128, True, True), ("fc", 32, 32, 128, True, True), ("fc", 125, 512, 8, True, False)]
CONVNET = [("conv", 64, 128, 14, 14, 3, 1, 1, 64, True, True), ("pool", 128, 14, 14, 2, 2),
           ("fc", 4, 98, 64, True, True), ("fc", 5, 128, 2, True, False)]
SMALLNET = [("conv", 8, 16, 12, 12, 3, 1, 1, 4, True, True), ("pool", 16, 12, 12, 2, 2), ("conv", 16, 16, 6, 6, 3, 1, 1, 8, False, False),
            ("pool", 16, 6, 6, 2, 2), ("fc", 4, 9, 16, True, True), ("fc", 5, 32, 2, True, False)]


@pytest.mark.parametrize("name,spec,batch", [("head 9216-4096-4096-1000", HEAD, 1), ("head 9216-4096-4096-1000", HEAD, 2),
                                             ("head 9216-4096-4096-1000", HEAD, 5), ("conv-pool-fc-fc", CONVNET, 1),
                                             ("conv-pool-fc-fc", CONVNET, 4), ("conv-pool-conv-pool-fc-fc", SMALLNET, 1),
                                             ("conv-pool-conv-pool-fc-fc", SMALLNET, 3)])
def test_chain_forward(name, spec, batch):
    rng = np.random.default_rng(41 + batch)
    olayers, dlayers, keep, x = _chain_inputs(rng, spec, batch)
    ref = O.chain_forward(olayers, x)
    y = torch.full(ref.shape, float("nan"), dtype=torch.float32, device=G.DEV)
    B.circ_chain_forward(dlayers, G.dev(x), y)
    torch.cuda.synchronize()
    check(y.cpu().numpy(), ref, f"chain {name} batch {batch}")
    # the chain is the single-layer entry points back to back: bit-identical to calling them one by one
    a = G.dev(x)
    for l, d in zip(spec, dlayers):
        if l[0] == "fc":
            a = B.circ_fc_forward(ctypes_tensor(keep, d.w_hat), a.reshape(batch, -1), ctypes_tensor(keep, d.bias), None, d.p, d.q, d.k, d.epilogue)
        elif l[0] == "conv":
            a = B.circ_conv_forward(ctypes_tensor(keep, d.w_hat), a, ctypes_tensor(keep, d.bias), None, d.C_out, d.r, d.stride, d.pad, d.k, d.epilogue)
        else:
            a = B.circ_maxpool_forward(a.reshape(batch, d.C_in, d.H, d.W), d.r, d.stride)
    torch.cuda.synchronize()
    assert torch.equal(a.reshape(y.shape), y)


@pytest.mark.parametrize("name,spec,batch", [("head 9216-4096-4096-1000", HEAD, 1), ("conv-pool-fc-fc", CONVNET, 1)])
def test_chain_recorded_in_a_graph_matches_eager(name, spec, batch):
    """A whole network for one input recorded into a HIP graph (the single-image serving loop):
    every replay, with eager work on the same buffers in between, reproduces the eager call bit for bit."""
    rng = np.random.default_rng(77)
    olayers, dlayers, keep, x = _chain_inputs(rng, spec, batch)
    ref = O.chain_forward(olayers, x)
    xd = G.dev(x)
    eager = torch.empty(ref.shape, dtype=torch.float32, device=G.DEV)
    B.circ_chain_forward(dlayers, xd, eager)
    torch.cuda.synchronize()
    check(eager.cpu().numpy(), ref, f"chain {name} eager")
    ws = torch.empty(B.circ_chain_workspace_bytes(dlayers, batch), dtype=torch.uint8, device=G.DEV)
    y = torch.zeros_like(eager)
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        B.circ_chain_forward(dlayers, xd, y, workspace=ws)
    for rep in range(3):
        y.fill_(-1.0)
        ws.fill_(0xFF)                         # the workspace carries nothing from one call to the next
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, eager), f"replay {rep} of {name} differs from the eager result"


def ctypes_tensor(keep, ptr):
    """The tensor in `keep` that starts at device address `ptr` (None for a NULL pointer)."""
    if not ptr:
        return None
    return next(t for t in keep if t is not None and t.data_ptr() == ptr)


def test_chain_rejects_ill_fitting_layers_and_short_workspace():
    rng = np.random.default_rng(5)
    _, dlayers, keep, x = _chain_inputs(rng, [("fc", 3, 4, 8, True, True), ("fc", 2, 3, 8, False, False)], 2)
    y = torch.empty(2, 16, device=G.DEV)
    B.circ_chain_forward(dlayers, G.dev(x), y)                        # fits
    bad = [dlayers[0], B.fc_layer(ctypes_tensor(keep, dlayers[1].w_hat), None, 2, 4, 8)]   # 24 outputs into 32 inputs
    assert B.circ_chain_workspace_bytes(bad, 2) == 0
    with pytest.raises(B.CircError) as e:
        B.circ_chain_forward(bad, G.dev(x), y, workspace=torch.empty(1 << 20, dtype=torch.uint8, device=G.DEV))
    assert e.value.status == B.CIRC_EINVAL
    with pytest.raises(B.CircError) as e:
        B.circ_chain_forward(dlayers, G.dev(x), y, workspace=torch.empty(256, dtype=torch.uint8, device=G.DEV))
    assert e.value.status == B.CIRC_EWORKSPACE
    with pytest.raises(B.CircError) as e:
        B.circ_maxpool_forward(G.dev(np.zeros((1, 1, 2, 2), np.float32)), 3, 1, y=torch.empty(1, 1, 1, 1, device=G.DEV))
    assert e.value.status == B.CIRC_EINVAL


# ---- error paths through the binding on the GPU machine ---------------------------------------
def test_errors_raise_through_binding():
    w, x, b = rand_fc(2, 2, 8, 2)
    wh = B.circ_precompute_spectra(G.dev(w))
    xd = G.dev(x)
    with pytest.raises(B.CircError) as e:
        B.circ_fc_forward(wh, xd, None, None, 2, 2, 8, B.EPI_BIAS)
    assert e.value.status == B.CIRC_EINVAL
    with pytest.raises(B.CircError) as e:
        B.circ_fc_forward(wh, xd, None, None, 2, 2, 8, 0, workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.status == B.CIRC_EWORKSPACE
    with pytest.raises(B.CircError) as e:
        B.circ_fc_forward(wh, xd, None, xd, 2, 2, 8, 0)
    assert e.value.status == B.CIRC_EINVAL

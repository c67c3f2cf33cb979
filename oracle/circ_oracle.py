"""CPU oracle for block-circulant layers (CirCNN, arXiv 1708.08917).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
HIP kernels are checked against.  Only tests, the smoke check and the
`cpu_baseline` leg of the benchmark may import it; the product path never does,
and this file imports nothing from the product package.

What it computes is the *definition*, in float64, with no FFT anywhere:
every k x k circulant block is written out as a dense matrix from its defining
vector and the layer is an ordinary dense matrix product (Sec. 3.1, Eq. 3;
Sec. 3.2, Eq. 6).  Because Eq. 3 and the circulant convolution theorem are
identities, the FFT route of Algorithms 1 and 2 must reproduce these numbers up
to rounding.  `numpy.matmul` is used as the matrix-product step.

Readings of the paper taken here (each also pinned by a CPU test):

* Orientation.  Sec. 3.1 calls w_ij the "first row" of W_ij and, in the same
  sentence, states W_ij x_j = IFFT(FFT(w_ij) o FFT(x_j)).  With rows that rotate
  to the right these two cannot both hold; the printed formula is kept:
  W_ij[a][b] = w_ij[(a - b) mod k], i.e. w_ij is the first *column* and
  W_ij x_j is the circular convolution of w_ij and x_j.
* Algorithm 2 has no batch index; gradients of the block vectors are summed
  over the batch, without a 1/B factor.
* CONV (Eq. 6, Eq. 7): for each spatial offset (dh, dw) the C_out x C_in
  channel-mixing matrix is block-circulant with k x k blocks; cross-correlation
  (no kernel flip), zero padding, stride 1.

Parity pins: all functions below are pinned (see tests/test_oracle_pins.py):
circulant definition, shift direction, DFT diagonalisation, brute-force
circular convolution, exact integers, k = 1 dense layer, bias and ReLU at k > 1 on a
matrix written entry by entry (also for the pre-expanded form), p = q = 1 library
circular convolution, finite differences and bilinear identities for the
gradients, library convolution and single-pixel response for CONV; the CONV
gradients and the bias gradient by finite differences, the library's own
convolution gradients, the bilinear identities and the r = 1 reduction to the
FC gradients; the gradient-descent steps by the library's own optimiser acting
on gathered dense weights, a closed form for k = 1 and the decrease of a
quadratic loss; max-pooling and chains of layers by the library's float64 pooling, dense
convolution and linear layers on weights written entry by entry, and a hand-worked window.
"""
from __future__ import annotations

import numpy as np


def circulant(w_vec: np.ndarray) -> np.ndarray:
    """Dense k x k circulant block from its defining vector (Sec. 3.1).

    C[a][b] = w[(a - b) mod k]: column 0 is w, each column is the previous one
    rotated down by one.
    """
    w_vec = np.asarray(w_vec, dtype=np.float64)
    k = w_vec.shape[0]
    a = np.arange(k).reshape(k, 1)
    b = np.arange(k).reshape(1, k)
    return w_vec[(a - b) % k]


def expand_block_circulant(w: np.ndarray) -> np.ndarray:
    """Dense (p*k) x (q*k) matrix W = [W_ij] from w[p][q][k] (Sec. 3.1, Eq. 3)."""
    w = np.asarray(w, dtype=np.float64)
    p, q, k = w.shape
    W = np.empty((p * k, q * k), dtype=np.float64)
    for i in range(p):
        for j in range(q):
            W[i * k:(i + 1) * k, j * k:(j + 1) * k] = circulant(w[i, j])
    return W


def fc_forward(w, x, bias=None, relu=False, block_rows=None) -> np.ndarray:
    """y = psi(W x + theta) for a batch (Eq. 1 with W from Eq. 3).

    w[p][q][k], x[B][q*k] -> y[B][p*k].  `block_rows` (a list of block-row
    indices i) restricts the result to the columns y[:, i*k:(i+1)*k] of those
    block rows, concatenated in the given order; the arithmetic per output is
    unchanged.
    """
    w = np.asarray(w, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64)
    p, q, k = w.shape
    rows = list(range(p)) if block_rows is None else list(block_rows)
    out = np.empty((x.shape[0], len(rows) * k), dtype=np.float64)
    for s, i in enumerate(rows):
        Wi = expand_block_circulant(w[i:i + 1])          # k x n : block row i of W
        a = np.matmul(x, Wi.T)
        if bias is not None:
            a = a + np.asarray(bias, dtype=np.float64)[i * k:(i + 1) * k]
        out[:, s * k:(s + 1) * k] = a
    if relu:
        out = np.maximum(out, 0.0)
    return out


def fc_forward_expanded(W, x, bias=None, relu=False) -> np.ndarray:
    """y = psi(W x + theta) (Eq. 1) on a matrix that has already been written out with
    expand_block_circulant: the same layer as fc_forward when the dense expansion of the blocks
    is done once and kept, the counterpart of keeping FFT(w_ij) instead of recomputing it.
    W[p*k][q*k], x[B][q*k] -> y[B][p*k]."""
    a = np.matmul(np.asarray(x, dtype=np.float64), np.asarray(W, dtype=np.float64).T)
    if bias is not None:
        a = a + np.asarray(bias, dtype=np.float64)
    return np.maximum(a, 0.0) if relu else a


def fc_backward_dx(w, dy, block_cols=None) -> np.ndarray:
    """dL/dx = W^T dL/da (Eq. 5).  dy[B][p*k] -> dx[B][q*k] (or the listed block columns)."""
    w = np.asarray(w, dtype=np.float64)
    dy = np.asarray(dy, dtype=np.float64)
    p, q, k = w.shape
    cols = list(range(q)) if block_cols is None else list(block_cols)
    out = np.empty((dy.shape[0], len(cols) * k), dtype=np.float64)
    for s, j in enumerate(cols):
        Wj = expand_block_circulant(w[:, j:j + 1])       # m x k : block column j of W
        out[:, s * k:(s + 1) * k] = np.matmul(dy, Wj)
    return out


def fc_backward_dw(x, dy, k, pairs=None) -> np.ndarray:
    """dL/dw_ij (Eq. 4), summed over the batch.

    The gradient of the dense matrix is G = dy^T x.  Since
    W_ij[a][b] = w_ij[(a - b) mod k], the chain rule collects every entry of
    block (i, j) that holds w_ij[t]:  dw_ij[t] = sum_a G_ij[a][(a - t) mod k].

    Returns dw[p][q][k], or dw[len(pairs)][k] for a list of (i, j) pairs.
    """
    x = np.asarray(x, dtype=np.float64)
    dy = np.asarray(dy, dtype=np.float64)
    q = x.shape[1] // k
    p = dy.shape[1] // k
    a = np.arange(k).reshape(k, 1)
    t = np.arange(k).reshape(1, k)
    col = (a - t) % k                                    # col[a][t] = (a - t) mod k

    def one(i, j):
        G = np.matmul(dy[:, i * k:(i + 1) * k].T, x[:, j * k:(j + 1) * k])   # k x k
        return G[a, col].sum(axis=0)

    if pairs is not None:
        return np.stack([one(i, j) for (i, j) in pairs])
    dw = np.empty((p, q, k), dtype=np.float64)
    for i in range(p):
        for j in range(q):
            dw[i, j] = one(i, j)
    return dw


def conv_out_size(n, r, pad, stride) -> int:
    """Output positions along one axis: the filter is placed every `stride` pixels as long as it
    fits the zero-padded input."""
    return (n + 2 * pad - r) // stride + 1


def conv_forward(w, x, bias=None, relu=False, pad=0, stride=1) -> np.ndarray:
    """Block-circulant CONV layer (Eq. 6 with the structure of Eq. 7; Eq. 6 itself is stride 1).

    w[r][r][p][q][k] (offset-major), x[N][C_in][H][W] ->
    y[N][C_out][(H + 2 pad - r) // stride + 1][(W + 2 pad - r) // stride + 1], with
    y[n, co, h, w] = sum_{dh, dw, ci} Wd[dh, dw][co, ci] * xpad[n, ci, h*stride + dh, w*stride + dw]
    where Wd[dh, dw] is the dense expansion of the p x q grid of that offset.
    """
    w = np.asarray(w, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64)
    r = w.shape[0]
    N, C_in, H, Wd_ = x.shape
    p, q, k = w.shape[2:]
    assert C_in == q * k
    C_out = p * k
    Ho, Wo = conv_out_size(H, r, pad, stride), conv_out_size(Wd_, r, pad, stride)
    xp = np.zeros((N, C_in, H + 2 * pad, Wd_ + 2 * pad), dtype=np.float64)
    xp[:, :, pad:pad + H, pad:pad + Wd_] = x
    y = np.zeros((N, C_out, Ho, Wo), dtype=np.float64)
    for dh in range(r):
        for dw in range(r):
            M = expand_block_circulant(w[dh, dw])        # C_out x C_in
            # the input pixel under tap (dh, dw) of every output position
            win = xp[:, :, dh:dh + (Ho - 1) * stride + 1:stride, dw:dw + (Wo - 1) * stride + 1:stride]
            # channel mixing at every pixel: y[n, :, h, w] += M @ win[n, :, h, w]
            y += np.matmul(M, win.reshape(N, C_in, Ho * Wo)).reshape(N, C_out, Ho, Wo)
    if bias is not None:
        y = y + np.asarray(bias, dtype=np.float64).reshape(1, C_out, 1, 1)
    if relu:
        y = np.maximum(y, 0.0)
    return y


def conv_backward_dx(w, dy, H, W, pad=0, stride=1) -> np.ndarray:
    """dL/dx of the block-circulant CONV layer (chain rule through Eq. 6; Sec. 3.2 notes that
    training of CONV layers follows the FC derivation).

    y[n, co, ho, wo] takes x[n, ci, ho*stride + dh - pad, wo*stride + dw - pad] with weight
    Wd[dh, dw][co, ci], so every (dh, dw) scatters Wd[dh, dw]^T dy[n, :, ho, wo] back to that
    input pixel; positions in the zero padding receive nothing.
    w[r][r][p][q][k], dy[N][C_out][Ho][Wo] -> dx[N][C_in][H][W].
    """
    w = np.asarray(w, dtype=np.float64)
    dy = np.asarray(dy, dtype=np.float64)
    r = w.shape[0]
    p, q, k = w.shape[2:]
    N, C_out, Ho, Wo = dy.shape
    assert C_out == p * k and Ho == conv_out_size(H, r, pad, stride) and Wo == conv_out_size(W, r, pad, stride)
    C_in = q * k
    dxp = np.zeros((N, C_in, H + 2 * pad, W + 2 * pad), dtype=np.float64)
    for dh in range(r):
        for dw in range(r):
            M = expand_block_circulant(w[dh, dw])        # C_out x C_in
            g = np.matmul(M.T, dy.reshape(N, C_out, Ho * Wo)).reshape(N, C_in, Ho, Wo)
            dxp[:, :, dh:dh + (Ho - 1) * stride + 1:stride, dw:dw + (Wo - 1) * stride + 1:stride] += g
    return dxp[:, :, pad:pad + H, pad:pad + W].copy()


def conv_backward_dw(x, dy, k, r, pad=0, stride=1) -> np.ndarray:
    """dL/dw of the block-circulant CONV layer, summed over images and pixels.

    For every offset the gradient of the dense channel-mixing matrix is
    G[dh, dw] = sum_{n, ho, wo} dy[n, :, ho, wo] xpad[n, :, ho*stride + dh, wo*stride + dw]^T, and, as for
    FC layers (Eq. 4), dw[dh][dw][i][j][t] collects the entries of block (i, j) that hold
    that weight: sum_a G_ij[a][(a - t) mod k].
    x[N][C_in][H][W], dy[N][C_out][Ho][Wo] -> dw[r][r][p][q][k].
    """
    x = np.asarray(x, dtype=np.float64)
    dy = np.asarray(dy, dtype=np.float64)
    N, C_in, H, W = x.shape
    _, C_out, Ho, Wo = dy.shape
    assert Ho == conv_out_size(H, r, pad, stride) and Wo == conv_out_size(W, r, pad, stride)
    p, q = C_out // k, C_in // k
    xp = np.zeros((N, C_in, H + 2 * pad, W + 2 * pad), dtype=np.float64)
    xp[:, :, pad:pad + H, pad:pad + W] = x
    a = np.arange(k).reshape(k, 1)
    t = np.arange(k).reshape(1, k)
    col = (a - t) % k
    dyf = dy.transpose(1, 0, 2, 3).reshape(C_out, N * Ho * Wo)
    dw = np.empty((r, r, p, q, k), dtype=np.float64)
    for dh in range(r):
        for dw_ in range(r):
            win = xp[:, :, dh:dh + (Ho - 1) * stride + 1:stride, dw_:dw_ + (Wo - 1) * stride + 1:stride]
            win = win.transpose(1, 0, 2, 3).reshape(C_in, N * Ho * Wo)
            G = np.matmul(dyf, win.T)                    # C_out x C_in
            for i in range(p):
                for j in range(q):
                    Gb = G[i * k:(i + 1) * k, j * k:(j + 1) * k]
                    dw[dh, dw_, i, j] = Gb[a, col].sum(axis=0)
    return dw


def maxpool_forward(x, window, stride) -> np.ndarray:
    """Max-pooling (the POOL layer of Sec. 2.1): x[N][C][H][W] ->
    y[n, c, ho, wo] = max over a, b < window of x[n, c, ho*stride + a, wo*stride + b];
    windows lie inside the image, (H - window) // stride + 1 output rows."""
    x = np.asarray(x, dtype=np.float64)
    N, C, H, W = x.shape
    Ho, Wo = (H - window) // stride + 1, (W - window) // stride + 1
    y = np.full((N, C, Ho, Wo), -np.inf)
    for a in range(window):
        for b in range(window):
            y = np.maximum(y, x[:, :, a:a + (Ho - 1) * stride + 1:stride, b:b + (Wo - 1) * stride + 1:stride])
    return y


def chain_forward(layers, x) -> np.ndarray:
    """A cascade of layers (Sec. 2.1), each the definition above applied to the previous output.
    `layers`: list of dicts, kind = "fc" (w[p][q][k], bias, relu), "conv" (w[r][r][p][q][k], bias,
    relu, pad, stride) or "pool" (window, stride).  An FC layer reads the preceding image as the
    vector [C*H*W] it is in NCHW order; a CONV / POOL layer after an FC layer needs "shape":
    (C, H, W) to view the vector as an image."""
    a = np.asarray(x, dtype=np.float64)
    for l in layers:
        if "shape" in l:
            a = a.reshape((a.shape[0],) + tuple(l["shape"]))
        if l["kind"] == "fc":
            a = fc_forward(l["w"], a.reshape(a.shape[0], -1), l.get("bias"), l.get("relu", False))
        elif l["kind"] == "conv":
            a = conv_forward(l["w"], a, l.get("bias"), l.get("relu", False), l.get("pad", 0), l.get("stride", 1))
        elif l["kind"] == "pool":
            a = maxpool_forward(a, l["window"], l["stride"])
        else:
            raise ValueError(l["kind"])
    return a


def bias_grad(dy, channel_axis=1) -> np.ndarray:
    """dL/dtheta (Eq. 1: a = Wx + theta, so the gradient of theta is dL/da summed over
    everything but the channel axis): dy[B][m] -> db[m]; dy[N][C][H][W] -> db[C]."""
    dy = np.asarray(dy, dtype=np.float64)
    axes = tuple(ax for ax in range(dy.ndim) if ax != channel_axis)
    return dy.sum(axis=axes)


def fc_sgd_step(w, x, dy, lr) -> np.ndarray:
    """One plain gradient-descent step on the block vectors of an FC layer.

    The training of Sec. 3.1 (Algorithm 2) ends in dL/dw_ij; the update itself is the
    ordinary one, w_ij <- w_ij - lr * dL/dw_ij, with the gradient summed over the batch.
    Because the FFT is linear, the same step applied to cached spectra,
    FFT(w_ij) <- FFT(w_ij) - lr * FFT(dL/dw_ij), must give FFT of this result.
    w[p][q][k], x[B][q*k], dy[B][p*k] -> w_new[p][q][k].
    """
    w = np.asarray(w, dtype=np.float64)
    return w - float(lr) * fc_backward_dw(x, dy, w.shape[2])


def conv_sgd_step(w, x, dy, lr, pad=0, stride=1) -> np.ndarray:
    """The same step for a block-circulant CONV layer (Sec. 3.2): w[r][r][p][q][k]."""
    w = np.asarray(w, dtype=np.float64)
    return w - float(lr) * conv_backward_dw(x, dy, w.shape[4], w.shape[0], pad, stride)


def max_norm_rel_err(got, ref) -> float:
    """max_e |got_e - ref_e| / max_e |ref_e| — the parity gate for one tensor."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    denom = float(np.max(np.abs(ref)))
    if denom == 0.0:
        return float(np.max(np.abs(got)))
    return float(np.max(np.abs(got - ref)) / denom)

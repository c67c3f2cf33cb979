"""Glue for the GPU parity tests: numpy in -> C ABI on cuda:0 -> numpy out."""
import numpy as np
import torch

from paper_1708_08917_amd import binding as B

DEV = "cuda:0"


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def epi_flags(bias, relu):
    return (B.EPI_BIAS if bias is not None else 0) | (B.EPI_RELU if relu else 0)


def gpu_fc_forward(w, x, bias=None, relu=False):
    p, q, k = w.shape
    wh = B.circ_precompute_spectra(dev(w))
    y = B.circ_fc_forward(wh, dev(x), dev(bias), None, p, q, k, epi_flags(bias, relu))
    torch.cuda.synchronize()
    return y.cpu().numpy()


def gpu_fc_backward(w, x, dy, need_dx=True, need_dw=True):
    p, q, k = w.shape
    wh = B.circ_precompute_spectra(dev(w))
    dx, dw = B.circ_fc_backward(wh, dev(x), dev(dy), p, q, k, need_dx, need_dw)
    torch.cuda.synchronize()
    return (None if dx is None else dx.cpu().numpy()), (None if dw is None else dw.cpu().numpy())


def gpu_conv_forward(w, x, bias=None, relu=False, pad=0, stride=1):
    r, _, p, q, k = w.shape
    wh = B.circ_precompute_spectra(dev(w))
    y = B.circ_conv_forward(wh, dev(x), dev(bias), None, p * k, r, stride, pad, k, epi_flags(bias, relu))
    torch.cuda.synchronize()
    return y.cpu().numpy()


def gpu_conv_backward(w, x, dy, pad=0, need_dx=True, need_dw=True, stride=1):
    r, _, p, q, k = w.shape
    N, C_in, H, W = x.shape
    wh = B.circ_precompute_spectra(dev(w))
    dx, dw = B.circ_conv_backward(wh, dev(x), dev(dy), C_in, H, W, r, stride, pad, k, need_dx, need_dw)
    torch.cuda.synchronize()
    return (None if dx is None else dx.cpu().numpy()), (None if dw is None else dw.cpu().numpy())


def gpu_bias_grad(dy):
    db = B.circ_bias_grad(dev(dy))
    torch.cuda.synchronize()
    return db.cpu().numpy()



def gpu_fc_sgd_steps(w, batches, lr, need_dx=False):
    """Precompute once, take one step per (x, dy) pair on the spectra, export the weights.
    Returns (w_new [p][q][k], blob, list of dx)."""
    p, q, k = w.shape
    wh = B.circ_precompute_spectra(dev(w.astype(np.float32)))
    dxs = []
    for x, dy in batches:
        dx = B.circ_fc_sgd_step(wh, dev(x.astype(np.float32)), dev(dy.astype(np.float32)), lr, p, q, k, need_dx=need_dx)
        dxs.append(None if dx is None else dx.cpu().numpy())
    w_new = B.circ_export_weights(wh, 1, p, q, k).cpu().numpy().reshape(p, q, k)
    return w_new, wh, dxs


def gpu_conv_sgd_steps(w, batches, lr, pad, need_dx=False, stride=1):
    r, _, p, q, k = w.shape
    wh = B.circ_precompute_spectra(dev(w.astype(np.float32)))
    dxs = []
    for x, dy in batches:
        _, C_in, H, W = x.shape
        dx = B.circ_conv_sgd_step(wh, dev(x.astype(np.float32)), dev(dy.astype(np.float32)), lr, C_in, H, W, r, stride, pad, k,
                                  need_dx=need_dx)
        dxs.append(None if dx is None else dx.cpu().numpy())
    w_new = B.circ_export_weights(wh, r * r, p, q, k).cpu().numpy().reshape(w.shape)
    return w_new, wh, dxs

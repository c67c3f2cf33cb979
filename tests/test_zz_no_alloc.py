"""circ_fc_forward_static (the entry point for callers that cannot allocate) against
circ_fc_forward and the oracle, through the C ABI: two calls in a row on the library's fixed
scratch array, the second with a smaller input, for both routes that really use scratch memory
(the three-kernel route and the split batch <= 2 kernel)."""
import numpy as np
import pytest
import torch

from oracle import circ_oracle as O
from paper_1708_08917_amd import binding as B
from tests import gpu_helpers as G

pytestmark = pytest.mark.gpu

GATE, TIGHT = 1e-4, 2e-5


def _layer(rng, p, q, k, batch):
    w = (rng.standard_normal((p, q, k)) / np.sqrt(q * k)).astype(np.float32)
    x = rng.uniform(-1, 1, (batch, q * k)).astype(np.float32)
    b = (0.1 * rng.standard_normal(p * k)).astype(np.float32)
    return w, x, b


def _both(w, x, b):
    p, q, k = w.shape
    wh = B.circ_precompute_spectra(G.dev(w))
    xd, bd = G.dev(x), G.dev(b)
    epi = B.EPI_BIAS | B.EPI_RELU
    assert B.circ_fc_workspace_bytes(p, q, k, x.shape[0]) > 0
    y_ws = B.circ_fc_forward(wh, xd, bd, None, p, q, k, epi)
    y_st = torch.full_like(y_ws, float("nan"))
    B.circ_fc_forward_static(wh, xd, bd, y_st, p, q, k, epi)
    torch.cuda.synchronize()
    return y_st.cpu().numpy(), y_ws.cpu().numpy()


# (first call, smaller second call); k = 16 with batch > 2 takes the three-kernel route (spectra of
# x and y in scratch), batch 1 on few block rows with long rows the split kernel (partial spectra)
@pytest.mark.parametrize("first,second", [((48, 40, 16, 70), (5, 3, 16, 9)),
                                           ((8, 130, 64, 1), (3, 128, 64, 2)),
                                           ((40, 3, 512, 130), (33, 34, 4, 70))])
def test_static_scratch_matches_workspace_entry_point(first, second):
    rng = np.random.default_rng(95)
    for shape in (first, second):
        w, x, b = _layer(rng, *shape)
        y_st, y_ws = _both(w, x, b)
        assert np.array_equal(y_st, y_ws), f"{shape}: differs from circ_fc_forward"      # same kernels, same order
        err = O.max_norm_rel_err(y_st, O.fc_forward(w, x, b, True))
        print(f"[parity] static scratch {shape} max-norm rel err = {err:.3e}", flush=True)
        assert err <= GATE and err <= TIGHT, (shape, err)


def test_static_scratch_rejects_what_does_not_fit():
    # 16384^2, k = 256, batch 1024 needs 135 MB of spectra: more than the fixed array
    p = q = 64; k = 256; batch = 1024
    assert B.circ_fc_workspace_bytes(p, q, k, batch) > B.STATIC_SCRATCH_BYTES
    wh = torch.empty(B.circ_spectra_bytes(1, p, q, k), dtype=torch.uint8, device=G.DEV)
    x = torch.empty(batch, q * k, device=G.DEV)
    y = torch.empty(batch, p * k, device=G.DEV)
    with pytest.raises(B.CircError) as e:
        B.circ_fc_forward_static(wh, x, None, y, p, q, k)
    assert e.value.status == B.CIRC_EWORKSPACE

"""gnn_loss_static (the entry point that allocates nothing) against gnn_loss, through the C ABI:
same bits for the gradient of the logits and for the loss, on two calls in a row, the second on
a smaller input (the static device array keeps the first call's contents)."""
import ctypes as C

import numpy as np
import pytest

from synth import features, glorot_weights, labels_and_mask, rmat_graph

pytestmark = pytest.mark.gpu


def _one(n, m_draw, seed, classes):
    import torch
    from paper_2605_11517_amd import Session

    rowptr, colidx = rmat_graph(n, m_draw, seed, symmetric=True, self_loops=True)
    dims = (32, 48, classes)
    X = features(n, dims[0], seed)
    y, m = labels_and_mask(n, classes, 0.3, seed)
    w = glorot_weights(dims, seed, sage=False, bias_scale=0.1)
    s = Session("gcn", dims, rowptr, colidx, 3, "random", seed, X, w, y, m)
    s.epoch()                                   # forward pass done: A^L holds the logits
    g = s.gact[-1]
    s.ctx.loss(s.stream)
    ref_loss = s.ctx.read_loss(s.stream)
    ref_grad = g.clone()
    g.fill_(7.0)                                # every element must be rewritten
    loss_dev = torch.full((1,), -1.0, dtype=torch.float32, device=s.dev)
    s.ctx.loss_static(s.stream, loss_dev.data_ptr())
    torch.cuda.synchronize()
    got_loss = float(loss_dev.cpu()[0])
    assert np.float32(got_loss).tobytes() == np.float32(ref_loss).tobytes(), (got_loss, ref_loss)
    assert torch.equal(g, ref_grad)
    assert float(ref_grad.abs().max()) > 0
    # the backward pass may follow either loss call
    s.ctx.gather_boundary(len(dims) - 1, 0, s.stream)
    s.ctx.layer_bwd(len(dims) - 1, 0, s.stream)
    torch.cuda.synchronize()
    return got_loss


def test_loss_static_matches_loss_twice_in_a_row():
    a = _one(20_000, 150_000, 5, 47)            # 313 block partial sums
    b = _one(1_500, 9_000, 6, 16)               # 24: the tail of the array still holds the first call's
    assert np.isfinite(a) and np.isfinite(b)


def test_loss_static_rejects_what_it_cannot_hold():
    from paper_2605_11517_amd import Session
    from paper_2605_11517_amd.binding import GnnError

    n = 300
    rowptr, colidx = rmat_graph(n, 1500, 7, symmetric=True, self_loops=True)
    dims = (8, 4)
    s = Session("gcn", dims, rowptr, colidx, 2, "random", 7, features(n, 8, 7),
                glorot_weights(dims, 7, sage=False), *labels_and_mask(n, 4, 0.5, 7))
    with pytest.raises(GnnError) as e:          # null output
        s.ctx.loss_static(s.stream, None)
    assert e.value.status == 1
    with pytest.raises(GnnError) as e:          # no forward pass yet
        s.ctx.loss_static(s.stream, C.c_void_p(16))
    assert e.value.status == 4

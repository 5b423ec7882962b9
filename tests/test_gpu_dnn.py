"""GPU parity of the first fully-connected layer under DES (Section 4.3): the matrix-core kernels,
through the C interface, against the CPU oracle on the same seeded inputs.  Shapes span several
128x128 output tiles with ragged edges in every dimension, shards with unequal numbers of fields,
shards with none, and enough samples that the weight gradient is computed in slices."""
import numpy as np
import pytest

from paper_1909_04823_amd import synth
from _harness import assert_close, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def des():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_1909_04823_amd import des as d
    return d


SHAPES = [
    # B, F, D, H, K
    (1, 2, 4, 4, 4),          # one sample, more shards than fields
    (300, 7, 8, 200, 3),      # ragged everywhere, D below the k tile
    (257, 26, 16, 256, 8),    # Criteo-like layer
    (130, 5, 64, 132, 2),     # D of several k tiles
    (5000, 3, 4, 132, 1),     # many samples: sliced weight gradient
    (2049, 10, 32, 64, 16),
    # contractions deeper than 1024 products take the two-level summation kernel
    (40000, 2, 4, 8, 1),      # weight gradient, 2512 samples per slice
    (64, 40, 32, 16, 1),      # forward, 1280 products per shard
    (8, 2, 4, 1100, 2),       # g_pool, 1100 hidden units
]


@pytest.mark.parametrize("B,F,D,H,K", SHAPES)
def test_dnn_layer_matches_oracle(oracle, des, B, F, D, H, K):
    import torch
    pool, W, dY = synth.dnn_layer_inputs(B * 31 + F, B, F, D, H)
    Y_ref = oracle.dnn_partial_forward(pool, W, K)
    g_ref, dW_ref = oracle.dnn_backward(pool, W, dY)
    print(f"dnn case B={B} F={F} D={D} H={H} K={K}", flush=True)
    pool_g, W_g, dY_g = dev(pool, torch), dev(W, torch), dev(dY, torch)
    nan = lambda *s: torch.full(s, float("nan"), dtype=torch.float32, device="cuda")
    Yp = des.dnn_partial_forward(pool_g, W_g, K, out=nan(K, B, H))
    Y = des.aggregate_partials(Yp)
    g_pool, dW = nan(B, F, D), nan(F * D, H)
    ws = torch.empty(des.dnn_backward_bytes(B, F, D, H), dtype=torch.uint8, device="cuda")
    des.dnn_backward(pool_g, W_g, dY_g, g_pool, dW, ws)
    torch.cuda.synchronize()
    assert_close(Yp.cpu().numpy(), Y_ref, "Y_partial")
    assert_close(Y.cpu().numpy(), oracle.aggregate(Y_ref), "Y")
    assert_close(g_pool.cpu().numpy(), g_ref, "g_pool")
    assert_close(dW.cpu().numpy(), dW_ref, "dW")
    # each output alone
    g2, dW2 = nan(B, F, D), nan(F * D, H)
    des.dnn_backward(pool_g, W_g, dY_g, g2, None, None)
    des.dnn_backward(pool_g, W_g, dY_g, None, dW2, ws)
    torch.cuda.synchronize()
    assert torch.equal(g2, g_pool) and torch.equal(dW2, dW)


def test_dnn_layer_argument_checks(des):
    import torch
    pool = torch.zeros((4, 2, 4), device="cuda"); W = torch.zeros((8, 8), device="cuda")
    with pytest.raises(des.DesError):
        des.dnn_partial_forward(pool, W, 0)                       # K < 1
    with pytest.raises(des.DesError):
        des.dnn_partial_forward(torch.zeros((4, 2, 6), device="cuda"), torch.zeros((12, 8), device="cuda"), 2)  # D % 4
    with pytest.raises(des.DesError):
        des.dnn_partial_forward(pool, torch.zeros((8, 6), device="cuda"), 2)   # H % 4
    dY = torch.zeros((4, 8), device="cuda")
    with pytest.raises(des.DesError):
        des.dnn_backward(pool, W, dY, None, None)                  # no output asked for
    big = torch.zeros((5000, 2, 4), device="cuda")
    with pytest.raises(des.DesError) as e:                         # dW summed over slices of samples needs the workspace
        des.dnn_backward(big, W, torch.zeros((5000, 8), device="cuda"), None, torch.zeros((8, 8), device="cuda"), None)
    assert e.value.code == des.ERR_WORKSPACE
    # empty batch: nothing launched, nothing written
    out = des.dnn_partial_forward(torch.zeros((0, 2, 4), device="cuda"), W, 2)
    assert out.shape == (2, 0, 8)

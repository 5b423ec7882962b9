"""des_bias_act_backward_static (the entry point that allocates nothing: its scratch is an array inside
the library's device image) against des_bias_act_backward (scratch in a caller's workspace), through the
C interface: same kernels, so the results must be identical bit for bit, and both must meet the oracle
within the library's fp32 bound.  Two calls in a row on the shared scratch, the second smaller."""
import numpy as np
import pytest

from _harness import assert_close, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def des():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_1909_04823_amd import des as d
    return d


def _case(oracle, des, torch, rows, H, relu, seed):
    rng = np.random.default_rng(seed)
    A = rng.standard_normal((rows, H)).astype(np.float32)
    dA = rng.standard_normal((rows, H)).astype(np.float32)
    dZ_ref, db_ref = oracle.bias_act_backward(A, dA, relu)
    A_g, dA_g = dev(A, torch), dev(dA, torch)
    ws = torch.empty(des.dense_workspace_bytes(H), dtype=torch.uint8, device="cuda")
    dZ_w = torch.full((rows, H), float("nan"), device="cuda"); db_w = torch.full((H,), float("nan"), device="cuda")
    des.bias_act_backward(A_g, dA_g, relu, dZ_w, db_w, ws)
    dZ_s = torch.full((rows, H), float("nan"), device="cuda"); db_s = torch.full((H,), float("nan"), device="cuda")
    print(f"no-alloc case rows={rows} H={H} relu={relu}", flush=True)
    des.bias_act_backward_static(A_g, dA_g, relu, dZ_s, db_s)
    torch.cuda.synchronize()
    assert torch.equal(dZ_s, dZ_w) and torch.equal(db_s, db_w), f"static scratch differs from workspace at rows={rows} H={H}"
    assert_close(dZ_s.cpu().numpy(), dZ_ref, "dZ")
    assert_close(db_s.cpu().numpy(), db_ref, "dbias")


def test_static_scratch_matches_workspace_entry_point(oracle, des):
    import torch
    # several tiles of 64 columns and a ragged tail, 64 row slices; then a smaller call on the same scratch,
    # whose partials from the first call are still there and must not leak into the result
    _case(oracle, des, torch, rows=20000, H=1000, relu=True, seed=1)
    _case(oracle, des, torch, rows=300, H=36, relu=False, seed=2)
    _case(oracle, des, torch, rows=1, H=1, relu=True, seed=3)


def test_static_scratch_limits(des):
    import torch
    A = torch.zeros((2, 4100), device="cuda")
    out, db = torch.zeros_like(A), torch.zeros(4100, device="cuda")
    with pytest.raises(des.DesError) as e:
        des.bias_act_backward_static(A, A, True, out, db)
    assert e.value.code == des.ERR_WORKSPACE
    A = torch.ones((4, 4096), device="cuda")
    out, db = torch.zeros_like(A), torch.zeros(4096, device="cuda")
    des.bias_act_backward_static(A, A, True, out, db)          # the widest layer the scratch holds
    torch.cuda.synchronize()
    assert bool((db == 4.0).all()) and torch.equal(out, A)

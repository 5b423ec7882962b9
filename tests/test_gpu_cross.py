"""GPU parity of the DCN cross layer under DES (per-shard scalar, aggregation, apply, backward) against the
CPU oracle, through the C interface.  Shapes span one lane group to many rows per slice, K above F,
every supported row width, ragged tails, empty batches, stacked layers, and the benchmark shapes
(sampled rows and columns, since the oracle cannot run 10^9 elements in seconds)."""
import numpy as np
import pytest

from paper_1909_04823_amd import synth
from _harness import assert_close

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def des():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_1909_04823_amd import des as d
    return d


def cross_inputs(seed, B, F, D):
    rng = np.random.default_rng(seed)
    d = F * D
    x0 = (0.3 * rng.standard_normal((B, F, D))).astype(np.float32)
    xl = (0.3 * rng.standard_normal((B, F, D))).astype(np.float32)
    w = (rng.standard_normal(d) / np.sqrt(d)).astype(np.float32)
    bias = (0.1 * rng.standard_normal(d)).astype(np.float32)
    g_y = (0.01 * rng.standard_normal((B, F, D))).astype(np.float32)
    return x0, xl, w, bias, g_y


@pytest.mark.parametrize("B,F,D,K", [(1, 1, 4, 1), (37, 5, 8, 3), (300, 26, 16, 8), (129, 7, 64, 4), (50, 3, 256, 2),
                                     (64, 5, 32, 9), (1000, 10, 128, 1), (2500, 3, 4, 2)])
def test_cross_layer_forward_and_backward(oracle, des, B, F, D, K):
    import torch
    d = F * D
    x0, xl, w, bias, g_y = cross_inputs(7 * B + K, B, F, D)
    t = lambda a: torch.from_numpy(a).cuda()
    tx0, txl, tw, tb, tg = t(x0), t(xl), t(w), t(bias), t(g_y)
    # forward: sub-operator, aggregation, remaining operator
    P = des.cross_partial(txl, tw, K)
    s = des.aggregate_partials(P)
    y = des.cross_apply(tx0, txl, s, tb)
    torch.cuda.synchronize()
    P_ref = oracle.cross_partial(xl, w, K)
    assert_close(P.cpu().numpy(), P_ref, "P")
    s_ref = oracle.aggregate(P_ref)
    assert_close(s.cpu().numpy(), s_ref, "s")
    s32 = s_ref.astype(np.float32)
    assert_close(des.cross_apply(tx0, txl, t(s32), tb).cpu().numpy(), oracle.cross_apply(x0, xl, s32, bias), "y")
    assert_close(y.cpu().numpy(), oracle.cross_apply(x0, xl, s.cpu().numpy(), bias), "y from the library's own s")
    # backward, overwriting and accumulating, and with g_xl written over g_y
    g_s, g_xl_ref, g_x0_ref, dw_ref, db_ref = oracle.cross_backward(x0, xl, w, s32, g_y)
    ws = torch.empty(des.cross_backward_bytes(B, d), dtype=torch.uint8, device="cuda")
    nan = lambda *shape: torch.full(shape, float("nan"), device="cuda")
    g_xl, g_x0, dw, db = nan(B, F, D), nan(B, F, D), nan(d), nan(d)
    des.cross_backward(tx0, txl, tw, t(s32), tg, g_xl, g_x0, False, dw, db, ws)
    torch.cuda.synchronize()
    assert_close(g_xl.cpu().numpy(), g_xl_ref, "g_xl")
    assert_close(g_x0.cpu().numpy(), g_x0_ref, "g_x0")
    assert_close(dw.cpu().numpy(), dw_ref, "dw")
    assert_close(db.cpu().numpy(), db_ref, "db")
    before = (0.01 * np.random.default_rng(1).standard_normal((B, F, D))).astype(np.float32)
    acc, alias = t(before.copy()), tg.clone()
    des.cross_backward(tx0, txl, tw, t(s32), alias, alias, acc, True, dw, db, ws)
    torch.cuda.synchronize()
    assert_close(acc.cpu().numpy(), before.astype(np.float64) + g_x0_ref, "g_x0 accumulated")
    assert_close(alias.cpu().numpy(), g_xl_ref, "g_xl in place of g_y")
    assert_close(dw.cpu().numpy(), dw_ref, "dw (second call)")


@pytest.mark.parametrize("B,F,D", [(3, 2, 4), (700, 9, 16), (130, 4, 64)])
def test_sub_operator_backward_and_first_layer_fold(oracle, des, B, F, D):
    """des_cross_partial_backward (gradient of the scalar only), and des_cross_backward without g_xl: the layer's
    input is x0 itself, so its input gradient lands in g_x0 together with the layer's own share."""
    import torch
    d = F * D
    x0, xl, w, bias, g_y = cross_inputs(11 * B, B, F, D)
    rng = np.random.default_rng(B)
    g_s = (0.1 * rng.standard_normal(B)).astype(np.float32)
    s32 = oracle.aggregate(oracle.cross_partial(x0, w, 3)).astype(np.float32)
    t = lambda a: torch.from_numpy(a).cuda()
    ws = torch.empty(des.cross_backward_bytes(B, d), dtype=torch.uint8, device="cuda")
    nan = lambda *shape: torch.full(shape, float("nan"), device="cuda")
    g_xl, dw, db = nan(B, F, D), nan(d), nan(d)
    des.cross_partial_backward(t(xl), t(w), t(g_s), g_xl, dw, ws)
    torch.cuda.synchronize()
    g_ref, dw_ref = oracle.cross_partial_backward(xl, w, g_s)
    assert_close(g_xl.cpu().numpy(), g_ref, "g_xl of the sub-operator")
    assert_close(dw.cpu().numpy(), dw_ref, "dw of the sub-operator")
    dw2 = nan(d)
    des.cross_partial_backward(t(xl), t(w), t(g_s), None, dw2, ws)
    torch.cuda.synchronize()
    assert torch.equal(dw, dw2)
    # first layer: xl is x0
    _, g_xl_ref, g_x0_ref, dw_ref, db_ref = oracle.cross_backward(x0, x0, w, s32, g_y)
    for accumulate in (False, True):
        before = (0.01 * rng.standard_normal((B, F, D))).astype(np.float32)
        g_x0 = t(before.copy())
        des.cross_backward(t(x0), t(x0), t(w), t(s32), t(g_y), None, g_x0, accumulate, dw, db, ws)
        torch.cuda.synchronize()
        assert_close(g_x0.cpu().numpy(), (before.astype(np.float64) if accumulate else 0.0) + g_x0_ref + g_xl_ref,
                     f"g_x0 with the input gradient folded in (accumulate={accumulate})")
        assert_close(dw.cpu().numpy(), dw_ref, "dw")
        assert_close(db.cpu().numpy(), db_ref, "db")


def test_stacked_cross_layers_chain(oracle, des):
    """Three layers forward and backward, each stage fed with the previous stage's fp32 output on both sides."""
    import torch
    B, F, D, K, n_layers = 200, 6, 16, 4, 3
    d = F * D
    rng = np.random.default_rng(5)
    x0 = (0.3 * rng.standard_normal((B, F, D))).astype(np.float32)
    ws = [(rng.standard_normal(d) / np.sqrt(d)).astype(np.float32) for _ in range(n_layers)]
    bs = [(0.1 * rng.standard_normal(d)).astype(np.float32) for _ in range(n_layers)]
    g_top = (0.01 * rng.standard_normal((B, F, D))).astype(np.float32)
    t = lambda a: torch.from_numpy(a).cuda()
    xs_o, ss_o = [x0], []
    xs_g, ss_g = [t(x0)], []
    for l in range(n_layers):
        P = des.cross_partial(xs_g[-1], t(ws[l]), K)
        ss_g.append(des.aggregate_partials(P))
        xs_g.append(des.cross_apply(xs_g[0], xs_g[-1], ss_g[-1], t(bs[l])))
        torch.cuda.synchronize()
        # the oracle continues from the library's fp32 activations, so every stage is compared on common inputs
        x_in = xs_g[l].cpu().numpy()
        s_ref = oracle.aggregate(oracle.cross_partial(x_in, ws[l], K))
        assert_close(ss_g[-1].cpu().numpy(), s_ref, f"s of layer {l}")
        s32 = ss_g[-1].cpu().numpy()
        assert_close(xs_g[-1].cpu().numpy(), oracle.cross_apply(x0, x_in, s32, bs[l]), f"x of layer {l + 1}")
        xs_o.append(x_in); ss_o.append(s32)
    wsb = torch.empty(des.cross_backward_bytes(B, d), dtype=torch.uint8, device="cuda")
    g = t(g_top)
    g_x0 = torch.empty((B, F, D), device="cuda")
    dw, db = torch.empty(d, device="cuda"), torch.empty(d, device="cuda")
    total_ref = np.zeros((B, F, D))
    for l in range(n_layers - 1, -1, -1):
        g_in = g.cpu().numpy()
        before = g_x0.cpu().numpy().astype(np.float64) if l < n_layers - 1 else 0.0
        des.cross_backward(xs_g[0], xs_g[l], t(ws[l]), ss_g[l], g, g, g_x0, l < n_layers - 1, dw, db, wsb)
        torch.cuda.synchronize()
        _, g_xl_ref, g_x0_ref, dw_ref, db_ref = oracle.cross_backward(x0, xs_g[l].cpu().numpy(), ws[l],
                                                                      ss_g[l].cpu().numpy(), g_in)
        assert_close(g.cpu().numpy(), g_xl_ref, f"g_xl of layer {l}")
        assert_close(g_x0.cpu().numpy(), before + g_x0_ref, f"g_x0 after layer {l}")
        assert_close(dw.cpu().numpy(), dw_ref, f"dw of layer {l}")
        assert_close(db.cpu().numpy(), db_ref, f"db of layer {l}")


def test_cross_empty_batch_and_argument_checks(des):
    import torch
    F, D = 3, 8
    d = F * D
    e = torch.empty((0, F, D), device="cuda")
    w, b = torch.ones(d, device="cuda"), torch.ones(d, device="cuda")
    P = des.cross_partial(e, w, 2)
    assert tuple(P.shape) == (2, 0)
    des.cross_apply(e, e, torch.empty(0, device="cuda"), b)
    ws = torch.empty(des.cross_backward_bytes(0, d), dtype=torch.uint8, device="cuda")
    dw, db = torch.full((d,), 7.0, device="cuda"), torch.full((d,), 7.0, device="cuda")
    des.cross_backward(e, e, w, torch.empty(0, device="cuda"), e, e.clone(), e.clone(), False, dw, db, ws)
    torch.cuda.synchronize()
    assert float(dw.abs().sum()) == 0.0 and float(db.abs().sum()) == 0.0
    # the whole-network calls on an empty batch: no-ops, and zero parameter gradients
    U, nb = torch.ones((3, d), device="cuda"), torch.ones((2, d), device="cuda")
    P3 = des.cross_net_partial(e, U, 2)
    assert tuple(P3.shape) == (2, 0, 3)
    nws = torch.empty(des.cross_net_bytes(0, d, 2), dtype=torch.uint8, device="cuda")
    t0, g0, c0 = torch.empty((0, 3), device="cuda"), torch.empty((0, 3), device="cuda"), torch.empty(0, device="cuda")
    des.cross_net_forward(t0, U, nb, g0, c0, nws)
    dU, dB = torch.full((3, d), 7.0, device="cuda"), torch.full((2, d), 7.0, device="cuda")
    des.cross_net_backward(e, U, nb, t0, g0, c0, e.clone(), False, dU, dB, nws)
    torch.cuda.synchronize()
    assert float(dU.abs().sum()) == 0.0 and float(dB.abs().sum()) == 0.0
    x = torch.ones((4, F, D), device="cuda")
    with pytest.raises(des.DesError) as err:                           # workspace too small
        des.cross_backward(x, x, w, torch.ones(4, device="cuda"), x, x.clone(), x.clone(), False, dw, db,
                           torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert err.value.code == des.ERR_WORKSPACE
    with pytest.raises(des.DesError) as err:                           # D not a multiple of 4
        des.cross_partial(torch.ones((4, 3, 6), device="cuda"), torch.ones(18, device="cuda"), 1)
    assert err.value.code == des.ERR_INVALID_ARG


@pytest.mark.parametrize("index", [2, 4])
def test_cross_layer_full_size_sampled(oracle, des, index):
    """One cross layer at the benchmark shapes (d = F*D up to 12800, B up to 131072): whole rows of sampled
    samples for P, s, y, g_xl and g_x0, and sampled columns of dw and db summed over the full batch."""
    import torch
    w_ = synth.workload(index)
    B, F, D, K = w_.B, w_.F, w_.D, w_.K
    d = F * D
    gen = torch.Generator(device="cuda"); gen.manual_seed(300 + index)
    x0 = torch.randn((B, F, D), device="cuda", generator=gen) * 0.3
    xl = torch.randn((B, F, D), device="cuda", generator=gen) * 0.3
    g_y = torch.randn((B, F, D), device="cuda", generator=gen) * 0.01
    w = torch.randn(d, device="cuda", generator=gen) / float(np.sqrt(d))
    bias = torch.randn(d, device="cuda", generator=gen) * 0.1
    P = des.cross_partial(xl, w, K)
    s = des.aggregate_partials(P)
    y = des.cross_apply(x0, xl, s, bias)
    g_xl, g_x0 = torch.empty_like(x0), torch.empty_like(x0)
    dw, db = torch.empty(d, device="cuda"), torch.empty(d, device="cuda")
    ws = torch.empty(des.cross_backward_bytes(B, d), dtype=torch.uint8, device="cuda")
    des.cross_backward(x0, xl, w, s, g_y, g_xl, g_x0, False, dw, db, ws)
    torch.cuda.synchronize()
    rng = np.random.default_rng(index)
    bsel = np.unique(np.concatenate([[0, 1, B - 1], rng.integers(0, B, 13)]))
    bt = torch.from_numpy(bsel).cuda()
    h = lambda a: a.cpu().numpy()
    x0_s, xl_s, g_s_, w_h, b_h = h(x0[bt]), h(xl[bt]), h(g_y[bt]), h(w), h(bias)
    P_ref = oracle.cross_partial(xl_s, w_h, K)
    assert_close(h(P[:, bt]), P_ref, "P rows")
    assert_close(h(s[bt]), oracle.aggregate(P_ref), "s rows")
    s32 = h(s[bt])
    assert_close(h(y[bt]), oracle.cross_apply(x0_s, xl_s, s32, b_h), "y rows")
    gs_ref, g_xl_ref, g_x0_ref, _, _ = oracle.cross_backward(x0_s, xl_s, w_h, s32, g_s_)
    assert_close(h(g_xl[bt]), g_xl_ref, "g_xl rows")
    assert_close(h(g_x0[bt]), g_x0_ref, "g_x0 rows")
    # columns of the batch sums: db[j] = sum_b g_y[b,j]; dw[j] = sum_b g_s[b] xl[b,j] with the oracle's g_s from
    # whole rows is out of reach for all B, so g_s comes from float64 row sums on the host in chunks
    jsel = np.unique(np.concatenate([[0, 3, 4, d - 1], rng.integers(0, d, 12)]))
    jt = torch.from_numpy(jsel).cuda()
    gs_all = np.empty(B, np.float64)
    step = 8192
    for b0 in range(0, B, step):
        gs_all[b0:b0 + step] = (h(g_y[b0:b0 + step]).reshape(-1, d).astype(np.float64) *
                                h(x0[b0:b0 + step]).reshape(-1, d)).sum(axis=1)
    np.testing.assert_allclose(gs_all[bsel], gs_ref, rtol=1e-12, atol=1e-15)       # the host sums are the oracle's g_s
    xl_cols = h(xl.reshape(B, d)[:, jt]).astype(np.float64)
    gy_cols = h(g_y.reshape(B, d)[:, jt]).astype(np.float64)
    assert_close(h(dw[jt]), (gs_all[:, None] * xl_cols).sum(axis=0), "dw columns")
    assert_close(h(db[jt]), gy_cols.sum(axis=0), "db columns")


def oracle_cross_network(oracle, x0, U, bias, g, K):
    """The network layer by layer with the oracle's functions (fp32 between the stages, as the layer-by-layer
    library calls hand tensors on): forward scalars, logit term, and every gradient for the gradient g of the term."""
    n = U.shape[0] - 1
    f32 = lambda a: np.ascontiguousarray(a, dtype=np.float32)
    xs, ss = [x0], []
    for l in range(n):
        s = f32(oracle.aggregate(oracle.cross_partial(xs[l], U[l], K)))
        ss.append(s)
        xs.append(f32(oracle.cross_apply(x0, xs[l], s, bias[l])))
    c = oracle.aggregate(oracle.cross_partial(xs[n], U[n], K))
    gx, dwc = oracle.cross_partial_backward(xs[n], U[n], g)
    dU, db = np.zeros(U.shape), np.zeros((n,) + U.shape[1:])
    dU[n] = dwc
    g_x0 = np.zeros(x0.shape)
    gx = f32(gx)
    for l in range(n - 1, -1, -1):
        _, g_xl, share, dU[l], db[l] = oracle.cross_backward(x0, xs[l], U[l], ss[l], gx)
        g_x0 += share
        gx = f32(g_xl)
    g_x0 += gx
    B = x0.shape[0]
    gamma = 1.0 + np.concatenate([np.zeros((1, B)), np.cumsum(np.array(ss, np.float64).reshape(n, B), axis=0)]).T
    return dict(c=c, gamma=gamma, g_x0=g_x0, dU=dU, db=db)


@pytest.mark.parametrize("B,F,D,K,n", [(5, 2, 4, 2, 1), (300, 26, 16, 8, 2), (129, 7, 64, 4, 3), (64, 5, 32, 9, 0),
                                       (1000, 3, 8, 1, 7), (40, 2, 256, 2, 2)])
def test_whole_cross_network_matches_the_layer_by_layer_oracle(oracle, des, B, F, D, K, n):
    import torch
    d, m = F * D, n + 1
    rng = np.random.default_rng(100 * B + n)
    x0 = (0.3 * rng.standard_normal((B, F, D))).astype(np.float32)
    U = (rng.standard_normal((m, d)) / np.sqrt(d)).astype(np.float32)
    bias = (0.1 * rng.standard_normal((n, d))).astype(np.float32)
    g = (0.05 * rng.standard_normal(B)).astype(np.float32)
    before = (0.01 * rng.standard_normal((B, F, D))).astype(np.float32)
    ref = oracle_cross_network(oracle, x0, U, bias, g, K)
    t_ = lambda a: torch.from_numpy(a).cuda()
    tx0, tU, tb = t_(x0), t_(U), (t_(bias) if n else None)
    P = des.cross_net_partial(tx0, tU, K)
    tt = des.aggregate_partials(P.view(K, B * m)).view(B, m)
    ws = torch.empty(des.cross_net_bytes(B, d, n), dtype=torch.uint8, device="cuda")
    gamma, c = torch.empty((B, m), device="cuda"), torch.empty(B, device="cuda")
    des.cross_net_forward(tt, tU, tb, gamma, c, ws)
    torch.cuda.synchronize()
    for k in range(m):                                   # every dot product is the layer sub-operator applied to x0
        assert_close(P[:, :, k].cpu().numpy(), oracle.cross_partial(x0, U[k], K), f"P of vector {k}")
    assert_close(gamma.cpu().numpy(), ref["gamma"], "gamma")
    assert_close(c.cpu().numpy(), ref["c"], "logit term")
    for accumulate in (False, True):
        g_x0 = t_(before.copy())
        dU, db = torch.full((m, d), float("nan"), device="cuda"), (torch.full((n, d), float("nan"), device="cuda") if n else None)
        des.cross_net_backward(tx0, tU, tb, tt, gamma, t_(g), g_x0, accumulate, dU, db, ws)
        torch.cuda.synchronize()
        assert_close(g_x0.cpu().numpy(), (before.astype(np.float64) if accumulate else 0.0) + ref["g_x0"], "g_x0")
        assert_close(dU.cpu().numpy(), ref["dU"], "dU")
        if n:
            assert_close(db.cpu().numpy(), ref["db"], "dbias")

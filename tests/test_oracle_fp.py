"""Pins for the floating-point half of the CPU oracle: expert FFN forward/backward, combine.

Expected values come from library routines on the CPU (torch float64 matmul, autograd,
index_add), from central finite differences, and from special cases with a closed form.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl


def _layer(seed=0, E=3, h=24, hff=20, rows=(5, 0, 9, 3), experts=(2, 1, 0, 2)):
    rng = np.random.default_rng(seed)
    go = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    ge = np.array(experts, np.int32)
    N = int(go[-1])
    bf = lambda x: torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16)
    X = bf(rng.standard_normal((N, h)))
    dY = bf(rng.standard_normal((N, h)))
    Wg = bf(0.3 * rng.standard_normal((E, hff, h)))
    Wu = bf(0.3 * rng.standard_normal((E, hff, h)))
    Wd = bf(0.3 * rng.standard_normal((E, h, hff)))
    return go, ge, X, dY, Wg, Wu, Wd


def _torch_ffn(X, go, ge, Wg, Wu, Wd):
    Y = torch.zeros(X.shape[0], Wd.shape[1], dtype=torch.float64)
    parts = []
    for g in range(len(ge)):
        a, b = int(go[g]), int(go[g + 1])
        e = int(ge[g])
        if e < 0 or a == b:
            continue
        Gt = X[a:b] @ Wg[e].T
        U = X[a:b] @ Wu[e].T
        parts.append((a, b, torch.nn.functional.silu(Gt) * U @ Wd[e].T))
    for a, b, y in parts:
        Y = Y + torch.nn.functional.pad(y, (0, 0, a, X.shape[0] - b))
    return Y


def test_ffn_fwd_equals_library_matmul_per_group():
    go, ge, X, dY, Wg, Wu, Wd = _layer()
    Gt, U, A, Y = oracle.ffn_fwd(X, go, ge, Wg, Wu, Wd)
    Xd, Wgd, Wud, Wdd = (t.double() for t in (X, Wg, Wu, Wd))
    for g in range(len(ge)):
        a, b, e = int(go[g]), int(go[g + 1]), int(ge[g])
        gt = Xd[a:b] @ Wgd[e].T
        u = Xd[a:b] @ Wud[e].T
        act = torch.nn.functional.silu(gt) * u
        np.testing.assert_allclose(Gt[a:b], gt.numpy(), rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(U[a:b], u.numpy(), rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(A[a:b], act.numpy(), rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(Y[a:b], (act @ Wdd[e].T).numpy(), rtol=1e-12, atol=1e-12)


def test_ffn_fwd_group_range_and_empty_slots():
    go, ge, X, dY, Wg, Wu, Wd = _layer(rows=(4, 0, 6, 0), experts=(1, -1, 0, -1))
    _, _, _, Y_all = oracle.ffn_fwd(X, go, ge, Wg, Wu, Wd)
    _, _, _, Y_part = oracle.ffn_fwd(X, go, ge, Wg, Wu, Wd, g_begin=2, g_end=3)
    assert np.isnan(Y_part[:4]).all()
    np.testing.assert_array_equal(Y_part[4:], Y_all[4:])
    assert not np.isnan(Y_all).any()


def test_ffn_bwd_equals_autograd():
    go, ge, X, dY, Wg, Wu, Wd = _layer(seed=1)
    dX, dWg, dWu, dWd = oracle.ffn_bwd(X, dY, go, ge, Wg, Wu, Wd)
    Xd = X.double().requires_grad_()
    Wgd, Wud, Wdd = (t.double().requires_grad_() for t in (Wg, Wu, Wd))
    Y = _torch_ffn(Xd, go, ge, Wgd, Wud, Wdd)
    (Y * dY.double()).sum().backward()
    np.testing.assert_allclose(dX, Xd.grad.numpy(), rtol=1e-10, atol=1e-12)
    # expert 2 owns two groups (a home copy and a replica): gradients must be their sum
    np.testing.assert_allclose(dWg, Wgd.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dWu, Wud.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dWd, Wdd.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_ffn_bwd_matches_central_finite_differences():
    # d/dp <Y(p), dY> by central differences on the oracle's own forward, in float64, at
    # bf16-representable points moved by a bf16-representable step.
    go, ge, X, dY, Wg, Wu, Wd = _layer(seed=2, E=2, h=8, hff=8, rows=(3, 2, 2), experts=(0, 1, 0))
    dX, dWg, dWu, dWd = oracle.ffn_bwd(X, dY, go, ge, Wg, Wu, Wd)

    def loss(Xv, Wgv, Wuv, Wdv):
        Y = _torch_ffn(Xv, go, ge, Wgv, Wuv, Wdv)
        return float((Y * dY.double()).sum())

    base = [t.double().clone() for t in (X, Wg, Wu, Wd)]
    grads = [dX, dWg, dWu, dWd]
    rng = np.random.default_rng(0)
    eps = 1e-5
    for which in range(4):
        flat_n = base[which].numel()
        for idx in rng.choice(flat_n, size=12, replace=False):
            plus = [t.clone() for t in base]
            minus = [t.clone() for t in base]
            plus[which].view(-1)[idx] += eps
            minus[which].view(-1)[idx] -= eps
            fd = (loss(*plus) - loss(*minus)) / (2 * eps)
            assert abs(fd - grads[which].reshape(-1)[idx]) <= 1e-6 * max(1.0, abs(fd))


def test_silu_derivative_special_points():
    # one expert, h = h' = 1, Wu = Wd = 1: y = silu(w x) * x; dy/dw at w x = 0 is x^2 / 2.
    go, ge = np.array([0, 1], np.int32), np.array([0], np.int32)
    one = torch.tensor([[[1.0]]], dtype=torch.bfloat16)
    X = torch.tensor([[2.0]], dtype=torch.bfloat16)
    Wg = torch.tensor([[[0.0]]], dtype=torch.bfloat16)
    dX, dWg, dWu, dWd = oracle.ffn_bwd(X, torch.tensor([[1.0]], dtype=torch.bfloat16), go, ge, Wg, one, one)
    assert dWg[0, 0, 0] == pytest.approx(0.5 * 2.0 * 2.0 * 2.0 / 2.0)   # dA*U*silu'(0)*x = 1*2*0.5*2
    assert dWu[0, 0, 0] == pytest.approx(0.0)                         # silu(0) = 0
    assert dX[0, 0] == pytest.approx(0.0)                             # Wg = 0 and silu(0) = 0


def test_combine_fwd_equals_index_add_and_dense_special_case():
    rng = np.random.default_rng(5)
    T, k, h = 11, 3, 7
    N = T * k
    row_of = rng.permutation(N).astype(np.int32)
    Y = rng.standard_normal((N, h))
    gates = rng.random((T, k)).astype(np.float32)
    out = oracle.combine_fwd(Y, gates, row_of, T, k)
    want = torch.zeros(T, h, dtype=torch.float64)
    want.index_add_(0, torch.arange(N) // k,
                    torch.from_numpy(Y[row_of]) * torch.from_numpy(gates.astype(np.float64)).reshape(-1, 1))
    np.testing.assert_allclose(out, want.numpy(), rtol=1e-13, atol=1e-13)
    # gate == 1 (the backward of the row gather) is a plain scatter-sum
    out1 = oracle.combine_fwd(Y, None, row_of, T, k)
    want1 = torch.zeros(T, h, dtype=torch.float64)
    want1.index_add_(0, torch.arange(N) // k, torch.from_numpy(Y[row_of]))
    np.testing.assert_allclose(out1, want1.numpy(), rtol=1e-13, atol=1e-13)
    # every slot of a token pointing at identical rows with gates 1/k gives that row back
    Ysame = np.repeat(rng.standard_normal((T, h)), k, axis=0)
    ident = np.arange(N, dtype=np.int32)
    out2 = oracle.combine_fwd(Ysame, np.full((T, k), 1.0 / k, np.float32), ident, T, k)
    np.testing.assert_allclose(out2, Ysame[::k], rtol=1e-6)


def test_combine_bwd_equals_autograd():
    rng = np.random.default_rng(6)
    T, k, h = 9, 2, 5
    N = T * k
    row_of = rng.permutation(N).astype(np.int32)
    Y = torch.from_numpy(rng.standard_normal((N, h))).requires_grad_()
    gates = torch.from_numpy(rng.random((T, k)).astype(np.float32)).double().requires_grad_()
    dOut = rng.standard_normal((T, h))
    out = (Y[torch.from_numpy(row_of).long()].reshape(T, k, h) * gates.unsqueeze(-1)).sum(1)
    (out * torch.from_numpy(dOut)).sum().backward()
    dY, dgate = oracle.combine_bwd(dOut, Y.detach().numpy(), gates.detach().numpy().astype(np.float32),
                                   row_of, T, k)
    np.testing.assert_allclose(dY, Y.grad.numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dgate, gates.grad.numpy(), rtol=1e-12, atol=1e-13)


def test_whole_layer_reduces_to_dense_ffn_when_experts_are_identical():
    # With identical experts and gates summing to one, the MoE layer is the dense SwiGLU FFN
    # of each token, whatever the routing, the plan and the replica split are.
    cfg = wl.small_config(E=8, k=2, EP=4, r=1, T=96, n_mb=1, h=32, hff=24)
    ids, gates = wl.make_routing(cfg, 0)
    X, _ = wl.make_tokens(cfg, 0)
    Wg, Wu, Wd = wl.make_weights(cfg)
    Wg, Wu, Wd = (W[:1].expand(cfg.E, -1, -1).contiguous() for W in (Wg, Wu, Wd))
    counts, _ = oracle.route_hist(ids[None], cfg.E)
    p = oracle.plan(counts, cfg.EP, cfg.rpn, cfg.r)
    row_of, src_of = oracle.permute(ids, cfg.E, p["inst_ptr"][0], p["inst_rows"][0],
                                    p["inst_group"][0], p["group_offset"][0])
    Xrows = oracle.gather_rows(X, src_of, cfg.k)
    _, _, _, Y = oracle.ffn_fwd(Xrows, p["group_offset"][0], p["group_expert"][0], Wg, Wu, Wd)
    out = oracle.combine_fwd(Y, gates, row_of, cfg.T, cfg.k)
    Xd = X.double()
    dense = (torch.nn.functional.silu(Xd @ Wg[0].double().T) * (Xd @ Wu[0].double().T)) @ Wd[0].double().T
    np.testing.assert_allclose(out, dense.numpy(), rtol=1e-6, atol=1e-9)

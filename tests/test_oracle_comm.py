"""Pins of the oracle's communication-aware cost model (Section 4.1, Eq. 1-6), its smoothed
objective and Algorithm 1 (Section 4.2) against things other than itself: the definitions
applied token by token, scipy's logsumexp, closed forms, brute force over all placements.
The annealing's trajectory is parity-unpinned (cooling rate, threshold, seeds and generator are
not published); what is pinned are its cost model and its invariants."""
import itertools

import numpy as np
import pytest
from scipy.special import logsumexp

import oracle
import workloads as wl


def model(h=2048, hff=768, F=5e14, B_intra=1.0e12, B_inter=5e10):
    return oracle.cost_model(h, hff, F, B_intra, B_inter)


def test_tau_on_the_two_node_two_gpu_example():
    """Figure of Section 4.1: two nodes of two GPUs; GPUs with the same index in their node share a rail."""
    LOC, NV, SR, CR = 0, 1, 2, 3
    want = [[LOC, NV, SR, CR],
            [NV, LOC, CR, SR],
            [SR, CR, LOC, NV],
            [CR, SR, NV, LOC]]
    got = [[oracle.tau(j, g, 2) for g in range(4)] for j in range(4)]
    assert got == want
    assert all(oracle.tau(j, g, 8) in (LOC, NV) for j in range(8) for g in range(8))     # one node: no RDMA


@pytest.mark.parametrize("EP,rpn,E", [(4, 2, 8), (8, 4, 16), (8, 8, 8), (6, 2, 12)])
def test_loads_equal_token_by_token_classification(EP, rpn, E):
    """Eq. 1-3 applied to every routed token separately (source rank, hosting rank -> type ->
    which links it loads) must give the aggregated loads."""
    rng = np.random.default_rng(EP * 100 + E)
    x = rng.integers(0, 9, size=(EP, E)).astype(np.int64)
    rank_of = rng.permutation(np.repeat(np.arange(EP), E // EP)).astype(np.int32)
    comp, nv_tx, nv_rx, rd_tx, rd_rx = [np.zeros(EP, np.int64) for _ in range(5)]
    for j in range(EP):
        for e in range(E):
            for _ in range(int(x[j, e])):                  # one token at a time
                g = int(rank_of[e])
                comp[g] += 1
                same_node = j // rpn == g // rpn
                if j == g:
                    continue
                if same_node:
                    nv_tx[j] += 1; nv_rx[g] += 1           # direct intra-node transfer
                elif j % rpn == g % rpn:
                    rd_tx[j] += 1; rd_rx[g] += 1           # same rail: RDMA only
                else:
                    nv_tx[j] += 1; nv_rx[g] += 1           # cross rail: intra-node relay ...
                    rd_tx[j] += 1; rd_rx[g] += 1           # ... then RDMA
    got = oracle.loads(x, rank_of, rpn)
    for a, b in zip(got, (comp, nv_tx, nv_rx, rd_tx, rd_rx)):
        assert np.array_equal(a, b)
    assert got[1].sum() == got[2].sum() and got[3].sum() == got[4].sum()      # every send is received
    assert got[0].sum() == x.sum()
    if rpn == EP:
        assert got[3].sum() == 0


def test_lse_matches_scipy_and_brackets_the_max():
    rng = np.random.default_rng(3)
    for n in (1, 4, 32):
        z = rng.uniform(0, 2, n)
        for beta in (1.0, 20.0, 400.0):
            got = oracle.lse(z, beta)
            assert got == pytest.approx(logsumexp(beta * z) / beta, rel=1e-13)
            assert z.max() <= got <= z.max() + np.log(n) / beta + 1e-15
    assert oracle.lse(np.array([0.3, 1.7, 1.2]), 5000.0) == pytest.approx(1.7, abs=1e-3)


def test_moe_time_hand_example():
    """2 nodes x 2 GPUs, 4 experts, expert e on rank e.  Loads by hand from Eq. 1-3, times by Eq. 4-6."""
    x = np.array([[10, 2, 3, 1],       # tokens on rank 0 for experts 0..3
                  [0, 8, 0, 4],
                  [5, 0, 6, 0],
                  [1, 1, 1, 7]], np.int64)
    rank_of = np.arange(4, dtype=np.int32)
    m = np.array([2.0, 0.5, 3.0])      # seconds per token: compute, intra-node link, RDMA
    comp = x.sum(0)                                       # [16, 11, 10, 12]
    # rank 0 sends: to rank 1 (nv) 2, to rank 2 (same rail) 3, to rank 3 (cross rail) 1
    assert oracle.loads(x, rank_of, 2)[1][0] == 2 + 1 and oracle.loads(x, rank_of, 2)[3][0] == 3 + 1
    nv_tx = np.array([2 + 1, 0 + 0, 0 + 0, 1 + 1]); nv_rx = np.array([0 + 1, 2 + 0, 1 + 0, 0 + 1])
    rd_tx = np.array([3 + 1, 0 + 4, 5 + 0, 1 + 1]); rd_rx = np.array([5 + 1, 1 + 0, 3 + 0, 4 + 1])
    L = oracle.loads(x, rank_of, 2)
    for a, b in zip(L, (comp, nv_tx, nv_rx, rd_tx, rd_rx)):
        assert np.array_equal(a, b)
    t_comp = 2.0 * 16
    t_comm = max(max(0.5 * nv_tx.max(), 0.5 * nv_rx.max()), max(3.0 * rd_tx.max(), 3.0 * rd_rx.max()))   # 18
    out = oracle.moe_time(x, rank_of, 2, m, beta=20.0, t_ref=1.0)
    assert out["T_comp"] == t_comp and out["T_comm"] == t_comm == 18.0 and out["T"] == 50.0
    # smoothing: LSE over ranks of the compute times plus LSE over ranks of the LSE of the four link times
    zc = 2.0 * comp
    zm = [logsumexp(20.0 * np.array([0.5 * nv_tx[g], 0.5 * nv_rx[g], 3.0 * rd_tx[g], 3.0 * rd_rx[g]])) / 20.0 for g in range(4)]
    want = logsumexp(20.0 * zc) / 20.0 + logsumexp(20.0 * np.array(zm)) / 20.0
    assert out["smooth"] == pytest.approx(want, rel=1e-13)
    # the smoothed objective scales with 1 / t_ref and tends to the exact one as beta grows
    sharp = oracle.moe_time(x, rank_of, 2, m, beta=1e4, t_ref=50.0)
    assert sharp["smooth"] == pytest.approx(1.0, abs=1e-3)


def test_route_hist_src_is_a_per_chunk_bincount():
    cfg = wl.small_config(T=512, k=4, E=16, EP=4)
    ids, _ = wl.make_routing(cfg, 0)
    x = oracle.route_hist_src(ids, cfg.E, cfg.EP)
    per = cfg.T // cfg.EP
    for j in range(cfg.EP):
        assert np.array_equal(x[j], np.bincount(ids[j * per:(j + 1) * per].ravel(), minlength=cfg.E))
    assert np.array_equal(x.sum(0), oracle.route_hist(ids[None], cfg.E)[0][0])
    with pytest.raises(ValueError):
        oracle.route_hist_src(ids[:510], cfg.E, cfg.EP)


def affinity_instance(seed, E, EP):
    """Every expert is mostly used by the tokens of one rank: placement decides the traffic."""
    rng = np.random.default_rng(seed)
    aff = rng.permutation(np.repeat(np.arange(EP), E // EP))
    x = rng.integers(5, 30, size=(EP, E)).astype(np.int64)
    for e in range(E):
        x[aff[e], e] += rng.integers(300, 600)
    return x, aff.astype(np.int32)


def test_sa_invariants_and_gain_over_lpt_when_placement_decides_traffic():
    E, EP, rpn = 32, 8, 4
    x, aff = affinity_instance(1, E, EP)
    m = model()
    rank, st = oracle.reorder_sa(x, rpn, m, gamma=0.999, eps=1e-3, n_seeds=4, seed=7)
    assert sorted(np.bincount(rank, minlength=EP).tolist()) == [E // EP] * EP           # capacity kept
    assert st["smooth"] <= st["smooth_start"]                                          # best-so-far starts at the start
    lp = oracle.lpt(x.sum(0), EP)
    assert st["T_start"] == oracle.moe_time(x, lp, rpn, m)["T"]                         # the start is greedy LPT
    assert st["T"] == oracle.moe_time(x, rank, rpn, m)["T"]
    assert st["T"] < 0.5 * st["T_start"]                                               # locality found
    assert st["T"] < 1.1 * oracle.moe_time(x, aff, rpn, m)["T"]
    assert st["iterations"] == int(np.ceil(np.log(1e-3 / st["smooth_start"]) / np.log(0.999)))
    again, st2 = oracle.reorder_sa(x, rpn, m, gamma=0.999, eps=1e-3, n_seeds=4, seed=7)
    assert np.array_equal(rank, again) and st2 == st                                   # deterministic


def test_sa_near_bruteforce_optimum_on_tiny_instances():
    """All placements of 6 experts on 3 ranks (2 each) enumerated; the annealing's result must be
    within 10 % of the best exact T_MoE (quality, not trajectory)."""
    E, EP, rpn = 6, 3, 3
    m = model(B_intra=2e10)
    worst = 0.0
    for seed in range(6):
        x, _ = affinity_instance(100 + seed, E, EP)
        best = np.inf
        for perm in set(itertools.permutations([0, 0, 1, 1, 2, 2])):
            best = min(best, oracle.moe_time(x, np.array(perm, np.int32), rpn, m)["T"])
        _, st = oracle.reorder_sa(x, rpn, m, gamma=0.995, eps=1e-3, n_seeds=4, seed=seed)
        worst = max(worst, st["T"] / best)
    assert worst <= 1.10

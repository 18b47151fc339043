"""Pins of the oracle's communication-aware cost model (Section 4.1, Eq. 1-6), its smoothed
objective and Algorithm 1 (Section 4.2) against things other than itself: the definitions
applied token by token, scipy's logsumexp, closed forms, brute force over all placements.
The annealing's constants (cooling rate, threshold, seeds, generator) are not published and are
arguments; its generator is pinned against published outputs and its acceptance rule, cooling and
draw order by a hand-worked three-step run (end of this file)."""
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


# ------------------------------------------------------------------ Algorithm 1, step by step
def test_splitmix64_published_vectors():
    """The generator of the annealing's draws against its published outputs: state 0 (the
    reference implementation's first values) and state 1234567 (the widely reproduced test vector)."""
    assert oracle.splitmix64(0, 5).tolist() == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F,
                                                0xF88BB8A8724C81EC, 0x1B39896A51A8749B]
    assert oracle.splitmix64(1234567, 5).tolist() == [6457827717110365317, 3203168211198807973, 9817491932198370423,
                                                      4593380528125082431, 16408922859458223821]


# A hand-worked run of Algorithm 1: 4 experts, 2 ranks in one node (every remote token crosses the
# intra-node link), one second per token of computation and per token over the link, beta = 20,
# gamma = 1/2, eps = 0.2 -> theta = T0, T0/2, T0/4 (> 0.2) and T0/8 (< 0.2): three iterations.
#   x[j][e]:  source 0 -> 8 1 1 6     loads l = 9 8 6 7
#             source 1 -> 1 7 5 1
# Greedy LPT: e0 (9) -> rank 0, e1 (8) -> rank 1, e3 (7) -> rank 1 (8 < 9; rank 1 is full), e2 -> rank 0.
# States met, as (computation load per rank | link send per rank | link receive per rank):
#   A = [0,1,0,1] start:      15 15 | 7 6 | 6 7     exact T = 15 + 7 = 22 = t_ref
#   B = [1,1,0,0] swap(0,3):  13 17 | 9 6 | 6 9
#   C = [0,1,1,0] swap(2,0):  16 14 | 2 2 | 2 2
#   D = [0,0,1,1] swap(1,3):  17 13 | 7 8 | 8 7
# Draws from splitmix64 started at 49 (e_a = o1 % 4, e_b = o2 % 4, u = (o3 >> 11) / 2^53, ...).
SA_HAND = dict(
    x=[[8, 1, 1, 6], [1, 7, 5, 1]], seed=49, gamma=0.5, eps=0.2, t_ref=22.0,
    start=[0, 1, 0, 1],
    draws=[(0, 3, 0.8379287921965335), (2, 0, 0.906503715108172), (1, 3, 0.4090126122385679)],
    loads={"A": ([15, 15], [7, 6], [6, 7]), "B": ([13, 17], [9, 6], [6, 9]),
           "C": ([16, 14], [2, 2], [2, 2]), "D": ([17, 13], [7, 8], [8, 7])},
    visited=["B", "C", "D"],            # the swapped state of each iteration
    accepted=[1, 1, 0],                 # B is worse but u < exp(-(T_B - T_A)/theta0); C improves; D is rejected
    final=[0, 1, 1, 0])


def sa_hand_smooth(name):
    """Smoothed objective of a hand-worked state from its loads (scipy's logsumexp, beta = 20, times / 22)."""
    from scipy.special import logsumexp
    comp, tx, rx = (np.array(v, np.float64) / SA_HAND["t_ref"] for v in SA_HAND["loads"][name])
    link = [logsumexp(20.0 * np.array([tx[g], rx[g], 0.0, 0.0])) / 20.0 for g in range(2)]   # no RDMA in one node
    return logsumexp(20.0 * comp) / 20.0 + logsumexp(20.0 * np.array(link)) / 20.0


def check_sa_hand_trace(tr):
    hw = SA_HAND
    assert tr["start"].tolist() == hw["start"] and tr["t_ref"] == hw["t_ref"] and tr["iterations"] == 3
    T = sa_hand_smooth("A")
    assert tr["smooth_start"] == pytest.approx(T, rel=1e-12)
    theta = T
    for i, ((ea, eb, u), name, acc) in enumerate(zip(hw["draws"], hw["visited"], hw["accepted"])):
        Tn = sa_hand_smooth(name)
        # the rule itself, on the hand-worked numbers: better, or u below the Metropolis threshold
        assert acc == int(Tn < T or u < np.exp(-(Tn - T) / theta))
        assert tr["moves"][i].tolist() == [ea, eb, acc]
        assert tr["vals"][i][0] == u
        assert tr["vals"][i][1] == pytest.approx(Tn, rel=1e-12)
        assert tr["vals"][i][2] == pytest.approx(theta, rel=1e-12)
        if acc:
            T = Tn
        theta *= hw["gamma"]
    assert tr["rank"].tolist() == hw["final"]


def test_sa_hand_worked_trajectory():
    hw = SA_HAND
    # the draws written above are what the pinned generator yields
    o = oracle.splitmix64(hw["seed"], 9)
    for i, (ea, eb, u) in enumerate(hw["draws"]):
        assert (int(o[3 * i]) % 4, int(o[3 * i + 1]) % 4) == (ea, eb)
        assert (int(o[3 * i + 2]) >> 11) / 2.0 ** 53 == u
    # the thresholds are not close calls made by rounding: 0.838 < 0.883 (accept), 0.409 > 0.348 (reject)
    TA, TB, TC, TD = (sa_hand_smooth(n) for n in "ABCD")
    assert TB > TA > TC and TD > TC
    assert np.exp(-(TB - TA) / TA) == pytest.approx(0.8834, abs=5e-4)
    assert np.exp(-(TD - TC) / (TA / 4)) == pytest.approx(0.3479, abs=5e-4)
    tr = oracle.reorder_sa_trace(np.array(hw["x"]), 2, np.array([1.0, 1.0, 1.0]), beta=20.0, gamma=hw["gamma"],
                                 eps=hw["eps"], seed=hw["seed"], cap=8)
    check_sa_hand_trace(tr)
    # and the multi-seed call's first seed is that run
    rank, st = oracle.reorder_sa(np.array(hw["x"]), 2, np.array([1.0, 1.0, 1.0]), gamma=hw["gamma"], eps=hw["eps"],
                                 n_seeds=1, seed=hw["seed"])
    assert rank.tolist() == hw["final"] and st["iterations"] == 3 and st["T_start"] == 22.0 and st["T"] == 18.0

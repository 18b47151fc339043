"""CPU-side checks of the product library: it loads, exports what the header declares, the
host planner equals the oracle's plan bit for bit, and bad arguments come back as status codes.
No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import workloads as wl
import paper_2605_08639_amd as rl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "relibra.h")).read()
    declared = set(re.findall(r"\b(relibra_[a-z_]+)\s*\(", header))
    declared -= {"relibra_stream"}
    assert {"relibra_route_hist", "relibra_plan", "relibra_permute", "relibra_moe_ffn_fwd",
            "relibra_moe_ffn_bwd", "relibra_unpermute_combine"} <= declared
    L = ctypes.CDLL(rl.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), name
    assert set(rl.EXPORTS) == declared


def _counts(cfg):
    ids = np.stack([wl.make_routing(cfg, mb)[0] for mb in range(cfg.n_mb)])
    return oracle.route_hist(ids, cfg.E)[0]


PLAN_KEYS = ("expert_to_slot", "replica_expert", "inst_ptr", "inst_rank", "inst_rows", "inst_group",
             "group_expert", "group_offset")


def _assert_same_plan(cfg, counts):
    want = oracle.plan(counts, cfg.EP, cfg.rpn, cfg.r)
    got = rl.relibra_plan(counts, cfg.k, cfg.EP, cfg.rpn, cfg.r)
    for key in PLAN_KEYS:
        assert np.array_equal(got[key], want[key]), key
    assert np.array_equal(got["max_load_before"], want["max_before"])
    assert np.array_equal(got["max_load_after"], want["max_after"])
    # gradient slots follow from the layout: home group -> its expert, replica slot j of rank g -> E + g*r + j
    M, r, E = cfg.M, cfg.r, cfg.E
    for mb in range(counts.shape[0]):
        for grp in range(cfg.G):
            rk, loc = divmod(grp, M + r)
            exp = want["group_expert"][mb, grp] if loc < M else E + rk * r + (loc - M)
            assert got["group_dw_slot"][mb, grp] == exp
    return got


@pytest.mark.parametrize("kw", [
    dict(),
    dict(E=8, k=2, EP=4, r=1, T=512, n_mb=1, routing="single"),
    dict(E=32, k=4, EP=16, r=2, T=300, n_mb=4, ranks_per_node=8),
    dict(E=32, k=4, EP=16, r=1, T=300, n_mb=3, ranks_per_node=4),
    dict(E=24, k=3, EP=4, r=0, T=200, n_mb=2),
    dict(E=16, k=8, EP=8, r=2, T=1000, n_mb=5, routing="stress", zipf_s=1.5),
    dict(E=64, k=6, EP=8, r=3, T=2000, n_mb=6, zipf_s=2.0),
    dict(E=12, k=1, EP=2, r=1, T=50, n_mb=2, ranks_per_node=1),
])
def test_planner_equals_oracle_plan(kw):
    cfg = wl.small_config(**kw)
    _assert_same_plan(cfg, _counts(cfg))


def test_planner_equals_oracle_on_random_histograms():
    rng = np.random.default_rng(42)
    for trial in range(60):
        EP = int(rng.choice([1, 2, 4, 8, 16]))
        M = int(rng.integers(1, 6))
        rpn = int(rng.choice([d for d in (1, 2, 4, 8) if EP % d == 0]))
        cfg = wl.small_config(E=EP * M, EP=EP, k=1, r=int(rng.integers(0, 4)), n_mb=int(rng.integers(1, 4)),
                              ranks_per_node=rpn)
        kind = trial % 3
        if kind == 0:
            counts = rng.integers(0, 50, size=(cfg.n_mb, cfg.E))
        elif kind == 1:
            counts = (rng.zipf(1.3, size=(cfg.n_mb, cfg.E)) % 5000)
        else:
            counts = rng.integers(0, 3, size=(cfg.n_mb, cfg.E)) * 7       # many ties and zeros
        _assert_same_plan(cfg, counts.astype(np.int32))


@pytest.mark.parametrize("idx", [0, 1, 2, 3, 4])
def test_planner_equals_oracle_on_paper_shaped_configs(idx):
    cfg = wl.CONFIGS[idx]
    got = _assert_same_plan(cfg, _counts(cfg))
    assert (got["max_load_after"] <= got["max_load_before"]).all() or cfg.n_mb > 1
    assert got["max_load_after"].sum() <= got["max_load_before"].sum()


def test_plan_argument_errors():
    c = np.zeros((1, 8), np.int32)
    for bad in (dict(EP=3), dict(rpn=3), dict(r=-1), dict(k=0), dict(k=9)):
        args = dict(k=2, EP=4, rpn=4, r=1)
        args.update(bad)
        with pytest.raises(rl.RelibraError) as ei:
            rl.relibra_plan(c, args["k"], args["EP"], args["rpn"], args["r"])
        assert ei.value.status == rl.EINVAL
    c[0, 3] = -1
    with pytest.raises(rl.RelibraError) as ei:
        rl.relibra_plan(c, 2, 4, 4, 1)
    assert ei.value.status == rl.ERANGE


def test_workspace_sizes_and_status_strings():
    assert rl.workspace_bytes(rl.WS_PERMUTE, 512, 2, 8, 12, 128, 256) >= ((1024 + 511) // 512) * 8 * 4
    fwd = rl.workspace_bytes(rl.WS_FFN_FWD, 512, 2, 8, 12, 128, 256)
    bwd = rl.workspace_bytes(rl.WS_FFN_BWD, 512, 2, 8, 12, 128, 256)
    assert bwd >= fwd + 2 * 1024 * 256 * 2                 # room for dGt and dU
    assert rl.workspace_bytes(99, 512, 2, 8, 12, 128, 256) == 0
    assert rl.status_string(rl.OK) == "ok" and "workspace" in rl.status_string(rl.EWORKSPACE)


def test_device_entry_points_reject_bad_sizes_before_touching_the_gpu():
    L = rl.lib()
    z = ctypes.c_void_p(0)
    assert L.relibra_route_hist(z, 1, 4, 2, 0, z, z, z) == rl.EINVAL          # E < 1
    assert L.relibra_route_hist(z, 1, 4, 9, 8, z, z, z) == rl.EINVAL          # k > E
    assert L.relibra_route_hist(z, 0, 4, 2, 8, z, z, z) == rl.OK              # empty batch
    assert L.relibra_permute(z, z, z, z, z, z, 4, 2, 5000, 12, 128, z, z, z, z, ctypes.c_size_t(0), z, z) == rl.EINVAL
    assert L.relibra_permute(z, z, z, z, z, z, 0, 2, 8, 12, 128, z, z, z, z, ctypes.c_size_t(0), z, z) == rl.OK
    assert L.relibra_moe_ffn_fwd(z, 16, z, z, 12, 0, 12, 8, z, z, z, 100, 256, z, z, z, z, 0, z,
                                 ctypes.c_size_t(0), z, z) == rl.EUNSUPPORTED  # h % 64
    assert L.relibra_moe_ffn_fwd(z, 16, z, z, 12, 5, 3, 8, z, z, z, 128, 256, z, z, z, z, 0, z,
                                 ctypes.c_size_t(0), z, z) == rl.EINVAL        # g_begin > g_end
    assert L.relibra_moe_ffn_fwd(z, 16, z, z, 9000, 0, 9000, 8, z, z, z, 128, 256, z, z, z, z, 0, z,
                                 ctypes.c_size_t(0), z, z) == rl.EUNSUPPORTED  # more than 8192 groups in one call
    assert L.relibra_moe_ffn_fwd(z, 16, z, z, 12, 0, 12, 8, z, z, z, 128, 256, z, z, z, z, 2, z,
                                 ctypes.c_size_t(0), z, z) == rl.EINVAL        # unknown flag bit
    assert L.relibra_unpermute_combine(7, z, z, z, z, 4, 2, 128, z, z, z, z, z) == rl.EINVAL
    assert L.relibra_unpermute_combine(0, z, z, z, z, 4, 2, 100, z, z, z, z, z) == rl.EINVAL
    # layer-shared replica buffer push
    assert L.relibra_replica_push(z, z, z, z, 8, 4, 2, 128, 256, 0, z, z) == rl.EINVAL      # no workgroups
    assert L.relibra_replica_push(z, z, z, z, 8, 4, 0, 128, 256, 4, z, z) == rl.OK          # r = 0: nothing to push
    assert L.relibra_replica_push(z, z, z, z, 8, 4, 2, 128, 256, 4, z, z) == rl.EINVAL      # null tensors
    # batched weight gradients
    one = (rl.WgradMb * 1)()
    f = ctypes.c_void_p(0)
    assert L.relibra_moe_ffn_wgrad_batched(one, 0, 16, 12, 10, 8, 128, 256, f, f, f, 0, z, ctypes.c_size_t(0), z, z) == rl.EINVAL
    assert L.relibra_moe_ffn_wgrad_batched(one, rl.MAX_WGRAD_MB + 1, 16, 12, 10, 8, 128, 256, f, f, f, 0, z,
                                           ctypes.c_size_t(0), z, z) == rl.EINVAL
    assert L.relibra_moe_ffn_wgrad_batched(one, 1, 16, 12, 10, 8, 100, 256, f, f, f, 0, z, ctypes.c_size_t(0), z, z) == rl.EUNSUPPORTED
    assert L.relibra_moe_ffn_wgrad_batched(one, 1, 16, 12, 10, 8, 128, 256, f, f, f, 8, z, ctypes.c_size_t(0), z, z) == rl.EINVAL   # unknown flag
    assert L.relibra_moe_ffn_wgrad_batched(one, 1, 16, 12, 10, 8, 128, 256, f, f, f, 6, z, ctypes.c_size_t(0), z, z) == rl.EINVAL   # both tiles
    assert L.relibra_moe_ffn_wgrad_batched(one, 1, 16, 12, 10, 8, 128, 256, f, f, f, 0, z, ctypes.c_size_t(0), z, z) == rl.EINVAL  # null dW
    assert rl.workspace_bytes(rl.WS_WGRAD_BATCHED, 0, 1, 8, 12, 128, 256) > 0
    # gate-fused forward / backward
    assert L.relibra_row_gates(z, z, -1, z, z, z) == rl.EINVAL
    assert L.relibra_row_gates(z, z, 0, z, z, z) == rl.OK
    assert L.relibra_row_gates(z, z, 8, z, z, z) == rl.EINVAL                               # null tensors
    assert L.relibra_moe_ffn_fwd_gated(z, 4, z, z, 16, z, z, 12, 0, 12, 8, z, z, z, 128, 256, z, z, z, z, z, 0, z,
                                       ctypes.c_size_t(0), z, z) == rl.EINVAL               # no row table, no gates
    sz = ctypes.c_size_t(0)
    assert L.relibra_moe_ffn_bwd_gated(z, 4, z, z, z, z, z, 16, z, z, z, 12, 0, 12, 8, 8, z, z, z, 128, 256, z, f, 1, z, sz, z, sz,
                                       z, z) == rl.EINVAL                                   # a flag of the ungated call only
    assert L.relibra_moe_ffn_bwd_gated(z, 4, z, z, z, z, z, 16, z, z, z, 12, 0, 12, 8, 8, z, z, z, 100, 256, z, f, 0, z, sz, z, sz,
                                       z, z) == rl.EUNSUPPORTED                             # h % 64
    assert L.relibra_moe_ffn_bwd_gated(z, 4, z, z, z, z, z, 16, z, z, z, 12, 0, 12, 8, 8, z, z, z, 128, 256, z, f, 0, z, sz, z, sz,
                                       z, z) == rl.EINVAL                                   # null tensors
    # partial row sums of dgate: four per row and 256-column tile of h'
    assert rl.workspace_bytes(rl.WS_DGATE, 512, 2, 8, 12, 128, 768) >= 4 * 3 * 1024 * 4


# ------------------------------------------------------------------ communication-aware model, Algorithm 1
def _src_hist(cfg):
    return sum(oracle.route_hist_src(wl.make_routing(cfg, mb)[0], cfg.E, cfg.EP) for mb in range(cfg.n_mb))


def _skewed_sources(seed, E, EP):
    rng = np.random.default_rng(seed)
    aff = rng.permutation(np.repeat(np.arange(EP), E // EP))
    x = rng.integers(5, 30, size=(EP, E)).astype(np.int64)
    for e in range(E):
        x[aff[e], e] += rng.integers(300, 600)
    return x


@pytest.mark.parametrize("EP,rpn,E", [(4, 2, 8), (8, 4, 32), (8, 8, 16), (16, 4, 64)])
def test_moe_time_equals_oracle(EP, rpn, E):
    """Eq. 1-6: integer loads identical, times and the smoothed objective to rounding."""
    rng = np.random.default_rng(E + EP)
    x = rng.integers(0, 5000, size=(EP, E)).astype(np.int64)
    rank_of = rng.permutation(np.repeat(np.arange(EP), E // EP)).astype(np.int32)
    m_or = oracle.cost_model(2048, 768, 5e14, 1.0e12, 5e10)
    m_lib = rl.cost_model(EP, rpn, 2048, 768, 5e14, 1.0e12, 5e10)
    for t_ref in (1.0, 3e-4):
        want = oracle.moe_time(x, rank_of, rpn, m_or, beta=20.0, t_ref=t_ref)
        got = rl.relibra_moe_time(x, rank_of, m_lib, beta=20.0, t_ref=t_ref, with_loads=True)
        for a, b in zip(got["loads"], oracle.loads(x, rank_of, rpn)):
            assert np.array_equal(a, b)
        for key in ("T", "T_comp", "T_comm", "smooth"):
            assert got[key] == pytest.approx(want[key], rel=1e-12), key


def test_reorder_sa_hand_worked_trajectory():
    """The library's Algorithm 1 on the hand-worked instance of tests/test_oracle_comm.py: draws,
    accept/reject sequence, objective values, cooling and final placement."""
    from test_oracle_comm import SA_HAND as hw, check_sa_hand_trace
    m = rl.CostModel(2, 2, 1.0, 1.0, 1.0)
    tr = rl.relibra_reorder_sa_trace(np.array(hw["x"]), m, gamma=hw["gamma"], eps=hw["eps"], seed=hw["seed"], cap=8)
    check_sa_hand_trace(tr)
    rank, st = rl.relibra_reorder_sa(np.array(hw["x"]), m, gamma=hw["gamma"], eps=hw["eps"], n_seeds=1, seed=hw["seed"])
    assert rank.tolist() == hw["final"] and st["iterations"] == 3 and st["T_start"] == 22.0 and st["T"] == 18.0


def test_reorder_sa_equals_oracle():
    """Algorithm 1 in the library (incremental O(|G|) state update, one thread per seed) against the
    oracle (objective recomputed from the definition at every step): same generator, same rule,
    so the same trajectory (every move and accept/reject decision of the first seed; objective
    values to rounding) and the same final placement."""
    for seed, (E, EP, rpn) in enumerate([(32, 8, 4), (16, 4, 2), (64, 8, 8)]):
        x = _skewed_sources(seed, E, EP)
        m_or = oracle.cost_model(2048, 768, 5e14, 1.0e12, 5e10)
        m_lib = rl.cost_model(EP, rpn, 2048, 768, 5e14, 1.0e12, 5e10)
        assert [m_lib.sec_per_token_comp, m_lib.sec_per_token_intra, m_lib.sec_per_token_inter] == pytest.approx(m_or.tolist(), rel=1e-15)
        t_or = oracle.reorder_sa_trace(x, rpn, m_or, gamma=0.999, eps=1e-3, seed=11, cap=4096)
        t_lib = rl.relibra_reorder_sa_trace(x, m_lib, gamma=0.999, eps=1e-3, seed=11, cap=4096)
        assert t_lib["iterations"] == t_or["iterations"] and len(t_or["moves"]) == 4096
        assert np.array_equal(t_lib["moves"], t_or["moves"])
        assert np.array_equal(t_lib["vals"][:, 0], t_or["vals"][:, 0])
        assert np.allclose(t_lib["vals"], t_or["vals"], rtol=1e-10, atol=0)
        assert np.array_equal(t_lib["start"], t_or["start"]) and np.array_equal(t_lib["rank"], t_or["rank"])
        assert 0 < t_or["moves"][:, 2].sum() < 4096            # both outcomes occur
        r_or, s_or = oracle.reorder_sa(x, rpn, m_or, gamma=0.999, eps=1e-3, n_seeds=4, seed=11)
        r_lib, s_lib = rl.relibra_reorder_sa(x, m_lib, gamma=0.999, eps=1e-3, n_seeds=4, seed=11)
        assert np.array_equal(r_lib, r_or)
        assert sorted(np.bincount(r_lib, minlength=EP).tolist()) == [E // EP] * EP
        assert s_lib["T_start"] == pytest.approx(s_or["T_start"], rel=1e-12)
        assert s_lib["smooth"] <= s_lib["smooth_start"]
        assert s_lib["iterations"] == s_or["iterations"]
        assert s_lib["T"] == pytest.approx(s_or["T"], rel=1e-12)
        again, s2 = rl.relibra_reorder_sa(x, m_lib, gamma=0.999, eps=1e-3, n_seeds=4, seed=11)
        assert np.array_equal(again, r_lib) and s2 == s_lib


def test_cost_model_init_follows_eq4_eq5():
    """6hh'/F seconds of computation per token (three GEMMs of 2hh' flops, Eq. 4) and one hidden vector of
    bf16 values over each link (Eq. 5), on numbers that divide evenly."""
    m = rl.cost_model(8, 4, 1024, 512, 2.0 ** 40, 2.0 ** 30, 2.0 ** 20)
    assert (m.EP, m.ranks_per_node) == (8, 4)
    assert m.sec_per_token_comp == 6 * 2.0 ** 19 / 2.0 ** 40
    assert m.sec_per_token_intra == 2048 / 2.0 ** 30 and m.sec_per_token_inter == 2048 / 2.0 ** 20
    for bad in (dict(EP=8, ranks_per_node=3), dict(F=0.0), dict(h=0)):
        kw = dict(EP=8, ranks_per_node=4, h=64, hff=64, F=1e12, B_intra=1e11, B_inter=1e10)
        kw.update(bad)
        with pytest.raises(rl.RelibraError):
            rl.cost_model(**kw)


def test_plan_placed_equals_oracle_under_the_annealed_placement():
    """Stage 2 under a placement found by Algorithm 1: every table bit-exact against the oracle."""
    cfg = wl.small_config(E=32, k=4, EP=8, r=2, T=1024, n_mb=3, ranks_per_node=4)
    counts = _counts(cfg)
    x = _src_hist(cfg)
    assert np.array_equal(x.sum(0), counts.sum(0))
    rank, _ = rl.relibra_reorder_sa(x, rl.cost_model(cfg.EP, cfg.rpn, cfg.h, cfg.hff, 5e14, 1e12, 5e10),
                                    gamma=0.995, eps=1e-2, n_seeds=2, seed=3)
    want = oracle.plan(counts, cfg.EP, cfg.rpn, cfg.r, placed=rank)
    got = rl.relibra_plan(counts, cfg.k, cfg.EP, cfg.rpn, cfg.r, expert_rank=rank)
    for key in PLAN_KEYS:
        assert np.array_equal(got[key], want[key]), key
    assert np.array_equal(got["max_load_after"], want["max_after"])
    assert np.array_equal(got["expert_to_slot"] // cfg.M, rank)
    bad = rank.copy()
    bad[0] = bad[1] = bad[2] = bad[3] = bad[4] = 0            # five experts on a rank that holds four
    with pytest.raises(rl.RelibraError):
        rl.relibra_plan(counts, cfg.k, cfg.EP, cfg.rpn, cfg.r, expert_rank=bad)


def test_comm_model_argument_errors():
    x = np.ones((4, 8), np.int64)
    rank = np.repeat(np.arange(4), 2).astype(np.int32)
    m = rl.cost_model(4, 2, 64, 64, 1e12, 1e11, 1e10)
    with pytest.raises(rl.RelibraError):
        rl.relibra_reorder_sa(x, m, gamma=1.0)
    with pytest.raises(rl.RelibraError):
        rl.relibra_reorder_sa(x, m, n_seeds=0)
    with pytest.raises(rl.RelibraError):
        rl.relibra_moe_time(-x, rank, m)
    with pytest.raises(rl.RelibraError):
        rl.relibra_moe_time(x, rank + 3, m)
    with pytest.raises(rl.RelibraError):
        rl.relibra_moe_time(x, rank, rl.cost_model(4, 3, 64, 64, 1e12, 1e11, 1e10))


@pytest.mark.parametrize("kw", [dict(E=16, k=2, EP=4, r=2, T=240, ranks_per_node=2),
                                dict(E=32, k=4, EP=8, r=1, T=512, ranks_per_node=4),
                                dict(E=128, k=8, EP=8, r=2, T=2048, ranks_per_node=8),
                                dict(E=64, k=4, EP=16, r=2, T=1024, ranks_per_node=4, routing="stress", zipf_s=1.5)])
def test_source_aware_split_and_its_times_equal_oracle(kw):
    """Section 5.2 split per source: integer tables identical to the oracle's, Eq. 1-6 on the split
    identical in loads and equal to rounding in times; the split never raises the modelled time's
    intra-node part over the token-order split's."""
    cfg = wl.small_config(n_mb=2, h=64, hff=64, **kw)
    ids = np.stack([wl.make_routing(cfg, mb)[0] for mb in range(cfg.n_mb)])
    counts, _ = oracle.route_hist(ids, cfg.E)
    p = rl.relibra_plan(counts, cfg.k, cfg.EP, cfg.rpn, cfg.r)
    m_or = oracle.cost_model(2048, 768, 5e14, 4e11, 5e10)
    m_lib = rl.cost_model(cfg.EP, cfg.rpn, 2048, 768, 5e14, 4e11, 5e10)
    for mb in range(cfg.n_mb):
        x = oracle.route_hist_src(ids[mb], cfg.E, cfg.EP)
        ptr, rank, rows = p["inst_ptr"][mb], p["inst_rank"][mb], p["inst_rows"][mb]
        n_inst = ptr[-1]
        want = oracle.assign_sources(x, cfg.rpn, ptr, rank, rows)
        got = rl.relibra_assign_sources(x, cfg.rpn, ptr, rank, rows)
        assert np.array_equal(got["inst_src_rows"][:n_inst], want[:n_inst])
        assert np.array_equal(got["inst_src_base"][:n_inst], np.cumsum(want[:n_inst], axis=1) - want[:n_inst])
        assert np.array_equal(got["src_first"], np.cumsum(x, axis=0) - x)
        t_or, l_or = oracle.moe_time_split(want[:n_inst], rank[:n_inst], cfg.rpn, m_or)
        t_lib = rl.relibra_moe_time_split(got["inst_src_rows"][:n_inst], rank[:n_inst], m_lib, with_loads=True)
        assert np.array_equal(t_lib["loads"], l_or)
        for key in ("T", "T_comp", "T_comm"):
            assert t_lib[key] == pytest.approx(t_or[key], rel=1e-12)


@pytest.mark.parametrize("kw", [dict(E=16, k=2, EP=4, r=2, T=240, ranks_per_node=2),
                                dict(E=32, k=4, EP=8, r=1, T=512, ranks_per_node=4),
                                dict(E=128, k=8, EP=8, r=2, T=2048, ranks_per_node=8),
                                dict(E=64, k=4, EP=16, r=2, T=1024, ranks_per_node=4, routing="stress", zipf_s=1.5)])
def test_timed_plan_equals_oracle(kw):
    """Algorithm 2 driven by T_MoE,g: every table identical to the oracle's, times equal to rounding;
    under an identity placement and under an annealed one."""
    cfg = wl.small_config(n_mb=3, h=64, hff=64, **kw)
    ids = np.stack([wl.make_routing(cfg, mb)[0] for mb in range(cfg.n_mb)])
    x = np.stack([oracle.route_hist_src(ids[mb], cfg.E, cfg.EP) for mb in range(cfg.n_mb)])
    m_or = oracle.cost_model(2048, 768, 5e14, 4e11, 5e10)
    m_lib = rl.cost_model(cfg.EP, cfg.rpn, 2048, 768, 5e14, 4e11, 5e10)
    ident = (np.arange(cfg.E) // cfg.M).astype(np.int32)
    annealed, _ = rl.relibra_reorder_sa(x.sum(0), m_lib, n_seeds=2, seed=3)
    for placed in (ident, annealed):
        want = oracle.plan_comm(x, cfg.rpn, cfg.r, placed, m_or)
        got = rl.relibra_plan_timed(x, cfg.k, m_lib, cfg.r, placed)
        for key in ("expert_to_slot", "replica_expert", "inst_ptr", "inst_rank", "inst_rows", "inst_group",
                    "group_expert", "group_offset"):
            assert np.array_equal(got[key], want[key]), key
        assert np.array_equal(got["max_load_after"], want["max_after"])
        assert np.allclose(got["t_before"], want["t_before"], rtol=1e-12)
        assert np.allclose(got["t_after"], want["t_after"], rtol=1e-12)
        assert (got["t_after"] <= got["t_before"]).all()
        # the tables are a valid plan: group sizes add up and every slot index is in range
        assert (got["group_offset"][:, -1] == cfg.T * cfg.k).all()
        assert ((got["group_dw_slot"] >= 0) & (got["group_dw_slot"] < cfg.E + cfg.EP * cfg.r)).all()


def test_timed_plan_argument_errors():
    x = np.ones((1, 4, 8), np.int64)
    m = rl.cost_model(4, 2, 64, 64, 1e12, 1e11, 1e10)
    rank = np.repeat(np.arange(4), 2).astype(np.int32)
    rl.relibra_plan_timed(x, 2, m, 1, rank)
    with pytest.raises(rl.RelibraError):
        rl.relibra_plan_timed(x, 2, m, 1, np.zeros(8, np.int32))         # more than M experts on a rank
    with pytest.raises(rl.RelibraError):
        rl.relibra_plan_timed(-x, 2, m, 1, rank)
    with pytest.raises(rl.RelibraError):
        rl.relibra_plan_timed(x, 2, m, -1, rank)


def test_source_aware_split_degenerate_cases():
    """Experts without tokens, a source without tokens, one token per source, a single rank."""
    # E = 4 on EP = 2 ranks of one node; expert 1 and source 1 are empty; expert 0 has a replica on rank 1
    x = np.array([[6, 0, 2, 1], [0, 0, 0, 0]], np.int64)
    ptr, rank, rows = [0, 2, 3, 4, 5], [0, 1, 0, 1, 1], [2, 4, 0, 2, 1]
    got = rl.relibra_assign_sources(x, 2, ptr, rank, rows)
    want = oracle.assign_sources(x, 2, ptr, rank, rows)
    assert np.array_equal(got["inst_src_rows"], want)
    assert got["inst_src_rows"].tolist() == [[2, 0], [4, 0], [0, 0], [2, 0], [1, 0]]
    # a single rank: everything is a local copy, no link is loaded
    x1 = np.array([[5, 7, 0]], np.int64)
    one = rl.relibra_assign_sources(x1, 1, [0, 1, 2, 3], [0, 0, 0], [5, 7, 0])
    t = rl.relibra_moe_time_split(one["inst_src_rows"], [0, 0, 0], rl.cost_model(1, 1, 64, 64, 1e12, 1e11, 1e10), with_loads=True)
    assert t["loads"].tolist() == [[12], [0], [0], [0], [0]] and t["T_comm"] == 0.0


def test_source_aware_split_argument_errors():
    x = np.array([[3], [1]], np.int64)
    with pytest.raises(rl.RelibraError):
        rl.relibra_assign_sources(x, 2, [0, 1], [0], [5])              # sizes do not add up
    with pytest.raises(rl.RelibraError):
        rl.relibra_assign_sources(x, 3, [0, 1], [0], [4])              # EP % ranks_per_node
    with pytest.raises(rl.RelibraError):
        rl.relibra_assign_sources(x, 2, [0, 1], [7], [4])              # rank out of range
    ok = rl.relibra_assign_sources(x, 2, [0, 1], [0], [4])
    assert ok["inst_src_rows"].tolist() == [[3, 1]] and ok["inst_src_base"].tolist() == [[0, 3]]
    m = rl.cost_model(2, 2, 64, 64, 1e12, 1e11, 1e10)
    with pytest.raises(rl.RelibraError):
        rl.relibra_moe_time_split(np.array([[1, -1]], np.int32), [0], m)
    L = rl.lib()
    z = ctypes.c_void_p(0)
    assert L.relibra_permute_src(z, z, z, z, 3, z, z, z, z, 8, 2, 4, 6, 0, z, z, z, z, ctypes.c_size_t(0), z, z) == rl.EINVAL  # T % EP
    assert L.relibra_permute_src(z, z, z, z, 4, z, z, z, z, 0, 2, 4, 6, 0, z, z, z, z, ctypes.c_size_t(0), z, z) == rl.OK      # empty


def test_load_stats_equal_oracle():
    for idx in (0, 1, 4):
        cfg = wl.CONFIGS[idx]
        counts = _counts(cfg)
        for top in (1, 4, min(8, cfg.E)):
            s_lib, i_lib = rl.relibra_load_stats(counts, top)
            s_or, i_or = oracle.load_stats(counts, top)
            assert np.allclose(s_lib, s_or, rtol=1e-14, atol=0) and np.array_equal(i_lib, i_or)
    with pytest.raises(rl.RelibraError):
        rl.relibra_load_stats(np.ones((2, 4), np.int32), top=5)

"""Pins of the oracle's source-aware token split (Section 5.2, y_{j,e,g}), of the cost model
evaluated on a split (Section 4.1, Eq. 1-6) and of the permutation that honours the split,
against things other than themselves: a hand-worked example on the two-node two-GPU topology of
Section 4.1, brute force over every feasible split of tiny cases, the already pinned
whole-expert cost model and permutation as the special case without replicas, and invariants."""
import itertools

import numpy as np
import pytest

import oracle
import workloads as wl

LOC, NV, SR, CR = 0, 1, 2, 3
TAU_2x2 = [[LOC, NV, SR, CR],          # Section 4.1's example: tau[source][destination]
           [NV, LOC, CR, SR],
           [SR, CR, LOC, NV],
           [CR, SR, NV, LOC]]


def test_hand_worked_split_and_times_on_the_two_node_example():
    """One expert, home rank 0, replica on rank 1, 7 tokens each; sources hold 5, 3, 4, 2 tokens.
    Rank 0 keeps its own 5 and takes 2 of source 2 (same rail); rank 1 keeps its own 3, takes the 2
    of source 3 (same rail) and the 2 that are left of source 2 (cross rail: one relay hop).
    Loads by hand: intra-node link send [0,0,2,0], receive [0,2,0,0]; RDMA send [0,0,4,2], receive
    [2,4,0,0].  With 1 s per computed token, 0.5 s per token on the intra-node link and 2 s on
    RDMA: T_comp = 7, T_comm = max(4, 8, 8, 4) = 8, T_MoE = 15."""
    x = np.array([[5], [3], [4], [2]], np.int64)
    inst_ptr, inst_rank, inst_rows = [0, 2], [0, 1], [7, 7]
    y = oracle.assign_sources(x, 2, inst_ptr, inst_rank, inst_rows)
    assert y.tolist() == [[5, 0, 2, 0], [0, 3, 2, 2]]
    t, loads = oracle.moe_time_split(y, inst_rank, 2, [1.0, 0.5, 2.0])
    assert loads.tolist() == [[7, 7, 0, 0], [0, 0, 2, 0], [0, 2, 0, 0], [0, 0, 4, 2], [2, 4, 0, 0]]
    assert (t["T_comp"], t["T_comm"], t["T"]) == (7.0, 8.0, 15.0)


def link_volumes(y, inst_rank, tau):
    nv = rd = 0
    for i, g in enumerate(inst_rank):
        for j, n in enumerate(y[i]):
            nv += n * (tau[j][g] in (NV, CR))
            rd += n * (tau[j][g] in (SR, CR))
    return nv, rd


@pytest.mark.parametrize("seed", range(12))
def test_split_has_the_smallest_intra_node_volume_of_all_feasible_splits(seed):
    """Brute force on the 2 x 2 topology: an expert with instances on both ranks of node 0, every
    integer split with the given instance sizes enumerated; the oracle's split must reach the
    minimum number of tokens crossing the intra-node link, and the RDMA volume must be the same
    for all of them."""
    rng = np.random.default_rng(seed)
    xs = rng.integers(0, 5, size=4)
    total = int(xs.sum())
    rows0 = int(rng.integers(0, total + 1))
    inst_rank, inst_rows = [0, 1], [rows0, total - rows0]
    best, rdma = None, set()
    for y0 in itertools.product(*[range(int(v) + 1) for v in xs]):
        if sum(y0) != rows0:
            continue
        y = [list(y0), [int(v) - a for v, a in zip(xs, y0)]]
        nv, rd = link_volumes(y, inst_rank, TAU_2x2)
        rdma.add(rd)
        best = nv if best is None else min(best, nv)
    got = oracle.assign_sources(xs.reshape(4, 1).astype(np.int64), 2, [0, 2], inst_rank, inst_rows)
    assert got.sum(axis=0).tolist() == xs.tolist() and got.sum(axis=1).tolist() == inst_rows
    assert link_volumes(got.tolist(), inst_rank, TAU_2x2)[0] == best
    assert len(rdma) == 1


def planned(cfg, mb=0):
    ids, _ = wl.make_routing(cfg, mb)
    counts = oracle.route_hist(ids[None], cfg.E)[0]
    p = oracle.plan(counts, cfg.EP, cfg.rpn, cfg.r)
    x = oracle.route_hist_src(ids, cfg.E, cfg.EP)
    return ids, p, x


@pytest.mark.parametrize("E,k,EP,rpn,r,T", [(16, 2, 4, 2, 2, 240), (32, 4, 8, 4, 1, 512), (8, 2, 8, 8, 2, 96)])
def test_split_conserves_tokens_and_never_moves_more_over_the_intra_node_link(E, k, EP, rpn, r, T):
    cfg = wl.small_config(E=E, k=k, EP=EP, r=r, T=T, n_mb=1, h=64, hff=64, ranks_per_node=rpn)
    ids, p, x = planned(cfg)
    ptr, rank, rows = p["inst_ptr"][0], p["inst_rank"][0], p["inst_rows"][0]
    y = oracle.assign_sources(x, rpn, ptr, rank, rows)
    n_inst = ptr[-1]
    assert (y[:n_inst].sum(axis=1) == rows[:n_inst]).all()
    for e in range(E):
        assert (y[ptr[e]:ptr[e + 1]].sum(axis=0) == x[:, e]).all()
    # the split in token order (what the plain permutation does): sources fill instances in turn
    y_plain = np.zeros_like(y)
    for e in range(E):
        i, room = ptr[e], rows[ptr[e]] if ptr[e + 1] > ptr[e] else 0
        for j in range(EP):
            n = int(x[j, e])
            while n:
                while room == 0:
                    i += 1
                    room = rows[i]
                m = min(n, room)
                y_plain[i, j] += m
                n -= m
                room -= m
    model = oracle.cost_model(2048, 768, 5e14, 4e11, 5e10)
    t_a, l_a = oracle.moe_time_split(y[:n_inst], rank[:n_inst], rpn, model)
    t_p, l_p = oracle.moe_time_split(y_plain[:n_inst], rank[:n_inst], rpn, model)
    assert (l_a[0] == l_p[0]).all()                            # same computation loads
    assert l_a[1].sum() <= l_p[1].sum()                        # never more intra-node traffic
    assert l_a[3].sum() == l_p[3].sum()                        # RDMA volume is not affected


def test_split_times_reduce_to_the_whole_expert_model_without_replicas():
    """One instance per expert: the split model must give what the (separately pinned) placement
    model gives."""
    rng = np.random.default_rng(5)
    EP, rpn, E = 8, 4, 16
    x = rng.integers(0, 50, size=(EP, E)).astype(np.int64)
    rank_of = rng.permutation(np.repeat(np.arange(EP), E // EP)).astype(np.int32)
    model = oracle.cost_model(1024, 512, 4e14, 3e11, 4e10)
    y = x.T.copy()                                             # instance e = expert e, all sources
    t, loads = oracle.moe_time_split(y, rank_of, rpn, model)
    want = oracle.moe_time(x, rank_of, rpn, model)
    assert np.isclose(t["T"], want["T"], rtol=1e-15) and np.isclose(t["T_comm"], want["T_comm"], rtol=1e-15)
    for got, ref in zip(loads, oracle.loads(x, rank_of, rpn)):
        assert (got == ref).all()


@pytest.mark.parametrize("E,k,EP,rpn,r,T", [(16, 2, 4, 2, 2, 240), (32, 4, 8, 4, 1, 512)])
def test_source_aware_permutation_is_a_bijection_that_realises_the_split(E, k, EP, rpn, r, T):
    cfg = wl.small_config(E=E, k=k, EP=EP, r=r, T=T, n_mb=1, h=64, hff=64, ranks_per_node=rpn)
    ids, p, x = planned(cfg)
    ptr, rank, rows, grp, off = (p[key][0] for key in ("inst_ptr", "inst_rank", "inst_rows", "inst_group", "group_offset"))
    y = oracle.assign_sources(x, rpn, ptr, rank, rows)
    row_of, src_of = oracle.permute_src(ids, E, EP, ptr, grp, off, y)
    N = T * k
    assert sorted(row_of.tolist()) == list(range(N))
    assert (src_of[row_of] == np.arange(N)).all()
    flat = ids.reshape(-1)
    per = T // EP
    for e in range(E):
        for i in range(ptr[e], ptr[e + 1]):
            lo = off[grp[i]]
            srcs = src_of[lo:lo + rows[i]]
            assert (flat[srcs] == e).all()
            js = (srcs // k) // per
            assert (np.bincount(js, minlength=EP) == y[i]).all()
            assert (np.diff(js) >= 0).all()                    # source after source
            for j in range(EP):
                assert (np.diff(srcs[js == j]) > 0).all()      # ascending inside a source


def test_source_aware_permutation_without_replicas_is_the_plain_permutation():
    cfg = wl.small_config(E=16, k=2, EP=4, r=0, T=200, n_mb=1, h=64, hff=64, ranks_per_node=2)
    ids, p, x = planned(cfg)
    ptr, rank, rows, grp, off = (p[key][0] for key in ("inst_ptr", "inst_rank", "inst_rows", "inst_group", "group_offset"))
    y = oracle.assign_sources(x, 2, ptr, rank, rows)
    a = oracle.permute_src(ids, 16, 4, ptr, grp, off, y)
    b = oracle.permute(ids, 16, ptr, rows, grp, off)
    assert (a[0] == b[0]).all() and (a[1] == b[1]).all()


def test_assign_sources_rejects_instance_sizes_that_do_not_add_up():
    x = np.array([[3], [1]], np.int64)
    with pytest.raises(ValueError):
        oracle.assign_sources(x, 2, [0, 1], [0], [5])


# ------------------------------------------------------------------ Algorithm 2 with the time of Section 4.1 as objective
def _inst_tables(z, a):
    E, EP = z.shape
    ptr, rank, rows = [0], [], []
    for e in range(E):
        for g in range(EP):
            if z[e, g]:
                rank.append(g)
                rows.append(int(a[e, g]))
        ptr.append(len(rank))
    return np.array(ptr, np.int32), np.array(rank, np.int32), np.array(rows, np.int32)


def _time_of(x, z, a, rpn, model):
    ptr, rank, rows = _inst_tables(z, a)
    y = oracle.assign_sources(x, rpn, ptr, rank, rows)
    return oracle.moe_time_split(y[:len(rank)], rank, rpn, model)[0]["T"]


def _hot_instance(seed, EP, E):
    rng = np.random.default_rng(seed)
    x = rng.integers(0, 30, size=(EP, E)).astype(np.int64)
    x[:, rng.integers(0, E)] += rng.integers(50, 150, size=EP)
    return x, np.repeat(np.arange(EP), E // EP).astype(np.int32)


@pytest.mark.parametrize("seed", range(10))
def test_time_aware_replication_reaches_the_brute_force_optimum_on_tiny_instances(seed):
    """Two nodes of two GPUs, eight experts, one replica slot per GPU: every placement of at most
    one replica per GPU is enumerated, each with the balanced split (pinned on its own) and the
    time of Eq. 1-6 on the source-aware split (pinned on its own); the greedy loop must end at the
    smallest T_MoE among them."""
    EP, rpn, E, r = 4, 2, 8, 1
    model = [1.0, 0.3, 1.5]
    x, rank_of = _hot_instance(seed, EP, E)
    z, a, st = oracle.replicate_comm(x, rank_of, rpn, r, model)
    assert st["T_after"] == pytest.approx(_time_of(x, z, a, rpn, model), rel=1e-12)
    best = None
    options = [[None] + [e for e in range(E) if rank_of[e] // rpn == g // rpn and rank_of[e] != g] for g in range(EP)]
    for choice in itertools.product(*options):
        zz = np.zeros((E, EP), np.uint8)
        aa = np.zeros((E, EP), np.int64)
        for e in range(E):
            zz[e, rank_of[e]] = 1
            aa[e, rank_of[e]] = x[:, e].sum()
        for g, e in enumerate(choice):
            if e is not None:
                zz[e, g] = 1
        for nd in range(EP // rpn):
            ex = [e for e in range(E) if rank_of[e] // rpn == nd]
            an = oracle.balance_split(zz[ex][:, nd * rpn:(nd + 1) * rpn].copy(), aa[ex][:, nd * rpn:(nd + 1) * rpn].copy())
            for i, e in enumerate(ex):
                aa[e, nd * rpn:(nd + 1) * rpn] = an[i]
        t = _time_of(x, zz, aa, rpn, model)
        best = t if best is None else min(best, t)
    assert st["T_after"] <= best * (1 + 1e-12)
    assert st["T_after"] <= st["T_before"]


@pytest.mark.parametrize("EP,rpn,E,r,seed", [(4, 2, 16, 2, 0), (8, 4, 32, 1, 1), (8, 8, 16, 2, 2), (16, 4, 64, 2, 3)])
def test_time_aware_replication_invariants(EP, rpn, E, r, seed):
    x, rank_of = _hot_instance(seed, EP, E)
    rng = np.random.default_rng(seed + 100)
    rank_of = rng.permutation(rank_of).astype(np.int32)
    model = oracle.cost_model(2048, 768, 5e14, 4e11, 5e10)
    z, a, st = oracle.replicate_comm(x, rank_of, rpn, r, model)
    assert (a.sum(axis=1) == x.sum(axis=0)).all()                           # every token served once
    assert (a[z == 0] == 0).all() and (a >= 0).all()
    for e in range(E):
        assert z[e, rank_of[e]] == 1                                        # the home copy stays
        assert all(g // rpn == rank_of[e] // rpn for g in np.flatnonzero(z[e]))   # replicas stay in the node
    replicas = z.sum(axis=0) - np.bincount(rank_of, minlength=EP)
    assert (replicas <= r).all()
    assert st["T_after"] <= st["T_before"]
    assert st["max_load"] == a.sum(axis=0).max()


@pytest.mark.parametrize("seed", range(6))
def test_time_aware_replication_without_communication_cost_balances_like_the_load_only_one(seed):
    """With free communication T_MoE is the largest computation load: the loop must then end no
    higher than the load-only Algorithm 2 (whose result is pinned to the brute-force optimum)."""
    EP, rpn, E, r = 4, 4, 16, 2
    x, rank_of = _hot_instance(seed, EP, E)
    cnt = x.sum(axis=0)
    z, a, st = oracle.replicate_comm(x, rank_of, rpn, r, [1.0, 0.0, 0.0])
    _, _, peak = oracle.replicate_node(cnt, rank_of, rpn, r)
    assert st["max_load"] <= peak
    assert st["max_load"] >= -(-int(cnt.sum()) // EP)

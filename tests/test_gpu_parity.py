"""GPU parity: every entry point of the C-ABI library against the CPU oracle on the same seeded
inputs.  Integer results (counts, plans, permutation indices, gathered rows) must be bit-exact;
floating-point results must be within relative L2 5e-3 of the oracle, which computes in double
precision on the same bf16-rounded inputs."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_2605_08639_amd as rl

pytestmark = pytest.mark.gpu
TOL = 5e-3
DEV = "cuda"


def rel_l2(got, want):
    got = got.double().cpu().numpy() if torch.is_tensor(got) else np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    den = np.linalg.norm(want)
    return float(np.linalg.norm(got - want) / den) if den > 0 else float(np.linalg.norm(got))


def dev_i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(DEV)


def routing(cfg):
    ids, gates = zip(*[wl.make_routing(cfg, mb) for mb in range(cfg.n_mb)])
    return np.stack(ids), np.stack(gates)


# ------------------------------------------------------------------ histogram
@pytest.mark.parametrize("kw", [
    dict(), dict(T=513, k=3, E=12, EP=4),                       # T*k not a multiple of 4: scalar loads
    dict(T=20000, k=8, E=256, EP=8, n_mb=2), dict(T=1, k=1, E=4, EP=4, n_mb=1)])
def test_route_hist_bit_exact(kw):
    cfg = wl.small_config(**kw)
    ids, _ = routing(cfg)
    want, _ = oracle.route_hist(ids, cfg.E)
    err = rl.new_err_flag()
    got = rl.relibra_route_hist(torch.from_numpy(ids).to(DEV), cfg.E, err_flag=err)
    assert np.array_equal(got.cpu().numpy(), want)
    assert err.item() == 0


def test_route_hist_flags_bad_ids_and_handles_empty():
    ids = torch.zeros((1, 64, 2), dtype=torch.int32, device=DEV)
    ids[0, 5, 1] = 9
    ids[0, 6, 0] = -1
    err = rl.new_err_flag()
    got = rl.relibra_route_hist(ids, 8, err_flag=err)
    assert err.item() == rl.ERR_ID_RANGE
    assert got.sum().item() == 126 and got[0, 0].item() == 126
    got = rl.relibra_route_hist(torch.zeros((2, 0, 2), dtype=torch.int32, device=DEV), 8)
    assert got.shape == (2, 8) and got.sum().item() == 0


def test_per_source_histogram_bit_exact():
    """x[j][e] of Section 4.1 (tokens on source rank j routed to e): the histogram kernel on the ids
    viewed as [n_mb*EP, T/EP, k] against the oracle's definition."""
    cfg = wl.small_config(T=1024, k=4, E=32, EP=8, n_mb=2)
    ids, _ = routing(cfg)
    err = rl.new_err_flag()
    got = rl.relibra_route_hist_src(torch.from_numpy(ids).to(DEV), cfg.E, cfg.EP, err_flag=err).cpu().numpy()
    assert err.item() == 0 and got.shape == (cfg.n_mb, cfg.EP, cfg.E)
    for mb in range(cfg.n_mb):
        assert np.array_equal(got[mb], oracle.route_hist_src(ids[mb], cfg.E, cfg.EP))


def test_histograms_of_several_layers_in_one_launch():
    """Replayed routing of every layer is known before training (Section 3): the histograms of
    [layers, n_mb] micro-batches come from one launch over ids of [layers * n_mb, T, k]."""
    layers = 3
    cfgs = [wl.small_config(T=640, k=4, E=64, EP=8, n_mb=4, index=90 + l) for l in range(layers)]
    ids = np.concatenate([routing(c)[0] for c in cfgs])                    # [layers * n_mb, T, k]
    got = rl.relibra_route_hist(torch.from_numpy(ids).to(DEV), 64).cpu().numpy().reshape(layers, 4, 64)
    for l, c in enumerate(cfgs):
        assert np.array_equal(got[l], oracle.route_hist(routing(c)[0], 64)[0])
    skew, inter = rl.relibra_load_stats(got[0], top=8)
    s_or, i_or = oracle.load_stats(got[0], top=8)
    assert np.allclose(skew, s_or, rtol=1e-14, atol=0) and np.array_equal(inter, i_or)


# ------------------------------------------------------------------ plan + permute
def plan_both(cfg, counts):
    want = oracle.plan(counts, cfg.EP, cfg.rpn, cfg.r)
    got = rl.relibra_plan(counts, cfg.k, cfg.EP, cfg.rpn, cfg.r)
    for key in ("expert_to_slot", "replica_expert", "inst_ptr", "inst_rank", "inst_rows", "inst_group",
                "group_expert", "group_offset"):
        assert np.array_equal(got[key], want[key]), key
    return got


@pytest.mark.parametrize("kw", [
    dict(), dict(E=8, k=2, EP=4, r=1, T=512, n_mb=1, routing="single"),
    dict(E=128, k=8, EP=8, r=2, T=3000, n_mb=2, h=64),
    dict(E=16, k=8, EP=8, r=2, T=1000, n_mb=2, routing="stress", zipf_s=1.5, h=64),
    dict(E=5, k=5, EP=1, r=0, T=37, n_mb=1, h=8)])
def test_hist_plan_permute_bit_exact(kw):
    cfg = wl.small_config(**kw)
    ids, _ = routing(cfg)
    counts = rl.relibra_route_hist(torch.from_numpy(ids).to(DEV), cfg.E).cpu().numpy()
    p = plan_both(cfg, counts)
    for mb in range(cfg.n_mb):
        X, _ = wl.make_tokens(cfg, mb)
        want_row, want_src = oracle.permute(ids[mb], cfg.E, p["inst_ptr"][mb], p["inst_rows"][mb],
                                            p["inst_group"][mb], p["group_offset"][mb])
        err = rl.new_err_flag()
        row_of, src_of, Xrows = rl.relibra_permute(
            torch.from_numpy(ids[mb]).to(DEV), dev_i32(p["inst_ptr"][mb]), dev_i32(p["inst_rows"][mb]),
            dev_i32(p["inst_group"][mb]), dev_i32(p["group_offset"][mb]), X.to(DEV), cfg.E, cfg.G, err_flag=err)
        assert err.item() == 0
        assert np.array_equal(row_of.cpu().numpy(), want_row)
        assert np.array_equal(src_of.cpu().numpy(), want_src)
        want_rows = oracle.gather_rows(X, want_src, cfg.k)
        got_rows = Xrows.cpu().view(torch.int16).numpy().view(np.uint16)
        assert np.array_equal(got_rows, want_rows)                     # bit copy


@pytest.mark.parametrize("kw", [dict(E=16, k=2, EP=4, r=2, T=240, ranks_per_node=2),
                                dict(E=128, k=8, EP=8, r=2, T=3000, n_mb=2, h=64, ranks_per_node=4),
                                dict(E=16, k=8, EP=8, r=2, T=1000, n_mb=2, routing="stress", zipf_s=1.5, h=64, ranks_per_node=8)])
def test_source_aware_permute_bit_exact(kw):
    """Permutation under the per-source split of Section 5.2: indices and gathered rows identical
    to the oracle's, and every instance holds exactly the tokens of each source the split gave it."""
    cfg = wl.small_config(**kw)
    ids, _ = routing(cfg)
    counts = oracle.route_hist(ids, cfg.E)[0]
    p = plan_both(cfg, counts)
    for mb in range(cfg.n_mb):
        X, _ = wl.make_tokens(cfg, mb)
        x = oracle.route_hist_src(ids[mb], cfg.E, cfg.EP)
        ptr, rank, rows, grp, off = (p[key][mb] for key in ("inst_ptr", "inst_rank", "inst_rows", "inst_group", "group_offset"))
        y = oracle.assign_sources(x, cfg.rpn, ptr, rank, rows)
        want_row, want_src = oracle.permute_src(ids[mb], cfg.E, cfg.EP, ptr, grp, off, y)
        tabs = rl.relibra_assign_sources(x, cfg.rpn, ptr, rank, rows)
        err = rl.new_err_flag()
        row_of, src_of, Xrows = rl.relibra_permute_src(
            torch.from_numpy(ids[mb]).to(DEV), dev_i32(ptr), dev_i32(grp), dev_i32(off), cfg.EP,
            dev_i32(tabs["src_first"]), dev_i32(tabs["inst_src_rows"]), dev_i32(tabs["inst_src_base"]),
            X.to(DEV), cfg.E, cfg.G, err_flag=err)
        assert err.item() == 0
        assert np.array_equal(row_of.cpu().numpy(), want_row)
        assert np.array_equal(src_of.cpu().numpy(), want_src)
        got_rows = Xrows.cpu().view(torch.int16).numpy().view(np.uint16)
        assert np.array_equal(got_rows, oracle.gather_rows(X, want_src, cfg.k))
    # a split table that does not cover the routing is flagged and the assignment skipped
    bad = tabs["inst_src_rows"].copy()
    i, j = np.argwhere(bad > 0)[0]
    bad[i, j] -= 1
    err = rl.new_err_flag()
    row_of, _, _ = rl.relibra_permute_src(
        torch.from_numpy(ids[-1]).to(DEV), dev_i32(ptr), dev_i32(grp), dev_i32(off), cfg.EP,
        dev_i32(tabs["src_first"]), dev_i32(bad), dev_i32(tabs["inst_src_base"]), None, cfg.E, cfg.G, err_flag=err)
    # one token of source j fewer than routed: exactly the source's last assignment of that expert has no row
    e_bad = int(np.searchsorted(np.asarray(ptr), i, side="right") - 1)
    tps = cfg.T // cfg.EP
    flat = ids[-1].reshape(-1)
    a_of = np.flatnonzero((flat == e_bad) & (np.arange(flat.size) // cfg.k // tps == j))
    assert err.item() == rl.ERR_PLAN_COVER
    assert np.array_equal(np.flatnonzero(row_of.cpu().numpy() < 0), a_of[-1:])


def test_source_aware_permute_one_token_per_source():
    """Smallest shape the source-aware permutation accepts: T = EP tokens, k = 1."""
    E = EP = 4
    ids = np.array([[2], [2], [0], [2]], np.int32)
    x = oracle.route_hist_src(ids, E, EP)
    # expert 2 (home rank 2) has a replica on rank 0 taking one of its three tokens
    ptr, rank, rows, grp = [0, 1, 2, 4, 5], [0, 1, 0, 2, 3], [1, 0, 1, 2, 0], [0, 2, 1, 4, 6]
    off = [0, 1, 2, 2, 2, 4, 4, 4, 4]                       # G = 8 groups: (home, replica) per rank
    y = oracle.assign_sources(x, 4, ptr, rank, rows)
    want_row, want_src = oracle.permute_src(ids, E, EP, ptr, grp, off, y)
    tabs = rl.relibra_assign_sources(x, 4, ptr, rank, rows)
    err = rl.new_err_flag()
    row_of, src_of, _ = rl.relibra_permute_src(torch.from_numpy(ids).to(DEV), dev_i32(ptr), dev_i32(grp), dev_i32(off), EP,
                                               dev_i32(tabs["src_first"]), dev_i32(tabs["inst_src_rows"]),
                                               dev_i32(tabs["inst_src_base"]), None, E, 8, err_flag=err)
    assert err.item() == 0
    assert row_of.cpu().tolist() == want_row.tolist() and src_of.cpu().tolist() == want_src.tolist()
    assert want_row.tolist() == [1, 2, 0, 3]                # token 0 (source 0) is the one the replica on rank 0 serves


def test_timed_plan_drives_the_device_path():
    """Tables of the time-driven Algorithm 2 (equal to the oracle's, checked on the host) through
    permutation and expert FFN forward: indices bit-exact, outputs within the bar."""
    cfg = wl.small_config(E=32, k=4, EP=8, r=2, T=1024, n_mb=1, h=128, hff=192, ranks_per_node=4)
    ids, _ = routing(cfg)
    x = np.stack([oracle.route_hist_src(ids[0], cfg.E, cfg.EP)])
    model = rl.cost_model(cfg.EP, cfg.rpn, 2048, 768, 5e14, 4e11, 5e10)
    placed = (np.arange(cfg.E) // cfg.M).astype(np.int32)
    p = rl.relibra_plan_timed(x, cfg.k, model, cfg.r, placed)
    want = oracle.plan_comm(x, cfg.rpn, cfg.r, placed, oracle.cost_model(2048, 768, 5e14, 4e11, 5e10))
    for key in ("inst_ptr", "inst_rank", "inst_rows", "inst_group", "group_expert", "group_offset"):
        assert np.array_equal(p[key], want[key]), key
    X, _ = wl.make_tokens(cfg, 0)
    Wg, Wu, Wd = wl.make_weights(cfg)
    tabs = {key: dev_i32(p[key][0]) for key in ("inst_ptr", "inst_rows", "inst_group", "group_offset", "group_expert")}
    err = rl.new_err_flag()
    row_of, src_of, Xrows = rl.relibra_permute(torch.from_numpy(ids[0]).to(DEV), tabs["inst_ptr"], tabs["inst_rows"],
                                               tabs["inst_group"], tabs["group_offset"], X.to(DEV), cfg.E, cfg.G, err_flag=err)
    want_row, want_src = oracle.permute(ids[0], cfg.E, p["inst_ptr"][0], p["inst_rows"][0], p["inst_group"][0], p["group_offset"][0])
    assert err.item() == 0
    assert np.array_equal(row_of.cpu().numpy(), want_row) and np.array_equal(src_of.cpu().numpy(), want_src)
    Y = rl.relibra_moe_ffn_fwd(Xrows, tabs["group_offset"], tabs["group_expert"], Wg.to(DEV), Wu.to(DEV), Wd.to(DEV), err_flag=err)[3]
    Y_o = oracle.ffn_fwd(oracle.gather_rows(X, want_src, cfg.k), p["group_offset"][0], p["group_expert"][0], Wg, Wu, Wd)[3]
    assert err.item() == 0
    assert rel_l2(Y, Y_o) <= TOL


def test_permute_flags_a_plan_that_does_not_cover_the_routing():
    cfg = wl.small_config(E=8, k=2, EP=4, r=1, T=200, n_mb=1, h=64)
    ids, _ = routing(cfg)
    counts, _ = oracle.route_hist(ids, cfg.E)
    p = rl.relibra_plan(counts, cfg.k, cfg.EP, cfg.rpn, cfg.r)
    rows = p["inst_rows"][0].copy()
    rows[p["inst_ptr"][0][3]] -= 1                                     # one row short for expert 3
    err = rl.new_err_flag()
    row_of, src_of, _ = rl.relibra_permute(
        torch.from_numpy(ids[0]).to(DEV), dev_i32(p["inst_ptr"][0]), dev_i32(rows), dev_i32(p["inst_group"][0]),
        dev_i32(p["group_offset"][0]), None, cfg.E, cfg.G, err_flag=err)
    assert err.item() & rl.ERR_PLAN_COVER
    assert (row_of == -1).sum().item() == 1


# ------------------------------------------------------------------ expert FFN
def ffn_case(seed, E, h, hff, rows, experts, wscale=0.05):
    rng = np.random.default_rng(seed)
    go = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    ge = np.array(experts, np.int32)
    N = int(go[-1])
    bf = lambda x: torch.from_numpy(np.asarray(x, np.float32)).to(torch.bfloat16)
    X = bf(rng.standard_normal((N, h)))
    dY = bf(rng.standard_normal((N, h)))
    Wg = bf(wscale * rng.standard_normal((E, hff, h)))
    Wu = bf(wscale * rng.standard_normal((E, hff, h)))
    Wd = bf(wscale * rng.standard_normal((E, h, hff)))
    return go, ge, X, dY, Wg, Wu, Wd


FFN_CASES = [
    # rows per group span: empty, 1, one short of a tile, a tile, one over, several tiles + tail
    dict(seed=1, E=4, h=256, hff=192, rows=(0, 1, 127, 128, 129, 300, 0, 65), experts=(0, 1, 2, 3, 0, 1, -1, 3)),
    dict(seed=2, E=3, h=128, hff=256, rows=(40, 513, 7), experts=(2, 0, 1)),
    dict(seed=3, E=2, h=64, hff=64, rows=(5, 3), experts=(1, 0)),
    dict(seed=4, E=2, h=320, hff=448, rows=(200, 0, 131), experts=(0, 1, 0)),
    # long groups: the large weight-gradient tile geometry (512 or more rows per group on average)
    dict(seed=7, E=2, h=128, hff=256, rows=(1100, 700), experts=(1, 0)),
    # widths that take the 512-column (eight-wave) tiles in every row-tiled kernel, ragged rows and a replica
    dict(seed=8, E=3, h=512, hff=512, rows=(1, 64, 65, 200, 0, 129), experts=(2, 0, 1, 0, -1, 2)),
    dict(seed=9, E=2, h=1024, hff=1536, rows=(300, 77), experts=(1, 0)),
    # the shortest contractions the wide tiles can meet (two slabs: fewer than the ring holds): gate/up and dA
    # over h = 64 with 512-wide outputs, then down over h' = 64 and dX over two phases of two slabs
    dict(seed=10, E=2, h=64, hff=512, rows=(130, 64), experts=(1, 0)),
    dict(seed=11, E=2, h=512, hff=64, rows=(129, 3), experts=(0, 1)),
]


def dw_slots(ge, E):
    """Home group of an expert = its first group; later groups of the same expert are replicas."""
    seen, slots, nxt = set(), [], E
    for e in ge.tolist():
        if e < 0:
            slots.append(nxt); nxt += 1
        elif e in seen:
            slots.append(nxt); nxt += 1
        else:
            seen.add(e); slots.append(e)
    return np.array(slots, np.int32), nxt


@pytest.mark.parametrize("case", FFN_CASES)
def test_ffn_fwd_bwd_within_tolerance(case):
    go, ge, X, dY, Wg, Wu, Wd = ffn_case(**case)
    E, hff, h = Wg.shape
    Gt_o, U_o, A_o, Y_o = oracle.ffn_fwd(X, go, ge, Wg, Wu, Wd)
    dX_o, dWg_o, dWu_o, dWd_o = oracle.ffn_bwd(X, dY, go, ge, Wg, Wu, Wd)
    live = np.concatenate([np.arange(go[g], go[g + 1]) for g in range(len(ge)) if ge[g] >= 0]).astype(np.int64)

    d = lambda t: t.to(DEV)
    err = rl.new_err_flag()
    Xd, dYd, Wgd, Wud, Wdd = d(X), d(dY), d(Wg), d(Wu), d(Wd)
    god, ged = dev_i32(go), dev_i32(ge)
    N = X.shape[0]
    sentinel = lambda cols: torch.full((N, cols), 7.0, dtype=torch.bfloat16, device=DEV)
    Gt, U, A, Y = rl.relibra_moe_ffn_fwd(Xd, god, ged, Wgd, Wud, Wdd, Gt=sentinel(hff), U=sentinel(hff),
                                         A=sentinel(hff), Yrows=sentinel(h), err_flag=err)
    for name, got, want in (("Gt", Gt, Gt_o), ("U", U, U_o), ("A", A, A_o), ("Y", Y, Y_o)):
        assert rel_l2(got[live], want[live]) <= TOL, name
        for g in range(len(ge)):                                   # per group, so a bad tile cannot hide
            if ge[g] >= 0 and go[g + 1] > go[g]:
                assert rel_l2(got[go[g]:go[g + 1]], want[go[g]:go[g + 1]]) <= TOL, (name, g)
    dead = np.setdiff1d(np.arange(N), live)
    if dead.size:                                                   # rows of empty slots stay untouched
        assert (Y[dead].float() == 7.0).all()

    slots, n_slots = dw_slots(ge, E)
    mk = lambda *s: torch.full(s, 3.0, dtype=torch.float32, device=DEV)
    dWg, dWu, dWd = mk(n_slots, hff, h), mk(n_slots, hff, h), mk(n_slots, h, hff)
    dX = rl.relibra_moe_ffn_bwd(dYd, Xd, Gt, U, A, god, ged, dev_i32(slots), Wgd, Wud, Wdd, dWg, dWu, dWd,
                                dXrows=sentinel(h), err_flag=err)
    assert err.item() == 0
    assert rel_l2(dX[live], dX_o[live]) <= TOL
    used = sorted(set(e for e in ge.tolist() if e >= 0))
    for name, got, want in (("dWg", dWg, dWg_o), ("dWu", dWu, dWu_o), ("dWd", dWd, dWd_o)):
        for e in used:
            if np.linalg.norm(want[e]) > 0:
                assert rel_l2(got[e], want[e]) <= TOL, (name, e)
            else:
                assert (got[e] == 0).all(), (name, e)              # expert seen only through empty groups
    # bit-reproducible
    dWg2, dWu2, dWd2 = mk(n_slots, hff, h), mk(n_slots, hff, h), mk(n_slots, h, hff)
    dX2 = rl.relibra_moe_ffn_bwd(dYd, Xd, Gt, U, A, god, ged, dev_i32(slots), Wgd, Wud, Wdd, dWg2, dWu2, dWd2)
    assert torch.equal(dX2[live], dX[live])
    for a, b in ((dWg2, dWg), (dWu2, dWu), (dWd2, dWd)):
        assert torch.equal(a[:E][used], b[:E][used])
    # accumulate mode adds the same gradient on top
    before = [w[:E].clone() for w in (dWg, dWu, dWd)]
    rl.relibra_moe_ffn_bwd(dYd, Xd, Gt, U, A, god, ged, dev_i32(slots), Wgd, Wud, Wdd, dWg, dWu, dWd,
                           flags=rl.BWD_ACCUMULATE, err_flag=err)
    for w, b in zip((dWg, dWu, dWd), before):
        for e in used:
            assert rel_l2(w[e], 2 * b[e].double().cpu().numpy()) <= 1e-6
    assert err.item() == 0


def test_ffn_group_range_runs_one_ranks_share_only():
    go, ge, X, dY, Wg, Wu, Wd = ffn_case(seed=5, E=4, h=128, hff=128, rows=(30, 50, 0, 20, 140, 9),
                                         experts=(0, 1, 2, 3, 0, 1))
    _, _, _, Y_o = oracle.ffn_fwd(X, go, ge, Wg, Wu, Wd)
    d = lambda t: t.to(DEV)
    N, h = X.shape
    Y = torch.full((N, h), 7.0, dtype=torch.bfloat16, device=DEV)
    rl.relibra_moe_ffn_fwd(d(X), dev_i32(go), dev_i32(ge), d(Wg), d(Wu), d(Wd), g_begin=3, g_end=5, Yrows=Y)
    a, b = int(go[3]), int(go[5])
    assert rel_l2(Y[a:b], Y_o[a:b]) <= TOL
    assert (Y[:a].float() == 7.0).all() and (Y[b:].float() == 7.0).all()


def test_ffn_flags_inconsistent_group_tables_without_faulting():
    go, ge, X, dY, Wg, Wu, Wd = ffn_case(seed=6, E=2, h=64, hff=64, rows=(10, 10), experts=(0, 1))
    d = lambda t: t.to(DEV)
    err = rl.new_err_flag()
    bad_go = go.copy()
    bad_go[2] = 5000                                                 # beyond the row buffer
    rl.relibra_moe_ffn_fwd(d(X), dev_i32(bad_go), dev_i32(ge), d(Wg), d(Wu), d(Wd), err_flag=err)
    assert err.item() & rl.ERR_GROUP_TABLE
    err.zero_()
    rl.relibra_moe_ffn_fwd(d(X), dev_i32(go), dev_i32(np.array([0, 9], np.int32)), d(Wg), d(Wu), d(Wd), err_flag=err)
    assert err.item() & rl.ERR_GROUP_TABLE


# ------------------------------------------------------------------ combine
@pytest.mark.parametrize("T,k,h", [(97, 4, 256), (5, 1, 8), (300, 8, 2048)])
def test_combine_modes(T, k, h):
    rng = np.random.default_rng(T)
    N = T * k
    row_of = rng.permutation(N).astype(np.int32)
    bf = lambda x: torch.from_numpy(np.asarray(x, np.float32)).to(torch.bfloat16)
    Y = bf(rng.standard_normal((N, h)))
    dOut = bf(rng.standard_normal((T, h)))
    gates = rng.random((T, k)).astype(np.float32)
    gates /= gates.sum(1, keepdims=True)
    Yd, gd, rd = Y.to(DEV), torch.from_numpy(gates).to(DEV), dev_i32(row_of)
    err = rl.new_err_flag()
    out = rl.relibra_unpermute_combine(rl.COMBINE_FWD, Yd, rd, T, k, gates=gd, err_flag=err)
    assert rel_l2(out, oracle.combine_fwd(Y.double().numpy(), gates, row_of, T, k)) <= TOL
    out = rl.relibra_unpermute_combine(rl.COMBINE_SUM, Yd, rd, T, k, err_flag=err)
    assert rel_l2(out, oracle.combine_fwd(Y.double().numpy(), None, row_of, T, k)) <= TOL
    dY, dgate = rl.relibra_unpermute_combine(rl.COMBINE_BWD, Yd, rd, T, k, gates=gd, tok=dOut.to(DEV), err_flag=err)
    dY_o, dgate_o = oracle.combine_bwd(dOut.double().numpy(), Y.double().numpy(), gates, row_of, T, k)
    assert rel_l2(dY, dY_o) <= TOL and rel_l2(dgate, dgate_o) <= TOL
    assert err.item() == 0


# ------------------------------------------------------------------ whole path
def run_layer_gpu(cfg, mb, ids, gates, p, Wg, Wu, Wd, X, dOut, dW):
    """One micro-batch through every entry point; returns what the layer hands back."""
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    err = rl.new_err_flag()
    ids_d, gates_d = t(ids), t(gates)
    tabs = {key: dev_i32(p[key][mb]) for key in ("inst_ptr", "inst_rows", "inst_group", "group_offset",
                                                 "group_expert", "group_dw_slot")}
    row_of, src_of, Xrows = rl.relibra_permute(ids_d, tabs["inst_ptr"], tabs["inst_rows"], tabs["inst_group"],
                                               tabs["group_offset"], X, cfg.E, cfg.G, err_flag=err)
    Gt, U, A, Y = rl.relibra_moe_ffn_fwd(Xrows, tabs["group_offset"], tabs["group_expert"], Wg, Wu, Wd, err_flag=err)
    Out = rl.relibra_unpermute_combine(rl.COMBINE_FWD, Y, row_of, cfg.T, cfg.k, gates=gates_d, err_flag=err)
    dY, dgate = rl.relibra_unpermute_combine(rl.COMBINE_BWD, Y, row_of, cfg.T, cfg.k, gates=gates_d, tok=dOut,
                                             err_flag=err)
    dXrows = rl.relibra_moe_ffn_bwd(dY, Xrows, Gt, U, A, tabs["group_offset"], tabs["group_expert"],
                                    tabs["group_dw_slot"], Wg, Wu, Wd, *dW, err_flag=err)
    dX = rl.relibra_unpermute_combine(rl.COMBINE_SUM, dXrows, row_of, cfg.T, cfg.k, err_flag=err)
    assert err.item() == 0
    return Out, dgate, dX


def run_layer_oracle(cfg, mb, ids, gates, p, Wg, Wu, Wd, X, dOut):
    row_of, src_of = oracle.permute(ids, cfg.E, p["inst_ptr"][mb], p["inst_rows"][mb], p["inst_group"][mb],
                                    p["group_offset"][mb])
    Xrows = oracle.gather_rows(X, src_of, cfg.k)
    go, ge = p["group_offset"][mb], p["group_expert"][mb]
    _, _, _, Y = oracle.ffn_fwd(Xrows, go, ge, Wg, Wu, Wd)
    Out = oracle.combine_fwd(Y, gates, row_of, cfg.T, cfg.k)
    dY, dgate = oracle.combine_bwd(dOut.double().numpy(), Y, gates, row_of, cfg.T, cfg.k)
    # the oracle's backward takes bf16 rows: round the upstream row gradients once, as the path does
    dY16 = torch.from_numpy(dY).to(torch.bfloat16)
    dXrows, dWg, dWu, dWd = oracle.ffn_bwd(Xrows, dY16, go, ge, Wg, Wu, Wd)
    dX = oracle.combine_fwd(dXrows, None, row_of, cfg.T, cfg.k)
    return Out, dgate, dX, dWg, dWu, dWd


@pytest.mark.parametrize("cfg", [wl.CONFIGS[0],
                                 wl.small_config(E=16, k=4, EP=4, r=2, T=777, n_mb=2, h=256, hff=192)],
                         ids=["config1-tiny", "ragged-small"])
def test_whole_layer_matches_oracle(cfg):
    ids, gates = routing(cfg)
    counts = rl.relibra_route_hist(torch.from_numpy(ids).to(DEV), cfg.E).cpu().numpy()
    assert np.array_equal(counts, oracle.route_hist(ids, cfg.E)[0])
    p = plan_both(cfg, counts)
    Wg, Wu, Wd = wl.make_weights(cfg)
    Wgd, Wud, Wdd = Wg.to(DEV), Wu.to(DEV), Wd.to(DEV)
    n_slots = cfg.E + cfg.EP * cfg.r
    for mb in range(cfg.n_mb):
        X, dOut = wl.make_tokens(cfg, mb)
        dW = [torch.empty((n_slots, cfg.hff, cfg.h), dtype=torch.float32, device=DEV),
              torch.empty((n_slots, cfg.hff, cfg.h), dtype=torch.float32, device=DEV),
              torch.empty((n_slots, cfg.h, cfg.hff), dtype=torch.float32, device=DEV)]
        Out, dgate, dX = run_layer_gpu(cfg, mb, ids[mb], gates[mb], p, Wgd, Wud, Wdd, X.to(DEV), dOut.to(DEV), dW)
        Out_o, dgate_o, dX_o, dWg_o, dWu_o, dWd_o = run_layer_oracle(cfg, mb, ids[mb], gates[mb], p, Wg, Wu, Wd, X, dOut)
        assert rel_l2(Out, Out_o) <= TOL
        assert rel_l2(dgate, dgate_o) <= TOL
        assert rel_l2(dX, dX_o) <= TOL
        assert rel_l2(dW[0][:cfg.E], dWg_o) <= TOL
        assert rel_l2(dW[1][:cfg.E], dWu_o) <= TOL
        assert rel_l2(dW[2][:cfg.E], dWd_o) <= TOL


# ------------------------------------------------------------------ layer-shared replica buffer
def test_replica_push_fills_slots_and_ffn_reads_them():
    """Section 5.1: the push copies each live replica's home parameters into its slot (bit copy,
    checked against the oracle); the FFN reading replica groups' parameters from those slots must
    give bit-identical results to reading them from the home blocks."""
    cfg = wl.small_config(E=16, k=4, EP=4, r=2, T=777, n_mb=2, h=256, hff=192)
    ids, gates = routing(cfg)
    counts = oracle.route_hist(ids, cfg.E)[0]
    p = plan_both(cfg, counts)
    Wg, Wu, Wd = wl.make_weights(cfg)
    n_slots = cfg.E + cfg.EP * cfg.r
    assert (p["replica_expert"] >= 0).any(), "the case must place replicas"

    def with_slots(W):      # home blocks followed by replica slots holding recognisable junk
        junk = torch.full((cfg.EP * cfg.r, *W.shape[1:]), 7.0, dtype=torch.bfloat16)
        return torch.cat([W, junk]).contiguous()

    big = [with_slots(W) for W in (Wg, Wu, Wd)]
    big_d = [W.to(DEV) for W in big]
    home_d = [W.to(DEV) for W in (Wg, Wu, Wd)]
    for mb in range(cfg.n_mb):
        rep = p["replica_expert"][mb].reshape(-1)
        err = rl.relibra_replica_push(*big_d, dev_i32(rep), cfg.E, cfg.EP, cfg.r, n_workgroups=3)
        assert err.item() == 0
        for W_d, W in zip(big_d, big):
            want = oracle.replica_push(W.view(torch.uint16).numpy(), rep, cfg.E)
            got = W_d.cpu().view(torch.uint16).numpy()
            live = np.concatenate([np.ones(cfg.E, bool), rep >= 0])
            assert np.array_equal(got[live], want[live])
            W.copy_(W_d.cpu())              # slots keep their contents from one micro-batch to the next
        X, dOut = wl.make_tokens(cfg, mb)
        t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
        tabs = {key: dev_i32(p[key][mb]) for key in ("inst_ptr", "inst_rows", "inst_group", "group_offset",
                                                     "group_expert", "group_dw_slot")}
        row_of, src_of, Xrows = rl.relibra_permute(t(ids[mb]), tabs["inst_ptr"], tabs["inst_rows"], tabs["inst_group"],
                                                   tabs["group_offset"], X.to(DEV), cfg.E, cfg.G)
        outs = []
        for use_slots in (False, True):
            err = rl.new_err_flag()
            W3 = big_d if use_slots else home_d
            ge = tabs["group_dw_slot"] if use_slots else tabs["group_expert"]
            Gt, U, A, Y = rl.relibra_moe_ffn_fwd(Xrows, tabs["group_offset"], ge, *W3, err_flag=err)
            dW = [torch.zeros((n_slots, cfg.hff, cfg.h), dtype=torch.float32, device=DEV),
                  torch.zeros((n_slots, cfg.hff, cfg.h), dtype=torch.float32, device=DEV),
                  torch.zeros((n_slots, cfg.h, cfg.hff), dtype=torch.float32, device=DEV)]
            dY = torch.randn(Y.shape, generator=torch.Generator().manual_seed(mb)).to(torch.bfloat16).to(DEV)
            dXrows = rl.relibra_moe_ffn_bwd(dY, Xrows, Gt, U, A, tabs["group_offset"], tabs["group_expert"],
                                            tabs["group_dw_slot"], *W3, *dW, err_flag=err, E=cfg.E,
                                            flags=rl.BWD_REPLICA_WEIGHTS if use_slots else 0)
            assert err.item() == 0
            outs.append((Y, dXrows, dW[0][:cfg.E], dW[1][:cfg.E], dW[2][:cfg.E]))
        for a, b in zip(*outs):
            assert torch.equal(a, b)
        # the same through the deferred and the gate-fused backward (no dW array: the slot table only
        # selects parameter blocks, and the wrapper must size it by the parameter arrays)
        row_tok = rl.relibra_row_tokens(src_of, cfg.k, cfg.T)
        row_gate = rl.relibra_row_gates(src_of, t(gates[mb]))
        Gt, U, A, Y = rl.relibra_moe_ffn_fwd(Xrows, tabs["group_offset"], tabs["group_expert"], *home_d)
        dY = torch.randn(Y.shape, generator=torch.Generator().manual_seed(100 + mb)).to(torch.bfloat16).to(DEV)
        got = []
        for use_slots in (False, True):
            err = rl.new_err_flag()
            W3 = big_d if use_slots else home_d
            fl = rl.BWD_REPLICA_WEIGHTS if use_slots else 0
            dXd = rl.relibra_moe_ffn_bwd(dY, None, Gt, U, A, tabs["group_offset"], tabs["group_expert"], tabs["group_dw_slot"],
                                         *W3, None, None, None, err_flag=err, E=cfg.E, flags=fl | rl.BWD_DEFER_WGRAD)
            dXg, dgate = rl.relibra_moe_ffn_bwd_gated(dOut.to(DEV), row_tok, row_gate, Gt, U, tabs["group_offset"],
                                                     tabs["group_expert"], tabs["group_dw_slot"], *W3, src_of=src_of,
                                                     err_flag=err, E=cfg.E, flags=fl)
            assert err.item() == 0
            got.append((dXd, dXg, dgate))
        for a, b in zip(*got):
            assert torch.equal(a, b)


def test_replica_pull_equals_the_inline_sum_and_two_layers_share_one_slot_buffer():
    """Section 5.1: one buffer of r slots per rank serves every layer in turn (parameters pushed
    before a layer's expert computation, gradients pulled back after its backward).  Two layers with
    their own weights and routing run through ONE shared slot buffer (parameters and gradients),
    the slots overwritten between layers; every result must equal, bit for bit, the run in which
    each layer has private slots and the backward call sums the replica gradients in line."""
    L = 2
    cfgs = [wl.small_config(E=16, k=4, EP=4, r=2, T=777, n_mb=1, h=256, hff=192, index=70 + l) for l in range(L)]
    E, EP, r, h, hff = cfgs[0].E, cfgs[0].EP, cfgs[0].r, cfgs[0].h, cfgs[0].hff
    n_rep = EP * r
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    layers = []
    for cfg in cfgs:
        ids, gates = routing(cfg)
        p = plan_both(cfg, oracle.route_hist(ids, cfg.E)[0])
        assert (p["replica_expert"] >= 0).any()
        X, dOut = wl.make_tokens(cfg, 0)
        tabs = {key: dev_i32(p[key][0]) for key in ("inst_ptr", "inst_rows", "inst_group", "group_offset",
                                                    "group_expert", "group_dw_slot")}
        row_of, src_of, Xrows = rl.relibra_permute(t(ids[0]), tabs["inst_ptr"], tabs["inst_rows"], tabs["inst_group"],
                                                   tabs["group_offset"], X.to(DEV), E, cfg.G)
        dY = torch.randn((cfg.N, h), generator=torch.Generator().manual_seed(cfg.index)).to(torch.bfloat16).to(DEV)
        layers.append(dict(p=p, tabs=tabs, Xrows=Xrows, dY=dY, W=[W.to(DEV) for W in wl.make_weights(cfg)],
                           rep=dev_i32(p["replica_expert"][0].reshape(-1))))

    def run_layer(ly, Wp, dWp, n_blocks, slot_table, pull):
        """forward + backward of one layer on parameter arrays Wp / gradient arrays dWp of n_blocks blocks whose
        first E are the layer's home blocks and whose last n_rep are the replica slots."""
        err = rl.new_err_flag()
        rl.relibra_replica_push(*Wp, ly["rep"], n_blocks - n_rep, EP, r, n_workgroups=5, err_flag=err)
        Gt, U, A, Y = rl.relibra_moe_ffn_fwd(ly["Xrows"], ly["tabs"]["group_offset"], slot_table, *Wp, err_flag=err)
        flags = rl.BWD_REPLICA_WEIGHTS | (rl.BWD_NO_REPLICA_SUM if pull else 0)
        dXrows = rl.relibra_moe_ffn_bwd(ly["dY"], ly["Xrows"], Gt, U, A, ly["tabs"]["group_offset"], ly["tabs"]["group_expert"],
                                        slot_table, *Wp, *dWp, err_flag=err, E=n_blocks - n_rep, flags=flags)
        if pull:
            rl.relibra_replica_pull(*dWp, ly["rep"], n_blocks - n_rep, EP, r, n_workgroups=3, err_flag=err)
        assert err.item() == 0
        return Y, dXrows

    shapes = [(hff, h), (hff, h), (h, hff)]
    # reference: private slots per layer, replica gradients summed inside the backward call
    want = []
    for ly in layers:
        Wp = [torch.cat([W, torch.zeros((n_rep, *W.shape[1:]), dtype=W.dtype, device=DEV)]) for W in ly["W"]]
        dWp = [torch.zeros((E + n_rep, *s), dtype=torch.float32, device=DEV) for s in shapes]
        Y, dXrows = run_layer(ly, Wp, dWp, E + n_rep, ly["tabs"]["group_dw_slot"], pull=False)
        want.append((Y, dXrows, *[d[:E].clone() for d in dWp]))
    # shared: [layer 0 home | layer 1 home | slots]; layer l sees the tail that starts at its home blocks, so a
    # replica slot's block index is (L - l) * E + s in its view
    W_all = [torch.cat([ly["W"][i] for ly in layers] + [torch.full((n_rep, *shapes[i]), 7.0, dtype=torch.bfloat16, device=DEV)])
             for i in range(3)]
    dW_all = [torch.full((L * E + n_rep, *s), float("nan"), dtype=torch.float32, device=DEV) for s in shapes]
    got = [None] * L
    for l in (0, 1, 1, 0):                                   # forward order, then backward order: slots refilled each time
        ly = layers[l]
        slot = ly["p"]["group_dw_slot"][0].copy()
        slot[slot >= E] += (L - l - 1) * E
        view_W = [W[l * E:] for W in W_all]
        view_dW = [d[l * E:] for d in dW_all]
        Y, dXrows = run_layer(ly, view_W, view_dW, (L - l) * E + n_rep, dev_i32(slot), pull=True)
        got[l] = (Y, dXrows, *[d[l * E:(l + 1) * E].clone() for d in dW_all])
    for l in range(L):
        for a, b in zip(got[l], want[l]):
            assert torch.equal(a, b), l
    # the home parameters were never written
    for i in range(3):
        for l, ly in enumerate(layers):
            assert torch.equal(W_all[i][l * E:(l + 1) * E], ly["W"][i])


def test_replica_push_flags_bad_table_and_leaves_empty_slots():
    E, EP, r, h, hff = 4, 2, 2, 64, 64
    W = [torch.arange((E + EP * r) * h * hff, dtype=torch.float32).reshape(E + EP * r, hff, h).to(torch.bfloat16).to(DEV)
         for _ in range(3)]
    before = [w.clone() for w in W]
    err = rl.relibra_replica_push(*W, dev_i32([2, -1, 99, 0]), E, EP, r, n_workgroups=1)
    assert err.item() == rl.ERR_ID_RANGE
    for w, b in zip(W, before):
        assert torch.equal(w[E + 0], b[2]) and torch.equal(w[E + 3], b[0])
        assert torch.equal(w[E + 1], b[E + 1]) and torch.equal(w[E + 2], b[E + 2])
        assert torch.equal(w[:E], b[:E])


# ------------------------------------------------------------------ batched weight gradients
def test_batched_weight_gradients_match_oracle_and_per_microbatch_path():
    """dW of a whole batch in one pass (Section 2.1: gradients accumulate over micro-batches):
    against the oracle's sum over micro-batches (all instances of an expert), and against the
    per-micro-batch accumulate path of the library, which differs only in fp32 summation order."""
    cfg = wl.small_config(E=16, k=4, EP=4, r=2, T=777, n_mb=3, h=256, hff=192)
    ids, gates = routing(cfg)
    counts = oracle.route_hist(ids, cfg.E)[0]
    p = plan_both(cfg, counts)
    Wg, Wu, Wd = wl.make_weights(cfg)
    W_d = [W.to(DEV) for W in (Wg, Wu, Wd)]
    n_slots = cfg.E + cfg.EP * cfg.r
    shapes = [(cfg.hff, cfg.h), (cfg.hff, cfg.h), (cfg.h, cfg.hff)]
    dW_ref = [np.zeros((cfg.E, *s)) for s in shapes]
    dW_mb = [torch.empty((n_slots, *s), dtype=torch.float32, device=DEV) for s in shapes]
    err = rl.new_err_flag()
    kept, fused_in = [], []
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    for mb in range(cfg.n_mb):
        X, _ = wl.make_tokens(cfg, mb)
        tabs = {key: dev_i32(p[key][mb]) for key in ("inst_ptr", "inst_rows", "inst_group", "group_offset",
                                                     "group_expert", "group_dw_slot")}
        Xd = X.to(DEV)
        row_of, src_of, Xrows = rl.relibra_permute(t(ids[mb]), tabs["inst_ptr"], tabs["inst_rows"], tabs["inst_group"],
                                                   tabs["group_offset"], Xd, cfg.E, cfg.G, err_flag=err)
        fused_in.append((Xd, rl.relibra_row_tokens(src_of, cfg.k, cfg.T, err_flag=err)))
        Gt, U, A, Y = rl.relibra_moe_ffn_fwd(Xrows, tabs["group_offset"], tabs["group_expert"], *W_d, err_flag=err)
        dY = torch.randn(Y.shape, generator=torch.Generator().manual_seed(100 + mb)).to(torch.bfloat16)
        dY_d = dY.to(DEV)
        ws = torch.empty(rl.workspace_bytes(rl.WS_FFN_BWD, cfg.N, 1, cfg.E, cfg.G, cfg.h, cfg.hff), dtype=torch.uint8, device=DEV)
        dX_deferred = rl.relibra_moe_ffn_bwd(dY_d, Xrows, Gt, U, A, tabs["group_offset"], tabs["group_expert"],
                                             tabs["group_dw_slot"], *W_d, None, None, None, err_flag=err, E=cfg.E,
                                             flags=rl.BWD_DEFER_WGRAD, workspace=ws)
        kept.append(dict(dYrows=dY_d, Xrows=Xrows, A=A, bwd_workspace=ws, inst_ptr=tabs["inst_ptr"],
                         inst_group=tabs["inst_group"], group_offset=tabs["group_offset"]))
        dX_full = rl.relibra_moe_ffn_bwd(dY_d, Xrows, Gt, U, A, tabs["group_offset"], tabs["group_expert"],
                                         tabs["group_dw_slot"], *W_d, *dW_mb, err_flag=err,
                                         flags=rl.BWD_ACCUMULATE if mb else 0)
        assert torch.equal(dX_deferred, dX_full)                 # the data gradients do not depend on the flag
        _, dWg_o, dWu_o, dWd_o = oracle.ffn_bwd(Xrows.cpu(), dY, p["group_offset"][mb], p["group_expert"][mb], Wg, Wu, Wd)
        for acc, o in zip(dW_ref, (dWg_o, dWu_o, dWd_o)):
            acc += o
    dW_b = [torch.full((cfg.E, *s), 3.0, dtype=torch.float32, device=DEV) for s in shapes]
    rl.relibra_moe_ffn_wgrad_batched(kept, cfg.E, *dW_b, err_flag=err)
    assert err.item() == 0
    for got, want, per_mb in zip(dW_b, dW_ref, dW_mb):
        assert rel_l2(got, want) <= TOL
        assert rel_l2(got, per_mb[:cfg.E].double().cpu().numpy()) <= 1e-5
    # the row gather fused in (token tensor + row -> token table instead of gathered rows): same operands,
    # same order, bit-identical weight gradients
    fused = [dict(m, Xrows=None, X=xd, row_tok=rt) for m, (xd, rt) in zip(kept, fused_in)]
    dW_f = [torch.empty((cfg.E, *s), dtype=torch.float32, device=DEV) for s in shapes]
    rl.relibra_moe_ffn_wgrad_batched(fused, cfg.E, *dW_f, err_flag=err)
    assert err.item() == 0
    for a_, b_ in zip(dW_f, dW_b):
        assert torch.equal(a_, b_)
    # both output tile shapes, forced (the default picks by contraction length): same sums, same order
    for tile in ("narrow", "wide"):
        for inputs in (kept, fused):
            dW_t = [torch.full((cfg.E, *s), float("nan"), dtype=torch.float32, device=DEV) for s in shapes]
            rl.relibra_moe_ffn_wgrad_batched(inputs, cfg.E, *dW_t, err_flag=err, tile=tile)
            assert err.item() == 0
            for a_, b_ in zip(dW_t, dW_b):
                assert torch.equal(a_, b_), tile
    once = [w.clone() for w in dW_b]
    rl.relibra_moe_ffn_wgrad_batched(kept, cfg.E, *dW_b, accumulate=True, err_flag=err)
    for got, one in zip(dW_b, once):
        assert torch.allclose(got, 2 * one, rtol=1e-6, atol=0)
    # a corrupted table is skipped and flagged, never dereferenced
    bad = dict(kept[1])
    bad["inst_group"] = kept[1]["inst_group"].clone()
    bad["inst_group"][0] = cfg.G + 5
    err2 = rl.relibra_moe_ffn_wgrad_batched([kept[0], bad, kept[2]], cfg.E, *dW_b)
    assert err2.item() == rl.ERR_GROUP_TABLE
    # an instance table that is not monotone (ranges of different experts overlap) lists more pieces than
    # a well-formed one can: the surplus is dropped and flagged, nothing is written past the piece arrays
    cap = kept[0]["inst_group"].shape[0]
    zig = dict(kept[0])
    zig["inst_ptr"] = dev_i32([0 if e % 2 == 0 else cap for e in range(cfg.E + 1)])
    err3 = rl.relibra_moe_ffn_wgrad_batched([zig] * rl.MAX_WGRAD_MB, cfg.E, *dW_b)
    torch.cuda.synchronize()
    assert err3.item() == rl.ERR_GROUP_TABLE


# ------------------------------------------------------------------ transposed weights for the data gradients
@pytest.mark.parametrize("n,a,b", [(3, 64, 64), (2, 192, 256), (5, 72, 136), (1, 8, 8)])
def test_transpose_experts_is_exact(n, a, b):
    W = torch.randn((n, a, b), generator=torch.Generator().manual_seed(a + b)).to(torch.bfloat16).to(DEV)
    got = rl.relibra_transpose_experts(W)
    assert torch.equal(got, W.transpose(1, 2).contiguous())


@pytest.mark.parametrize("case", [FFN_CASES[0], FFN_CASES[3], FFN_CASES[4]])
def test_backward_with_transposed_weights_matches_oracle_and_the_plain_layout(case):
    """The data gradients read their weights from transposed copies: same mathematics, so the
    result must meet the oracle's bar and agree with the plain-layout kernels."""
    go, ge, X, dY, Wg, Wu, Wd = ffn_case(**case)
    E = case["E"]
    slots, n_slots = dw_slots(ge, E)
    dev = lambda a: a.to(DEV)
    Xd, dYd, W_d = dev(X), dev(dY), [dev(W) for W in (Wg, Wu, Wd)]
    W_t = [rl.relibra_transpose_experts(W) for W in W_d]
    go_d, ge_d, sl_d = dev_i32(go), dev_i32(ge), dev_i32(slots)
    err = rl.new_err_flag()
    Gt, U, A, Y = rl.relibra_moe_ffn_fwd(Xd, go_d, ge_d, *W_d, err_flag=err)
    outs = []
    for W3, flags in ((W_d, 0), (W_t, rl.BWD_TRANSPOSED_WEIGHTS)):
        dW = [torch.zeros((n_slots, *s), dtype=torch.float32, device=DEV)
              for s in ((case["hff"], case["h"]), (case["hff"], case["h"]), (case["h"], case["hff"]))]
        dX = rl.relibra_moe_ffn_bwd(dYd, Xd, Gt, U, A, go_d, ge_d, sl_d, *W3, *dW, flags=flags, err_flag=err, E=E)
        outs.append((dX, *dW))
    assert err.item() == 0
    live = np.concatenate([np.arange(go[g], go[g + 1]) for g in range(len(ge)) if ge[g] >= 0 and go[g + 1] > go[g]])
    lv = torch.from_numpy(live).to(DEV)
    assert rel_l2(outs[1][0][lv], outs[0][0][lv].double().cpu().numpy()) <= 1e-6      # data gradients: same sums
    for a_, b_ in zip(outs[0][1:], outs[1][1:]):
        assert torch.equal(a_, b_)                                                    # weight gradients do not read W
    dX_o, _, _, _ = oracle.ffn_bwd(X, dY, go, ge, Wg, Wu, Wd)
    assert rel_l2(outs[1][0][lv], dX_o[live]) <= TOL


@pytest.mark.parametrize("case", [FFN_CASES[0], FFN_CASES[3], FFN_CASES[4]])
def test_forward_with_transposed_weights_is_bit_identical(case):
    """Forward GEMMs reading transposed weight copies multiply the same operands in the same
    order: every stored tensor must equal the plain-layout result bit for bit (which the other
    tests hold against the oracle)."""
    go, ge, X, dY, Wg, Wu, Wd = ffn_case(**case)
    Xd, W_d = X.to(DEV), [W.to(DEV) for W in (Wg, Wu, Wd)]
    W_t = [rl.relibra_transpose_experts(W) for W in W_d]
    go_d, ge_d = dev_i32(go), dev_i32(ge)
    err = rl.new_err_flag()
    plain = rl.relibra_moe_ffn_fwd(Xd, go_d, ge_d, *W_d, err_flag=err)
    mk = lambda t: torch.zeros_like(t)
    swapped = rl.relibra_moe_ffn_fwd(Xd, go_d, ge_d, *W_t, Gt=mk(plain[0]), U=mk(plain[1]), A=mk(plain[2]), Yrows=mk(plain[3]),
                                     err_flag=err, flags=rl.FWD_TRANSPOSED_WEIGHTS)
    assert err.item() == 0
    live = np.concatenate([np.arange(go[g], go[g + 1]) for g in range(len(ge)) if ge[g] >= 0 and go[g + 1] > go[g]])
    lv = torch.from_numpy(live).to(DEV)
    for a_, b_ in zip(plain, swapped):
        assert torch.equal(a_[lv], b_[lv])
    Y_o = oracle.ffn_fwd(X, go, ge, Wg, Wu, Wd)[3]
    assert rel_l2(swapped[3][lv], Y_o[live]) <= TOL


# ------------------------------------------------------------------ row gather fused into the GEMMs
def test_forward_with_fused_row_gather_is_bit_identical():
    """relibra_moe_ffn_fwd_gather reads row `row` as X[row_tok[row]]: the same operands in the same
    order as the two-step form (gather, then forward), so every output must match bit for bit;
    row_tok itself is checked against the oracle's permutation."""
    cfg = wl.small_config(E=16, k=4, EP=4, r=2, T=777, n_mb=2, h=256, hff=192)
    ids, gates = routing(cfg)
    counts = oracle.route_hist(ids, cfg.E)[0]
    p = plan_both(cfg, counts)
    Wg, Wu, Wd = [W.to(DEV) for W in wl.make_weights(cfg)]
    for mb in range(cfg.n_mb):
        X, _ = wl.make_tokens(cfg, mb)
        Xd = X.to(DEV)
        tabs = {key: dev_i32(p[key][mb]) for key in ("inst_ptr", "inst_rows", "inst_group", "group_offset", "group_expert")}
        ids_d = torch.from_numpy(ids[mb]).to(DEV)
        err = rl.new_err_flag()
        row_of, src_of, Xrows = rl.relibra_permute(ids_d, tabs["inst_ptr"], tabs["inst_rows"], tabs["inst_group"],
                                                   tabs["group_offset"], Xd, cfg.E, cfg.G, err_flag=err)
        row_tok = rl.relibra_row_tokens(src_of, cfg.k, cfg.T, err_flag=err)
        _, src_o = oracle.permute(ids[mb], cfg.E, p["inst_ptr"][mb], p["inst_rows"][mb], p["inst_group"][mb], p["group_offset"][mb])
        assert np.array_equal(row_tok.cpu().numpy(), src_o // cfg.k)
        two_step = rl.relibra_moe_ffn_fwd(Xrows, tabs["group_offset"], tabs["group_expert"], Wg, Wu, Wd, err_flag=err)
        fused = rl.relibra_moe_ffn_fwd_gather(Xd, row_tok, tabs["group_offset"], tabs["group_expert"], Wg, Wu, Wd, err_flag=err)
        assert err.item() == 0
        for a, b in zip(two_step, fused):
            assert torch.equal(a, b)
        # and together with transposed weight copies (the benchmark's default forward)
        W_t = [rl.relibra_transpose_experts(W) for W in (Wg, Wu, Wd)]
        both = rl.relibra_moe_ffn_fwd_gather(Xd, row_tok, tabs["group_offset"], tabs["group_expert"], *W_t, err_flag=err,
                                             flags=rl.FWD_TRANSPOSED_WEIGHTS)
        assert err.item() == 0
        for a, b in zip(two_step, both):
            assert torch.equal(a, b)
    bad = src_of.clone()
    bad[3] = cfg.T * cfg.k + 7
    err = rl.new_err_flag()
    rt = rl.relibra_row_tokens(bad, cfg.k, cfg.T, err_flag=err)
    assert err.item() == rl.ERR_PLAN_COVER and rt[3].item() == 0


# ------------------------------------------------------------------ gate-side fusion of the backward
@pytest.mark.parametrize("hff", [320, 512], ids=["narrow-dA-tiles", "wide-dA-tiles"])
@pytest.mark.parametrize("weights_t", [False, True], ids=["stored-layout", "transposed-copies"])
def test_gate_fused_backward_matches_the_unfused_definition(weights_t, hff):
    """The combine (Section 2.1: gate-weighted sum of the selected experts' outputs) is linear, so its
    backward may move into the expert backward: dOut rows read straight from the token tensor, the gate
    applied to dA, dgate as a row reduction of dA' against A, dWd from dOut rows against gate * A.  The
    oracle computes the unfused definition (combine backward, then expert backward); the fused path must
    agree within the floating-point tolerance on dX, dgate and all three weight gradients, its forward
    outputs must equal the unfused forward's bit for bit, and two runs must agree bit for bit."""
    cfg = wl.small_config(E=16, k=4, EP=4, r=2, T=777, n_mb=2, h=512, hff=hff)
    ids, gates = routing(cfg)
    counts = oracle.route_hist(ids, cfg.E)[0]
    p = plan_both(cfg, counts)
    Wg, Wu, Wd = wl.make_weights(cfg)
    W_d = [W.to(DEV) for W in (Wg, Wu, Wd)]
    W_f = [rl.relibra_transpose_experts(W) for W in W_d] if weights_t else W_d       # forward operands
    f_flags = rl.FWD_TRANSPOSED_WEIGHTS if weights_t else 0
    shapes = [(cfg.hff, cfg.h), (cfg.hff, cfg.h), (cfg.h, cfg.hff)]
    dW_ref = [np.zeros((cfg.E, *s)) for s in shapes]
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    err = rl.new_err_flag()
    kept = []
    for mb in range(cfg.n_mb):
        X, dOut = wl.make_tokens(cfg, mb)
        Xd, dOut_d, gates_d = X.to(DEV), dOut.to(DEV), t(gates[mb])
        tabs = {key: dev_i32(p[key][mb]) for key in ("inst_ptr", "inst_rows", "inst_group", "group_offset",
                                                     "group_expert", "group_dw_slot")}
        row_of, src_of, _ = rl.relibra_permute(t(ids[mb]), tabs["inst_ptr"], tabs["inst_rows"], tabs["inst_group"],
                                               tabs["group_offset"], Xd, cfg.E, cfg.G, err_flag=err)
        row_tok = rl.relibra_row_tokens(src_of, cfg.k, cfg.T, err_flag=err)
        row_gate = rl.relibra_row_gates(src_of, gates_d, err_flag=err)
        row_of_o, src_o = oracle.permute(ids[mb], cfg.E, p["inst_ptr"][mb], p["inst_rows"][mb], p["inst_group"][mb],
                                         p["group_offset"][mb])
        assert np.array_equal(row_gate.cpu().numpy(), gates[mb].reshape(-1)[src_o])
        # forward: everything the ungated call writes, bit for bit, plus Ag = gate * A
        plain = rl.relibra_moe_ffn_fwd_gather(Xd, row_tok, tabs["group_offset"], tabs["group_expert"], *W_f, err_flag=err, flags=f_flags)
        Gt, U, A, Ag, Y = rl.relibra_moe_ffn_fwd_gated(Xd, row_tok, row_gate, tabs["group_offset"], tabs["group_expert"], *W_f,
                                                       err_flag=err, flags=f_flags)
        for a_, b_ in zip(plain, (Gt, U, A, Y)):
            assert torch.equal(a_, b_)
        Xrows_o = oracle.gather_rows(X, src_o, cfg.k)
        go, ge = p["group_offset"][mb], p["group_expert"][mb]
        _, _, A_o, Y_o = oracle.ffn_fwd(Xrows_o, go, ge, Wg, Wu, Wd)
        assert rel_l2(Ag, gates[mb].reshape(-1)[src_o][:, None].astype(np.float64) * A_o) <= TOL
        # gated in place (A and Ag the same tensor): same Gt, U and Ag; rows come out gate-scaled, the combine is a sum
        A_ip = torch.empty_like(A)
        Gt_p, U_p, _, Ag_p, Y_p = rl.relibra_moe_ffn_fwd_gated(Xd, row_tok, row_gate, tabs["group_offset"], tabs["group_expert"],
                                                               *W_f, A=A_ip, Ag=A_ip, err_flag=err, flags=f_flags)
        assert torch.equal(Gt_p, Gt) and torch.equal(U_p, U) and torch.equal(Ag_p, Ag)
        Out_p = rl.relibra_unpermute_combine(rl.COMBINE_SUM, Y_p, row_of, cfg.T, cfg.k, err_flag=err)
        assert rel_l2(Out_p, oracle.combine_fwd(Y_o, gates[mb], row_of_o, cfg.T, cfg.k)) <= TOL
        # backward
        ws = torch.empty(rl.workspace_bytes(rl.WS_FFN_BWD, cfg.N, 1, cfg.E, cfg.G, cfg.h, cfg.hff), dtype=torch.uint8, device=DEV)
        b_flags = rl.BWD_TRANSPOSED_WEIGHTS if weights_t else 0
        W_b = W_f if weights_t else W_d
        dgate = torch.full((cfg.T, cfg.k), float("nan"), dtype=torch.float32, device=DEV)
        dXrows, _ = rl.relibra_moe_ffn_bwd_gated(dOut_d, row_tok, row_gate, Gt, U, tabs["group_offset"], tabs["group_expert"],
                                                 tabs["group_dw_slot"], *W_b, src_of=src_of, flags=b_flags, dgate=dgate,
                                                 workspace=ws, err_flag=err, E=cfg.E)
        dXrows2, dgate_rows = rl.relibra_moe_ffn_bwd_gated(dOut_d, row_tok, row_gate, Gt, U, tabs["group_offset"],
                                                           tabs["group_expert"], tabs["group_dw_slot"], *W_b, flags=b_flags,
                                                           err_flag=err, E=cfg.E)
        assert torch.equal(dXrows, dXrows2)                                       # reproducible
        assert torch.equal(dgate.reshape(-1)[src_of.long()], dgate_rows)          # the two dgate layouts
        dX = rl.relibra_unpermute_combine(rl.COMBINE_SUM, dXrows, row_of, cfg.T, cfg.k, err_flag=err)
        # oracle: the unfused definition
        dY_o, dgate_o = oracle.combine_bwd(dOut.double().numpy(), Y_o, gates[mb], row_of_o, cfg.T, cfg.k)
        dY16 = torch.from_numpy(dY_o).to(torch.bfloat16)
        dXrows_o, dWg_o, dWu_o, dWd_o = oracle.ffn_bwd(Xrows_o, dY16, go, ge, Wg, Wu, Wd)
        dX_o = oracle.combine_fwd(dXrows_o, None, row_of_o, cfg.T, cfg.k)
        assert rel_l2(dX, dX_o) <= TOL
        assert rel_l2(dgate, dgate_o) <= TOL
        for acc, o in zip(dW_ref, (dWg_o, dWu_o, dWd_o)):
            acc += o
        kept.append(dict(dOut=dOut_d, X=Xd, row_tok=row_tok, A=Ag, bwd_workspace=ws, inst_ptr=tabs["inst_ptr"],
                         inst_group=tabs["inst_group"], group_offset=tabs["group_offset"]))
    assert err.item() == 0
    for tile in (None, "narrow", "wide"):
        dW = [torch.full((cfg.E, *s), float("nan"), dtype=torch.float32, device=DEV) for s in shapes]
        rl.relibra_moe_ffn_wgrad_batched(kept, cfg.E, *dW, err_flag=err, tile=tile)
        assert err.item() == 0
        for got, want in zip(dW, dW_ref):
            assert rel_l2(got, want) <= TOL, tile
        if tile is None:
            first = dW
        else:
            for a_, b_ in zip(dW, first):
                assert torch.equal(a_, b_), tile
    # argument checks: the fused backward needs its scratch, and a bad src_of entry is flagged, not followed
    with pytest.raises(rl.RelibraError):
        rl.relibra_moe_ffn_bwd_gated(dOut_d, row_tok, row_gate, Gt, U, tabs["group_offset"], tabs["group_expert"],
                                     tabs["group_dw_slot"], *W_b, flags=b_flags, E=cfg.E,
                                     dgate_scratch=torch.empty(256, dtype=torch.uint8, device=DEV))
    bad = src_of.clone()
    bad[5] = cfg.N + 3
    err2 = rl.new_err_flag()
    rl.relibra_moe_ffn_bwd_gated(dOut_d, row_tok, row_gate, Gt, U, tabs["group_offset"], tabs["group_expert"],
                                 tabs["group_dw_slot"], *W_b, src_of=bad, flags=b_flags, err_flag=err2, E=cfg.E,
                                 dgate=torch.zeros(cfg.N, dtype=torch.float32, device=DEV))
    assert err2.item() == rl.ERR_PLAN_COVER

"""ctypes face of the CPU oracle (oracle/relibra_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the CPU-baseline
leg of the benchmark.  The product package never imports this module and this module
never imports the product package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "relibra_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over rows; no BLAS, no intrinsics)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-std=c99", "-shared", "-fPIC",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.oracle_replicate_node.restype = C.c_longlong
        _lib.oracle_lse.restype = C.c_double
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


def _u16(a):
    """bf16 torch tensor or uint16 array -> contiguous uint16 numpy array (bit patterns)."""
    if hasattr(a, "view") and hasattr(a, "dtype") and str(a.dtype) == "torch.bfloat16":
        import torch
        return a.contiguous().view(torch.int16).numpy().view(np.uint16)
    return np.ascontiguousarray(a, dtype=np.uint16)


# ------------------------------------------------------------------ integer path
def route_hist(ids, E):
    """ids[n_mb,T,k] -> (counts[n_mb,E] int32, total[E] int64)."""
    ids = _i32(ids)
    n_mb, T, k = ids.shape
    counts = np.empty((n_mb, E), np.int32)
    total = np.empty(E, np.int64)
    rc = lib().oracle_route_hist(_p(ids), n_mb, T, k, E, _p(counts), _p(total))
    if rc:
        raise ValueError(f"oracle_route_hist: status {rc}")
    return counts, total


def lpt(l, EP):
    l = _i64(l)
    out = np.empty(l.shape[0], np.int32)
    lib().oracle_lpt(_p(l), l.shape[0], EP, _p(out))
    return out


def swap_descent(l, EP, rank_of):
    l = _i64(l)
    out = _i32(rank_of).copy()
    lib().oracle_swap_descent(_p(l), l.shape[0], EP, _p(out))
    return out


def reorder(l, EP):
    l = _i64(l)
    out = np.empty(l.shape[0], np.int32)
    lib().oracle_reorder(_p(l), l.shape[0], EP, _p(out))
    return out


def balance_split(z, a):
    """Balance the split a[ne,n] (warm start) under placement z[ne,n]; returns the new split."""
    z = np.ascontiguousarray(z, dtype=np.uint8)
    a = _i64(a).copy()
    ne, n = z.shape
    lib().oracle_balance_split(_p(z), ne, n, _p(a))
    return a


def replicate_node(cnt, home, n, r):
    cnt = _i64(cnt)
    home = _i32(home)
    ne = cnt.shape[0]
    z = np.empty((ne, n), np.uint8)
    a = np.empty((ne, n), np.int64)
    mx = lib().oracle_replicate_node(_p(cnt), _p(home), ne, n, r, _p(z), _p(a))
    return z, a, int(mx)


def plan(counts, EP, rpn, r, placed=None):
    """counts[n_mb,E] -> dict of plan tables (see oracle_plan in the C file).
    placed [E]: use this placement instead of the oracle's own stage 1."""
    counts = _i32(counts)
    n_mb, E = counts.shape
    M = E // EP if EP > 0 else 0
    G = EP * (M + r)
    cap = E + EP * r
    out = dict(
        expert_to_slot=np.empty(E, np.int32),
        replica_expert=np.empty((n_mb, EP, r), np.int32),
        inst_ptr=np.empty((n_mb, E + 1), np.int32),
        inst_rank=np.empty((n_mb, cap), np.int32),
        inst_rows=np.empty((n_mb, cap), np.int32),
        inst_group=np.empty((n_mb, cap), np.int32),
        group_expert=np.empty((n_mb, G), np.int32),
        group_offset=np.empty((n_mb, G + 1), np.int32),
        max_before=np.empty(n_mb, np.int64),
        max_after=np.empty(n_mb, np.int64),
    )
    placed = None if placed is None else _i32(placed)
    rc = lib().oracle_plan_ex(_p(counts), n_mb, E, EP, rpn, r, _p(placed),
                           _p(out["expert_to_slot"]), _p(out["replica_expert"]),
                           _p(out["inst_ptr"]), _p(out["inst_rank"]), _p(out["inst_rows"]),
                           _p(out["inst_group"]), _p(out["group_expert"]), _p(out["group_offset"]),
                           _p(out["max_before"]), _p(out["max_after"]))
    if rc:
        raise ValueError(f"oracle_plan: status {rc}")
    return out


def replicate_comm(x, rank_of, rpn, r, model):
    """Algorithm 2 with the time of Section 4.1 as objective, one micro-batch:
    x [EP,E] -> (z [E,EP] uint8, a [E,EP] int64, dict(T_before, T_after, max_load))."""
    x, rank_of = _i64(x), _i32(rank_of)
    EP, E = x.shape
    model = np.ascontiguousarray(model, dtype=np.float64)
    z = np.zeros((E, EP), np.uint8)
    a = np.zeros((E, EP), np.int64)
    T2 = np.zeros(2, np.float64)
    lib().oracle_replicate_comm.restype = C.c_longlong
    mx = lib().oracle_replicate_comm(_p(x), _p(rank_of), E, EP, int(rpn), int(r), _p(model), _p(z), _p(a), _p(T2))
    return z, a, dict(T_before=T2[0], T_after=T2[1], max_load=int(mx))


def plan_comm(x, rpn, r, placed, model):
    """x [n_mb,EP,E] per-source histograms + placement -> plan tables with the time-aware replication."""
    x = _i64(x)
    n_mb, EP, E = x.shape
    M = E // EP
    G = EP * (M + r)
    cap = E + EP * r
    out = dict(
        expert_to_slot=np.empty(E, np.int32), replica_expert=np.empty((n_mb, EP, r), np.int32),
        inst_ptr=np.empty((n_mb, E + 1), np.int32), inst_rank=np.empty((n_mb, cap), np.int32),
        inst_rows=np.empty((n_mb, cap), np.int32), inst_group=np.empty((n_mb, cap), np.int32),
        group_expert=np.empty((n_mb, G), np.int32), group_offset=np.empty((n_mb, G + 1), np.int32),
        max_before=np.empty(n_mb, np.int64), max_after=np.empty(n_mb, np.int64),
        t_before=np.empty(n_mb, np.float64), t_after=np.empty(n_mb, np.float64))
    model = np.ascontiguousarray(model, dtype=np.float64)
    rc = lib().oracle_plan_comm(_p(x), n_mb, E, EP, int(rpn), int(r), _p(_i32(placed)), _p(model),
                                _p(out["expert_to_slot"]), _p(out["replica_expert"]),
                                _p(out["inst_ptr"]), _p(out["inst_rank"]), _p(out["inst_rows"]),
                                _p(out["inst_group"]), _p(out["group_expert"]), _p(out["group_offset"]),
                                _p(out["max_before"]), _p(out["max_after"]), _p(out["t_before"]), _p(out["t_after"]))
    if rc:
        raise ValueError(f"oracle_plan_comm: status {rc}")
    return out


def permute(ids, E, inst_ptr, inst_rows, inst_group, group_offset):
    """ids[T,k] + one micro-batch's plan tables -> (row_of[N], src_of[N])."""
    ids = _i32(ids)
    T, k = ids.shape
    row_of = np.full(T * k, -1, np.int32)
    src_of = np.full(T * k, -1, np.int32)
    rc = lib().oracle_permute(_p(ids), T, k, E, _p(_i32(inst_ptr)), _p(_i32(inst_rows)),
                              _p(_i32(inst_group)), _p(_i32(group_offset)), _p(row_of), _p(src_of))
    if rc:
        raise ValueError(f"oracle_permute: status {rc}")
    return row_of, src_of


def load_stats(counts, top=8):
    """-> (skewness [n_mb], intersection ratio of adjacent micro-batches' top hot sets [n_mb-1])."""
    counts = _i32(counts)
    n_mb, E = counts.shape
    skew = np.empty(n_mb, np.float64)
    inter = np.empty(max(n_mb - 1, 0), np.float64)
    lib().oracle_load_stats(_p(counts), n_mb, E, int(top), _p(skew), _p(inter))
    return skew, inter


# ------------------------------------------------------------------ communication-aware model, Algorithm 1
def cost_model(h, hff, F, B_intra, B_inter, bytes_per_value=2):
    """[seconds per token of computation (Eq. 4), per token over the intra-node link, over RDMA (Eq. 5)]."""
    return np.array([6.0 * h * hff / F, bytes_per_value * h / B_intra, bytes_per_value * h / B_inter], np.float64)


def route_hist_src(ids_mb, E, EP):
    """ids [T,k] of one micro-batch -> x [EP,E] int64 (tokens of source rank j routed to expert e)."""
    ids_mb = _i32(ids_mb)
    T, k = ids_mb.shape
    x = np.empty((EP, E), np.int64)
    rc = lib().oracle_route_hist_src(_p(ids_mb), T, k, E, EP, _p(x))
    if rc:
        raise ValueError(f"oracle_route_hist_src: status {rc}")
    return x


def tau(j, g, rpn):
    return int(lib().oracle_tau(int(j), int(g), int(rpn)))


def loads(x, rank_of, rpn):
    """-> comp, nv_tx, nv_rx, rd_tx, rd_rx [EP] int64 (Eq. 1-3)."""
    x, rank_of = _i64(x), _i32(rank_of)
    EP, E = x.shape
    out = [np.empty(EP, np.int64) for _ in range(5)]
    lib().oracle_loads(_p(x), E, EP, int(rpn), _p(rank_of), *[_p(o) for o in out])
    return out


def lse(z, beta):
    z = np.ascontiguousarray(z, dtype=np.float64)
    return float(lib().oracle_lse(_p(z), z.shape[0], C.c_double(beta)))


def moe_time(x, rank_of, rpn, model, beta=20.0, t_ref=1.0):
    """-> dict(T, T_comp, T_comm in seconds (Eq. 4-6), smooth = LSE-smoothed objective on times / t_ref)."""
    x, rank_of = _i64(x), _i32(rank_of)
    EP, E = x.shape
    model = np.ascontiguousarray(model, dtype=np.float64)
    out = np.empty(4, np.float64)
    lib().oracle_moe_time(_p(x), E, EP, int(rpn), _p(rank_of), _p(model), C.c_double(beta), C.c_double(t_ref), _p(out))
    return dict(T=out[0], T_comp=out[1], T_comm=out[2], smooth=out[3])


def assign_sources(x, rpn, inst_ptr, inst_rank, inst_rows):
    """x [EP,E] + one micro-batch's instance tables -> y [n_inst, EP] int64 (tokens of source j served by instance i)."""
    x = _i64(x)
    EP, E = x.shape
    inst_ptr, inst_rank, inst_rows = _i32(inst_ptr), _i32(inst_rank), _i32(inst_rows)
    y = np.zeros((inst_rank.shape[0], EP), np.int64)
    rc = lib().oracle_assign_sources(_p(x), E, EP, int(rpn), _p(inst_ptr), _p(inst_rank), _p(inst_rows), _p(y))
    if rc:
        raise ValueError(f"oracle_assign_sources: status {rc}")
    return y


def moe_time_split(y, inst_rank, rpn, model):
    """-> dict(T, T_comp, T_comm) in seconds (Eq. 4-6) and loads [5, EP] in tokens under the split y."""
    y, inst_rank = _i64(y), _i32(inst_rank)
    n_inst, EP = y.shape
    model = np.ascontiguousarray(model, dtype=np.float64)
    out = np.empty(3, np.float64)
    loads_ = np.empty((5, EP), np.int64)
    lib().oracle_moe_time_split(_p(y), n_inst, EP, int(rpn), _p(inst_rank), _p(model), _p(out), _p(loads_))
    return dict(T=out[0], T_comp=out[1], T_comm=out[2]), loads_


def permute_src(ids, E, EP, inst_ptr, inst_group, group_offset, y):
    """Permutation that honours the per-source split y -> (row_of[N], src_of[N])."""
    ids = _i32(ids)
    T, k = ids.shape
    row_of = np.full(T * k, -1, np.int32)
    src_of = np.full(T * k, -1, np.int32)
    rc = lib().oracle_permute_src(_p(ids), T, k, E, EP, _p(_i32(inst_ptr)), _p(_i32(inst_group)),
                                  _p(_i32(group_offset)), _p(_i64(y)), _p(row_of), _p(src_of))
    if rc:
        raise ValueError(f"oracle_permute_src: status {rc}")
    return row_of, src_of


def splitmix64(seed, n):
    """First n outputs of the annealing's generator started at state `seed` (uint64)."""
    out = np.empty(n, np.uint64)
    lib().oracle_splitmix64(C.c_uint64(seed), int(n), _p(out))
    return out


def reorder_sa_trace(x, rpn, model, beta=20.0, gamma=0.999, eps=1e-3, seed=0, cap=64):
    """One seed of Algorithm 1 with its trajectory: dict(start, rank, t_ref, smooth_start, iterations,
    moves [n,3] = (e_a, e_b, accepted), vals [n,3] = (u, T', theta)) for the first n = min(cap, iterations) steps."""
    x = _i64(x)
    EP, E = x.shape
    model = np.ascontiguousarray(model, dtype=np.float64)
    moves = np.zeros((cap, 3), np.int32)
    vals = np.zeros((cap, 3), np.float64)
    start, rank = np.empty(E, np.int32), np.empty(E, np.int32)
    st = np.empty(2, np.float64)
    fn = lib().oracle_reorder_sa_trace
    fn.restype = C.c_longlong
    it = fn(_p(x), E, EP, int(rpn), _p(model), C.c_double(beta), C.c_double(gamma), C.c_double(eps), C.c_uint64(seed),
            int(cap), _p(moves), _p(vals), _p(start), _p(rank), _p(st))
    if it < 0:
        raise ValueError("oracle_reorder_sa_trace: bad arguments")
    n = min(int(it), cap)
    return dict(start=start, rank=rank, t_ref=st[0], smooth_start=st[1], iterations=int(it), moves=moves[:n], vals=vals[:n])


def reorder_sa(x, rpn, model, beta=20.0, gamma=0.999, eps=1e-3, n_seeds=8, seed=0):
    """Algorithm 1 -> (rank_of [E], dict(T_start, T, smooth_start, smooth, iterations))."""
    x = _i64(x)
    EP, E = x.shape
    model = np.ascontiguousarray(model, dtype=np.float64)
    rank_of = np.empty(E, np.int32)
    st = np.empty(5, np.float64)
    rc = lib().oracle_reorder_sa(_p(x), E, EP, int(rpn), _p(model), C.c_double(beta), C.c_double(gamma),
                                 C.c_double(eps), int(n_seeds), C.c_uint64(seed), _p(rank_of), _p(st))
    if rc:
        raise ValueError(f"oracle_reorder_sa: status {rc}")
    return rank_of, dict(T_start=st[0], T=st[1], smooth_start=st[2], smooth=st[3], iterations=int(st[4]))


# ------------------------------------------------------------------ floating point
def gather_rows(X, src_of, k):
    X = _u16(X)
    src_of = _i32(src_of)
    N, h = src_of.shape[0], X.shape[1]
    out = np.empty((N, h), np.uint16)
    lib().oracle_gather_rows(_p(X), _p(src_of), N, k, h, _p(out))
    return out


def replica_push(W, replica_expert, E):
    """W [E + slots, ...] bf16 bit patterns -> copy with every live replica slot filled from its home block."""
    W = _u16(W).copy()
    rep = _i32(replica_expert).reshape(-1)
    assert W.shape[0] == E + rep.shape[0]
    block = int(np.prod(W.shape[1:]))
    lib().oracle_replica_push(_p(W), _p(rep), int(E), int(rep.shape[0]), C.c_size_t(block))
    return W


def ffn_fwd(Xrows, group_offset, group_expert, Wg, Wu, Wd, g_begin=0, g_end=None):
    """-> Gt, U, A [N,h'] and Y [N,h], float64 (rows outside the group range are NaN)."""
    Xrows, Wg, Wu, Wd = _u16(Xrows), _u16(Wg), _u16(Wu), _u16(Wd)
    go, ge = _i32(group_offset), _i32(group_expert)
    if g_end is None:
        g_end = ge.shape[0]
    N, h = Xrows.shape
    hff = Wg.shape[1]
    assert Wg.shape[2] == h and Wd.shape[1] == h and Wd.shape[2] == hff
    Gt = np.full((N, hff), np.nan)
    U = np.full((N, hff), np.nan)
    A = np.full((N, hff), np.nan)
    Y = np.full((N, h), np.nan)
    lib().oracle_ffn_fwd(_p(Xrows), _p(go), _p(ge), g_begin, g_end, _p(Wg), _p(Wu), _p(Wd),
                         h, hff, _p(Gt), _p(U), _p(A), _p(Y))
    return Gt, U, A, Y


def ffn_bwd(Xrows, dYrows, group_offset, group_expert, Wg, Wu, Wd, g_begin=0, g_end=None):
    """-> dXrows [N,h], dWg, dWu [E,h',h], dWd [E,h,h'], float64."""
    Xrows, dYrows, Wg, Wu, Wd = _u16(Xrows), _u16(dYrows), _u16(Wg), _u16(Wu), _u16(Wd)
    go, ge = _i32(group_offset), _i32(group_expert)
    if g_end is None:
        g_end = ge.shape[0]
    N, h = Xrows.shape
    E, hff = Wg.shape[0], Wg.shape[1]
    dX = np.full((N, h), np.nan)
    dWg = np.empty((E, hff, h))
    dWu = np.empty((E, hff, h))
    dWd = np.empty((E, h, hff))
    lib().oracle_ffn_bwd(_p(Xrows), _p(dYrows), _p(go), _p(ge), g_begin, g_end, E,
                         _p(Wg), _p(Wu), _p(Wd), h, hff, _p(dX), _p(dWg), _p(dWu), _p(dWd))
    return dX, dWg, dWu, dWd


def combine_fwd(Yrows, gates, row_of, T, k):
    Yrows = np.ascontiguousarray(Yrows, dtype=np.float64)
    g = None if gates is None else np.ascontiguousarray(gates, dtype=np.float32)
    h = Yrows.shape[1]
    out = np.empty((T, h))
    lib().oracle_combine_fwd(_p(Yrows), _p(g), _p(_i32(row_of)), T, k, h, _p(out))
    return out


def combine_bwd(dOut, Yrows, gates, row_of, T, k):
    dOut = np.ascontiguousarray(dOut, dtype=np.float64)
    Yrows = np.ascontiguousarray(Yrows, dtype=np.float64)
    g = np.ascontiguousarray(gates, dtype=np.float32)
    h = Yrows.shape[1]
    dY = np.empty_like(Yrows)
    dgate = np.empty((T, k))
    lib().oracle_combine_bwd(_p(dOut), _p(Yrows), _p(g), _p(_i32(row_of)), T, k, h, _p(dY), _p(dgate))
    return dY, dgate


def num_threads():
    """Threads the oracle's OpenMP loops use."""
    return int(lib().oracle_num_threads())

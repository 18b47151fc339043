"""Thin Python binding of librelibra.so (see include/relibra.h).

Argument marshalling only: every step of the path runs in the library's HIP kernels (or, for
relibra_plan, its host C++).  PyTorch supplies device memory and the current HIP stream.
There is no fallback: if the shared library is missing, importing the binding's functions
raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librelibra.so")

OK, EINVAL, ERANGE, EWORKSPACE, EHIP, EUNSUPPORTED = 0, -1, -2, -3, -4, -5
ERR_ID_RANGE, ERR_PLAN_COVER, ERR_GROUP_TABLE = 1, 2, 4
WS_PERMUTE, WS_FFN_FWD, WS_FFN_BWD, WS_WGRAD_BATCHED, WS_DGATE = 0, 1, 2, 3, 4
BWD_ACCUMULATE, BWD_NO_REPLICA_SUM, BWD_REPLICA_WEIGHTS, BWD_DEFER_WGRAD, BWD_TRANSPOSED_WEIGHTS = 1, 2, 4, 8, 16
FWD_TRANSPOSED_WEIGHTS = 1
WGRAD_ACCUMULATE, WGRAD_TILE_NARROW, WGRAD_TILE_WIDE = 1, 2, 4
MAX_WGRAD_MB = 48
COMBINE_FWD, COMBINE_BWD, COMBINE_SUM = 0, 1, 2

EXPORTS = ("relibra_route_hist", "relibra_plan", "relibra_plan_placed", "relibra_moe_time", "relibra_reorder_sa", "relibra_load_stats",
           "relibra_cost_model_init", "relibra_reorder_sa_trace",
           "relibra_assign_sources", "relibra_moe_time_split", "relibra_permute_src", "relibra_plan_timed",
           "relibra_permute", "relibra_permute_static", "relibra_row_tokens", "relibra_row_gates", "relibra_moe_ffn_fwd_gather", "relibra_moe_ffn_fwd_gated",
           "relibra_moe_ffn_bwd_gated", "relibra_moe_ffn_fwd",
           "relibra_moe_ffn_bwd", "relibra_moe_ffn_wgrad_batched", "relibra_transpose_experts", "relibra_unpermute_combine", "relibra_replica_push", "relibra_replica_pull",
           "relibra_workspace_bytes",
           "relibra_status_string", "relibra_prof_start", "relibra_prof_stop")

KERNELS = ("hist", "perm_count", "perm_scan", "perm_rank", "gather", "combine_fwd", "combine_bwd",
           "combine_sum", "sched", "fwd_gate_up", "fwd_down", "bwd_act", "bwd_dx", "wgrad_down",
           "wgrad_gate_up", "replica_sum", "replica_push", "wgrad_order", "transpose", "row_tokens", "row_gates",
           "dgate_reduce", "replica_pull")

_lib = None


class RelibraError(RuntimeError):
    def __init__(self, fn, status):
        self.status = status
        super().__init__(f"{fn}: status {status} ({status_string(status)})")


def lib():
    """The loaded C-ABI library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                              "(hipcc, gfx950) first; there is no fallback path")
        L = C.CDLL(LIB_PATH)
        L.relibra_workspace_bytes.restype = C.c_size_t
        L.relibra_status_string.restype = C.c_char_p
        for name in EXPORTS:
            getattr(L, name)
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().relibra_status_string(int(status)).decode()


def _check(fn, rc):
    if rc != OK:
        raise RelibraError(fn, rc)


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dp(t, dtype=None):
    """Device pointer of a contiguous CUDA tensor (None -> NULL)."""
    if t is None:
        return C.c_void_p(0)
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous"
    if dtype is not None:
        assert t.dtype == dtype, f"expected {dtype}, got {t.dtype}"
    return C.c_void_p(t.data_ptr())


def _hp(a):
    return a.ctypes.data_as(C.c_void_p)


def workspace_bytes(which, T, k, E, G, h, hff):
    return int(lib().relibra_workspace_bytes(which, T, k, E, G, h, hff))


def new_err_flag(device="cuda"):
    return torch.zeros(1, dtype=torch.int32, device=device)


# ---------------------------------------------------------------------------------------------
def relibra_route_hist(ids, E, counts=None, err_flag=None):
    """ids [n_mb,T,k] int32 (device) -> counts [n_mb,E] int32 (device)."""
    n_mb, T, k = ids.shape
    if counts is None:
        counts = torch.empty((n_mb, E), dtype=torch.int32, device=ids.device)
    if err_flag is None:
        err_flag = new_err_flag(ids.device)
    rc = lib().relibra_route_hist(_dp(ids, torch.int32), n_mb, T, k, E, _dp(counts, torch.int32),
                                  _dp(err_flag, torch.int32), _stream())
    _check("relibra_route_hist", rc)
    return counts


def relibra_plan(counts_host, k, EP, ranks_per_node, r, expert_rank=None):
    """counts_host [n_mb,E] int32 numpy (host) -> dict of host numpy plan tables.
    expert_rank [E] (optional): take this placement instead of running stage 1 (relibra_plan_placed)."""
    counts_host = np.ascontiguousarray(counts_host, dtype=np.int32)
    n_mb, E = counts_host.shape
    M = E // EP if EP > 0 and E % EP == 0 else 0
    G = max(EP * (M + r), 1) if EP > 0 and r >= 0 else 1
    cap = max(E + max(EP, 0) * max(r, 0), 1)
    out = dict(
        expert_to_slot=np.empty(E, np.int32),
        replica_expert=np.empty((n_mb, max(EP, 0), max(r, 0)), np.int32),
        inst_ptr=np.empty((n_mb, E + 1), np.int32),
        inst_rank=np.empty((n_mb, cap), np.int32),
        inst_rows=np.empty((n_mb, cap), np.int32),
        inst_group=np.empty((n_mb, cap), np.int32),
        group_expert=np.empty((n_mb, G), np.int32),
        group_offset=np.empty((n_mb, G + 1), np.int32),
        group_dw_slot=np.empty((n_mb, G), np.int32),
        max_load_before=np.empty(n_mb, np.int64),
        max_load_after=np.empty(n_mb, np.int64),
    )
    rep = out["replica_expert"]
    tail = (_hp(out["expert_to_slot"]), _hp(rep) if rep.size else C.c_void_p(0),
            _hp(out["inst_ptr"]), _hp(out["inst_rank"]), _hp(out["inst_rows"]),
            _hp(out["inst_group"]), _hp(out["group_expert"]), _hp(out["group_offset"]),
            _hp(out["group_dw_slot"]), _hp(out["max_load_before"]), _hp(out["max_load_after"]))
    if expert_rank is None:
        rc = lib().relibra_plan(_hp(counts_host), n_mb, E, k, EP, ranks_per_node, r, *tail)
        _check("relibra_plan", rc)
    else:
        expert_rank = np.ascontiguousarray(expert_rank, dtype=np.int32)
        assert expert_rank.shape == (E,)
        rc = lib().relibra_plan_placed(_hp(counts_host), n_mb, E, k, EP, ranks_per_node, r, _hp(expert_rank), *tail)
        _check("relibra_plan_placed", rc)
    return out


def relibra_plan_timed(x_host, k, model, r, expert_rank):
    """x_host [n_mb,EP,E] int64 per-source histograms + placement -> plan tables with Algorithm 2 driven by
    T_MoE,g (Section 4.1), plus t_before / t_after [n_mb] (seconds)."""
    x_host = np.ascontiguousarray(x_host, dtype=np.int64)
    n_mb, EP, E = x_host.shape
    assert EP == model.EP
    expert_rank = np.ascontiguousarray(expert_rank, dtype=np.int32)
    assert expert_rank.shape == (E,)
    M = E // EP if E % EP == 0 else 0
    G = max(EP * (M + r), 1) if r >= 0 else 1
    cap = max(E + EP * max(r, 0), 1)
    out = dict(
        expert_to_slot=np.empty(E, np.int32), replica_expert=np.empty((n_mb, EP, max(r, 0)), np.int32),
        inst_ptr=np.empty((n_mb, E + 1), np.int32), inst_rank=np.empty((n_mb, cap), np.int32),
        inst_rows=np.empty((n_mb, cap), np.int32), inst_group=np.empty((n_mb, cap), np.int32),
        group_expert=np.empty((n_mb, G), np.int32), group_offset=np.empty((n_mb, G + 1), np.int32),
        group_dw_slot=np.empty((n_mb, G), np.int32),
        max_load_before=np.empty(n_mb, np.int64), max_load_after=np.empty(n_mb, np.int64),
        t_before=np.empty(n_mb, np.float64), t_after=np.empty(n_mb, np.float64))
    rep = out["replica_expert"]
    rc = lib().relibra_plan_timed(_hp(x_host), n_mb, E, int(k), C.byref(model), int(r), _hp(expert_rank),
                                  _hp(out["expert_to_slot"]), _hp(rep) if rep.size else C.c_void_p(0),
                                  _hp(out["inst_ptr"]), _hp(out["inst_rank"]), _hp(out["inst_rows"]),
                                  _hp(out["inst_group"]), _hp(out["group_expert"]), _hp(out["group_offset"]),
                                  _hp(out["group_dw_slot"]), _hp(out["max_load_before"]), _hp(out["max_load_after"]),
                                  _hp(out["t_before"]), _hp(out["t_after"]))
    _check("relibra_plan_timed", rc)
    return out


def relibra_load_stats(counts_host, top=8):
    """counts [n_mb,E] int32 (host) -> (skewness [n_mb], intersection ratio of the top hot sets [n_mb-1])."""
    counts_host = np.ascontiguousarray(counts_host, dtype=np.int32)
    n_mb, E = counts_host.shape
    skew = np.empty(n_mb, np.float64)
    inter = np.empty(max(n_mb - 1, 0), np.float64)
    rc = lib().relibra_load_stats(_hp(counts_host), n_mb, E, int(top), _hp(skew), _hp(inter) if n_mb > 1 else C.c_void_p(0))
    _check("relibra_load_stats", rc)
    return skew, inter


class CostModel(C.Structure):
    """relibra_cost_model (Section 4.1): seconds per routed token of computation, over the
    intra-node link and over RDMA, on EP ranks in nodes of ranks_per_node."""
    _fields_ = [("EP", C.c_int), ("ranks_per_node", C.c_int), ("sec_per_token_comp", C.c_double),
                ("sec_per_token_intra", C.c_double), ("sec_per_token_inter", C.c_double)]


def cost_model(EP, ranks_per_node, h, hff, F, B_intra, B_inter, bytes_per_value=2):
    m = CostModel()
    rc = lib().relibra_cost_model_init(C.byref(m), int(EP), int(ranks_per_node), int(h), int(hff), C.c_double(F),
                                       C.c_double(B_intra), C.c_double(B_inter), int(bytes_per_value))
    _check("relibra_cost_model_init", rc)
    return m


def relibra_route_hist_src(ids, E, EP, err_flag=None):
    """ids [n_mb,T,k] int32 (device) -> x [n_mb,EP,E] int32 (device): tokens on source rank
    j = t // (T/EP) routed to expert e.  The histogram kernel on ids viewed as [n_mb*EP, T/EP, k]."""
    n_mb, T, k = ids.shape
    assert T % EP == 0, "tokens must split evenly over the source ranks"
    x = relibra_route_hist(ids.view(n_mb * EP, T // EP, k), E, err_flag=err_flag)
    return x.view(n_mb, EP, E)


def relibra_moe_time(x_host, expert_rank, model, beta=20.0, t_ref=1.0, with_loads=False):
    """x_host [EP,E] int64 -> dict(T, T_comp, T_comm, smooth[, loads [5,EP]]) (Eq. 1-6)."""
    x_host = np.ascontiguousarray(x_host, dtype=np.int64)
    expert_rank = np.ascontiguousarray(expert_rank, dtype=np.int32)
    EP, E = x_host.shape
    assert EP == model.EP and expert_rank.shape == (E,)
    out = np.empty(4, np.float64)
    loads = np.empty((5, EP), np.int64) if with_loads else None
    rc = lib().relibra_moe_time(_hp(x_host), E, C.byref(model), _hp(expert_rank), C.c_double(beta), C.c_double(t_ref),
                                _hp(out), _hp(loads) if with_loads else C.c_void_p(0))
    _check("relibra_moe_time", rc)
    res = dict(T=out[0], T_comp=out[1], T_comm=out[2], smooth=out[3])
    if with_loads:
        res["loads"] = loads
    return res


def relibra_reorder_sa(x_host, model, beta=20.0, gamma=0.9995, eps=1e-4, n_seeds=8, seed=0):
    """Algorithm 1 -> (expert_rank [E] int32, dict(T_start, T, smooth_start, smooth, iterations))."""
    x_host = np.ascontiguousarray(x_host, dtype=np.int64)
    EP, E = x_host.shape
    assert EP == model.EP
    rank = np.empty(E, np.int32)
    st = np.empty(5, np.float64)
    rc = lib().relibra_reorder_sa(_hp(x_host), E, C.byref(model), C.c_double(beta), C.c_double(gamma), C.c_double(eps),
                                  int(n_seeds), C.c_uint64(seed), _hp(rank), _hp(st))
    _check("relibra_reorder_sa", rc)
    return rank, dict(T_start=st[0], T=st[1], smooth_start=st[2], smooth=st[3], iterations=int(st[4]))


def relibra_reorder_sa_trace(x_host, model, beta=20.0, gamma=0.9995, eps=1e-4, seed=0, cap=64):
    """One seed of Algorithm 1 with its trajectory -> dict(start, rank, t_ref, smooth_start, iterations,
    moves [n,3] = (e_a, e_b, accepted), vals [n,3] = (u, T', theta))."""
    x_host = np.ascontiguousarray(x_host, dtype=np.int64)
    EP, E = x_host.shape
    assert EP == model.EP
    moves, vals = np.zeros((cap, 3), np.int32), np.zeros((cap, 3), np.float64)
    start, rank, st = np.empty(E, np.int32), np.empty(E, np.int32), np.empty(2, np.float64)
    fn = lib().relibra_reorder_sa_trace
    fn.restype = C.c_longlong
    it = fn(_hp(x_host), E, C.byref(model), C.c_double(beta), C.c_double(gamma), C.c_double(eps), C.c_uint64(seed),
            int(cap), _hp(moves), _hp(vals), _hp(start), _hp(rank), _hp(st))
    if it < 0:
        raise RelibraError("relibra_reorder_sa_trace", int(it))
    n = min(int(it), cap)
    return dict(start=start, rank=rank, t_ref=st[0], smooth_start=st[1], iterations=int(it), moves=moves[:n], vals=vals[:n])


def relibra_permute(ids, inst_ptr, inst_rows, inst_group, group_offset, X, E, G,
                    row_of=None, src_of=None, Xrows=None, workspace=None, err_flag=None):
    """One micro-batch: ids [T,k], plan tables (device int32), X [T,h] bf16 -> row_of, src_of, Xrows."""
    T, k = ids.shape
    N = T * k
    h = 0 if X is None else X.shape[1]
    dev = ids.device
    if row_of is None:
        row_of = torch.empty(N, dtype=torch.int32, device=dev)
    if src_of is None:
        src_of = torch.empty(N, dtype=torch.int32, device=dev)
    if Xrows is None and X is not None:
        Xrows = torch.empty((N, h), dtype=torch.bfloat16, device=dev)
    need = workspace_bytes(WS_PERMUTE, T, k, E, G, h, 0)
    if workspace is None:
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=dev)
    if err_flag is None:
        err_flag = new_err_flag(dev)
    rc = lib().relibra_permute(_dp(ids, torch.int32), _dp(inst_ptr, torch.int32), _dp(inst_rows, torch.int32),
                               _dp(inst_group, torch.int32), _dp(group_offset, torch.int32),
                               _dp(X), T, k, E, G, h, _dp(row_of), _dp(src_of), _dp(Xrows),
                               _dp(workspace), C.c_size_t(workspace.numel()), _dp(err_flag), _stream())
    _check("relibra_permute", rc)
    return row_of, src_of, Xrows


PERMUTE_STATIC_BYTES = 4 << 20


def relibra_permute_static(ids, inst_ptr, inst_rows, inst_group, group_offset, X, E, G, row_of, src_of, Xrows=None, err_flag=None):
    """relibra_permute with the library's static device scratch instead of a workspace: nothing is allocated, so
    every output (row_of, src_of [N] int32, Xrows [N,h] bf16 when X is given, err_flag) is the caller's."""
    T, k = ids.shape
    h = 0 if X is None else X.shape[1]
    assert row_of.shape == (T * k,) and src_of.shape == (T * k,) and err_flag is not None
    rc = lib().relibra_permute_static(_dp(ids, torch.int32), _dp(inst_ptr, torch.int32), _dp(inst_rows, torch.int32),
                                      _dp(inst_group, torch.int32), _dp(group_offset, torch.int32),
                                      _dp(X), T, k, E, G, h, _dp(row_of, torch.int32), _dp(src_of, torch.int32), _dp(Xrows),
                                      _dp(err_flag, torch.int32), _stream())
    _check("relibra_permute_static", rc)
    return row_of, src_of, Xrows


def relibra_assign_sources(x_host, ranks_per_node, inst_ptr, inst_rank, inst_rows):
    """x_host [EP,E] int64 + one micro-batch's plan tables (host) -> dict(src_first [EP,E],
    inst_src_rows, inst_src_base [n_inst,EP]) int32: which sources fill which instance (Section 5.2)."""
    x_host = np.ascontiguousarray(x_host, dtype=np.int64)
    inst_ptr, inst_rank, inst_rows = (np.ascontiguousarray(a, dtype=np.int32) for a in (inst_ptr, inst_rank, inst_rows))
    EP, E = x_host.shape
    n_inst = int(inst_ptr[E])
    out = dict(src_first=np.zeros((EP, E), np.int32), inst_src_rows=np.zeros((max(n_inst, 1), EP), np.int32),
               inst_src_base=np.zeros((max(n_inst, 1), EP), np.int32))
    rc = lib().relibra_assign_sources(_hp(x_host), E, EP, int(ranks_per_node), _hp(inst_ptr), _hp(inst_rank), _hp(inst_rows),
                                      _hp(out["src_first"]), _hp(out["inst_src_rows"]), _hp(out["inst_src_base"]))
    _check("relibra_assign_sources", rc)
    return out


def relibra_moe_time_split(inst_src_rows, inst_rank, model, with_loads=False):
    """Eq. 1-6 on a split -> dict(T, T_comp, T_comm[, loads [5,EP]])."""
    inst_src_rows = np.ascontiguousarray(inst_src_rows, dtype=np.int32)
    inst_rank = np.ascontiguousarray(inst_rank, dtype=np.int32)
    n_inst = min(inst_src_rows.shape[0], inst_rank.shape[0])
    assert inst_src_rows.shape[1] == model.EP
    out = np.empty(3, np.float64)
    loads = np.empty((5, model.EP), np.int64) if with_loads else None
    rc = lib().relibra_moe_time_split(_hp(inst_src_rows), n_inst, _hp(inst_rank), C.byref(model), _hp(out),
                                      _hp(loads) if with_loads else C.c_void_p(0))
    _check("relibra_moe_time_split", rc)
    res = dict(T=out[0], T_comp=out[1], T_comm=out[2])
    if with_loads:
        res["loads"] = loads
    return res


def relibra_permute_src(ids, inst_ptr, inst_group, group_offset, EP, src_first, inst_src_rows, inst_src_base, X, E, G,
                        row_of=None, src_of=None, Xrows=None, workspace=None, err_flag=None):
    """relibra_permute under a source-aware split (device int32 copies of relibra_assign_sources' tables)."""
    T, k = ids.shape
    N = T * k
    h = 0 if X is None else X.shape[1]
    dev = ids.device
    if row_of is None:
        row_of = torch.empty(N, dtype=torch.int32, device=dev)
    if src_of is None:
        src_of = torch.empty(N, dtype=torch.int32, device=dev)
    if Xrows is None and X is not None:
        Xrows = torch.empty((N, h), dtype=torch.bfloat16, device=dev)
    if workspace is None:
        workspace = torch.empty(max(workspace_bytes(WS_PERMUTE, T, k, E, G, h, 0), 1), dtype=torch.uint8, device=dev)
    if err_flag is None:
        err_flag = new_err_flag(dev)
    rc = lib().relibra_permute_src(_dp(ids, torch.int32), _dp(inst_ptr, torch.int32), _dp(inst_group, torch.int32),
                                   _dp(group_offset, torch.int32), int(EP), _dp(src_first, torch.int32),
                                   _dp(inst_src_rows, torch.int32), _dp(inst_src_base, torch.int32),
                                   _dp(X), T, k, E, G, h, _dp(row_of), _dp(src_of), _dp(Xrows),
                                   _dp(workspace), C.c_size_t(workspace.numel()), _dp(err_flag), _stream())
    _check("relibra_permute_src", rc)
    return row_of, src_of, Xrows


def relibra_moe_ffn_fwd(Xrows, group_offset, group_expert, Wg, Wu, Wd, g_begin=0, g_end=None,
                        Gt=None, U=None, A=None, Yrows=None, workspace=None, err_flag=None, flags=0):
    """Xrows [n_rows,h] bf16, weights bf16 -> (Gt, U, A [n_rows,h'], Yrows [n_rows,h]) bf16.
    group_expert indexes the parameter blocks of Wg/Wu/Wd (all Wg.shape[0] of them are addressable).
    flags = FWD_TRANSPOSED_WEIGHTS: the weights are the transposed copies ([E,h,h'], [E,h,h'], [E,h',h])."""
    n_rows, h = Xrows.shape
    E, hff = Wg.shape[0], (Wg.shape[2] if flags & FWD_TRANSPOSED_WEIGHTS else Wg.shape[1])
    G = group_expert.shape[0]
    g_end = G if g_end is None else g_end
    dev = Xrows.device
    mk = lambda cols: torch.empty((n_rows, cols), dtype=torch.bfloat16, device=dev)
    Gt = mk(hff) if Gt is None else Gt
    U = mk(hff) if U is None else U
    A = mk(hff) if A is None else A
    Yrows = mk(h) if Yrows is None else Yrows
    if workspace is None:
        need = workspace_bytes(WS_FFN_FWD, max(n_rows, 1), 1, E, G, h, hff)
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=dev)
    if err_flag is None:
        err_flag = new_err_flag(dev)
    rc = lib().relibra_moe_ffn_fwd(_dp(Xrows, torch.bfloat16), n_rows, _dp(group_offset, torch.int32),
                                   _dp(group_expert, torch.int32), G, g_begin, g_end, E,
                                   _dp(Wg, torch.bfloat16), _dp(Wu, torch.bfloat16), _dp(Wd, torch.bfloat16),
                                   h, hff, _dp(Gt), _dp(U), _dp(A), _dp(Yrows), int(flags),
                                   _dp(workspace), C.c_size_t(workspace.numel()), _dp(err_flag), _stream())
    _check("relibra_moe_ffn_fwd", rc)
    return Gt, U, A, Yrows


def relibra_row_tokens(src_of, k, T, row_tok=None, err_flag=None):
    """src_of [N] int32 (device, from relibra_permute) -> row_tok [N] int32: the token of every row."""
    N = src_of.shape[0]
    if row_tok is None:
        row_tok = torch.empty(N, dtype=torch.int32, device=src_of.device)
    if err_flag is None:
        err_flag = new_err_flag(src_of.device)
    rc = lib().relibra_row_tokens(_dp(src_of, torch.int32), N, int(k), int(T), _dp(row_tok, torch.int32), _dp(err_flag), _stream())
    _check("relibra_row_tokens", rc)
    return row_tok


def relibra_row_gates(src_of, gates, row_gate=None, err_flag=None):
    """src_of [N] int32, gates [T,k] fp32 (device) -> row_gate [N] fp32: the gate of the assignment every row serves."""
    N = src_of.shape[0]
    assert gates.numel() == N and gates.is_contiguous()
    if row_gate is None:
        row_gate = torch.empty(N, dtype=torch.float32, device=src_of.device)
    if err_flag is None:
        err_flag = new_err_flag(src_of.device)
    rc = lib().relibra_row_gates(_dp(src_of, torch.int32), _dp(gates, torch.float32), N, _dp(row_gate, torch.float32),
                                 _dp(err_flag), _stream())
    _check("relibra_row_gates", rc)
    return row_gate


def relibra_moe_ffn_fwd_gated(X, row_tok, row_gate, group_offset, group_expert, Wg, Wu, Wd, g_begin=0, g_end=None,
                              Gt=None, U=None, A=None, Ag=None, Yrows=None, workspace=None, err_flag=None, flags=0):
    """relibra_moe_ffn_fwd_gather that also stores Ag = row_gate * A (the operand of the gate-fused weight gradient).
    Passing the same tensor as A and Ag gates in place: Yrows then come out gate-scaled (combine with COMBINE_SUM)."""
    T, h = X.shape
    n_rows = row_tok.shape[0]
    E, hff = Wg.shape[0], (Wg.shape[2] if flags & FWD_TRANSPOSED_WEIGHTS else Wg.shape[1])
    G = group_expert.shape[0]
    g_end = G if g_end is None else g_end
    dev = X.device
    mk = lambda cols: torch.empty((n_rows, cols), dtype=torch.bfloat16, device=dev)
    Gt = mk(hff) if Gt is None else Gt
    U = mk(hff) if U is None else U
    A = mk(hff) if A is None else A
    Ag = mk(hff) if Ag is None else Ag
    Yrows = mk(h) if Yrows is None else Yrows
    if workspace is None:
        workspace = torch.empty(max(workspace_bytes(WS_FFN_FWD, max(n_rows, 1), 1, E, G, h, hff), 1), dtype=torch.uint8, device=dev)
    if err_flag is None:
        err_flag = new_err_flag(dev)
    rc = lib().relibra_moe_ffn_fwd_gated(_dp(X, torch.bfloat16), T, _dp(row_tok, torch.int32), _dp(row_gate, torch.float32), n_rows,
                                         _dp(group_offset, torch.int32), _dp(group_expert, torch.int32), G, g_begin, g_end, E,
                                         _dp(Wg, torch.bfloat16), _dp(Wu, torch.bfloat16), _dp(Wd, torch.bfloat16),
                                         h, hff, _dp(Gt), _dp(U), _dp(A), _dp(Ag), _dp(Yrows), int(flags),
                                         _dp(workspace), C.c_size_t(workspace.numel()), _dp(err_flag), _stream())
    _check("relibra_moe_ffn_fwd_gated", rc)
    return Gt, U, A, Ag, Yrows


def relibra_moe_ffn_bwd_gated(dOut, row_tok, row_gate, Gt, U, group_offset, group_expert, group_dw_slot, Wg, Wu, Wd,
                              src_of=None, g_begin=0, g_end=None, flags=0, dXrows=None, dgate=None, workspace=None,
                              dgate_scratch=None, err_flag=None, E=None):
    """Gate-fused data gradients (weight gradients deferred to relibra_moe_ffn_wgrad_batched): dOut [T,h] bf16 is the
    gradient of the combined output; -> dXrows [n_rows,h] bf16, dgate fp32 ([n_rows] by row, or with src_of in the
    gates' [T*k] layout).  The workspace holds dGt, dU for the batched weight gradients."""
    T, h = dOut.shape
    n_rows = row_tok.shape[0]
    hff = Wg.shape[2] if flags & BWD_TRANSPOSED_WEIGHTS else Wg.shape[1]
    E = Wg.shape[0] if E is None else int(E)
    G = group_expert.shape[0]
    g_end = G if g_end is None else g_end
    dev = dOut.device
    if dXrows is None:
        dXrows = torch.empty((n_rows, h), dtype=torch.bfloat16, device=dev)
    if dgate is None:
        dgate = torch.zeros(n_rows, dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = torch.empty(max(workspace_bytes(WS_FFN_BWD, max(n_rows, 1), 1, E, G, h, hff), 1), dtype=torch.uint8, device=dev)
    if dgate_scratch is None:
        dgate_scratch = torch.empty(max(workspace_bytes(WS_DGATE, max(n_rows, 1), 1, E, G, h, hff), 1), dtype=torch.uint8, device=dev)
    if err_flag is None:
        err_flag = new_err_flag(dev)
    rc = lib().relibra_moe_ffn_bwd_gated(_dp(dOut, torch.bfloat16), T, _dp(row_tok, torch.int32), _dp(row_gate, torch.float32),
                                         _dp(src_of, torch.int32), _dp(Gt, torch.bfloat16), _dp(U, torch.bfloat16), n_rows,
                                         _dp(group_offset, torch.int32), _dp(group_expert, torch.int32),
                                         _dp(group_dw_slot, torch.int32), G, g_begin, g_end, E,
                                         Wg.shape[0] if flags & BWD_REPLICA_WEIGHTS else E,   # parameter blocks addressable by slot
                                         _dp(Wg, torch.bfloat16), _dp(Wu, torch.bfloat16), _dp(Wd, torch.bfloat16), h, hff,
                                         _dp(dXrows), _dp(dgate, torch.float32), int(flags),
                                         _dp(workspace), C.c_size_t(workspace.numel()),
                                         _dp(dgate_scratch), C.c_size_t(dgate_scratch.numel()), _dp(err_flag), _stream())
    _check("relibra_moe_ffn_bwd_gated", rc)
    return dXrows, dgate


def relibra_moe_ffn_fwd_gather(X, row_tok, group_offset, group_expert, Wg, Wu, Wd, g_begin=0, g_end=None,
                               Gt=None, U=None, A=None, Yrows=None, workspace=None, err_flag=None, flags=0):
    """relibra_moe_ffn_fwd with the row gather fused in: X [T,h] token tensor, row_tok [n_rows]."""
    T, h = X.shape
    n_rows = row_tok.shape[0]
    E, hff = Wg.shape[0], (Wg.shape[2] if flags & FWD_TRANSPOSED_WEIGHTS else Wg.shape[1])
    G = group_expert.shape[0]
    g_end = G if g_end is None else g_end
    dev = X.device
    mk = lambda cols: torch.empty((n_rows, cols), dtype=torch.bfloat16, device=dev)
    Gt = mk(hff) if Gt is None else Gt
    U = mk(hff) if U is None else U
    A = mk(hff) if A is None else A
    Yrows = mk(h) if Yrows is None else Yrows
    if workspace is None:
        workspace = torch.empty(max(workspace_bytes(WS_FFN_FWD, max(n_rows, 1), 1, E, G, h, hff), 1), dtype=torch.uint8, device=dev)
    if err_flag is None:
        err_flag = new_err_flag(dev)
    rc = lib().relibra_moe_ffn_fwd_gather(_dp(X, torch.bfloat16), T, _dp(row_tok, torch.int32), n_rows,
                                          _dp(group_offset, torch.int32), _dp(group_expert, torch.int32), G, g_begin, g_end, E,
                                          _dp(Wg, torch.bfloat16), _dp(Wu, torch.bfloat16), _dp(Wd, torch.bfloat16),
                                          h, hff, _dp(Gt), _dp(U), _dp(A), _dp(Yrows), int(flags),
                                          _dp(workspace), C.c_size_t(workspace.numel()), _dp(err_flag), _stream())
    _check("relibra_moe_ffn_fwd_gather", rc)
    return Gt, U, A, Yrows


def relibra_moe_ffn_bwd(dYrows, Xrows, Gt, U, A, group_offset, group_expert, group_dw_slot,
                        Wg, Wu, Wd, dWg, dWu, dWd, g_begin=0, g_end=None, flags=0,
                        dXrows=None, workspace=None, err_flag=None, E=None):
    """-> dXrows [n_rows,h] bf16; dWg, dWu [slots,h',h] and dWd [slots,h,h'] fp32 are written in place.
    E = number of home experts (default Wg.shape[0]; pass it when the weights carry replica slots)."""
    n_rows, h = dYrows.shape                 # Xrows may be None when the weight gradients are deferred
    hff = Wg.shape[2] if flags & BWD_TRANSPOSED_WEIGHTS else Wg.shape[1]
    E = Wg.shape[0] if E is None else int(E)
    if flags & BWD_REPLICA_WEIGHTS and dWg is not None:
        assert Wg.shape[0] >= dWg.shape[0] and Wu.shape[0] >= dWg.shape[0] and Wd.shape[0] >= dWg.shape[0]
    G = group_expert.shape[0]
    g_end = G if g_end is None else g_end
    dev = dYrows.device
    if dXrows is None:
        dXrows = torch.empty((n_rows, h), dtype=torch.bfloat16, device=dev)
    if workspace is None:
        need = workspace_bytes(WS_FFN_BWD, max(n_rows, 1), 1, E, G, h, hff)
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=dev)
    if err_flag is None:
        err_flag = new_err_flag(dev)
    if flags & BWD_DEFER_WGRAD:
        # no dW is written: the slot table only selects parameter blocks (replica slots included)
        n_slots = dWg.shape[0] if dWg is not None else (Wg.shape[0] if flags & BWD_REPLICA_WEIGHTS else E)
    else:
        n_slots = dWg.shape[0]
        assert dWu.shape[0] == n_slots and dWd.shape[0] == n_slots
    rc = lib().relibra_moe_ffn_bwd(_dp(dYrows, torch.bfloat16), _dp(Xrows),
                                   _dp(Gt, torch.bfloat16), _dp(U, torch.bfloat16), _dp(A, torch.bfloat16), n_rows,
                                   _dp(group_offset, torch.int32), _dp(group_expert, torch.int32),
                                   _dp(group_dw_slot, torch.int32), G, g_begin, g_end, E, n_slots,
                                   _dp(Wg, torch.bfloat16), _dp(Wu, torch.bfloat16), _dp(Wd, torch.bfloat16),
                                   h, hff, _dp(dXrows), _dp(dWg, torch.float32), _dp(dWu, torch.float32),
                                   _dp(dWd, torch.float32), int(flags),
                                   _dp(workspace), C.c_size_t(workspace.numel()), _dp(err_flag), _stream())
    _check("relibra_moe_ffn_bwd", rc)
    return dXrows


def relibra_transpose_experts(W, out=None):
    """W [n, a, b] bf16 (device) -> out [n, b, a] with out[e] = W[e].T."""
    n, a, b = W.shape
    if out is None:
        out = torch.empty((n, b, a), dtype=torch.bfloat16, device=W.device)
    assert out.shape == (n, b, a)
    rc = lib().relibra_transpose_experts(_dp(W, torch.bfloat16), n, a, b, _dp(out, torch.bfloat16), _stream())
    _check("relibra_transpose_experts", rc)
    return out


class WgradMb(C.Structure):
    """relibra_wgrad_mb: one micro-batch's device pointers for the batched weight gradients."""
    _fields_ = [("dYrows_dev", C.c_void_p), ("Xrows_dev", C.c_void_p), ("A_save_dev", C.c_void_p),
                ("bwd_workspace_dev", C.c_void_p), ("inst_ptr_dev", C.c_void_p), ("inst_group_dev", C.c_void_p),
                ("group_offset_dev", C.c_void_p), ("X_dev", C.c_void_p), ("row_tok_dev", C.c_void_p), ("n_tokens", C.c_int),
                ("dOut_dev", C.c_void_p)]


def relibra_moe_ffn_wgrad_batched(mbs, E, dWg, dWu, dWd, accumulate=False, workspace=None, err_flag=None, tile=None):
    """mbs: list of dicts(dYrows, Xrows (or X and row_tok: fused gather), A, bwd_workspace, inst_ptr,
    inst_group, group_offset) of device tensors, one per micro-batch whose backward ran with BWD_DEFER_WGRAD.  Writes dWg, dWu [E,h',h],
    dWd [E,h,h'] fp32 in place (sum over all micro-batches and instances)."""
    n_mb = len(mbs)
    first = mbs[0]
    n_rows, hff = first["A"].shape
    # gate-fused form: dOut [T,h] (with X, row_tok) instead of dYrows, and A holding the gate-scaled activations
    h = (first["dYrows"] if first.get("dYrows") is not None else first["dOut"]).shape[1]
    G = first["group_offset"].shape[0] - 1
    inst_cap = first["inst_group"].shape[0]
    dev = dWg.device
    arr = (WgradMb * n_mb)()
    for i, m in enumerate(mbs):
        assert m["A"].shape == (n_rows, hff)
        if m.get("dYrows") is not None:
            assert m["dYrows"].shape == (n_rows, h)
            dy, dout = _dp(m["dYrows"], torch.bfloat16), C.c_void_p(0)
        else:
            assert m.get("Xrows") is None and m["dOut"].shape == m["X"].shape
            dy, dout = C.c_void_p(0), _dp(m["dOut"], torch.bfloat16)
        assert m["group_offset"].shape[0] == G + 1 and m["inst_group"].shape[0] == inst_cap and m["inst_ptr"].shape[0] == E + 1
        assert m["bwd_workspace"].numel() >= workspace_bytes(WS_FFN_BWD, max(n_rows, 1), 1, E, G, h, hff)
        if m.get("Xrows") is not None:          # group-ordered rows
            assert m["Xrows"].shape == (n_rows, h)
            x_rows, x_tok, rtok, n_tok = _dp(m["Xrows"], torch.bfloat16), C.c_void_p(0), C.c_void_p(0), 0
        else:                                   # token tensor + row -> token table (fused gather)
            assert m["X"].shape[1] == h and m["row_tok"].shape == (n_rows,)
            x_rows, x_tok, rtok, n_tok = C.c_void_p(0), _dp(m["X"], torch.bfloat16), _dp(m["row_tok"], torch.int32), m["X"].shape[0]
        arr[i] = WgradMb(dy, x_rows, _dp(m["A"], torch.bfloat16),
                         _dp(m["bwd_workspace"]), _dp(m["inst_ptr"], torch.int32), _dp(m["inst_group"], torch.int32),
                         _dp(m["group_offset"], torch.int32), x_tok, rtok, n_tok, dout)
    if workspace is None:
        workspace = torch.empty(max(workspace_bytes(WS_WGRAD_BATCHED, 0, 1, E, G, h, hff), 1), dtype=torch.uint8, device=dev)
    if err_flag is None:
        err_flag = new_err_flag(dev)
    rc = lib().relibra_moe_ffn_wgrad_batched(arr, n_mb, n_rows, G, inst_cap, int(E), h, hff,
                                             _dp(dWg, torch.float32), _dp(dWu, torch.float32), _dp(dWd, torch.float32),
                                             (WGRAD_ACCUMULATE if accumulate else 0) | {None: 0, "narrow": WGRAD_TILE_NARROW, "wide": WGRAD_TILE_WIDE}[tile],
                                             _dp(workspace), C.c_size_t(workspace.numel()),
                                             _dp(err_flag), _stream())
    _check("relibra_moe_ffn_wgrad_batched", rc)
    return err_flag


def relibra_replica_push(Wg, Wu, Wd, replica_expert, E, EP, r, n_workgroups=16, err_flag=None):
    """Fill the EP*r replica slots behind the E home blocks of Wg, Wu, Wd (in place) for one micro-batch."""
    assert Wg.shape[0] >= E + EP * r and Wu.shape[0] >= E + EP * r and Wd.shape[0] >= E + EP * r
    assert replica_expert.numel() == EP * r
    hff, h = Wg.shape[1], Wg.shape[2]
    if err_flag is None:
        err_flag = new_err_flag(Wg.device)
    rc = lib().relibra_replica_push(_dp(Wg, torch.bfloat16), _dp(Wu, torch.bfloat16), _dp(Wd, torch.bfloat16),
                                    _dp(replica_expert, torch.int32), int(E), int(EP), int(r), h, hff,
                                    int(n_workgroups), _dp(err_flag), _stream())
    _check("relibra_replica_push", rc)
    return err_flag


def relibra_replica_pull(dWg, dWu, dWd, replica_expert, E, EP, r, n_workgroups=16, err_flag=None):
    """Add the EP*r replica-slot gradients behind the E home blocks of dWg, dWu, dWd into their home blocks (in place)."""
    assert dWg.shape[0] >= E + EP * r and dWu.shape[0] >= E + EP * r and dWd.shape[0] >= E + EP * r
    assert replica_expert.numel() == EP * r
    hff, h = dWg.shape[1], dWg.shape[2]
    if err_flag is None:
        err_flag = new_err_flag(dWg.device)
    rc = lib().relibra_replica_pull(_dp(dWg, torch.float32), _dp(dWu, torch.float32), _dp(dWd, torch.float32),
                                    _dp(replica_expert, torch.int32), int(E), int(EP), int(r), h, hff,
                                    int(n_workgroups), _dp(err_flag), _stream())
    _check("relibra_replica_pull", rc)
    return err_flag


def relibra_unpermute_combine(mode, rows, row_of, T, k, gates=None, tok=None,
                              out_tok=None, out_rows=None, dgate=None, err_flag=None):
    """FWD/SUM -> out_tok [T,h] bf16; BWD -> (out_rows [N,h] bf16, dgate [T,k] fp32)."""
    h = rows.shape[1]
    dev = rows.device
    if err_flag is None:
        err_flag = new_err_flag(dev)
    if mode == COMBINE_BWD:
        if out_rows is None:
            out_rows = torch.empty((T * k, h), dtype=torch.bfloat16, device=dev)
        if dgate is None:
            dgate = torch.empty((T, k), dtype=torch.float32, device=dev)
    elif out_tok is None:
        out_tok = torch.empty((T, h), dtype=torch.bfloat16, device=dev)
    rc = lib().relibra_unpermute_combine(int(mode), _dp(rows, torch.bfloat16), _dp(tok), _dp(gates),
                                         _dp(row_of, torch.int32), T, k, h, _dp(out_tok), _dp(out_rows),
                                         _dp(dgate), _dp(err_flag), _stream())
    _check("relibra_unpermute_combine", rc)
    return (out_rows, dgate) if mode == COMBINE_BWD else out_tok


def prof_start(level=1, max_records=4096):
    """Bracket kernel launches with HIP events (level 1: grouped GEMMs, 2: every kernel)."""
    _check("relibra_prof_start", lib().relibra_prof_start(int(level), int(max_records)))


def prof_stop():
    """-> {kernel name: (total ms, launches)} for the launches recorded since prof_start."""
    ms = np.zeros(len(KERNELS), np.float64)
    n = np.zeros(len(KERNELS), np.int64)
    _check("relibra_prof_stop", lib().relibra_prof_stop(_hp(ms), _hp(n)))
    return {name: (float(ms[i]), int(n[i])) for i, name in enumerate(KERNELS) if n[i]}

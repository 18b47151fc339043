"""The permutation's entry point that allocates nothing (static device scratch) against the
workspace form, through the C ABI: two calls in a row on one GPU, the second on a smaller input,
bit-exact indices and gathered rows; sizes beyond the static array are refused."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_2605_08639_amd as rl

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _case(cfg):
    ids, _ = wl.make_routing(cfg, 0)
    counts = oracle.route_hist(ids[None], cfg.E)[0]
    p = rl.relibra_plan(counts, cfg.k, cfg.EP, cfg.rpn, cfg.r)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    tabs = [t(p[key][0]) for key in ("inst_ptr", "inst_rows", "inst_group", "group_offset")]
    X, _ = wl.make_tokens(cfg, 0)
    return t(ids), tabs, X.to(DEV)


def test_permute_static_equals_permute_on_two_calls_in_a_row():
    big = wl.small_config(E=128, k=8, EP=8, r=2, T=6000, n_mb=1, h=128, index=61)     # 375 units of 128 assignments + a ragged one
    small = wl.small_config(E=16, k=4, EP=4, r=2, T=777, n_mb=1, h=64, index=62)
    for cfg in (big, small):                                    # the second call finds the first one's leftovers in the array
        ids_d, tabs, X_d = _case(cfg)
        want_row, want_src, want_rows = rl.relibra_permute(ids_d, *tabs, X_d, cfg.E, cfg.G)
        row_of = torch.full((cfg.N,), -7, dtype=torch.int32, device=DEV)
        src_of = torch.full((cfg.N,), -7, dtype=torch.int32, device=DEV)
        Xrows = torch.zeros((cfg.N, cfg.h), dtype=torch.bfloat16, device=DEV)
        err = rl.new_err_flag()
        rl.relibra_permute_static(ids_d, *tabs, X_d, cfg.E, cfg.G, row_of, src_of, Xrows, err_flag=err)
        torch.cuda.synchronize()
        assert err.item() == 0
        assert torch.equal(row_of, want_row) and torch.equal(src_of, want_src)
        assert torch.equal(Xrows.view(torch.int16), want_rows.view(torch.int16))
        # and against the oracle's definition of the permutation
        p_row, p_src = oracle.permute(ids_d.cpu().numpy(), cfg.E, *[x.cpu().numpy() for x in tabs])
        assert np.array_equal(row_of.cpu().numpy(), p_row) and np.array_equal(src_of.cpu().numpy(), p_src)


def test_permute_static_refuses_sizes_beyond_its_array():
    E, k = 4096, 1
    T = 128 * 300                                               # (300 + 4) units x 4096 experts x 4 bytes > 4 MiB
    assert rl.workspace_bytes(rl.WS_PERMUTE, T, k, E, E, 0, 0) > rl.PERMUTE_STATIC_BYTES
    z = lambda n: torch.zeros(n, dtype=torch.int32, device=DEV)
    with pytest.raises(rl.RelibraError) as ei:
        rl.relibra_permute_static(z(T).view(T, k), z(E + 1), z(E), z(E), z(E + 1), None, E, E, z(T), z(T), err_flag=rl.new_err_flag())
    assert ei.value.status == rl.EWORKSPACE

"""tns_run_static (the entry point for callers that cannot allocate) against tns_run: same outputs,
bit for bit, on two calls in a row, the second with a smaller input (the static scratch keeps the
first call's contents)."""
import numpy as np
import pytest

from paper_2311_17410_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2311_17410_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("policy", [0, 1])
def test_static_scratch_entry_point_equals_tns_run(B, policy):
    import torch
    from _harness import build_plan
    wl = W.c2()
    plan = build_plan(B, wl, policy, 0, seed=7)
    targets, t_start, t_end, _ = wl.queries(window_frac=0.25)
    dev = torch.device("cuda", 0)
    d_t, d_b, d_e = (torch.from_numpy(a).to(dev) for a in (targets, t_start, t_end))
    p = lambda t: 0 if t is None else t.data_ptr()
    stream = torch.cuda.current_stream().cuda_stream
    names = ("nbr", "eid", "ts", "count", "rowptr", "cmp_nbr", "cmp_eid", "cmp_ts")
    for Q, tb in ((len(targets), None), (100_003, d_b), (0, None)):     # several tiles + ragged tail, then smaller, then empty
        ref = plan.run(d_t[:Q], None if tb is None else tb[:Q], d_e[:Q], query_id_base=5)
        got = plan.alloc_outputs(Q, compact=True)
        for k in names:
            got[k].fill_(-7)
        B.tns_run_static(plan.handle, Q, p(d_t), p(tb), p(d_e), 0, 5, p(got["nbr"]), p(got["eid"]), p(got["ts"]),
                         p(got["count"]), p(got["rowptr"]), p(got["cmp_nbr"]), p(got["cmp_eid"]), p(got["cmp_ts"]), stream)
        torch.cuda.synchronize()
        assert not plan.status(None) and not plan.status(ref["workspace"])
        total = int(ref["rowptr"][-1].item())
        assert int(got["rowptr"][-1].item()) == total
        for k in ("nbr", "eid", "count", "rowptr"):
            assert torch.equal(got[k], ref[k]), (Q, k)
        assert torch.equal(got["ts"].view(torch.int32), ref["ts"].view(torch.int32)), (Q, "ts")
        for k in ("cmp_nbr", "cmp_eid"):
            assert torch.equal(got[k][:total], ref[k][:total]), (Q, k)
        assert torch.equal(got["cmp_ts"][:total].view(torch.int32), ref["cmp_ts"][:total].view(torch.int32)), (Q, "cmp_ts")
    # sizes beyond the static array are refused, nothing is launched
    got = plan.alloc_outputs(16, compact=True)
    with pytest.raises(B.TnsError) as ei:
        B.tns_run_static(plan.handle, (1 << 24) + 1, p(d_t), 0, p(d_e), 0, 0, p(got["nbr"]), p(got["eid"]), p(got["ts"]),
                         p(got["count"]), p(got["rowptr"]), p(got["cmp_nbr"]), p(got["cmp_eid"]), p(got["cmp_ts"]), stream)
    assert ei.value.status == B.TNS_ESIZE
    plan.close()

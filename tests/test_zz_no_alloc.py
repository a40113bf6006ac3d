"""The entry point that allocates nothing (mmbp_local_search_static), called through the C ABI,
against mmbp_local_search with a caller-provided workspace: bit-exact on every output, on two calls in
a row that share the library's static scratch, the second with a smaller input."""
import numpy as np
import pytest

from paper_2502_15763_amd import workloads as W
from gpu_util import say, to_dev, u64, gpu_local_search

pytestmark = pytest.mark.gpu


def _static_local_search(cost, assign0, M, cap, max_passes):
    import torch
    from paper_2502_15763_amd import api
    dcost, dassign = to_dev(cost), to_dev(assign0.astype(np.int32))
    S, N = cost.shape
    dev = dcost.device
    load = torch.empty((S, M), dtype=torch.int64, device=dev)
    mk = torch.empty(S, dtype=torch.int64, device=dev)
    passes = torch.empty(S, dtype=torch.int32, device=dev)
    evals = torch.empty(S, dtype=torch.int64, device=dev)
    status = torch.empty(S, dtype=torch.int32, device=dev)
    log = torch.full((S, max_passes), -1, dtype=torch.int64, device=dev)
    rc = api.mmbp_local_search_static(dcost, M, cap, max_passes, dassign, load, mk, passes, status, evals_out=evals,
                                      applied_log=log, raise_on_error=False)
    torch.cuda.synchronize()
    return dict(rc=rc, assign=dassign.cpu().numpy(), load=load.cpu().numpy(), makespan=mk.cpu().numpy(),
                passes=passes.cpu().numpy(), evals=u64(evals), status=status.cpu().numpy(), log=u64(log))


def _same(a, b, label):
    assert a["rc"] == 0 and b["rc"] == 0, (label, a["rc"], b["rc"])
    for k in ("status", "passes", "makespan", "evals", "load", "assign", "log"):
        assert np.array_equal(a[k], b[k]), f"{label}: {k} differs between the static-scratch call and the workspace call"


def test_static_scratch_entry_matches_workspace_entry():
    from paper_2502_15763_amd import api
    rng = np.random.default_rng(2718)
    # two calls in a row on shapes that need the scratch (too large for one workgroup's LDS), the
    # second smaller, so that it runs over what the first left behind; then one that prefers it
    # and one that needs none
    for (S, N, M, cap, passes, hi) in [(3, 14000, 6, 2500, 8, 30000), (2, 13000, 5, 2700, 6, 4),
                                       (1, 4096, 16, 256, 20, 50000), (4, 300, 5, 70, 50, 1000)]:
        need = api.mmbp_workspace_bytes(S, N, M)
        say(f"static scratch S={S} N={N} M={M} workspace_bytes={need}")
        assert need <= api.STATIC_SCRATCH_BYTES
        cost, assign = W.random_offline(rng, S, N, M, cap, cost_hi=hi, dtype=np.int32)
        ref = gpu_local_search(cost, assign, M, cap, passes)
        got = _static_local_search(cost, assign, M, cap, passes)
        _same(got, ref, f"S={S} N={N} M={M}")
        assert int(ref["passes"].sum()) > 0


def test_static_scratch_entry_rejects_what_does_not_fit():
    from paper_2502_15763_amd import api
    S, N, M, cap = 8, 65536, 64, 1024
    assert api.mmbp_workspace_bytes(S, N, M) > api.STATIC_SCRATCH_BYTES
    cost = np.ones((S, N), np.int32)
    assign = W.round_robin(S, N, M)
    r = _static_local_search(cost, assign, M, cap, 1)
    assert r["rc"] == api.EWORKSPACE
    assert "MMBP_STATIC_SCRATCH_BYTES" in api.mmbp_strerror(r["rc"])

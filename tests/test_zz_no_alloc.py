"""The entry point that allocates nothing (am_subset_indices_static) against the ordinary one
(am_subset_indices), through the C ABI: same index list and count bit for bit, on two calls in a row,
the second on a smaller stage, so that what the first call left in the library's static scratch
array must not leak into the second."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _both(am, st, t, capacity):
    want, k = st.subset_indices(t, capacity=capacity)
    out = torch.full((capacity,), -1, dtype=torch.int64, device="cuda")
    count = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    st.subset_indices_static(t, out, count)
    torch.cuda.synchronize()
    got_k = int(count.item())
    assert got_k == k, (got_k, k)
    assert torch.equal(out[:min(k, capacity)], want)
    assert bool((out[min(k, capacity):] == -1).all())          # nothing written past the list
    return k


def test_static_scratch_entry_point_matches_the_ordinary_one(amlib):
    am = amlib
    big = am.init_state(am.make_config(3_000_017, 1, fraction=0.05, seed=21, optimizer=am.OPT_SGD, beta1=0.0,
                                       correction=am.CORR_NONE), None)
    small = am.init_state(am.make_config(70_001, 1, fraction=0.3, seed=22, optimizer=am.OPT_SGD, beta1=0.0,
                                         correction=am.CORR_NONE), None)
    print("static scratch: big stage", flush=True)
    k1 = _both(am, big, 7, 200_000)
    print("static scratch: small stage", flush=True)
    k2 = _both(am, small, 7, 30_000)
    assert k1 > k2 > 0
    print("static scratch: big stage again, truncated output", flush=True)
    _both(am, big, (1 << 33) + 1, 1000)
    # the stratified rule and a stage of one coordinate go through the same scratch
    one = am.init_state(am.make_config(1, 1, fraction=1.0, seed=3, optimizer=am.OPT_SGD, beta1=0.0,
                                       correction=am.CORR_NONE), None)
    assert _both(am, one, 1, 4) == 1
    strat = am.init_state(am.make_config(500_003, 1, fraction=0.01, seed=4, optimizer=am.OPT_SGD, beta1=0.0,
                                         correction=am.CORR_NONE, subset_kind=am.SUBSET_STRATIFIED), None)
    _both(am, strat, 5, 6000)


def test_static_scratch_entry_point_refuses_a_stage_beyond_its_limit(amlib):
    am = amlib
    n = (1 << 27) + 1
    st = am.init_state(am.make_config(n, 1, fraction=1e-6, seed=1, optimizer=am.OPT_SGD, beta1=0.0,
                                      correction=am.CORR_NONE), None)
    out = torch.zeros(1024, dtype=torch.int64, device="cuda")
    count = torch.zeros(1, dtype=torch.int64, device="cuda")
    with pytest.raises(am.AsyncMeshError) as e:
        st.subset_indices_static(1, out, count)
    assert e.value.status == -1 and "static scratch" in str(e.value)
    idx, k = st.subset_indices(1, capacity=1024)                # the ordinary entry point still serves it
    assert k == idx.numel()

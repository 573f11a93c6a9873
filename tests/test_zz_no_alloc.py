"""stalloc_lower_bound_static (the entry point without workspace, for callers that cannot
allocate) against stalloc_lower_bound, through the C ABI: two calls in a row, the second on a
smaller trace, so that whatever the first call left in the library's buffer is in the way."""
import ctypes

import numpy as np
import pytest

from workloads import make_trace

pytestmark = pytest.mark.gpu


def _raw_trace(S, size, ta, tf, t_end):
    return S._Trace(size.numel(), int(t_end), size.data_ptr(), ta.data_ptr(), tf.data_ptr())


def _both(S, torch, tr_np):
    """(lower bound, earliest t, status) of the two entry points on one trace, raw ctypes calls."""
    size, ta, tf = S.trace_to_device(tr_np)
    tr = _raw_trace(S, size, ta, tf, tr_np.t_end)
    stream = torch.cuda.current_stream().cuda_stream
    res = []
    for static in (False, True):
        lb = torch.full((1,), -7, dtype=torch.int64, device="cuda")
        t = torch.full((1,), -7, dtype=torch.int32, device="cuda")
        st = torch.full((1,), -7, dtype=torch.int32, device="cuda")
        if static:
            rc = S.lib.stalloc_lower_bound_static(ctypes.byref(tr), lb.data_ptr(), t.data_ptr(), st.data_ptr(), stream)
        else:
            need = ctypes.c_size_t(0)
            assert S.lib.stalloc_lower_bound(ctypes.byref(tr), None, None, None, None, ctypes.byref(need), None) == 0
            ws = torch.empty(need.value, dtype=torch.uint8, device="cuda")
            rc = S.lib.stalloc_lower_bound(ctypes.byref(tr), lb.data_ptr(), t.data_ptr(), st.data_ptr(),
                                           ws.data_ptr(), ctypes.byref(need), stream)
        assert rc == 0
        torch.cuda.synchronize()
        res.append((int(lb.cpu().numpy().view(np.uint64)[0]), int(t.item()), int(st.item())))
    return res


def test_static_entry_point_matches_on_two_calls_in_a_row(oracle):
    import torch
    assert torch.cuda.is_available(), "this test needs the GPU"
    import paper_2507_16274_amd as S
    # config 5 first (t_end = 399 496 fills most of the buffer), then the 96 requests of config 1,
    # then a trace with tied timestamps in between the two sizes
    rng = np.random.default_rng(5)
    n = 3000
    ts = rng.integers(0, 500, size=n)
    tied = type("T", (), {})()
    tied.size = (rng.integers(1, 1 << 33, size=n) * 512).astype(np.uint64)
    tied.t_alloc = ts.astype(np.uint32)
    tied.t_free = (ts + rng.integers(1, 300, size=n)).astype(np.uint32)
    tied.t_end = int(tied.t_free.max())
    for tr_np in (make_trace(5), make_trace(1), tied):
        with_ws, static = _both(S, torch, tr_np)
        assert static == with_ws
        want = oracle.lower_bound(tr_np.size, tr_np.t_alloc, tr_np.t_free, tr_np.t_end)
        assert static[2] == 0 and static[:2] == want


def test_static_entry_point_rejects_what_it_cannot_hold():
    import torch
    import paper_2507_16274_amd as S
    size = torch.ones(4, dtype=torch.int64, device="cuda")
    ta = torch.zeros(4, dtype=torch.int32, device="cuda")
    tf = torch.ones(4, dtype=torch.int32, device="cuda")
    out = torch.zeros(4, dtype=torch.int64, device="cuda")
    tr = _raw_trace(S, size, ta, tf, S.STATIC_MAX_T_END + 1)
    assert S.lib.stalloc_lower_bound_static(ctypes.byref(tr), out.data_ptr(), None, out[1:].data_ptr(), None) == 9
    assert S.lib.stalloc_status_string(9).decode() == "STALLOC_ERR_TOO_LARGE"
    tr = _raw_trace(S, size, ta, tf, S.STATIC_MAX_T_END)
    assert S.lib.stalloc_lower_bound_static(ctypes.byref(tr), None, None, out.data_ptr(), None) == 1   # no output
    # a malformed trace is reported through the status word like in stalloc_lower_bound
    tf0 = torch.zeros(4, dtype=torch.int32, device="cuda")
    st = torch.zeros(1, dtype=torch.int32, device="cuda")
    tr = _raw_trace(S, size, ta, tf0, 8)
    assert S.lib.stalloc_lower_bound_static(ctypes.byref(tr), out.data_ptr(), None, st.data_ptr(),
                                            torch.cuda.current_stream().cuda_stream) == 0
    torch.cuda.synchronize()
    assert int(st.item()) == 2

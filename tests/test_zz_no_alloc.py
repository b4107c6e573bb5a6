"""tg_assign_static (the entry point that allocates nothing: its workspace is an array in the library's
own device data) against tg_assign on the same problems, through the C ABI: every integer output bit
for bit, the floats of the summaries bit for bit as well (same kernels, same inputs).  Two calls in a
row on the same GPU, the second on a smaller problem, so that whatever the first call left in the
shared array must not matter; then a problem that is too large for the array is refused."""
import numpy as np
import pytest

import gen

pytestmark = pytest.mark.gpu

KEYS = ("node", "units", "act_us", "defer_reason", "node_used", "task_sum_us", "node_obj", "summary")


def _run(tg, p, static):
    import torch
    P = tg.Problem(p)
    bufs = P.alloc_assign()
    if static:
        assert P.assign_ws_bytes <= 32 << 20
        del bufs["ws"]
    for k in KEYS:
        bufs[k].fill_(77 if bufs[k].dtype == torch.uint8 else -3)
    if static:
        P.assign_static(None, bufs)
    else:
        P.assign(None, bufs)
    torch.cuda.synchronize()
    out = {k: bufs[k].cpu().numpy().copy() for k in KEYS}
    P.free()
    return out


def test_assign_static_matches_assign_twice_in_a_row():
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    from paper_2603_13019_amd import tg
    tg.load()
    big = gen.make_config(2, B=96)                                   # 96 x 1024 actions: 5.6 MB of workspace
    small = gen.make_random_problem(11, B=3, N=150, n_cpu=3, n_gpu=2, n_api=2)
    got_big = _run(tg, big, True)
    got_small = _run(tg, small, True)                                # second call, smaller input, same array
    for name, p, got in (("workload-2 shape", big, got_big), ("small", small, got_small)):
        want = _run(tg, p, False)
        for k in KEYS:
            np.testing.assert_array_equal(got[k], want[k], err_msg=f"{name} {k}")
    # and once more the larger one after the smaller one
    again = _run(tg, big, True)
    for k in KEYS:
        np.testing.assert_array_equal(again[k], got_big[k], err_msg=f"repeat {k}")


def test_assign_static_refuses_what_does_not_fit():
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    from paper_2603_13019_amd import tg
    p = gen.make_config(2, B=700)                                    # 41 MB of workspace
    P = tg.Problem(p)
    assert P.assign_ws_bytes > 32 << 20
    bufs = P.alloc_assign()
    bufs["node"].fill_(-3)
    with pytest.raises(tg.TgError) as e:
        P.assign_static(None, bufs)
    assert e.value.code == -7
    torch.cuda.synchronize()
    assert bool((bufs["node"] == -3).all())                          # nothing was launched
    P.free()

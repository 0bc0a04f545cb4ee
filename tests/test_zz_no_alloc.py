"""GPU test of lohan_grad_sqnorm_static, the entry point for callers that cannot allocate: its
results must equal lohan_grad_sqnorm's (same kernels, the workspace being a static device array
of the library) on calls in a row that share that array, the later ones on smaller inputs."""
import numpy as np
import pytest
import torch

import paper_2403_06504_amd as lohan
from paper_2403_06504_amd import synthetic_inputs as synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
RTOL_SQNORM = 1e-5          # the bar on the squared norm; the flag is bit-exact


def gradients(n, seed, plant=None):
    wl = synth.WORKLOADS["gpt13b"].with_n(n)
    g = synth.make_block(wl, seed=seed, device=DEV)["g"]
    if plant is not None:
        index, bits = plant
        g.view(torch.int16)[index] = np.int16(np.uint16(bits).view(np.int16))
    return g


def run_both(g, n, loss_scale, ws):
    """(flag, sqnorm bits) from the workspace entry point and from the static one."""
    out = []
    for static in (False, True):
        flag = torch.full((1,), 7, dtype=torch.int32, device=DEV)           # stale on purpose
        sqnorm = torch.full((1,), -1.0, dtype=torch.float64, device=DEV)
        if static:
            lohan.lohan_grad_sqnorm_static(g, n, loss_scale, sqnorm, flag)
        else:
            lohan.lohan_grad_sqnorm(g, n, loss_scale, sqnorm, flag, ws)
        torch.cuda.synchronize()
        out.append((int(flag.cpu().item()), sqnorm.cpu().numpy().view(np.uint64)[0]))
    return out


def test_static_workspace_matches_caller_workspace_on_calls_in_a_row(oracle):
    ws = lohan.new_workspace(DEV)
    # n spans many tiles with a ragged tail; each later call is smaller than the one before, and
    # the first one overflows, so nothing stale may survive in the shared array.
    cases = [(5_000_003, 1, (5_000_002, 0x7C00)), (1_234_567, 2, None), (70_001, 3, None),
             (9, 4, (3, 0xFE00)), (0, 5, None)]
    for n, seed, plant in cases:
        g = gradients(max(n, 8), seed, plant)[:n] if n else torch.empty(0, dtype=torch.float16,
                                                                        device=DEV)
        (f_ws, s_ws), (f_st, s_st) = run_both(g, n, 65536.0, ws)
        want_flag = 1 if plant is not None else 0
        assert f_ws == want_flag and f_st == want_flag, (n, f_ws, f_st)
        if want_flag == 0:
            assert s_st == s_ws, (n, s_st, s_ws)                   # same kernels, same order
            host = synth.to_numpy_bits(g) if n else np.zeros(0, dtype=np.uint16)
            want = oracle.grad_sqnorm(host, 65536.0)
            got = float(np.uint64(s_st).view(np.float64))
            assert abs(got - want) <= RTOL_SQNORM * want, (n, got, want)


def test_static_entry_point_rejects_what_it_cannot_do():
    g = gradients(1024, 0)
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    sqnorm = torch.zeros(1, dtype=torch.float64, device=DEV)
    with pytest.raises(lohan.LohanError) as e:
        lohan.lohan_grad_sqnorm_static(g.data_ptr(), (1 << 40) + 1, 1.0, sqnorm, flag)
    assert e.value.status == 6 and "maximum" in str(e.value)
    with pytest.raises(lohan.LohanError) as e:
        lohan.lohan_grad_sqnorm_static(g, 1024, 0.0, sqnorm, flag)
    assert e.value.status == 3

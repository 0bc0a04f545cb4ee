"""GPU parity of the one-launch step for small blocks (lohan_adam_small_block_step): the same
oracle, the same bar as the two-call step, plus what is particular to it -- the depth boundaries
of the register-resident kernels, the grid-wide wait and its bounded give-up path."""
import sys

import numpy as np
import pytest
import torch

import paper_2403_06504_amd as lohan
from paper_2403_06504_amd import synthetic_inputs as synth

from gpu_util import RTOL_SQNORM, DeviceBlock, assert_state_parity, oracle_steps

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TILE = 1024
ZERO_ULP = {"p": 0, "m": 0, "v": 0, "p16": 0}


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module", autouse=True)
def _library_is_native():
    assert torch.cuda.is_available(), "these tests need a GPU"
    lohan.load_library()
    lohan.lohan_tuning_set_launch_config()
    lohan.lohan_tuning_set_wait_limit()
    yield
    lohan.lohan_tuning_set_wait_limit()


def workload(n, step=100, S=65536.0):
    return synth.Workload(name=f"n{n}", n=n, step=step, loss_scale=S, zero_moments=False)


def small_step(blk: DeviceBlock, hy: dict, flags=0, want_norm=True, stream=None):
    lohan.lohan_adam_small_block_step(blk.p, blk.m, blk.v, blk.g, blk.p16, blk.n, hy["lr"],
                                      hy["beta1"], hy["beta2"], hy["eps"], hy["weight_decay"],
                                      hy["step"], hy["loss_scale"],
                                      blk.sqnorm if want_norm else None, blk.flag, flags, blk.ws,
                                      stream=stream)


def small_steps(blk, hy, steps, flags=0):
    out = []
    for k in range(steps):
        blk.flag.fill_(9)                                   # stale on purpose
        small_step(blk, dict(hy, step=hy["step"] + k), flags=flags)
        torch.cuda.synchronize()
        out.append(blk.flag_value())
    return out


def check_norm(oracle, blk, host, S, what):
    want = oracle.grad_sqnorm(host["g"], S)
    got = float(blk.sqnorm.cpu().item())
    assert abs(got - want) <= RTOL_SQNORM * want, (what, got, want)


def depth_boundaries():
    """Sizes around every point where the launcher changes depth or reaches a workgroup's last
    slot: the capacity of each depth follows from the largest n by the depths' ratios, so take a
    spread of tile counts instead of re-deriving the library's table here."""
    max_n = lohan.lohan_adam_small_block_max_n()
    tiles_max = max_n // TILE
    picks = {tiles_max, tiles_max - 1, tiles_max * 3 // 4, tiles_max * 4 // 5 + 1,
             tiles_max * 14 // 15, tiles_max * 2 // 3 - 1, tiles_max // 2 + 3}
    return max_n, sorted(t * TILE + r for t, r in zip(sorted(picks), (0, 1, 1023, 517, 4, 0, 3)))


@pytest.mark.parametrize("l2_mode", [False, True])
def test_small_sizes_ten_chained_steps(oracle, l2_mode):
    """Every residue of the 4-wide vectors and of the 1024-element tile, one workgroup and a few,
    ten chained steps each."""
    sizes = list(range(0, 10)) + [255, 256, 257, 1023, 1024, 1025, 2047, 2048, 3071, 3072, 3073,
                                  4099, 7 * 1024 + 5, 65_537, 1_000_003]
    flags = lohan.LOHAN_FLAG_L2_MODE if l2_mode else 0
    for n in sizes:
        say(f"[small-block] n={n} l2={l2_mode}")
        wl = workload(n)
        blk = DeviceBlock(synth.make_block(wl, seed=n, device=DEV))
        host = blk.host()
        hy = wl.hyper()
        assert small_steps(blk, hy, 10, flags=flags) == [0] * 10
        assert oracle_steps(oracle, host, hy, 10, l2_mode=l2_mode, nthreads=4) == [0] * 10
        assert assert_state_parity(blk.host(), host, what=f"n={n}") == ZERO_ULP
        if n:
            check_norm(oracle, blk, host, wl.loss_scale, f"n={n}")
        else:
            assert float(blk.sqnorm.cpu().item()) == 0.0


def test_config1_h768_block_and_depth_boundaries(oracle):
    """The h=768 block (the workload this entry point exists for) and sizes around every depth
    boundary up to the largest the device takes, three chained steps each."""
    max_n, sizes = depth_boundaries()
    say(f"[small-block] max_n={max_n}")
    assert max_n >= synth.WORKLOADS["gpt_h768"].n, "the h=768 block must fit"
    for n in [synth.WORKLOADS["gpt_h768"].n] + sizes + [max_n]:
        say(f"[small-block] n={n}")
        wl = workload(n)
        blk = DeviceBlock(synth.make_block(wl, seed=n % 1009, device=DEV))
        host = blk.host()
        hy = wl.hyper()
        assert small_steps(blk, hy, 3) == [0] * 3
        assert oracle_steps(oracle, host, hy, 3) == [0] * 3
        assert assert_state_parity(blk.host(), host, what=f"n={n}") == ZERO_ULP
        check_norm(oracle, blk, host, wl.loss_scale, f"n={n}")


def test_same_state_as_the_two_call_step_and_same_bits_twice():
    n = synth.WORKLOADS["gpt_h768"].n
    wl = workload(n)
    hy = wl.hyper()
    runs = []
    for which in ("small", "small", "two-call"):
        blk = DeviceBlock(synth.make_block(wl, seed=5, device=DEV))
        for k in range(2):
            h = dict(hy, step=hy["step"] + k)
            if which == "small":
                small_step(blk, h)
            else:
                blk.norm(wl.loss_scale)
                blk.step(h, flags=lohan.LOHAN_FLAG_PRECHECKED)
        torch.cuda.synchronize()
        assert blk.flag_value() == 0
        runs.append((blk.host(), float(blk.sqnorm.cpu().item())))
    for k in ("p", "m", "v", "p16"):
        assert np.array_equal(runs[0][0][k], runs[1][0][k]), k
        assert np.array_equal(runs[0][0][k], runs[2][0][k]), k
    assert runs[0][1] == runs[1][1]                                   # fixed order of its own
    assert abs(runs[0][1] - runs[2][1]) <= RTOL_SQNORM * runs[2][1]


@pytest.mark.parametrize("n", [1, 1023, 1024, 4099, 1_000_003, 7_077_888])
def test_overflow_anywhere_skips_the_whole_block(oracle, n):
    """A non-finite gradient in the first or last workgroup's share, on a tile boundary or in the
    ragged tail must keep every workgroup from writing: state bit-identical, flag 1.  The largest
    finite values must not."""
    wl = workload(n)
    hy = wl.hyper()
    base = synth.make_block(wl, seed=3, device=DEV)
    positions = sorted({0, n - 1, n // 2, (n // TILE) * TILE % n, max(0, (n // TILE) * TILE - 1)})
    for pat in (0x7C00, 0xFC00, 0x7E01, 0x7BFF, 0xFBFF):
        for pos in positions:
            blk = DeviceBlock({k: t.clone() for k, t in base.items()})
            blk.g.view(torch.int16)[pos] = pat if pat < 0x8000 else pat - 0x10000
            host = blk.host()
            want = oracle.grad_overflow_check(host["g"])
            assert want == (0 if pat in (0x7BFF, 0xFBFF) else 1)
            assert small_steps(blk, hy, 1) == [want]
            assert oracle_steps(oracle, host, hy, 1, nthreads=8) == [want]
            after = blk.host()
            for k in ("p", "m", "v", "p16"):
                assert np.array_equal(after[k].view(np.uint8), host[k].view(np.uint8)), (k, pat, pos)


def test_fp16_copy_and_no_norm(oracle):
    n = 3_000_001
    wl = workload(n)
    hy = wl.hyper()
    blk = DeviceBlock(synth.make_block(wl, seed=11, device=DEV))
    host = blk.host()
    blk.sqnorm.fill_(-3.0)
    small_step(blk, hy, flags=lohan.LOHAN_FLAG_P16_FP16, want_norm=False)
    torch.cuda.synchronize()
    assert blk.flag_value() == 0 and float(blk.sqnorm.cpu().item()) == -3.0
    f = oracle.adam_block_step(host["p"], host["m"], host["v"], host["g"], host["p16"],
                               lr=hy["lr"], beta1=hy["beta1"], beta2=hy["beta2"], eps=hy["eps"],
                               weight_decay=hy["weight_decay"], step=hy["step"],
                               loss_scale=hy["loss_scale"], half_out=True, nthreads=8)
    assert f == 0
    assert assert_state_parity(blk.host(), host, what="fp16 copy") == ZERO_ULP


def test_limits_and_argument_errors():
    max_n = lohan.lohan_adam_small_block_max_n()
    n = 4096
    wl = workload(n)
    hy = wl.hyper()
    blk = DeviceBlock(synth.make_block(wl, seed=0, device=DEV))
    before = blk.host()

    # beyond the limit nothing is launched (the arrays here are far shorter: nothing may run)
    too_large = lohan.load_library().lohan_adam_small_block_step(
        blk.p.data_ptr(), blk.m.data_ptr(), blk.v.data_ptr(), blk.g.data_ptr(),
        blk.p16.data_ptr(), max_n + 1, hy["lr"], hy["beta1"], hy["beta2"], hy["eps"],
        hy["weight_decay"], hy["step"], hy["loss_scale"], blk.sqnorm.data_ptr(),
        blk.flag.data_ptr(), 0, blk.ws.data_ptr(), blk.ws.numel(), None)
    assert too_large == 6 and "maximum" in lohan.lohan_status_string(6)
    with pytest.raises(lohan.LohanError):
        small_step(blk, hy, flags=lohan.LOHAN_FLAG_PRECHECKED)
    with pytest.raises(lohan.LohanError):
        small_step(blk, dict(hy, step=0))
    torch.cuda.synchronize()
    after = blk.host()
    for k in ("p", "m", "v", "p16"):
        assert np.array_equal(after[k].view(np.uint8), before[k].view(np.uint8))


def test_unprepared_workspace_fails_on_the_safe_side():
    n = 50_000
    wl = workload(n)
    blk = DeviceBlock(synth.make_block(wl, seed=2, device=DEV))
    before = blk.host()
    blk.ws.fill_(0x5A)                                     # never prepared
    blk.flag.fill_(0)
    small_step(blk, wl.hyper())
    torch.cuda.synchronize()
    assert blk.flag_value() == 1 and np.isnan(float(blk.sqnorm.cpu().item()))
    after = blk.host()
    for k in ("p", "m", "v", "p16"):
        assert np.array_equal(after[k].view(np.uint8), before[k].view(np.uint8))


def test_a_wait_that_is_given_up_is_reported_and_leaves_the_workspace_usable(oracle):
    """The wait bound forced to zero polls from the host: every workgroup but the last to arrive
    gives up at once, all wavefronts exit normally, the flag carries the incomplete bit, and the
    counters are back at zero so that the next call on the same workspace is a correct step."""
    n = 2_000_003
    wl = workload(n)
    hy = wl.hyper()
    blk = DeviceBlock(synth.make_block(wl, seed=4, device=DEV))
    fresh = {k: getattr(blk, k).clone() for k in ("p", "m", "v", "p16")}
    try:
        lohan.lohan_tuning_set_wait_limit(0)
        small_step(blk, hy)
        torch.cuda.synchronize()
    finally:
        lohan.lohan_tuning_set_wait_limit()
    flag = blk.flag_value() & 0xFFFFFFFF
    assert flag & lohan.LOHAN_OVERFLOW_INCOMPLETE, hex(flag)
    # the state is unspecified now: restore it, then the same workspace must work as before
    for k, t in fresh.items():
        getattr(blk, k).copy_(t)
    host = blk.host()
    assert small_steps(blk, hy, 2) == [0, 0]
    assert oracle_steps(oracle, host, hy, 2) == [0, 0]
    assert assert_state_parity(blk.host(), host, what="after a given-up wait") == ZERO_ULP
    # and the other users of the workspace find their counters at zero too
    blk.norm(wl.loss_scale)
    torch.cuda.synchronize()
    check_norm(oracle, blk, host, wl.loss_scale, "norm after")


def test_alternating_with_the_other_reductions_on_one_workspace(oracle):
    n = 5_000_011
    wl = workload(n)
    hy = wl.hyper()
    blk = DeviceBlock(synth.make_block(wl, seed=6, device=DEV))
    host = blk.host()
    for k in range(3):
        h = dict(hy, step=hy["step"] + k)
        blk.check()
        small_step(blk, h)
        blk.norm(wl.loss_scale)
    torch.cuda.synchronize()
    assert blk.flag_value() == 0
    assert oracle_steps(oracle, host, hy, 3) == [0] * 3
    assert assert_state_parity(blk.host(), host, what="alternating") == ZERO_ULP
    check_norm(oracle, blk, host, wl.loss_scale, "alternating")


def test_small_step_replayed_from_a_hip_graph(oracle):
    """One kernel, no memset, no allocation: capturable.  Three replays with eager work and
    synchronisations in between, each checked against the oracle."""
    n = synth.WORKLOADS["gpt_h768"].n
    wl = workload(n)
    hy = wl.hyper()
    blk = DeviceBlock(synth.make_block(wl, seed=8, device=DEV))
    host = blk.host()
    warm = DeviceBlock(synth.make_block(workload(4096), seed=1, device=DEV))
    small_step(warm, workload(4096).hyper())
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            small_step(blk, hy, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    assert np.array_equal(blk.host()["p"].view(np.uint32), host["p"].view(np.uint32))

    scratch = torch.zeros(1 << 20, device=DEV)
    for r in range(3):
        graph.replay()
        torch.cuda.synchronize()
        assert blk.flag_value() == 0
        assert oracle_steps(oracle, host, hy, 1) == [0]
        assert assert_state_parity(blk.host(), host, what=f"replay {r}") == ZERO_ULP
        check_norm(oracle, blk, host, wl.loss_scale, f"replay {r}")
        scratch.add_(1.0)
        small_step(warm, workload(4096).hyper())
        torch.cuda.synchronize()
    assert float(scratch[0].cpu()) == 3.0


def test_small_steps_on_a_side_stream_while_gemms_run(oracle):
    """The one-launch step needs its whole grid resident, so compute units held by another
    stream's kernels delay it; kernels that finish by themselves (GEMMs here) must do no more
    than that.  h=768 blocks, each step behind its GEMM's event, GEMMs kept running on the main
    stream: every step complete (no incomplete bit) and equal to the oracle."""
    nblocks, n = 6, synth.WORKLOADS["gpt_h768"].n
    wl = workload(n)
    hy = wl.hyper()
    blocks = [DeviceBlock(synth.make_block(wl, seed=200 + i, device=DEV)) for i in range(nblocks)]
    hosts = [b.host() for b in blocks]
    side = torch.cuda.Stream()
    a = torch.randn(4096, 4096, device=DEV, dtype=torch.bfloat16)
    b = torch.randn(4096, 8192, device=DEV, dtype=torch.bfloat16)
    main = torch.cuda.current_stream()
    for i in reversed(range(nblocks)):
        torch.matmul(a, b)
        ev = torch.cuda.Event()
        ev.record(main)
        side.wait_event(ev)
        small_step(blocks[i], hy, stream=side)
        for _ in range(4):                      # GEMMs that overlap the step
            torch.matmul(a, b)
    side.synchronize()
    torch.cuda.synchronize()
    for i in range(nblocks):
        assert blocks[i].flag_value() == 0, hex(blocks[i].flag_value() & 0xFFFFFFFF)
        assert oracle_steps(oracle, hosts[i], hy, 1) == [0]
        assert assert_state_parity(blocks[i].host(), hosts[i], what=f"block {i}") == ZERO_ULP


def test_two_streams_with_grids_that_fit_together(oracle):
    """Two one-launch steps may run at the same time when their grids fit the device together
    (here 98 workgroups each); grids that do not fit together must be ordered by the caller."""
    n = 300_001
    wl = workload(n)
    hy = wl.hyper()
    blocks = [DeviceBlock(synth.make_block(wl, seed=300 + i, device=DEV)) for i in range(8)]
    hosts = [b.host() for b in blocks]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for s in streams:
        s.wait_stream(torch.cuda.current_stream())
    for k in range(3):
        for i, blk in enumerate(blocks):
            small_step(blk, dict(hy, step=hy["step"] + k), stream=streams[i % 2])
    for s in streams:
        s.synchronize()
    for i, blk in enumerate(blocks):
        assert blk.flag_value() == 0
        assert oracle_steps(oracle, hosts[i], hy, 3, nthreads=8) == [0] * 3
        assert assert_state_parity(blk.host(), hosts[i], what=f"block {i}") == ZERO_ULP

"""GPU parity of the ring form of the out-of-place step (B blocks in B + 1 slots, the slot table in
device memory): after any number of passes every block's state, found through the table, must be
what the oracle computes for that block alone, a block whose gradients overflowed must still sit
in its old slot bit-identical, and the table must stay a permutation of the slots."""
import sys

import numpy as np
import pytest
import torch

import paper_2403_06504_amd as lohan
from paper_2403_06504_amd import synthetic_inputs as synth

from gpu_util import assert_state_parity

pytestmark = pytest.mark.gpu

DEV = "cuda"
ZERO = {"p": 0, "m": 0, "v": 0, "p16": 0}


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


class Ring:
    def __init__(self, n, num_blocks, seed0=0, half=False, keep_host=True):
        self.n, self.B = n, num_blocks
        self.wl = synth.Workload(name=f"n{n}", n=n, step=100, loss_scale=65536.0,
                                 zero_moments=False)
        self.hy = self.wl.hyper()
        self.slots, self.g = [], []
        for b in range(num_blocks + 1):
            t = synth.make_block(self.wl, seed=seed0 + b, device=DEV)
            if b == num_blocks:                                  # the spare starts as garbage
                for k in ("p", "m", "v"):
                    t[k].fill_(float("nan"))
            else:
                self.g.append(t["g"])
            self.slots.append({k: t[k] for k in ("p", "m", "v", "p16")})
        self.ring = torch.empty(lohan.lohan_ring_bytes(num_blocks, 1), dtype=torch.uint8,
                                device=DEV)
        lohan.lohan_ring_init(self.ring,
                              [(s["p"], s["m"], s["v"], s["p16"], n) for s in self.slots],
                              num_blocks)
        self.host = [self.host_of_slot(b, b) for b in range(num_blocks)] if keep_host else None
        self.half = half

    def host_of_slot(self, slot, block):
        out = {k: synth.to_numpy_bits(self.slots[slot][k]) for k in ("p", "m", "v", "p16")}
        out["g"] = synth.to_numpy_bits(self.g[block])
        return out

    def one_pass(self, step, flags=0, stream=None):
        hy = self.hy
        for b in reversed(range(self.B)):             # gradients arrive with decreasing index
            lohan.lohan_ring_adam_block_step(self.ring, self.B, 1, b, self.g[b], self.n, hy["lr"],
                                             hy["beta1"], hy["beta2"], hy["eps"],
                                             hy["weight_decay"], step, hy["loss_scale"], flags,
                                             stream=stream)

    def read(self):
        slot_of, spares, last = lohan.lohan_ring_read(self.ring, self.B, 1)
        assert sorted(slot_of + spares) == list(range(self.B + 1)), (slot_of, spares)
        return slot_of, spares[0], last

    def oracle_pass(self, oracle, step, l2=False):
        flags = []
        for b in range(self.B):
            h = self.host[b]
            h["g"] = synth.to_numpy_bits(self.g[b])
            flags.append(oracle.adam_block_step(h["p"], h["m"], h["v"], h["g"], h["p16"],
                                                nthreads=4, l2_mode=l2, half_out=self.half,
                                                **dict(self.hy, step=step)))
        return flags

    def check(self, slot_of, what):
        for b in range(self.B):
            got = self.host_of_slot(slot_of[b], b)
            worst = assert_state_parity(got, self.host[b], what=f"{what} block {b}")
            assert worst == ZERO, (what, b, worst)


@pytest.mark.parametrize("n", [300_001, 4_096, 7])
def test_three_passes_with_an_overflow_in_the_second(oracle, n):
    r = Ring(n, 5, seed0=10)
    assert r.read() == ([0, 1, 2, 3, 4], 5, [0] * 5)
    t = r.hy["step"]
    # pass 1: every block moves into the spare in turn (4 first), so everything shifts by one
    r.one_pass(t)
    slot_of, spare, last = r.read()
    assert r.oracle_pass(oracle, t) == [0] * 5
    assert slot_of == [1, 2, 3, 4, 5] and spare == 0 and last == [0] * 5
    r.check(slot_of, "pass 1")
    # pass 2: block 2 overflows and stays where it is
    pos = n // 2
    saved = r.g[2][pos].clone()
    r.g[2].view(torch.int16)[pos] = 0x7C00
    before = r.host_of_slot(slot_of[2], 2)
    r.one_pass(t + 1)
    slot_of2, spare2, last2 = r.read()
    assert r.oracle_pass(oracle, t + 1) == [0, 0, 1, 0, 0]
    assert last2 == [0, 0, 1, 0, 0]
    assert slot_of2[2] == slot_of[2]
    after = r.host_of_slot(slot_of2[2], 2)
    for k in ("p", "m", "v", "p16"):
        assert np.array_equal(after[k].view(np.uint8), before[k].view(np.uint8)), k
    r.check(slot_of2, "pass 2")
    # pass 3: the gradient is finite again; block 2 repeats step t + 1, the others take t + 2
    r.g[2][pos] = saved
    hy = r.hy
    for b in reversed(range(5)):
        step = t + 1 if b == 2 else t + 2
        lohan.lohan_ring_adam_block_step(r.ring, 5, 1, b, r.g[b], n, hy["lr"], hy["beta1"],
                                         hy["beta2"], hy["eps"], hy["weight_decay"], step,
                                         hy["loss_scale"], 0)
        h = r.host[b]
        h["g"] = synth.to_numpy_bits(r.g[b])
        assert oracle.adam_block_step(h["p"], h["m"], h["v"], h["g"], h["p16"], nthreads=4,
                                      **dict(hy, step=step)) == 0
    slot_of3, _, last3 = r.read()
    assert last3 == [0] * 5                        # the repeated step went through
    r.check(slot_of3, "pass 3")


def test_a_block_whose_every_gradient_is_non_finite_stays_put(oracle):
    """Every wavefront of the step records the overflow (the usual way a block overflows); the
    block keeps its slot bit for bit and the next clean pass goes through."""
    n = 3_000_001
    r = Ring(n, 3, seed0=30)
    t = r.hy["step"]
    clean = r.g[1].clone()
    r.g[1].view(torch.int16).fill_(0x7E00)
    before = r.host_of_slot(1, 1)
    r.one_pass(t)
    slot_of, _, last = r.read()
    assert r.oracle_pass(oracle, t) == [0, 1, 0] and last == [0, 1, 0]
    assert slot_of[1] == 1
    after = r.host_of_slot(1, 1)
    for k in ("p", "m", "v", "p16"):
        assert np.array_equal(after[k].view(np.uint8), before[k].view(np.uint8)), k
    r.check(slot_of, "pass with an all-NaN block")
    r.g[1].copy_(clean)
    hy = r.hy
    for b in reversed(range(3)):
        step = t if b == 1 else t + 1
        lohan.lohan_ring_adam_block_step(r.ring, 3, 1, b, r.g[b], n, hy["lr"], hy["beta1"],
                                         hy["beta2"], hy["eps"], hy["weight_decay"], step,
                                         hy["loss_scale"], 0)
        h = r.host[b]
        h["g"] = synth.to_numpy_bits(r.g[b])
        assert oracle.adam_block_step(h["p"], h["m"], h["v"], h["g"], h["p16"], nthreads=4,
                                      **dict(hy, step=step)) == 0
    slot_of2, _, last2 = r.read()
    assert last2 == [0, 0, 0]
    r.check(slot_of2, "clean pass after it")


@pytest.mark.parametrize("flags", [lohan.LOHAN_FLAG_L2_MODE, lohan.LOHAN_FLAG_P16_FP16,
                                   lohan.LOHAN_FLAG_L2_MODE | lohan.LOHAN_FLAG_P16_FP16])
def test_ring_mode_flags(oracle, flags):
    r = Ring(123_457, 3, seed0=20, half=bool(flags & lohan.LOHAN_FLAG_P16_FP16))
    t = r.hy["step"]
    for k in range(2):
        r.one_pass(t + k, flags=flags)
        assert r.oracle_pass(oracle, t + k, l2=bool(flags & lohan.LOHAN_FLAG_L2_MODE)) == [0] * 3
    slot_of, _, _ = r.read()
    r.check(slot_of, f"flags={flags}")


def test_a_captured_pass_replays_through_the_rotating_slots(oracle):
    """The slot table lives on the device, so a captured pass stays valid while the slots rotate
    underneath it: three replays, each checked against the oracle (the step index is baked into
    the captured launches, so every replay repeats step 100 on the evolving state)."""
    r = Ring(200_003, 4, seed0=30)
    warm = Ring(4_096, 2, seed0=1)
    warm.one_pass(100)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            r.one_pass(100, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    assert r.read() == ([0, 1, 2, 3], 4, [0] * 4)              # capture executes nothing
    scratch = torch.zeros(1 << 20, device=DEV)
    for k in range(3):
        graph.replay()
        torch.cuda.synchronize()
        assert r.oracle_pass(oracle, 100) == [0] * 4
        slot_of, _, _ = r.read()
        r.check(slot_of, f"replay {k}")
        scratch.add_(1.0)
        warm.one_pass(101 + k)
    assert float(scratch[0].cpu()) == 3.0


def test_13b_blocks_in_a_ring_sampled(oracle):
    """Three blocks of the benchmark's shape in four slots (17.6 GB of slots), two passes, block 1
    overflowing in the second; sampled ranges against the oracle."""
    wl = synth.WORKLOADS["gpt13b"]
    n = wl.n
    r = Ring(n, 3, seed0=40, keep_host=False)
    span = 1 << 20
    rng = np.random.default_rng(21)
    starts = [0, n - span] + [int(x) for x in rng.integers(span, n - 2 * span, size=2)]

    def sample(slot, block, s):
        out = {k: synth.to_numpy_bits(r.slots[slot][k][s:s + span]) for k in ("p", "m", "v", "p16")}
        out["g"] = synth.to_numpy_bits(r.g[block][s:s + span])
        return out

    hosts = [{s: sample(b, b, s) for s in starts} for b in range(3)]
    t = wl.step
    r.one_pass(t)
    r.g[1].view(torch.int16)[n - 1] = -1                        # NaN in the last element
    r.one_pass(t + 1)
    slot_of, spare, last = r.read()
    assert last == [0, 1, 0]
    for b in range(3):
        for s in starts:
            h = hosts[b][s]
            for step in ((t,) if b == 1 else (t, t + 1)):
                assert oracle.adam_block_step(h["p"], h["m"], h["v"], h["g"], h["p16"],
                                              nthreads=8, **dict(r.hy, step=step)) == 0
            worst = assert_state_parity(sample(slot_of[b], b, s), h, what=f"ring 13B block {b}")
            assert worst == ZERO, (b, s, worst)


# One transformer layer as the gradient handler of Sec. IV-C sees it: one tensor at a time.  The
# weight matrices of a GPT block with hidden size h (QKV 3h^2, attention output h^2, the two MLP
# matrices 4h^2 each) and its bias / LayerNorm vectors.
def layer_tensor_lengths(h):
    return [3 * h * h, 3 * h, h * h, h, 4 * h * h, 4 * h, 4 * h * h, h, h, h, h, h]


class TensorRing:
    """Two layers' tensors in a ring with one spare per distinct length, all arrays placed by
    lohan_tensor_placement in one slab."""

    def __init__(self, h, layers=2, seed0=0):
        self.lengths = layer_tensor_lengths(h) * layers
        self.B = len(self.lengths)
        self.spare_lengths = sorted(set(self.lengths), reverse=True)
        self.S = len(self.spare_lengths)
        all_lengths = self.lengths + self.spare_lengths
        offsets, slab_bytes, align = lohan.lohan_tensor_placement(all_lengths)
        self.slab = torch.empty(slab_bytes + align, dtype=torch.uint8, device=DEV)
        start = (-self.slab.data_ptr()) % align

        def view(i, field, dtype, width):
            off = start + offsets[i][field]
            return self.slab[off: off + all_lengths[i] * width].view(dtype)

        self.slots, self.g, self.host = [], [], []
        self.hy = synth.Workload("t", 1, 100, 65536.0, False).hyper()
        for i, n in enumerate(all_lengths):
            slot = {"p": view(i, "param_fp32", torch.float32, 4),
                    "m": view(i, "exp_avg", torch.float32, 4),
                    "v": view(i, "exp_avg_sq", torch.float32, 4),
                    "p16": view(i, "param_bf16", torch.bfloat16, 2)}
            if i < self.B:
                wl = synth.Workload(f"t{i}", n, 100, 65536.0, False)
                t = synth.make_block(wl, seed=seed0 + i, device=DEV)
                for k in slot:
                    slot[k].copy_(t[k])
                g = view(i, "grad_fp16", torch.float16, 2)
                g.copy_(t["g"])
                self.g.append(g)
                self.host.append({k: synth.to_numpy_bits(t[k]) for k in ("p", "m", "v", "g", "p16")})
            else:
                for k in ("p", "m", "v"):
                    slot[k].fill_(float("nan"))
            self.slots.append(slot)
        self.ring = torch.empty(lohan.lohan_ring_bytes(self.B, self.S), dtype=torch.uint8,
                                device=DEV)
        lohan.lohan_ring_init(
            self.ring, [(s["p"], s["m"], s["v"], s["p16"], n)
                        for s, n in zip(self.slots, all_lengths)], self.B)
        self.all_lengths = all_lengths

    def read(self):
        slot_of, spares, skipped = lohan.lohan_ring_read(self.ring, self.B, self.S)
        assert sorted(slot_of + spares) == list(range(self.B + self.S))
        for b, s in enumerate(slot_of):                     # a block only ever sits in a slot
            assert self.all_lengths[s] == self.lengths[b]   # of its own length
        return slot_of, spares, skipped

    def check(self, slot_of, what):
        for b in range(self.B):
            got = {k: synth.to_numpy_bits(self.slots[slot_of[b]][k]) for k in ("p", "m", "v", "p16")}
            worst = assert_state_parity(got, self.host[b], what=f"{what} tensor {b}")
            assert worst == ZERO, (what, b, self.lengths[b], worst)


def test_ring_of_unequal_tensors_with_one_spare_per_length(oracle):
    """The handler fires per gradient tensor, and a layer's tensors have four different lengths:
    B tensors in B slots plus one spare per distinct length.  Three passes (tensors taken last to
    first), one tensor overflowing in the second, per-tensor clipping in the third."""
    r = TensorRing(256, layers=2, seed0=70)
    hy = r.hy
    assert r.S == 6 and r.read()[0] == list(range(r.B))    # 3h^2, h^2, 4h^2, 3h, h, 4h
    t = hy["step"]
    sq = torch.zeros(r.B, dtype=torch.float64, device=DEV)
    fl = torch.zeros(r.B, dtype=torch.int32, device=DEV)
    ws = lohan.new_workspace(DEV)
    bad = 4                                              # a 4h^2 matrix of the first layer
    for k, step in enumerate((t, t + 1, t + 2)):
        if k == 1:
            r.g[bad].view(torch.int16)[17] = 0x7C00
        clip = k == 2
        max_norm = 0.01
        for b in reversed(range(r.B)):
            n = r.lengths[b]
            if clip:
                lohan.lohan_grad_sqnorm(r.g[b], n, hy["loss_scale"], sq[b:b + 1], fl[b:b + 1], ws)
                lohan.lohan_ring_adam_block_step_clipped(
                    r.ring, r.B, r.S, b, r.g[b], n, hy["lr"], hy["beta1"], hy["beta2"], hy["eps"],
                    hy["weight_decay"], step, hy["loss_scale"], sq[b:b + 1], max_norm, 0)
            else:
                lohan.lohan_ring_adam_block_step(r.ring, r.B, r.S, b, r.g[b], n, hy["lr"],
                                                 hy["beta1"], hy["beta2"], hy["eps"],
                                                 hy["weight_decay"], step, hy["loss_scale"], 0)
        slot_of, spares, skipped = r.read()
        norms = sq.cpu().numpy()
        for b in range(r.B):
            h = r.host[b]
            h["g"] = synth.to_numpy_bits(r.g[b])
            scale = hy["loss_scale"]
            if clip and not (b == bad):
                scale = lohan.lohan_clip_loss_scale(float(norms[b]), hy["loss_scale"], max_norm)
                sq_orc = oracle.grad_sqnorm(h["g"], hy["loss_scale"])
                assert abs(float(norms[b]) - sq_orc) <= 1e-5 * sq_orc
                s_orc = float(oracle.clip_loss_scale(sq_orc, hy["loss_scale"], max_norm))
                assert abs(int(np.float32(scale).view(np.uint32)) -
                           int(np.float32(s_orc).view(np.uint32))) <= 1
            f = oracle.adam_block_step(h["p"], h["m"], h["v"], h["g"], h["p16"], nthreads=4,
                                       **dict(hy, step=step, loss_scale=scale))
            assert skipped[b] == f == (1 if (b == bad and k >= 1) else 0), (k, b)
        r.check(slot_of, f"pass {k}")


def test_ring_step_with_the_wrong_length_touches_nothing(oracle):
    r = TensorRing(128, layers=1, seed0=90)
    hy = r.hy
    before = [{k: synth.to_numpy_bits(s[k]) for k in ("p", "m", "v", "p16")} for s in r.slots[:r.B]]
    b = 0                                                # registered with 3h^2 elements
    lohan.lohan_ring_adam_block_step(r.ring, r.B, r.S, b, r.g[b], r.lengths[b] - 256, hy["lr"],
                                     hy["beta1"], hy["beta2"], hy["eps"], hy["weight_decay"],
                                     hy["step"], hy["loss_scale"], 0)
    slot_of, spares, skipped = r.read()
    assert slot_of == list(range(r.B)) and skipped[b] == 1
    for i in range(r.B):
        for k in ("p", "m", "v", "p16"):
            got = synth.to_numpy_bits(r.slots[i][k])
            assert np.array_equal(got.view(np.uint8), before[i][k].view(np.uint8)), (i, k)

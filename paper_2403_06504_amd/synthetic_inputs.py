"""Seeded synthetic block inputs, shared by the tests (oracle and GPU side) and the benchmark.

Data only: none of the method's arithmetic lives here.  The paper evaluates on randomly
initialised parameters and random data (Sec. V-A "Workloads") with the GPT-style shapes of
Table IV; a transformer block of hidden size h carries 12*h^2 weights, which is the flat element
count used here.  N(0, x) below always means standard deviation x.

Workloads (hyper-parameters are AdamW lr 1e-4, betas (0.9, 0.999), eps 1e-8, wd 0.01):
  gpt_h768    n = 12*768^2          m = v = 0,                    step 1,    loss scale 1024
  gpt13b      n = 12*5120^2         m ~ N(0,1e-4), v ~ |N(0,1e-7)|, step 100,  loss scale 65536
  gpt175b     n = 12*12288^2        as gpt13b,                     step 1000, loss scale 65536
  gpt13b_ragged  n = 12*5120^2 + 1  as gpt13b (overflow / clipping cases)
p ~ N(0, 0.02) fp32; stored gradients are fp16(N(0,1e-3) * loss_scale).
"""
from dataclasses import dataclass, replace

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    n: int
    step: int
    loss_scale: float
    zero_moments: bool
    lr: float = 1e-4
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.01
    p_std: float = 0.02
    g_std: float = 1e-3
    m_std: float = 1e-4
    v_std: float = 1e-7

    def hyper(self, step=None, loss_scale=None) -> dict:
        return dict(lr=self.lr, beta1=self.beta1, beta2=self.beta2, eps=self.eps,
                    weight_decay=self.weight_decay, step=self.step if step is None else step,
                    loss_scale=self.loss_scale if loss_scale is None else loss_scale)

    def with_n(self, n: int) -> "Workload":
        return replace(self, n=int(n))


WORKLOADS = {
    "gpt_h768": Workload("gpt_h768", 12 * 768 ** 2, 1, 1024.0, True),
    "gpt13b": Workload("gpt13b", 12 * 5120 ** 2, 100, 65536.0, False),
    "gpt175b": Workload("gpt175b", 12 * 12288 ** 2, 1000, 65536.0, False),
    "gpt13b_ragged": Workload("gpt13b_ragged", 12 * 5120 ** 2 + 1, 100, 65536.0, False),
}

# Block shapes of the paper's evaluation models: (name, layers, hidden size).  A GPT-style
# decoder block carries 12*h^2 weights (Table IV); a DiT block carries 18*h^2 (attention 4h^2,
# MLP 8h^2, adaLN modulation 6h^2 -- this reproduces the model sizes of Table VI).
TABLE_IV_GPT = (("6B", 28, 4096), ("13B", 40, 5120), ("30B", 48, 7168), ("70B", 80, 8192),
                ("135B", 88, 11264), ("175B", 96, 12288), ("276B", 112, 14336),
                ("412B", 128, 16384))
TABLE_VI_DIT = (("0.67B", 28, 1152), ("0.90B", 30, 1280), ("1.4B", 32, 1536), ("10B", 28, 4096),
                ("20B", 40, 5120), ("40B", 48, 7168))


def shape_workloads():
    """One Workload per evaluation-model block shape, value distributions as gpt13b."""
    out = []
    for name, _, h in TABLE_IV_GPT:
        out.append(Workload(f"gpt{name}_h{h}", 12 * h * h, 100, 65536.0, False))
    for name, _, h in TABLE_VI_DIT:
        out.append(Workload(f"dit{name}_h{h}", 18 * h * h, 100, 65536.0, False))
    return out


# fp16 bit patterns with an all-ones exponent: +inf, -inf, quiet NaN, all-ones NaN, signalling NaN
NONFINITE_FP16 = (0x7C00, 0xFC00, 0x7E00, 0xFFFF, 0x7C01)

_CHUNK = 1 << 26


def _randn_into(out: torch.Tensor, std: float, gen: torch.Generator, absolute=False):
    """Fill a flat tensor with N(0, std) in bounded-size pieces (keeps temporaries small)."""
    n = out.numel()
    for lo in range(0, n, _CHUNK):
        hi = min(n, lo + _CHUNK)
        piece = torch.randn(hi - lo, generator=gen, device=out.device, dtype=torch.float32)
        piece.mul_(std)
        if absolute:
            piece.abs_()
        out[lo:hi].copy_(piece)      # converts when `out` is fp16
    return out


def make_block(workload: Workload, seed: int = 0, device="cpu") -> dict:
    """Tensors of one block on `device`: p, m, v (fp32), g (fp16, already multiplied by the loss
    scale), p16 (bf16, filled with a sentinel so that an unwritten output is visible)."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(int(seed))
    n = workload.n
    p = _randn_into(torch.empty(n, dtype=torch.float32, device=dev), workload.p_std, gen)
    g = _randn_into(torch.empty(n, dtype=torch.float16, device=dev),
                    workload.g_std * workload.loss_scale, gen)
    if workload.zero_moments:
        m = torch.zeros(n, dtype=torch.float32, device=dev)
        v = torch.zeros(n, dtype=torch.float32, device=dev)
    else:
        m = _randn_into(torch.empty(n, dtype=torch.float32, device=dev), workload.m_std, gen)
        v = _randn_into(torch.empty(n, dtype=torch.float32, device=dev), workload.v_std, gen,
                        absolute=True)
    p16 = torch.full((n,), -3.0, dtype=torch.bfloat16, device=dev)
    return {"p": p, "m": m, "v": v, "g": g, "p16": p16}


def plant_nonfinite(g: torch.Tensor, fraction: float, seed: int, always=()) -> torch.Tensor:
    """Overwrite a seeded set of positions of an fp16 gradient tensor with inf/NaN bit patterns
    (cycling through NONFINITE_FP16).  `always` lists indices that are hit regardless
    (e.g. 0 and n-1).  Returns the sorted positions (CPU int64)."""
    n = g.numel()
    count = int(round(n * fraction))
    gen = torch.Generator(device="cpu")
    gen.manual_seed(int(seed) + 7919)
    pos = torch.randint(0, n, (count,), generator=gen, dtype=torch.int64) if count else \
        torch.empty(0, dtype=torch.int64)
    if len(always):
        pos = torch.cat([pos, torch.tensor([i % n for i in always], dtype=torch.int64)])
    pos = torch.unique(pos)
    pats = torch.tensor(NONFINITE_FP16, dtype=torch.int32)
    vals = pats[torch.arange(pos.numel()) % len(NONFINITE_FP16)].to(torch.int16)  # wraps > 0x7FFF
    g.view(torch.int16)[pos.to(g.device)] = vals.to(g.device)
    return pos


def to_numpy_bits(t: torch.Tensor):
    """Host numpy copy; 16-bit float tensors come back as uint16 bit patterns."""
    c = t.detach().cpu().contiguous()
    if c.dtype in (torch.float16, torch.bfloat16):
        return c.view(torch.int16).numpy().view("uint16").copy()
    return c.numpy().copy()

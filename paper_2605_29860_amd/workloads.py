"""Seeded synthetic inputs shaped like the paper's rollout workload.

The paper trains R1-Distill-Qwen models (vocabulary 152064) with 8 rollouts x 64 prompts
= 512 trajectories per batch and a target stop rate of 0.25 (Section 5.1, Appendix A).
Neither the weights nor the data exist here, so logits, critic values, rewards and
lengths are drawn from seeded distributions of the same shapes.  This module only
*generates inputs*: it contains none of the method's arithmetic and is the one piece of
code that the tests hand to both the GPU path and the CPU oracle.

Every generator takes a torch device; whatever bits it produces on that device are the
ground truth for both sides (the oracle receives a host copy of the same bits).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np
import torch

QWEN_VOCAB = 152064


def _gen(device, *key) -> torch.Generator:
    """A torch generator on `device` keyed by a tuple of small integers."""
    h = 0x9E3779B97F4A7C15
    for k in key:
        h = (h ^ (int(k) + 0x632BE59BD9B4E019)) * 0xD6E8FEB86659FD93 % (1 << 63)
        h ^= h >> 29
    g = torch.Generator(device=device)
    g.manual_seed(h % (1 << 62))
    return g


def to_host_bits(logits: torch.Tensor) -> np.ndarray:
    """Host copy for the oracle: float32 stays float32, bf16 becomes its uint16 bit pattern."""
    t = logits.detach()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    if t.dtype == torch.float32:
        return t.cpu().numpy()
    raise TypeError(t.dtype)


# --------------------------------------------------------------------------- paper hyper-parameters
@dataclass
class RolloutParams:
    """Values of Appendix A (Table of hyper-parameters); c and delta are not given there."""
    mu_g: float = 1.0
    var_g: float = 2.0
    delta: float = 1e-8
    clip_c: float = 10.0
    alpha_s: float = 0.9
    beta: float = 7.0
    eps: float = 0.2
    stop_enabled: int = 1
    eos_id: int = -1

    def as_dict(self):
        return dict(self.__dict__)


# --------------------------------------------------------------------------- config 1 (small reference)
@dataclass
class SmallReference:
    """B=4, V=32768 fp32, T=128: N(0, 2^2) noise with one planted peak per row.

    Rows 0-1 keep a tall peak (the mode holds almost all the mass, so the regret stays
    near zero).  In rows 2-3 the peak shrinks linearly from `peak_hi` at step 0 to
    `peak_lo` (+8.0) at the last step, which moves mass onto the noise tokens and makes
    the regret grow until the stop rule fires.
    """
    B: int = 4
    V: int = 32768
    T: int = 128
    sigma: float = 2.0
    peak_hi: float = 20.0
    peak_lo: float = 8.0
    temperature: float = 1.0
    seed: int = 0
    params: RolloutParams = field(default_factory=lambda: RolloutParams(mu_g=0.5, var_g=1.0))
    r_fail: float = -1.0
    gamma: float = 1.0
    lam: float = 0.95

    def peak_index(self) -> np.ndarray:
        g = _gen("cpu", self.seed, 101)
        return torch.randint(0, self.V, (self.B,), generator=g).numpy()

    def logits(self, step: int, device="cpu") -> torch.Tensor:
        g = _gen("cpu", self.seed, 102, step)
        x = torch.randn(self.B, self.V, generator=g, dtype=torch.float32) * self.sigma
        idx = self.peak_index()
        frac = step / max(self.T - 1, 1)
        for b in range(self.B):
            h = self.peak_hi if b < 2 else self.peak_hi + (self.peak_lo - self.peak_hi) * frac
            x[b, idx[b]] = h
        return x.to(device)

    def values(self, device="cpu") -> torch.Tensor:
        """[B, T] critic values ~ U(-1, 1); column t gates step t and the same array feeds GAE."""
        g = _gen("cpu", self.seed, 103)
        return (torch.rand(self.B, self.T, generator=g, dtype=torch.float32) * 2 - 1).to(device)


# --------------------------------------------------------------------------- config 2-4 (Qwen-vocabulary rows)
class ZipfLogits:
    """bf16 logits = N(0, 3^2) noise + a Zipf(s)-shaped boost over a seeded permutation.

    boost(v) = -s * ln(rank(v)), rank a seeded permutation of 1..V: the logarithm of an
    unnormalised Zipf pmf, so a few tokens carry most of the mass as in a language-model
    head, and the bf16 grid produces many exact logit ties.
    """

    def __init__(self, V: int = QWEN_VOCAB, seed: int = 0, sigma: float = 3.0, s: float = 1.1,
                 device="cpu", dtype=torch.bfloat16):
        self.V, self.seed, self.sigma, self.s = V, seed, sigma, s
        self.device, self.dtype = device, dtype
        g = _gen("cpu", seed, 201)
        rank = torch.randperm(V, generator=g).to(torch.float32) + 1.0
        self.boost = (-s * torch.log(rank)).to(device)

    def rows(self, B: int, step: int = 0, out: torch.Tensor | None = None) -> torch.Tensor:
        g = _gen(self.device, self.seed, 202, step)
        x = torch.randn(B, self.V, generator=g, device=self.device, dtype=torch.float32)
        x.mul_(self.sigma).add_(self.boost)
        if out is None:
            return x.to(self.dtype)
        out.copy_(x)
        return out


@dataclass
class RegretPlant:
    """Rows whose regret is forced up from a seeded onset step on ("peak + plateau").

    From its onset step a planted row gets one peak token at height P and a plateau of
    every even vocabulary index at P - D.  P is far above the noise, so the row's mass
    sits on the plateau while the mode is the peak: the sampled token is a plateau token
    with probability K e^{-D/tau} / (1 + K e^{-D/tau}) and the regret is then D / tau.
    """
    rows: np.ndarray          # planted row ids
    onset: np.ndarray         # first planted step of each such row
    peak: np.ndarray          # peak token of each such row
    P: float = 40.0
    D: float = 4.25

    @staticmethod
    def make(B: int, V: int, fraction: float, onset_lo: int, onset_hi: int, seed: int) -> "RegretPlant":
        g = _gen("cpu", seed, 301)
        n = int(round(B * fraction))
        rows = torch.randperm(B, generator=g)[:n].sort().values.numpy()
        onset = torch.randint(onset_lo, onset_hi + 1, (n,), generator=g).numpy()
        peak = (torch.randint(0, V // 2, (n,), generator=g) * 2 + 1).numpy()  # odd index
        return RegretPlant(rows=rows, onset=onset, peak=peak)

    def apply(self, x: torch.Tensor, step: int) -> torch.Tensor:
        on = self.onset <= step
        if not on.any():
            return x
        r = torch.as_tensor(self.rows[on], device=x.device, dtype=torch.long)
        pk = torch.as_tensor(self.peak[on], device=x.device, dtype=torch.long)
        sub = x[r]
        sub[:, 0::2] = self.P - self.D
        sub[torch.arange(r.numel(), device=x.device), pk] = self.P
        x[r] = sub
        return x


def step_values(B: int, seed: int, step: int, lo: float, hi: float, device="cpu") -> torch.Tensor:
    """Critic values V_phi(s_t) of one step, ~ U(lo, hi)."""
    g = _gen(device, seed, 401, step)
    return torch.rand(B, generator=g, device=device, dtype=torch.float32) * (hi - lo) + lo


def initial_state(B: int, device="cpu"):
    """State before step 0 of Algorithm 1: z = 0, every row live, no stop step yet."""
    return (torch.zeros(B, dtype=torch.float32, device=device),
            torch.ones(B, dtype=torch.uint8, device=device),
            torch.full((B,), -1, dtype=torch.int32, device=device))


def seeded_state(B: int, seed: int, device="cpu", dead_every: int = 8):
    """Mid-rollout state for the single-step config: z ~ U(-1,1), every `dead_every`-th row dead."""
    g = _gen("cpu", seed, 501)
    z = torch.rand(B, generator=g, dtype=torch.float32) * 2 - 1
    alive = torch.ones(B, dtype=torch.uint8)
    if dead_every > 0:
        alive[dead_every - 1::dead_every] = 0
    stop_step = torch.full((B,), -1, dtype=torch.int32)
    return z.to(device), alive.to(device), stop_step.to(device)


# --------------------------------------------------------------------------- config 5 (advantages)
def advantage_batch(B: int = 1024, T: int = 16384, len_lo: int = 512, len_hi: int = 16384,
                    stop_fraction: float = 0.3, seed: int = 0, device="cpu", poison: bool = False):
    """values ~ U(-1,1); lengths ~ U{len_lo..len_hi}; `stop_fraction` of rows early-stopped;
    survivors carry a Bernoulli(0.5) reward in {0,1} on their last token, zero elsewhere.

    With `poison` everything at t >= length is NaN, which proves that it is never read.
    Returns (rewards [B,T] f32, values [B,T] f32, lengths [B] i32, stopped [B] u8).
    """
    g = _gen("cpu", seed, 601)
    lengths = torch.randint(len_lo, min(len_hi, T) + 1, (B,), generator=g, dtype=torch.int64)
    stopped = (torch.rand(B, generator=g) < stop_fraction)
    term = (torch.rand(B, generator=g) < 0.5).to(torch.float32)
    gd = _gen(device, seed, 602)
    values = torch.rand(B, T, generator=gd, device=device, dtype=torch.float32) * 2 - 1
    rewards = torch.zeros(B, T, device=device, dtype=torch.float32)
    idx = (lengths - 1).clamp(min=0).to(device)
    rows = torch.arange(B, device=device)
    rewards[rows, idx] = torch.where(stopped, torch.zeros(B), term).to(device)
    if poison:
        t = torch.arange(T, device=device)[None, :]
        pad = t >= lengths.to(device)[:, None]
        values[pad] = math.nan
        rewards[pad] = math.nan
    return (rewards, values, lengths.to(torch.int32).to(device),
            stopped.to(torch.uint8).to(device))


# --------------------------------------------------------------------------- batch-boundary statistics
def regret_batch(B: int = 512, T: int = 8192, len_lo: int = 64, stop_fraction: float = 0.25, seed: int = 0,
                 device="cpu", poison: bool = False):
    """Per-token regrets of a finished rollout batch, shaped like what espo_step emits on the
    Qwen-vocabulary rows: zero when the mode was sampled (a bit more than half of the tokens),
    otherwise exponential with mean 2.2; lengths ~ U{len_lo..T}; `stop_fraction` of the rows
    ended by the stop rule.  With `poison` everything at t >= length is NaN.
    Returns (regret [B,T] f32, lengths [B] i32, stopped [B] u8).
    """
    g = _gen("cpu", seed, 701)
    lengths = torch.randint(min(len_lo, T), T + 1, (B,), generator=g, dtype=torch.int64)
    stopped = torch.rand(B, generator=g) < stop_fraction
    gd = _gen(device, seed, 702)
    u = torch.rand(B, T, generator=gd, device=device, dtype=torch.float32)
    e = torch.rand(B, T, generator=gd, device=device, dtype=torch.float32)
    regret = torch.where(u < 0.55, torch.zeros_like(u), -2.2 * torch.log1p(-e))
    if poison:
        t = torch.arange(T, device=device)[None, :]
        regret[t >= lengths.to(device)[:, None]] = float("nan")
    return regret, lengths.to(torch.int32).to(device), stopped.to(torch.uint8).to(device)

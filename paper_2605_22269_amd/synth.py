"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws random tensors; it holds none of the method's
arithmetic and is the one module that both the HIP path's tests / benchmark and
the CPU oracle's tests may use.  The paper measures on LLaVA-OneVision style
streams (P = 196 visual tokens per frame, 10 minute to 1 hour videos sampled at
0.5-3 fps, Sec. 4.1 "Configurations"); the real videos and model weights are
not available, so these streams stand in for the K, V and last-layer Q tensors
a Video-LLM prefill would hand over:

* K, V, Q follow an AR(1) process across frames, independently per (layer,
  head, position, feature):  x_f = r*x_{f-1} + sqrt(1-r^2)*eps_f, eps ~ N(0,1),
  so consecutive frames are strongly correlated like video;
* optionally a Bernoulli(spike_prob) subset of (frame, position) tokens has its
  K and V rows scaled by spike_scale in every layer and head ("salient"
  tokens with a spiked norm);
* questions are N(0,1) query tokens, optionally with a planted direction so
  that known target frames should be retrieved.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str                 # "bf16" | "f32"
    n_frames: int
    tokens_per_frame: int
    frames_per_segment: int
    superpatches_per_frame: int = 4
    chunk_frames: int = 8
    ar_rho: float = 0.9
    spike_prob: float = 0.0
    spike_scale: float = 3.0
    keep_ratio: float = 0.25
    alpha: float = 0.7
    lambda_frame: float = 0.3
    k_seg: int = 2
    k_frame: int = 4
    question_tokens: int = 16
    n_questions: int = 1

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == "bf16" else torch.float32

    @property
    def elem_bytes(self):
        return 2 if self.dtype == "bf16" else 4

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


# The five configurations the build is measured and parity-tested on.
WORKLOADS = {
    "tiny": Workload("tiny", 1, 4, 1, 64, "f32", 32, 49, 8, keep_ratio=0.25,
                     k_seg=2, k_frame=4, question_tokens=16),
    "7b": Workload("7b", 28, 28, 4, 128, "bf16", 256, 196, 16, spike_prob=0.05,
                   keep_ratio=0.25, k_seg=4, k_frame=16, question_tokens=32),
    "hour": Workload("hour", 28, 28, 4, 128, "bf16", 3600, 196, 32, spike_prob=0.05,
                     keep_ratio=0.125, k_seg=8, k_frame=32, question_tokens=32),
    "retrieval": Workload("retrieval", 28, 28, 4, 128, "bf16", 3600, 196, 32, spike_prob=0.05,
                          keep_ratio=0.125, k_seg=8, k_frame=32, question_tokens=64, n_questions=64),
    "72b": Workload("72b", 80, 64, 8, 128, "bf16", 3600, 64, 32, ar_rho=0.95,
                    keep_ratio=0.125, k_seg=8, k_frame=32, question_tokens=32),
}


class SynthStream:
    """Frame-by-frame generator of (K, V, Q_last) chunks.

    Draw order per frame is fixed (K noise, V noise, Q noise, spike mask), so
    the stream does not depend on how it is cut into chunks.
    """

    def __init__(self, w: Workload, seed: int, device="cpu", with_q: bool = True):
        self.w = w
        self.device = torch.device(device)
        self.gen = torch.Generator(device=self.device)
        self.gen.manual_seed(seed)
        self.with_q = with_q
        self._k = self._v = self._q = None
        self.frame = 0

    def _randn(self, *shape):
        return torch.randn(*shape, generator=self.gen, device=self.device, dtype=torch.float32)

    def _step(self, prev, shape):
        eps = self._randn(*shape)
        if prev is None:
            return eps
        r = self.w.ar_rho
        return prev.mul_(r).add_(eps, alpha=math.sqrt(1.0 - r * r))

    def next_chunk(self, n_frames: int):
        """Returns k, v: [L][Hkv][n*P][D] and q_last: [Hq][n*P][D] (or None)."""
        w = self.w
        L, Hq, Hkv, D, P = w.n_layers, w.n_q_heads, w.n_kv_heads, w.head_dim, w.tokens_per_frame
        dt = w.torch_dtype
        k = torch.empty(L, Hkv, n_frames * P, D, dtype=dt, device=self.device)
        v = torch.empty_like(k)
        q = torch.empty(Hq, n_frames * P, D, dtype=dt, device=self.device) if self.with_q else None
        for f in range(n_frames):
            self._k = self._step(self._k, (L, Hkv, P, D))
            self._v = self._step(self._v, (L, Hkv, P, D))
            if self.with_q:
                self._q = self._step(self._q, (Hq, P, D))
            sl = slice(f * P, (f + 1) * P)
            if w.spike_prob > 0.0:
                u = torch.rand(P, generator=self.gen, device=self.device)
                scale = torch.where(u < w.spike_prob, w.spike_scale, 1.0).view(1, 1, P, 1)
                k[:, :, sl] = (self._k * scale).to(dt)
                v[:, :, sl] = (self._v * scale).to(dt)
            else:
                k[:, :, sl] = self._k.to(dt)
                v[:, :, sl] = self._v.to(dt)
            if self.with_q:
                q[:, sl] = self._q.to(dt)
            self.frame += 1
        return k, v, q


def random_question(w: Workload, n_tokens: int, seed: int, device="cpu"):
    """[n_tokens][Hq][D] query states drawn N(0,1)."""
    g = torch.Generator(device=torch.device(device))
    g.manual_seed(seed)
    x = torch.randn(n_tokens, w.n_q_heads, w.head_dim, generator=g, device=device, dtype=torch.float32)
    return x.to(w.torch_dtype)


def planted_question(w: Workload, target_keys: torch.Tensor, n_tokens: int, seed: int,
                     cosine: float = 0.5, device="cpu"):
    """Question whose mean query has cosine ~`cosine` with the direction of the
    given target block keys.

    target_keys: [n_targets][Hkv*D] block keys of the frames to plant (float).
    The direction u is the normalised mean of the keys after repeating each KV
    head for its group of query heads; q_bar = (cosine*u + sqrt(1-cosine^2)*n)
    * sqrt(Hq*D) with n a unit vector orthogonal to u; tokens are q_bar plus
    N(0,1) noise that sums to zero over the tokens.
    """
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(seed)
    Hq, Hkv, D = w.n_q_heads, w.n_kv_heads, w.head_dim
    G = Hq // Hkv
    t = target_keys.to(device=dev, dtype=torch.float32).view(-1, Hkv, 1, D).expand(-1, Hkv, G, D)
    u = t.reshape(-1, Hq * D).mean(dim=0)
    u = u / u.norm()
    n = torch.randn(Hq * D, generator=g, device=dev)
    n = n - (n @ u) * u
    n = n / n.norm()
    q_bar = (cosine * u + math.sqrt(1.0 - cosine * cosine) * n) * math.sqrt(Hq * D)
    eps = torch.randn(n_tokens, Hq * D, generator=g, device=dev)
    eps = eps - eps.mean(dim=0, keepdim=True)
    return (q_bar.unsqueeze(0) + eps).view(n_tokens, Hq, D).to(w.torch_dtype)


def handed_over_attention(n_units: int, tokens_per_unit: int, seed: int, tie_fraction: float = 0.3):
    """Stand-in for the attention-received signal (Eq. 1) that a prefill hands over for units it
    has just processed: float32 [n_units][tokens_per_unit], positive, heavy-tailed, a sink at the
    first token of every unit, and a fraction of the values snapped to a coarse grid so that exact
    ties occur.  No arithmetic of the method is in here: just numbers with that shape."""
    g = torch.Generator().manual_seed(seed)
    a = torch.rand(n_units, tokens_per_unit, generator=g, dtype=torch.float64)
    a = (a * a * a) / tokens_per_unit
    a[:, 0] += 20.0 / tokens_per_unit
    snap = torch.rand(n_units, tokens_per_unit, generator=g) < tie_fraction
    grid = 2.0 ** -14
    a = torch.where(snap, torch.round(a / grid) * grid, a)
    return a.to(torch.float32)


def question_lengths(n_questions: int, lo: int, hi: int, seed: int):
    """Uniform integer lengths in [lo, hi] for a batch of questions."""
    g = torch.Generator()
    g.manual_seed(seed)
    return torch.randint(lo, hi + 1, (n_questions,), generator=g).tolist()


def as_numpy(t: torch.Tensor):
    """Host numpy view of a tensor; bfloat16 is returned as uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view("uint16")
    return t.numpy()

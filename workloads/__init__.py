"""Seeded synthetic KV-cache tensors shaped like the paper's models.

This module serves both the CPU oracle's tests and the GPU library's tests / bench.  It
holds no HQMQ arithmetic: only random tensors with the shapes and value structure of the
workloads (Gaussian activations with per-channel scales, a few hot channels, heavy-tailed
spikes), cast to fp16.  Real caches, datasets and checkpoints are not available; these
tensors stand in for them.

A tensor is identified by (config, layer, role); its seed is a hash of those, so any
tensor can be regenerated alone, on the CPU or on the GPU (the two devices draw different
random streams; a parity test generates once and feeds the same bytes to both sides).
"""
from __future__ import annotations

from dataclasses import dataclass

import torch

FP16_MAX = 65504.0


@dataclass(frozen=True)
class Workload:
    name: str
    config_id: int
    layers: int
    B: int
    H: int
    T: int
    D: int
    S: int
    b_r: int = 6
    C: float = 3.0
    law: str = "lognormal"      # value structure of K ("lognormal" | "hot_channels" | "heavy")
    sigma_g: float = 0.5        # LogNormal(0, sigma_g) per-channel scale
    hot: int = 0                # number of hot channels per head (K only)
    hot_scale: float = 1.0
    spike_prob: float = 0.0     # per-element probability of an added Cauchy spike (K only)
    spike_scale: float = 0.0

    @property
    def elems_per_tensor(self) -> int:
        return self.B * self.H * self.T * self.D

    @property
    def n_tensors(self) -> int:
        return 2 * self.layers

    def with_T(self, T: int, layers: int | None = None) -> "Workload":
        """Same value law at a reduced sequence length / layer count (for parity tests)."""
        d = dict(self.__dict__)
        d["T"] = T
        if layers is not None:
            d["layers"] = layers
        return Workload(**d)


WORKLOADS = {
    "tiny": Workload("tiny", 1, 1, 1, 8, 1024, 128, 16),
    "llama3_8b_32k": Workload("llama3_8b_32k", 2, 32, 1, 8, 32768, 128, 256),
    "mistral7b_outlier": Workload("mistral7b_outlier", 3, 32, 4, 8, 8192, 128, 64,
                                  law="hot_channels", hot=4, hot_scale=20.0),
    "qwen25_7b_heavy": Workload("qwen25_7b_heavy", 4, 28, 1, 4, 32768, 128, 256, law="heavy",
                                hot=3, hot_scale=100.0, spike_prob=1e-3, spike_scale=10.0),
    "llama3_70b_128k": Workload("llama3_70b_128k", 5, 80, 1, 8, 131072, 128, 256, sigma_g=0.75),
    # the two other head dimensions of the paper's models, at the paper's own codebook sizes
    # (S = 192, b_r = 4): 96 (a full multi-head model with 32 kv heads) and 64 (8 kv heads)
    "mha32_d96_8k": Workload("mha32_d96_8k", 6, 32, 1, 32, 8192, 96, 192, b_r=4),
    "gqa8_d64_32k": Workload("gqa8_d64_32k", 7, 24, 1, 8, 32768, 64, 192, b_r=4, law="hot_channels",
                             hot=2, hot_scale=20.0),
}


def _mix64(z: int) -> int:
    m = (1 << 64) - 1
    z &= m
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & m
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & m
    return z ^ (z >> 31)


def tensor_seed(base_seed: int, config_id: int, layer: int, role: int) -> int:
    """63-bit seed of one (config, layer, role) tensor."""
    z = _mix64(base_seed)
    for v in (config_id, layer, role):
        z = _mix64(z ^ ((v + 1) * 0x9E3779B97F4A7C15))
    return z >> 1


def channel_scales(wl: Workload, layer: int, role: int, base_seed: int = 0) -> torch.Tensor:
    """Per-(head, channel) factor g[H, D], fixed over batch and tokens.  Drawn on the CPU so
    it is the same whatever device the activations are drawn on."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(tensor_seed(base_seed, wl.config_id, layer, role) ^ 0x5EED)
    if wl.law == "lognormal":
        return torch.exp(wl.sigma_g * torch.randn(wl.H, wl.D, generator=gen))
    g = torch.ones(wl.H, wl.D)
    if role == 0 and wl.hot > 0:  # hot channels on K only
        for h in range(wl.H):
            idx = torch.randperm(wl.D, generator=gen)[: wl.hot]
            g[h, idx] = wl.hot_scale
    return g


def make_tensor(wl: Workload, layer: int, role: int, device="cpu", base_seed: int = 0) -> torch.Tensor:
    """fp16 tensor [B, H, T, D] of one (layer, role); role 0 = K, 1 = V."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(tensor_seed(base_seed, wl.config_id, layer, role))
    g = channel_scales(wl, layer, role, base_seed).to(dev)
    x = torch.randn(wl.B, wl.H, wl.T, wl.D, generator=gen, device=dev, dtype=torch.float32)
    x *= g.view(1, wl.H, 1, wl.D)
    if role == 0 and wl.spike_prob > 0.0:
        hit = torch.rand(x.shape, generator=gen, device=dev) < wl.spike_prob
        spikes = torch.empty_like(x).cauchy_(0.0, 1.0, generator=gen) * wl.spike_scale
        x += torch.where(hit, spikes, torch.zeros_like(spikes))
    return x.clamp_(-FP16_MAX, FP16_MAX).to(torch.float16)


def sample_rows(wl: Workload, n_head: int = 256, n_tail: int = 256, n_rand: int = 4096,
                seed: int = 0) -> torch.Tensor:
    """Boolean mask over the B*H*T rows: the first and last token rows and a seeded random
    set of token positions, for every (batch, head).  Used where the exhaustive CPU search
    cannot cover a full-size tensor."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(seed ^ 0xA11CE)
    tok = torch.zeros(wl.T, dtype=torch.bool)
    tok[: min(n_head, wl.T)] = True
    tok[max(0, wl.T - n_tail):] = True
    if n_rand > 0:
        tok[torch.randint(0, wl.T, (n_rand,), generator=gen)] = True
    return tok.view(1, 1, wl.T).expand(wl.B, wl.H, wl.T).reshape(-1).clone()

"""Seeded synthetic Q/K/V for the workloads, and the workload table itself.

Holds none of the method's arithmetic: only shapes and a random smooth-field
generator.  Both the HIP path and the CPU oracle are fed the SAME bf16 bytes
produced here (the oracle receives them copied to host memory).

Real DiT activations (Wan2.2, HunyuanVideo1.5, Qwen-image-edit; Sec. 4 "setup")
are not available, so each tensor is a spatially/temporally correlated random
field of the same shape: per (head, channel) a sum of 8 random sinusoids of
(t, h, w) with at most 2 cycles per axis, scaled to unit variance over tokens,
plus i.i.d. Gaussian noise of standard deviation `sigma`, rescaled to unit
variance and rounded to bf16.  Neighbouring tokens are therefore similar, the
property Sec. 3.2 relies on.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import torch

SEED_BASE = 0x5F2D0000
N_WAVES = 8
MAX_CYCLES = 2.0


@dataclass(frozen=True)
class Workload:
    name: str
    index: int                 # 1-based position in the workload list (seeds depend on it)
    batch: int
    heads: int
    head_dim: int
    T: int
    H: int
    W: int
    block: int
    sparsity: float
    sink_frames: int
    sigma: float
    sweep: tuple = field(default=())   # extra sparsity points
    text_tokens: int = 0               # tokens of the other modality appended after the video tokens

    @property
    def N(self) -> int:
        return self.T * self.H * self.W + self.text_tokens

    @property
    def n_blocks(self) -> int:
        return -(-self.N // self.block)


WORKLOADS = {
    "tiny": Workload("tiny", 1, 1, 2, 64, 6, 16, 16, 64, 0.5, 1, 0.3),
    "image": Workload("image", 2, 1, 24, 128, 1, 64, 64, 128, 0.5, 0, 0.3),
    "video480p": Workload("video480p", 3, 1, 40, 128, 21, 30, 52, 128, 0.8, 1, 0.3),
    "video720p": Workload("video720p", 4, 1, 40, 128, 21, 45, 80, 128, 0.8, 1, 0.3),
    "longvideo": Workload("longvideo", 5, 1, 24, 128, 33, 45, 80, 128, 0.8, 1, 0.5,
                          sweep=(0.5, 0.7, 0.8, 0.9)),
}


def _field(gen_cpu: torch.Generator, T: int, H: int, W: int, d: int, sigma: float,
           device: torch.device, noise_seed: int, chunk: int = 16384) -> torch.Tensor:
    """One (batch, head) slice [N, d] float32 on `device`."""
    amp = torch.randn(d, N_WAVES, generator=gen_cpu)
    freq = (torch.rand(3, d, N_WAVES, generator=gen_cpu) * 2.0 - 1.0) * MAX_CYCLES
    if T == 1:
        freq[0].zero_()
    phase = torch.rand(d, N_WAVES, generator=gen_cpu) * (2.0 * math.pi)
    amp, freq, phase = amp.to(device), freq.to(device), phase.to(device)
    N = T * H * W
    out = torch.empty(N, d, dtype=torch.float32, device=device)
    idx = torch.arange(N, device=device)
    t = (idx // (H * W)).float() / T
    h = ((idx // W) % H).float() / H
    w = (idx % W).float() / W
    for s in range(0, N, chunk):
        e = min(N, s + chunk)
        arg = (t[s:e, None, None] * freq[0] + h[s:e, None, None] * freq[1]
               + w[s:e, None, None] * freq[2]) * (2.0 * math.pi) + phase
        out[s:e] = (torch.cos(arg) * amp).sum(-1)
    out = out / out.std(dim=0, keepdim=True).clamp_min(1e-6)
    gen_dev = torch.Generator(device=device)
    gen_dev.manual_seed(noise_seed)
    out = out + sigma * torch.randn(N, d, generator=gen_dev, device=device)
    out = out / out.std(dim=0, keepdim=True).clamp_min(1e-6)
    return out


def make_tensor(wl: Workload, tensor_index: int, device="cpu", heads=None) -> torch.Tensor:
    """Tensor `tensor_index` (0=Q, 1=K, 2=V) of workload `wl`: [B, heads, N, d] bf16,
    video tokens in [T, H, W] raster order, then the text tokens if any.  `heads` limits generation to a list of
    head numbers (each head's values do not depend on which others are made)."""
    device = torch.device(device)
    head_list = list(range(wl.heads)) if heads is None else list(heads)
    out = torch.empty(wl.batch, len(head_list), wl.N, wl.head_dim, dtype=torch.bfloat16, device=device)
    for b in range(wl.batch):
        for k, hd in enumerate(head_list):
            seed = SEED_BASE + wl.index * 16 + tensor_index
            gen = torch.Generator(device="cpu")
            gen.manual_seed(seed * 100003 + (b * wl.heads + hd))
            x = _field(gen, wl.T, wl.H, wl.W, wl.head_dim, wl.sigma, device,
                       noise_seed=seed * 7919 + (b * wl.heads + hd))
            if wl.text_tokens:
                # text tokens have no spatial structure: i.i.d. unit-variance rows (drawn after the field)
                x = torch.cat([x, torch.randn(wl.text_tokens, wl.head_dim, generator=gen).to(device)])
            out[b, k] = x.to(torch.bfloat16)
    return out


def make_qkv(wl: Workload, device="cpu", heads=None):
    return tuple(make_tensor(wl, i, device=device, heads=heads) for i in range(3))


def bf16_bits(x: torch.Tensor):
    """Host numpy uint16 view of a bf16 tensor's bytes (what the oracle reads)."""
    return x.detach().contiguous().cpu().view(torch.int16).numpy().view("uint16")

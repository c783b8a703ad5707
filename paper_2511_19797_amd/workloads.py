"""Seeded synthetic inputs with the attention shapes of the paper's DiT workloads.

This module holds no arithmetic of the method: it only draws numbers.  Both the
tests' oracle side and the GPU side are fed from here so they see identical
bits (values are rounded to the storage dtype on the host, once, before either
side touches them).

The paper trains DiT-XL/2 on ImageNet 256x256 / 512x512 latents with patch
size 2 (Sec. 6, App. F), i.e. self-attention over 16x16 = 256 or 32x32 = 1024
tokens, hidden 1152 split in 16 heads of 72 (the original DiT split).  Those
datasets and weights are not used; iid Gaussian tensors of the same shapes
stand in for the activations.

Recipe for every config: one numpy PCG64 stream seeded with `seed`; float32
standard normals drawn in the order q, k, v, tq, tk, tv, gO, gTO, each as a
whole [B,H,N,d] array; then the per-config scaling (tangent std, key scale);
then round-to-nearest-even to the storage dtype.
"""
from dataclasses import dataclass

import numpy as np
import torch

NAMES = ("q", "k", "v", "tq", "tk", "tv", "gO", "gTO")


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    N: int
    d: int
    dtype: str            # "f32" or "bf16"
    tangent_std: float = 1.0
    key_scale: float = 1.0
    note: str = ""
    M: int = 0            # queries, where they differ in number from the N keys (0: self-attention, M = N)

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def heads(self):
        return self.B * self.H

    @property
    def Mq(self):
        return self.M or self.N

    def fwd_flops(self):
        """Six N x N x d products (S, two for Sdot, and three PV-type)."""
        return 12.0 * self.B * self.H * self.Mq * self.N * self.d

    def bwd_flops(self):
        """Fifteen N x N x d products (six score-type incl. the recompute, nine output)."""
        return 30.0 * self.B * self.H * self.Mq * self.N * self.d

    def elem_bytes(self):
        return 4 if self.dtype == "f32" else 2

    def fwd_bytes(self):
        """Reads q,k,v,tq,tk,tv; writes o,to and two fp32 row vectors."""
        nq, nk = self.B * self.H * self.Mq, self.B * self.H * self.N
        return (4 * nq + 4 * nk) * self.d * self.elem_bytes() + 8 * nq

    def bwd_bytes(self):
        """Reads ten [B,H,N,d] tensors and two row vectors; writes six tensors."""
        nq, nk = self.B * self.H * self.Mq, self.B * self.H * self.N
        return (8 * nq + 8 * nk) * self.d * self.elem_bytes() + 8 * nq


CONFIGS = {
    "C1": Workload("C1", 1, 2, 64, 32, "f32", note="tiny plumbing case"),
    "C2": Workload("C2", 32, 12, 256, 64, "bf16", note="DiT-B/2, 256px latents"),
    "C3": Workload("C3", 32, 16, 256, 72, "bf16", note="DiT-XL/2, 256px latents"),
    "C4": Workload("C4", 16, 16, 1024, 72, "bf16", tangent_std=0.1, note="DiT-XL/2, 512px latents"),
    "C5": Workload("C5", 2, 24, 4096, 128, "bf16", key_scale=2.0, note="long-sequence stress"),
    # the head split the paper itself trains DiT-XL/2 with (hidden 1152 as 18 heads of 64, App. F:
    # its kernel ran 1.25x slower with 16 heads of 72)
    "X3": Workload("X3", 32, 18, 256, 64, "bf16", note="DiT-XL/2 as 18 x 64, 256px latents"),
    "X4": Workload("X4", 16, 18, 1024, 64, "bf16", tangent_std=0.1, note="DiT-XL/2 as 18 x 64, 512px latents"),
    # queries and keys differing in number (the paper's Background allows it; its models do not use it):
    # 1024 image tokens attending to 256 conditioning tokens, DiT-XL/2 head shape
    "XA": Workload("XA", 16, 16, 256, 72, "bf16", tangent_std=0.1, note="cross-attention, 1024 queries x 256 keys", M=1024),
}

# The shapes of the paper's own kernel benchmark (App. C "Evaluation": backward latency over heads H
# and sequence length S).  The table states neither batch size nor head dim: batch 1 and head dim 64
# are this repository's choice, so its rows give context, not a comparison.
SWEEP_H = (1, 24)
SWEEP_S = (128, 1024, 4096, 8192, 16384, 32768)


def sweep_configs():
    return [Workload(f"H{h}S{s}", 1, h, s, 64, "bf16", note="kernel-benchmark shape, batch 1, head dim 64")
            for h in SWEEP_H for s in SWEEP_S]


def custom(B, H, N, d, dtype="bf16", tangent_std=1.0, key_scale=1.0, name=None):
    return Workload(name or f"B{B}H{H}N{N}d{d}{dtype}", B, H, N, d, dtype, tangent_std, key_scale)


def make_inputs(w: Workload, seed: int):
    """dict name -> CPU torch tensor [B,H,N,d] ([B,H,M,d] for the query side) in the workload's storage dtype."""
    rng = np.random.Generator(np.random.PCG64(seed))
    out = {}
    for name in NAMES:
        rows = w.Mq if name in ("q", "tq", "gO", "gTO") else w.N  # query-side tensors have M rows
        x = rng.standard_normal((w.B, w.H, rows, w.d), dtype=np.float32)
        if name in ("tq", "tk", "tv") and w.tangent_std != 1.0:
            x *= np.float32(w.tangent_std)
        if name == "k" and w.key_scale != 1.0:
            x *= np.float32(w.key_scale)
        out[name] = torch.from_numpy(x).to(w.torch_dtype).contiguous()
    return out


def make_gains(w: Workload, seed: int):
    """(gain_q, gain_k): float32 [d] gains of the QK-norm, around one as after some training."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return tuple(torch.from_numpy((1.0 + 0.2 * rng.standard_normal(w.d)).astype(np.float32)) for _ in range(2))


def make_adaln_inputs(B: int, T: int, C: int, dtype: str, seed: int):
    """Inputs of the normalised AdaLN modulation: token features x with tangent tx and upstream gradients gy, gty
    ([B,T,C], storage dtype), scale a and shift b per batch element with tangents ta, tb ([B,C] float32)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    out = {}
    for name in ("x", "tx", "gy", "gty"):
        out[name] = torch.from_numpy(rng.standard_normal((B, T, C), dtype=np.float32)).to(td).contiguous()
    for name in ("a", "ta", "b", "tb"):
        out[name] = torch.from_numpy(rng.standard_normal((B, C), dtype=np.float32)).contiguous()
    return out


def make_gate_inputs(B: int, T: int, C: int, dtype: str, seed: int):
    """Inputs of the normalised residual gate: the stream x and the branch output h with tangents tx, th and upstream
    gradients gz, gtz ([B,T,C], storage dtype), the gate c per batch element with tangent tc ([B,C] float32)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    out = {}
    for name in ("x", "tx", "h", "th", "gz", "gtz"):
        out[name] = torch.from_numpy(rng.standard_normal((B, T, C), dtype=np.float32)).to(td).contiguous()
    for name in ("c", "tc"):
        out[name] = torch.from_numpy(rng.standard_normal((B, C), dtype=np.float32)).contiguous()
    return out


def make_gelu_inputs(shape, dtype: str, seed: int):
    """Inputs of the MLP's activation: pre-activations u (standard normal, what a normalised, modulated token times a
    freshly initialised weight gives), their tangent tu and the upstream gradients ga, gta, all of `shape`."""
    rng = np.random.Generator(np.random.PCG64(seed))
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    return {name: torch.from_numpy(rng.standard_normal(shape, dtype=np.float32)).to(td).contiguous()
            for name in ("u", "tu", "ga", "gta")}


def make_linear_inputs(R: int, K: int, F: int, dtype: str, seed: int):
    """Inputs of a linear layer with tangent: tokens x [R,K] with tangent tx, upstream gradients gy, gty [R,F] (standard
    normal), a weight w [F,K] of standard deviation 1/sqrt(K) (a freshly initialised layer: outputs of unit size) and
    a bias b [F] of standard deviation 0.1, all in the storage dtype."""
    rng = np.random.Generator(np.random.PCG64(seed))
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    out = {}
    for name, shape, scale in (("x", (R, K), 1.0), ("tx", (R, K), 1.0), ("w", (F, K), K ** -0.5), ("b", (F,), 0.1),
                               ("gy", (R, F), 1.0), ("gty", (R, F), 1.0)):
        out[name] = torch.from_numpy(rng.standard_normal(shape, dtype=np.float32) * np.float32(scale)).to(td).contiguous()
    return out


def make_block_inputs(B: int, T: int, H: int, d: int, hidden: int, seed: int):
    """Inputs of one normalised DiT block with tangent: the stream x [B,T,C] (C = H d) with tangent tx and upstream
    gradients gz, gtz (standard normal, bf16); the six modulation vectors a1 ... c2 [B,C] and their tangents (standard
    normal, float32); weights of standard deviation 1/sqrt(fan-in) and biases of 0.1 (bf16); QK-norm gains 1 + 0.2 x
    standard normal (float32).  Returns (x, tx, mods, tmods, params, gz, gtz)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    C = H * d
    bf = lambda *s, scale=1.0: torch.from_numpy(rng.standard_normal(s, dtype=np.float32) * np.float32(scale)).to(torch.bfloat16)
    f32 = lambda *s, scale=1.0, shift=0.0: torch.from_numpy((shift + scale * rng.standard_normal(s)).astype(np.float32))
    x, tx = bf(B, T, C), bf(B, T, C)
    mods = {k: f32(B, C) for k in ("a1", "b1", "c1", "a2", "b2", "c2")}
    tmods = {k: f32(B, C) for k in ("a1", "b1", "c1", "a2", "b2", "c2")}
    params = {"wqkv": bf(3 * C, C, scale=C ** -0.5), "bqkv": bf(3 * C, scale=0.1), "gq": f32(d, scale=0.2, shift=1.0),
              "gk": f32(d, scale=0.2, shift=1.0), "wo": bf(C, C, scale=C ** -0.5), "bo": bf(C, scale=0.1),
              "w1": bf(hidden, C, scale=C ** -0.5), "b1": bf(hidden, scale=0.1), "w2": bf(C, hidden, scale=hidden ** -0.5),
              "b2": bf(C, scale=0.1)}
    return x, tx, mods, tmods, params, bf(B, T, C), bf(B, T, C)


def to_f64(t: torch.Tensor) -> np.ndarray:
    """Exact widening of a stored tensor to float64 (what the oracle consumes)."""
    return t.detach().cpu().to(torch.float64).numpy()

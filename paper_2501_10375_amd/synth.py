"""Seeded synthetic inputs for the MoE layer (shared by tests, bench and smoke).

This module holds none of the method's arithmetic.  It only manufactures
tensors with the shapes of the models in Table III of the DAOP paper (Mixtral
8x7B: hidden 4096, 8 experts of FFN width 14336, top-2; Phi-3.5-MoE: hidden
4096, 16 experts of width 6400, top-2) and the value distributions the
benchmark configurations ask for: hidden states ~ N(0,1), weights
~ N(0, 1/fan_in), and a per-expert gate bias that skews routing like a Zipf
profile.  They stand in for the real checkpoints and the ShareGPT prompts the
paper measures on (Sec. V-A), none of which are available offline.

The generator is counter based and integer exact, so the same (seed, tensor
id, element index) gives the same bits on the CPU and on the GPU, and any slice
can be regenerated without the whole tensor:

  key      = mix64(seed * 2^32 + tensor_id)
  u_j(i)   = mix64(key + (3 i + j + 1) * GOLDEN),  j = 0, 1, 2     (splitmix64 stream)
  S(i)     = sum of the twelve 16-bit fields of u_0, u_1, u_2      (Irwin-Hall(12))
  value(i) = fp32(2 S - 786420) * fp32(scale / 131072)  -> rounded once to the storage type

(2 S - 786420) / 131072 has mean 0 and variance 1 - 2^-32, support about +-6.
All steps are 64-bit integer operations except one exact int->fp32 conversion
and one fp32 multiply.
"""
from __future__ import annotations

import math

import torch

_GOLDEN = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB
_MASK64 = (1 << 64) - 1

# Tensor ids (distinguish tensors generated under one seed).
TID_X, TID_WG, TID_WG_NEXT, TID_W1, TID_W3, TID_W2 = 1, 2, 3, 4, 5, 6


def _s64(v: int) -> int:
    """Python int -> the signed value with the same low 64 bits."""
    v &= _MASK64
    return v - (1 << 64) if v >= (1 << 63) else v


def _mix64_py(z: int) -> int:
    z &= _MASK64
    z = ((z ^ (z >> 30)) * _M1) & _MASK64
    z = ((z ^ (z >> 27)) * _M2) & _MASK64
    return z ^ (z >> 31)


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of an int64 tensor."""
    return (z >> s) & ((1 << (64 - s)) - 1)


def _mix64(z: torch.Tensor) -> torch.Tensor:
    z = (z ^ _lsr(z, 30)) * _s64(_M1)
    z = (z ^ _lsr(z, 27)) * _s64(_M2)
    return z ^ _lsr(z, 31)


def _field_sum(u: torch.Tensor) -> torch.Tensor:
    return (u & 0xFFFF) + (_lsr(u, 16) & 0xFFFF) + (_lsr(u, 32) & 0xFFFF) + _lsr(u, 48)


def element_py(seed: int, tensor_id: int, index: int) -> int:
    """Reference for one element in pure Python: returns the integer 2 S - 786420."""
    key = _mix64_py((seed << 32) + tensor_id)
    s = 0
    for j in range(3):
        u = _mix64_py(key + (3 * index + j + 1) * _GOLDEN)
        s += (u & 0xFFFF) + ((u >> 16) & 0xFFFF) + ((u >> 32) & 0xFFFF) + (u >> 48)
    return 2 * s - 786420


def normal(shape, seed: int, tensor_id: int, std: float, dtype: torch.dtype, device="cpu",
           chunk: int = 1 << 24) -> torch.Tensor:
    """Tensor of the given shape with entries ~ N(0, std^2) (Irwin-Hall(12) stand-in)."""
    n = 1
    for s in shape:
        n *= int(s)
    out = torch.empty(n, dtype=dtype, device=device)
    key = _s64(_mix64_py((seed << 32) + tensor_id))
    scale = torch.tensor(std / 131072.0, dtype=torch.float32, device=device)
    golden = _s64(_GOLDEN)
    for start in range(0, n, chunk):
        stop = min(n, start + chunk)
        i3 = torch.arange(start, stop, dtype=torch.int64, device=device) * 3
        s = torch.zeros(stop - start, dtype=torch.int64, device=device)
        for j in range(3):
            s += _field_sum(_mix64((i3 + (j + 1)) * golden + key))
        v = (2 * s - 786420).to(torch.float32) * scale
        out[start:stop] = v.to(dtype)
    return out.reshape(*shape)


def zipf_gate_bias(n_experts: int, s: float, device="cpu", perm_seed: int | None = None) -> torch.Tensor:
    """fp32 gate bias b[e] = -s * ln(rank_e); rank_e = e + 1, or a seeded permutation of 1..E."""
    ranks = list(range(1, n_experts + 1))
    if perm_seed is not None:
        keys = [_mix64_py((perm_seed << 32) + 977 + e) for e in range(n_experts)]
        order = sorted(range(n_experts), key=lambda e: keys[e])
        ranks = [0] * n_experts
        for r, e in enumerate(order):
            ranks[e] = r + 1
    return torch.tensor([-s * math.log(r) for r in ranks], dtype=torch.float32, device=device)


def moe_layer_inputs(T: int, H: int, F: int, E: int, dtype: torch.dtype, device="cpu", seed: int = 0,
                     zipf_s: float | None = 1.2, with_next: bool = True, x_seed: int | None = None):
    """All tensors of one layer call: x, gate, next-layer gate, experts, biases."""
    d = {
        "x": normal((T, H), seed if x_seed is None else x_seed, TID_X, 1.0, dtype, device),
        "wg": normal((E, H), seed, TID_WG, H ** -0.5, dtype, device),
        "w1": normal((E, F, H), seed, TID_W1, H ** -0.5, dtype, device),
        "w3": normal((E, F, H), seed, TID_W3, H ** -0.5, dtype, device),
        "w2": normal((E, H, F), seed, TID_W2, F ** -0.5, dtype, device),
        "bias": None if zipf_s is None else zipf_gate_bias(E, zipf_s, device),
        "wg_next": None,
        "bias_next": None,
    }
    if with_next:
        d["wg_next"] = normal((E, H), seed, TID_WG_NEXT, H ** -0.5, dtype, device)
        d["bias_next"] = None if zipf_s is None else zipf_gate_bias(E, zipf_s, device, perm_seed=seed + 1)
    return d


def to_numpy(t: torch.Tensor):
    """Host numpy view of a tensor's stored values; bf16 comes back as uint16 bit patterns."""
    if t is None:
        return None
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view("uint16")
    return t.numpy()

"""Seeded synthetic inputs for the HOT linear-backward path.

This module only draws numbers.  It holds none of the method's arithmetic (no
transform, no quantizer, no GEMM) and is the single piece of code that both the
CPU oracle's tests and the HIP path's tests / benchmark use, so that both sides
see byte-identical fp32 tensors.  Tensors are produced on the requested device
with a ``torch.Generator`` keyed by (seed, tensor name); callers that feed both
sides generate once and copy the same tensor.

The shapes follow the layer tuples (L, O, I) of the paper's latency table
(ViT-B qkv / proj / fc1 / fc2) scaled to batched token counts, and the value
distributions follow the qualitative structure the paper shows for g_y
(Gaussian bulk, heavy tails, a few outlier channels or tokens).
"""
from __future__ import annotations

import zlib
from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import torch


def _gen(seed: int, name: str, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1_000_003 + zlib.crc32(name.encode())) & 0x7FFF_FFFF_FFFF)
    return g


def normal(shape, std: float, seed: int, name: str, device="cpu") -> torch.Tensor:
    """fp32 N(0, std^2)."""
    g = _gen(seed, name, device)
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32) * std


def student_t(shape, df: int, scale: float, seed: int, name: str, device="cpu") -> torch.Tensor:
    """fp32 Student-t with integer df: z / sqrt(chi2_df / df), times scale."""
    g = _gen(seed, name, device)
    z = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    chi2 = torch.zeros(shape, device=device, dtype=torch.float32)
    for _ in range(df):
        c = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
        chi2 += c * c
    return (z / torch.sqrt(chi2 / df)) * scale


def bf16_round(t: torch.Tensor) -> torch.Tensor:
    """Round to bf16 (nearest even) and widen back to fp32."""
    return t.to(torch.bfloat16).to(torch.float32)


def scale_columns(t: torch.Tensor, count: int, factor: float, seed: int, name: str) -> torch.Tensor:
    """Multiply `count` seed-chosen columns (channels) by `factor`, in place."""
    g = _gen(seed, name + ".cols", "cpu")
    cols = torch.randperm(t.shape[1], generator=g)[:count].to(t.device)
    t[:, cols] *= factor
    return t


def scale_rows(t: torch.Tensor, count: int, factor: float, seed: int, name: str) -> torch.Tensor:
    """Multiply `count` seed-chosen rows (tokens) by `factor`, in place."""
    g = _gen(seed, name + ".rows", "cpu")
    rows = torch.randperm(t.shape[0], generator=g)[:count].to(t.device)
    t[rows, :] *= factor
    return t


@dataclass
class Layer:
    name: str
    L: int
    O: int
    I: int


@dataclass
class Workload:
    """One benchmark / parity configuration: layers plus HOT hyper-parameters."""
    name: str
    layers: List[Layer]
    block: int          # n, WHT block size
    keep: int           # r, HLA rows kept per block
    x_kind: str         # "normal" | "bf16" | "chan_outlier"
    gy_kind: str        # "chan_outlier" | "t4" | "t3" | "normal"
    quantizer: str      # "token" | "tensor" | "select"
    extra: Dict = field(default_factory=dict)


# The five configurations named by the benchmark definition.
WORKLOADS: Dict[str, Workload] = {
    "cfg1_single_512x768x768": Workload(
        "cfg1_single_512x768x768", [Layer("lin", 512, 768, 768)], 16, 8,
        "normal", "chan_outlier", "token"),
    "cfg2_vitb_fc1": Workload(
        "cfg2_vitb_fc1", [Layer("fc1", 64 * 197, 3072, 768)], 32, 16,
        "bf16", "t4", "token"),
    "cfg3_vitb_block_b256": Workload(
        "cfg3_vitb_block_b256",
        [Layer("qkv", 256 * 197, 2304, 768), Layer("proj", 256 * 197, 768, 768),
         Layer("fc1", 256 * 197, 3072, 768), Layer("fc2", 256 * 197, 768, 3072)],
        16, 8, "normal", "chan_outlier", "token"),
    "cfg4_llm7b_mlp": Workload(
        "cfg4_llm7b_mlp",
        [Layer("up", 8 * 2048, 11008, 4096), Layer("down", 8 * 2048, 4096, 11008)],
        64, 32, "chan_outlier", "t3", "select"),
    "cfg5_vitl_chain": Workload(
        "cfg5_vitl_chain",
        [Layer("fc1", 1024 * 197, 4096, 1024), Layer("fc2", 1024 * 197, 1024, 4096)],
        16, 8, "bf16", "normal", "token", {"depth": 24}),
}


def make_x(kind: str, L: int, I: int, seed: int, name: str, device="cpu") -> torch.Tensor:
    x = normal((L, I), 1.0, seed, name + ".x", device)
    if kind == "bf16":
        x = bf16_round(x)
    elif kind == "chan_outlier":
        scale_columns(x, max(1, I // 100), 20.0, seed, name + ".x")
    elif kind != "normal":
        raise ValueError(kind)
    return x


def make_w(O: int, I: int, seed: int, name: str, device="cpu") -> torch.Tensor:
    return normal((O, I), 0.02, seed, name + ".w", device)


def make_gy(kind: str, L: int, O: int, seed: int, name: str, device="cpu") -> torch.Tensor:
    if kind == "normal":
        return normal((L, O), 1e-3, seed, name + ".gy", device)
    if kind == "chan_outlier":
        g = normal((L, O), 1e-3, seed, name + ".gy", device)
        return scale_columns(g, 4, 50.0, seed, name + ".gy")
    if kind == "tok_outlier":
        g = normal((L, O), 1e-3, seed, name + ".gy", device)
        return scale_rows(g, max(1, L // 64), 50.0, seed, name + ".gy")
    if kind == "t4":
        return student_t((L, O), 4, 1e-3, seed, name + ".gy", device)
    if kind == "t3":
        return student_t((L, O), 3, 1e-3, seed, name + ".gy", device)
    raise ValueError(kind)


def make_layer(wl: Workload, layer: Layer, seed: int = 0, device="cpu",
               L: int | None = None) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """(x [L,I], w [O,I], g_y [L,O]) for one layer; `L` overrides the token count."""
    L = layer.L if L is None else L
    tag = f"{wl.name}.{layer.name}"
    return (make_x(wl.x_kind, L, layer.I, seed, tag, device),
            make_w(layer.O, layer.I, seed, tag, device),
            make_gy(wl.gy_kind, L, layer.O, seed, tag, device))

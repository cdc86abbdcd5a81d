"""Seeded synthetic inputs shaped like the paper's workloads.

This module holds NO arithmetic of the method: it only draws random tensors
(activations, weights, upstream gradients, and the multiplicative / additive
noise used to move freshly initialised step sizes and zero points into a
"trained" state) and lists the linear-layer shapes of a Llama-2 decoder block.
Both the GPU tests and the CPU oracle's tests take their inputs from here, so
they see the same bytes.

The paper trains on RedPajama activations flowing through Llama-2 weights
(Sec. 4.1); neither is available offline, so N(0,1) activations / gradients
and N(0, sigma^2) weights of the same shapes stand in for them.
"""
from __future__ import annotations

import zlib
from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class Linear:
    name: str
    out_features: int
    in_features: int


def llama_block(hidden: int, inter: int, kv: int | None = None):
    """The seven quantised linears of one decoder block (out x in)."""
    kv = hidden if kv is None else kv
    return [
        Linear("q", hidden, hidden), Linear("k", kv, hidden), Linear("v", kv, hidden),
        Linear("o", hidden, hidden), Linear("gate", inter, hidden), Linear("up", inter, hidden),
        Linear("down", hidden, inter),
    ]


def llama_block_fused(hidden: int, inter: int, kv: int | None = None):
    """The same block with the linears that share an input stacked along the output dimension (q|k|v and gate|up).
    Groups run along the input dimension, so a stack of weight matrices is quantised exactly like its parts."""
    kv = hidden if kv is None else kv
    return [
        Linear("qkv", hidden + 2 * kv, hidden), Linear("o", hidden, hidden),
        Linear("gate_up", 2 * inter, hidden), Linear("down", hidden, inter),
    ]


@dataclass(frozen=True)
class Workload:
    name: str
    layers: tuple
    tokens: int
    bits: int
    group: int
    w_std: float
    act_dtype: str      # "f32" | "bf16"
    phases: tuple       # subset of ("block_ap", "e2e_qp")


WORKLOADS = {
    # one small fp32 linear: the case the CPU oracle finishes in well under a second
    "single_fp32_w4g128": Workload("single_fp32_w4g128", (Linear("lin", 512, 512),), 256, 4, 128, 0.02, "f32",
                                   ("block_ap",)),
    "llama2_7b_block_ap_w2g64": Workload("llama2_7b_block_ap_w2g64", tuple(llama_block(4096, 11008)), 8192, 2, 64,
                                         0.02, "bf16", ("block_ap",)),
    "llama2_7b_e2e_qp_w2g64": Workload("llama2_7b_e2e_qp_w2g64", tuple(llama_block(4096, 11008)), 4096, 2, 64,
                                       0.02, "bf16", ("e2e_qp",)),
    "llama2_13b_w3g128": Workload("llama2_13b_w3g128", tuple(llama_block(5120, 13824)), 4096, 3, 128, 0.02, "bf16",
                                  ("block_ap", "e2e_qp")),
    # the paper's 4-bit setting (w4g128) on the 7B shapes; not a BASELINE configuration, used by the full-size parity tests
    "llama2_7b_w4g128": Workload("llama2_7b_w4g128", tuple(llama_block(4096, 11008)), 4096, 4, 128, 0.02, "bf16",
                                 ("block_ap", "e2e_qp")),
    # one group per row (the paper's group-size table ends at 256; per-channel is the limit case): the dW kernel then
    # writes per-32-column partials and a second kernel reduces them
    "llama2_7b_w2_per_channel": Workload("llama2_7b_w2_per_channel", tuple(llama_block(4096, 11008)), 4096, 2, -1, 0.02,
                                         "bf16", ("block_ap", "e2e_qp")),
    "llama2_70b_w2g64": Workload("llama2_70b_w2g64", tuple(llama_block(8192, 28672, 1024)), 4096, 2, 64, 0.015,
                                 "bf16", ("block_ap", "e2e_qp")),
    "llama2_7b_block_ap_w2g64_fused": Workload("llama2_7b_block_ap_w2g64_fused", tuple(llama_block_fused(4096, 11008)),
                                               8192, 2, 64, 0.02, "bf16", ("block_ap",)),
    "llama2_70b_w2g64_fused": Workload("llama2_70b_w2g64_fused", tuple(llama_block_fused(8192, 28672, 1024)), 4096, 2,
                                       64, 0.015, "bf16", ("block_ap", "e2e_qp")),
}


def seed_of(*parts) -> int:
    """Stable 31-bit seed from a tuple of names / numbers."""
    return zlib.crc32("/".join(str(p) for p in parts).encode()) & 0x7FFFFFFF


def normal(shape, std: float, seed: int, dtype=torch.float32) -> torch.Tensor:
    """N(0, std^2) on the CPU, drawn in fp32 and then rounded to ``dtype``."""
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    t = torch.empty(tuple(shape), dtype=torch.float32)
    t.normal_(0.0, 1.0, generator=g)
    if std != 1.0:
        t.mul_(std)
    return t.to(dtype)


def uniform(shape, lo: float, hi: float, seed: int) -> torch.Tensor:
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    return torch.empty(tuple(shape), dtype=torch.float32).uniform_(lo, hi, generator=g)


def trained_state_noise(shape, seed: int):
    """Noise that turns min/max-initialised (s, z) into a plausible mid-training state.

    Returns (u, d): multiply s by u ~ U[0.7, 1.1) and add d ~ U{-1, 0, +1} to z.
    Right after min/max initialisation no weight is clamped, so without this
    the two clamped branches of the gradients would never run.
    """
    u = uniform(shape, 0.7, 1.1, seed)
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed) ^ 0x5A5A5A5)
    d = torch.randint(-1, 2, tuple(shape), generator=g).to(torch.float32)
    return u, d


def torch_dtype(name: str):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]

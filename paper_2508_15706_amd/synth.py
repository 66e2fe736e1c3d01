"""Seeded synthetic workloads: tensor lists and pseudo-gradient fills.

This module holds NO arithmetic of the method.  It only describes shapes and
draws random inputs, so it may serve both the HIP library's callers and the
tests that feed the same buffers to the CPU oracle.

The tensor lists are synthetic stand-ins for the trained pseudo-gradients the
paper's experiments (Section 4; LLaMA-style 178M-2B dense models and a MoE
model) produced: same kind of shapes (embedding, attention and SwiGLU matrices,
norm vectors, experts and routers), values drawn from seeded distributions.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Optional

import torch

LAYOUT_FLAT = 0    # runs of 4096 consecutive elements (the paper's rule for 1-D tensors)
LAYOUT_TILE64 = 1  # 64x64 blocks (the paper's rule for 2-D tensors)

ARENA_ALIGN = 64   # tensors start on 256-byte boundaries inside an arena


@dataclass
class TensorSpec:
    name: str
    rows: int
    cols: int
    offset: int = 0          # element offset in the arena
    layout: int = LAYOUT_TILE64
    kind: str = "linear"     # "embed" | "linear" | "norm" | "router" | "expert"
    group: int = -1          # expert id for kind == "expert"

    @property
    def numel(self) -> int:
        return self.rows * self.cols

    def desc(self):
        return (self.rows, self.cols, self.offset, self.layout)


def _finish(specs: List[TensorSpec], flat: bool = False) -> List[TensorSpec]:
    off = 0
    for s in specs:
        s.layout = LAYOUT_FLAT if (flat or s.rows == 1) else LAYOUT_TILE64
        s.offset = off
        off += (s.numel + ARENA_ALIGN - 1) // ARENA_ALIGN * ARENA_ALIGN
    return specs


def arena_numel(specs: List[TensorSpec]) -> int:
    return max((s.offset + (s.numel + ARENA_ALIGN - 1) // ARENA_ALIGN * ARENA_ALIGN for s in specs),
               default=0)


def total_numel(specs: List[TensorSpec]) -> int:
    return sum(s.numel for s in specs)


def dense_llama_list(d: int, n_layers: int, ff: int, vocab: int, kv_dim: Optional[int] = None,
                     flat: bool = False) -> List[TensorSpec]:
    """Embedding, per layer q,k,v,o + SwiGLU gate,up,down + two RMSNorm vectors,
    final norm, untied head."""
    kv = d if kv_dim is None else kv_dim
    sp = [TensorSpec("embed", vocab, d, kind="embed")]
    for l in range(n_layers):
        sp += [
            TensorSpec(f"l{l}.q", d, d), TensorSpec(f"l{l}.k", d, kv),
            TensorSpec(f"l{l}.v", d, kv), TensorSpec(f"l{l}.o", d, d),
            TensorSpec(f"l{l}.gate", d, ff), TensorSpec(f"l{l}.up", d, ff),
            TensorSpec(f"l{l}.down", ff, d),
            TensorSpec(f"l{l}.norm1", 1, d, kind="norm"), TensorSpec(f"l{l}.norm2", 1, d, kind="norm"),
        ]
    sp += [TensorSpec("final_norm", 1, d, kind="norm"), TensorSpec("head", vocab, d, kind="embed")]
    return _finish(sp, flat)


def moe_list(d: int = 1024, n_layers: int = 12, n_experts: int = 16, ff: int = 1408,
             vocab: int = 50257, mats_per_expert: int = 2, flat: bool = False) -> List[TensorSpec]:
    """Tied embedding, per layer q,k,v,o, router d x E, E experts of
    `mats_per_expert` matrices (d x ff ... ff x d), two norm vectors; final norm."""
    sp = [TensorSpec("embed", vocab, d, kind="embed")]
    for l in range(n_layers):
        sp += [TensorSpec(f"l{l}.{n}", d, d) for n in "qkvo"]
        sp.append(TensorSpec(f"l{l}.router", d, n_experts, kind="router"))
        for x in range(n_experts):
            g = l * n_experts + x
            for m in range(mats_per_expert - 1):
                sp.append(TensorSpec(f"l{l}.x{x}.w_in{m}", d, ff, kind="expert", group=g))
            sp.append(TensorSpec(f"l{l}.x{x}.w_out", ff, d, kind="expert", group=g))
        sp += [TensorSpec(f"l{l}.norm1", 1, d, kind="norm"), TensorSpec(f"l{l}.norm2", 1, d, kind="norm")]
    sp.append(TensorSpec("final_norm", 1, d, kind="norm"))
    return _finish(sp, flat)


@dataclass
class Workload:
    name: str
    config_id: int
    specs: List[TensorSpec]
    k: int
    R: int
    beta: float
    lr: float
    rounds: int
    dist: str          # "gauss" | "gauss_fanin" | "mix_t3" | "moe"
    scale: float

    @property
    def N(self) -> int:
        return total_numel(self.specs)

    @property
    def arena(self) -> int:
        return arena_numel(self.specs)


def workload(config_id: int, k: Optional[int] = None, flat: bool = False) -> Workload:
    """The five benchmark configurations (sizes and distributions as configured
    for this build; outer learning rates follow the paper's tuned values for the
    worker count - hyper-parameter appendix - where the configuration names none)."""
    if config_id == 1:
        sp = _finish([TensorSpec("w", 1024, 1024)], flat)
        return Workload("1M-single", 1, sp, k or 64, 4, 0.95, 0.7, 3, "gauss", 1e-3)
    if config_id == 2:
        sp = dense_llama_list(768, 12, 3072, 50257, flat=flat)
        return Workload("190M-dense", 2, sp, k or 64, 8, 0.95, 1.0, 1, "gauss_fanin", 1e-3)
    if config_id == 3:
        sp = dense_llama_list(1024, 24, 4096, 50257, flat=flat)
        return Workload("510M-dense", 3, sp, k or 64, 8, 0.95, 1.0, 5, "mix_t3", 1e-3)
    if config_id == 4:
        sp = dense_llama_list(2048, 24, 8192, 50257, flat=flat)
        return Workload("1.8B-dense", 4, sp, k or 64, 8, 0.95, 1.0, 3, "gauss", 5e-4)
    if config_id == 5:
        sp = moe_list(flat=flat)
        return Workload("645M-moe", 5, sp, k or 32, 16, 0.95, 0.8, 1, "moe", 1e-3)
    raise ValueError(f"unknown config {config_id}")


def paper_shape_list(which: str) -> List[TensorSpec]:
    """The paper's own three dense architectures (hyper-parameter appendix:
    178M, 512M and 2B LLaMA-style models, vocabulary 32000)."""
    if which == "178M":
        return dense_llama_list(1024, 9, 2688, 32000)
    if which == "512M":
        return dense_llama_list(1536, 12, 5440, 32000)
    if which == "2B":
        return dense_llama_list(2560, 24, 7680, 32000, kv_dim=5 * 128)
    raise ValueError(which)


PAPER_LISTS = {"paper178M": ("178M", 6, 8, 1.0), "paper512M": ("512M", 7, 8, 1.0), "paper2B": ("2B", 8, 16, 0.8)}


def paper_workload(name: str, k: Optional[int] = None, flat: bool = False) -> Workload:
    """One of the paper's own three architectures as a workload: Gaussian pseudo-gradients, the
    worker counts and outer learning rates of the paper's runs on that model (R = 8 and 1.0 for
    178M and 512M, R = 16 and 0.8 for 2B), k = 64 unless given."""
    which, cid, R, lr = PAPER_LISTS[name]
    sp = paper_shape_list(which)
    if flat:
        sp = _finish(sp, True)
    return Workload(f"paper-{which}", cid, sp, k or 64, R, 0.95, lr, 1, "gauss", 1e-3)


def seed_for(config_id: int, rnd: int, worker: int) -> int:
    return 1000 * config_id + 100 * rnd + worker


def fill_delta(w: Workload, out: torch.Tensor, rnd: int, worker: int) -> None:
    """Fill the arena `out` (fp32, any device) with the pseudo-gradient of
    (round, worker).  Padding between tensors is left at zero."""
    dev = out.device
    g = torch.Generator(device=dev)
    g.manual_seed(seed_for(w.config_id, rnd, worker))
    out.zero_()
    expert_scale = {}
    expert_dead = set()
    if w.dist == "moe":
        groups = sorted({s.group for s in w.specs if s.kind == "expert"})
        gc = torch.Generator(device="cpu")
        gc.manual_seed(seed_for(w.config_id, 0, 0) + 7)  # which experts are idle: fixed per config
        dead = torch.randperm(len(groups), generator=gc)[: len(groups) // 5].tolist()
        expert_dead = {groups[i] for i in dead}
        gu = torch.Generator(device="cpu")
        gu.manual_seed(seed_for(w.config_id, rnd, worker) + 13)
        u = torch.rand(len(groups), generator=gu) * 0.9 + 0.1
        expert_scale = {grp: float(u[i]) for i, grp in enumerate(groups)}
    for s in w.specs:
        view = out[s.offset:s.offset + s.numel]
        if w.dist == "gauss":
            view.normal_(0.0, w.scale, generator=g)
        elif w.dist == "gauss_fanin":
            fan_in = s.rows if s.kind == "linear" else s.cols
            view.normal_(0.0, w.scale / math.sqrt(fan_in), generator=g)
        elif w.dist == "mix_t3":
            view.normal_(0.0, w.scale, generator=g)
            z = torch.empty_like(view).normal_(0.0, 1.0, generator=g)
            chi = torch.zeros_like(view)
            for _ in range(3):
                chi += torch.empty_like(view).normal_(0.0, 1.0, generator=g) ** 2
            t3 = z / torch.sqrt(chi / 3.0) * w.scale
            pick = torch.empty_like(view).uniform_(0.0, 1.0, generator=g) < 0.1
            view[pick] = t3[pick]
            del z, chi, t3, pick
        elif w.dist == "moe":
            if s.kind == "expert":
                if s.group in expert_dead:
                    continue
                view.normal_(0.0, w.scale * expert_scale[s.group], generator=g)
            else:
                view.normal_(0.0, w.scale, generator=g)
        else:
            raise ValueError(w.dist)


def fill_theta(w: Workload, out: torch.Tensor) -> None:
    g = torch.Generator(device=out.device)
    g.manual_seed(seed_for(w.config_id, 99, 99))
    out.normal_(0.0, 0.02, generator=g)

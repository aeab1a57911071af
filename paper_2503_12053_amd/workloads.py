"""Seeded synthetic workloads for the gradient-compensation path.

This module only *describes* parameter sets (tensor sizes, stage split, staleness per
stage, ring depth) and draws random weights / gradients / weight versions for them.  It
holds none of the method's arithmetic, so both the CPU oracle's tests and the HIP path's
tests can feed from it without sharing anything else.

The paper's workloads are image/tabular classifiers split into P pipeline stages
(Sec. "Experiments"; notation in the appendix "Notations": stage j owns the layers
[L_j, L_{j+1}) and |w_j| parameters, and with maximum staleness P-1 it keeps P-j weight
versions).  None of its datasets or weights are needed here: the path only ever sees
parameter-shaped arrays.  The five workloads below stand in for them, using the public
parameter shapes of ResNet-18 and ViT-B/16.

Value recipe (all "N(0, s)" use s as the standard deviation):
  newest version  W ~ N(0, 0.05)
  older versions  V[k-1] = V[k] - N(0, 1e-3)        (one independent drift per version step)
  gradient        g ~ N(0, 0.01)                    (optionally 1 % of entries x100)
  "amplified"     g ~ N(0, 1), drift ~ N(0, 0.05): makes the compensation term a few
                  per cent of the gradient so that a kernel that skipped it would fail.
bf16 workloads: values are drawn in fp32; master = W, newest version = bf16(W), older
versions bf16(float(V[k]) - drift), gradients rounded to bf16.

Random streams: one torch CPU generator per (workload seed, stage, stream) with
  generator seed = (seed * 4099 + stage) * 1_000_003 + stream
  stream 0 = weights, 1 = gradients, 2 + k = drift between versions k and k+1
  (k = 0 is the oldest version step), 99 = heavy-tail mask; gradients of later
  optimisation steps (multi-step tests) use stream + 1000 * step.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import torch

__all__ = ["Workload", "StageData", "make_workload", "generate_stage", "generate",
           "WORKLOAD_NAMES", "custom_workload"]


@dataclass
class Workload:
    name: str
    tensors: List[Tuple[str, int, int]]          # (name, numel, stage) in model order
    staleness: List[int]                         # tau_j per stage
    ring_depth: int                              # R (stored versions per stage)
    n_iters: int                                 # K (compensation iterations; -1 = one per version step)
    lam: float                                   # lambda, compensation coefficient
    lr: float                                    # eta
    precision: str = "f32"                       # "f32" | "bf16" (bf16 storage + fp32 master)
    seed: int = 0
    weight_std: float = 0.05
    grad_std: float = 0.01
    drift_std: float = 1e-3
    heavy_tail: Optional[Tuple[float, float]] = None   # (probability, scale)
    note: str = ""

    @property
    def n_stages(self) -> int:
        return len(self.staleness)

    def stage_numel(self) -> List[int]:
        out = [0] * self.n_stages
        for _, n, s in self.tensors:
            out[s] += n
        return out

    @property
    def numel(self) -> int:
        return sum(n for _, n, _ in self.tensors)

    def stage_tensors(self, j: int) -> List[Tuple[str, int]]:
        return [(nm, n) for nm, n, s in self.tensors if s == j]


@dataclass
class StageData:
    """Logical (unpadded) data of one stage: the stage's tensors concatenated in order."""
    versions: List[torch.Tensor]                 # R tensors, oldest first, newest last
    grads: torch.Tensor
    master: Optional[torch.Tensor] = None        # fp32, only for bf16 workloads


# ----------------------------------------------------------------------------------------
# parameter shapes
# ----------------------------------------------------------------------------------------
def _resnet18_tensors() -> List[Tuple[str, int, int]]:
    """62 parameter tensors of ResNet-18 (conv / bn weight+bias / fc), 4 stages."""
    t: List[Tuple[str, int, int]] = []

    def conv(name, cout, cin, k, stage):
        t.append((name, cout * cin * k * k, stage))

    def bn(name, c, stage):
        t.append((name + ".weight", c, stage))
        t.append((name + ".bias", c, stage))

    conv("conv1", 64, 3, 7, 0)
    bn("bn1", 64, 0)
    widths = [64, 128, 256, 512]
    cin = 64
    for li, c in enumerate(widths):
        stage = li
        for b in range(2):
            pre = f"layer{li + 1}.{b}"
            conv(pre + ".conv1", c, cin if b == 0 else c, 3, stage)
            bn(pre + ".bn1", c, stage)
            conv(pre + ".conv2", c, c, 3, stage)
            bn(pre + ".bn2", c, stage)
            if b == 0 and cin != c:
                conv(pre + ".downsample.0", c, cin, 1, stage)
                bn(pre + ".downsample.1", c, stage)
        cin = c
    t.append(("fc.weight", 512 * 1000, 3))
    t.append(("fc.bias", 1000, 3))
    return t


def _vit_b_tensors() -> List[Tuple[str, int, int]]:
    """ViT-B/16 (12 blocks, width 768, MLP 3072, 1000 classes) split by block into 8 stages."""
    d, mlp = 768, 3072
    block_stage = [0, 0, 1, 1, 2, 2, 3, 3, 4, 5, 6, 7]
    t: List[Tuple[str, int, int]] = [
        ("patch_embed.weight", d * 3 * 16 * 16, 0), ("patch_embed.bias", d, 0),
        ("cls_token", d, 0), ("pos_embed", 197 * d, 0)]
    for b in range(12):
        s = block_stage[b]
        p = f"blocks.{b}"
        t += [(p + ".norm1.weight", d, s), (p + ".norm1.bias", d, s),
              (p + ".attn.qkv.weight", d * 3 * d, s), (p + ".attn.qkv.bias", 3 * d, s),
              (p + ".attn.proj.weight", d * d, s), (p + ".attn.proj.bias", d, s),
              (p + ".norm2.weight", d, s), (p + ".norm2.bias", d, s),
              (p + ".mlp.fc1.weight", d * mlp, s), (p + ".mlp.fc1.bias", mlp, s),
              (p + ".mlp.fc2.weight", mlp * d, s), (p + ".mlp.fc2.bias", d, s)]
    t += [("norm.weight", d, 7), ("norm.bias", d, 7),
          ("head.weight", d * 1000, 7), ("head.bias", 1000, 7)]
    return t


WORKLOAD_NAMES = {
    1: "tiny_100k_f32",
    2: "resnet18_flat4_f32",
    3: "resnet18_62tensors_f32",
    4: "vit_b_8stage_f32",
    5: "mixed_350m_bf16_master",
}


def make_workload(idx: int) -> Workload:
    """The five benchmark configurations (1-based, in the order they are listed)."""
    if idx == 1:
        return Workload(WORKLOAD_NAMES[1], [("w", 100_000, 0)], [1], 2, 1, 0.5, 0.01, seed=0,
                        note="1 stage, 1 tensor; launch-latency bound")
    if idx == 2:
        n = 2_794_128  # (ResNet-18 without fc: 11,176,512) / 4
        return Workload(WORKLOAD_NAMES[2], [(f"stage{j}", n, j) for j in range(4)],
                        [3, 2, 1, 0], 4, 3, 0.5, 0.01, seed=1,
                        note="4 equal flat stages, K >= tau: one iteration per version step")
    if idx == 3:
        return Workload(WORKLOAD_NAMES[3], _resnet18_tensors(), [3, 2, 1, 0], 4, 2, 0.5, 0.01,
                        seed=2, note="62 tensors of very different size over 4 stages")
    if idx == 4:
        return Workload(WORKLOAD_NAMES[4], _vit_b_tensors(), [7, 6, 5, 4, 3, 2, 1, 0], 8, 3,
                        0.5, 0.01, seed=3, note="86.6 M fp32 parameters, ring 2.77 GB")
    if idx == 5:
        n = 21_875_000
        return Workload(WORKLOAD_NAMES[5], [(f"stage{j}", n, j) for j in range(16)],
                        list(range(15, -1, -1)), 16, 4, 0.3, 0.005, precision="bf16", seed=4,
                        heavy_tail=(0.01, 100.0),
                        note="350 M params, bf16 grads/versions + fp32 master")
    raise ValueError(f"no workload {idx}")


def custom_workload(name, tensor_numels_per_stage, staleness, ring_depth, n_iters, lam=0.5,
                    lr=0.01, precision="f32", seed=1234, **kw) -> Workload:
    """Small ad-hoc workloads for tests: tensor_numels_per_stage = [[n, n, ...], ...]."""
    tensors = []
    for j, sizes in enumerate(tensor_numels_per_stage):
        for i, n in enumerate(sizes):
            tensors.append((f"s{j}.t{i}", int(n), j))
    return Workload(name, tensors, list(staleness), ring_depth, n_iters, lam, lr,
                    precision=precision, seed=seed, **kw)


# ----------------------------------------------------------------------------------------
# random draws
# ----------------------------------------------------------------------------------------
def _gen(seed: int, stage: int, stream: int, device="cpu") -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((seed * 4099 + stage) * 1_000_003 + stream)
    return g


def _normal(n: int, std: float, gen: torch.Generator) -> torch.Tensor:
    x = torch.empty(n, dtype=torch.float32, device=gen.device)
    x.normal_(0.0, std, generator=gen)
    return x


def draw_grads(w: Workload, j: int, n: int, amplified: bool = False, step: int = 0, device="cpu") -> torch.Tensor:
    """Gradient of stage j for optimisation step `step` (fp32 values; caller rounds)."""
    std = 1.0 if amplified else w.grad_std
    g = _normal(n, std, _gen(w.seed, j, 1 + 1000 * step, device))
    if w.heavy_tail is not None:
        p, scale = w.heavy_tail
        u = torch.empty(n, dtype=torch.float32, device=g.device)
        mask = u.uniform_(0, 1, generator=_gen(w.seed, j, 99 + 1000 * step, device)) < p
        g[mask] *= scale
    return g


def generate_stage(w: Workload, j: int, amplified: bool = False,
                   n_versions: Optional[int] = None, device="cpu") -> StageData:
    """Versions (oldest first), gradient and master of stage j, as flat logical arrays.

    device="cpu" (default) draws with torch's CPU generators: bit-reproducible everywhere, what every parity
    test uses.  Another device draws the same recipe with that device's generator (same seeds, different
    streams): for timing runs of the largest workload, where only the distributions matter."""
    n = w.stage_numel()[j]
    R = w.ring_depth if n_versions is None else n_versions
    drift_std = 0.05 if amplified else w.drift_std
    bf16 = w.precision == "bf16"

    W = _normal(n, w.weight_std, _gen(w.seed, j, 0, device))
    master = W.clone() if bf16 else None
    newest = W.to(torch.bfloat16) if bf16 else W
    versions = [newest]
    for k in range(R - 2, -1, -1):           # version step k: between versions k and k+1
        d = _normal(n, drift_std, _gen(w.seed, j, 2 + k, device))
        if bf16:
            older = (versions[0].to(torch.float32) - d).to(torch.bfloat16)
        else:
            older = versions[0] - d
        versions.insert(0, older)
    g = draw_grads(w, j, n, amplified, device=device)
    if bf16:
        g = g.to(torch.bfloat16)
    return StageData(versions, g, master)


def generate(w: Workload, amplified: bool = False) -> List[StageData]:
    return [generate_stage(w, j, amplified) for j in range(w.n_stages)]

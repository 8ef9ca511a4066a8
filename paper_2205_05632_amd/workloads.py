"""Seeded synthetic workloads: tensor-shape tables and gradient generators.

This module holds none of the method's arithmetic.  It only says how large the
flattened parameter vector is, where the layer tensors start, and how the
per-worker gradients (the inputs of one optimizer step) are drawn.  Both the GPU
library's callers and the CPU checker are fed from here, with the same bytes.

The paper trains a CNN, LeNet-5, an LSTM and ResNet-18 on MNIST, CIFAR-10 and
IMDB (Section 5.1, Appendix A).  None of those datasets is used here: a step's
cost and result depend only on shapes and value distributions, so seeded random
gradients with the layer structure of ResNet-18 / ResNet-50 / a GPT-2-small-sized
transformer stand in for them.
"""
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch


def resnet18_shapes(num_classes: int = 10) -> List[int]:
    """Element counts of the 62 parameter tensors of a ResNet-18 (10-way head)."""
    sizes = [64 * 3 * 7 * 7, 64, 64]
    widths = [64, 128, 256, 512]
    cin = 64
    for s, w in enumerate(widths):
        for blk in range(2):
            sizes += [w * cin * 9, w, w, w * w * 9, w, w]
            if blk == 0 and s > 0:
                sizes += [w * cin, w, w]  # 1x1 projection + norm
            cin = w
    sizes += [512 * num_classes, num_classes]
    return sizes


def resnet50_shapes(num_classes: int = 1000) -> List[int]:
    """Element counts of the 161 parameter tensors of a ResNet-50."""
    sizes = [64 * 3 * 7 * 7, 64, 64]
    cin = 64
    for w, reps in zip([64, 128, 256, 512], [3, 4, 6, 3]):
        for blk in range(reps):
            sizes += [w * cin, w, w, w * w * 9, w, w, 4 * w * w, 4 * w, 4 * w]
            if blk == 0:
                sizes += [4 * w * cin, 4 * w, 4 * w]
            cin = 4 * w
    sizes += [2048 * num_classes, num_classes]
    return sizes


def gpt2_small_shapes() -> List[int]:
    """Element counts of the 148 parameter tensors of a 12-layer, 768-wide transformer."""
    h, v, p = 768, 50257, 1024
    sizes = [v * h, p * h]
    for _ in range(12):
        sizes += [h, h, h * 3 * h, 3 * h, h * h, h, h, h, h * 4 * h, 4 * h, 4 * h * h, h]
    sizes += [h, h]
    return sizes


@dataclass
class Workload:
    name: str
    n: int                      # workers
    sizes: List[int]            # layer tensor sizes, flattened in this order
    dist: str                   # "normal" | "student_t3"
    compressor: str             # "topk" | "blocksign" | "none" | "topk_blocks" (top-k inside every layer tensor)
    k: int = 0
    block: str = "layer"        # blocksign: "layer" or an integer block length as string
    steps: int = 10
    unit_std: bool = False      # tiny: N(0,1) everywhere
    sparse_rows: Optional[tuple] = None  # (tensor index, row length, keep probability)
    lr: float = 1e-3
    seed: int = 20220511
    d: int = field(init=False)

    def __post_init__(self):
        self.d = int(sum(self.sizes))
        if self.compressor == "topk_blocks":
            self.k = int(self.block_k().sum())

    def layer_offsets(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(np.asarray(self.sizes, dtype=np.int64))])

    def block_k(self, num: int = 1, den: int = 100) -> np.ndarray:
        """Top-k per layer tensor: floor(size * num / den) coordinates, at least one."""
        sizes = np.asarray(self.sizes, dtype=np.int64)
        return np.maximum(1, (sizes * num) // den)

    def block_offsets(self) -> Optional[np.ndarray]:
        if self.compressor == "topk_blocks":
            return self.layer_offsets()
        if self.compressor != "blocksign":
            return None
        if self.block == "layer":
            return self.layer_offsets()
        b = int(self.block)
        off = np.arange(0, self.d, b, dtype=np.int64)
        return np.concatenate([off, [self.d]])

    def layer_stds(self) -> np.ndarray:
        """One scale per layer tensor, log-uniform in [1e-4, 1e-1], drawn once per run."""
        if self.unit_std:
            return np.ones(len(self.sizes), dtype=np.float32)
        rng = np.random.Generator(np.random.Philox(key=self.seed))
        return (10.0 ** rng.uniform(-4.0, -1.0, size=len(self.sizes))).astype(np.float32)


def _ratio_k(d: int, num: int, den: int) -> int:
    return (d * num) // den


def get(name: str) -> Workload:
    r18, r50, g2 = resnet18_shapes(), resnet50_shapes(), gpt2_small_shapes()
    d18, d50, dg = sum(r18), sum(r50), sum(g2)
    table = {
        "tiny": lambda: Workload("tiny", 4, [65536], "normal", "topk", k=655, steps=10, unit_std=True),
        "tiny_blocksign": lambda: Workload("tiny_blocksign", 4, [65536], "normal", "blocksign",
                                           block="4096", steps=10, unit_std=True),
        "r18_blocksign": lambda: Workload("r18_blocksign", 16, r18, "normal", "blocksign", steps=20),
        "r18_topk1": lambda: Workload("r18_topk1", 16, r18, "normal", "topk",
                                      k=_ratio_k(d18, 1, 100), steps=20),
        "r18_topk01": lambda: Workload("r18_topk01", 16, r18, "normal", "topk",
                                       k=_ratio_k(d18, 1, 1000), steps=20),
        "r18_none": lambda: Workload("r18_none", 16, r18, "normal", "none", steps=20),
        "r18_topk1_layers": lambda: Workload("r18_topk1_layers", 16, r18, "normal", "topk_blocks", steps=20),
        "r50_topk1": lambda: Workload("r50_topk1", 8, r50, "student_t3", "topk",
                                      k=_ratio_k(d50, 1, 100), steps=20),
        "gpt2s_topk01": lambda: Workload("gpt2s_topk01", 8, g2, "normal", "topk",
                                         k=_ratio_k(dg, 1, 1000), steps=10,
                                         sparse_rows=(0, 768, 0.1)),
        "gpt2s_blocksign": lambda: Workload("gpt2s_blocksign", 8, g2, "normal", "blocksign",
                                            block="4096", steps=10, sparse_rows=(0, 768, 0.1)),
    }
    if name not in table:
        raise KeyError(f"unknown workload {name!r}; have {sorted(table)}")
    return table[name]()


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def theta0(w: Workload, device="cpu") -> torch.Tensor:
    """Initial parameter: N(0, 0.01) read as variance 0.01, i.e. std 0.1."""
    g = _gen(device, w.seed * 7919 + 1)
    return torch.randn(w.d, generator=g, device=device, dtype=torch.float32) * 0.1


def coordinate_scale(w: Workload, device="cpu") -> torch.Tensor:
    """Per-coordinate gradient scale (the layer's std repeated over its elements)."""
    stds = torch.from_numpy(w.layer_stds())
    reps = torch.tensor(w.sizes, dtype=torch.int64)
    return torch.repeat_interleave(stds, reps).to(device)


def gradients(w: Workload, step: int, device="cpu", ld: Optional[int] = None,
              scale: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Gradients of all n workers for one step: an n x ld fp32 tensor (columns >= d are 0).

    Values are a pure function of (workload seed, step): worker i's row is drawn
    from its own generator seeded by (seed, step, i).
    """
    ld = w.d if ld is None else int(ld)
    out = torch.zeros((w.n, ld), dtype=torch.float32, device=device)
    if scale is None:
        scale = coordinate_scale(w, device)
    for i in range(w.n):
        g = _gen(device, (w.seed * 1000003 + step) * 1009 + i)
        row = out[i, : w.d]
        if w.dist == "normal":
            row.normal_(generator=g)
        elif w.dist == "student_t3":
            # t with 3 degrees of freedom = z / sqrt(chi2_3 / 3)
            row.normal_(generator=g)
            chi = torch.zeros_like(row)
            tmp = torch.empty_like(row)
            for _ in range(3):
                tmp.normal_(generator=g)
                chi.addcmul_(tmp, tmp)
            row.div_(torch.sqrt(chi / 3.0))
            del chi, tmp
        else:
            raise ValueError(w.dist)
        if not w.unit_std:
            row.mul_(scale)
        if w.sparse_rows is not None:
            t_idx, row_len, keep_p = w.sparse_rows
            off = int(w.layer_offsets()[t_idx])
            nrows = w.sizes[t_idx] // row_len
            keep = torch.rand(nrows, generator=g, device=device) < keep_p
            blk = row[off: off + nrows * row_len].view(nrows, row_len)
            blk.mul_(keep.to(torch.float32).unsqueeze(1))
            # dropped rows are exactly +0.0f (x * 0 may give -0.0f; adding 0 clears the sign)
            blk.add_(0.0)
    return out

"""Seeded synthetic pipeline-stage workloads (shapes, hyper-parameters, fills).

This module holds none of the method's arithmetic: only the ragged tensor
lists of the five benchmark configurations, the optimizer hyper-parameters
each one runs with, and the seeded normal fills of W, g, m, v.  Both the GPU
tests / benchmark and the CPU oracle's tests draw their inputs from here, so
that the two sides see bit-identical values.

The lists stand in for the stage partitions the paper trains (Sec. V-A): the
path's cost depends only on tensor count, sizes and dtypes, and its values
only need realistic magnitudes.  "N(0, x)" means standard deviation x; the
second moment is the square of a normal draw, so some entries are close to 0.
"""
from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import torch

SEED_BASE = 231200839


@dataclass(frozen=True)
class Workload:
    config: int                       # 1..5
    name: str
    optimizer: str                    # "sgdm" | "adam" | "adamw"
    hyper: Dict[str, float]           # lr, beta1, beta2, eps, weight_decay
    t: int
    s_values: Tuple[int, ...]         # version differences the config sweeps
    what_dtype: str                   # "f32" | "bf16"
    shapes: List[Tuple[str, Tuple[int, ...]]]
    sigma: Dict[str, float] = field(default_factory=dict)   # std of W, g, m, and of the draw squared into v

    @property
    def numels(self) -> List[int]:
        out = []
        for _, shp in self.shapes:
            n = 1
            for d in shp:
                n *= d
            out.append(n)
        return out

    @property
    def n_params(self) -> int:
        return sum(self.numels)

    @property
    def bytes_per_param(self) -> int:
        """Algorithmic HBM bytes per parameter: every input read once, every output written once."""
        streams = 3 if self.optimizer == "sgdm" else 4          # W, g, m (, v)
        rd = 4 * streams
        wr = 4 * (streams - 1) + (2 if self.what_dtype == "bf16" else 4)
        return rd + wr


def _resnet50_stages_3_4_fc():
    shapes = []

    def bottleneck(prefix, cin, width, cout, project):
        shapes.append((prefix + ".conv1", (width, cin, 1, 1)))
        shapes.append((prefix + ".norm1.scale", (width,)))
        shapes.append((prefix + ".norm1.shift", (width,)))
        shapes.append((prefix + ".conv2", (width, width, 3, 3)))
        shapes.append((prefix + ".norm2.scale", (width,)))
        shapes.append((prefix + ".norm2.shift", (width,)))
        shapes.append((prefix + ".conv3", (cout, width, 1, 1)))
        shapes.append((prefix + ".norm3.scale", (cout,)))
        shapes.append((prefix + ".norm3.shift", (cout,)))
        if project:
            shapes.append((prefix + ".proj", (cout, cin, 1, 1)))
            shapes.append((prefix + ".proj_norm.scale", (cout,)))
            shapes.append((prefix + ".proj_norm.shift", (cout,)))

    for b in range(6):
        bottleneck("stage3.%d" % b, 512 if b == 0 else 1024, 256, 1024, b == 0)
    for b in range(3):
        bottleneck("stage4.%d" % b, 1024 if b == 0 else 2048, 512, 2048, b == 0)
    shapes.append(("fc.weight", (1000, 2048)))
    shapes.append(("fc.bias", (1000,)))
    return shapes


def _bert_large_layers(n_layers=6, h=1024, ffn=4096):
    shapes = []
    for l in range(n_layers):
        p = "layer%d." % l
        for nm in ("q", "k", "v", "o"):
            shapes.append((p + "attn." + nm + ".weight", (h, h)))
            shapes.append((p + "attn." + nm + ".bias", (h,)))
        shapes.append((p + "ffn.in.weight", (ffn, h)))
        shapes.append((p + "ffn.in.bias", (ffn,)))
        shapes.append((p + "ffn.out.weight", (h, ffn)))
        shapes.append((p + "ffn.out.bias", (h,)))
        for nm in ("ln1", "ln2"):
            shapes.append((p + nm + ".scale", (h,)))
            shapes.append((p + nm + ".shift", (h,)))
    return shapes


def _gpt_layers(n_layers=3, h=2048):
    shapes = []
    for l in range(n_layers):
        p = "layer%d." % l
        shapes.append((p + "qkv.weight", (3 * h, h)))
        shapes.append((p + "qkv.bias", (3 * h,)))
        shapes.append((p + "out.weight", (h, h)))
        shapes.append((p + "out.bias", (h,)))
        shapes.append((p + "mlp.in.weight", (4 * h, h)))
        shapes.append((p + "mlp.in.bias", (4 * h,)))
        shapes.append((p + "mlp.out.weight", (h, 4 * h)))
        shapes.append((p + "mlp.out.bias", (h,)))
        for nm in ("ln1", "ln2"):
            shapes.append((p + nm + ".scale", (h,)))
            shapes.append((p + nm + ".shift", (h,)))
    return shapes


def _llama7b_layers_plus_embedding(n_layers=3, h=4096, ffn=11008, vocab=32000):
    shapes = []
    for l in range(n_layers):
        p = "layer%d." % l
        for nm in ("q", "k", "v", "o"):
            shapes.append((p + "attn." + nm, (h, h)))
        shapes.append((p + "ffn.gate", (ffn, h)))
        shapes.append((p + "ffn.up", (ffn, h)))
        shapes.append((p + "ffn.down", (h, ffn)))
        shapes.append((p + "norm1", (h,)))
        shapes.append((p + "norm2", (h,)))
    shapes.append(("embedding", (vocab, h)))
    return shapes


_ADAM = {"lr": 1e-3, "beta1": 0.9, "beta2": 0.999, "eps": 1e-8, "weight_decay": 0.0}
_ADAMW = dict(_ADAM, weight_decay=0.01)


def workload(config: int) -> Workload:
    if config == 1:
        return Workload(1, "flat-1Mi", "adam", dict(_ADAM), 100, (3,), "f32",
                        [("flat", (1048576,))],
                        {"W": 0.02, "g": 1e-3, "m": 1e-4, "v": 1e-3})
    if config == 2:
        return Workload(2, "resnet50-stages3-4-fc", "sgdm",
                        {"lr": 0.1, "beta1": 0.9, "beta2": 0.0, "eps": 0.0, "weight_decay": 1e-4},
                        1, (0, 1, 2, 3), "f32", _resnet50_stages_3_4_fc(),
                        {"W": 0.05, "g": 1e-2, "m": 1e-2, "v": 0.0})
    if config == 3:
        return Workload(3, "bert-large-6-layers", "adam", dict(_ADAM), 1000, (2,), "bf16",
                        _bert_large_layers(), {"W": 0.02, "g": 1e-4, "m": 1e-5, "v": 1e-4})
    if config == 4:
        return Workload(4, "gpt-2048-3-layers", "adamw", dict(_ADAMW), 1000, tuple(range(8)), "bf16",
                        _gpt_layers(), {"W": 0.02, "g": 1e-4, "m": 1e-5, "v": 1e-4})
    if config == 5:
        return Workload(5, "llama7b-3-layers-embedding", "adamw", dict(_ADAMW), 5000, (7,), "bf16",
                        _llama7b_layers_plus_embedding(),
                        {"W": 0.02, "g": 1e-5, "m": 1e-6, "v": 1e-5})
    raise ValueError("config must be 1..5")


def tensor_seed(config: int, tensor_index: int, which: str) -> int:
    return SEED_BASE + 1000 * config + 4 * tensor_index + {"W": 0, "g": 1, "m": 2, "v": 3}[which]


def fill_tensor(config: int, tensor_index: int, which: str, numel: int, sigma: float, device, out=None) -> torch.Tensor:
    """One flat fp32 tensor of seeded normal draws with std `sigma` (squared for v); into `out` if given."""
    gen = torch.Generator(device=device)
    gen.manual_seed(tensor_seed(config, tensor_index, which))
    x = torch.randn(numel, generator=gen, device=device, dtype=torch.float32)
    if out is not None:
        out.copy_(x)
        x = out
    x.mul_(sigma)
    if which == "v":
        x.mul_(x)
    return x


def make_inputs(wl: Workload, device, tensors=None, layout="packed", optimizer=None):
    """Separately allocated flat tensors for the stage: dict of lists W, g, m, v (v is None for SGDM).

    `optimizer` runs the config's tensor list under another optimizer than its own: the state lists are the ones
    that optimizer has (m is None for RMSprop and Adagrad, v is None for SGDM and Nesterov), and a second moment
    the config gives no scale for is the square of a draw with the first moment's scale.

    `tensors` optionally restricts the list to a subset of tensor indices (same seeds as in the full list).
    layout "packed": plain allocations, which the allocator places back to back.  "skewed" (GPU only): the
    same values, with the W, g, m, v buffers of a tensor placed so that their addresses differ in bits 12-13
    (`stage.alloc_skewed`), the placement the memory system of MI355X prefers.  "local" (GPU only): the same
    values in a near-memory arena (`stage.StageArena`), which also holds the What buffers; the result then has
    the extra keys "What", "arena" (hand both to `Stage`) and "stage_arena" (close it when done).
    """
    idx = range(len(wl.shapes)) if tensors is None else tensors
    numels = wl.numels
    opt = optimizer or wl.optimizer
    sigma = dict(wl.sigma)
    if not sigma.get("v"):
        sigma["v"] = sigma["m"]
    out = {"W": [], "g": [], "m": [] if opt not in ("rmsprop", "adagrad") else None,
           "v": [] if opt not in ("sgdm", "nesterov") else None, "index": list(idx)}
    if layout not in ("packed", "skewed", "local"):
        raise ValueError("layout must be 'packed', 'skewed' or 'local'")
    sa = None
    if layout == "local":
        from .stage import StageArena
        sa = StageArena([numels[i] for i in out["index"]], wl.what_dtype, has_m=out["m"] is not None,
                        has_v=out["v"] is not None, device=device)
        out.update(What=sa.What, arena=sa.arena, stage_arena=sa)
    for pos, i in enumerate(out["index"]):
        for slot, which in enumerate(("W", "g", "m", "v")):
            if out[which] is None:
                continue
            dst = None
            if layout == "skewed":
                from .stage import alloc_skewed
                dst = alloc_skewed(numels[i], torch.float32, device, slot)
            elif layout == "local":
                dst = getattr(sa, which)[pos]
            out[which].append(fill_tensor(wl.config, i, which, numels[i], sigma[which], device, out=dst))
    return out

"""A pipeline stage's tensors bound to a libpipeoptim plan (PyTorch used for device memory only)."""
import warnings
from typing import List, Optional

import torch

from . import binding


# On MI355X the four or five streams of a tensor (W, g, m, v, What at the SAME element offset) are best placed so
# that their addresses differ in bits 12-13 (4 KiB granularity, four values): buffers packed back to back with
# power-of-two sizes agree in those bits and run about 5 % slower on stages made of 4-16 MiB tensors.
SKEW_GRANULE = 4096
SKEW_SLOTS = 4


def address_slot(ptr: int) -> int:
    """Bits 12-13 of a device address."""
    return (ptr // SKEW_GRANULE) % SKEW_SLOTS


def alloc_skewed(n: int, dtype: torch.dtype, device, slot: int) -> torch.Tensor:
    """A contiguous, 4 KiB-aligned tensor of n elements whose address has bits 12-13 equal to `slot`
    (a view into an allocation that is up to 16 KiB larger)."""
    esize = torch.empty(0, dtype=dtype).element_size()
    period = SKEW_GRANULE * SKEW_SLOTS
    buf = torch.empty(n + period // esize, dtype=dtype, device=device)
    shift = ((slot % SKEW_SLOTS) * SKEW_GRANULE - buf.data_ptr()) % period
    assert shift % esize == 0
    return buf[shift // esize: shift // esize + n]


class _DeviceSpan:
    """Describes raw device memory to PyTorch through the array interface it accepts for zero-copy import."""

    def __init__(self, ptr: int, numel: int, typestr: str, owner):
        self.owner = owner      # PyTorch keeps this object for as long as the imported storage lives
        self.__cuda_array_interface__ = {"shape": (numel,), "typestr": typestr, "data": (ptr, False), "version": 3,
                                         "strides": None}


def tensor_at(ptr: int, numel: int, dtype: torch.dtype, device, owner) -> torch.Tensor:
    """A flat tensor over numel elements of device memory at `ptr` that PyTorch did not allocate (no copy).
    `owner` is whatever keeps that memory alive; the tensor's storage holds a reference to it, so the owner is
    not collected while the tensor or any view of it exists (closing the owner explicitly still invalidates them)."""
    if numel == 0:
        return torch.empty(0, dtype=dtype, device=device)
    if dtype == torch.float32:
        t = torch.as_tensor(_DeviceSpan(ptr, numel, "<f4", owner), device=device)
    elif dtype == torch.bfloat16:          # the array interface has no bf16: import the bits, reinterpret
        t = torch.as_tensor(_DeviceSpan(ptr, numel, "<i2", owner), device=device).view(torch.bfloat16)
    else:
        raise ValueError("tensor_at supports float32 and bfloat16")
    if t.data_ptr() != ptr:
        raise RuntimeError("PyTorch copied the arena memory instead of wrapping it")
    return t


class StageArena:
    """All five streams of a stage's tensors (W, g, m, v, What) in one near-memory arena (MI355X).

    The streams of tensor i come from one ``pipeoptim_arena_alloc`` call, so they share one block-to-die layout and a
    plan over them can be localized (``Plan.localize``).  The tensors are uninitialised views of arena memory;
    they stay valid until ``close()``.
    """

    def __init__(self, numels, what_dtype: str, grad_dtype: str = "f32", has_m: bool = True, has_v: bool = True,
                 device="cuda", skew_bytes: Optional[int] = None):
        dev = torch.device(device)
        if dev.index is None:
            dev = torch.device("cuda", torch.cuda.current_device())
        wsz = 2 if what_dtype == "bf16" else 4
        gsz = 2 if grad_dtype == "bf16" else 4
        per_param = 4 + gsz + (4 if has_m else 0) + (4 if has_v else 0) + wsz
        # every buffer is 16 KiB aligned and big ones are followed by a gap: leave room for both
        capacity = sum(n * per_param + 5 * 16384 + 5 * (4 << 20) for n in numels) + (64 << 20)
        with torch.cuda.device(dev):
            self.arena = binding.Arena(capacity)
            if skew_bytes is not None:
                self.arena.set_skew(skew_bytes)
            self.W, self.g, self.What = [], [], []
            self.m = [] if has_m else None
            self.v = [] if has_v else None
            gdt = torch.bfloat16 if grad_dtype == "bf16" else torch.float32
            wdt = torch.bfloat16 if what_dtype == "bf16" else torch.float32
            for n in numels:
                sizes = [4 * n, gsz * n] + ([4 * n] if has_m else []) + ([4 * n] if has_v else []) + [wsz * n]
                ptrs = self.arena.alloc(sizes)
                k = iter(ptrs)
                self.W.append(tensor_at(next(k), n, torch.float32, dev, self.arena))
                self.g.append(tensor_at(next(k), n, gdt, dev, self.arena))
                if has_m:
                    self.m.append(tensor_at(next(k), n, torch.float32, dev, self.arena))
                if has_v:
                    self.v.append(tensor_at(next(k), n, torch.float32, dev, self.arena))
                self.What.append(tensor_at(next(k), n, wdt, dev, self.arena))
        self.what_dtype = what_dtype

    def stage(self) -> "Stage":
        """A Stage (plan) over this arena's tensors, localized for the current stream.  Close it before the arena."""
        return Stage(self.W, self.g, self.m, self.v, self.what_dtype, What=self.What, arena=self.arena)

    def close(self) -> None:
        """Frees the arena's memory.  Every tensor it handed out is invalid from here on."""
        self.arena.destroy()


class Stage:
    """Holds flat fp32 W, g, m, v tensors (m or v may be None) and the What buffers, plus the plan over their addresses.

    All arithmetic happens inside ``pipeoptim_step_predict``; this class only keeps the
    tensors alive, allocates What, and passes pointers and the current stream.
    """

    def __init__(self, W: List[torch.Tensor], g: List[torch.Tensor], m: Optional[List[torch.Tensor]],
                 v: Optional[List[torch.Tensor]], what_dtype: str, skew_what: bool = True,
                 What: Optional[List[torch.Tensor]] = None, arena: Optional[binding.Arena] = None,
                 learn_layout: bool = False):
        """`What`: prediction buffers the caller already holds (else the stage allocates them).  `arena`: the
        near-memory arena the tensors came from, if any; the plan is then localized over it.  `learn_layout`
        (without an arena): let the library find the die layout of these buffers by timing and order its tiles
        accordingly (`pipeoptim_plan_learn_layout`; a blocking set-up step)."""
        for lst in (W,) + ((m,) if m is not None else ()) + ((v,) if v is not None else ()):
            for x in lst:
                if x.dtype != torch.float32 or not x.is_contiguous() or x.device.type != "cuda":
                    raise ValueError("W, m, v must be contiguous fp32 tensors on the GPU")
        gdt = {x.dtype for x in g} or {torch.float32}
        if len(gdt) != 1 or not gdt <= {torch.float32, torch.bfloat16}:
            raise ValueError("gradients must all be fp32 or all be bf16")
        if any(not x.is_contiguous() or x.device.type != "cuda" for x in g):
            raise ValueError("gradients must be contiguous tensors on the GPU")
        self.grad_dtype = "bf16" if gdt == {torch.bfloat16} else "f32"
        self.W, self.g, self.m, self.v = W, g, m, v
        self.what_dtype = what_dtype
        tdt = torch.bfloat16 if what_dtype == "bf16" else torch.float32
        if What is not None:
            if len(What) != len(W) or any(h.dtype != tdt or h.numel() != x.numel() or not h.is_contiguous()
                                          for h, x in zip(What, W)):
                raise ValueError("What must match W in length and sizes and have the prediction's dtype")
            self.What = What
        elif skew_what and not (learn_layout and arena is None):
            # What takes an address slot (bits 12-13) that no other stream of its tensor uses, else the gradient's.
            # (Not under a learnt layout: a stream has a say in the vote only if it starts on a chunk boundary, and an
            # fp32 What 4 KiB off the others' blocks took the learnt order's gain away on the 0.74B-parameter stage.)
            self.What = []
            for i, x in enumerate(W):
                used = {address_slot(lst[i].data_ptr()) for lst in (W, g, m, v) if lst is not None}
                free = [k for k in range(SKEW_SLOTS) if k not in used]
                slot = free[0] if free else address_slot(g[i].data_ptr())
                self.What.append(alloc_skewed(x.numel(), tdt, x.device, slot))
        else:
            self.What = [torch.empty(x.numel(), dtype=tdt, device=x.device) for x in W]
        self.numel = [x.numel() for x in W]
        ptrs = lambda lst: [x.data_ptr() for x in lst]
        self.plan = binding.Plan(self.numel, ptrs(W), ptrs(g), ptrs(m) if m is not None else None,
                                 ptrs(v) if v is not None else None,
                                 ptrs(self.What), what_dtype, torch.cuda.current_stream().cuda_stream,
                                 grad_dtype=self.grad_dtype)
        self.n_local_params = (self.plan.localize(arena, torch.cuda.current_stream().cuda_stream)
                               if arena is not None else 0)
        if arena is None and learn_layout:
            try:
                self.n_local_params = self.plan.learn_layout(torch.cuda.current_stream().cuda_stream)
            except binding.PipeOptimError as e:         # e.g. not an MI355X in one partition: the plain order still works
                warnings.warn("the layout of the buffers could not be learnt (%s): using the plain tile order" % e)

    @property
    def n_params(self) -> int:
        return sum(self.numel)

    def step_predict(self, hyper: binding.po_hyper, t: int, s: int) -> None:
        self.plan.step_predict(hyper, t, s, torch.cuda.current_stream().cuda_stream)

    def predict(self, hyper: binding.po_hyper, t: int, s: int) -> None:
        self.plan.predict(hyper, t, s, torch.cuda.current_stream().cuda_stream)

    def close(self) -> None:
        self.plan.destroy()

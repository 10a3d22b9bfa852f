"""A pipeline stage's tensors bound to a libpipeoptim plan (PyTorch used for device memory only)."""
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


class Stage:
    """Holds flat fp32 W, g, m, v tensors (m or v may be None) and the What buffers, plus the plan over their addresses.

    All arithmetic happens inside ``pipeoptim_step_predict``; this class only keeps the
    tensors alive, allocates What, and passes pointers and the current stream.
    """

    def __init__(self, W: List[torch.Tensor], g: List[torch.Tensor], m: Optional[List[torch.Tensor]],
                 v: Optional[List[torch.Tensor]], what_dtype: str, skew_what: bool = True):
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
        if skew_what:
            # What takes an address slot (bits 12-13) that no other stream of its tensor uses, else the gradient's
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

    @property
    def n_params(self) -> int:
        return sum(self.numel)

    def step_predict(self, hyper: binding.po_hyper, t: int, s: int) -> None:
        self.plan.step_predict(hyper, t, s, torch.cuda.current_stream().cuda_stream)

    def predict(self, hyper: binding.po_hyper, t: int, s: int) -> None:
        self.plan.predict(hyper, t, s, torch.cuda.current_stream().cuda_stream)

    def close(self) -> None:
        self.plan.destroy()

"""A pipeline stage's tensors bound to a libpipeoptim plan (PyTorch used for device memory only)."""
from typing import List, Optional

import torch

from . import binding


class Stage:
    """Holds flat fp32 W, g, m, v tensors (m or v may be None) and the What buffers, plus the plan over their addresses.

    All arithmetic happens inside ``pipeoptim_step_predict``; this class only keeps the
    tensors alive, allocates What, and passes pointers and the current stream.
    """

    def __init__(self, W: List[torch.Tensor], g: List[torch.Tensor], m: Optional[List[torch.Tensor]],
                 v: Optional[List[torch.Tensor]], what_dtype: str):
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

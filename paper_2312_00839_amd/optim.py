"""The weight-handling part of paper Algorithm 1 for the parameters of a ``torch.nn.Module`` pipeline stage.

``StageOptimizer`` binds a stage's parameters to a libpipeoptim plan and exposes what a 1F1B runtime needs
each iteration (the runtime itself, its schedule and its transfers are not part of this library):

    opt = StageOptimizer(stage_module.parameters(), "adamw", lr=1e-3, weight_decay=0.01, rank=r, depth=D)
    ...
    with opt.predicted_weights():        # Algorithm 1: forward pass with What_{t+s}
        y = stage_module(x)
    ...                                  # backward pass fills the gradient buffers
    opt.step()                           # Eq. 1 and, in the same kernel, next iteration's What (Eq. 5)

All arithmetic runs in the library's kernels: this class allocates buffers, points ``param.grad`` at them,
swaps ``param.data`` between W and What (pointer swaps, no copies: the cache / restore of Algorithm 1 costs
nothing), and passes pointers.  Parameters must be contiguous fp32 tensors on the GPU.

With ``arena=True`` (the default for stages of 4 Mi parameters and more; smaller ones gain nothing from it) the
optimizer owns the stage's memory the way flat-parameter optimizers do: the parameters are moved once into the
library's near-memory arena, next to their gradient, state and What buffers, so that both kernels run with every
XCC on its own die's HBM.  ``close()`` moves them back out.  With ``arena=False, learn_layout=True`` the parameters
stay where the caller put them, the other buffers are plain PyTorch allocations, and the plan finds out by timing
which die each 2 MiB piece lies on (``pipeoptim_plan_learn_layout``): most of the arena's gain, depending on how
the allocator happened to place the buffers.
"""
import contextlib
import warnings
from typing import Iterable, List, Optional

import torch

from . import binding
from .stage import Stage, StageArena, address_slot, alloc_skewed, SKEW_SLOTS


class StageOptimizer:
    def __init__(self, params: Iterable[torch.nn.Parameter], optimizer: str = "adamw", lr: float = 1e-3,
                 betas=(0.9, 0.999), eps: float = 1e-8, weight_decay: float = 0.0, momentum: float = 0.9,
                 dampening: float = 0.0, alpha: float = 0.99, rank: int = 0, depth: int = 1,
                 decay_in_prediction: bool = True, arena: Optional[bool] = None, learn_layout: bool = False):
        self.params: List[torch.nn.Parameter] = [p for p in params]
        if not self.params:
            raise ValueError("no parameters")
        for p in self.params:
            if p.dtype != torch.float32 or not p.is_contiguous() or p.device.type != "cuda":
                raise ValueError("parameters must be contiguous fp32 tensors on the GPU")
        if optimizer not in binding.OPTIMIZERS:
            raise ValueError("unknown optimizer %r" % optimizer)
        self.optimizer = optimizer
        self.s = binding.pipeoptim_version_difference(depth, rank)            # paper Eq. 4
        self.rank, self.depth = rank, depth
        self.t = 0                                                            # steps taken; the next step is t + 1
        self._warned_moved = False
        if optimizer == "sgdm":
            b1, b2 = momentum, dampening
        elif optimizer == "nesterov":
            b1, b2 = momentum, 0.0
        elif optimizer == "rmsprop":
            b1, b2 = 0.0, alpha
        elif optimizer == "adagrad":
            b1, b2 = 0.0, 0.0
        else:
            b1, b2 = betas
        self.hyper = binding.make_hyper(optimizer, lr, b1, b2, eps, weight_decay, decay_in_prediction)
        binding.pipeoptim_coefficients(self.hyper, 1, self.s)                 # validates the hyper-parameters now

        dev = self.params[0].device
        has_m = optimizer not in ("rmsprop", "adagrad")
        has_v = optimizer not in ("sgdm", "nesterov")
        self._arena: Optional[StageArena] = None
        if arena is None:
            arena = sum(p.numel() for p in self.params) >= (1 << 22)
        if arena:
            try:
                self._arena = StageArena([p.numel() for p in self.params], "f32", has_m=has_m, has_v=has_v, device=dev)
            except binding.PipeOptimError as e:
                warnings.warn("near-memory arena unavailable (%s): using plain allocations" % e)
        if self._arena is not None:
            sa = self._arena
            for p, w in zip(self.params, sa.W):
                w.copy_(p.data.view(-1))
                p.data = w.view_as(p)                                          # the parameter now lives in the arena
            for lst in (sa.g, sa.m, sa.v):
                for x in lst or ():
                    x.zero_()
            self._W, self._g, self._m, self._v = sa.W, sa.g, sa.m, sa.v
            for p, g in zip(self.params, self._g):
                p.grad = g.view_as(p)
            self._stage = Stage(self._W, self._g, self._m, self._v, "f32", What=sa.What, arena=sa.arena)
            self._What = self._stage.What
            self._swapped = False
            return
        self._W = [p.data.view(-1) for p in self.params]

        def state_like(slot_offset):
            # gradient and state buffers: zero-filled, placed in address slots (bits 12-13) next to W's; under a learnt
            # layout plain allocations instead (a stream has a say there only if it starts on a chunk boundary)
            if learn_layout:
                return [torch.zeros(w.numel(), dtype=torch.float32, device=dev) for w in self._W]
            out = []
            for w in self._W:
                x = alloc_skewed(w.numel(), torch.float32, dev, (address_slot(w.data_ptr()) + slot_offset) % SKEW_SLOTS)
                out.append(x.zero_())
            return out

        self._g = state_like(1)
        self._m: Optional[List[torch.Tensor]] = state_like(2) if has_m else None
        self._v: Optional[List[torch.Tensor]] = state_like(3 if has_m else 2) if has_v else None
        for p, g in zip(self.params, self._g):
            p.grad = g.view_as(p)                                              # autograd accumulates in place
        # the prediction is consumed by an fp32 module, so What is fp32 here (the C ABI also offers bf16)
        self._stage = Stage(self._W, self._g, self._m, self._v, "f32", skew_what=not learn_layout, learn_layout=learn_layout)
        self._What = self._stage.What
        self._swapped = False

    # ------------------------------------------------------------------ Algorithm 1
    def step(self) -> None:
        """W_{t+1} = W_t - lr*dW_t (Eq. 1) and What = W_t - lr*s*dW_t (Eq. 5), one kernel."""
        if self._swapped:
            raise RuntimeError("step() inside predicted_weights(): the parameters currently alias What")
        moved = False
        for p, g, w in zip(self.params, self._g, self._W):
            if p.grad is None:
                raise RuntimeError("a parameter has no gradient: run the backward pass before step()")
            moved = moved or p.grad.data_ptr() != g.data_ptr()
            if p.data_ptr() != w.data_ptr():
                raise RuntimeError("a parameter's storage was replaced after this optimizer was created "
                                   "(e.g. by module.to() or by assigning .data): create the optimizer afterwards")
        if moved:
            # autograd put the gradients into buffers of its own (e.g. after zero_grad(set_to_none=True)): hand the new
            # addresses to the plan, on the current stream, ahead of the step; nothing is waited for
            new = []
            for p in self.params:
                gr = p.grad
                if gr.dtype != torch.float32 or not gr.is_contiguous() or gr.device != p.device or gr.numel() != p.numel():
                    raise RuntimeError("gradients must be contiguous fp32 tensors of the parameter's size on its device")
                new.append(gr.view(-1))
            self._stage.plan.set_pointers(1, [x.data_ptr() for x in new], torch.cuda.current_stream().cuda_stream)
            still_local = self._stage.plan.local_params()         # a learnt order survives new gradient buffers, the arena's does not
            if self._stage.n_local_params and not still_local and not self._warned_moved:
                warnings.warn("gradients left the near-memory arena: the step runs in the plain tile order from here on "
                              "(keep the buffers this optimizer handed out, e.g. zero_grad(set_to_none=False), to avoid that)")
                self._warned_moved = True
            self._stage.n_local_params = still_local
            self._g = new
            self._stage.g = new
        self.t += 1
        self._stage.step_predict(self.hyper, self.t, self.s)

    def refresh_prediction(self, s: Optional[int] = None) -> None:
        """What = W - lr*s*dW from the cached state alone (Table 1 optimizers), e.g. for another version difference."""
        if self.t < 1:
            raise RuntimeError("no optimizer state yet: call step() first")
        self._stage.predict(self.hyper, self.t, self.s if s is None else s)

    def zero_grad(self) -> None:
        for g in self._g:
            g.zero_()

    @contextlib.contextmanager
    def predicted_weights(self):
        """Inside the block the module's parameters ARE the predicted weights (their storage is What); on exit
        they are W again.  Before the first step(), or on the last stage (s = 0), What is not used and the
        block runs with W itself, as Algorithm 1's else-branch does."""
        use = self.s > 0 and self.t > 0
        if use:
            for p, h in zip(self.params, self._What):
                p.data = h.view_as(p)
            self._swapped = True
        try:
            yield
        finally:
            if use:
                for p, w in zip(self.params, self._W):
                    p.data = w.view_as(p)
                self._swapped = False

    # ------------------------------------------------------------------ state access
    def state(self):
        """The optimizer's buffers (flat views, by parameter order): dict with W, g, m, v, What and the step count."""
        return {"W": self._W, "g": self._g, "m": self._m, "v": self._v, "What": self._What, "t": self.t, "s": self.s}

    @property
    def n_local_params(self) -> int:
        """Parameters whose streams the kernels process in the near-memory tile order."""
        return self._stage.n_local_params

    def close(self) -> None:
        """Destroys the plan.  With an arena, first gives every parameter an ordinary allocation again (a copy of
        its current value) and drops the gradient views, since the arena's memory goes away."""
        self._stage.close()
        if self._arena is not None:
            for p in self.params:
                p.data = p.data.clone()
                p.grad = None
            torch.cuda.synchronize()
            self._arena.close()
            self._arena = None

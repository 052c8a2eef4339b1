"""torch.optim-style front ends over the C ABI: they own the state buffers and one plan per parameter group and
call lpmm_adamw4_step_multi / lpmm_sgdm4_step_multi.  Orchestration only -- every number is computed by lpmm4.so.

    opt = AdamW4bit(model.parameters(), lr=1e-3, weight_decay=0.01)
    loss.backward(); opt.step(); opt.zero_grad()

Parameters must be fp32, contiguous and on one GPU; gradients fp32 or bf16 (one type per optimizer).  A plan
refers to parameter and gradient buffers by address, so it is rebuilt whenever one of them has moved (keep
gradients in place with zero_grad(set_to_none=False) to avoid that).
"""
from __future__ import annotations

import torch

from . import binding as _b

QUANT_MIN_NUMEL = 4096          # App. C.1: tensors of at most 4096 elements keep fp32 states


def _default_no_decay(p: torch.Tensor) -> bool:
    return p.ndim <= 1              # biases and normalization weights


class _PlanOptimizer:
    def __init__(self, params, no_decay):
        self.params = [p for p in params if p.requires_grad]
        if not self.params:
            raise ValueError("no parameters")
        dev = self.params[0].device
        for p in self.params:
            if p.dtype != torch.float32 or not p.is_contiguous() or p.device != dev or dev.type != "cuda":
                raise ValueError("parameters must be contiguous fp32 tensors on one GPU")
        self.device = dev
        self.no_decay = no_decay if callable(no_decay) else (lambda p, flag=bool(no_decay): flag and p.ndim <= 1)
        self.t = 0
        self._plan = None
        self._key = None
        self._states = None

    # subclasses: _new_state(p) -> state, _desc(p, g, state) -> TensorDesc, _step(plan)
    def _ensure_plan(self):
        grads = []
        for p in self.params:
            if p.grad is None:
                raise ValueError("every parameter needs a gradient (frozen parameters: requires_grad=False)")
            g = p.grad
            if not g.is_contiguous() or g.dtype not in (torch.float32, torch.bfloat16):
                raise ValueError("gradients must be contiguous fp32 or bf16")
            grads.append(g)
        if len({g.dtype for g in grads}) != 1:
            raise ValueError("one gradient type per optimizer")
        key = tuple((p.data_ptr(), g.data_ptr()) for p, g in zip(self.params, grads)) + (grads[0].dtype,)
        if key == self._key:
            return
        with torch.cuda.device(self.device):
            _b.ensure_init(4096)            # lookup tables; a plan carries its own workspace
            if self._states is None:
                self._states = [self._new_state(p) for p in self.params]
            if self._plan is not None:
                torch.cuda.synchronize(self.device)
                _b.lpmm_adamw4_plan_release(self._plan)
            descs = [self._desc(p, g, st) for p, g, st in zip(self.params, grads, self._states)]
            self._plan = _b.new_plan(descs, _b.GRAD_BF16 if grads[0].dtype == torch.bfloat16 else _b.GRAD_F32,
                                     self.device)
        self._key = key

    @torch.no_grad()
    def step(self):
        self._ensure_plan()
        self.t += 1
        with torch.cuda.device(self.device):
            self._step(self._plan)

    def zero_grad(self, set_to_none: bool = False):
        for p in self.params:
            if p.grad is not None:
                if set_to_none:
                    p.grad = None
                else:
                    p.grad.zero_()

    def state_buffers(self):
        """The device buffers that make up the optimizer state, per parameter (for checkpoints)."""
        return self._states

    @staticmethod
    def _tensors_of(st):
        if torch.is_tensor(st):
            return {"m": st}
        if isinstance(st, tuple):
            return {"m": st[0], "v": st[1]}
        return {k: v for k, v in vars(st).items() if torch.is_tensor(v)}

    def state_dict(self):
        """Step count and a copy of every state buffer (the buffers ARE the whole optimizer state).  States exist
        after the first step."""
        # a capturable optimizer counts its steps on the device (graph replays do not run step())
        t = int(self.step_dev.item()) if getattr(self, "capturable", False) else self.t
        if self._states is None:
            return {"t": t, "states": None}
        return {"t": t, "states": [{k: v.clone() for k, v in self._tensors_of(st).items()} for st in self._states]}

    def load_state_dict(self, sd):
        """Into an optimizer over the same parameters (same shapes, same second-moment kind); the buffers keep
        their addresses, so the plan stays valid."""
        if sd["states"] is None:
            return
        if self._states is None:
            with torch.cuda.device(self.device):
                _b.ensure_init(4096)
                self._states = [self._new_state(p) for p in self.params]
        if len(sd["states"]) != len(self._states):
            raise ValueError("state of a different parameter list")
        for st, saved in zip(self._states, sd["states"]):
            mine = self._tensors_of(st)
            if set(mine) != set(saved) or any(mine[k].shape != saved[k].shape for k in mine):
                raise ValueError("state of a different shape or kind")
            for k in mine:
                mine[k].copy_(saved[k])
        self.t = int(sd["t"])
        if getattr(self, "capturable", False):
            self.step_dev.fill_(self.t)

    def __del__(self):
        try:
            if self._plan is not None:
                _b.lpmm_adamw4_plan_release(self._plan)
        except Exception:
            pass


class AdamW4bit(_PlanOptimizer):
    """4-bit AdamW.  second_moment: "rank1" (rank-1/Linear for matrices, the paper's 4-bit AdamW), "factor" (row and
    column statistics for matrices, the paper's 4-bit Factor) or "b128" (every tensor flat, block-wise).  Tensors
    with 3 to 8 dimensions get one statistic per index of every dimension under "rank1" and are taken as
    (shape[0], rest) matrices under "factor" (and beyond 8 dimensions); tensors of at most 4096 elements keep fp32
    states, larger 1-dimensional ones block-wise 4-bit states."""

    def __init__(self, params, lr=1e-3, betas=(0.9, 0.999), eps=1e-8, weight_decay=1e-2, second_moment="rank1",
                 no_decay=_default_no_decay, capturable=False):
        super().__init__(params, no_decay)
        if second_moment not in ("rank1", "factor", "b128"):
            raise ValueError("second_moment must be rank1, factor or b128")
        self.lr, self.betas, self.eps, self.weight_decay, self.second_moment = lr, betas, eps, weight_decay, second_moment
        # capturable: the learning rate and the step number live on the device, so that step() can be captured
        # into a graph and replayed (run one step eagerly first: the plan is built then); change the rate with set_lr
        self.capturable = capturable
        if capturable:
            self.lr_dev = torch.full((1,), float(lr), device=self.device)
            self.step_dev = torch.zeros(1, dtype=torch.int64, device=self.device)

    def set_lr(self, lr: float):
        self.lr = lr
        if self.capturable:
            self.lr_dev.fill_(float(lr))

    def _new_state(self, p):
        n = p.numel()
        if n <= QUANT_MIN_NUMEL:
            return (torch.zeros(n, device=p.device), torch.zeros(n, device=p.device))
        if p.ndim <= 1 or self.second_moment == "b128":
            return _b.new_state_b128(n, p.device)
        rows, cols = p.shape[0], n // p.shape[0]
        if self.second_moment == "factor":
            return _b.new_state_factor(rows, cols, p.device)
        if 3 <= p.ndim <= 8:
            return _b.new_state_nd(tuple(p.shape), p.device)      # rank-1 normalization over every dimension
        return _b.new_state(rows, cols, p.device)

    def _desc(self, p, g, st):
        nd = bool(self.no_decay(p))
        if isinstance(st, tuple):
            return _b.make_desc(p, g, st, 1, p.numel(), no_decay=nd)
        return _b.make_desc(p, g, st, no_decay=nd)

    def _step(self, plan):
        if self.capturable:
            self.step_dev += 1
            _b.lpmm_adamw4_step_multi_capturable(plan, self.lr_dev, self.step_dev, self.betas[0], self.betas[1],
                                                 self.eps, self.weight_decay)
        else:
            _b.lpmm_adamw4_step_multi(plan, self.lr, self.betas[0], self.betas[1], self.eps, self.weight_decay, self.t)


class SGDM4bit(_PlanOptimizer):
    """SGD with momentum, momentum in 4 bits (fp32 for tensors of at most 4096 elements); no weight decay."""

    def __init__(self, params, lr=1e-2, momentum=0.9):
        super().__init__(params, no_decay=False)
        self.lr, self.momentum = lr, momentum

    def _new_state(self, p):
        n = p.numel()
        return torch.zeros(n, device=p.device) if n <= QUANT_MIN_NUMEL else _b.new_state_sgdm(n, p.device)

    def _desc(self, p, g, st):
        return _b.make_desc_sgdm(p, g, st, p.numel())

    def _step(self, plan):
        _b.lpmm_sgdm4_step_multi(plan, self.lr, self.momentum)

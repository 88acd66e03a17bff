"""torch.optim front end of the fused 8-bit optimizer step (Sec. IV: "SGD (8-bit)", "Adam (8-bit)").

Host orchestration only: state allocation, parameter lists and hyper-parameters.  Every
arithmetic step runs in libq8opt.so through one multi-tensor launch per parameter group
(`q8opt.Plan`); there is no CPU or eager-PyTorch fallback.

    opt = Adam8bit(model.parameters(), lr=1e-3)            # Eq. adam as printed
    opt = Adam8bit(..., weight_decay=0.05, decoupled_weight_decay=True, bias_correction=True)   # AdamW
    opt = SGD8bit(model.parameters(), lr=0.1, momentum=0.9, weight_decay=1e-4)

Parameters must be contiguous CUDA tensors, all float32, all bfloat16 or all float16 within a group
(gradients in the same dtype).  Tensors with fewer than `min_8bit_size` elements keep
32-bit states (same formulas, no quantization).  Optimizer state lives in ordinary torch
tensors, so `state_dict()` / `load_state_dict()` checkpoint and resume it.
"""
from __future__ import annotations

import torch

from . import q8opt

__all__ = ["Adam8bit", "SGD8bit"]

_TABLES = {}


def _tables(device):
    """Search tables of the two dynamic-tree codebooks, built once per device."""
    key = (device.type, device.index)
    if key not in _TABLES:
        with torch.cuda.device(device):
            _TABLES[key] = (q8opt.upload_qtable(q8opt.build_qtable(q8opt.build_codebook(True)), device),
                            q8opt.upload_qtable(q8opt.build_qtable(q8opt.build_codebook(False)), device))
    return _TABLES[key]


class _Keep:
    """Opaque holder: torch's load_state_dict casts every state *tensor* to the parameter's dtype,
    which would turn the uint8 codes into floats (and float32 block maxima into bfloat16)."""

    def __init__(self, t):
        self.t = t


class _Q8Optimizer(torch.optim.Optimizer):
    _adam = True

    def __init__(self, params, defaults, block_size, min_8bit_size):
        if block_size < 64 or block_size > 4096 or block_size & (block_size - 1):
            raise ValueError("block_size must be a power of two in [64, 4096]")
        defaults = dict(defaults, block_size=block_size, min_8bit_size=min_8bit_size)
        super().__init__(params, defaults)
        self._plans = {}

    # ------------------------------------------------------------------ state
    def _init_state(self, p, group):
        st = self.state[p]
        if st:
            return st
        n, B = p.numel(), group["block_size"]
        dev = p.device
        if n < group["min_8bit_size"]:
            st["m_f32"] = torch.zeros(n, dtype=torch.float32, device=dev)
            if self._adam:
                st["r_f32"] = torch.zeros(n, dtype=torch.float32, device=dev)
        else:
            nb = -(-n // B)
            st["m_q"] = torch.full((n,), 127, dtype=torch.uint8, device=dev)      # code of 0.0, signed map
            st["N_m"] = torch.zeros(nb, dtype=torch.float32, device=dev)
            if self._adam:
                st["r_q"] = torch.zeros(n, dtype=torch.uint8, device=dev)         # code of 0.0, unsigned map
                st["N_r"] = torch.zeros(nb, dtype=torch.float32, device=dev)
        return st

    def _plan(self, gi, group):
        """(plan, device) for the group's parameters that have gradients; rebuilt only when a buffer
        address changed (the table holds raw device pointers)."""
        entries, sig = [], []
        dtype = device = None
        for p in group["params"]:
            if p.grad is None:
                continue
            g = p.grad
            if g.is_sparse:
                raise RuntimeError("sparse gradients are not supported")
            if not p.is_cuda or not p.is_contiguous() or not g.is_contiguous():
                raise RuntimeError("parameters and gradients must be contiguous CUDA tensors")
            if p.dtype not in (torch.float32, torch.bfloat16, torch.float16) or g.dtype != p.dtype:
                raise RuntimeError("parameters and gradients must share one of float32, bfloat16, float16")
            if dtype is None:
                dtype, device = p.dtype, p.device
            elif p.dtype != dtype or p.device != device:
                raise RuntimeError("one parameter group must hold one dtype on one device")
            st = self._init_state(p, group)
            e = dict(w=p.data, g=g)
            e.update({k: v for k, v in st.items() if k in ("m_q", "r_q", "N_m", "N_r", "m_f32", "r_f32")})
            entries.append(e)
            sig.append((p.data_ptr(), g.data_ptr(), p.numel()) + tuple(st[k].data_ptr() for k in sorted(st)
                                                                       if torch.is_tensor(st[k])))
        if not entries:
            return None
        sig = (tuple(sig), group["block_size"], dtype)
        cached = self._plans.get(gi)
        if cached is None or cached[0] != sig:
            if cached is not None:
                torch.cuda.current_stream(device).synchronize()     # work using the old table may be in flight
                cached[1].destroy()
            with torch.cuda.device(device):
                plan = q8opt.Plan(entries, group["block_size"], wg_dtype=str(dtype).replace("torch.", ""))
            self._plans[gi] = cached = (sig, plan, device)
        return cached[1], cached[2]

    def _launch(self, plan, tabs, group):
        raise NotImplementedError

    def _drop_plans(self):
        for _, plan, device in self._plans.values():
            torch.cuda.current_stream(device).synchronize()
            plan.destroy()
        self._plans = {}

    def load_state_dict(self, state_dict):
        """As torch's, but state tensors keep their own dtypes (uint8 codes, float32 maxima)."""
        held = {pid: {k: (_Keep(v) if torch.is_tensor(v) else v) for k, v in st.items()}
                for pid, st in state_dict["state"].items()}
        super().load_state_dict({"state": held, "param_groups": state_dict["param_groups"]})
        for p, st in self.state.items():
            for k, v in list(st.items()):
                if isinstance(v, _Keep):
                    st[k] = v.t.detach().clone().to(p.device)
        self._drop_plans()           # the tables hold the addresses of the replaced state tensors

    @torch.no_grad()
    def step(self, closure=None):
        loss = None
        if closure is not None:
            with torch.enable_grad():
                loss = closure()
        for gi, group in enumerate(self.param_groups):
            got = self._plan(gi, group)
            if got is None:
                continue
            plan, device = got
            with torch.cuda.device(device):
                self._launch(plan, _tables(device), group)
        return loss

    def __del__(self):
        for _, plan, _ in getattr(self, "_plans", {}).values():
            try:
                plan.destroy()
            except Exception:
                pass


class Adam8bit(_Q8Optimizer):
    """Adam with 8-bit block-wise quantized states (Eq. adam + Eq. quant1-quant3).

    Defaults reproduce the printed update: no bias correction, weight decay (if any) added
    to the gradient.  `bias_correction=True` and `decoupled_weight_decay=True` select the
    two extensions of the C ABI (together: AdamW)."""
    _adam = True

    def __init__(self, params, lr=1e-3, betas=(0.9, 0.999), eps=1e-8, weight_decay=0.0,
                 bias_correction=False, decoupled_weight_decay=False, block_size=2048, min_8bit_size=4096):
        defaults = dict(lr=lr, betas=betas, eps=eps, weight_decay=weight_decay, bias_correction=bias_correction,
                        decoupled_weight_decay=decoupled_weight_decay, step=0)
        super().__init__(params, defaults, block_size, min_8bit_size)

    def _launch(self, plan, tabs, group):
        group["step"] += 1
        flags = (q8opt.FLAG_BIAS_CORRECTION if group["bias_correction"] else 0) | \
                (q8opt.FLAG_DECOUPLED_WD if group["decoupled_weight_decay"] else 0)
        plan.multi_adam8bit_step(tabs[0], tabs[1], group["lr"], group["betas"][0], group["betas"][1], group["eps"],
                                 weight_decay=group["weight_decay"], t=group["step"], flags=flags)


class SGD8bit(_Q8Optimizer):
    """SGD with momentum, the momentum held in 8 bits (Eq. sgd + Eq. quant1-quant3)."""
    _adam = False

    def __init__(self, params, lr=0.1, momentum=0.9, weight_decay=0.0, block_size=2048, min_8bit_size=4096):
        defaults = dict(lr=lr, momentum=momentum, weight_decay=weight_decay)
        super().__init__(params, defaults, block_size, min_8bit_size)

    def _launch(self, plan, tabs, group):
        plan.multi_sgd8bit_step(tabs[0], group["lr"], group["momentum"], weight_decay=group["weight_decay"])

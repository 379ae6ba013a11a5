"""torch.autograd integration: ISOPO gradients for the linear layers of a model.

Both listings of the paper are written as a full backward hook of a linear
module: the forward pass registers the layer's input activations, backprop runs
on objective = sum(log_prob) WITHOUT advantages, and the hook turns the layer's
(act_in, grad_out) into the ISOPO microbatch gradient, which is accumulated into
the module's gradient.  This module is that harness, and nothing more: it
collects the two matrices and the ragged sequence layout and hands them to the
layer step of the HIP library (`isopo.py`); no arithmetic of the method happens
here.

    hooks = IsopoHooks(model, seq_offsets, advantages, variant="interacting", lam=1e-3)
    loss = log_prob.sum()          # no advantages
    loss.backward()
    hooks.apply()                  # weight.grad <- ISOPO gradient of every hooked layer
    hooks.remove()

Token layout: a hooked layer sees inputs of shape [N, d_in] (packed, ragged:
sequence i owns rows seq_offsets[i]:seq_offsets[i+1]) or [B, T, d_in] (B
sequences of T tokens; seq_offsets is then implied).
"""
from __future__ import annotations

from typing import Callable, Dict, Iterable, Optional

import numpy as np
import torch
from torch import nn

VARIANTS = ("interacting", "interacting_ema", "fisher", "fisher_token_samples", "rescaled")


def _hip_layer_step(X, Delta, seq_offsets, A, cfg) -> torch.Tensor:
    """The layer step on the GPU through the C ABI (imported lazily so the
    harness can be imported, and its plumbing tested, without the library)."""
    from . import isopo
    layer = isopo.Layer(X, Delta, seq_offsets)
    reg_mode = isopo.REG_REL_TRACE if cfg["relative_reg"] else isopo.REG_ABSOLUTE
    variant = cfg["variant"]
    if variant in ("interacting", "fisher"):
        return isopo.layer_step(layer, A, variant, cfg["lam"], reg_mode, "auto")["dW"]
    if variant == "interacting_ema":
        # the interacting experiment's regulariser: lam * trailing mean over steps of the layer's mean eigenvalue,
        # the state living on the device with the hooks object (one per module)
        K, ws = isopo.layer_gram(layer, "materialised", keep_stash=isopo.KEEP_FAST)
        c, _ = isopo.transform_ema(K, A, "interacting", cfg["lam"], cfg["ema_state"], cfg["ema_decay"])
        return isopo.weighted_grad(layer, c, ws, layout=isopo.stash_layout(layer)[0])
    if variant == "fisher_token_samples":
        n_s = min(cfg["n_samples"], layer.n_tokens)
        idx = torch.randperm(layer.n_tokens, generator=cfg["generator"], device="cpu")[:n_s]
        c, _ = isopo.fisher_samples(layer, idx.to(torch.int32).to(X.device), A, cfg["lam"], reg_mode)
        return isopo.weighted_grad(layer, c)            # one weighted contraction from X and Delta, no stash
    if variant == "rescaled":
        K, ws = isopo.layer_gram(layer, "materialised", keep_stash=isopo.KEEP_FAST)
        f2, g2 = isopo.gram_norms(K)
        p, q, r = cfg["pqr"]
        c = isopo.rescale(f2, g2, A, p, q, r, reg=cfg["reg3"])
        return isopo.weighted_grad(layer, c, ws, layout=isopo.stash_layout(layer)[0])
    raise ValueError(f"unknown variant {variant!r}")


class IsopoHooks:
    """Forward and full-backward hooks on the nn.Linear modules of `model`.

    layer_step: callable (X [N, d_in], Delta [N, d_out], seq_offsets (host int32),
    A [m], cfg dict) -> dW [d_out, d_in]; defaults to the HIP library.  Tests of
    the plumbing may pass another implementation.
    """

    def __init__(self, model: nn.Module, seq_offsets, advantages: torch.Tensor, variant: str = "interacting",
                 lam: float = 1e-3, relative_reg: bool = True, n_samples: int = 32, pqr=(0.0, -1.0, -2.0),
                 reg3=(0.0, 0.0, 0.0), modules: Optional[Iterable[nn.Linear]] = None, seed: int = 0,
                 layer_step: Optional[Callable] = None, ema_decay: float = 0.9,
                 ema_states: Optional[Dict[nn.Linear, torch.Tensor]] = None):
        if variant not in VARIANTS:
            raise ValueError(f"variant must be one of {VARIANTS}")
        self.seq_offsets = None if seq_offsets is None else np.ascontiguousarray(np.asarray(seq_offsets, dtype=np.int32))
        self.A = advantages
        self.cfg = {"variant": variant, "lam": float(lam), "relative_reg": bool(relative_reg),
                    "n_samples": int(n_samples), "pqr": tuple(pqr), "reg3": tuple(reg3),
                    "generator": torch.Generator(device="cpu").manual_seed(seed), "ema_decay": float(ema_decay)}
        # variant "interacting_ema": per-module {trailing mean, steps seen} on the device; pass the dict of a
        # previous step's hooks object (its .ema_states) to carry the means over training steps
        self.ema_states: Dict[nn.Linear, torch.Tensor] = ema_states if ema_states is not None else {}
        self.layer_step = layer_step or _hip_layer_step
        self.grads: Dict[nn.Linear, torch.Tensor] = {}
        self.captured: Dict[nn.Linear, tuple] = {}
        self._act: Dict[nn.Linear, torch.Tensor] = {}
        self._handles = []
        mods = list(modules) if modules is not None else [m for m in model.modules() if isinstance(m, nn.Linear)]
        for m in mods:
            self._handles.append(m.register_forward_hook(self._forward))
            self._handles.append(m.register_full_backward_hook(self._backward))
        self.modules = mods

    def _forward(self, mod, inputs, output):
        self._act[mod] = inputs[0].detach()

    def _offsets_for(self, x: torch.Tensor) -> np.ndarray:
        if x.dim() == 3:
            b, t = x.shape[0], x.shape[1]
            return (np.arange(b + 1, dtype=np.int64) * t).astype(np.int32)
        if self.seq_offsets is None:
            raise ValueError("packed [N, d] inputs need seq_offsets")
        return self.seq_offsets

    def _backward(self, mod, grad_input, grad_output):
        x = self._act.pop(mod)
        off = self._offsets_for(x)
        X = x.reshape(-1, x.shape[-1]).contiguous()
        Delta = grad_output[0].detach().reshape(-1, grad_output[0].shape[-1]).contiguous()
        if int(off[-1]) != X.shape[0]:
            raise ValueError(f"seq_offsets cover {int(off[-1])} tokens, the layer saw {X.shape[0]}")
        self.captured[mod] = (X, Delta, off)
        if self.cfg["variant"] == "interacting_ema":
            if mod not in self.ema_states:
                self.ema_states[mod] = torch.zeros(2, dtype=torch.float32, device=X.device)
            self.cfg["ema_state"] = self.ema_states[mod]
        dW = self.layer_step(X, Delta, off, self.A, self.cfg)
        if mod in self.grads:
            self.grads[mod] += dW           # a second microbatch accumulates, as `mod.grad += grad` does
        else:
            self.grads[mod] = dW

    def apply(self) -> None:
        """weight.grad <- the accumulated ISOPO gradient (replacing what plain
        backprop of sum(log_prob) left there)."""
        for mod, dW in self.grads.items():
            mod.weight.grad = dW.to(mod.weight.dtype).reshape(mod.weight.shape)

    def remove(self) -> None:
        for h in self._handles:
            h.remove()
        self._handles = []

"""Shared set-up of the GPU parity tests: same synthetic weights to the oracle (host, float64)
and to the HIP library (device, storage dtype)."""
import numpy as np

from synth import get_config, make_weights, make_prompt
from synth.gpu import weights_to_device


def have_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


class Pair:
    """Oracle + library context over identical weights."""

    def __init__(self, name, act="auto", storage=None, lib_over=None, **cfg_over):
        import paper_2506_03566_amd as P
        from oracle.model import Weights
        self.cfg = get_config(name, **cfg_over)
        self.storage = storage if storage is not None else make_weights(self.cfg)
        self.W = Weights(self.cfg, self.storage)
        # fp32 storage is compared against exact arithmetic; 16-bit storage against the oracle's
        # mixed-precision model (activations rounded where they become GEMM operands)
        self.act = (None if self.cfg.dtype == 0 else self.cfg.dtype) if act == "auto" else act
        self.dev_weights = weights_to_device(self.cfg, self.storage)
        self.ctx = P.Poss(self.cfg, self.dev_weights, **(lib_over or {}))

    def oracle(self):
        from oracle.poss import PossOracle
        return PossOracle(self.W, self.cfg, act=self.act)

    def close(self):
        self.ctx.close()


def tol_for(cfg):
    """Max-abs logit error allowed: 1e-4 in float32 mode, 2e-2 with 16-bit storage."""
    return 1e-4 if cfg.dtype == 0 else 2e-2


# End-to-end error of 16-bit logits after the whole target at the 8B / 13B shapes.  The 2e-2 bound holds per
# layer and per Head on identical inputs; through 32-40 random-initialised layers every flipped rounding of
# an activation is carried on and amplified, and two summation orders (the oracle's float64 sums, the
# kernels' float32 sums; consecutive or scattered cache slots) flip different ones.  Measured against the
# teacher-forced oracle at the 8B shape: max|dlogit| 0.14 - 0.20 over 12 positions across builds (logit std 1.28);
# tests allow 0.30, and two runs of the library may therefore disagree where a top-2 gap is below twice that.
E2E_LOGIT_TOL = 0.30


def tree_from_gpu(tr):
    from oracle.tree import Tree
    d = tr.as_dict()
    return Tree(d["token"], d["parent"]), d

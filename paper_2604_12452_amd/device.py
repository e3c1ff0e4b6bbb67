"""Device plumbing shared by the benchmark, the smoke check and the GPU tests: moves seeded inputs to
the GPU, allocates outputs with torch and calls liblca through its binding.  No arithmetic of the method."""
from __future__ import annotations

import numpy as np

from . import inputs


def to_dev(a: np.ndarray, dtype: str):
    import torch
    if dtype == "bf16":
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def from_dev(t, dtype: str) -> np.ndarray:
    """Device tensor -> float64 numpy, exactly."""
    import torch
    if dtype == "bf16":
        return inputs.to_f64(t.view(torch.int16).cpu().numpy().view(np.uint16), "bf16")
    return t.cpu().numpy().astype(np.float64)


def lca_desc(wl: inputs.Workload, **over):
    from . import lca
    kw = dict(B=wl.B, L=wl.L, H=wl.H, S=wl.S, d_pool=wl.d_pool, d_sel=wl.d_sel, g=wl.g, w=wl.w, n_q=wl.n_q, mode=wl.mode,
              dtype={"bf16": lca.BF16, "f32": lca.F32, "f16": lca.F16}[wl.dtype], scale=wl.scale)
    kw.update(over)
    return lca.Desc(**kw)


class GpuRun:
    """Inputs of a workload on the device plus the outputs of the liblca calls made on them."""

    def __init__(self, wl: inputs.Workload, Q: np.ndarray, POOL: np.ndarray, SEL: np.ndarray, rep_logit_bias: float = 0.0):
        from . import lca
        self.lca, self.wl = lca, wl
        self.desc = lca_desc(wl, rep_logit_bias=rep_logit_bias)
        self.Q, self.POOL, self.SEL = to_dev(Q, wl.dtype), to_dev(POOL, wl.dtype), to_dev(SEL, wl.dtype)
        self.ws = lca.alloc_workspace(self.desc)

    def condense(self, alpha: bool = True):
        import torch
        self.pool_rep, self.sel_rep, self.anchor, self.alpha = self.lca.alloc_condensed(self.desc, alpha=alpha)
        self.lca.condense(self.desc, self.Q, self.POOL, self.SEL, self.pool_rep, self.sel_rep, self.anchor, self.alpha, self.ws)
        torch.cuda.synchronize()
        return self

    def prefill(self, lse: bool = True):
        import torch
        d = self.desc
        self.O = torch.full((d.B, d.L, d.H, d.d_pool), float("nan"), dtype=self.lca.torch_dtype(d), device="cuda")
        self.lse = torch.full((d.B, d.L, d.H), float("nan"), dtype=torch.float32, device="cuda") if lse else None
        self.lca.prefill_attn(d, self.Q, self.POOL, self.SEL, self.pool_rep, self.sel_rep, self.O, self.lse, self.ws)
        torch.cuda.synchronize()
        return self

    def dense(self, lse: bool = True):
        import torch
        d = self.desc
        self.O_dense = torch.full((d.B, d.L, d.H, d.d_pool), float("nan"), dtype=self.lca.torch_dtype(d), device="cuda")
        self.lse_dense = torch.full((d.B, d.L, d.H), float("nan"), dtype=torch.float32, device="cuda") if lse else None
        self.lca.dense_attn(d, self.Q, self.POOL, self.SEL, self.O_dense, self.lse_dense, self.ws)
        torch.cuda.synchronize()
        return self

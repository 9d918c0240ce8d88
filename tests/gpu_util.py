"""Helpers for the GPU parity tests: move seeded numpy inputs to the device as bf16, run the HIP
path through the binding, bring results back as float64."""
import numpy as np
import torch

import paper_2407_20761_amd as ob
import synth_inputs as si

DEV = "cuda"


def to_dev(a, dtype=torch.bfloat16):
    """bf16-representable float32 numpy -> bf16 (or fp32) device tensor (exact)."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV).to(dtype)


def to_np(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def bytes_buf(n):
    return torch.empty(max(int(n), 256), dtype=torch.uint8, device=DEV)


def saved_view(desc, T, saved, name, shape, dtype=torch.bfloat16):
    off = ob.ob_block_saved_offset(desc, T, name)
    n = int(np.prod(shape)) * (2 if dtype == torch.bfloat16 else 4)
    return saved[off:off + n].view(dtype).view(*shape)


class BlockRun:
    """One block's device state: weights, grads, saved, workspace."""

    def __init__(self, shape, w_np, T, dtype=torch.bfloat16):
        self.shape, self.T = shape, T
        self.desc = ob.make_desc(shape, ob.OB_BF16 if dtype == torch.bfloat16 else ob.OB_FP32)
        self.w = {n: to_dev(a, dtype) for n, a in w_np.items()}
        self.g = {n: torch.zeros_like(t) for n, t in self.w.items()}
        self.saved = bytes_buf(ob.ob_block_saved_bytes(self.desc, T))
        self.ws = bytes_buf(ob.ob_block_workspace_bytes(self.desc, T))

    def fwd(self, x, seg):
        y = torch.empty_like(x)
        ob.ob_block_fwd(self.desc, self.w, x, y, self.saved, seg, self.ws)
        return y

    def bwd(self, x, dy, seg, accumulate=False):
        dx = torch.empty_like(x)
        ob.ob_block_bwd(self.desc, self.w, self.g, accumulate, x, dy, dx, self.saved, seg, self.ws)
        return dx


def run_block(shape, w_np, x_np, dy_np, cu, dtype=torch.bfloat16):
    T = x_np.shape[0]
    seg = ob.Segments(cu)
    run = BlockRun(shape, w_np, T, dtype)
    x, dy = to_dev(x_np, dtype), to_dev(dy_np, dtype)
    y = run.fwd(x, seg)
    dx = run.bwd(x, dy, seg)
    torch.cuda.synchronize()
    return run, to_np(y), to_np(dx), {n: to_np(t) for n, t in run.g.items()}

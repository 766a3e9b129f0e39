"""torch.autograd wrapper over the C ABI, so that the head drops into an encoder (Sec. 5 of the paper
trains through it).  Argument marshalling only: forward and backward both run in the HIP library, and
only (Y, I) are saved between them (Sec. 3 "Backward Pass")."""
from __future__ import annotations

import torch

from . import binding as lsr


class _LsrHead(torch.autograd.Function):
    @staticmethod
    def forward(ctx, H, W, bias, mask):
        if not (H.is_cuda and W.is_cuda and bias.is_cuda and mask.is_cuda):
            raise RuntimeError("lsr_head: all tensors must live on the GPU; there is no CPU path")
        if H.dtype != W.dtype or H.dtype not in (torch.bfloat16, torch.float32):
            raise TypeError("lsr_head: H and W must both be bfloat16 or both float32")
        H, W = H.contiguous(), W.contiguous()
        bias = bias.contiguous().float()
        mask = (mask != 0).to(torch.uint8).contiguous()
        B, S, D = H.shape
        V = W.shape[0]
        dt = lsr.LSR_BF16 if H.dtype == torch.bfloat16 else lsr.LSR_F32
        Y = torch.empty((B, V), dtype=torch.float32, device=H.device)
        I = torch.empty((B, V), dtype=torch.int32, device=H.device)
        ws = torch.empty(lsr.lsr_head_workspace_bytes(B, S, D, V, dt, False), dtype=torch.uint8, device=H.device)
        lsr.lsr_head_forward(B, S, D, V, dt, H, W, bias, mask, Y, I, ws)
        ctx.save_for_backward(H, W, Y, I)
        ctx.shape = (B, S, D, V, dt)
        ctx.mark_non_differentiable(I)
        return Y, I

    @staticmethod
    def backward(ctx, dY, _dI):
        H, W, Y, I = ctx.saved_tensors
        B, S, D, V, dt = ctx.shape
        need_h, need_w, need_b = ctx.needs_input_grad[0], ctx.needs_input_grad[1], ctx.needs_input_grad[2]
        dY = dY.contiguous().float()
        dev = H.device
        # the library stores dH and dW in the parameters' own dtype (float32 sums, rounded once)
        dH = torch.empty((B, S, D), dtype=H.dtype, device=dev) if need_h else None
        dW = torch.empty((V, D), dtype=W.dtype, device=dev) if need_w else None
        db = torch.empty((V,), dtype=torch.float32, device=dev) if need_b else None
        if need_h or need_w or need_b:
            ws = torch.empty(lsr.lsr_head_backward_ex_workspace_bytes(B, S, D, V, dt, dt), dtype=torch.uint8, device=dev)
            lsr.lsr_head_backward_ex(B, S, D, V, dt, H, W, dY, Y, I, dH, dW, db, dt, False, ws)
        return dH, dW, db, None


def lsr_head(H: torch.Tensor, W: torch.Tensor, bias: torch.Tensor, mask: torch.Tensor):
    """Y[b,v] = max over valid s of log(1 + ReLU(H[b,s,:] . W[v,:] + bias[v]))  (Eq. 1), differentiable
    in H, W and bias.  Returns (Y float32 [B,V], I int32 [B,V]); I is the arg-max position.
    Gradients are summed in float32 and stored by the library in the dtype of the parameter they belong to."""
    return _LsrHead.apply(H, W, bias, mask)

"""torch.autograd front end of the HIP library: plumbing only.

`cat_loss(H, W, y, B, K, ...)` returns the scalar CAT-weighted loss as a tensor that back-propagates
into H and W through `pard2_cat_fwd` / `pard2_cat_bwd`; `cat_kd_loss(...)` does the same for the
Eq.12 token loss with the distillation term.  Every number is produced by the library's kernels; this
module only saves the forward's `lse` / `w` for the backward and hands the upstream gradient over as
`grad_loss`.  The CAT weight is a constant of the backward (stop-gradient), as the library defines it.
"""
from __future__ import annotations

import torch

from . import binding as b


def _dtype_code(t):
    if t.dtype == torch.bfloat16:
        return b.PARD2_BF16
    if t.dtype == torch.float32:
        return b.PARD2_FP32
    raise b.Pard2Error(f"unsupported storage type {t.dtype}")


class _CatLoss(torch.autograd.Function):
    @staticmethod
    def forward(ctx, H, W, y, conf_in, valid_len, desc):
        out = b.pard2_cat_fwd(desc, H, W, y, conf_in=conf_in, valid_len=valid_len)
        ctx.desc = desc
        ctx.save_for_backward(H, W, y, valid_len if valid_len is not None else torch.empty(0), out["lse"], out["w"])
        ctx.has_vl = valid_len is not None
        ctx.aux = out
        return out["loss"].reshape(())

    @staticmethod
    def backward(ctx, grad):
        H, W, y, vl, lse, w = ctx.saved_tensors
        gl = grad.reshape(1).to(torch.float32).contiguous()
        dH, dW = b.pard2_cat_bwd(ctx.desc, H, W, y, lse, w, valid_len=vl if ctx.has_vl else None, grad_loss=gl)
        return dH, dW, None, None, None, None


class _CatKdLoss(torch.autograd.Function):
    @staticmethod
    def forward(ctx, H, W, Ht, Wt, y, conf_in, valid_len, desc):
        out = b.pard2_cat_kd_fwd(desc, H, W, Ht, Wt, y, conf_in=conf_in, valid_len=valid_len)
        ctx.desc = desc
        ctx.save_for_backward(H, W, Ht, Wt, y, valid_len if valid_len is not None else torch.empty(0), out["lse"],
                              out["lse_t"], out["w"])
        ctx.has_vl = valid_len is not None
        ctx.aux = out
        return out["loss"].reshape(())

    @staticmethod
    def backward(ctx, grad):
        H, W, Ht, Wt, y, vl, lse, lse_t, w = ctx.saved_tensors
        gl = grad.reshape(1).to(torch.float32).contiguous()
        dH, dW = b.pard2_cat_kd_bwd(ctx.desc, H, W, Ht, Wt, y, lse, lse_t, w, valid_len=vl if ctx.has_vl else None,
                                    grad_loss=gl)
        return dH, dW, None, None, None, None, None, None


def _desc(H, W, B, K, weight_mode, reduction, beta, gamma, ignore_index):
    T, d = H.shape
    if T != B * K or W.shape[1] != d or H.stride(1) != 1 or W.stride(1) != 1:
        raise b.Pard2Error("H must be [B*K, d] and W [V, d], unit stride along d")
    return b.make_desc(T, d, W.shape[0], B, K, _dtype_code(H), weight_mode=weight_mode, reduction=reduction, beta=beta,
                       gamma=gamma, ignore_index=ignore_index, ldH=H.stride(0), ldW=W.stride(0))


def cat_loss(H, W, y, B, K, conf_in=None, valid_len=None, weight_mode=b.PARD2_W_CAT, reduction=b.PARD2_RED_MEAN_VALID,
             beta=0.1, gamma=1.0, ignore_index=-100):
    """CAT-weighted cross-entropy (Eq.9-11) of the head W over hidden states H; differentiable in H and W."""
    return _CatLoss.apply(H, W, y, conf_in, valid_len, _desc(H, W, B, K, weight_mode, reduction, beta, gamma,
                                                           ignore_index))


def cat_kd_loss(H, W, Ht, Wt, y, B, K, conf_in=None, valid_len=None, weight_mode=b.PARD2_W_CAT,
                reduction=b.PARD2_RED_MEAN_VALID, beta=0.1, gamma=1.0, ignore_index=-100):
    """Eq.12 token loss s (beta CE + KL(teacher || draft)); differentiable in the draft's H and W only."""
    return _CatKdLoss.apply(H, W, Ht, Wt, y, conf_in, valid_len, _desc(H, W, B, K, weight_mode, reduction, beta, gamma,
                                                                     ignore_index))

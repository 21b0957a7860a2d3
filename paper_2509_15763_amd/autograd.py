"""torch.autograd wrappers around the C ABI (argument marshalling and tape bookkeeping only: the forward
and the backward both run in the HIP kernels of libunigist).

    out = gist_attention(q, k, v, r, W)                         # [B,Hq,L,D], [B,Hkv,L,D] -> [B,Hq,L,D]
    out = gist_attention(q, k, v, r, W, sinks=128, window_mode=UNIGIST_WINDOW_UNITS)
    out = gist_attention_varlen(q, k, v, r, W, cu_seqlens)      # [Hq,T,D], [Hkv,T,D] -> [Hq,T,D]
    out = gist_attention_varlen(q, k, v, r, W, cu_seqlens, sinks=128, window_mode=UNIGIST_WINDOW_UNITS)

The backward of the attention needs q, k, v, out and the row-wise log-sum-exp, which the forward saves
(Sec. 4.2: no attention matrix is ever materialised).
"""
import torch

from . import binding as _b


class _GistAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, r, W, sinks, window_mode):
        # a q in the projection layout ([B, L, Hq, D] in memory, passed as its [B, Hq, L, D] view) is used as it is
        # and out comes back in the same layout; everything else is made contiguous
        q = q if _b._q_strided(q) else q.contiguous()
        k, v = k.contiguous(), v.contiguous()
        out, lse = _b.attn_fwd(q, k, v, r, W, sinks=sinks, window_mode=window_mode)
        ctx.save_for_backward(q, k, v, out, lse)
        ctx.mask = (int(r), int(W), int(sinks), int(window_mode))
        return out

    @staticmethod
    def backward(ctx, dout):
        q, k, v, out, lse = ctx.saved_tensors
        r, W, sinks, window_mode = ctx.mask
        if not _b._q_strided(q):
            dout = dout.contiguous()
        dq, dk, dv = _b.attn_bwd(q, k, v, out, lse, dout, r, W, sinks=sinks, window_mode=window_mode)
        return dq, dk, dv, None, None, None, None


class _GistAttentionVarlen(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, r, W, cu_seqlens, sinks, window_mode):
        q = q if _b._q_strided(q) else q.contiguous()      # a [T, Hq, D] tensor passed as its [Hq, T, D] view stays
        k, v = k.contiguous(), v.contiguous()
        cu = [int(x) for x in cu_seqlens]
        out, lse = _b.attn_fwd_varlen(q, k, v, r, W, cu, sinks=sinks, window_mode=window_mode)
        ctx.save_for_backward(q, k, v, out, lse)
        ctx.mask = (int(r), int(W), cu, int(sinks), int(window_mode))
        return out

    @staticmethod
    def backward(ctx, dout):
        q, k, v, out, lse = ctx.saved_tensors
        r, W, cu, sinks, window_mode = ctx.mask
        if not _b._q_strided(q):
            dout = dout.contiguous()
        dq, dk, dv = _b.attn_bwd_varlen(q, k, v, out, lse, dout, r, W, cu, sinks=sinks, window_mode=window_mode)
        return dq, dk, dv, None, None, None, None, None


def gist_attention(q, k, v, r, W, sinks=0, window_mode=_b.UNIGIST_WINDOW_SLIDING):
    """Differentiable gist-masked causal attention (Sec. 4.1, Eq. 3) on GPU tensors."""
    return _GistAttention.apply(q, k, v, r, W, sinks, window_mode)


def gist_attention_varlen(q, k, v, r, W, cu_seqlens, sinks=0, window_mode=_b.UNIGIST_WINDOW_SLIDING):
    """The same for documents packed along the token axis; cu_seqlens is a host sequence of boundaries."""
    return _GistAttentionVarlen.apply(q, k, v, r, W, cu_seqlens, sinks, window_mode)

"""torch.autograd bindings of the WERSA hot path (argument marshalling only: every step runs in
the HIP kernels behind the C ABI).

    out = wersa_attention(q, k, v, omega_rf, sigma, gate_w, gate_b, scale_w, L)
    y = wersa_attention_block(x, wq, wk, wv, wo, H, omega_rf, sigma, gate_w, gate_b, scale_w, L)

q, k, v: (B, H, n, d) with a shared layout (any strides, last dimension contiguous); gradients
flow to q, k, v, sigma, gate_w, gate_b, scale_w (omega_rf is a fixed random matrix) and, for the
block, to x and the four weight matrices (float32 gradients cast to the weights' dtype).
"""
import torch

from . import binding


class _WersaAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, omega_rf, sigma, gate_w, gate_b, scale_w, L, eps, bw_floor):
        out, saved = binding.wersa_forward(q, k, v, omega_rf, sigma, gate_w, gate_b, scale_w, L, eps=eps,
                                           bw_floor=bw_floor)
        ctx.save_for_backward(q, k, v, omega_rf, sigma, gate_w, gate_b, scale_w, out, saved)
        ctx.cfg = (L, eps, bw_floor)
        return out

    @staticmethod
    def backward(ctx, dout):
        q, k, v, omega_rf, sigma, gate_w, gate_b, scale_w, out, saved = ctx.saved_tensors
        L, eps, bw_floor = ctx.cfg
        if dout.stride() != q.stride():
            dout = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device).copy_(dout)
        g = binding.wersa_backward(q, k, v, omega_rf, sigma, gate_w, gate_b, scale_w, out, dout, saved, L,
                                   eps=eps, bw_floor=bw_floor)
        return (g["dq"], g["dk"], g["dv"], None, g["dsigma"], g["dgate_w"], g["dgate_b"], g["dscale_w"],
                None, None, None)


def wersa_attention(q, k, v, omega_rf, sigma, gate_w, gate_b, scale_w, L, eps=1e-6, bw_floor=1e-6):
    return _WersaAttention.apply(q, k, v, omega_rf, sigma, gate_w, gate_b, scale_w, L, eps, bw_floor)


class _WersaBlock(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, wq, wk, wv, wo, H, omega_rf, sigma, gate_w, gate_b, scale_w, L, eps, bw_floor):
        y, saved = binding.wersa_block_forward(x, wq, wk, wv, wo, H, omega_rf, sigma, gate_w, gate_b, scale_w, L,
                                               eps=eps, bw_floor=bw_floor)
        ctx.save_for_backward(x, wq, wk, wv, wo, omega_rf, sigma, gate_w, gate_b, scale_w, saved)
        ctx.cfg = (H, L, eps, bw_floor)
        return y

    @staticmethod
    def backward(ctx, dy):
        x, wq, wk, wv, wo, omega_rf, sigma, gate_w, gate_b, scale_w, saved = ctx.saved_tensors
        H, L, eps, bw_floor = ctx.cfg
        g = binding.wersa_block_backward(x, wq, wk, wv, wo, H, omega_rf, sigma, gate_w, gate_b, scale_w,
                                         dy.contiguous(), saved, L, eps=eps, bw_floor=bw_floor)
        cast = lambda t: t.to(wq.dtype)
        return (g["dx"], cast(g["dwq"]), cast(g["dwk"]), cast(g["dwv"]), cast(g["dwo"]), None, None, g["dsigma"],
                g["dgate_w"], g["dgate_b"], g["dscale_w"], None, None, None)


def wersa_attention_block(x, wq, wk, wv, wo, H, omega_rf, sigma, gate_w, gate_b, scale_w, L, eps=1e-6,
                          bw_floor=1e-6):
    return _WersaBlock.apply(x, wq, wk, wv, wo, H, omega_rf, sigma, gate_w, gate_b, scale_w, L, eps, bw_floor)

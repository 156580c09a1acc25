"""Oracle of the backward pass through a span of frozen blocks (test infrastructure).

Section 2.2 ("Distributed fine-tuning"): a server backpropagates through the blocks it holds and
returns the gradient with respect to its input activations; server-side parameters get no gradient.
The paper fixes no arithmetic for it.  Readings taken here:

 - the derivative is that of the forward pass as computed, evaluated at the tensors the forward pass
   produced, with every rounding and every int8 quantization of an ACTIVATION treated as the identity
   (straight-through);
 - a linear is y = x Wd^T + bias with Wd = fp16(Wq * (s_w / 127)), the weights dequantized from int8
   (the same matrix the forward pass applies to outlier columns; there is no other copy of the
   weights), so dx = dy Wd for all columns;
 - LayerNorm, the ALiBi causal softmax attention, tanh-GeLU and the residual sums are differentiated
   exactly, in fp64; GeLU's derivative is taken at the unrounded sum the forward pass fed to GeLU;
 - gradients are fp16 tensors where the backward pass, fused like the forward pass, stores one:
   the gradient of the GeLU input, of x1 (block input plus attention branch), of the attention
   context, of the fused query/key/value tensor and of the block input.  Everything between two such
   points is fp64.

Plain numpy, fp64; the forward tensors come from the C oracle's traced step.
"""
import numpy as np

from . import oracle as O

__all__ = ["dequantized_weight", "linear_pre_activation", "gelu_grad", "layernorm_backward",
           "attention_backward", "block_backward", "span_backward"]

_C0 = 0.7978845608028654     # sqrt(2 / pi)
_C1 = 0.044715


def _r16(a, on=True):
    """fp64 -> fp16 -> fp64 (one rounding to nearest even), or the identity."""
    return np.asarray(a, np.float64).astype(np.float16).astype(np.float64) if on else np.asarray(a, np.float64)


def dequantized_weight(wq, sw):
    """Wd[N,K] as fp64: the fp32 product code * (s_w / 127) rounded to fp16."""
    scale = (np.asarray(sw, np.float32) / np.float32(127.0)).astype(np.float32)
    prod = np.asarray(wq, np.int8).astype(np.float32) * scale[:, None]      # fp32 product
    return prod.astype(np.float16).astype(np.float64)


def linear_pre_activation(X, wq, sw, bias, theta):
    """fp64 [M,N]: what the mixed int8/fp16 linear sums before its fused tail and its fp16 rounding
    (int32 accumulator times the two scales, plus the outlier columns times Wd, plus the bias)."""
    _, dbg = O.linear(X, wq, sw, bias, theta, want_debug=True)
    sx = (dbg["sx"] / np.float32(127.0)).astype(np.float32).astype(np.float64)
    swd = (np.asarray(sw, np.float32) / np.float32(127.0)).astype(np.float32).astype(np.float64)
    pre = dbg["acc"].astype(np.float64) * sx[:, None] * swd[None, :]
    cols = np.flatnonzero(dbg["mask"])
    if cols.size:
        Wd = dequantized_weight(wq, sw)
        pre = pre + np.asarray(X, np.float16).astype(np.float64)[:, cols] @ Wd[:, cols].T
    return pre + np.asarray(bias, np.float16).astype(np.float64)[None, :]


def gelu_grad(p):
    """d/dp of 0.5 p (1 + tanh(c0 (p + c1 p^3)))."""
    p = np.asarray(p, np.float64)
    t = np.tanh(_C0 * (p + _C1 * p ** 3))
    return 0.5 * (1.0 + t) + 0.5 * p * (1.0 - t * t) * _C0 * (1.0 + 3.0 * _C1 * p * p)


def layernorm_backward(dy, x, g, eps):
    """Gradient w.r.t. x of y = (x - mean) / sqrt(var + eps) * g + b, rows independently (biased variance)."""
    dy, x, g = (np.asarray(a, np.float64) for a in (dy, x, g))
    mu = x.mean(axis=1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=1, keepdims=True)
    inv = 1.0 / np.sqrt(var + eps)
    xh = (x - mu) * inv
    dxh = dy * g[None, :]
    return inv * (dxh - dxh.mean(axis=1, keepdims=True) - xh * (dxh * xh).mean(axis=1, keepdims=True))


def attention_backward(dctx, qkv, nh, slopes):
    """One sequence of T tokens attending to itself (no earlier cache).  dctx [T,H]; qkv [T,3H] with
    column h*3d + p*d + j (p = 0 query, 1 key, 2 value).  Returns dqkv [T,3H] in the same layout."""
    dctx, qkv = np.asarray(dctx, np.float64), np.asarray(qkv, np.float64)
    T, H3 = qkv.shape
    H = H3 // 3
    d = H // nh
    out = np.zeros((T, H3))
    pos = np.arange(T)
    dist = pos[:, None] - pos[None, :]                     # i - j
    causal = dist >= 0
    for h in range(nh):
        q = qkv[:, h * 3 * d: h * 3 * d + d]
        k = qkv[:, h * 3 * d + d: h * 3 * d + 2 * d]
        v = qkv[:, h * 3 * d + 2 * d: h * 3 * d + 3 * d]
        z = q @ k.T / np.sqrt(float(d)) - slopes[h] * dist
        z = np.where(causal, z, -np.inf)
        z = z - z.max(axis=1, keepdims=True)
        P = np.exp(z)
        P = P / P.sum(axis=1, keepdims=True)
        dO = dctx[:, h * d: (h + 1) * d]
        dP = dO @ v.T
        dS = P * (dP - (P * dP).sum(axis=1, keepdims=True))
        out[:, h * 3 * d: h * 3 * d + d] = dS @ k / np.sqrt(float(d))
        out[:, h * 3 * d + d: h * 3 * d + 2 * d] = dS.T @ q / np.sqrt(float(d))
        out[:, h * 3 * d + 2 * d: h * 3 * d + 3 * d] = P.T @ dO
    return out


def block_backward(Wd, ln1_g, ln2_g, saved, dy, B, T, nh, eps, slopes, round16=True):
    """Wd: the four dequantized weights (qkv, dense, up, down) as fp64.  saved: x [M,H] block input,
    qkv [M,3H], x1 [M,H], pre [M,F] (the sum fed to GeLU).  dy [M,H] -> gradient w.r.t. x."""
    r = lambda a: _r16(a, round16)
    dy = np.asarray(dy, np.float64)
    x, qkv, x1, pre = (np.asarray(saved[k], np.float64) for k in ("x", "qkv", "x1", "pre"))
    H = x.shape[1]
    # x2 = x1 + down(gelu(pre)),  pre = up(LN2(x1))
    dpre = r((dy @ Wd[3]) * gelu_grad(pre))
    dx1 = r(dy + layernorm_backward(dpre @ Wd[2], x1, ln2_g, eps))
    # x1 = x + dense(ctx),  ctx = attention(qkv),  qkv = Lin(LN1(x))
    dctx = r(dx1 @ Wd[1])
    dqkv = np.empty((B * T, 3 * H))
    for s in range(B):
        rows = slice(s * T, (s + 1) * T)
        dqkv[rows] = attention_backward(dctx[rows], qkv[rows], nh, slopes)
    dqkv = r(dqkv)
    return r(dx1 + layernorm_backward(dqkv @ Wd[0], x, ln1_g, eps))


def span_backward(span, params, X, dY):
    """span: oracle Span with params (the list of block parameter dicts) loaded.  X, dY: [B,T,H] fp16.
    Runs the traced forward pass on fresh sessions, then the blocks in reverse.  Returns (Y, dX) fp16."""
    X = np.ascontiguousarray(X, np.float16)
    B, T, H = X.shape
    M = B * T
    sessions = [span.open_session(T) for _ in range(B)]
    try:
        Y, taps = span.step(sessions, X, trace=True)
    finally:
        for s in sessions:
            s.close()
    slopes = O.alibi_slopes(span.nh)
    g = np.asarray(dY, np.float16).astype(np.float64).reshape(M, H)
    for b in range(span.NB - 1, -1, -1):
        p = params[b]
        w = [span.get_weight(b, i) for i in range(4)]
        Wd = [dequantized_weight(wq, sw) for wq, sw in w]
        pre = linear_pre_activation(taps["u"][b], w[2][0], w[2][1], p["b_up"], span.theta)
        x_in = X.reshape(M, H) if b == 0 else taps["x2"][b - 1]
        saved = dict(x=x_in.astype(np.float64), qkv=taps["qkv"][b].astype(np.float64),
                     x1=taps["x1"][b].astype(np.float64), pre=pre)
        g = block_backward(Wd, np.asarray(p["ln1_g"], np.float16).astype(np.float64),
                           np.asarray(p["ln2_g"], np.float16).astype(np.float64),
                           saved, g, B, T, span.nh, span.eps, slopes)
    return Y, g.astype(np.float16).reshape(B, T, H)

"""Velocity / noise network of the sampling loop, fp64 NumPy (test infrastructure only).

The paper evaluates a pretrained backbone at every step (the drift of Eq. 12
needs v_theta or the score); trained weights are not available, so the
workload is a randomly initialised patch-2 diffusion transformer with adaLN
conditioning -- the public DiT block structure -- in three variants:
  "adaln": conditioning vector only;
  "cross": an extra cross-attention sub-block over projected context tokens;
  "joint": context tokens are projected to the model width and appended to the
           image tokens, the whole sequence runs through every block and the
           image tokens are read out;
  "mmdit": as "joint", but image and context tokens keep separate streams with
           their own modulation, projection and MLP weights in every block and
           meet only in the joint attention, whose queries and keys are
           RMS-normalised per head with a learnt per-channel scale (the
           public dual-stream block of the flow-model family the paper trains).
All arithmetic is fp64; the weights passed in are already rounded to bf16 by
the input generator, so only activation rounding separates this from a bf16
implementation.  **Parity unpinned** as a whole (there is no reference
implementation of this synthetic network); every building block is pinned in
the tests against PyTorch CPU fp64 library routines (layer_norm, gelu(tanh),
scaled_dot_product_attention, linear) and against structural invariants.
"""
import math
import numpy as np


def silu(x):
    return x / (1.0 + np.exp(-x))


def gelu_tanh(x):
    return 0.5 * x * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (x + 0.044715 * x ** 3)))


def layer_norm(x, eps=1e-6):
    """LayerNorm over the last axis, no affine, biased variance."""
    mu = np.mean(x, axis=-1, keepdims=True)
    var = np.mean((x - mu) ** 2, axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps)


def rms_norm(x, g, eps=1e-6):
    """x / sqrt(mean(x^2) + eps) * g over the last axis."""
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * np.asarray(g, dtype=np.float64)


def linear(x, w, b):
    """y = x W^T + b with W stored [out, in]."""
    return x @ np.asarray(w, dtype=np.float64).T + np.asarray(b, dtype=np.float64)


def timestep_embedding(t_in, dim=256, max_period=10000.0):
    """Sinusoidal embedding: [cos(t f_i), sin(t f_i)], f_i = max_period^(-i/half)."""
    half = dim // 2
    f = np.exp(-math.log(max_period) * np.arange(half, dtype=np.float64) / half)
    a = float(t_in) * f
    return np.concatenate([np.cos(a), np.sin(a)])


def patchify(x, C, H, W):
    """[M, C*H*W] -> [M, (H/2)(W/2), 4C]; patch vector index = c*4 + dy*2 + dx."""
    M = x.shape[0]
    v = x.reshape(M, C, H // 2, 2, W // 2, 2)          # m c py dy px dx
    v = v.transpose(0, 2, 4, 1, 3, 5)                   # m py px c dy dx
    return v.reshape(M, (H // 2) * (W // 2), 4 * C)


def unpatchify(tok, C, H, W):
    """Inverse of patchify: [M, L_i, 4C] -> [M, C*H*W]."""
    M = tok.shape[0]
    v = tok.reshape(M, H // 2, W // 2, C, 2, 2)         # m py px c dy dx
    v = v.transpose(0, 3, 1, 4, 2, 5)                   # m c py dy px dx
    return v.reshape(M, C * H * W)


def attention(q, k, v, heads):
    """Multi-head softmax attention. q [M, Lq, D], k, v [M, Lk, D]; head h owns
    columns h*hd .. (h+1)*hd; logits scaled by 1/sqrt(hd)."""
    M, Lq, D = q.shape
    Lk = k.shape[1]
    hd = D // heads
    qh = q.reshape(M, Lq, heads, hd).transpose(0, 2, 1, 3)
    kh = k.reshape(M, Lk, heads, hd).transpose(0, 2, 1, 3)
    vh = v.reshape(M, Lk, heads, hd).transpose(0, 2, 1, 3)
    s = qh @ kh.transpose(0, 1, 3, 2) / math.sqrt(hd)
    s = s - np.max(s, axis=-1, keepdims=True)
    p = np.exp(s)
    p = p / np.sum(p, axis=-1, keepdims=True)
    o = p @ vh
    return o.transpose(0, 2, 1, 3).reshape(M, Lq, D)


def conditioning(wts, t_in, y):
    """c = MLP(sincos(t)) + y : the adaLN conditioning vector of one prompt."""
    e = timestep_embedding(t_in)
    h = silu(linear(e, wts["t_w1"], wts["t_b1"]))
    return linear(h, wts["t_w2"], wts["t_b2"]) + np.asarray(y, dtype=np.float64)


def _mmdit_blocks(wts, cfg, hx, hc, sc):
    """Dual-stream blocks: hx [M, Li, D] image tokens, hc [M, Lc, D] context tokens."""
    heads, D = cfg["heads"], cfg["D"]
    hd = D // heads
    Li = hx.shape[1]
    qk_norm = cfg.get("qk_norm", True)
    for blk in wts["blocks"]:
        streams = []
        for h, pre in ((hx, ""), (hc, "c_")):
            mod = np.split(linear(sc, blk[pre + "mod_w"], blk[pre + "mod_b"]), 6)
            a = layer_norm(h) * (1.0 + mod[1]) + mod[0]
            q, k, v = np.split(linear(a, blk[pre + "qkv_w"], blk[pre + "qkv_b"]), 3, axis=-1)
            if qk_norm:
                shp = q.shape
                q = rms_norm(q.reshape(shp[:-1] + (heads, hd)), blk[pre + "qn_g"]).reshape(shp)
                k = rms_norm(k.reshape(shp[:-1] + (heads, hd)), blk[pre + "kn_g"]).reshape(shp)
            streams.append((mod, q, k, v))
        q = np.concatenate([streams[0][1], streams[1][1]], axis=1)       # image tokens first
        k = np.concatenate([streams[0][2], streams[1][2]], axis=1)
        v = np.concatenate([streams[0][3], streams[1][3]], axis=1)
        att = attention(q, k, v, heads)
        out = []
        for (h, pre), (mod, _, _, _), a in zip(((hx, ""), (hc, "c_")), streams, (att[:, :Li], att[:, Li:])):
            h = h + mod[2] * linear(a, blk[pre + "o_w"], blk[pre + "o_b"])
            m = layer_norm(h) * (1.0 + mod[4]) + mod[3]
            h = h + mod[5] * linear(gelu_tanh(linear(m, blk[pre + "fc1_w"], blk[pre + "fc1_b"])),
                                    blk[pre + "fc2_w"], blk[pre + "fc2_b"])
            out.append(h)
        hx, hc = out
    return hx


def forward(wts, cfg, x, t_in, y, ctx=None):
    """Network output u for M trajectories of ONE prompt.

    x [M, C*H*W] fp64, t_in scalar network time, y [D] prompt vector,
    ctx [L_c, D_c] context tokens (cross / joint / mmdit variants).  Returns [M, C*H*W]."""
    C, H, W, D, heads = cfg["C"], cfg["H"], cfg["W"], cfg["D"], cfg["heads"]
    kind = cfg["kind"]
    x = np.asarray(x, dtype=np.float64)
    M = x.shape[0]
    Li = (H // 2) * (W // 2)
    h = linear(patchify(x, C, H, W), wts["pe_w"], wts["pe_b"]) + np.asarray(wts["pos"], np.float64)
    sc = silu(conditioning(wts, t_in, y))
    if kind == "mmdit":
        hc = linear(np.asarray(ctx, np.float64), wts["ctx_w"], wts["ctx_b"])
        h = _mmdit_blocks(wts, cfg, h, np.broadcast_to(hc, (M,) + hc.shape), sc)
    else:
        if kind == "joint":
            hc = linear(np.asarray(ctx, np.float64), wts["ctx_w"], wts["ctx_b"])
            h = np.concatenate([h, np.broadcast_to(hc, (M,) + hc.shape)], axis=1)
        for blk in wts["blocks"]:
            sh1, sc1, g1, sh2, sc2, g2 = np.split(linear(sc, blk["mod_w"], blk["mod_b"]), 6)
            a = layer_norm(h) * (1.0 + sc1) + sh1
            q, k, v = np.split(linear(a, blk["qkv_w"], blk["qkv_b"]), 3, axis=-1)
            h = h + g1 * linear(attention(q, k, v, heads), blk["o_w"], blk["o_b"])
            if kind == "cross":
                cq = linear(layer_norm(h), blk["cq_w"], blk["cq_b"])
                ck, cv = np.split(linear(np.asarray(ctx, np.float64), blk["ckv_w"], blk["ckv_b"]), 2, axis=-1)
                ck = np.broadcast_to(ck, (M,) + ck.shape)
                cv = np.broadcast_to(cv, (M,) + cv.shape)
                h = h + linear(attention(cq, ck, cv, heads), blk["co_w"], blk["co_b"])
            m = layer_norm(h) * (1.0 + sc2) + sh2
            h = h + g2 * linear(gelu_tanh(linear(m, blk["fc1_w"], blk["fc1_b"])), blk["fc2_w"], blk["fc2_b"])
    shf, scf = np.split(linear(sc, wts["fmod_w"], wts["fmod_b"]), 2)
    o = layer_norm(h[:, :Li]) * (1.0 + scf) + shf
    return unpatchify(linear(o, wts["f_w"], wts["f_b"]), C, H, W)

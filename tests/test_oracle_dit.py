"""Pins for oracle/dit.py (CPU only): each building block against PyTorch CPU fp64
library routines and structural invariants; the whole forward against a forward
assembled from those library routines."""
import math
import numpy as np
import torch
import torch.nn.functional as F

from oracle import dit
from paper_2512_15347_amd import workloads

T64 = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))


def test_elementwise_blocks_vs_torch():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 96)) * 3
    np.testing.assert_allclose(dit.silu(x), F.silu(T64(x)).numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(dit.gelu_tanh(x), F.gelu(T64(x), approximate="tanh").numpy(), rtol=1e-12, atol=1e-14)
    ln = dit.layer_norm(x)
    np.testing.assert_allclose(ln, F.layer_norm(T64(x), (96,), eps=1e-6).numpy(), rtol=1e-11, atol=1e-13)
    assert np.max(np.abs(ln.mean(-1))) < 1e-12 and np.max(np.abs(ln.var(-1) - 1)) < 1e-5
    w = rng.standard_normal((7, 96)); b = rng.standard_normal(7)
    np.testing.assert_allclose(dit.linear(x, w, b), F.linear(T64(x), T64(w), T64(b)).numpy(), rtol=1e-12, atol=1e-12)
    # triple loop on a corner
    assert abs(dit.linear(x, w, b)[2, 3] - (sum(x[2, i] * w[3, i] for i in range(96)) + b[3])) < 1e-12


def test_attention_vs_torch_and_invariants():
    rng = np.random.default_rng(1)
    M, Lq, Lk, D, h = 2, 9, 13, 32, 4
    q = rng.standard_normal((M, Lq, D)); k = rng.standard_normal((M, Lk, D)); v = rng.standard_normal((M, Lk, D))
    got = dit.attention(q, k, v, h)
    sp = lambda a, L: T64(a).reshape(M, L, h, D // h).transpose(1, 2)
    want = F.scaled_dot_product_attention(sp(q, Lq), sp(k, Lk), sp(v, Lk)).transpose(1, 2).reshape(M, Lq, D).numpy()
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-13)
    # identical keys -> uniform weights -> the mean of V
    k_same = np.broadcast_to(k[:, :1], k.shape)
    np.testing.assert_allclose(dit.attention(q, k_same, v, h), np.broadcast_to(v.mean(1, keepdims=True), (M, Lq, D)), atol=1e-12)


def test_patchify_roundtrip_and_layout():
    C, H, W = 3, 4, 6
    x = np.arange(2 * C * H * W, dtype=np.float64).reshape(2, C * H * W)
    p = dit.patchify(x, C, H, W)
    assert p.shape == (2, 6, 12)
    np.testing.assert_array_equal(dit.unpatchify(p, C, H, W), x)
    img = x[1].reshape(C, H, W)
    # token (py=1, px=2), entry c=2, dy=1, dx=0
    assert p[1, 1 * 3 + 2, 2 * 4 + 1 * 2 + 0] == img[2, 2 * 1 + 1, 2 * 2 + 0]
    # matches unfold: patch vector index = c*4 + dy*2 + dx
    unf = F.unfold(T64(img)[None], kernel_size=2, stride=2)[0].T.numpy()
    np.testing.assert_array_equal(p[1], unf)


def test_timestep_embedding():
    e = dit.timestep_embedding(0.0)
    np.testing.assert_array_equal(e[:128], 1.0); np.testing.assert_array_equal(e[128:], 0.0)
    e = dit.timestep_embedding(500.0)
    assert abs(e[0] - math.cos(500.0)) < 1e-12 and abs(e[128] - math.sin(500.0)) < 1e-12
    assert abs(e[64] - math.cos(500.0 * 10000 ** -0.5)) < 1e-12
    assert np.allclose(e[:128] ** 2 + e[128:] ** 2, 1.0)


def _torch_forward(w, cfg, x, t_in, y, ctx):
    """The same network assembled from torch library routines only."""
    C, H, W, D, h = cfg["C"], cfg["H"], cfg["W"], cfg["D"], cfg["heads"]
    M = x.shape[0]; Li = cfg["Li"]
    lin = lambda a, wn, bn, d=w: F.linear(a, T64(d[wn]), T64(d[bn]))
    img = T64(x).reshape(M, C, H, W)
    tok = F.unfold(img, kernel_size=2, stride=2).transpose(1, 2)
    hdn = lin(tok, "pe_w", "pe_b") + T64(w["pos"])
    if cfg["kind"] == "joint":
        hdn = torch.cat([hdn, lin(T64(ctx), "ctx_w", "ctx_b").expand(M, -1, -1)], 1)
    half = 128
    f = torch.exp(-math.log(10000.0) * torch.arange(half, dtype=torch.float64) / half)
    emb = torch.cat([torch.cos(t_in * f), torch.sin(t_in * f)])
    c = lin(F.silu(lin(emb, "t_w1", "t_b1")), "t_w2", "t_b2") + T64(y)
    sc = F.silu(c)
    heads = lambda a: a.reshape(M, a.shape[1], h, D // h).transpose(1, 2)
    for blk in w["blocks"]:
        sh1, sc1, g1, sh2, sc2, g2 = lin(sc, "mod_w", "mod_b", blk).chunk(6)
        a = F.layer_norm(hdn, (D,), eps=1e-6) * (1 + sc1) + sh1
        q, k, v = lin(a, "qkv_w", "qkv_b", blk).chunk(3, dim=-1)
        o = F.scaled_dot_product_attention(heads(q), heads(k), heads(v)).transpose(1, 2).reshape(M, -1, D)
        hdn = hdn + g1 * lin(o, "o_w", "o_b", blk)
        if cfg["kind"] == "cross":
            cq = lin(F.layer_norm(hdn, (D,), eps=1e-6), "cq_w", "cq_b", blk)
            ck, cv = lin(T64(ctx), "ckv_w", "ckv_b", blk).expand(M, -1, -1).chunk(2, dim=-1)
            o = F.scaled_dot_product_attention(heads(cq), heads(ck), heads(cv)).transpose(1, 2).reshape(M, -1, D)
            hdn = hdn + lin(o, "co_w", "co_b", blk)
        m = F.layer_norm(hdn, (D,), eps=1e-6) * (1 + sc2) + sh2
        hdn = hdn + g2 * lin(F.gelu(lin(m, "fc1_w", "fc1_b", blk), approximate="tanh"), "fc2_w", "fc2_b", blk)
    shf, scf = lin(sc, "fmod_w", "fmod_b").chunk(2)
    o = F.layer_norm(hdn[:, :Li], (D,), eps=1e-6) * (1 + scf) + shf
    out = lin(o, "f_w", "f_b").transpose(1, 2)
    return F.fold(out, (H, W), kernel_size=2, stride=2).reshape(M, -1).numpy()


def test_forward_all_variants_vs_torch_assembly():
    for name in ("cfg1", "cfg2_small", "cfg3_small"):
        cfg = workloads.get_config(name)
        w = workloads.make_weights(cfg)
        inp = workloads.make_inputs(cfg, w)
        rng = np.random.default_rng(3)
        x = rng.standard_normal((3, cfg["d"]))
        ctx = inp["ctx"][0] if inp["ctx"] is not None else None
        got = dit.forward(w, cfg, x, 700.0, inp["y"][0], ctx)
        want = _torch_forward(w, cfg, x, 700.0, inp["y"][0], ctx)
        assert got.shape == (3, cfg["d"])
        np.testing.assert_allclose(got, want, rtol=1e-9, atol=1e-12)
        assert np.std(got) > 1e-3                      # a live output, not zeros


def _torch_forward_mmdit(w, cfg, x, t_in, y, ctx):
    """The dual-stream network assembled from torch library routines only."""
    C, H, W, D, h = cfg["C"], cfg["H"], cfg["W"], cfg["D"], cfg["heads"]
    M = x.shape[0]; Li = cfg["Li"]; hd = D // h
    lin = lambda a, wn, bn, d=w: F.linear(a, T64(d[wn]), T64(d[bn]))
    img = T64(x).reshape(M, C, H, W)
    hx = lin(F.unfold(img, kernel_size=2, stride=2).transpose(1, 2), "pe_w", "pe_b") + T64(w["pos"])
    hc = lin(T64(ctx), "ctx_w", "ctx_b").expand(M, -1, -1)
    half = 128
    f = torch.exp(-math.log(10000.0) * torch.arange(half, dtype=torch.float64) / half)
    emb = torch.cat([torch.cos(t_in * f), torch.sin(t_in * f)])
    sc = F.silu(lin(F.silu(lin(emb, "t_w1", "t_b1")), "t_w2", "t_b2") + T64(y))
    heads = lambda a: a.reshape(M, a.shape[1], h, hd).transpose(1, 2)
    for blk in w["blocks"]:
        parts = []
        for hs, pre in ((hx, ""), (hc, "c_")):
            mod = lin(sc, pre + "mod_w", pre + "mod_b", blk).chunk(6)
            a = F.layer_norm(hs, (D,), eps=1e-6) * (1 + mod[1]) + mod[0]
            q, k, v = lin(a, pre + "qkv_w", pre + "qkv_b", blk).chunk(3, dim=-1)
            q = F.rms_norm(heads(q), (hd,), T64(blk[pre + "qn_g"]), eps=1e-6)
            k = F.rms_norm(heads(k), (hd,), T64(blk[pre + "kn_g"]), eps=1e-6)
            parts.append((mod, q, k, heads(v)))
        q = torch.cat([parts[0][1], parts[1][1]], 2); k = torch.cat([parts[0][2], parts[1][2]], 2)
        v = torch.cat([parts[0][3], parts[1][3]], 2)
        o = F.scaled_dot_product_attention(q, k, v).transpose(1, 2).reshape(M, -1, D)
        new = []
        for (hs, pre), (mod, _, _, _), a in zip(((hx, ""), (hc, "c_")), parts, (o[:, :Li], o[:, Li:])):
            hs = hs + mod[2] * lin(a, pre + "o_w", pre + "o_b", blk)
            m = F.layer_norm(hs, (D,), eps=1e-6) * (1 + mod[4]) + mod[3]
            hs = hs + mod[5] * lin(F.gelu(lin(m, pre + "fc1_w", pre + "fc1_b", blk), approximate="tanh"),
                                   pre + "fc2_w", pre + "fc2_b", blk)
            new.append(hs)
        hx, hc = new
    shf, scf = lin(sc, "fmod_w", "fmod_b").chunk(2)
    o = F.layer_norm(hx, (D,), eps=1e-6) * (1 + scf) + shf
    return F.fold(lin(o, "f_w", "f_b").transpose(1, 2), (H, W), kernel_size=2, stride=2).reshape(M, -1).numpy()


def test_rms_norm_vs_torch():
    rng = np.random.default_rng(8)
    x = rng.standard_normal((3, 5, 4, 32)); g = 1.0 + 0.1 * rng.standard_normal(32)
    want = F.rms_norm(T64(x), (32,), T64(g), eps=1e-6).numpy()
    np.testing.assert_allclose(dit.rms_norm(x, g), want, rtol=1e-12, atol=1e-14)
    # unit scale: every row has mean square 1 (up to eps)
    assert np.allclose(np.mean(dit.rms_norm(x, np.ones(32)) ** 2, axis=-1), 1.0, atol=1e-5)


def test_dual_stream_forward_vs_torch_assembly_and_joint_special_case():
    cfg = workloads.get_config("cfg3_mmdit_small")
    w = workloads.make_weights(cfg); inp = workloads.make_inputs(cfg, w)
    rng = np.random.default_rng(5)
    x = rng.standard_normal((3, cfg["d"]))
    got = dit.forward(w, cfg, x, 650.0, inp["y"][1], inp["ctx"][1])
    want = _torch_forward_mmdit(w, cfg, x, 650.0, inp["y"][1], inp["ctx"][1])
    np.testing.assert_allclose(got, want, rtol=1e-9, atol=1e-12)
    assert np.std(got) > 1e-3
    # the norm scales are live inputs
    w2 = {**w, "blocks": [dict(b) for b in w["blocks"]]}
    w2["blocks"][0]["c_kn_g"] = w2["blocks"][0]["c_kn_g"] * 1.5
    assert np.max(np.abs(dit.forward(w2, cfg, x, 650.0, inp["y"][1], inp["ctx"][1]) - got)) > 1e-7
    # special case that reduces to the single-stream network: both streams share one set of weights and the
    # query / key norms are switched off
    cj = workloads.get_config("cfg3_small")
    wj = workloads.make_weights(cj); ij = workloads.make_inputs(cj, wj)
    wm = {**wj, "blocks": [{**b, **{"c_" + k: v for k, v in b.items()}} for b in wj["blocks"]]}
    cm = {**cj, "kind": "mmdit", "qk_norm": False}
    xj = rng.standard_normal((2, cj["d"]))
    np.testing.assert_allclose(dit.forward(wm, cm, xj, 400.0, ij["y"][0], ij["ctx"][0]),
                               dit.forward(wj, cj, xj, 400.0, ij["y"][0], ij["ctx"][0]), rtol=1e-10, atol=1e-13)


def test_forward_trajectories_are_independent_and_context_matters():
    cfg = workloads.get_config("cfg3_small")
    w = workloads.make_weights(cfg); inp = workloads.make_inputs(cfg, w)
    rng = np.random.default_rng(4)
    x = rng.standard_normal((4, cfg["d"]))
    full = dit.forward(w, cfg, x, 300.0, inp["y"][0], inp["ctx"][0])
    one = dit.forward(w, cfg, x[2:3], 300.0, inp["y"][0], inp["ctx"][0])
    np.testing.assert_allclose(full[2:3], one, rtol=1e-12, atol=1e-14)
    other = dit.forward(w, cfg, x[2:3], 300.0, inp["y"][0], inp["ctx"][0] * 0.5)
    assert np.max(np.abs(other - one)) > 1e-6
    other_t = dit.forward(w, cfg, x[2:3], 900.0, inp["y"][0], inp["ctx"][0])
    assert np.max(np.abs(other_t - one)) > 1e-6


def test_weights_are_bf16_representable():
    cfg = workloads.get_config("cfg1")
    w = workloads.make_weights(cfg)
    for a in [w["pe_w"], w["pos"], w["blocks"][1]["qkv_w"]]:
        assert np.all((a.view(np.uint32) & 0xFFFF) == 0)
        np.testing.assert_array_equal(a, torch.tensor(a).to(torch.bfloat16).float().numpy())
    raw = np.random.default_rng(0).standard_normal(1000, dtype=np.float32)
    np.testing.assert_array_equal(workloads.bf16_round(raw), torch.tensor(raw).to(torch.bfloat16).float().numpy())

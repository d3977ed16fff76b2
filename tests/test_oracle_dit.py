"""Pins of the DiT oracle's pieces against brute force, special cases and
PyTorch's CPU library routines (no GPU, no HIP library)."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import speca_inputs as si
from oracle import dit


def test_attention_vs_brute_force_loops():
    rng = np.random.default_rng(0)
    r, H, T, hd = 2, 3, 5, 4
    q, k, v = (rng.standard_normal((r, H, T, hd)) for _ in range(3))
    got = dit.attention(q, k, v)
    for a in range(r):
        for h in range(H):
            for i in range(T):
                w = [math.exp(sum(q[a, h, i, d] * k[a, h, j, d] for d in range(hd)) / math.sqrt(hd)) for j in range(T)]
                z = sum(w)
                for d in range(hd):
                    exp = sum(w[j] * v[a, h, j, d] for j in range(T)) / z
                    assert got[a, h, i, d] == pytest.approx(exp, rel=1e-12, abs=1e-12)


def test_attention_special_cases_and_library():
    rng = np.random.default_rng(1)
    q, v = rng.standard_normal((1, 2, 6, 8)), rng.standard_normal((1, 2, 6, 8))
    # identical keys -> uniform weights -> mean of V
    k = np.repeat(rng.standard_normal((1, 2, 1, 8)), 6, axis=2)
    np.testing.assert_allclose(dit.attention(q, k, v), np.repeat(v.mean(axis=2, keepdims=True), 6, axis=2), rtol=1e-12)
    # library routine
    k = rng.standard_normal((1, 2, 6, 8))
    ref = F.scaled_dot_product_attention(torch.tensor(q), torch.tensor(k), torch.tensor(v)).numpy()
    np.testing.assert_allclose(dit.attention(q, k, v), ref, rtol=1e-10, atol=1e-12)
    # not symmetric in q/k: a transposed operand fails this
    assert np.max(np.abs(dit.attention(k, q, v) - ref)) > 1e-3


def test_linear_vs_triple_loop():
    rng = np.random.default_rng(2)
    a, w, b = rng.standard_normal((3, 4)), rng.standard_normal((5, 4)), rng.standard_normal(5)
    got = dit.linear(a, w, b)
    for i in range(3):
        for n in range(5):
            assert got[i, n] == pytest.approx(sum(a[i, kk] * w[n, kk] for kk in range(4)) + b[n], rel=1e-13)


def test_pointwise_vs_library():
    x = torch.linspace(-6, 6, 101, dtype=torch.float64)
    np.testing.assert_allclose(dit.gelu_tanh(x.numpy()), F.gelu(x, approximate="tanh").numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(dit.silu(x.numpy()), F.silu(x).numpy(), rtol=1e-12, atol=1e-14)
    # tanh form stays within 1e-3 of the erf definition; exact limits
    assert np.max(np.abs(dit.gelu_tanh(x.numpy()) - F.gelu(x).numpy())) < 1e-3
    assert dit.gelu_tanh(np.array([0.0]))[0] == 0.0 and dit.gelu_tanh(np.array([30.0]))[0] == 30.0
    a = torch.randn(4, 7, 32, dtype=torch.float64, generator=torch.Generator().manual_seed(0))
    np.testing.assert_allclose(dit.layer_norm(a.numpy()), F.layer_norm(a, (32,), eps=1e-6).numpy(), rtol=1e-10, atol=1e-12)


def test_timestep_sinusoid():
    e = dit.timestep_sinusoid(np.array([0.0, 3.0]), 8)
    np.testing.assert_array_equal(e[0], [1, 1, 1, 1, 0, 0, 0, 0])
    w = [1.0, 10.0 ** -1, 10.0 ** -2, 10.0 ** -3]
    np.testing.assert_allclose(e[1], [math.cos(3 * x) for x in w] + [math.sin(3 * x) for x in w], rtol=1e-12)


def test_patchify_ordering_vs_conv2d():
    s = si.dit_tiny()
    w = si.make_dit_weights(s, seed=3)
    m = dit.DiTOracle(s, w)
    x = si.make_latents(2, s.in_channels, s.latent_hw, seed=3).astype(np.float64)
    tok = m.patchify(x)
    # explicit indexing
    p, g = s.patch, s.grid
    for (i, j, c, pi, pj) in [(0, 0, 0, 0, 0), (1, 2, 3, 1, 0), (3, 3, 2, 0, 1)]:
        assert tok[1, i * g + j, (c * p + pi) * p + pj] == x[1, c, i * p + pi, j * p + pj]
    np.testing.assert_array_equal(m.unpatchify(tok), x)
    # patch embedding == strided convolution with the weight viewed as [D, C, p, p]
    wp = torch.tensor(w["patch_w"], dtype=torch.float64).reshape(s.hidden, s.in_channels, p, p)
    conv = F.conv2d(torch.tensor(x), wp, torch.tensor(w["patch_b"], dtype=torch.float64), stride=p)
    conv = conv.flatten(2).transpose(1, 2).numpy() + w["pos"][None].astype(np.float64)
    np.testing.assert_allclose(m.embed(x), conv, rtol=1e-10, atol=1e-12)


def _torch_block(s, w, l, h, c):
    """The same adaLN-Zero block assembled from PyTorch library routines."""
    t = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))
    D = s.hidden
    mod = F.linear(F.silu(t(c)), t(w[f"blk{l}.mod_w"]), t(w[f"blk{l}.mod_b"]))
    sa, ca, ga, sm, cm, gm = [a[:, None, :] for a in mod.chunk(6, dim=1)]
    x = t(h)
    xn = F.layer_norm(x, (D,), eps=1e-6) * (1 + ca) + sa
    mha = torch.nn.MultiheadAttention(D, s.heads, batch_first=True, dtype=torch.float64)
    with torch.no_grad():
        mha.in_proj_weight.copy_(t(w[f"blk{l}.qkv_w"])); mha.in_proj_bias.copy_(t(w[f"blk{l}.qkv_b"]))
        mha.out_proj.weight.copy_(t(w[f"blk{l}.proj_w"])); mha.out_proj.bias.copy_(t(w[f"blk{l}.proj_b"]))
        fa = mha(xn, xn, xn, need_weights=False)[0]
        x = x + ga * fa
        xn = F.layer_norm(x, (D,), eps=1e-6) * (1 + cm) + sm
        fm = F.linear(F.gelu(F.linear(xn, t(w[f"blk{l}.fc1_w"]), t(w[f"blk{l}.fc1_b"])), approximate="tanh"),
                      t(w[f"blk{l}.fc2_w"]), t(w[f"blk{l}.fc2_b"]))
        x = x + gm * fm
    return x.numpy(), fa.numpy(), fm.numpy()


def test_block_vs_library_assembly():
    s = si.dit_tiny()
    w = si.make_dit_weights(s, seed=1, std=0.2)          # larger weights so every term matters
    m = dit.DiTOracle(s, w)
    x = si.make_latents(3, s.in_channels, s.latent_hw, seed=1)
    h, c = m.begin(x, 417.0, [1, 2, s.num_classes])
    for l in range(s.depth):
        h2, feats = m.block_real(l, h, c)
        rh, rfa, rfm = _torch_block(s, w, l, h, c)
        np.testing.assert_allclose(feats[0], rfa, rtol=1e-9, atol=1e-11)
        np.testing.assert_allclose(feats[1], rfm, rtol=1e-9, atol=1e-11)
        np.testing.assert_allclose(h2, rh, rtol=1e-9, atol=1e-11)
        # folding the block's own real features reproduces the real hidden state
        np.testing.assert_allclose(m.block_fold(l, h, c, feats), h2, rtol=1e-12, atol=1e-13)
        h = h2


def test_zero_modulation_makes_blocks_identity():
    s = si.dit_tiny()
    w = si.make_dit_weights(s, seed=2)
    for l in range(s.depth):
        w[f"blk{l}.mod_w"] = np.zeros_like(w[f"blk{l}.mod_w"]); w[f"blk{l}.mod_b"] = np.zeros_like(w[f"blk{l}.mod_b"])
    m = dit.DiTOracle(s, w)
    x = si.make_latents(1, s.in_channels, s.latent_hw, seed=2)
    out, feats = m.forward(x, 10.0, [3])
    h, c = m.begin(x, 10.0, [3])
    np.testing.assert_array_equal(out, m.finish(h, c))
    assert len(feats) == m.n_slots == 2 * s.depth and feats[0].shape == (1, s.tokens, s.hidden)


def test_rows_are_independent():
    s = si.dit_tiny()
    m = dit.DiTOracle(s, si.make_dit_weights(s, seed=4))
    x = si.make_latents(3, s.in_channels, s.latent_hw, seed=4)
    out, _ = m.forward(x, 500.0, [0, 1, 2])
    out1, _ = m.forward(x[1:2], 500.0, [1])
    np.testing.assert_allclose(out[1:2], out1, rtol=1e-12, atol=1e-14)


def test_flop_count_matches_paper_table():
    # Table 3: DiT-XL/2 DDIM-50 = 23.74 TFLOPs per trajectory = 0.4748 T per step for
    # the guidance pair; the linear + attention contractions of the DiT-XL/2-shaped
    # model give it from shapes alone (the paper's count adds the small layers).
    m = dit.DiTOracle(si.dit_xl2(), {})
    per_pair = 2 * m.flops_per_row()
    assert per_pair / 1e12 == pytest.approx(23.74 / 50, rel=5e-3)


def _torch_conditioning(s, w, t, labels):
    """c = MLP_t(sinusoid(t)) + y_table[label] from library routines: torch.cos/sin of the angles written
    out frequency by frequency, F.linear, F.silu, F.embedding."""
    T64 = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))
    half = s.freq_dim // 2
    ang = torch.tensor([[float(t) * 10000.0 ** (-j / half) for j in range(half)]] * len(labels), dtype=torch.float64)
    emb = torch.cat([torch.cos(ang), torch.sin(ang)], dim=1)
    temb = F.linear(F.silu(F.linear(emb, T64(w["t_w1"]), T64(w["t_b1"]))), T64(w["t_w2"]), T64(w["t_b2"]))
    return (temb + F.embedding(torch.tensor(list(labels), dtype=torch.long), T64(w["y_table"]))).numpy()


def _torch_final(s, w, h, c):
    """(shift, scale) = chunk(Linear(SiLU(c)), 2); Linear(LN(h)(1+scale)+shift); un-patchify by explicit
    indexing: out[r, ch, i p + pi, j p + pj] = tok[r, i g + j, (ch p + pi) p + pj]."""
    T64 = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))
    D, p, g, C = s.hidden, s.patch, s.grid, s.in_channels
    mod = F.linear(F.silu(T64(c)), T64(w["fmod_w"]), T64(w["fmod_b"]))
    shift, scale = mod[:, None, :D], mod[:, None, D:]
    tok = F.linear(F.layer_norm(T64(h), (D,), eps=1e-6) * (1 + scale) + shift, T64(w["final_w"]), T64(w["final_b"])).numpy()
    out = np.zeros((h.shape[0], C, g * p, g * p))
    for i in range(g):
        for j in range(g):
            for ch in range(C):
                for pi in range(p):
                    for pj in range(p):
                        out[:, ch, i * p + pi, j * p + pj] = tok[:, i * g + j, (ch * p + pi) * p + pj]
    return out


def test_conditioning_vs_library_assembly():
    s = si.dit_tiny()
    w = si.make_dit_weights(s, seed=5, std=0.2)          # every bias and table row matters at this scale
    m = dit.DiTOracle(s, w)
    labels = [0, 3, s.num_classes, 3]                    # includes the null row and a repeated label
    for t in (0.0, 1.0, 417.0, 980.0):
        got = m.conditioning(t, labels)
        np.testing.assert_allclose(got, _torch_conditioning(s, w, t, labels), rtol=1e-10, atol=1e-12)
    # what a plausible mistake changes: dropping a bias, the wrong table row, sin before cos
    c = m.conditioning(417.0, labels)
    assert np.max(np.abs(c[1] - c[3])) == 0.0 and np.max(np.abs(c[0] - c[1])) > 1e-2
    w2 = dict(w); w2["t_b2"] = np.zeros_like(w["t_b2"])
    assert np.max(np.abs(dit.DiTOracle(s, w2).conditioning(417.0, labels) - c)) > 1e-2
    w3 = dict(w); w3["t_w1"] = np.concatenate([w["t_w1"][:, s.freq_dim // 2:], w["t_w1"][:, : s.freq_dim // 2]], axis=1)
    assert np.max(np.abs(dit.DiTOracle(s, w3).conditioning(417.0, labels) - c)) > 1e-2
    # t = 0: the embedding is (1,..,1,0,..,0), so only the cosine half of t_w1 enters
    half = s.freq_dim // 2
    e0 = w["t_w1"][:, :half].astype(np.float64).sum(axis=1) + w["t_b1"]
    c0 = (e0 / (1 + np.exp(-e0))) @ w["t_w2"].astype(np.float64).T + w["t_b2"] + w["y_table"][3]
    np.testing.assert_allclose(m.conditioning(0.0, [3])[0], c0, rtol=1e-10, atol=1e-12)


def test_final_layer_vs_library_assembly():
    s = si.dit_tiny()
    w = si.make_dit_weights(s, seed=6, std=0.2)
    m = dit.DiTOracle(s, w)
    x = si.make_latents(3, s.in_channels, s.latent_hw, seed=6)
    h, c = m.begin(x, 250.0, [1, 2, s.num_classes])
    got = m.final(h, c)
    ref = _torch_final(s, w, h, c)
    assert got.shape == x.shape
    np.testing.assert_allclose(got, ref, rtol=1e-9, atol=1e-11)
    # the (shift, scale) order matters at this weight scale: the swapped split is far from the reference
    D = s.hidden
    w_sw = dict(w)
    w_sw["fmod_w"] = np.concatenate([w["fmod_w"][D:], w["fmod_w"][:D]])
    w_sw["fmod_b"] = np.concatenate([w["fmod_b"][D:], w["fmod_b"][:D]])
    assert np.max(np.abs(dit.DiTOracle(s, w_sw).final(h, c) - ref)) > 1e-2 * np.max(np.abs(ref))
    # zero modulation: a plain LayerNorm + linear layer
    w0 = dict(w); w0["fmod_w"] = np.zeros_like(w["fmod_w"]); w0["fmod_b"] = np.zeros_like(w["fmod_b"])
    tok = F.linear(F.layer_norm(torch.tensor(h), (D,), eps=1e-6), torch.tensor(w["final_w"], dtype=torch.float64),
                   torch.tensor(w["final_b"], dtype=torch.float64)).numpy()
    np.testing.assert_allclose(dit.DiTOracle(s, w0).final(h, c), m.unpatchify(tok), rtol=1e-10, atol=1e-12)
    # forward = begin -> blocks -> final, with nothing else in between
    out, _ = m.forward(x, 250.0, [1, 2, s.num_classes])
    hh = h
    for l in range(s.depth):
        hh, _ = m.block_real(l, hh, c)
    np.testing.assert_allclose(out, _torch_final(s, w, hh, c), rtol=1e-9, atol=1e-11)

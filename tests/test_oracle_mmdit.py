"""Pins of the MMDiT oracle's pieces against closed forms, special cases and PyTorch's CPU
library routines (no GPU, no HIP library)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import speca_inputs as si
from oracle import mmdit, sampler, speca_core as core

T64 = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))


def test_rms_norm_vs_library():
    rng = np.random.default_rng(0)
    x, sc = rng.standard_normal((2, 3, 5, 16)), rng.standard_normal(16)
    np.testing.assert_allclose(mmdit.rms_norm(x, sc), F.rms_norm(T64(x), (16,), T64(sc), eps=1e-6).numpy(), rtol=1e-12)
    assert mmdit.rms_norm(np.full((1, 8), 3.0), np.ones(8))[0, 0] == pytest.approx(1.0, rel=1e-6)


def test_rope_is_complex_rotation_and_relative():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((1, 2, 6, 8))
    ang = rng.uniform(0, 6, size=(6, 4))
    got = mmdit.apply_rope(x, np.cos(ang), np.sin(ang))
    z = (x[..., 0::2] + 1j * x[..., 1::2]) * np.exp(1j * ang)
    np.testing.assert_allclose(got[..., 0::2], z.real, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(got[..., 1::2], z.imag, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(np.linalg.norm(got, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-12)   # a rotation
    # zero angle = identity (text tokens sit at the origin)
    np.testing.assert_array_equal(mmdit.apply_rope(x, np.ones((6, 4)), np.zeros((6, 4))), x)
    # q.k after rotation depends only on the position difference
    om = 1.0 / 100.0 ** (np.arange(4) / 4)
    q, k = rng.standard_normal(8), rng.standard_normal(8)
    def dot(pq, pk):
        rq = mmdit.apply_rope(q[None, None, None], np.cos(pq * om)[None], np.sin(pq * om)[None])
        rk = mmdit.apply_rope(k[None, None, None], np.cos(pk * om)[None], np.sin(pk * om)[None])
        return float((rq * rk).sum())
    assert dot(3, 1) == pytest.approx(dot(10, 8), rel=1e-12) and dot(3, 1) != pytest.approx(dot(3, 2), rel=1e-3)


def test_rope_tables():
    s = si.mmdit_tiny_video()
    c, sn = si.rope_tables(s)
    assert c.shape == (s.tokens, s.head_dim // 2)
    assert np.all(c[: s.txt_tokens] == 1) and np.all(sn[: s.txt_tokens] == 0)
    gh, gw = s.latent_h // s.patch, s.latent_w // s.patch
    tok = s.txt_tokens + (2 * gh + 1) * gw + 3                          # (f, i, j) = (2, 1, 3)
    a0, a1 = s.rope_axes[0] // 2, (s.rope_axes[0] + s.rope_axes[1]) // 2
    assert c[tok, 0] == pytest.approx(np.cos(2.0)) and c[tok, a0] == pytest.approx(np.cos(1.0)) and sn[tok, a1] == pytest.approx(np.sin(3.0))


def test_patchify_vs_conv3d_and_roundtrip():
    s = si.mmdit_tiny_video()
    w = si.make_mmdit_weights(s, 2)
    m = mmdit.MMDiTOracle(s, w)
    x = si.make_video_latents(2, s, 2).astype(np.float64)
    np.testing.assert_array_equal(m.unpatchify(m.patchify(x)), x)
    p = s.patch
    wp = T64(w["img_in_w"]).reshape(s.hidden, s.in_channels, 1, p, p)
    conv = F.conv3d(T64(x), wp, T64(w["img_in_b"]), stride=(1, p, p)).flatten(2).transpose(1, 2).numpy()
    txt, vec = si.make_text(2, s, 2)
    h, _ = m.begin(x, 100.0, (txt, vec))
    np.testing.assert_allclose(h[:, s.txt_tokens:], conv, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(h[:, : s.txt_tokens], F.linear(T64(txt), T64(w["txt_in_w"]), T64(w["txt_in_b"])).numpy(), rtol=1e-10, atol=1e-12)


def _torch_attention(s, w, q, k, v, qn, kn):
    """Joint attention assembled from library routines: per-token RMS scales, rotation as a
    complex product, scaled_dot_product_attention."""
    r, T, D = q.shape
    H, hd = s.heads, s.head_dim
    def prep(a, sc):
        a = T64(a).reshape(r, T, H, hd).transpose(1, 2)
        a = a * torch.rsqrt((a * a).mean(-1, keepdim=True) + 1e-6) * T64(sc)[None, None]
        z = torch.view_as_complex(a.reshape(r, H, T, hd // 2, 2).contiguous())
        z = z * torch.complex(T64(w["rope_cos"]), T64(w["rope_sin"]))
        return torch.view_as_real(z).reshape(r, H, T, hd)
    o = F.scaled_dot_product_attention(prep(q, qn), prep(k, kn), T64(v).reshape(r, T, H, hd).transpose(1, 2))
    return o.transpose(1, 2).reshape(r, T, D).numpy()


def test_blocks_vs_library_assembly():
    s = si.mmdit_tiny()
    w = si.make_mmdit_weights(s, 1, std=0.15)
    m = mmdit.MMDiTOracle(s, w)
    x = si.make_video_latents(2, s, 1); txt, vec = si.make_text(2, s, 1)
    h, c = m.begin(x, 321.0, (txt, vec))
    D, Tt = s.hidden, s.txt_tokens
    lin = lambda a, wn, bn: F.linear(T64(a), T64(w[wn]), T64(w[bn])).numpy()
    ln = lambda a: F.layer_norm(T64(a), (D,), eps=1e-6).numpy()
    sc = F.silu(T64(c)).numpy()
    # dual block 0
    mods = {st: [a[:, None] for a in np.split(lin(sc, f"dual0.{st}_mod_w", f"dual0.{st}_mod_b"), 6, axis=1)] for st in ("txt", "img")}
    hs = {"txt": h[:, :Tt], "img": h[:, Tt:]}
    qkv = np.concatenate([lin(ln(hs[st]) * (1 + mods[st][1]) + mods[st][0], f"dual0.{st}_qkv_w", f"dual0.{st}_qkv_b") for st in ("txt", "img")], axis=1)
    T = qkv.shape[1]
    qn = np.concatenate([np.tile(w["dual0.txt_qnorm"], (Tt, 1)), np.tile(w["dual0.img_qnorm"], (T - Tt, 1))])
    kn = np.concatenate([np.tile(w["dual0.txt_knorm"], (Tt, 1)), np.tile(w["dual0.img_knorm"], (T - Tt, 1))])
    a = _torch_attention(s, w, qkv[..., :D], qkv[..., D:2 * D], qkv[..., 2 * D:], qn, kn)
    fa = np.concatenate([lin(a[:, :Tt], "dual0.txt_proj_w", "dual0.txt_proj_b"), lin(a[:, Tt:], "dual0.img_proj_w", "dual0.img_proj_b")], axis=1)
    h1 = {"txt": hs["txt"] + mods["txt"][2] * fa[:, :Tt], "img": hs["img"] + mods["img"][2] * fa[:, Tt:]}
    fm = np.concatenate([lin(F.gelu(T64(lin(ln(h1[st]) * (1 + mods[st][4]) + mods[st][3], f"dual0.{st}_fc1_w", f"dual0.{st}_fc1_b")),
                                    approximate="tanh").numpy(), f"dual0.{st}_fc2_w", f"dual0.{st}_fc2_b") for st in ("txt", "img")], axis=1)
    h2 = np.concatenate([h1["txt"] + mods["txt"][5] * fm[:, :Tt], h1["img"] + mods["img"][5] * fm[:, Tt:]], axis=1)
    got_h, got_f = m.block_real(0, h, c)
    np.testing.assert_allclose(got_f[0], fa, rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(got_f[1], fm, rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(got_h, h2, rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(m.block_fold(0, h, c, got_f), got_h, rtol=1e-12, atol=1e-13)
    # single block 0 (block index depth_dual)
    b = s.depth_dual
    sh, scl, g = [a_[:, None] for a_ in np.split(lin(sc, "single0.mod_w", "single0.mod_b"), 3, axis=1)]
    y = lin(ln(got_h) * (1 + scl) + sh, "single0.lin1_w", "single0.lin1_b")
    a = _torch_attention(s, w, y[..., :D], y[..., D:2 * D], y[..., 2 * D:3 * D], np.tile(w["single0.qnorm"], (T, 1)), np.tile(w["single0.knorm"], (T, 1)))
    f = lin(np.concatenate([a, F.gelu(T64(y[..., 3 * D:]), approximate="tanh").numpy()], axis=-1), "single0.lin2_w", "single0.lin2_b")
    gh, gf = m.block_real(b, got_h, c)
    np.testing.assert_allclose(gf[0], f, rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(gh, got_h + g * f, rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(m.block_fold(b, got_h, c, gf), gh, rtol=1e-12, atol=1e-13)


def test_text_and_image_streams_interact_only_through_attention():
    s = si.mmdit_tiny()
    m = mmdit.MMDiTOracle(s, si.make_mmdit_weights(s, 3))
    x = si.make_video_latents(1, s, 3); txt, vec = si.make_text(1, s, 3)
    out1, feats1 = m.forward(x, 700.0, (txt, vec))
    txt2 = txt.copy(); txt2[0, 0] += 1.0
    out2, feats2 = m.forward(x, 700.0, (txt2, vec))
    assert np.max(np.abs(out1 - out2)) > 1e-6                         # text reaches the image through joint attention
    assert out1.shape == x.shape and len(feats1) == s.n_slots and feats1[-1].shape == (1, s.tokens, s.hidden)
    # rows are independent
    x2 = si.make_video_latents(2, s, 4); t2, v2 = si.make_text(2, s, 4)
    oa, _ = m.forward(x2, 10.0, (t2, v2)); ob, _ = m.forward(x2[1:], 10.0, (t2[1:], v2[1:]))
    np.testing.assert_allclose(oa[1:], ob, rtol=1e-12, atol=1e-14)


def test_flop_counts_match_paper_tables():
    # Table 1: FLUX.1-dev 50 steps = 3719.50 TFLOPs -> 74.39 T per step; the FLUX-shaped model's
    # linear + attention contractions give it from shapes alone.
    f = mmdit.MMDiTOracle(si.mmdit_flux(), {}).flops_per_row()
    assert f / 1e12 == pytest.approx(3719.50 / 50, rel=2e-3)
    # verification cost ratio = one block of the stack: 1/57 and 1/60 (appendix: 0.0175, 0.0167)
    assert 1 / (si.mmdit_flux().depth_dual + si.mmdit_flux().depth_single) == pytest.approx(0.0175, abs=2e-4)
    assert 1 / (si.mmdit_hunyuan().depth_dual + si.mmdit_hunyuan().depth_single) == pytest.approx(0.0167, abs=2e-4)
    assert si.mmdit_hunyuan().img_tokens == 27030 and si.mmdit_flux().img_tokens == 4096


def test_flow_trajectory_tau_zero_is_plain_sampling_and_schedules():
    s = si.mmdit_tiny()
    m = mmdit.MMDiTOracle(s, si.make_mmdit_weights(s, 0))
    B, S = 2, 8
    x = si.make_video_latents(B, s, 0); txt, vec = si.make_text(B, s, 0)
    ts, sg = si.flow_tables(S)
    sol = sampler.Solver("flow", ts, sg)
    conds = [(txt[b], vec[b]) for b in range(B)]
    plain = sampler.sample_plain(m, sol, x, conds)
    out, tr = sampler.sample(m, sampler.SpecaConfig(order=2, interval=3), sol, np.zeros(S, np.float32), x, conds)
    assert np.array_equal(out, plain) and np.all(tr.kind == 0)
    out, tr = sampler.sample(m, sampler.SpecaConfig(order=2, interval=3), sol, np.full(S, np.inf, np.float32), x, conds)
    assert tr.kind[0].tolist() == [0, 1, 1, 0, 1, 1, 0, 1]
    out, tr = sampler.sample(m, sampler.SpecaConfig(order=1, interval=4), sol, core.tau_linear(0.02, 0.004, S), x, conds)
    assert (tr.kind == 1).sum() > 0 and (tr.kind == 2).sum() > 0


def _torch_mm_conditioning(s, w, t, pooled):
    """vec = MLP_t(sinusoid(t)) + MLP_v(pooled) from library routines, angles written out frequency by frequency."""
    half = s.freq_dim // 2
    ang = torch.tensor([[float(t) * 10000.0 ** (-j / half) for j in range(half)]] * pooled.shape[0], dtype=torch.float64)
    emb = torch.cat([torch.cos(ang), torch.sin(ang)], dim=1)
    tv = F.linear(F.silu(F.linear(emb, T64(w["t_w1"]), T64(w["t_b1"]))), T64(w["t_w2"]), T64(w["t_b2"]))
    pv = F.linear(F.silu(F.linear(T64(pooled), T64(w["v_w1"]), T64(w["v_b1"]))), T64(w["v_w2"]), T64(w["v_b2"]))
    return (tv + pv).numpy()


def _torch_mm_finish(s, w, h, vec):
    """Final layer on the image tokens only; un-patchify by explicit indexing:
    out[r, c, f, i p + pi, j p + pj] = tok[r, (f gh + i) gw + j, (c p + pi) p + pj]."""
    D, p = s.hidden, s.patch
    gh, gw = s.latent_h // p, s.latent_w // p
    mod = F.linear(F.silu(T64(vec)), T64(w["fmod_w"]), T64(w["fmod_b"]))
    shift, scale = mod[:, None, :D], mod[:, None, D:]
    tok = F.linear(F.layer_norm(T64(h[:, s.txt_tokens:]), (D,), eps=1e-6) * (1 + scale) + shift, T64(w["final_w"]), T64(w["final_b"])).numpy()
    out = np.zeros((h.shape[0], s.in_channels, s.latent_t, s.latent_h, s.latent_w))
    for f in range(s.latent_t):
        for i in range(gh):
            for j in range(gw):
                for c in range(s.in_channels):
                    for pi in range(p):
                        for pj in range(p):
                            out[:, c, f, i * p + pi, j * p + pj] = tok[:, (f * gh + i) * gw + j, (c * p + pi) * p + pj]
    return out


@pytest.mark.parametrize("shape_fn", [si.mmdit_tiny, si.mmdit_tiny_video])
def test_conditioning_and_finish_vs_library_assembly(shape_fn):
    s = shape_fn()
    w = si.make_mmdit_weights(s, 7, std=0.15)
    m = mmdit.MMDiTOracle(s, w)
    x = si.make_video_latents(2, s, 7); txt, pooled = si.make_text(2, s, 7)
    for t in (0.0, 37.0, 1000.0):
        np.testing.assert_allclose(m.conditioning(t, pooled), _torch_mm_conditioning(s, w, t, pooled), rtol=1e-10, atol=1e-12)
    vec = m.conditioning(37.0, pooled)
    # both halves enter: another pooled vector or another timestep changes the result; a dropped bias does too
    assert np.max(np.abs(m.conditioning(38.0, pooled) - vec)) > 1e-4 and np.max(np.abs(m.conditioning(37.0, pooled[::-1]) - vec)) > 1e-3
    w2 = dict(w); w2["v_b2"] = np.zeros_like(w["v_b2"])
    assert np.max(np.abs(mmdit.MMDiTOracle(s, w2).conditioning(37.0, pooled) - vec)) > 1e-2
    h, vec = m.begin(x, 37.0, (txt, pooled))
    got = m.finish(h, vec)
    ref = _torch_mm_finish(s, w, h, vec)
    assert got.shape == x.shape
    np.testing.assert_allclose(got, ref, rtol=1e-9, atol=1e-11)
    # the text rows never reach the output of the final layer
    h2 = h.copy(); h2[:, : s.txt_tokens] += 1.0
    np.testing.assert_array_equal(m.finish(h2, vec), got)
    # swapped (shift, scale) is far from the reference
    D = s.hidden
    w_sw = dict(w)
    w_sw["fmod_w"] = np.concatenate([w["fmod_w"][D:], w["fmod_w"][:D]]); w_sw["fmod_b"] = np.concatenate([w["fmod_b"][D:], w["fmod_b"][:D]])
    assert np.max(np.abs(mmdit.MMDiTOracle(s, w_sw).finish(h, vec) - ref)) > 1e-2 * np.max(np.abs(ref))
    # forward = begin -> blocks -> finish
    out, _ = m.forward(x, 37.0, (txt, pooled))
    hh = h
    for b in range(m.n_blocks):
        hh, _ = m.block_real(b, hh, vec)
    np.testing.assert_allclose(out, _torch_mm_finish(s, w, hh, vec), rtol=1e-9, atol=1e-11)

"""CPU oracle of the second target-model family: a rectified-flow MMDiT (dual-stream
blocks with joint attention over text + image tokens, then single-stream blocks),
rotary positions, per-head RMS-norm on q and k.

TEST INFRASTRUCTURE ONLY (see oracle/speca_core.py).  Plain float64 NumPy.

The paper only names the architectures it accelerates (FLUX, HunyuanVideo; Sec. 4 and
the appendix "Model Configurations"); the definition below is fixed here and both sides
implement it:

  vec = MLP_t(sinusoid(t)) + MLP_v(pooled);  h = [txt_in(text) ; img_in(patchify(x))]
  dual block (per stream s in {txt, img}, own weights and own 6-way modulation of vec):
      qkv_s = (LN(h_s)(1+scale_a)+shift_a) Wqkv_s + b;  q,k <- RoPE(RMSnorm(q,k))
      a = attention over the joint sequence
      F_attn = [a_txt Wproj_txt + b ; a_img Wproj_img + b]          (cached slot 2l, joint rows)
      h += gate_a(stream) * F_attn
      F_mlp  = [mlp_txt(LNmod(h_txt)) ; mlp_img(LNmod(h_img))]      (cached slot 2l+1)
      h += gate_m(stream) * F_mlp
  single block (3-way modulation):
      [qkv | m] = (LN(h)(1+scale)+shift) W1 + b1;  a = attention(RoPE(RMSnorm(q,k)), v)
      F = [a | GELU_tanh(m)] W2 + b2                                (cached slot 2*n_dual + l)
      h += gate * F
  out = unpatchify((LN(h_img)(1+scale_f)+shift_f) Wf + bf)          (the model's velocity)

RMS-norm: x / sqrt(mean(x^2) + 1e-6) * scale.  RoPE rotates the pairs (2i, 2i+1) of every
head by the angle whose cos/sin the model ships as tables [tokens, head_dim/2].
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

import numpy as np

from .dit import attention, gelu_tanh, layer_norm, linear, silu, timestep_sinusoid

RMS_EPS = 1e-6


def rms_norm(x, scale, eps: float = RMS_EPS):
    return x / np.sqrt((x ** 2).mean(axis=-1, keepdims=True) + eps) * scale


def apply_rope(x, cos, sin):
    """x: [rows, H, T, hd]; cos/sin: [T, hd/2].  (x0, x1) -> (x0 c - x1 s, x0 s + x1 c) per pair."""
    x0, x1 = x[..., 0::2], x[..., 1::2]
    out = np.empty_like(x)
    out[..., 0::2] = x0 * cos - x1 * sin
    out[..., 1::2] = x0 * sin + x1 * cos
    return out


class MMDiTOracle:
    def __init__(self, shape, weights: Dict[str, np.ndarray]):
        self.s = shape
        self.w = {k: np.asarray(v, dtype=np.float64) for k, v in weights.items()}
        self.n_blocks = shape.depth_dual + shape.depth_single
        self.slots_per_block = [2] * shape.depth_dual + [1] * shape.depth_single
        self.n_slots = shape.n_slots

    def rows_cond(self, cond, guided: bool):
        """cond = (text [Tt, txt_dim], pooled [vec_dim]) of one sample -> batch-of-one arrays."""
        assert not guided, "guidance is not part of the rectified-flow configurations"
        txt, pooled = cond
        return np.asarray(txt)[None], np.asarray(pooled)[None]

    # ---- pieces ---------------------------------------------------------------
    def conditioning(self, t: float, pooled: np.ndarray) -> np.ndarray:
        w = self.w
        rows = pooled.shape[0]
        emb = timestep_sinusoid(np.full(rows, float(t)), self.s.freq_dim)
        tv = linear(silu(linear(emb, w["t_w1"], w["t_b1"])), w["t_w2"], w["t_b2"])
        pv = linear(silu(linear(np.asarray(pooled, np.float64), w["v_w1"], w["v_b1"])), w["v_w2"], w["v_b2"])
        return tv + pv

    def patchify(self, x: np.ndarray) -> np.ndarray:
        """[rows, C, F, H, W] -> [rows, F*gh*gw, C*p*p]; token (f, i, j), features (c, pi, pj)."""
        r, C, Fr, H, W = x.shape
        p = self.s.patch
        gh, gw = H // p, W // p
        a = x.reshape(r, C, Fr, gh, p, gw, p).transpose(0, 2, 3, 5, 1, 4, 6)      # r f i j c pi pj
        return a.reshape(r, Fr * gh * gw, C * p * p)

    def unpatchify(self, tok: np.ndarray) -> np.ndarray:
        s = self.s
        r, p = tok.shape[0], s.patch
        gh, gw = s.latent_h // p, s.latent_w // p
        a = tok.reshape(r, s.latent_t, gh, gw, s.in_channels, p, p).transpose(0, 4, 1, 2, 5, 3, 6)   # r c f i pi j pj
        return a.reshape(r, s.in_channels, s.latent_t, s.latent_h, s.latent_w)

    def begin(self, x: np.ndarray, t: float, cond):
        """cond = (text [rows, Tt, txt_dim], pooled [rows, vec_dim]).  x: [rows, C, F, H, W] (F = 1 for images)."""
        w, s = self.w, self.s
        txt, pooled = cond
        x = np.asarray(x, np.float64)
        assert x.ndim == 5
        vec = self.conditioning(t, pooled)
        img = linear(self.patchify(x), w["img_in_w"], w["img_in_b"])
        tx = linear(np.asarray(txt, np.float64), w["txt_in_w"], w["txt_in_b"])
        return np.concatenate([tx, img], axis=1), vec

    def _heads(self, a):   # [r,T,D] -> [r,H,T,hd]
        r, T, _ = a.shape
        return a.reshape(r, T, self.s.heads, self.s.head_dim).transpose(0, 2, 1, 3)

    def _joint_attention(self, q, k, v, qn, kn):
        """q,k,v: [r,T,D] joint; qn/kn: per-token RMS scales [T, hd] (stream-dependent)."""
        w = self.w
        q, k, v = self._heads(q), self._heads(k), self._heads(v)
        q = apply_rope(rms_norm(q, qn[None, None]), w["rope_cos"], w["rope_sin"])
        k = apply_rope(rms_norm(k, kn[None, None]), w["rope_cos"], w["rope_sin"])
        o = attention(q, k, v)
        r, H, T, hd = o.shape
        return o.transpose(0, 2, 1, 3).reshape(r, T, H * hd)

    def _mod(self, vec, wname, bname, n):
        m = linear(silu(vec), self.w[wname], self.w[bname])
        return [a[:, None, :] for a in np.split(m, n, axis=1)]

    def dual_real(self, l: int, h: np.ndarray, vec: np.ndarray):
        w, s = self.w, self.s
        Tt, D = s.txt_tokens, s.hidden
        P = {st: f"dual{l}.{st}_" for st in ("txt", "img")}
        mods = {st: self._mod(vec, P[st] + "mod_w", P[st] + "mod_b", 6) for st in P}
        rng = {"txt": slice(0, Tt), "img": slice(Tt, None)}
        qkv = np.concatenate([linear(layer_norm(h[:, rng[st]]) * (1 + mods[st][1]) + mods[st][0],
                                     w[P[st] + "qkv_w"], w[P[st] + "qkv_b"]) for st in ("txt", "img")], axis=1)
        T = qkv.shape[1]
        qn = np.concatenate([np.repeat(w[P["txt"] + "qnorm"][None], Tt, 0), np.repeat(w[P["img"] + "qnorm"][None], T - Tt, 0)])
        kn = np.concatenate([np.repeat(w[P["txt"] + "knorm"][None], Tt, 0), np.repeat(w[P["img"] + "knorm"][None], T - Tt, 0)])
        a = self._joint_attention(qkv[..., :D], qkv[..., D:2 * D], qkv[..., 2 * D:], qn, kn)
        fa = np.concatenate([linear(a[:, rng[st]], w[P[st] + "proj_w"], w[P[st] + "proj_b"]) for st in ("txt", "img")], axis=1)
        ga = np.concatenate([np.broadcast_to(mods["txt"][2], (h.shape[0], Tt, D)),
                             np.broadcast_to(mods["img"][2], (h.shape[0], T - Tt, D))], axis=1)
        h = h + ga * fa
        fm = np.concatenate([linear(gelu_tanh(linear(layer_norm(h[:, rng[st]]) * (1 + mods[st][4]) + mods[st][3],
                                                     w[P[st] + "fc1_w"], w[P[st] + "fc1_b"])), w[P[st] + "fc2_w"], w[P[st] + "fc2_b"])
                             for st in ("txt", "img")], axis=1)
        gm = np.concatenate([np.broadcast_to(mods["txt"][5], (h.shape[0], Tt, D)),
                             np.broadcast_to(mods["img"][5], (h.shape[0], T - Tt, D))], axis=1)
        h = h + gm * fm
        return h, [fa, fm]

    def dual_fold(self, l, h, vec, feats):
        s = self.s
        Tt, D = s.txt_tokens, s.hidden
        T = h.shape[1]
        mods = {st: self._mod(vec, f"dual{l}.{st}_mod_w", f"dual{l}.{st}_mod_b", 6) for st in ("txt", "img")}
        for which, f in ((2, feats[0]), (5, feats[1])):
            g = np.concatenate([np.broadcast_to(mods["txt"][which], (h.shape[0], Tt, D)),
                                np.broadcast_to(mods["img"][which], (h.shape[0], T - Tt, D))], axis=1)
            h = h + g * f
        return h

    def single_real(self, l: int, h: np.ndarray, vec: np.ndarray):
        w, s = self.w, self.s
        D = s.hidden
        p = f"single{l}."
        shift, scale, gate = self._mod(vec, p + "mod_w", p + "mod_b", 3)
        y = linear(layer_norm(h) * (1 + scale) + shift, w[p + "lin1_w"], w[p + "lin1_b"])
        T = h.shape[1]
        qn = np.repeat(w[p + "qnorm"][None], T, 0)
        kn = np.repeat(w[p + "knorm"][None], T, 0)
        a = self._joint_attention(y[..., :D], y[..., D:2 * D], y[..., 2 * D:3 * D], qn, kn)
        f = linear(np.concatenate([a, gelu_tanh(y[..., 3 * D:])], axis=-1), w[p + "lin2_w"], w[p + "lin2_b"])
        return h + gate * f, [f]

    def single_fold(self, l, h, vec, feats):
        _, _, gate = self._mod(vec, f"single{l}.mod_w", f"single{l}.mod_b", 3)
        return h + gate * feats[0]

    # ---- block-level interface used by the sampler -----------------------------------
    def block_real(self, b: int, h, vec):
        nd = self.s.depth_dual
        return self.dual_real(b, h, vec) if b < nd else self.single_real(b - nd, h, vec)

    def block_fold(self, b: int, h, vec, feats):
        nd = self.s.depth_dual
        return self.dual_fold(b, h, vec, feats) if b < nd else self.single_fold(b - nd, h, vec, feats)

    def finish(self, h, vec):
        w, s = self.w, self.s
        shift, scale = self._mod(vec, "fmod_w", "fmod_b", 2)
        tok = linear(layer_norm(h[:, s.txt_tokens:]) * (1 + scale) + shift, w["final_w"], w["final_b"])
        out = self.unpatchify(tok)
        return out

    def forward(self, x, t, cond):
        h, vec = self.begin(x, t, cond)
        feats: List[np.ndarray] = []
        for b in range(self.n_blocks):
            h, f = self.block_real(b, h, vec)
            feats += f
        return self.finish(h, vec), feats

    def flops_per_row(self) -> float:
        """2 FLOPs per multiply-add of the linear layers and the attention of all blocks."""
        s = self.s
        D, Dm, T, Ti, Tt, hd, H = s.hidden, s.mlp_hidden, s.tokens, s.img_tokens, s.txt_tokens, s.head_dim, s.heads
        attn = 2.0 * 2.0 * H * T * T * hd
        dual = 2.0 * T * D * (3 * D + D + 2 * Dm) + attn
        single = 2.0 * T * D * (3 * D + Dm) + 2.0 * T * (D + Dm) * D + attn
        return s.depth_dual * dual + s.depth_single * single

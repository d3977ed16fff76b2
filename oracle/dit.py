"""CPU oracle of the target model: a class-conditional DiT in adaLN-Zero form.

TEST INFRASTRUCTURE ONLY (see oracle/speca_core.py).  Plain float64 NumPy, one
obvious operation per line; no blocking, fusion or reordering.

The paper only names the architecture (Sec. 3.1.2: blocks of attention and MLP in
residual form F(x) = x + AdaLN o f(x)); the block below is the standard
adaLN-Zero DiT block, fixed here as the definition both sides implement:

  c      = MLP_t(sinusoid(t)) + y_table[label]
  h0     = patchify(x) W_p^T + b_p + pos
  per block l, with (shift_a, scale_a, gate_a, shift_m, scale_m, gate_m) = SiLU(c) W_mod^T + b_mod:
      F_attn = proj( MHA( LN(h)*(1+scale_a)+shift_a ) )         (cached slot 2l)
      h      = h + gate_a * F_attn
      F_mlp  = fc2( GELU_tanh( fc1( LN(h)*(1+scale_m)+shift_m ) ) )   (cached slot 2l+1)
      h      = h + gate_m * F_mlp
  out    = unpatchify( (LN(h)*(1+scale_f)+shift_f) W_f^T + b_f ),  (shift_f, scale_f) = SiLU(c) W_fmod^T + b_fmod

LN has no affine parameters and eps = 1e-6.  The cached features are the
pre-gate branch outputs F_attn / F_mlp, because the gates depend on the current
timestep and can be applied exactly on speculative steps.
Linear weights are [out, in].
"""
from __future__ import annotations

import math
from typing import Dict, List, Sequence, Tuple

import numpy as np

LN_EPS = 1e-6


def silu(a):
    return a / (1.0 + np.exp(-a))


def gelu_tanh(a):
    return 0.5 * a * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (a + 0.044715 * a ** 3)))


def layer_norm(a, eps: float = LN_EPS):
    mu = a.mean(axis=-1, keepdims=True)
    var = ((a - mu) ** 2).mean(axis=-1, keepdims=True)
    return (a - mu) / np.sqrt(var + eps)


def linear(a, w, b=None):
    out = a @ w.T
    return out if b is None else out + b


def attention(q, k, v):
    """softmax(q k^T / sqrt(hd)) v, no mask.  q,k,v: [rows, H, T, hd]."""
    hd = q.shape[-1]
    s = np.einsum("rhid,rhjd->rhij", q, k) / math.sqrt(hd)
    s = s - s.max(axis=-1, keepdims=True)
    p = np.exp(s)
    p = p / p.sum(axis=-1, keepdims=True)
    return np.einsum("rhij,rhjd->rhid", p, v)


def timestep_sinusoid(t: np.ndarray, dim: int, max_period: float = 10000.0) -> np.ndarray:
    """[rows] -> [rows, dim]: (cos(t w_j), sin(t w_j)), w_j = max_period^(-j/(dim/2))."""
    half = dim // 2
    w = np.exp(-math.log(max_period) * np.arange(half, dtype=np.float64) / half)
    ang = np.asarray(t, dtype=np.float64)[:, None] * w[None, :]
    return np.concatenate([np.cos(ang), np.sin(ang)], axis=1)


class DiTOracle:
    """Weights: dict name -> array as produced by speca_inputs.make_dit_weights."""

    def __init__(self, shape, weights: Dict[str, np.ndarray]):
        self.s = shape
        self.w = {k: np.asarray(v, dtype=np.float64) for k, v in weights.items()}
        self.n_blocks = shape.depth
        self.slots_per_block = [2] * shape.depth
        self.n_slots = 2 * shape.depth

    # ---- pieces ---------------------------------------------------------------
    def conditioning(self, t: float, labels: Sequence[int]) -> np.ndarray:
        w = self.w
        rows = len(labels)
        emb = timestep_sinusoid(np.full(rows, float(t)), self.s.freq_dim)
        temb = linear(silu(linear(emb, w["t_w1"], w["t_b1"])), w["t_w2"], w["t_b2"])
        return temb + w["y_table"][np.asarray(labels, dtype=np.int64)]

    def patchify(self, x: np.ndarray) -> np.ndarray:
        """[rows, C, H, W] -> [rows, T, C*p*p]; token = (i, j) row-major over the
        patch grid, features ordered (c, pi, pj)."""
        r, C, H, W = x.shape
        p, g = self.s.patch, self.s.grid
        a = x.reshape(r, C, g, p, g, p)             # r c i pi j pj
        a = a.transpose(0, 2, 4, 1, 3, 5)           # r i j c pi pj
        return a.reshape(r, g * g, C * p * p)

    def unpatchify(self, tok: np.ndarray) -> np.ndarray:
        r = tok.shape[0]
        p, g, C = self.s.patch, self.s.grid, self.s.in_channels
        a = tok.reshape(r, g, g, C, p, p)           # r i j c pi pj
        a = a.transpose(0, 3, 1, 4, 2, 5)           # r c i pi j pj
        return a.reshape(r, C, g * p, g * p)

    def embed(self, x: np.ndarray) -> np.ndarray:
        w = self.w
        return linear(self.patchify(np.asarray(x, dtype=np.float64)), w["patch_w"], w["patch_b"]) + w["pos"][None]

    def modulation(self, c: np.ndarray, l: int) -> List[np.ndarray]:
        w = self.w
        m = linear(silu(c), w[f"blk{l}.mod_w"], w[f"blk{l}.mod_b"])
        return [a[:, None, :] for a in np.split(m, 6, axis=1)]   # each [rows,1,D]

    def attn_branch(self, l: int, h: np.ndarray, shift, scale) -> np.ndarray:
        w, s = self.w, self.s
        r, T, D = h.shape
        xn = layer_norm(h) * (1.0 + scale) + shift
        qkv = linear(xn, w[f"blk{l}.qkv_w"], w[f"blk{l}.qkv_b"])          # [r,T,3D] = (q|k|v), each (head, hd)
        qkv = qkv.reshape(r, T, 3, s.heads, s.head_dim).transpose(2, 0, 3, 1, 4)
        o = attention(qkv[0], qkv[1], qkv[2])                              # [r,H,T,hd]
        o = o.transpose(0, 2, 1, 3).reshape(r, T, D)
        return linear(o, w[f"blk{l}.proj_w"], w[f"blk{l}.proj_b"])

    def mlp_branch(self, l: int, h: np.ndarray, shift, scale) -> np.ndarray:
        w = self.w
        xn = layer_norm(h) * (1.0 + scale) + shift
        a = gelu_tanh(linear(xn, w[f"blk{l}.fc1_w"], w[f"blk{l}.fc1_b"]))
        return linear(a, w[f"blk{l}.fc2_w"], w[f"blk{l}.fc2_b"])

    def final(self, h: np.ndarray, c: np.ndarray) -> np.ndarray:
        w = self.w
        m = linear(silu(c), w["fmod_w"], w["fmod_b"])
        shift, scale = [a[:, None, :] for a in np.split(m, 2, axis=1)]
        tok = linear(layer_norm(h) * (1.0 + scale) + shift, w["final_w"], w["final_b"])
        return self.unpatchify(tok)

    # ---- block-level interface used by the sampler ---------------------------------
    def begin(self, x: np.ndarray, t: float, labels: Sequence[int]):
        """-> (hidden state, per-call context)."""
        c = self.conditioning(t, labels)
        return self.embed(x), c

    def block_real(self, l: int, h: np.ndarray, c: np.ndarray) -> Tuple[np.ndarray, List[np.ndarray]]:
        """Run block l for real: -> (new hidden, [F_attn, F_mlp])."""
        sa, ca, ga, sm, cm, gm = self.modulation(c, l)
        fa = self.attn_branch(l, h, sa, ca)
        h = h + ga * fa
        fm = self.mlp_branch(l, h, sm, cm)
        h = h + gm * fm
        return h, [fa, fm]

    def block_fold(self, l: int, h: np.ndarray, c: np.ndarray, feats: Sequence[np.ndarray]) -> np.ndarray:
        """Advance the hidden state through block l using given (forecast)
        branch outputs in place of computed ones; gates are those of the current step."""
        _, _, ga, _, _, gm = self.modulation(c, l)
        return h + ga * feats[0] + gm * feats[1]

    def finish(self, h: np.ndarray, c: np.ndarray) -> np.ndarray:
        return self.final(h, c)

    def forward(self, x: np.ndarray, t: float, labels: Sequence[int]):
        """Full forward: -> (model output [rows,C,H,W], features of all slots)."""
        h, c = self.begin(x, t, labels)
        feats: List[np.ndarray] = []
        for l in range(self.n_blocks):
            h, f = self.block_real(l, h, c)
            feats += f
        return self.finish(h, c), feats

    # ---- cost model (2 FLOPs per multiply-add) ---------------------------------------
    def flops_per_row(self) -> float:
        s = self.s
        T, D, Dm, hd, H = s.tokens, s.hidden, s.mlp_hidden, s.head_dim, s.heads
        per_block = 2.0 * T * D * (3 * D) + 2.0 * T * D * D + 2.0 * T * D * Dm * 2 + 2.0 * 2.0 * H * T * T * hd
        return s.depth * per_block

"""Seeded synthetic inputs for the SpeCa sampling step (weights, latents, labels,
text embeddings, cached-feature trajectories, solver tables).

This module is the ONLY code shared between the CPU oracle and the HIP library's
tests/benchmarks.  It holds no arithmetic of the method itself: it only draws
random tensors of the shapes, value distributions and structure of the paper's
workloads (class-conditional DiT, forecast/verify tensors) and builds the constant
tables a model ships with (positional table, noise schedule).  Everything is a
pure function of its seed.

All arrays are float32 (or int32) NumPy arrays.  With ``dtype="bf16"`` the values
are rounded to the nearest bfloat16-representable number (ties to even) so that a
bf16 device tensor and an fp64 oracle array hold exactly the same values.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, asdict
from typing import Dict, List, Tuple

import numpy as np

# ----------------------------------------------------------------------------- dtypes


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round a float32 array to the nearest bfloat16 value (ties to even); result
    is float32 holding a bf16-representable value."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 array (already bf16-representable) -> uint16 raw bf16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


def from_bf16_bits(u: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(u, dtype=np.uint16)
    return (u.astype(np.uint32) << 16).view(np.float32).reshape(u.shape)


def _store(a: np.ndarray, dtype: str) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "bf16":
        return round_to_bf16(a)
    if dtype == "f32":
        return a
    raise ValueError(f"unknown dtype {dtype!r}")


def _rng(seed: int, *stream: int) -> np.random.Generator:
    """Independent generator per (seed, stream...) so that a tensor's values do
    not depend on which other tensors were drawn before it."""
    return np.random.default_rng(np.random.SeedSequence([int(seed), *[int(s) for s in stream]]))


# ----------------------------------------------------------------------------- DiT


@dataclass(frozen=True)
class DiTShape:
    """Class-conditional DiT in adaLN-Zero form (shape only)."""
    depth: int            # L blocks
    hidden: int           # D
    heads: int            # H, head_dim = D / H
    mlp_hidden: int       # Dm
    in_channels: int      # C
    latent_hw: int        # latent height = width
    patch: int            # p
    num_classes: int = 1000
    freq_dim: int = 256   # sinusoidal timestep embedding width
    dtype: str = "f32"    # "f32" | "bf16": storage type of weights / activations / cache

    @property
    def head_dim(self) -> int:
        return self.hidden // self.heads

    @property
    def grid(self) -> int:
        return self.latent_hw // self.patch

    @property
    def tokens(self) -> int:
        return self.grid * self.grid

    @property
    def patch_dim(self) -> int:
        return self.patch * self.patch * self.in_channels

    @property
    def n_slots(self) -> int:
        return 2 * self.depth

    def as_dict(self) -> dict:
        return asdict(self)


def dit_tiny(dtype: str = "f32") -> DiTShape:
    """Configuration 1: tiny class-conditional DiT."""
    return DiTShape(depth=2, hidden=64, heads=4, mlp_hidden=256, in_channels=4,
                    latent_hw=8, patch=2, num_classes=10, freq_dim=32, dtype=dtype)


def dit_xl2(dtype: str = "bf16") -> DiTShape:
    """Configuration 3: DiT-XL/2-shaped model."""
    return DiTShape(depth=28, hidden=1152, heads=16, mlp_hidden=4608, in_channels=4,
                    latent_hw=32, patch=2, num_classes=1000, freq_dim=256, dtype=dtype)


def sincos_2d_table(grid: int, dim: int) -> np.ndarray:
    """Fixed 2-D sine/cosine positional table [grid*grid, dim]: first half of the
    channels encodes the row index, second half the column index; each half is
    [sin(pos*w_j), cos(pos*w_j)] with w_j = 10000^(-j/(dim/4))."""
    assert dim % 4 == 0
    q = dim // 4
    omega = 1.0 / (10000.0 ** (np.arange(q, dtype=np.float64) / q))
    ii, jj = np.meshgrid(np.arange(grid, dtype=np.float64), np.arange(grid, dtype=np.float64), indexing="ij")

    def enc(pos):
        ang = pos.reshape(-1)[:, None] * omega[None, :]
        return np.concatenate([np.sin(ang), np.cos(ang)], axis=1)

    return np.concatenate([enc(ii), enc(jj)], axis=1).astype(np.float32)


# Draw order of the DiT parameters.  Every tensor has its own stream index, so the
# list below is the complete recipe: tensor k is N(0, std^2) from stream
# (seed, 1, k) unless noted.
_DIT_GLOBAL = ["t_w1", "t_b1", "t_w2", "t_b2", "y_table", "patch_w", "patch_b",
               "fmod_w", "fmod_b", "final_w", "final_b"]
_DIT_BLOCK = ["mod_w", "mod_b", "qkv_w", "qkv_b", "proj_w", "proj_b",
              "fc1_w", "fc1_b", "fc2_w", "fc2_b"]


def dit_param_shapes(s: DiTShape) -> Dict[str, Tuple[int, ...]]:
    """Name -> shape.  Linear weights are [out_features, in_features], row-major
    (the input dimension is contiguous)."""
    D, Dm = s.hidden, s.mlp_hidden
    shp = {
        "t_w1": (D, s.freq_dim), "t_b1": (D,), "t_w2": (D, D), "t_b2": (D,),
        "y_table": (s.num_classes + 1, D),
        "patch_w": (D, s.patch_dim), "patch_b": (D,),
        "pos": (s.tokens, D),
        "fmod_w": (2 * D, D), "fmod_b": (2 * D,),
        "final_w": (s.patch_dim, D), "final_b": (s.patch_dim,),
    }
    for l in range(s.depth):
        shp[f"blk{l}.mod_w"] = (6 * D, D)
        shp[f"blk{l}.mod_b"] = (6 * D,)
        shp[f"blk{l}.qkv_w"] = (3 * D, D)
        shp[f"blk{l}.qkv_b"] = (3 * D,)
        shp[f"blk{l}.proj_w"] = (D, D)
        shp[f"blk{l}.proj_b"] = (D,)
        shp[f"blk{l}.fc1_w"] = (Dm, D)
        shp[f"blk{l}.fc1_b"] = (Dm,)
        shp[f"blk{l}.fc2_w"] = (D, Dm)
        shp[f"blk{l}.fc2_b"] = (D,)
    return shp


def make_dit_weights(s: DiTShape, seed: int = 0, std: float = 0.02) -> Dict[str, np.ndarray]:
    """All parameters (biases and modulation weights included) ~ N(0, std^2),
    stored in the model dtype; ``pos`` is the fixed sin-cos table."""
    shapes = dit_param_shapes(s)
    out: Dict[str, np.ndarray] = {}
    k = 0
    for name in _DIT_GLOBAL:
        out[name] = _store(_rng(seed, 1, k).standard_normal(shapes[name], dtype=np.float32) * std, s.dtype)
        k += 1
    for l in range(s.depth):
        for nm in _DIT_BLOCK:
            name = f"blk{l}.{nm}"
            out[name] = _store(_rng(seed, 1, k).standard_normal(shapes[name], dtype=np.float32) * std, s.dtype)
            k += 1
    out["pos"] = _store(sincos_2d_table(s.grid, s.hidden), s.dtype)
    return out


def make_latents(batch: int, channels: int, hw: int, seed: int = 0) -> np.ndarray:
    """Initial latent noise N(0,1), float32 [batch, C, hw, hw]."""
    return _rng(seed, 2).standard_normal((batch, channels, hw, hw), dtype=np.float32)


def make_solver_noise(steps: int, latent_shape: Tuple[int, ...], seed: int = 0) -> np.ndarray:
    """Standard-normal draws of a stochastic solver, float32 [steps, *latent_shape] (latent_shape
    starts with the batch).  Both sides of a parity test read the same array."""
    return _rng(seed, 4).standard_normal((steps,) + tuple(latent_shape), dtype=np.float32)


def make_labels(batch: int, num_classes: int, seed: int = 0) -> np.ndarray:
    return _rng(seed, 3).integers(0, num_classes, size=(batch,), dtype=np.int64).astype(np.int32)


# ----------------------------------------------------------------------------- solver tables


def ddim_tables(steps: int, train_steps: int = 1000, beta_start: float = 1e-4,
                beta_end: float = 2e-2) -> Tuple[np.ndarray, np.ndarray]:
    """Noise-schedule tables handed to the sampler as data.

    Linear beta schedule over ``train_steps``; sampling step s uses timestep
    t_s = (S-1-s) * train_steps // S.  Returns (timesteps[S] float32,
    alpha_bar[S+1] float32) where alpha_bar[s] is the cumulative product at t_s and
    alpha_bar[S] = 1 (the clean end of the trajectory)."""
    betas = np.linspace(beta_start, beta_end, train_steps, dtype=np.float64)
    abar = np.cumprod(1.0 - betas)
    ts = np.array([(steps - 1 - s) * train_steps // steps for s in range(steps)], dtype=np.int64)
    ab = np.concatenate([abar[ts], [1.0]])
    return ts.astype(np.float32), ab.astype(np.float32)


def flow_tables(steps: int, time_scale: float = 1000.0) -> Tuple[np.ndarray, np.ndarray]:
    """Rectified-flow tables: sigma[s] = 1 - s/S (sigma[S] = 0); the model is
    conditioned on timesteps[s] = sigma[s] * time_scale."""
    sig = np.array([1.0 - s / steps for s in range(steps + 1)], dtype=np.float64)
    return (sig[:steps] * time_scale).astype(np.float32), sig.astype(np.float32)


# ----------------------------------------------------------------------------- forecast / verify tensors


def feature_trajectory(slots: int, batch: int, tokens: int, hidden: int, ref_steps: List[int],
                       seed: int = 0, dtype: str = "bf16", noise: float = 1e-3) -> List[np.ndarray]:
    """Cached-feature stand-in for configuration 2.  Every element follows
    F(u) = a + b*u + c*u^2 + n(u) with a~N(0,1), b~N(0,0.1^2), c~N(0,0.01^2) and
    n~N(0,noise^2) drawn independently per reference step.  Returns one array
    [slots, batch, tokens, hidden] per entry of ``ref_steps`` (same order)."""
    shape = (slots, batch, tokens, hidden)
    a = _rng(seed, 10).standard_normal(shape, dtype=np.float32)
    b = _rng(seed, 11).standard_normal(shape, dtype=np.float32) * np.float32(0.1)
    c = _rng(seed, 12).standard_normal(shape, dtype=np.float32) * np.float32(0.01)
    out = []
    for j, u in enumerate(ref_steps):
        n = _rng(seed, 13, j).standard_normal(shape, dtype=np.float32) * np.float32(noise)
        f = a + b * np.float32(u) + c * np.float32(u * u) + n
        out.append(_store(f, dtype))
    return out


VERIFY_DELTAS = (0.01, 0.02, 0.03, 0.04, 0.06, 0.07, 0.08, 0.10)


def perturbed_target(pred: np.ndarray, deltas, seed: int = 0, dtype: str = "bf16") -> np.ndarray:
    """Verification target for configuration 2: for sample b,
    truth = pred + delta_b * rms(pred_b) * z with z~N(0,1).  ``pred`` is
    [batch, ...]; the perturbation size is chosen, not computed by the method, so
    that the relative error of sample b is close to delta_b."""
    pred = np.asarray(pred, dtype=np.float32)
    out = np.empty_like(pred)
    for b in range(pred.shape[0]):
        z = _rng(seed, 20, b).standard_normal(pred[b].shape, dtype=np.float32)
        rms = float(np.sqrt(np.mean(pred[b].astype(np.float64) ** 2)))
        out[b] = pred[b] + np.float32(deltas[b % len(deltas)] * rms) * z
    return _store(out, dtype)


# ----------------------------------------------------------------------------- MMDiT


@dataclass(frozen=True)
class MMDiTShape:
    """Rectified-flow MMDiT (shape only): dual-stream blocks over (text, image) tokens with
    joint attention, then single-stream blocks over the concatenated sequence; rotary
    positions; per-head RMS-norm on q and k."""
    depth_dual: int
    depth_single: int
    hidden: int            # D
    heads: int             # head_dim = D / heads
    mlp_hidden: int        # Dm
    in_channels: int       # latent channels C
    latent_t: int          # latent frames (1 = image)
    latent_h: int
    latent_w: int
    patch: int             # spatial patch (temporal patch is 1)
    txt_tokens: int
    txt_dim: int
    vec_dim: int
    rope_axes: Tuple[int, int, int]   # head_dim split over (t, y, x); sums to head_dim
    freq_dim: int = 256
    dtype: str = "bf16"

    @property
    def head_dim(self) -> int:
        return self.hidden // self.heads

    @property
    def img_tokens(self) -> int:
        return self.latent_t * (self.latent_h // self.patch) * (self.latent_w // self.patch)

    @property
    def tokens(self) -> int:
        return self.txt_tokens + self.img_tokens

    @property
    def patch_dim(self) -> int:
        return self.in_channels * self.patch * self.patch

    @property
    def n_slots(self) -> int:
        return 2 * self.depth_dual + self.depth_single

    @property
    def mod_width(self) -> int:
        return self.depth_dual * 12 * self.hidden + self.depth_single * 3 * self.hidden + 2 * self.hidden


def mmdit_tiny(dtype: str = "f32") -> MMDiTShape:
    """Reduced MMDiT for end-to-end parity (the full shapes are far beyond a CPU oracle)."""
    return MMDiTShape(depth_dual=2, depth_single=2, hidden=128, heads=2, mlp_hidden=512, in_channels=4, latent_t=1,
                      latent_h=8, latent_w=12, patch=2, txt_tokens=8, txt_dim=32, vec_dim=24, rope_axes=(16, 24, 24),
                      freq_dim=32, dtype=dtype)


def mmdit_tiny_video(dtype: str = "f32") -> MMDiTShape:
    return MMDiTShape(depth_dual=1, depth_single=2, hidden=128, heads=2, mlp_hidden=512, in_channels=4, latent_t=3,
                      latent_h=4, latent_w=8, patch=2, txt_tokens=5, txt_dim=32, vec_dim=24, rope_axes=(16, 24, 24),
                      freq_dim=32, dtype=dtype)


def mmdit_flux(dtype: str = "bf16") -> MMDiTShape:
    """Configuration 4: FLUX-shaped, 1024x1024 (latent 16 x 128 x 128, patch 2 -> 4096 tokens), 512 text tokens."""
    return MMDiTShape(depth_dual=19, depth_single=38, hidden=3072, heads=24, mlp_hidden=12288, in_channels=16, latent_t=1,
                      latent_h=128, latent_w=128, patch=2, txt_tokens=512, txt_dim=4096, vec_dim=768, rope_axes=(16, 56, 56),
                      dtype=dtype)


def mmdit_hunyuan(dtype: str = "bf16") -> MMDiTShape:
    """Configuration 5: HunyuanVideo-shaped, 480p 2 s (latent 16 x 17 x 60 x 106, patch 1x2x2 -> 27030 tokens), 256 text tokens."""
    return MMDiTShape(depth_dual=20, depth_single=40, hidden=3072, heads=24, mlp_hidden=12288, in_channels=16, latent_t=17,
                      latent_h=60, latent_w=106, patch=2, txt_tokens=256, txt_dim=4096, vec_dim=768, rope_axes=(16, 56, 56),
                      dtype=dtype)


def rope_tables(s: MMDiTShape, theta: float = 10000.0) -> Tuple[np.ndarray, np.ndarray]:
    """cos/sin tables [tokens, head_dim/2] of the rotary embedding: text tokens sit at the
    origin, image token (f, i, j) at position (f, i, j); axis a owns rope_axes[a]/2 frequency
    pairs with omega_q = theta^(-2q/rope_axes[a])."""
    assert sum(s.rope_axes) == s.head_dim and all(a % 2 == 0 for a in s.rope_axes)
    gh, gw = s.latent_h // s.patch, s.latent_w // s.patch
    f, i, j = np.meshgrid(np.arange(s.latent_t), np.arange(gh), np.arange(gw), indexing="ij")
    ids = np.stack([f.ravel(), i.ravel(), j.ravel()], axis=1).astype(np.float64)
    ids = np.concatenate([np.zeros((s.txt_tokens, 3)), ids], axis=0)
    ang = []
    for a, d in enumerate(s.rope_axes):
        omega = 1.0 / theta ** (np.arange(0, d, 2, dtype=np.float64) / d)
        ang.append(ids[:, a:a + 1] * omega[None, :])
    ang = np.concatenate(ang, axis=1)
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def mmdit_param_shapes(s: MMDiTShape) -> Dict[str, Tuple[int, ...]]:
    D, Dm, hd = s.hidden, s.mlp_hidden, s.head_dim
    shp = {
        "t_w1": (D, s.freq_dim), "t_b1": (D,), "t_w2": (D, D), "t_b2": (D,),
        "v_w1": (D, s.vec_dim), "v_b1": (D,), "v_w2": (D, D), "v_b2": (D,),
        "img_in_w": (D, s.patch_dim), "img_in_b": (D,), "txt_in_w": (D, s.txt_dim), "txt_in_b": (D,),
        "fmod_w": (2 * D, D), "fmod_b": (2 * D,), "final_w": (s.patch_dim, D), "final_b": (s.patch_dim,),
    }
    for l in range(s.depth_dual):
        for st in ("img", "txt"):
            p = f"dual{l}.{st}_"
            shp.update({p + "mod_w": (6 * D, D), p + "mod_b": (6 * D,), p + "qkv_w": (3 * D, D), p + "qkv_b": (3 * D,),
                        p + "qnorm": (hd,), p + "knorm": (hd,), p + "proj_w": (D, D), p + "proj_b": (D,),
                        p + "fc1_w": (Dm, D), p + "fc1_b": (Dm,), p + "fc2_w": (D, Dm), p + "fc2_b": (D,)})
    for l in range(s.depth_single):
        p = f"single{l}."
        shp.update({p + "mod_w": (3 * D, D), p + "mod_b": (3 * D,), p + "lin1_w": (3 * D + Dm, D), p + "lin1_b": (3 * D + Dm,),
                    p + "qnorm": (hd,), p + "knorm": (hd,), p + "lin2_w": (D, D + Dm), p + "lin2_b": (D,)})
    return shp


def make_mmdit_weights(s: MMDiTShape, seed: int = 0, std: float = 0.02) -> Dict[str, np.ndarray]:
    """All parameters ~ N(0, std^2) in dict order of mmdit_param_shapes (stream (seed, 4, k)),
    except the RMS-norm scales which are 1 + N(0, std^2); plus the rotary tables
    "rope_cos"/"rope_sin" (float32, not rounded)."""
    out: Dict[str, np.ndarray] = {}
    for k, (name, shape) in enumerate(mmdit_param_shapes(s).items()):
        a = _rng(seed, 4, k).standard_normal(shape, dtype=np.float32) * np.float32(std)
        if name.endswith("norm"):
            a = a + np.float32(1.0)
        out[name] = _store(a, s.dtype)
    out["rope_cos"], out["rope_sin"] = rope_tables(s)
    return out


def make_text(batch: int, s: MMDiTShape, seed: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """Stand-ins for the text encoder outputs: token embeddings [batch, txt_tokens, txt_dim]
    and pooled vector [batch, vec_dim], N(0,1), stored in the model dtype."""
    txt = _rng(seed, 5).standard_normal((batch, s.txt_tokens, s.txt_dim), dtype=np.float32)
    vec = _rng(seed, 6).standard_normal((batch, s.vec_dim), dtype=np.float32)
    return _store(txt, s.dtype), _store(vec, s.dtype)


def make_video_latents(batch: int, s: MMDiTShape, seed: int = 0) -> np.ndarray:
    """Initial noise N(0,1), float32 [batch, C, T, H, W]."""
    return _rng(seed, 2).standard_normal((batch, s.in_channels, s.latent_t, s.latent_h, s.latent_w), dtype=np.float32)

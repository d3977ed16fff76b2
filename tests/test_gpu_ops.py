"""Parity of the dense contractions (linear layers, attention) with the oracle's
plain definitions, through the C ABI (speca_linear, speca_attention).

Tolerance: inputs are bf16-representable on both sides, products are exact in fp32,
sums differ by fp32 rounding (<= K * 2^-24 relative to the sum of magnitudes), and the
bf16 result is rounded once: the device value must lie within one bf16 step of the
oracle's value rounded to bf16, plus that fp32 noise."""
import numpy as np
import pytest

import speca_inputs as si
from oracle import dit as odit, speca_core as core

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _bd():
    from paper_2509_11628_amd import binding as bd
    return bd


def _dev(a, dtype):
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).cuda().to(td).contiguous()


def _check(got, exp, dtype, K):
    got = got.float().cpu().numpy().astype(np.float64)
    scale = np.max(np.abs(exp))
    if dtype == "f32":
        assert np.max(np.abs(got - exp)) <= 1e-5 * scale
    else:
        expb = core.bf16_round(exp)
        tol = np.abs(expb) * 2.0 ** -7 + K * 2.0 ** -22 * scale + 1e-30
        bad = np.abs(got - expb) > tol
        assert not bad.any(), (int(bad.sum()), float(np.max(np.abs(got - expb))))


SHAPES = [  # M, N, K
    (128, 128, 64), (256, 64, 128), (200, 192, 72), (1, 64, 64), (130, 1152, 1152), (515, 256, 4608), (16, 2304, 1152),
    (300, 16, 64),
    # the direct-to-LDS tiles, each with ragged M and N: 128x128, 256x128 (3-stage ring, K-steps 3n+1 and 3n+2), 256x256
    (1000, 3304, 128), (4000, 1160, 256), (4000, 1160, 320), (4000, 3400, 2048),
    # one and two K-steps (the rings re-read the last tile into a free stage past the end of K): 3-stage and 2-stage
    # 256x128, and the shortest K the 256x256 tile takes
    (4096, 3456, 64), (4000, 1160, 64), (4096, 3456, 128), (4608, 3072, 2048),
    # the MLP GEMMs of configuration 3 at full size
    (4096, 4608, 1152), (4096, 1152, 4608),
]


@pytest.mark.parametrize("M,N,K", SHAPES)
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("act", [0, 1, 2])
def test_linear(M, N, K, dtype, act):
    # activations: two register-staged shapes and, for the direct-to-LDS loop, one 256x128 tile (2- and 3-stage ring),
    # one 256x256 tile and the fc1 shape of configuration 3 (one wave of 256x256 tiles plus a remainder launch)
    if act and (M, N, K) not in ((200, 192, 72), (130, 1152, 1152), (4000, 1160, 256), (4000, 3400, 2048), (4096, 3456, 128),
                                 (4096, 4608, 1152)):
        return
    bd = _bd()
    rng = np.random.default_rng(M * 7 + N * 3 + K)
    a = si._store(rng.standard_normal((M, K)).astype(np.float32), dtype)
    w = si._store((rng.standard_normal((N, K)) * 0.05).astype(np.float32), dtype)
    b = si._store(rng.standard_normal(N).astype(np.float32) * 0.1, dtype)
    out = bd.linear(_dev(a, dtype), _dev(w, dtype), _dev(b, dtype), act)
    exp = odit.linear(a.astype(np.float64), w.astype(np.float64), b.astype(np.float64))
    if act == 1:
        exp = odit.gelu_tanh(exp)
    if act == 2:
        exp = odit.silu(exp)
    _check(out, exp, dtype, K)


def test_linear_row_result_independent_of_m():
    bd = _bd()
    rng = np.random.default_rng(0)
    a = _dev(rng.standard_normal((700, 1152)), "bf16"); w = _dev(rng.standard_normal((1152, 1152)) * 0.03, "bf16")
    full = bd.linear(a, w)
    part = bd.linear(a[300:333].contiguous(), w)
    assert torch.equal(full[300:333], part)         # bitwise: fixed K order, no split-K
    # the same across main loops and tile shapes: 4096 rows take the 256x128 direct-to-LDS tiles, 33 rows
    # the register-staged 128x64 ones; K = 2048 with 4096 x 3072 outputs takes 256x256
    a = _dev(rng.standard_normal((4096, 1152)), "bf16")
    full = bd.linear(a, w)
    assert torch.equal(full[1000:1033], bd.linear(a[1000:1033].contiguous(), w))
    a = _dev(rng.standard_normal((4096, 2048)), "bf16"); w = _dev(rng.standard_normal((3072, 2048)) * 0.03, "bf16")
    full = bd.linear(a, w)
    assert torch.equal(full[4000:4096], bd.linear(a[4000:4096].contiguous(), w))


@pytest.mark.parametrize("rows,T,H,hd", [(2, 16, 4, 16), (1, 100, 2, 72), (2, 256, 3, 72), (1, 77, 2, 64), (1, 300, 2, 128), (1, 64, 1, 32),
                                          (1, 256, 2, 128), (3, 200, 2, 64), (1, 257, 2, 72), (1, 33, 1, 128),
                                          (1, 2000, 2, 128), (1, 1111, 1, 72),       # many key tiles, ragged tail
                                          (2, 641, 3, 128), (1, 320, 1, 128)])       # several rows and heads; whole tiles only
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_attention(rows, T, H, hd, dtype):
    bd = _bd()
    rng = np.random.default_rng(T + hd)
    qkv = si._store(rng.standard_normal((rows, T, 3, H, hd)).astype(np.float32), dtype)
    out = bd.attention(_dev(qkv.reshape(rows, T, 3 * H * hd), dtype), H)
    q, k, v = (qkv[:, :, i].transpose(0, 2, 1, 3).astype(np.float64) for i in range(3))
    exp = odit.attention(q, k, v).transpose(0, 2, 1, 3).reshape(rows, T, H * hd)
    got = out.float().cpu().numpy().astype(np.float64)
    scale = np.max(np.abs(exp))
    # bf16: probabilities and the output are rounded to bf16 on the device (2^-9 relative each)
    assert np.max(np.abs(got - exp)) <= (2e-5 if dtype == "f32" else 1.2e-2) * scale


@pytest.mark.parametrize("T,hd", [(256, 72), (200, 72), (96, 64)])
def test_attention_short_sequence_into_an_output_at_8_byte_alignment(T, hd):
    """The whole-sequence kernel (T <= 256) stores 16-byte chunks; an output that is only 8-byte aligned takes the tiled
    kernel instead.  Same values either way."""
    bd = _bd()
    rows, H = 3, 4
    rng = np.random.default_rng(7 * T + hd)
    qkv = si._store(rng.standard_normal((rows, T, 3, H, hd)).astype(np.float32), "bf16")
    dq = _dev(qkv.reshape(rows, T, 3 * H * hd), "bf16")
    aligned = bd.attention(dq, H)
    pool = torch.zeros(rows * T * H * hd + 4, dtype=torch.bfloat16, device="cuda")
    shifted = pool[4:].view(rows, T, H * hd)                   # data pointer 8 bytes past a 16-byte boundary
    assert shifted.data_ptr() % 16 == 8
    bd.attention(dq, H, out=shifted)
    q, k, v = (qkv[:, :, i].transpose(0, 2, 1, 3).astype(np.float64) for i in range(3))
    exp = odit.attention(q, k, v).transpose(0, 2, 1, 3).reshape(rows, T, H * hd)
    scale = np.max(np.abs(exp))
    for got in (aligned, shifted):
        assert np.max(np.abs(got.float().cpu().numpy().astype(np.float64) - exp)) <= 1.2e-2 * scale
    assert float(pool[:4].abs().max()) == 0.0                  # nothing written in front of the output


@pytest.mark.parametrize("M,N,K,act", [(27286, 3072, 3072, 0), (27286, 12288, 3072, 1), (4608, 3072, 12288, 0), (4608, 15360 // 5 * 3, 3072, 0)])
def test_linear_at_mmdit_sizes_sampled_rows(M, N, K, act):
    """The linear layers at the row counts of configurations 4 and 5 (4608 / 27286 tokens, hidden 3072, MLP 12288):
    the device computes the whole product, the oracle a sample of its rows (first and last tile, ragged tail
    included) by the plain definition."""
    bd = _bd()
    g = torch.Generator(device="cuda").manual_seed(M + N + K)
    a = torch.randn((M, K), generator=g, device="cuda").to(torch.bfloat16)
    w = (torch.randn((N, K), generator=g, device="cuda") * 0.03).to(torch.bfloat16)
    b = (torch.randn((N,), generator=g, device="cuda") * 0.1).to(torch.bfloat16)
    out = bd.linear(a, w, b, act)
    rng = np.random.default_rng(M)
    rows = np.unique(np.concatenate([np.arange(0, 8), np.arange(M - 40, M), rng.integers(0, M, 80)]))
    ridx = torch.from_numpy(rows).cuda()
    exp = odit.linear(a[ridx].float().cpu().numpy().astype(np.float64), w.float().cpu().numpy().astype(np.float64),
                      b.float().cpu().numpy().astype(np.float64))
    if act == 1:
        exp = odit.gelu_tanh(exp)
    _check(out[ridx], exp, "bf16", K)


@pytest.mark.parametrize("T,H", [(4608, 2), (27286, 1)])
def test_attention_at_mmdit_lengths_sampled_queries(T, H):
    """Attention at the sequence lengths of configurations 4 (4096 + 512 tokens) and 5 (27030 + 256), head_dim 128:
    the device computes every query; the oracle's plain softmax over ALL keys is evaluated for a few hundred sampled
    query rows (first tile, ragged last tile, random ones).  Keys are given a per-key offset along one direction so
    that the scores are far from uniform and the running maximum really moves along the hundreds of key tiles."""
    bd = _bd()
    hd = 128
    g = torch.Generator(device="cuda").manual_seed(T)
    qkv = torch.randn((1, T, 3, H, hd), generator=g, device="cuda")
    qkv[:, :, 1, :, 0] += torch.linspace(-3.0, 3.0, T, device="cuda")[None, :, None]        # keys drift along dim 0
    qkv[:, :, 0, :, 0] += 2.0                                                                 # every query looks along it
    qkv[:, :, 0] *= 2.5                                                                       # peaked softmax (score std 2.5)
    qkv[:, :, 2, :, 1] += torch.linspace(-2.0, 2.0, T, device="cuda")[None, :, None]        # values say which keys were attended
    qkv = qkv.to(torch.bfloat16)
    out = bd.attention(qkv.reshape(1, T, 3 * H * hd).contiguous(), H)
    rng = np.random.default_rng(T)
    qs = np.unique(np.concatenate([np.arange(0, 70), np.arange(T - 150, T), rng.integers(0, T, 160)]))
    host = qkv.float().cpu().numpy().astype(np.float64)
    q = host[:, qs, 0].transpose(0, 2, 1, 3)                       # [1, H, nq, hd]
    k = host[:, :, 1].transpose(0, 2, 1, 3)                        # [1, H, T, hd]
    v = host[:, :, 2].transpose(0, 2, 1, 3)
    exp = odit.attention(q, k, v).transpose(0, 2, 1, 3).reshape(len(qs), H * hd)
    got = out[0, torch.from_numpy(qs).cuda()].float().cpu().numpy().astype(np.float64)
    scale = np.max(np.abs(exp))
    assert np.max(np.abs(got - exp)) <= 1.2e-2 * scale, float(np.max(np.abs(got - exp)) / scale)


def test_linear_rejects_bad_arguments():
    bd = _bd()
    a = torch.zeros((4, 8), device="cuda"); w = torch.zeros((6, 8), device="cuda")
    with pytest.raises(bd.SpecaError) as e:
        bd.linear(a, w)                              # N not a multiple of 4
    assert e.value.code == bd.EINVAL

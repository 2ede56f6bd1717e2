"""Pins for the oracle's primitives: closed forms, textbook identities and library routines.
Each is chosen so that a plausible slip (dropped term, wrong sign or index, transposed operand)
fails at least one assertion."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workloads as wl
from oracle import binding as ob
from oracle import definition as od

KINDS = [("f32", 2e-6), ("f64", 1e-13)]


@pytest.mark.parametrize("kind,rtol", KINDS)
def test_matvec_is_row_times_vector(kind, rtol):
    rng = np.random.default_rng(0)
    w = rng.standard_normal((7, 13)).astype(np.float32)   # non-square: a transposed read fails
    x = rng.standard_normal(13)
    if kind == "f32":
        x = x.astype(np.float32).astype(np.float64)
    want = w.astype(np.float64) @ x
    got = ob.prim_matvec(w, x, kind)
    assert np.allclose(got, want, rtol=0, atol=rtol * 20)
    # one-hot input picks a column
    e3 = np.zeros(13); e3[3] = 1.0
    assert np.array_equal(ob.prim_matvec(w, e3, kind), w[:, 3].astype(np.float64))


@pytest.mark.parametrize("kind,rtol", KINDS)
def test_matvec_bf16_bits(kind, rtol):
    rng = np.random.default_rng(1)
    wf = rng.standard_normal((5, 16)).astype(np.float32)
    bits = wl.f32_to_bf16_bits(wf)
    # the bit patterns mean what torch says they mean
    as_torch = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(as_torch, wl.bf16_bits_to_f32(bits).astype(np.float64))
    assert np.array_equal(as_torch, torch.from_numpy(wf).to(torch.bfloat16).to(torch.float64).numpy())
    x = np.arange(16, dtype=np.float64) - 7.0
    got = ob.prim_matvec(bits, x, kind)
    assert np.allclose(got, as_torch @ x, rtol=0, atol=1e-4 if kind == "f32" else 1e-12)


@pytest.mark.parametrize("kind,rtol", KINDS)
def test_bf16_round_matches_library(kind, rtol):
    rng = np.random.default_rng(2)
    xs = np.concatenate([rng.standard_normal(200) * 10.0 ** rng.integers(-6, 6, 200),
                         [0.0, 1.0, 1.00390625, 1.01171875, -3.0e38]]).astype(np.float32)
    want = torch.from_numpy(xs).to(torch.bfloat16).to(torch.float32).numpy()
    got = np.array([ob.prim_bf16_round(float(x), kind) for x in xs], dtype=np.float32)
    assert np.array_equal(got, want)   # includes the two halfway cases (ties to even)


@pytest.mark.parametrize("kind,rtol", KINDS)
def test_rmsnorm_closed_forms(kind, rtol):
    d = 24
    gamma = np.linspace(0.5, 1.5, d).astype(np.float32)
    # constant vector c: mean square c^2 -> out = sign(c) * gamma (eps = 0)
    out = ob.prim_rmsnorm(np.full(d, -3.0), gamma, 0.0, kind)
    assert np.allclose(out, -gamma, rtol=rtol * 4, atol=0)
    # eps matters: x = 0 gives 0; tiny x is damped by eps, not blown up
    assert np.all(ob.prim_rmsnorm(np.zeros(d), gamma, 1e-6, kind) == 0)
    x = np.zeros(d); x[5] = 2.0
    out = ob.prim_rmsnorm(x, gamma, 0.25, kind)           # mean sq = 4/24
    assert out[5] == pytest.approx(2.0 / np.sqrt(4.0 / d + 0.25) * gamma[5], rel=rtol * 4)
    # library routine
    rng = np.random.default_rng(3)
    x = rng.standard_normal(d)
    if kind == "f32":
        x = x.astype(np.float32).astype(np.float64)
    want = F.rms_norm(torch.from_numpy(x), (d,), torch.from_numpy(gamma.astype(np.float64)),
                      1e-6).numpy()
    assert np.allclose(ob.prim_rmsnorm(x, gamma, 1e-6, kind), want, rtol=rtol * 8, atol=0)
    assert np.allclose(od.rmsnorm(x, gamma, 1e-6), want, rtol=1e-13, atol=0)


@pytest.mark.parametrize("kind,rtol", KINDS)
def test_silu(kind, rtol):
    assert ob.prim_silu(0.0, kind) == 0.0
    for x in (-20.0, -1.5, -0.1, 0.3, 2.0, 15.0):
        want = float(F.silu(torch.tensor(x, dtype=torch.float64)))
        assert ob.prim_silu(x, kind) == pytest.approx(want, rel=rtol * 4, abs=1e-12)
        assert float(od.silu(np.float64(x))) == pytest.approx(want, rel=1e-14)
    # silu(x) - silu(-x) = x
    assert ob.prim_silu(1.25, kind) - ob.prim_silu(-1.25, kind) == pytest.approx(1.25, rel=rtol * 4)


@pytest.mark.parametrize("kind,rtol", KINDS)
def test_rope_is_a_rotation_by_pos_theta(kind, rtol):
    hd, base = 8, 10000.0
    half = hd // 2
    rng = np.random.default_rng(4)
    v = rng.standard_normal(hd)
    if kind == "f32":
        v = v.astype(np.float32).astype(np.float64)
    # position 0 is the identity
    assert np.array_equal(ob.prim_rope(v, 0, base, kind), v)
    # pair (i, i + hd/2) turns by pos * base^(-2i/hd): complex multiplication
    pos = 7
    z = (v[:half] + 1j * v[half:]) * np.exp(1j * pos * base ** (-2.0 * np.arange(half) / hd))
    got = ob.prim_rope(v, pos, base, kind)
    assert np.allclose(got[:half], z.real, rtol=0, atol=rtol * 8)
    assert np.allclose(got[half:], z.imag, rtol=0, atol=rtol * 8)
    # pair 0 has frequency 1: a quarter turn-ish check of the sign convention
    e0 = np.zeros(hd); e0[0] = 1.0
    r = ob.prim_rope(e0, 1, base, kind)
    assert r[0] == pytest.approx(np.cos(1.0), abs=rtol * 4)
    assert r[half] == pytest.approx(np.sin(1.0), abs=rtol * 4)   # +sin on the partner
    # norm is kept and rotations compose: R(a) R(b) = R(a+b)
    assert np.linalg.norm(got) == pytest.approx(np.linalg.norm(v), rel=rtol * 8)
    twice = ob.prim_rope(ob.prim_rope(v, 3, base, kind), 4, base, kind)
    assert np.allclose(twice, got, rtol=0, atol=rtol * 16)
    # relative-position property: <R(m) q, R(n) k> depends on m - n only
    q, k = rng.standard_normal(hd), rng.standard_normal(hd)
    d1 = ob.prim_rope(q, 9, base, kind) @ ob.prim_rope(k, 4, base, kind)
    d2 = ob.prim_rope(q, 25, base, kind) @ ob.prim_rope(k, 20, base, kind)
    assert d1 == pytest.approx(d2, abs=rtol * 64)
    # numpy definition agrees (it is vectorised over positions and heads)
    dv = od.rope(v.reshape(1, 1, hd), np.array([pos]), base).reshape(hd)
    assert np.allclose(dv, np.concatenate([z.real, z.imag]), rtol=0, atol=1e-14)


@pytest.mark.parametrize("kind,rtol", KINDS)
def test_attention_head_closed_forms(kind, rtol):
    hd, n = 4, 6
    rng = np.random.default_rng(5)
    k = rng.standard_normal((n, hd)); v = rng.standard_normal((n, hd))
    # q = 0 -> uniform weights -> mean of the values
    out = ob.prim_attend(np.zeros(hd), k, v, kind)
    assert np.allclose(out, v.mean(axis=0), rtol=0, atol=rtol * 8)
    # one context entry -> that value exactly
    out = ob.prim_attend(rng.standard_normal(hd), k[:1], v[:1], kind)
    assert np.allclose(out, v[0], rtol=0, atol=rtol * 4)
    # two entries: logistic weight with the 1/sqrt(hd) scale
    q = np.array([1.0, -2.0, 0.5, 3.0])
    s = (k[:2] @ q) / np.sqrt(hd)
    p1 = 1.0 / (1.0 + np.exp(s[0] - s[1]))
    out = ob.prim_attend(q, k[:2], v[:2], kind)
    assert np.allclose(out, (1 - p1) * v[0] + p1 * v[1], rtol=0, atol=rtol * 16)
    # large scores do not overflow
    out = ob.prim_attend(q * 400.0, k, v, kind)
    assert np.all(np.isfinite(out))
    # library: scaled dot product attention
    want = F.scaled_dot_product_attention(torch.from_numpy(q).view(1, 1, 1, hd),
                                          torch.from_numpy(k).view(1, 1, n, hd),
                                          torch.from_numpy(v).view(1, 1, n, hd)).view(hd).numpy()
    assert np.allclose(ob.prim_attend(q, k, v, kind), want, rtol=0, atol=rtol * 16)


@pytest.mark.parametrize("kind,rtol", KINDS)
def test_argmax_lowest_index_and_nan(kind, rtol):
    assert ob.prim_argmax([0.0, 3.0, 3.0, -1.0], kind) == 1
    assert ob.prim_argmax([-5.0, -7.0], kind) == 0
    assert ob.prim_argmax([2.0], kind) == 0
    assert ob.prim_argmax([1.0, float("nan"), 5.0], kind) == -1
    assert ob.prim_argmax([-np.inf, -np.inf, -1e30], kind) == 2


def test_definition_attention_matches_library_gqa():
    """causal grouped-query attention of the numpy definition vs torch's SDPA with the KV heads
    repeated per group (consecutive query heads share a KV head)"""
    rng = np.random.default_rng(6)
    T, nq, nkv, hd = 9, 6, 2, 8
    q = rng.standard_normal((T, nq, hd)); k = rng.standard_normal((T, nkv, hd))
    v = rng.standard_normal((T, nkv, hd))
    got = od.causal_attention(q, k, v)
    tq = torch.from_numpy(q).permute(1, 0, 2).unsqueeze(0)
    tk = torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(nq // nkv, dim=0).unsqueeze(0)
    tv = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(nq // nkv, dim=0).unsqueeze(0)
    want = F.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
    assert np.allclose(got, want, rtol=0, atol=1e-13)
    # first position sees only itself
    assert np.allclose(got[0], np.repeat(v[0], nq // nkv, axis=0), rtol=0, atol=1e-14)

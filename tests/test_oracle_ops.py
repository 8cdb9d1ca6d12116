"""Pins of the oracle's single operations against closed forms, invariants and numpy/scipy fp64 routines.

Each check is chosen so that a plausible slip in the oracle (dropped term, wrong sign or index,
transposed operand, wrong pairing) fails it.  CPU only.
"""
import numpy as np
import pytest
import scipy.special
import torch

from oracle import oracle as O

RNG = np.random.default_rng(1234)


def f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def bf16_bits(a32: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns via torch's conversion (a library routine, round-to-nearest-even)."""
    return torch.from_numpy(a32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def bf16_vals(a32: np.ndarray) -> np.ndarray:
    return torch.from_numpy(a32).to(torch.bfloat16).to(torch.float32).numpy()


# ---------------------------------------------------------------- bf16 rounding

def test_bf16_round_matches_library_conversion():
    v = f32(RNG.standard_normal(4096) * np.exp(RNG.uniform(-20, 20, 4096)))
    ours = np.array([O.bf16_round(float(x)) for x in v], np.float32)
    assert np.array_equal(ours, bf16_vals(v))


def test_bf16_round_ties_to_even():
    # 1 + 2^-8 is exactly halfway between bf16 neighbours 1 and 1+2^-7: ties go to the even mantissa (1.0)
    assert O.bf16_round(1.0 + 2.0 ** -8) == 1.0
    # 1 + 3*2^-8 is halfway between 1+2^-7 (odd) and 1+2^-6 (even)
    assert O.bf16_round(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6
    assert O.bf16_round(-(1.0 + 2.0 ** -8)) == -1.0
    assert O.bf16_round(0.0) == 0.0


# ---------------------------------------------------------------- rmsnorm + matvec

def test_matvec_matches_numpy_fp64_nonsquare():
    N, K = 37, 352  # non-square: a transposed operand cannot pass
    W = f32(RNG.standard_normal((N, K)))
    x = f32(RNG.standard_normal(K))
    y = O.norm_matvec(O.EO_F32, W, x, None, 0.0)
    ref = W.astype(np.float64) @ x.astype(np.float64)
    assert np.max(np.abs(y - ref)) <= 1e-6 * np.max(np.abs(ref))


def test_norm_matvec_matches_definition_fp64():
    N, K, eps = 96, 128, 1e-5
    W = f32(RNG.standard_normal((N, K)) * 0.05)
    x = f32(RNG.standard_normal(K) * 3.0)
    g = f32(1.0 + 0.2 * RNG.standard_normal(K))
    y = O.norm_matvec(O.EO_F32, W, x, g, eps)
    xd = x.astype(np.float64)
    h = g * xd / np.sqrt(np.mean(xd * xd) + eps)
    ref = W.astype(np.float64) @ h
    assert np.max(np.abs(y - ref)) <= 1e-6 * np.max(np.abs(ref))


def test_rmsnorm_constant_vector_closed_form():
    K, eps = 64, 1e-5
    g = f32(RNG.uniform(0.5, 1.5, K))
    eye = f32(np.eye(K))
    for c in (2.5, -0.01):
        y = O.norm_matvec(O.EO_F32, eye, f32(np.full(K, c)), g, eps)
        ref = g * np.sign(c) / np.sqrt(1.0 + eps / (c * c))
        assert np.allclose(y, ref, rtol=1e-6, atol=0)


def test_rmsnorm_scale_invariance():
    K = 128
    W = f32(RNG.standard_normal((16, K)))
    x = f32(RNG.standard_normal(K))
    g = f32(np.ones(K))
    y1 = O.norm_matvec(O.EO_F32, W, x, g, 1e-12)
    y2 = O.norm_matvec(O.EO_F32, W, f32(x * 8.0), g, 1e-12)
    assert np.allclose(y1, y2, rtol=1e-6)


def test_norm_matvec_bf16_contract():
    """bf16 storage: weights are bf16 bit patterns; the input x*g and the RMS scale stay fp32."""
    N, K, eps = 48, 128, 1e-5
    W32 = f32(RNG.standard_normal((N, K)) * 0.05)
    Wb = bf16_bits(W32)
    x = f32(RNG.standard_normal(K))
    g = f32(1.0 + 0.1 * RNG.standard_normal(K))
    y = O.norm_matvec(O.EO_BF16, Wb, x, g, eps)
    h = f32(x * g).astype(np.float64)
    r = np.float32(1.0 / np.sqrt(np.mean(x.astype(np.float64) ** 2) + eps))
    ref = float(r) * (bf16_vals(W32).astype(np.float64) @ h)
    assert np.max(np.abs(y - ref)) <= 1e-6 * np.max(np.abs(ref))
    # and it is close to the un-rounded definition (bf16 has 8 bits of mantissa)
    full = W32.astype(np.float64) @ (g * x / np.sqrt(np.mean(x.astype(np.float64) ** 2) + eps))
    assert np.max(np.abs(y - full)) <= 2e-2 * np.max(np.abs(full))


# ---------------------------------------------------------------- RoPE

def test_rope_position_zero_is_identity():
    v = f32(RNG.standard_normal(4 * 32))
    assert np.array_equal(O.rope(v, 4, 32, 0, 10000.0), v)


def test_rope_textbook_rotation_and_pairing():
    # head_dim 4, half-split pairs (0,2) and (1,3); angles pos*base^0 and pos*base^(-2/4)
    base, pos = 10000.0, 3
    v = f32([1.0, 2.0, 0.0, 0.0])
    out = O.rope(v, 1, 4, pos, base)
    a0, a1 = pos * 1.0, pos * base ** (-0.5)
    ref = np.array([np.cos(a0), 2 * np.cos(a1), np.sin(a0), 2 * np.sin(a1)])
    assert np.allclose(out, ref, atol=1e-7)
    # a vector on the second element of a pair rotates the other way round the circle
    out = O.rope(f32([0, 0, 1.0, 0]), 1, 4, pos, base)
    assert np.allclose(out, [-np.sin(a0), 0, np.cos(a0), 0], atol=1e-7)


def test_rope_preserves_norm_and_depends_on_relative_position():
    H, hd = 2, 32
    q = f32(RNG.standard_normal(H * hd))
    k = f32(RNG.standard_normal(H * hd))
    for h in range(H):
        sl = slice(h * hd, (h + 1) * hd)
        assert np.isclose(np.linalg.norm(O.rope(q, H, hd, 77, 10000.0)[sl]), np.linalg.norm(q[sl]),
                          rtol=1e-6)
    s1 = O.rope(q, H, hd, 9, 10000.0)[:hd] @ O.rope(k, H, hd, 4, 10000.0)[:hd]
    s2 = O.rope(q, H, hd, 109, 10000.0)[:hd] @ O.rope(k, H, hd, 104, 10000.0)[:hd]
    s3 = O.rope(q, H, hd, 9, 10000.0)[:hd] @ O.rope(k, H, hd, 5, 10000.0)[:hd]
    assert np.isclose(s1, s2, rtol=1e-4, atol=1e-5)
    assert not np.isclose(s1, s3, rtol=1e-3)


def test_rope_heads_use_the_same_angles():
    hd = 8
    one = f32(RNG.standard_normal(hd))
    two = np.concatenate([one, one])
    out = O.rope(two, 2, hd, 5, 10000.0)
    assert np.array_equal(out[:hd], out[hd:])


# ---------------------------------------------------------------- attention

def test_attention_single_position_returns_v():
    H, hd = 4, 32
    q = f32(RNG.standard_normal(H * hd))
    K = f32(RNG.standard_normal((1, H * hd)))
    V = f32(RNG.standard_normal((1, H * hd)))
    assert np.allclose(O.attention_row(q, K, V, H, hd), V[0], rtol=1e-7)


def test_attention_uniform_keys_gives_mean_of_values():
    H, hd, n = 2, 16, 37
    q = f32(RNG.standard_normal(H * hd))
    K = f32(np.tile(RNG.standard_normal(H * hd), (n, 1)))
    V = f32(RNG.standard_normal((n, H * hd)))
    assert np.allclose(O.attention_row(q, K, V, H, hd), V.mean(0), rtol=1e-5, atol=1e-6)


def test_attention_matches_scipy_softmax_fp64_per_head():
    H, hd, n = 4, 32, 53
    q = f32(RNG.standard_normal(H * hd))
    K = f32(RNG.standard_normal((n, H * hd)))
    V = f32(RNG.standard_normal((n, H * hd)))
    out = O.attention_row(q, K, V, H, hd)
    Kd = K.astype(np.float64).reshape(n, H, hd)
    Vd = V.astype(np.float64).reshape(n, H, hd)
    qd = q.astype(np.float64).reshape(H, hd)
    s = np.einsum("hc,nhc->hn", qd, Kd) / np.sqrt(hd)
    p = scipy.special.softmax(s, axis=1)
    ref = np.einsum("hn,nhc->hc", p, Vd).reshape(-1)
    assert np.max(np.abs(out - ref)) <= 2e-6 * np.max(np.abs(ref))


def test_attention_heads_do_not_mix():
    H, hd, n = 2, 8, 5
    q = f32(RNG.standard_normal(H * hd))
    K = f32(RNG.standard_normal((n, H * hd)))
    V = f32(RNG.standard_normal((n, H * hd)))
    a = O.attention_row(q, K, V, H, hd)
    K2, V2 = K.copy(), V.copy()
    K2[:, hd:] += 1.0
    V2[:, hd:] *= 2.0
    b = O.attention_row(q, K2, V2, H, hd)
    assert np.array_equal(a[:hd], b[:hd])
    assert not np.allclose(a[hd:], b[hd:])


# ---------------------------------------------------------------- SwiGLU

def test_swiglu_zero_gate_and_fp64_formula():
    n = 257
    up = f32(RNG.standard_normal(n))
    assert np.array_equal(O.swiglu(f32(np.zeros(n)), up), np.zeros(n, np.float32))
    gate = f32(RNG.standard_normal(n) * 4)
    ref = gate.astype(np.float64) * scipy.special.expit(gate.astype(np.float64)) * up.astype(np.float64)
    assert np.allclose(O.swiglu(gate, up), ref, rtol=1e-6, atol=1e-9)
    # large negative gate: silu -> 0-, large positive: silu -> t
    assert abs(O.swiglu(f32([-60.0]), f32([1.0]))[0]) < 1e-20
    assert O.swiglu(f32([60.0]), f32([1.0]))[0] == 60.0


# ---------------------------------------------------------------- softmax max

def test_softmax_max_all_equal_and_dominant():
    n = 1024
    d = O.softmax_max(f32(np.full(n, 0.7)))
    assert d["argmax"] == 0 and d["conf"] == np.float32(1.0 / n)
    z = f32(np.zeros(n))
    z[417] = 200.0
    d = O.softmax_max(z)
    assert d["argmax"] == 417 and d["conf"] == 1.0


def test_softmax_max_matches_scipy_and_reports_runner_up():
    z = f32(RNG.standard_normal(1000) * 3.4)
    d = O.softmax_max(z)
    p = scipy.special.softmax(z.astype(np.float64))
    assert d["argmax"] == int(np.argmax(z))
    assert np.isclose(d["conf"], p.max(), rtol=1e-6)
    assert 1.0 / len(z) <= d["conf"] <= 1.0
    order = np.argsort(-z, kind="stable")
    assert d["arg2"] == order[1] and d["top1"] == z[order[0]] and d["top2"] == z[order[1]]


def test_softmax_max_tie_takes_lowest_index():
    z = f32(np.zeros(16))
    z[5] = z[11] = 2.0
    d = O.softmax_max(z)
    assert d["argmax"] == 5 and d["arg2"] == 11 and d["top1"] == d["top2"]


def test_softmax_max_two_logits_closed_form():
    # conf = 1/(1+exp(-gap)) (logistic): a textbook special case
    for gap in (0.0, 0.3, 2.0, 9.0):
        d = O.softmax_max(f32([1.0, 1.0 + gap]))
        assert np.isclose(d["conf"], scipy.special.expit(gap), rtol=1e-6)

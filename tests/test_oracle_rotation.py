"""Pins of the oracle's key-only Hadamard rotation (Sec. 4 "Integration with Rotation-Based Methods", Sec. 5.3)
against things other than itself: the dense Sylvester matrix from scipy, exact +-1/sqrt(n) columns, orthogonality,
score invariance, the format (a rotated cache is the plain cache of pre-rotated rows), and the effect the paper
uses it for (outlier channels stop dominating the key groups, so key error and attention error drop)."""
import math

import numpy as np
import pytest
import scipy.linalg
import torch

from paper_2502_15075_amd import synth

SIGNS = (0x9E3779B9, 0x7F4A7C15, 0xF39CC060, 0x5CEDC834)


def _sign_vector(signs, n=128):
    return np.array([-1.0 if (signs[d // 32] >> (d % 32)) & 1 else 1.0 for d in range(n)])


def _fwht_f32(x):
    """numpy butterflies in binary32, strides 1, 2, ..., n/2 (written independently of the C loop: whole-array
    reshapes instead of index tests)."""
    y = np.array(x, dtype=np.float32)
    n = y.size
    h = 1
    while h < n:
        v = y.reshape(n // (2 * h), 2, h)
        a, b = v[:, 0, :].copy(), v[:, 1, :].copy()
        v[:, 0, :] = a + b
        v[:, 1, :] = a - b
        h *= 2
    return y


@pytest.mark.parametrize("n", [32, 64, 128])
def test_rotation_is_the_dense_hadamard_matrix(oracle, n):
    rng = np.random.default_rng(n)
    H = scipy.linalg.hadamard(n).astype(np.float64)
    signs = SIGNS
    s = _sign_vector(signs, n)
    for _ in range(20):
        x = (rng.standard_normal(n) * rng.choice([1.0, 30.0], size=n)).astype(np.float32)
        want = H @ (s * x.astype(np.float64)) / math.sqrt(n)
        got = oracle.rotate(x, signs)
        assert np.abs(got - want).max() <= 2e-6 * np.abs(x).sum() / math.sqrt(n) + 1e-30
        back = oracle.unrotate(got, signs)
        assert np.abs(back - x).max() <= 4e-6 * np.abs(x).max()


def test_unit_vectors_give_exact_columns(oracle):
    c = np.float32(1.0 / math.sqrt(128.0))
    H = scipy.linalg.hadamard(128)
    s = _sign_vector(SIGNS)
    for j in (0, 1, 5, 64, 127):
        e = np.zeros(128, dtype=np.float32)
        e[j] = 1.0
        got = oracle.rotate(e, SIGNS)
        assert np.array_equal(got, (H[:, j] * s[j]).astype(np.float32) * c)
        # R^T R = I on the same unit vector, up to the rounding of c*c*128
        back = oracle.unrotate(got, SIGNS)
        assert abs(back[j] - 1.0) < 1e-6 and np.abs(np.delete(back, j)).max() < 1e-7


def test_rotation_matches_numpy_butterflies_bit_for_bit(oracle):
    rng = np.random.default_rng(4)
    s = _sign_vector(SIGNS).astype(np.float32)
    c = np.float32(1.0 / math.sqrt(128.0))
    for _ in range(50):
        x = (rng.standard_normal(128) * 7).astype(np.float16).astype(np.float32)
        assert np.array_equal(oracle.rotate(x, SIGNS), _fwht_f32(s * x) * c)
        assert np.array_equal(oracle.unrotate(x, SIGNS), (_fwht_f32(x) * c) * s)


def test_norms_and_scores_are_preserved(oracle):
    rng = np.random.default_rng(5)
    for _ in range(20):
        k = (rng.standard_normal(128) * 4).astype(np.float32)
        k[[5, 37, 69, 101]] *= 20
        q = rng.standard_normal(128).astype(np.float32)
        kr, qr = oracle.rotate(k, SIGNS).astype(np.float64), oracle.rotate(q, SIGNS).astype(np.float64)
        assert np.linalg.norm(kr) == pytest.approx(np.linalg.norm(k.astype(np.float64)), rel=1e-6)
        assert float(qr @ kr) == pytest.approx(float(q.astype(np.float64) @ k.astype(np.float64)), abs=1e-5 * np.linalg.norm(k) * np.linalg.norm(q))
        # outliers are spread: the largest rotated entry is far below the largest original one
        assert np.abs(kr).max() < 0.5 * np.abs(k).max()


def test_rotated_cache_is_the_plain_cache_of_prerotated_rows(oracle):
    """Format pin: with rotate_k the key planes hold exactly what a plain append of the rows R k (computed here with
    numpy butterflies, handed over as binary32) would hold; the value planes do not change at all."""
    B, H, T = 1, 2, 70
    K, V, _ = synth.make_kvq(11, B, H, H, T, dtype=torch.float16)
    Kn, Vn = K.numpy(), V.numpy()
    s = _sign_vector(SIGNS).astype(np.float32)
    c = np.float32(1.0 / math.sqrt(128.0))
    Krot = np.stack([_fwht_f32(s * r) * c for r in Kn.astype(np.float32).reshape(-1, 128)]).reshape(Kn.shape)
    for bk, bv, gk, gv in ((4, 2, 64, 64), (2, 4, 32, 128), (8, 8, 128, 32)):
        Lr = oracle.Layout(B, H, T, 128, bk, bv, gk, gv, rotate_k=1, signs_k=SIGNS)
        Lp = oracle.Layout(B, H, T, 128, bk, bv, gk, gv)
        pr, pp, p0 = oracle.new_planes(Lr), oracle.new_planes(Lp), oracle.new_planes(Lp)
        oracle.quantize_append(Lr, pr, Kn, Vn, 0)
        oracle.quantize_append(Lp, pp, np.ascontiguousarray(Krot), np.ascontiguousarray(Vn.astype(np.float32)), 0)
        oracle.quantize_append(Lp, p0, Kn, Vn, 0)
        for a, b in zip(pr, pp):
            assert np.array_equal(a, b)
        assert np.array_equal(pr[2], p0[2]) and np.array_equal(pr[3], p0[3])
        assert not np.array_equal(pr[0], p0[0])
        # dequantize: stored basis is the plain reconstruction; input basis is its inverse rotation
        ks, _ = oracle.dequantize(Lr, pr, 0, T, stored=True)
        kp, _ = oracle.dequantize(Lp, pp, 0, T)
        assert np.array_equal(ks, kp)
        ku, _ = oracle.dequantize(Lr, pr, 0, T)
        want = np.stack([(_fwht_f32(r) * c) * s for r in ks.reshape(-1, 128)]).reshape(ks.shape)
        assert np.array_equal(ku, want)


def test_rotation_needs_quantized_keys(oracle):
    L = oracle.Layout(1, 1, 32, 128, 16, 16, 64, 64, rotate_k=1, signs_k=SIGNS)
    K = np.zeros((1, 1, 4, 128), dtype=np.float16)
    with pytest.raises(ValueError):
        oracle.quantize_append(L, oracle.new_planes(L), K, K, 0)


def test_decode_attention_of_a_rotated_cache(oracle):
    """The oracle's rotated decode equals dense attention computed here from the stored reconstruction and a query
    rotated with scipy's matrix (binary64) and rounded to binary16; and with 8-bit keys it is close to exact
    attention on the original tensors (the rotation changes the basis, not the function)."""
    B, Hk, Hq, T = 1, 2, 4, 96
    K, V, q = synth.make_kvq(12, B, Hk, Hq, T, dtype=torch.float16)
    scale = 1 / math.sqrt(128)
    L = oracle.Layout(B, Hk, T, 128, 8, 8, 32, 32, rotate_k=1, signs_k=SIGNS)
    planes = oracle.new_planes(L)
    oracle.quantize_append(L, planes, K.numpy(), V.numpy(), 0)
    got = oracle.decode_attention(L, planes, q.numpy(), T, scale)
    Ks, Vs = oracle.dequantize(L, planes, 0, T, stored=True)
    Hm = scipy.linalg.hadamard(128).astype(np.float64)
    s = _sign_vector(SIGNS)
    qr = (q.numpy().astype(np.float64) * s) @ Hm.T / math.sqrt(128)
    qr16 = qr.astype(np.float32).astype(np.float16)
    # the binary64 rotation and the oracle's binary32 butterflies may round a few entries to neighbouring binary16
    # numbers; compare through the attention output with a tolerance that covers one binary16 ulp of the query
    want = oracle.attention_dense(Ks, Vs, qr16, scale)
    assert np.abs(got - want).max() <= 3e-3 * np.abs(want).max()
    exact = oracle.attention_dense(K.float().numpy(), V.float().numpy(), q.numpy(), scale)
    err_rot = np.abs(got - exact).max() / np.abs(exact).max()
    assert err_rot < 0.1


def test_rotation_lowers_key_error_and_attention_error(oracle):
    """Sec. 5.3: key-only rotation is what brings K4V2 towards K4V4.  On keys with a few large channels the rotated
    4-bit cache has a much smaller key MSE, and over many (sequence, head) pairs a smaller attention-output error."""
    B, H, T = 8, 8, 128
    scale = 1 / math.sqrt(128)
    K, V, q = synth.make_kvq(13, B, H, H, T, dtype=torch.float16)
    Kn, Vn, qn = K.numpy(), V.numpy(), q.numpy()
    exact = oracle.attention_dense(Kn.astype(np.float32), Vn.astype(np.float32), qn, scale).astype(np.float64)
    res = {}
    for rot in (0, 1):
        L = oracle.Layout(B, H, T, 128, 4, 2, 64, 64, rotate_k=rot, signs_k=SIGNS)
        planes = oracle.new_planes(L)
        oracle.quantize_append(L, planes, Kn, Vn, 0)
        Kh, _ = oracle.dequantize(L, planes, 0, T)
        out = oracle.decode_attention(L, planes, qn, T, scale).astype(np.float64)
        res[rot] = (oracle.mse(Kn.astype(np.float32), Kh),
                    float((np.linalg.norm(out - exact, axis=-1) / np.linalg.norm(exact, axis=-1)).mean()))
    assert res[1][0] < 0.5 * res[0][0]
    assert res[1][1] < res[0][1]


SIGNS_V = (0x243F6A88, 0x85A308D3, 0x13198A2E, 0x03707344)


def test_value_rotation_format_and_inverse(oracle):
    """rotate_v: the value planes are the plain planes of the rows R_v v (numpy butterflies), the key planes do not
    move, and dequantize hands back R_v^T of the stored reconstruction."""
    B, H, T = 1, 2, 70
    K, V, _ = synth.make_kvq(14, B, H, H, T, dtype=torch.float16)
    Kn, Vn = K.numpy(), V.numpy()
    s = _sign_vector(SIGNS_V).astype(np.float32)
    c = np.float32(1.0 / math.sqrt(128.0))
    Vrot = np.stack([_fwht_f32(s * r) * c for r in Vn.astype(np.float32).reshape(-1, 128)]).reshape(Vn.shape)
    for bk, bv, gk, gv in ((4, 2, 64, 64), (2, 4, 32, 128)):
        Lr = oracle.Layout(B, H, T, 128, bk, bv, gk, gv, rotate_v=1, signs_v=SIGNS_V)
        Lp = oracle.Layout(B, H, T, 128, bk, bv, gk, gv)
        pr, pp, p0 = oracle.new_planes(Lr), oracle.new_planes(Lp), oracle.new_planes(Lp)
        oracle.quantize_append(Lr, pr, Kn, Vn, 0)
        oracle.quantize_append(Lp, pp, np.ascontiguousarray(Kn.astype(np.float32)), np.ascontiguousarray(Vrot), 0)
        oracle.quantize_append(Lp, p0, Kn, Vn, 0)
        for a, b in zip(pr, pp):
            assert np.array_equal(a, b)
        assert np.array_equal(pr[0], p0[0]) and np.array_equal(pr[1], p0[1]) and not np.array_equal(pr[2], p0[2])
        _, vs = oracle.dequantize(Lr, pr, 0, T, stored=True)
        _, vu = oracle.dequantize(Lr, pr, 0, T)
        want = np.stack([(_fwht_f32(r) * c) * s for r in vs.reshape(-1, 128)]).reshape(vs.shape)
        assert np.array_equal(vu, want)


def test_attention_with_both_rotations_is_the_same_function(oracle):
    """out = R_v^T (softmax(q' K'^T) V') with q' = R_k q: with 8-bit codes it stays close to exact attention on the
    original tensors, and it equals the matrix form evaluated here with scipy's Hadamard matrix in binary64."""
    B, Hk, Hq, T = 1, 2, 4, 96
    K, V, q = synth.make_kvq(15, B, Hk, Hq, T, dtype=torch.float16)
    scale = 1 / math.sqrt(128)
    L = oracle.Layout(B, Hk, T, 128, 8, 8, 32, 32, rotate_k=1, signs_k=SIGNS, rotate_v=1, signs_v=SIGNS_V)
    planes = oracle.new_planes(L)
    oracle.quantize_append(L, planes, K.numpy(), V.numpy(), 0)
    got = oracle.decode_attention(L, planes, q.numpy(), T, scale).astype(np.float64)
    exact = oracle.attention_dense(K.float().numpy(), V.float().numpy(), q.numpy(), scale)
    assert np.abs(got - exact).max() / np.abs(exact).max() < 0.1
    Ks, Vs = oracle.dequantize(L, planes, 0, T, stored=True)
    Hm = scipy.linalg.hadamard(128).astype(np.float64)
    sk, sv = _sign_vector(SIGNS), _sign_vector(SIGNS_V)
    qr = np.stack([oracle.rotate(r, SIGNS) for r in q.numpy().astype(np.float32).reshape(-1, 128)]).astype(np.float16)
    out_rot = oracle.attention_dense(Ks, Vs, qr.reshape(B, Hq, 128), scale).astype(np.float64)
    want = (out_rot @ Hm) / math.sqrt(128) * sv                         # R_v^T y = diag(s_v) H y / sqrt(n)
    assert np.abs(got - want).max() <= 1e-5 * np.abs(want).max()


def test_rotating_values_does_not_help(oracle):
    """Sec. 5.3: the gains come from the keys; value rotation alone is unnecessary.  On values without outlier
    channels the rotated 2-bit value cache has the same reconstruction error (a rotation keeps an isotropic
    distribution isotropic), so the attention error of value-only rotation stays at the unrotated level while
    key-only rotation lowers it."""
    B, H, T = 8, 8, 128
    scale = 1 / math.sqrt(128)
    K, V, q = synth.make_kvq(16, B, H, H, T, dtype=torch.float16)
    Kn, Vn, qn = K.numpy(), V.numpy(), q.numpy()
    exact = oracle.attention_dense(Kn.astype(np.float32), Vn.astype(np.float32), qn, scale).astype(np.float64)
    err, mse_v = {}, {}
    for name, rk, rv in (("none", 0, 0), ("key", 1, 0), ("value", 0, 1), ("both", 1, 1)):
        L = oracle.Layout(B, H, T, 128, 4, 2, 64, 64, rotate_k=rk, signs_k=SIGNS, rotate_v=rv, signs_v=SIGNS_V)
        planes = oracle.new_planes(L)
        oracle.quantize_append(L, planes, Kn, Vn, 0)
        _, Vh = oracle.dequantize(L, planes, 0, T)
        mse_v[name] = oracle.mse(Vn.astype(np.float32), Vh)
        out = oracle.decode_attention(L, planes, qn, T, scale).astype(np.float64)
        err[name] = float((np.linalg.norm(out - exact, axis=-1) / np.linalg.norm(exact, axis=-1)).mean())
    assert 0.9 < mse_v["value"] / mse_v["none"] < 1.1
    assert err["key"] < err["none"] and err["both"] < err["none"]
    assert err["value"] > 0.9 * err["none"]
    assert err["both"] > 0.9 * err["key"]

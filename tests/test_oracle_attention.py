"""Pins for the CPU oracle's decode attention and for the paper's claims about bit allocation.

The attention oracle is the textbook definition (App. A: S = Q K^T / sqrt(d), A = softmax(S),
output A V); it is pinned to brute-force loops, to special cases with a closed form, and to
torch's own scaled-dot-product attention.  The bit-allocation tests check Theorem 2 (more bits
for keys beats the swapped allocation when ||K|| > ||V||) on the synthetic workload.
"""
import math

import numpy as np
import pytest
import torch

from paper_2502_15075_amd import synth


def _brute(K, V, q, scale):
    B, Hk, T, D = K.shape
    Hq = q.shape[1]
    R = Hq // Hk
    out = np.zeros((B, Hq, D))
    for b in range(B):
        for h in range(Hq):
            kh = h // R
            logits = [scale * sum(float(q[b, h, d]) * float(K[b, kh, t, d]) for d in range(D)) for t in range(T)]
            m = max(logits)
            w = [math.exp(l - m) for l in logits]
            tot = sum(w)
            for d in range(D):
                out[b, h, d] = sum(w[t] * float(V[b, kh, t, d]) for t in range(T)) / tot
    return out


def test_dense_attention_matches_brute_force_gqa(oracle):
    rng = np.random.default_rng(0)
    B, Hk, Hq, T, D = 2, 2, 6, 7, 32                      # 3 query heads per KV head
    K = rng.standard_normal((B, Hk, T, D)).astype(np.float32)
    V = rng.standard_normal((B, Hk, T, D)).astype(np.float32)
    q = rng.standard_normal((B, Hq, D)).astype(np.float32)
    got = oracle.attention_dense(K, V, q, 0.3)
    assert np.allclose(got, _brute(K, V, q, 0.3), rtol=1e-6, atol=1e-7)
    # a transposed operand or a wrong head map would show here: make KV heads very different
    K[:, 1] *= 5
    V[:, 1] += 3
    got = oracle.attention_dense(K, V, q, 0.3)
    assert np.allclose(got, _brute(K, V, q, 0.3), rtol=1e-6, atol=1e-7)


def test_dense_attention_matches_torch_sdpa(oracle):
    torch.manual_seed(1)
    B, Hk, Hq, T, D = 2, 2, 8, 50, 64
    K = torch.randn(B, Hk, T, D, dtype=torch.float64)
    V = torch.randn(B, Hk, T, D, dtype=torch.float64)
    q = torch.randn(B, Hq, D, dtype=torch.float64)
    R = Hq // Hk
    want = torch.nn.functional.scaled_dot_product_attention(
        q[:, :, None, :], K.repeat_interleave(R, dim=1), V.repeat_interleave(R, dim=1), scale=0.2)[:, :, 0]
    got = oracle.attention_dense(K.float().numpy(), V.float().numpy(), q.float().numpy(), 0.2)
    assert np.allclose(got, want.numpy(), rtol=2e-5, atol=2e-6)


def test_special_cases_with_closed_forms(oracle):
    rng = np.random.default_rng(2)
    B, Hk, Hq, T, D = 1, 2, 4, 33, 64
    K = rng.standard_normal((B, Hk, T, D)).astype(np.float32)
    V = rng.standard_normal((B, Hk, T, D)).astype(np.float32)
    q = rng.standard_normal((B, Hq, D)).astype(np.float32)
    # one cached token: the output is that token's value row
    out = oracle.attention_dense(K[:, :, :1], V[:, :, :1], q, 0.125)
    assert np.array_equal(out, np.repeat(V[:, :, 0], 2, axis=1))
    # zero query: uniform weights, output is the mean value row
    out = oracle.attention_dense(K, V, np.zeros_like(q), 0.125)
    assert np.allclose(out, np.repeat(V.astype(np.float64).mean(axis=2), 2, axis=1), rtol=1e-6, atol=1e-7)
    # identical key rows: uniform weights whatever the query
    Ksame = np.repeat(K[:, :, :1], T, axis=2)
    out = oracle.attention_dense(Ksame, V, q, 0.125)
    assert np.allclose(out, np.repeat(V.astype(np.float64).mean(axis=2), 2, axis=1), rtol=1e-6, atol=1e-7)
    # softmax is invariant to adding the same number to every logit: shift every key row by c*q/|q|^2-like row
    base = oracle.attention_dense(K, V, q[:, :1].repeat(4, axis=1), 0.125)
    shift = (q[:, 0] / np.linalg.norm(q[:, 0]))[:, None, None, :] * 3.0
    shifted = oracle.attention_dense(K + shift.astype(np.float32), V, q[:, :1].repeat(4, axis=1), 0.125)
    assert np.allclose(base, shifted, rtol=2e-4, atol=2e-5)
    # a very large logit on one token selects its value row
    Kbig = K.copy()
    Kbig[0, 0, 5] = 1000 * q[0, 0]
    out = oracle.attention_dense(Kbig, V, q, 1.0)
    assert np.allclose(out[0, 0], V[0, 0, 5], rtol=1e-6)


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
def test_decode_attention_over_cache_is_dense_attention_on_reconstruction(oracle, dtype):
    K, V, q = synth.make_kvq(4, 2, 2, 8, 100, 128, dtype=dtype)
    bf = dtype == torch.bfloat16
    L = oracle.Layout(2, 2, 100, 128, 4, 2, 64, 64)
    planes = oracle.new_planes(L)
    oracle.quantize_append(L, planes, synth.to_numpy_bits(K), synth.to_numpy_bits(V), 0, bf16=bf)
    scale = 1 / math.sqrt(128)
    got = oracle.decode_attention(L, planes, synth.to_numpy_bits(q), 100, scale, bf16=bf)
    kd, vd = oracle.dequantize(L, planes, 0, 100)
    R = 4
    want = torch.nn.functional.scaled_dot_product_attention(
        q.double()[:, :, None, :], torch.from_numpy(kd).double().repeat_interleave(R, dim=1),
        torch.from_numpy(vd).double().repeat_interleave(R, dim=1), scale=scale)[:, :, 0].numpy()
    assert np.allclose(got, want, rtol=1e-5, atol=1e-6)
    # seq_len shorter than what is cached: only the first tokens count
    got50 = oracle.decode_attention(L, planes, synth.to_numpy_bits(q), 50, scale, bf16=bf)
    want50 = oracle.attention_dense(kd[:, :, :50], vd[:, :, :50], q.float().numpy(), scale)
    assert np.array_equal(got50, want50)


def test_unquantized_cache_equals_plain_attention(oracle):
    K, V, q = synth.make_kvq(5, 1, 2, 4, 70, 128, dtype=torch.float16)
    L = oracle.Layout(1, 2, 70, 128, 16, 16, 64, 64)
    planes = oracle.new_planes(L)
    oracle.quantize_append(L, planes, K.numpy(), V.numpy(), 0)
    scale = 1 / math.sqrt(128)
    got = oracle.decode_attention(L, planes, q.numpy(), 70, scale)
    want = torch.nn.functional.scaled_dot_product_attention(
        q.double()[:, :, None, :], K.double().repeat_interleave(2, dim=1), V.double().repeat_interleave(2, dim=1),
        scale=scale)[:, :, 0].numpy()
    assert np.allclose(got, want, rtol=1e-5, atol=1e-6)


@pytest.mark.parametrize("bk,bv,dtype", [(16, 2, torch.float16), (16, 4, torch.bfloat16), (4, 16, torch.float16), (2, 16, torch.bfloat16)])
def test_one_tensor_unquantized(oracle, bk, bv, dtype):
    """The ablation that quantizes only keys or only values (Table 1's discussion): the 16-bit tensor is kept exactly
    (its plane holds the input patterns, its scale/zero plane is empty), and attention is the library routine on the
    exact tensor and the other one's reconstruction."""
    K, V, q = synth.make_kvq(6 + bk, 1, 2, 4, 70, 128, dtype=dtype)
    bf = dtype == torch.bfloat16
    L = oracle.Layout(1, 2, 70, 128, bk, bv, 64, 64, raw_dtype=1 if bf else 0)
    planes = oracle.new_planes(L)
    assert planes[1 if bk == 16 else 3].size == 0 and planes[0 if bk == 16 else 2].size == 2 * 96 * 256
    oracle.quantize_append(L, planes, synth.to_numpy_bits(K), synth.to_numpy_bits(V), 0, bf16=bf)
    kd, vd = oracle.dequantize(L, planes, 0, 70)
    exact, other = (kd, K) if bk == 16 else (vd, V)
    assert np.array_equal(exact, other.float().numpy())
    Lq = oracle.Layout(1, 2, 70, 128, 4 if bk == 16 else bk, 4 if bv == 16 else bv, 64, 64)     # the quantized tensor alone
    pq = oracle.new_planes(Lq)
    oracle.quantize_append(Lq, pq, synth.to_numpy_bits(K), synth.to_numpy_bits(V), 0, bf16=bf)
    kq, vq = oracle.dequantize(Lq, pq, 0, 70)
    assert np.array_equal(vd, vq) if bk == 16 else np.array_equal(kd, kq)
    scale = 1 / math.sqrt(128)
    got = oracle.decode_attention(L, planes, synth.to_numpy_bits(q), 70, scale, bf16=bf)
    want = torch.nn.functional.scaled_dot_product_attention(
        q.double()[:, :, None, :], torch.from_numpy(kd).double().repeat_interleave(2, dim=1),
        torch.from_numpy(vd).double().repeat_interleave(2, dim=1), scale=scale)[:, :, 0].numpy()
    assert np.allclose(got, want, rtol=1e-5, atol=1e-6)


# --------------------------------------------------------------------------- bit allocation (Theorem 2)

def _alloc_error(oracle, K, V, q, bk, bv, G, bf16):
    B, Hk, T, D = K.shape
    L = oracle.Layout(B, Hk, T, D, bk, bv, G, G)
    planes = oracle.new_planes(L)
    oracle.quantize_append(L, planes, synth.to_numpy_bits(K), synth.to_numpy_bits(V), 0, bf16=bf16)
    scale = 1 / math.sqrt(D)
    got = oracle.decode_attention(L, planes, synth.to_numpy_bits(q), T, scale, bf16=bf16).astype(np.float64)
    want = oracle.attention_dense(K.float().numpy(), V.float().numpy(), q.float().numpy(), scale).astype(np.float64)
    rel = np.linalg.norm(got - want, axis=-1) / np.linalg.norm(want, axis=-1)
    return rel.mean()                                    # mean over (batch, query head) pairs


@pytest.mark.parametrize("sigma_k", [2.0, 4.0, 6.0])
def test_more_bits_for_keys_beats_the_swapped_allocation(oracle, sigma_k):
    """Theorem 2 is a statement about the expectation, so the error is averaged over 256
    (sequence, query head) pairs.  ||K||_F > ||V||_F by construction (sigma_k >= 2, outlier channels)."""
    K, V, q = synth.make_kvq(int(sigma_k), 32, 2, 8, 256, 128, dtype=torch.bfloat16, sigma_k=sigma_k)
    assert K.float().norm() > 2 * V.float().norm()
    e42 = _alloc_error(oracle, K, V, q, 4, 2, 64, True)
    e24 = _alloc_error(oracle, K, V, q, 2, 4, 64, True)
    e44 = _alloc_error(oracle, K, V, q, 4, 4, 64, True)
    e22 = _alloc_error(oracle, K, V, q, 2, 2, 64, True)
    assert e42 < e24
    assert e44 < e42 < e22 and e44 < e24 < e22 * 1.05


def test_without_norm_disparity_the_ordering_disappears(oracle):
    """The proviso of Theorem 2: with ||K|| = ||V|| neither allocation is clearly ahead."""
    K, V, q = synth.make_kvq(7, 32, 2, 8, 256, 128, dtype=torch.bfloat16, sigma_k=1.0, outlier_scale=1.0)
    e42 = _alloc_error(oracle, K, V, q, 4, 2, 64, True)
    e24 = _alloc_error(oracle, K, V, q, 2, 4, 64, True)
    assert 0.6 < e42 / e24 < 1.6


def test_eight_bits_approach_full_precision(oracle):
    K, V, q = synth.make_kvq(8, 4, 2, 8, 256, 128, dtype=torch.bfloat16, sigma_k=1.0, outlier_scale=1.0)
    e88 = _alloc_error(oracle, K, V, q, 8, 8, 64, True)
    e44 = _alloc_error(oracle, K, V, q, 4, 4, 64, True)
    e22 = _alloc_error(oracle, K, V, q, 2, 2, 64, True)
    assert e88 < 1e-2 and e88 < e44 < e22
    Ko, Vo, qo = synth.make_kvq(9, 4, 2, 8, 256, 128, dtype=torch.bfloat16)      # the heavy-outlier workload
    assert _alloc_error(oracle, Ko, Vo, qo, 8, 8, 64, True) < _alloc_error(oracle, Ko, Vo, qo, 4, 4, 64, True)


def test_per_sequence_lengths_are_independent_batches_of_one(oracle):
    """Ragged batch: element b of the result is what a cache holding ONLY that sequence's tokens gives (built from
    scratch with batch 1), equal lengths reproduce the uniform call bit for bit, and per-element appends land where a
    batch-1 append would put them."""
    rng = np.random.default_rng(77)
    B, Hk, Hq, T, D = 3, 2, 4, 90, 128
    K = (rng.standard_normal((B, Hk, T, D)) * 2).astype(np.float16)
    V = rng.standard_normal((B, Hk, T, D)).astype(np.float16)
    q = rng.standard_normal((B, Hq, D)).astype(np.float16)
    scale = 1 / np.sqrt(D)
    L = oracle.Layout(B, Hk, T, D, 4, 2, 64, 64)
    planes = oracle.new_planes(L)
    oracle.quantize_append(L, planes, K, V, 0)
    lens = [90, 1, 47]
    got = oracle.decode_attention_varlen(L, planes, q, lens, scale)
    for b, n in enumerate(lens):
        L1 = oracle.Layout(1, Hk, T, D, 4, 2, 64, 64)
        p1 = oracle.new_planes(L1)
        oracle.quantize_append(L1, p1, np.ascontiguousarray(K[b:b + 1, :, :n]), np.ascontiguousarray(V[b:b + 1, :, :n]), 0)
        want = oracle.decode_attention(L1, p1, q[b:b + 1], n, scale)
        assert np.array_equal(got[b], want[0])
    same = oracle.decode_attention_varlen(L, planes, q, [60, 60, 60], scale)
    assert np.array_equal(same, oracle.decode_attention(L, planes, q, 60, scale))
    # appends at per-element positions
    pa = oracle.new_planes(L, fill=0x11)
    pos = [5, 0, 33]
    oracle.quantize_append_at(L, pa, np.ascontiguousarray(K[:, :, 7:8]), np.ascontiguousarray(V[:, :, 7:8]), pos)
    for b, t in enumerate(pos):
        L1 = oracle.Layout(1, Hk, T, D, 4, 2, 64, 64)
        p1 = oracle.new_planes(L1, fill=0x11)
        oracle.quantize_append(L1, p1, np.ascontiguousarray(K[b:b + 1, :, 7:8]), np.ascontiguousarray(V[b:b + 1, :, 7:8]), t)
        for a, c in zip(pa, p1):
            assert np.array_equal(a.reshape(B, -1)[b], c)

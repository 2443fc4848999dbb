"""Pins of the oracle's channel-wise key groups with a full-precision residual buffer (Sec. 4 "Downstream Task
Accuracy": the per-column back-end and its 64-token residual buffer) against things other than itself: a vectorized
numpy statement of the same quantizer applied to columns, array-transpose statements of the plane layouts, the
buffer's life cycle (what is stored raw, what is flushed, when), attention through torch on numpy-built tensors, and
the reason the per-column form exists (a few large key channels stop inflating every group's range)."""
import math

import numpy as np
import pytest
import torch

from paper_2502_15075_amd import synth
from test_oracle_quantizer import _expected_planes, _pack_fields_le


def _quantize_columns_numpy(X, bits):
    """Asymmetric min-max quantizer of App. B applied to every column of X [G, D], binary32 operations on whole
    arrays: returns codes [G, D], scale and zero as binary16 patterns [D]."""
    X = X.astype(np.float32)
    mn, mx = X.min(axis=0), X.max(axis=0)
    mn = np.where(mn == 0, np.float32(0), mn)
    levels = np.float32(2 ** bits - 1)
    s16 = ((mx - mn) / levels).astype(np.float32).astype(np.float16)
    s16 = np.where(s16 == 0, np.float16(0), s16)
    z16 = mn.astype(np.float16)
    s, z = s16.astype(np.float32), z16.astype(np.float32)
    with np.errstate(divide="ignore", invalid="ignore"):
        rcp = (np.float32(1) / s).astype(np.float32)
        t = ((X - z).astype(np.float32) * rcp).astype(np.float32)
    codes = np.clip(np.rint(t), 0, levels)
    codes = np.where(s == 0, 0, codes).astype(np.uint8)
    return codes, s16.view(np.uint16), z16.view(np.uint16)


def _quantize_rows_numpy(X, bits, G):
    T, D = X.shape
    codes = np.zeros((T, D), np.uint8)
    S = np.zeros((T, D // G), np.uint16)
    Z = np.zeros((T, D // G), np.uint16)
    for g in range(D // G):
        c, s, z = _quantize_columns_numpy(X[:, g * G:(g + 1) * G].T, bits)
        codes[:, g * G:(g + 1) * G], S[:, g], Z[:, g] = c.T, s, z
    return codes, S, Z


@pytest.mark.parametrize("G,bk,bv,gv", [(64, 4, 2, 64), (32, 2, 4, 128), (128, 8, 8, 32), (64, 6, 1, 64), (64, 3, 6, 32),
                                        (32, 1, 3, 64)])
def test_flushed_blocks_match_numpy_and_the_residual_holds_the_tail(oracle, G, bk, bv, gv):
    rng = np.random.default_rng(G + bk)
    B, H, D = 2, 2, 128
    T = 2 * G + 37 if G < 128 else 2 * G + 5
    cap = -(-T // max(32, G)) * max(32, G)
    K = (rng.standard_normal((B, H, T, D)) * 3).astype(np.float16)
    K[..., [5, 37]] *= 20
    V = rng.standard_normal((B, H, T, D)).astype(np.float16)
    L = oracle.Layout(B, H, T, D, bk, bv, G, gv, axis_k=1)
    planes = oracle.new_seq_planes(L, fill=0xA5)
    assert [p.size for p in planes] == [B * H * cap * 16 * bk, B * H * (cap // G) * D * 4, B * H * cap * 16 * bv,
                                        B * H * cap * (D // gv) * 4, B * H * G * D * 2, B * H * G * D * 2]
    oracle.seq_append(L, planes, K, V, 0)
    nq = T // G * G
    for bh in range(B * H):
        Kb, Vb = K.reshape(B * H, T, D)[bh], V.reshape(B * H, T, D)[bh]
        codes = np.zeros((cap, D), np.uint8)
        meta = np.zeros((cap // G, D, 2), np.uint16)
        for blk in range(nq // G):
            c, s, z = _quantize_columns_numpy(Kb[blk * G:(blk + 1) * G], bk)
            codes[blk * G:(blk + 1) * G] = c
            meta[blk, :, 0], meta[blk, :, 1] = s, z
        k_plane = _pack_key_rows_numpy(codes, bk)
        got_k = planes[0].reshape(B * H, -1)[bh]
        assert np.array_equal(got_k[:nq * 16 * bk], k_plane[:nq * 16 * bk])
        assert (got_k[nq * 16 * bk:] == 0xA5).all()                       # nothing beyond the flushed blocks is written
        got_m = planes[1].reshape(B * H, -1)[bh]
        assert np.array_equal(got_m[:(nq // G) * D * 4], meta[:nq // G].view(np.uint8).ravel())
        assert (got_m[(nq // G) * D * 4:] == 0xA5).all()
        # values: the token-wise planes of the flushed tokens
        vcodes, S, Z = _quantize_rows_numpy(np.concatenate([Vb[:nq].astype(np.float32), np.zeros((cap - nq, D), np.float32)]), bv, gv)
        vmeta, v_plane = _expected_planes(vcodes, S, Z, 8, gv)[1], _pack_value_blocks_numpy(vcodes, S, Z, bv, gv)
        got_v = planes[2].reshape(B * H, -1)[bh]
        assert np.array_equal(got_v[:nq * 16 * bv], v_plane[:nq * 16 * bv]) and (got_v[nq * 16 * bv:] == 0xA5).all()
        got_vm = planes[3].reshape(B * H, -1)[bh]
        assert np.array_equal(got_vm[:nq * (D // gv) * 4], vmeta[:nq * (D // gv) * 4])
        # residual: slot t % G of the newest tokens; keys row-major, values in the 16-bit block order
        kr = planes[4].reshape(B * H, G, D * 2)[bh].view(np.float16).reshape(G, D)
        for t in range(nq, T):
            assert np.array_equal(kr[t % G], Kb[t])
        slots = np.zeros((G, D), np.uint16)
        live = np.zeros((G, D), bool)
        for t in range(T - G if T >= G else 0, T):                       # last writer of every slot
            slots[t % G] = Vb[t].view(np.uint16)
            live[t % G] = True
        _, _, vr_plane = _expected_planes(slots, np.zeros((G, 1), np.uint16), np.zeros((G, 1), np.uint16), 16, 128)
        _, _, live_plane = _expected_planes(live.astype(np.uint16) * 0xFFFF, np.zeros((G, 1), np.uint16), np.zeros((G, 1), np.uint16), 16, 128)
        got_vr = planes[5].reshape(B * H, -1)[bh]
        assert np.array_equal(got_vr & live_plane, vr_plane & live_plane)
        assert ((got_vr | live_plane) == np.where(live_plane == 0xFF, 0xFF, 0xA5)).all()


def test_chunked_appends_compose(oracle):
    rng = np.random.default_rng(3)
    B, H, T, D, G = 1, 2, 200, 128, 64
    K = rng.standard_normal((B, H, T, D)).astype(np.float16)
    V = rng.standard_normal((B, H, T, D)).astype(np.float16)
    L = oracle.Layout(B, H, T, D, 4, 2, G, 64, axis_k=1)
    whole = oracle.new_seq_planes(L, fill=0x5A)
    oracle.seq_append(L, whole, K, V, 0)
    parts = oracle.new_seq_planes(L, fill=0x5A)
    for a, b in ((0, 1), (1, 63), (63, 64), (64, 65), (65, 191), (191, 192), (192, 200)):
        oracle.seq_append(L, parts, np.ascontiguousarray(K[:, :, a:b]), np.ascontiguousarray(V[:, :, a:b]), a)
    for p, w in zip(parts, whole):
        assert np.array_equal(p, w)


def test_what_attention_sees(oracle):
    """Flushed tokens: code * scale + zero with the column's scale/zero (numpy); newest tokens: the inputs exactly.
    Attention over the mix equals torch's softmax attention on those tensors; below one block nothing is quantized."""
    rng = np.random.default_rng(8)
    B, Hk, Hq, T, D, G = 1, 2, 4, 150, 128, 64
    K = (rng.standard_normal((B, Hk, T, D)) * 2).astype(np.float16)
    V = rng.standard_normal((B, Hk, T, D)).astype(np.float16)
    q = rng.standard_normal((B, Hq, D)).astype(np.float16)
    scale = 1 / math.sqrt(D)
    L = oracle.Layout(B, Hk, T, D, 4, 2, G, 64, axis_k=1)
    planes = oracle.new_seq_planes(L)
    oracle.seq_append(L, planes, K, V, 0)
    for seq_len in (150, 128, 127, 64, 63, 1):
        # the cache state at seq_len tokens: rebuild by appending only that many
        pl = oracle.new_seq_planes(L)
        oracle.seq_append(L, pl, np.ascontiguousarray(K[:, :, :seq_len]), np.ascontiguousarray(V[:, :, :seq_len]), 0)
        kd, vd = oracle.seq_dequantize(L, pl, seq_len, 0, seq_len)
        nq = seq_len // G * G
        want_k = K[:, :, :seq_len].astype(np.float32).copy()
        want_v = V[:, :, :seq_len].astype(np.float32).copy()
        for h in range(Hk):
            for blk in range(nq // G):
                X = K[0, h, blk * G:(blk + 1) * G]
                c, s, z = _quantize_columns_numpy(X, 4)
                want_k[0, h, blk * G:(blk + 1) * G] = c.astype(np.float32) * s.view(np.float16).astype(np.float32) + z.view(np.float16).astype(np.float32)
            if nq:
                c, S, Z = _quantize_rows_numpy(V[0, h, :nq].astype(np.float32), 2, 64)
                sv = np.repeat(S.view(np.float16).astype(np.float32), 64, axis=1)
                zv = np.repeat(Z.view(np.float16).astype(np.float32), 64, axis=1)
                want_v[0, h, :nq] = c.astype(np.float32) * sv + zv
        assert np.array_equal(kd, want_k) and np.array_equal(vd, want_v)
        got = oracle.seq_decode_attention(L, pl, q, seq_len, scale)
        Kt = torch.from_numpy(want_k).double().repeat_interleave(Hq // Hk, dim=1)
        Vt = torch.from_numpy(want_v).double().repeat_interleave(Hq // Hk, dim=1)
        qt = torch.from_numpy(q.astype(np.float64)).unsqueeze(2)
        ref = torch.nn.functional.scaled_dot_product_attention(qt, Kt, Vt, scale=scale).squeeze(2).numpy()
        assert np.abs(got - ref).max() <= 2e-6 * np.abs(ref).max()
        if seq_len < G:
            exact = oracle.attention_dense(K[:, :, :seq_len].astype(np.float32), V[:, :, :seq_len].astype(np.float32), q, scale)
            assert np.array_equal(got, exact)


def test_per_channel_groups_tame_outlier_channels(oracle):
    """Keys with a few large channels: a token-wise group containing one of them spends its whole range on it, a
    channel-wise group does not.  Key MSE at 4 bits drops by a large factor; the half-step bound holds per column."""
    B, H, T, D, G = 2, 4, 256, 128, 64
    K, V, _ = synth.make_kvq(21, B, H, H, T, dtype=torch.float16)
    Kn, Vn = K.numpy(), V.numpy()
    Ls = oracle.Layout(B, H, T, D, 4, 2, G, 64, axis_k=1)
    ps = oracle.new_seq_planes(Ls)
    oracle.seq_append(Ls, ps, Kn, Vn, 0)
    ks, _ = oracle.seq_dequantize(Ls, ps, T, 0, T)
    Lt = oracle.Layout(B, H, T, D, 4, 2, 64, 64)
    pt = oracle.new_planes(Lt)
    oracle.quantize_append(Lt, pt, Kn, Vn, 0)
    kt, _ = oracle.dequantize(Lt, pt, 0, T)
    mse_seq, mse_tok = oracle.mse(Kn.astype(np.float32), ks), oracle.mse(Kn.astype(np.float32), kt)
    assert mse_seq < 0.4 * mse_tok
    quiet = np.setdiff1d(np.arange(D), [5, 37, 69, 101])                 # the channels that are not outliers gain most
    assert oracle.mse(Kn.astype(np.float32)[..., quiet], ks[..., quiet]) < 0.05 * oracle.mse(Kn.astype(np.float32)[..., quiet], kt[..., quiet])
    rng_col = (Kn.astype(np.float32).reshape(B, H, T // G, G, D).max(axis=3) - Kn.astype(np.float32).reshape(B, H, T // G, G, D).min(axis=3))
    step = rng_col / 15
    err = np.abs(Kn.astype(np.float32) - ks).reshape(B, H, T // G, G, D).max(axis=3)
    assert (err <= step / 2 * (1 + 2 ** -9) + 1e-6).all()


def test_token_wise_entry_points_refuse_channel_wise_layouts(oracle):
    L = oracle.Layout(1, 1, 64, 128, 4, 2, 64, 64, axis_k=1)
    x = np.zeros((1, 1, 4, 128), np.float16)
    with pytest.raises(ValueError):
        oracle.quantize_append(L, oracle.new_planes(L), x, x, 0)
    with pytest.raises(ValueError):
        oracle.seq_append(oracle.Layout(1, 1, 64, 128, 16, 2, 64, 64, axis_k=1), oracle.new_seq_planes(L), x, x, 0)


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
def test_group_quantizer_equals_the_numpy_statement_bit_for_bit(oracle, bits):
    """The oracle's one-group routine (a C loop) against the whole-array numpy statement of the same arithmetic
    (binary32, one rounding per operation) on groups built to hit ties, constant groups, tiny and huge ranges."""
    rng = np.random.default_rng(bits)
    groups = []
    for n in (32, 64, 128):
        for _ in range(60):
            scale = 2.0 ** rng.integers(-12, 10)
            x = rng.standard_normal(n) * scale
            kind = rng.integers(0, 5)
            if kind == 0:
                x = np.round(x / scale * 4) / 4 * scale                # dyadic grid: exact ties
            elif kind == 1:
                x[:] = x[0]                                            # constant group
            elif kind == 2:
                x[rng.integers(0, n)] *= 50                            # one outlier
            elif kind == 3:
                x = np.abs(x)                                          # minimum near zero, -0 never
            groups.append(x.astype(np.float16).astype(np.float32))
    for x in groups:
        codes, S, Z = oracle.quantize_group(x, bits)
        c2, s2, z2 = _quantize_columns_numpy(x[:, None], bits)
        assert S == int(s2[0]) and Z == int(z2[0])
        assert np.array_equal(codes, c2[:, 0])


def _pack_key_rows_numpy(codes, bits):
    """Key rows at their own width.  1 bit: a plain bit string.  3 and 6 bits: per chunk of 32 channels the low 2 (4)
    bits of the 32 codes as one run of fields, then their high 1 (2) bits as a second run."""
    if bits not in (3, 6):
        return _pack_fields_le(codes.ravel(), bits)
    lo = 2 if bits == 3 else 4
    T, D = codes.shape
    chunks = codes.reshape(T, D // 32, 32).astype(np.uint16)
    low = _pack_fields_le((chunks & ((1 << lo) - 1)).ravel(), lo).reshape(T, D // 32, 4 * lo)
    high = _pack_fields_le((chunks >> lo).ravel(), bits - lo).reshape(T, D // 32, 4 * (bits - lo))
    return np.concatenate([low, high], axis=2).ravel()


def _pack_value_blocks_numpy(codes, S, Z, bits, G):
    """Value blocks at their own width.  3 and 6 bits: per 32-token block the block of the codes' low 2 (4) bits in the
    2-bit (4-bit) layout, then the block of their high 1 (2) bits in the 1-bit (2-bit) layout."""
    if bits not in (3, 6):
        return _expected_planes(codes, S, Z, bits, G)[2]
    lo = 2 if bits == 3 else 4
    T = codes.shape[0]
    low = _expected_planes(codes & ((1 << lo) - 1), S, Z, lo, G)[2].reshape(T // 32, 512 * lo)
    high = _expected_planes(codes >> lo, S, Z, bits - lo, G)[2].reshape(T // 32, 512 * (bits - lo))
    return np.concatenate([low, high], axis=1).ravel()


@pytest.mark.parametrize("bits", [1, 3, 6])
def test_odd_widths_are_packed_at_their_own_width(oracle, bits):
    """1-, 3- and 6-bit codes (the per-column back-end's grid {1,2,4,6,8}, Table 1's 3-bit keys) are quantized with
    2^b - 1 steps and take b bits in both tensors: key rows D*b/8 bytes (3 and 6 bits as a low and a high run per 32
    channels), value blocks 512*b bytes (3 and 6 bits as a block of low parts and a block of high parts).  Planes =
    numpy's packing of numpy's b-bit codes, sizes accordingly, reconstruction = code * scale + zero."""
    rng = np.random.default_rng(bits)
    B, H, T, D, G = 1, 2, 64, 128, 64
    x = (rng.standard_normal((B, H, T, D)) * 2).astype(np.float16)
    L = oracle.Layout(B, H, T, D, bits, bits, G, G)
    sizes, fsizes = oracle.plane_bytes(L), oracle.plane_bytes(oracle.Layout(B, H, T, D, 8, 8, G, G))
    assert sizes[0] == sizes[2] == B * H * T * D * bits // 8 and sizes[1::2] == fsizes[1::2]
    planes = oracle.new_planes(L)
    oracle.quantize_append(L, planes, x, x, 0)
    kd, vd = oracle.dequantize(L, planes, 0, T)
    for bh in range(B * H):
        rows = x.reshape(B * H, T, D)[bh].astype(np.float32)
        codes, S, Z = _quantize_rows_numpy(rows, bits, G)
        assert codes.max() <= 2 ** bits - 1
        meta, v_plane = _expected_planes(codes, S, Z, 8, G)[1], _pack_value_blocks_numpy(codes, S, Z, bits, G)
        got = [p.reshape(B * H, -1)[bh] for p in planes]
        assert np.array_equal(got[0], _pack_key_rows_numpy(codes, bits)) and np.array_equal(got[1], meta)
        assert np.array_equal(got[2], v_plane) and np.array_equal(got[3], meta)
        want = codes.astype(np.float32) * np.repeat(S.view(np.float16).astype(np.float32), G, axis=1) \
            + np.repeat(Z.view(np.float16).astype(np.float32), G, axis=1)
        assert np.array_equal(kd.reshape(B * H, T, D)[bh], want) and np.array_equal(vd.reshape(B * H, T, D)[bh], want)


def test_three_bit_keys_against_four_bit_keys_through_the_cache(oracle):
    """Table 1 reports key MSE at 3 and 4 bits with a ratio of 4.5-4.7; (15/7)^2 = 4.59 for 2^b - 1 steps.  Through
    the whole cache path (append, planes, dequantize) on dense Gaussian keys the ratio lands there."""
    rng = np.random.default_rng(33)
    B, H, T, D = 2, 4, 256, 128
    K = rng.standard_normal((B, H, T, D)).astype(np.float16)
    mse = {}
    for b in (3, 4):
        L = oracle.Layout(B, H, T, D, b, 2, 64, 64)
        planes = oracle.new_planes(L)
        oracle.quantize_append(L, planes, K, K, 0)
        kd, _ = oracle.dequantize(L, planes, 0, T)
        mse[b] = oracle.mse(K.astype(np.float32), kd)
    assert mse[3] / mse[4] == pytest.approx((15 / 7) ** 2, rel=0.06)


def test_ragged_batch_is_each_sequence_on_its_own(oracle):
    """Per-sequence lengths with channel-wise keys: a batch whose elements have had different numbers of tokens appended
    (one of them exactly a block, one below a block, one several blocks plus a tail) holds, element by element, the
    planes of a batch of one filled the same way, and attends like it."""
    B, H, R, D = 3, 2, 2, 128
    lens = [64, 37, 150]
    K, V, q = synth.make_kvq(77, B, H, H * R, max(lens), dtype=torch.float16)
    L = oracle.Layout(B, H, 160, D, 4, 2, 64, 64, axis_k=1)
    planes = oracle.new_seq_planes(L, fill=0x5A)
    Kn, Vn, qn = K.numpy(), V.numpy(), q.numpy()
    for t in range(max(lens)):                               # token by token, only the sequences that still grow
        live = [b for b in range(B) if t < lens[b]]
        for b in live:                                       # element by element, on that element's slice of the planes
            Lb, pb = _element_of(oracle, L, planes, b)
            oracle.seq_append(Lb, pb, np.ascontiguousarray(Kn[b:b + 1, :, t:t + 1]), np.ascontiguousarray(Vn[b:b + 1, :, t:t + 1]), t)
    scale = 1 / math.sqrt(D)
    got = oracle.seq_decode_attention_varlen(L, planes, qn, lens, scale)
    for b in range(B):
        L1 = oracle.Layout(1, H, 160, D, 4, 2, 64, 64, axis_k=1)
        p1 = oracle.new_seq_planes(L1, fill=0x5A)
        oracle.seq_append(L1, p1, np.ascontiguousarray(Kn[b:b + 1, :, :lens[b]]), np.ascontiguousarray(Vn[b:b + 1, :, :lens[b]]), 0)
        want = oracle.seq_decode_attention(L1, p1, qn[b:b + 1], lens[b], scale)
        assert np.array_equal(got[b], want[0])
        for whole, single in zip(planes, p1):
            assert np.array_equal(whole.reshape(B, -1)[b], single)
    # one more token for every element at its own position
    Kx, Vx, _ = synth.make_kvq(78, B, H, H * R, 1, dtype=torch.float16)
    oracle.seq_append_at(L, planes, Kx.numpy(), Vx.numpy(), lens)
    got = oracle.seq_decode_attention_varlen(L, planes, qn, [n + 1 for n in lens], scale)
    assert np.isfinite(got).all() and got.shape == (B, H * R, D)


def _element_of(oracle, L, planes, b):
    from dataclasses import replace
    return replace(L, batch=1), [p.reshape(L.batch, -1)[b] if p.size else p for p in planes]


# --------------------------------------------------------------------------- key rotation on the per-column back-end

ROT_SIGNS = (0x9E3779B9, 0x7F4A7C15, 0xF39CC060, 0x5CEDC834)


def _rotate_rows(oracle, X, signs):
    """R x for every row of X (the oracle's single-vector rotation, itself pinned against scipy's Hadamard matrix)."""
    return np.stack([oracle.rotate(r, signs) for r in X.astype(np.float32)])


@pytest.mark.parametrize("G,bk,bv", [(64, 4, 2), (32, 2, 4), (128, 8, 8), (64, 3, 2)])
def test_rotated_channelwise_planes_are_those_of_the_rotated_rows(oracle, G, bk, bv):
    """Sec. 5.3's best setting (key-only rotation) on Sec. 4's per-column keys: the flushed code and scale/zero planes
    of a cache with rotate_k equal those of a cache WITHOUT rotation that is fed the rotated rows R k (binary32, no
    rounding on the way to the quantizer); the residual buffers keep the input rows; value planes do not change."""
    rng = np.random.default_rng(G * 7 + bk)
    B, H, D = 1, 2, 128
    T = 2 * G + 19
    K = (rng.standard_normal((B, H, T, D)) * 3).astype(np.float16)
    K[..., [5, 37, 69, 101]] *= 20
    V = rng.standard_normal((B, H, T, D)).astype(np.float16)
    Lr = oracle.Layout(B, H, T, D, bk, bv, G, 64, axis_k=1, rotate_k=1, signs_k=ROT_SIGNS)
    Lp = oracle.Layout(B, H, T, D, bk, bv, G, 64, axis_k=1)
    rot = oracle.new_seq_planes(Lr, fill=0xA5)
    oracle.seq_append(Lr, rot, K, V, 0)
    nq = T // G * G
    for h in range(H):
        Kr = _rotate_rows(oracle, K[0, h, :nq], ROT_SIGNS)                       # binary32 rows R k
        for blk in range(nq // G):
            c, s, z = _quantize_columns_numpy(Kr[blk * G:(blk + 1) * G], bk)
            meta = rot[1].reshape(B * H, -1)[h].view(np.uint16).reshape(-1, D, 2)[blk]
            assert np.array_equal(meta[:, 0], s) and np.array_equal(meta[:, 1], z)
            rows = rot[0].reshape(B * H, -1, 16 * bk)[h][blk * G:(blk + 1) * G]
            assert np.array_equal(rows.ravel(), _pack_key_rows_numpy(c, bk)[:G * 16 * bk])
        kr = rot[4].reshape(B * H, G, D * 2)[h].view(np.float16).reshape(G, D)
        for t in range(nq, T):
            assert np.array_equal(kr[t % G], K[0, h, t])                         # the buffer keeps the input row
    plain = oracle.new_seq_planes(Lp, fill=0xA5)
    oracle.seq_append(Lp, plain, K, V, 0)
    for i in (2, 3, 5):
        assert np.array_equal(rot[i], plain[i])                                  # values: untouched by the key rotation
    assert not np.array_equal(rot[0], plain[0])


def test_rotated_channelwise_attention(oracle):
    """What attention computes with rotated channel-wise keys, written out with numpy and torch: flushed tokens score
    binary16(R q) against the stored reconstruction of R k, tail tokens score q against the input rows, one softmax
    over all, values as always.  And the reconstruction handed out is in the input basis: R^T of what is stored."""
    rng = np.random.default_rng(21)
    B, Hk, Hq, T, D, G = 1, 2, 4, 150, 128, 64
    K = (rng.standard_normal((B, Hk, T, D)) * 2).astype(np.float16)
    K[..., [5, 37]] *= 15
    V = rng.standard_normal((B, Hk, T, D)).astype(np.float16)
    q = rng.standard_normal((B, Hq, D)).astype(np.float16)
    scale = 1 / math.sqrt(D)
    L = oracle.Layout(B, Hk, T, D, 4, 2, G, 64, axis_k=1, rotate_k=1, signs_k=ROT_SIGNS)
    for seq_len in (150, 128, 70, 63):
        pl = oracle.new_seq_planes(L)
        oracle.seq_append(L, pl, np.ascontiguousarray(K[:, :, :seq_len]), np.ascontiguousarray(V[:, :, :seq_len]), 0)
        nq = seq_len // G * G
        kd, vd = oracle.seq_dequantize(L, pl, seq_len, 0, seq_len)
        got = oracle.seq_decode_attention(L, pl, q, seq_len, scale)
        ref = np.zeros((B, Hq, D))
        for hq in range(Hq):
            hk = hq // (Hq // Hk)
            stored = np.zeros((seq_len, D), np.float32)
            for blk in range(nq // G):
                Kr = _rotate_rows(oracle, K[0, hk, blk * G:(blk + 1) * G], ROT_SIGNS)
                c, s, z = _quantize_columns_numpy(Kr, 4)
                stored[blk * G:(blk + 1) * G] = c.astype(np.float32) * s.view(np.float16).astype(np.float32) + z.view(np.float16).astype(np.float32)
            stored[nq:] = K[0, hk, nq:seq_len].astype(np.float32)
            # the reconstruction in the input basis: R^T of the stored flushed rows, the tail as it is
            back = stored.copy()
            for t in range(nq):
                back[t] = oracle.unrotate(stored[t], ROT_SIGNS)
            assert np.array_equal(kd[0, hk], back)
            qr = oracle.rotate(q[0, hq].astype(np.float32), ROT_SIGNS).astype(np.float16).astype(np.float64)
            logits = np.concatenate([stored[:nq].astype(np.float64) @ qr, stored[nq:].astype(np.float64) @ q[0, hq].astype(np.float64)]) * scale
            p = torch.softmax(torch.from_numpy(logits), dim=0).numpy()
            ref[0, hq] = p @ vd[0, hk].astype(np.float64)
        assert np.abs(got - ref).max() <= 2e-6 * np.abs(ref).max()
    # the rotation leaves the scores where they were: with 8-bit keys the output stays close to exact attention
    L8 = oracle.Layout(B, Hk, T, D, 8, 8, G, 64, axis_k=1, rotate_k=1, signs_k=ROT_SIGNS)
    pl = oracle.new_seq_planes(L8)
    oracle.seq_append(L8, pl, K, V, 0)
    exact = oracle.attention_dense(K.astype(np.float32), V.astype(np.float32), q, scale)
    got = oracle.seq_decode_attention(L8, pl, q, T, scale)
    assert np.abs(got - exact).max() < 0.05 * np.abs(exact).max()


def test_rotation_and_per_column_groups_on_outlier_channels(oracle):
    """The two remedies for a few large key channels, and their combination (Sec. 5.3 on Sec. 4's back-end), on keys
    that are independent draws with four channels scaled by 20: token-wise groups waste their range on the large
    channel (MSE 1.5 at 4 bits), per-column groups isolate it (0.42), the rotation spreads it over all channels
    (0.22); rotating in front of per-column groups neither helps nor hurts on such keys (columns of R k all have the
    same spread): the combination is there for keys whose columns differ, not expected to win here."""
    rng = np.random.default_rng(5)
    B, H, T, D, G = 1, 4, 256, 128, 64
    K = (rng.standard_normal((B, H, T, D)) * 2).astype(np.float32)
    K[..., [5, 37, 69, 101]] *= 20
    K16 = K.astype(np.float16)
    V = rng.standard_normal((B, H, T, D)).astype(np.float16)
    err = {}
    for axis in (0, 1):
        for rot in (0, 1):
            L = oracle.Layout(B, H, T, D, 4, 2, G, 64, axis_k=axis, rotate_k=rot, signs_k=ROT_SIGNS if rot else (0, 0, 0, 0))
            if axis:
                pl = oracle.new_seq_planes(L)
                oracle.seq_append(L, pl, K16, V, 0)
                kd, _ = oracle.seq_dequantize(L, pl, T, 0, T)
            else:
                pl = oracle.new_planes(L)
                oracle.quantize_append(L, pl, K16, V, 0)
                kd, _ = oracle.dequantize(L, pl, 0, T)
            err[axis, rot] = oracle.mse(K16.astype(np.float32), kd)
    assert err[0, 1] < err[1, 0] < 0.5 * err[0, 0]
    assert abs(err[1, 1] / err[1, 0] - 1) < 0.15


# --------------------------------------------------------------------------- the buffer's length as a parameter of its own

@pytest.mark.parametrize("G,RL,bk,bv", [(128, 64, 4, 2), (64, 64, 2, 4), (32, 128, 8, 8), (128, 32, 3, 2)])
def test_token_wise_keys_behind_a_residual_buffer(oracle, G, RL, bk, bv):
    """The downstream runs' pairing (Sec. 4: a 64-token full-precision buffer in front of 128-element groups, which can
    only run along head_dim): keys token-wise as on the plain path, the newest n mod RL tokens still in the buffer.
    Flushed planes = the plain token-wise planes of the same tokens (that path has its own numpy pins), nothing is
    written beyond them, the buffer holds the tail, attention sees reconstruction + tail."""
    rng = np.random.default_rng(G + RL)
    B, Hk, Hq, D = 1, 2, 4, 128
    T = 2 * RL + 21
    K = (rng.standard_normal((B, Hk, T, D)) * 3).astype(np.float16)
    V = rng.standard_normal((B, Hk, T, D)).astype(np.float16)
    q = rng.standard_normal((B, Hq, D)).astype(np.float16)
    L = oracle.Layout(B, Hk, T, D, bk, bv, G, 64, resid_len=RL)
    pl = oracle.new_seq_planes(L, fill=0xA5)
    cap = -(-T // max(32, RL)) * max(32, RL)
    assert [p.size for p in pl] == [B * Hk * cap * 16 * bk, B * Hk * cap * (D // G) * 4, B * Hk * cap * 16 * bv,
                                    B * Hk * cap * 2 * 4, B * Hk * RL * D * 2, B * Hk * RL * D * 2]
    for a, b in ((0, 1), (1, RL - 1), (RL - 1, RL + 3), (RL + 3, T)):
        oracle.seq_append(L, pl, np.ascontiguousarray(K[:, :, a:b]), np.ascontiguousarray(V[:, :, a:b]), a)
    nq = T // RL * RL
    Lp = oracle.Layout(B, Hk, cap, D, bk, bv, G, 64)
    plain = oracle.new_planes(Lp, fill=0xA5)
    oracle.quantize_append(Lp, plain, np.ascontiguousarray(K[:, :, :nq]), np.ascontiguousarray(V[:, :, :nq]), 0)
    for got, want in zip(pl[:4], plain):
        assert np.array_equal(got, want)                                 # flushed tokens as on the plain path, the rest untouched
    kr = pl[4].reshape(B * Hk, RL, D * 2).view(np.float16).reshape(B * Hk, RL, D)
    for t in range(nq, T):
        assert np.array_equal(kr[:, t % RL], K.reshape(B * Hk, T, D)[:, t])
    kd, vd = oracle.seq_dequantize(L, pl, T, 0, T)
    kp, vp = oracle.dequantize(Lp, plain, 0, nq)
    assert np.array_equal(kd[:, :, :nq], kp) and np.array_equal(vd[:, :, :nq], vp)
    assert np.array_equal(kd[:, :, nq:], K[:, :, nq:].astype(np.float32)) and np.array_equal(vd[:, :, nq:], V[:, :, nq:].astype(np.float32))
    got = oracle.seq_decode_attention(L, pl, q, T, 1 / math.sqrt(D))
    Kt = torch.from_numpy(kd).double().repeat_interleave(Hq // Hk, dim=1)
    Vt = torch.from_numpy(vd).double().repeat_interleave(Hq // Hk, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(torch.from_numpy(q.astype(np.float64)).unsqueeze(2), Kt, Vt,
                                                           scale=1 / math.sqrt(D)).squeeze(2).numpy()
    assert np.abs(got - ref).max() <= 2e-6 * np.abs(ref).max()
    # the plain entry points refuse a layout with a buffer (its tail is not in the planes)
    with pytest.raises(ValueError):
        oracle.quantize_append(L, pl[:4], K, V, 0)


@pytest.mark.parametrize("G,RL,bk", [(32, 64, 4), (32, 128, 2), (64, 128, 8), (128, 128, 4)])
def test_channel_wise_groups_shorter_than_the_buffer(oracle, G, RL, bk):
    """A flush of RL tokens quantizes RL / G groups per channel (numpy column quantizer per group), and happens only
    when the buffer is full: with 32-token groups and a 64-token buffer, tokens 64..95 of a 100-token sequence are
    still in the buffer although they would fill a group."""
    rng = np.random.default_rng(G * 3 + RL)
    B, H, D = 1, 2, 128
    T = 2 * RL + RL // 2 + 5
    K = (rng.standard_normal((B, H, T, D)) * 3).astype(np.float16)
    K[..., [5, 37]] *= 20
    V = rng.standard_normal((B, H, T, D)).astype(np.float16)
    L = oracle.Layout(B, H, T, D, bk, 2, G, 64, axis_k=1, resid_len=RL)
    pl = oracle.new_seq_planes(L, fill=0xA5)
    oracle.seq_append(L, pl, K, V, 0)
    nq = T // RL * RL
    cap = -(-T // RL) * RL
    assert pl[1].size == B * H * (cap // G) * D * 4 and pl[4].size == B * H * RL * D * 2
    for h in range(H):
        for grp in range(nq // G):
            c, s, z = _quantize_columns_numpy(K[0, h, grp * G:(grp + 1) * G], bk)
            meta = pl[1].reshape(B * H, -1)[h].view(np.uint16).reshape(-1, D, 2)[grp]
            assert np.array_equal(meta[:, 0], s) and np.array_equal(meta[:, 1], z)
            rows = pl[0].reshape(B * H, -1, 16 * bk)[h][grp * G:(grp + 1) * G]
            assert np.array_equal(rows.ravel(), _pack_key_rows_numpy(c, bk)[:G * 16 * bk])
        assert (pl[0].reshape(B * H, -1)[h][nq * 16 * bk:] == 0xA5).all()            # nothing beyond the flushed tokens
        assert (pl[1].reshape(B * H, -1)[h][(nq // G) * D * 4:] == 0xA5).all()
        kr = pl[4].reshape(B * H, RL, D * 2)[h].view(np.float16).reshape(RL, D)
        for t in range(nq, T):
            assert np.array_equal(kr[t % RL], K[0, h, t])
    parts = oracle.new_seq_planes(L, fill=0xA5)
    for a, b in ((0, 3), (3, RL), (RL, RL + 1), (RL + 1, T)):
        oracle.seq_append(L, parts, np.ascontiguousarray(K[:, :, a:b]), np.ascontiguousarray(V[:, :, a:b]), a)
    for x, y in zip(parts, pl):
        assert np.array_equal(x, y)

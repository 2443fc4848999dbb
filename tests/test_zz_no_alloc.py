"""kvq_decode_attention_static, the entry point for callers that cannot allocate (its partial records live in a static
device array of the library): through the C ABI, against kvq_decode_attention with a caller workspace, on two calls in a
row, the second with a smaller input.  Both run the same kernels, so the outputs must be identical bit for bit; the
first is also held to the oracle's bar."""
import math

import numpy as np
import pytest
import torch

from paper_2502_15075_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kvq():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2502_15075_amd import kvq as m
    m.load()
    return m


def _one_call(kvq, oracle, seed, B, Hkv, Hq, T, bk, bv, check_oracle):
    scale = 1 / math.sqrt(128)
    K, V, q = synth.make_kvq(seed, B, Hkv, Hq, T, dtype=torch.bfloat16)
    L = kvq.Layout(B, Hkv, T, 128, bk, bv, 64, 64)
    cache = kvq.Cache(L, fill=0)
    kvq.quantize_append(L, cache, K.cuda(), V.cuda(), 0)
    need = kvq.decode_workspace_bytes(L, Hq, T)
    assert 0 < need <= kvq.STATIC_SCRATCH_BYTES, "the case must split the sequence, or the scratch array is not used"
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    want = torch.empty(B, Hq, 128, dtype=torch.float32, device="cuda")
    got = torch.full((B, Hq, 128), float("nan"), dtype=torch.float32, device="cuda")
    kvq.decode_attention(L, cache, q.cuda(), T, scale, want, ws)
    kvq.decode_attention_static(L, cache, q.cuda(), T, scale, got)
    torch.cuda.synchronize()
    assert torch.equal(got, want), float((got - want).abs().max())
    if check_oracle:
        Lo = oracle.Layout(B, Hkv, T, 128, bk, bv, 64, 64)
        planes = oracle.new_planes(Lo)
        oracle.quantize_append(Lo, planes, synth.to_numpy_bits(K), synth.to_numpy_bits(V), 0, bf16=True)
        ref = oracle.decode_attention(Lo, planes, synth.to_numpy_bits(q), T, scale, bf16=True).astype(np.float64)
        err = float((np.abs(got.cpu().numpy() - ref).max(axis=-1) / np.abs(ref).max(axis=-1)).max())
        assert err < 2e-3, err


def test_static_scratch_matches_the_workspace_call_twice_in_a_row(kvq, oracle):
    # B=2, 2 KV heads: 4 streams, so the sequence is split many ways and the merge kernel reads the records
    _one_call(kvq, oracle, 71, 2, 2, 8, 3000, 4, 2, True)
    # a smaller input right after it: fewer splits, fewer records; what the first call left behind must not be read
    _one_call(kvq, oracle, 72, 1, 2, 4, 1500, 2, 4, True)


def test_static_scratch_rejects_what_does_not_fit(kvq):
    """Token-wise caches never need more than about 1 MiB of records (the plan splits a sequence only while there are
    fewer than 256 streams).  Channel-wise keys add one record per query head for the residual tail whatever the batch:
    1024 sequences of 8 heads need 2 x 8192 records = 8.25 MiB, more than the array holds."""
    B, Hq, T = 1024, 8, 100
    L = kvq.Layout(B, 1, T, 128, 4, 2, 64, 64, axis_k=kvq.AXIS_SEQ)
    assert kvq.decode_workspace_bytes(L, Hq, T) > kvq.STATIC_SCRATCH_BYTES
    cache = kvq.Cache(L, fill=0)
    q = torch.zeros(B, Hq, 128, dtype=torch.float16, device="cuda")
    out = torch.empty(B, Hq, 128, dtype=torch.float32, device="cuda")
    with pytest.raises(kvq.KvqError) as e:
        kvq.decode_attention_static(L, cache, q, T, 0.1, out)
    assert e.value.status == kvq.ERR_STATIC_SCRATCH
    # the same layout with fewer sequences fits and runs (63 tokens: nothing flushed, no record at all)
    assert kvq.decode_workspace_bytes(L, Hq, 63) == 0

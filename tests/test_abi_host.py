"""Host-side checks of libkvq's C ABI that need no GPU: the library loads, exports every symbol the header
declares, sizes follow the closed forms, and every argument error is reported before anything is launched."""
import ctypes as C
import os
import re

import pytest
from dataclasses import replace

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def kvq():
    from paper_2502_15075_amd import kvq as m
    if not os.path.exists(m.LIB_PATH):
        from paper_2502_15075_amd import build
        build.build_lib()
    m.load()
    return m


def test_every_declared_symbol_is_exported(kvq):
    header = open(os.path.join(ROOT, "include", "kvq.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(kvq_[a-z_]+)\s*\(", header))
    assert {"kvq_cache_bytes", "kvq_decode_workspace_bytes", "kvq_quantize_append", "kvq_decode_attention",
            "kvq_decode_step", "kvq_dequantize", "kvq_reconstruction_error", "kvq_residual_bytes", "kvq_selftest_quantizer",
            "kvq_decode_attention_varlen", "kvq_decode_step_varlen", "kvq_status_string"} <= declared
    lib = C.CDLL(kvq.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_status_strings(kvq):
    seen = {kvq.status_string(i) for i in range(7)}
    assert len(seen) == 7 and "ok" in seen
    assert kvq.status_string(99) == "unknown status"


def test_cache_bytes_closed_forms(kvq):
    """bytes per (b, h, token): 16 b_K + 16 b_V code bytes and 4 bytes per group of scale/zero (Sec. 1: K4V2 code
    bytes are 3/4 of K4V4's)."""
    rows = 8 * 8 * 8192
    a = kvq.cache_bytes(kvq.Layout(8, 8, 8192, 128, 4, 2, 64, 64))
    b = kvq.cache_bytes(kvq.Layout(8, 8, 8192, 128, 4, 4, 64, 64))
    assert a == [rows * 64, rows * 8, rows * 32, rows * 8] and sum(a) == rows * 112
    assert (a[0] + a[2]) / (b[0] + b[2]) == 0.75 and sum(b) == rows * 144
    assert sum(kvq.cache_bytes(kvq.Layout(1, 8, 1024, 128, 4, 2, 32, 32))) == 8 * 1024 * 128
    assert sum(kvq.cache_bytes(kvq.Layout(32, 8, 32768, 128, 4, 2, 64, 64))) == 896 << 20
    assert sum(kvq.cache_bytes(kvq.Layout(1, 1, 65, 128, 8, 8, 64, 64))) == 96 * 272        # capacity rounds up to 32
    raw = kvq.cache_bytes(kvq.Layout(2, 2, 64, 128, 16, 16, 64, 64))
    assert raw == [2 * 2 * 64 * 256, 0, 2 * 2 * 64 * 256, 0]
    # paged planes: pool of n_pages pages, each one head's share of a 256-token cache per KV head
    assert kvq.cache_bytes(kvq.Layout(5, 2, 1000, 128, 4, 2, 64, 64, page_tokens=256, n_pages=11)) == \
        [11 * 2 * 256 * 64, 11 * 2 * 256 * 8, 11 * 2 * 256 * 32, 11 * 2 * 256 * 8]
    # codes of both tensors take 16 b bytes per token at every width
    k3v1 = kvq.cache_bytes(kvq.Layout(2, 2, 64, 128, 3, 1))
    assert k3v1 == [4 * 64 * 48, k3v1[1], 4 * 64 * 16, k3v1[3]] and k3v1[1::2] == kvq.cache_bytes(kvq.Layout(2, 2, 64, 128, 4, 2))[1::2]
    assert sum(kvq.cache_bytes(kvq.Layout(32, 8, 32768, 128, 4, 1, 64, 64))) == 96 * 32 * 8 * 32768
    assert kvq.cache_bytes(kvq.Layout(2, 2, 64, 128, 6, 6))[0::2] == [4 * 64 * 96, 4 * 64 * 96]
    assert kvq.cache_bytes(kvq.Layout(2, 2, 64, 128, 1, 3))[0::2] == [4 * 64 * 16, 4 * 64 * 48]
    # channel-wise keys: capacity in blocks of 64 tokens, 4 bytes per channel and block, two 64-slot residual buffers
    Ls = kvq.Layout(2, 3, 100, 128, 4, 2, 64, 32, axis_k=kvq.AXIS_SEQ)
    assert kvq.cache_bytes(Ls) == [6 * 128 * 64, 6 * 2 * 512, 6 * 128 * 32, 6 * 128 * 16]
    assert kvq.residual_bytes(Ls) == [6 * 64 * 256, 6 * 64 * 256]
    # ... in paged planes: the pool holds the code and scale/zero planes (128/64 blocks of scale/zero per page and head),
    # the residual buffers stay per sequence
    Lp = kvq.Layout(2, 3, 1000, 128, 4, 2, 64, 32, axis_k=kvq.AXIS_SEQ, page_tokens=128, n_pages=20)
    assert kvq.cache_bytes(Lp) == [20 * 3 * 128 * 64, 20 * 3 * 2 * 512, 20 * 3 * 128 * 32, 20 * 3 * 128 * 16]
    assert kvq.residual_bytes(Lp) == [6 * 64 * 256, 6 * 64 * 256]
    # the workspace of a channel-wise cache always counts the record of the residual tail once there are flushed blocks
    assert kvq.decode_workspace_bytes(Ls, 12, 63) == 0
    assert kvq.decode_workspace_bytes(Ls, 12, 64) == kvq.decode_workspace_bytes(Ls, 12, 100) > 0
    assert kvq.residual_bytes(kvq.Layout(2, 3, 100)) == [0, 0]
    # key groups of 32 tokens behind a 64-slot buffer, of 128 tokens behind a 128-slot one (the capacity is rounded up to
    # the buffer's length; 4 bytes per channel and group)
    L32 = kvq.Layout(2, 3, 100, 128, 4, 2, 32, 32, axis_k=kvq.AXIS_SEQ, resid_len=64)
    assert kvq.cache_bytes(L32) == [6 * 128 * 64, 6 * 4 * 512, 6 * 128 * 32, 6 * 128 * 16] and kvq.residual_bytes(L32) == [6 * 64 * 256] * 2
    L128 = kvq.Layout(2, 3, 130, 128, 4, 2, 128, 32, axis_k=kvq.AXIS_SEQ)
    assert kvq.cache_bytes(L128) == [6 * 256 * 64, 6 * 2 * 512, 6 * 256 * 32, 6 * 256 * 16] and kvq.residual_bytes(L128) == [6 * 128 * 256] * 2
    assert kvq.cache_bytes(replace(L128, resid_len=128)) == kvq.cache_bytes(L128)


def test_sizes_agree_with_the_oracle(kvq, oracle):
    for args in ((1, 8, 1024, 128, 4, 2, 32, 32), (3, 2, 77, 128, 2, 8, 128, 64), (2, 2, 33, 128, 16, 4, 64, 32)):
        assert kvq.cache_bytes(kvq.Layout(*args)) == oracle.plane_bytes(oracle.Layout(*args))
    for gk, rl in ((64, 0), (32, 64), (128, 128), (128, 0), (64, 128), (32, 128)):
        Lg = kvq.Layout(3, 2, 77, 128, 4, 2, gk, 32, axis_k=kvq.AXIS_SEQ, resid_len=rl)
        Lo = oracle.Layout(3, 2, 77, 128, 4, 2, gk, 32, axis_k=1, resid_len=rl)
        assert kvq.cache_bytes(Lg) + kvq.residual_bytes(Lg) == [p.size for p in oracle.new_seq_planes(Lo)], (gk, rl)


def test_workspace_plan(kvq):
    # 256 (b,h) streams fill the chip without splitting the sequence: no workspace at all
    assert kvq.decode_workspace_bytes(kvq.Layout(32, 8, 32768), 64, 32768) == 0
    # few streams, long context: (splits) x (B x H_q) records of 132 floats, then one 8-byte counter per (b, h_kv)
    n = kvq.decode_workspace_bytes(kvq.Layout(1, 8, 131072), 32, 131072)
    assert n > 64 and (n - 64) % (32 * 132 * 4) == 0
    assert kvq.decode_workspace_bytes(kvq.Layout(1, 8, 131072), 32, 40) <= n


def _status(fn, *a):
    with pytest.raises(Exception) as e:
        fn(*a)
    return e.value.status


def test_layout_errors(kvq):
    bad = [
        (kvq.Layout(0, 8, 64), kvq.ERR_INVALID_ARG), (kvq.Layout(1, 8, 0), kvq.ERR_INVALID_ARG),
        (kvq.Layout(1, 8, 64, 128, 7, 2), kvq.ERR_INVALID_ARG), (kvq.Layout(1, 8, 64, 128, 4, 5), kvq.ERR_INVALID_ARG),
        (kvq.Layout(1, 8, 64, 128, 4, 2, 48, 64), kvq.ERR_INVALID_ARG), (kvq.Layout(1, 8, 64, 128, 4, 2, 64, 256), kvq.ERR_INVALID_ARG),
        (kvq.Layout(1, 8, 64, 64), kvq.ERR_UNSUPPORTED), (kvq.Layout(1, 8, 64, 128, 4, 2, 32, 64, axis_k=1), kvq.ERR_UNSUPPORTED),
        (kvq.Layout(1, 8, 64, 128, 4, 2, 64, 64, axis_v=1), kvq.ERR_UNSUPPORTED),
        (kvq.Layout(1, 8, 64, 128, 16, 16, 64, 64, axis_k=1), kvq.ERR_INVALID_ARG),      # residual buffer + unquantized planes
        (kvq.Layout(1, 8, 64, 128, 4, 2, 64, 64, axis_v=7), kvq.ERR_INVALID_ARG),
        (kvq.Layout(1, 8, 64, 128, 4, 2, 64, 64, raw_dtype=2), kvq.ERR_INVALID_ARG),
        (kvq.Layout(1, 8, 1 << 25), kvq.ERR_UNSUPPORTED),
        (kvq.Layout(1, 8, 64, page_tokens=48, n_pages=4), kvq.ERR_INVALID_ARG), (kvq.Layout(1, 8, 64, page_tokens=32, n_pages=4), kvq.ERR_INVALID_ARG),
        (kvq.Layout(1, 8, 64, page_tokens=64, n_pages=0), kvq.ERR_INVALID_ARG),
        (kvq.Layout(1, 8, 64, rotate_k=2), kvq.ERR_INVALID_ARG), (kvq.Layout(1, 8, 64, rotate_v=-1), kvq.ERR_INVALID_ARG),
        (kvq.Layout(1, 8, 64, 128, 4, 16, rotate_v=1), kvq.ERR_INVALID_ARG),
        (kvq.Layout(1, 8, 64, 128, 4, 2, 64, 64, axis_k=1, rotate_v=1), kvq.ERR_INVALID_ARG),
        (kvq.Layout(1, 8, 64, 128, 16, 16, rotate_k=1), kvq.ERR_INVALID_ARG),        # rotation needs quantized keys
        # residual buffers: 64 or 128 slots that whole key groups fill; 64 in front of token-wise keys; paged with 64/64 only
        (kvq.Layout(1, 8, 256, 128, 4, 2, 128, 64, axis_k=1, resid_len=64), kvq.ERR_INVALID_ARG),
        (kvq.Layout(1, 8, 256, 128, 4, 2, 32, 64, axis_k=1, resid_len=32), kvq.ERR_UNSUPPORTED),
        (kvq.Layout(1, 8, 256, 128, 4, 2, 64, 64, axis_k=1, resid_len=256), kvq.ERR_UNSUPPORTED),
        (kvq.Layout(1, 8, 256, 128, 4, 2, 64, 64, resid_len=128), kvq.ERR_UNSUPPORTED),
        (kvq.Layout(1, 8, 256, 128, 4, 2, 64, 64, resid_len=-64), kvq.ERR_INVALID_ARG),
        (kvq.Layout(1, 8, 256, 128, 4, 2, 32, 64, axis_k=1, resid_len=64, page_tokens=64, n_pages=8), kvq.ERR_UNSUPPORTED),
        (kvq.Layout(1, 8, 256, 128, 4, 2, 128, 64, axis_k=1, page_tokens=128, n_pages=8), kvq.ERR_UNSUPPORTED),
    ]
    for layout, want in bad:
        assert _status(kvq.cache_bytes, layout) == want, layout


def test_call_errors_are_caught_before_any_launch(kvq):
    """Fake (never dereferenced) device addresses: every one of these calls must fail on the host."""
    lib = kvq.load()
    L = kvq.Layout(2, 2, 100)
    cl = L.c()
    good = kvq._CCache(0x10000, 0x20000, 0x30000, 0x40000, v_scale_exp=0x48000)
    p = C.c_void_p
    def qa(cache, k, v, dt, sb, sh, st, pos, n):
        return lib.kvq_quantize_append(C.byref(cl), C.byref(cache), p(k), p(v), dt, sb, sh, st, pos, n, None)
    assert qa(good, 0x50000, 0x60000, 0, 25600, 12800, 128, 95, 8) == kvq.ERR_CAPACITY
    assert qa(good, 0x50000, 0x60000, 0, 25600, 12800, 128, -1, 1) == kvq.ERR_INVALID_ARG
    assert qa(good, 0, 0x60000, 0, 25600, 12800, 128, 0, 1) == kvq.ERR_INVALID_ARG
    assert qa(good, 0x50000, 0x60000, 2, 25600, 12800, 128, 0, 1) == kvq.ERR_INVALID_ARG          # fp32 input
    assert qa(good, 0x50002, 0x60000, 0, 25600, 12800, 128, 0, 1) == kvq.ERR_INVALID_ARG          # misaligned rows
    assert qa(good, 0x50000, 0x60000, 0, 25600, 12800, 100, 0, 1) == kvq.ERR_INVALID_ARG          # rows overlap
    assert qa(kvq._CCache(0x10000, 0, 0x30000, 0x40000, v_scale_exp=0x48000), 0x50000, 0x60000, 0, 25600, 12800, 128, 0, 1) == kvq.ERR_INVALID_ARG
    # quantized values need the stream's value-scale exponents (part of the cache's state)
    assert qa(kvq._CCache(0x10000, 0x20000, 0x30000, 0x40000), 0x50000, 0x60000, 0, 25600, 12800, 128, 0, 1) == kvq.ERR_INVALID_ARG
    assert qa(kvq._CCache(0x10000, 0x20000, 0x30000, 0x40000, v_scale_exp=0x48002), 0x50000, 0x60000, 0, 25600, 12800, 128, 0, 1) == kvq.ERR_INVALID_ARG
    assert qa(good, 0x50000, 0x60000, 0, 25600, 12800, 128, 100, 0) == kvq.OK                     # empty append: no launch
    Lp = kvq.Layout(2, 2, 100, page_tokens=64, n_pages=8).c()                                       # paged layout without a table
    assert lib.kvq_quantize_append(C.byref(Lp), C.byref(good), p(0x50000), p(0x60000), 0, 25600, 12800, 128, 0, 1, None) == kvq.ERR_INVALID_ARG

    def da(q, heads, seq, scale, out, odt, ws, wsb):
        return lib.kvq_decode_attention(C.byref(cl), C.byref(good), p(q), 1, heads, seq, C.c_float(scale), p(out), odt, p(ws), wsb, None)
    assert da(0x50000, 8, 101, 0.1, 0x60000, 2, 0x70000, 1 << 20) == kvq.ERR_CAPACITY
    assert da(0x50000, 8, 0, 0.1, 0x60000, 2, 0x70000, 1 << 20) == kvq.ERR_INVALID_ARG
    assert da(0x50000, 3, 50, 0.1, 0x60000, 2, 0x70000, 1 << 20) == kvq.ERR_INVALID_ARG          # 3 heads over 2 kv heads
    assert da(0x50000, 18, 50, 0.1, 0x60000, 2, 0x70000, 1 << 20) == kvq.ERR_UNSUPPORTED         # 9 query heads per kv head
    assert da(0x50000, 8, 50, -1.0, 0x60000, 2, 0x70000, 1 << 20) == kvq.ERR_INVALID_ARG
    assert da(0x50000, 8, 50, float("nan"), 0x60000, 2, 0x70000, 1 << 20) == kvq.ERR_INVALID_ARG
    assert da(0, 8, 50, 0.1, 0x60000, 2, 0x70000, 1 << 20) == kvq.ERR_INVALID_ARG
    need = kvq.decode_workspace_bytes(L, 8, 100)
    if need:
        assert da(0x50000, 8, 100, 0.1, 0x60000, 2, 0x70000, need - 1) == kvq.ERR_WORKSPACE
        assert da(0x50000, 8, 100, 0.1, 0x60000, 2, 0, need) == kvq.ERR_WORKSPACE
    assert da(0x50000, 32, 50, 0.1, 0x60000, 2, 0x70000, 1 << 20) == kvq.ERR_UNSUPPORTED         # 16 query heads per kv head
    # one tensor unquantized: attention exists with one column set and token-wise keys; the query of a 16-bit key plane has
    # the plane's type; the fused step is for caches with both tensors quantized
    mixc = kvq._CCache(0x10000, 0, 0x30000, 0x40000, v_scale_exp=0x48000)
    def dmix(layout, q_dtype, heads, fn=lib.kvq_decode_attention):
        return fn(C.byref(layout.c()), C.byref(mixc), p(0x50000), q_dtype, heads, 50, C.c_float(0.1), p(0x60000), 2, p(0x70000), 1 << 20, None)
    assert dmix(kvq.Layout(2, 2, 100, 128, 16, 2, 64, 64), 1, 8) == kvq.ERR_UNSUPPORTED            # bfloat16 query, binary16 keys
    assert dmix(kvq.Layout(2, 2, 100, 128, 16, 2, 64, 32), 0, 16) == kvq.ERR_UNSUPPORTED           # 8 heads x 4 value groups
    Lm = kvq.Layout(2, 2, 100, 128, 16, 2, 64, 64).c()
    assert lib.kvq_decode_step(C.byref(Lm), C.byref(mixc), p(0x50000), p(0x51000), 0, 256, 128, 5, p(0x52000), 0, 8,
                               C.c_float(0.1), p(0x60000), 2, p(0x70000), 1 << 20, None) == kvq.ERR_UNSUPPORTED

    def ds(pos, k=0x50000):
        return lib.kvq_decode_step(C.byref(cl), C.byref(good), p(k), p(0x51000), 1, 256, 128, pos, p(0x52000), 1, 8,
                                   C.c_float(0.1), p(0x60000), 2, p(0x70000), 1 << 20, None)
    assert ds(100) == kvq.ERR_CAPACITY and ds(-1) == kvq.ERR_INVALID_ARG and ds(5, 0) == kvq.ERR_INVALID_ARG

    def dv(lens, bound):
        return lib.kvq_decode_attention_varlen(C.byref(cl), C.byref(good), p(0x50000), 1, 8, p(lens), bound, C.c_float(0.1),
                                               p(0x60000), 2, p(0x70000), 1 << 20, None)
    assert dv(0, 50) == kvq.ERR_INVALID_ARG and dv(0x80002, 50) == kvq.ERR_INVALID_ARG
    assert dv(0x80000, 101) == kvq.ERR_CAPACITY and dv(0x80000, 0) == kvq.ERR_INVALID_ARG

    def dsv(pos, bound):
        return lib.kvq_decode_step_varlen(C.byref(cl), C.byref(good), p(0x50000), p(0x51000), 1, 256, 128, p(pos), bound,
                                          p(0x52000), 1, 8, C.c_float(0.1), p(0x60000), 2, p(0x70000), 1 << 20, None)
    assert dsv(0, 5) == kvq.ERR_INVALID_ARG and dsv(0x80000, -1) == kvq.ERR_INVALID_ARG and dsv(0x80000, 100) == kvq.ERR_CAPACITY

    def dq(t0, t1, ko, vo, dt):
        return lib.kvq_dequantize(C.byref(cl), C.byref(good), t0, t1, p(ko), p(vo), dt, None)
    assert dq(0, 101, 0x50000, 0x60000, 2) == kvq.ERR_CAPACITY
    assert dq(5, 4, 0x50000, 0x60000, 2) == kvq.ERR_INVALID_ARG
    assert dq(0, 4, 0, 0, 2) == kvq.ERR_INVALID_ARG
    assert dq(0, 4, 0x50000, 0, 7) == kvq.ERR_INVALID_ARG
    assert dq(4, 4, 0x50000, 0, 2) == kvq.OK                                                       # empty range: no launch

    def re_(k, v, dt, st, t0, t1, sums):
        return lib.kvq_reconstruction_error(C.byref(cl), C.byref(good), p(k), p(v), dt, 25600, 12800, st, t0, t1, p(sums), None)
    assert re_(0x50000, 0x60000, 0, 128, 0, 101, 0x70000) == kvq.ERR_CAPACITY
    assert re_(0x50000, 0x60000, 0, 128, 9, 3, 0x70000) == kvq.ERR_INVALID_ARG
    assert re_(0, 0, 0, 128, 0, 4, 0x70000) == kvq.ERR_INVALID_ARG
    assert re_(0x50000, 0x60000, 2, 128, 0, 4, 0x70000) == kvq.ERR_INVALID_ARG                   # fp32 reference rows
    assert re_(0x50000, 0x60000, 0, 120, 0, 4, 0x70000) == kvq.ERR_INVALID_ARG                   # rows overlap
    assert re_(0x50000, 0x60000, 0, 128, 0, 4, 0) == kvq.ERR_INVALID_ARG
    assert re_(0x50000, 0x60000, 0, 128, 0, 4, 0x70004) == kvq.ERR_INVALID_ARG                   # misaligned doubles


def test_product_path_never_touches_the_oracle():
    """The library, its binding and the benchmark's GPU leg must not import the CPU oracle."""
    pat = re.compile(r"^\s*(from|import)\s+oracle|kvq_oracle|libkvq_oracle", re.M)
    for rel in ("paper_2502_15075_amd/kvq.py", "paper_2502_15075_amd/synth.py", "paper_2502_15075_amd/build.py",
                "paper_2502_15075_amd/__init__.py"):
        assert not pat.search(open(os.path.join(ROOT, rel)).read()), rel
    for f in os.listdir(os.path.join(ROOT, "paper_2502_15075_amd", "csrc")):
        assert not pat.search(open(os.path.join(ROOT, "paper_2502_15075_amd", "csrc", f)).read()), f


def test_inline_assembly_stays_away_from_transcendental_results():
    """The compiler keeps the wait states between an instruction and a hazardous reader of its result (a transcendental
    result read by the next instruction, a register read through a lane permute right after it was written) only for
    instructions it emits itself.  The decode kernels, whose softmax weights come straight from v_exp_f32, therefore
    carry no instruction in inline assembly at all, and the assembly of the quantizer is limited to minimum / maximum
    instructions (their operands are converted inputs, never a reciprocal or exponential); the lane-permuted forms come
    in blocks that open with their own pause and never read a register written by the instruction just before."""
    csrc = os.path.join(ROOT, "paper_2502_15075_amd", "csrc")
    texts = {}
    for name in sorted(os.listdir(csrc)):
        src = open(os.path.join(csrc, name)).read()
        blocks = []
        for m in re.finditer(r'\basm\s*(?:volatile)?\s*\(((?:\s*"(?:[^"\\]|\\.)*")+)', src):
            text = "".join(re.findall(r'"((?:[^"\\]|\\.)*)"', m.group(1))).replace("\\n", "\n").replace("\\t", " ")
            if text.strip():
                blocks.append([l.strip() for l in text.split("\n") if l.strip()])
        texts[name] = blocks
    assert texts["kvq_decode.hip"] == [] and texts["kvq_api.hip"] == []
    allowed = ("v_min3_f32", "v_max3_f32", "v_min_f32", "v_max_f32", "v_min_f32_dpp", "v_max_f32_dpp", "s_nop")
    n_dpp = 0
    for name, blocks in texts.items():
        for lines in blocks:
            ops = [l.split()[0] for l in lines]
            assert all(op in allowed for op in ops), (name, lines)
            if any(op.endswith("_dpp") for op in ops):
                n_dpp += 1
                assert ops[0] == "s_nop", (name, lines)
                # a permuted read of %k needs two wait states after the write of %k: between two instructions on the
                # same operand lie the other operand's instruction and a pause, or the block's opening pause
                last_write = {}
                for i, l in enumerate(lines):
                    if not l.split()[0].endswith("_dpp"):
                        continue
                    dst = l.split()[1].rstrip(",")
                    if dst in last_write:
                        assert i - last_write[dst] >= 3, (name, lines)
                    last_write[dst] = i
    assert n_dpp >= 1


def test_workspace_never_shrinks_as_the_sequence_grows(kvq):
    """A caller sizes the workspace once for its longest sequence: the figure for a shorter one must not be larger
    (the number of records a call actually writes is not monotone in the length; the reported size is its bound)."""
    for B, H, Hq, axis in ((8, 8, 32, 0), (2, 8, 32, 0), (1, 8, 8, 0), (1, 1, 8, 0), (3, 2, 16, 1), (1, 8, 32, 1)):
        L = kvq.Layout(B, H, 1 << 17, 128, 4, 2, 64, 64, axis_k=axis)
        sizes = [kvq.decode_workspace_bytes(L, Hq, t) for t in list(range(1, 6000, 7)) + list(range(6000, 1 << 17, 997))]
        assert all(a <= b for a, b in zip(sizes, sizes[1:])), (B, H, axis)
        counters = (B * H * 8 + 15) // 16 * 16
        assert sizes[-1] > counters and (sizes[-1] - counters) % (132 * 4 * B * Hq) == 0

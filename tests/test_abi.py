"""CPU-side checks of the C ABI: the library loads, exports everything the header declares,
and rejects bad arguments with the documented status before touching a GPU."""
import ctypes
import os
import re

import pytest

from paper_2408_16978_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2408_16978_amd import build
        build.build()
    return B.load()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "fpdt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fpdt_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(lib):
    names = declared_functions()
    assert {"fpdt_attn_fwd", "fpdt_attn_bwd", "fpdt_attn_merge", "fpdt_attn_workspace_bytes",
            "fpdt_last_error", "fpdt_last_link_bytes", "fpdt_version"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert "gfx950" in B.fpdt_version()


def test_binding_names_match_header():
    for n in declared_functions():
        assert callable(getattr(B, n)), n


def test_header_constants_match_binding():
    text = open(os.path.join(ROOT, "include", "fpdt.h")).read()
    for name in ("FPDT_KV_ON_HOST", "FPDT_ACT_ON_HOST", "FPDT_BWD_KV_OUTER", "FPDT_BWD_Q_OUTER",
                 "FPDT_PAIRWISE", "FPDT_BWD_STORE_DS"):
        m = re.search(name + r"\s*=\s*1u\s*<<\s*(\d+)", text)
        assert m and getattr(B, name) == 1 << int(m.group(1)), name
    assert re.search(r"FPDT_CHUNK_MULTIPLE\s*=\s*256", text) and B.FPDT_CHUNK_MULTIPLE == 256
    assert re.search(r"FPDT_PREFERRED_CHUNK\s*=\s*65536", text) and B.FPDT_PREFERRED_CHUNK == 65536
    assert re.search(r"FPDT_NOALLOC_SCRATCH_BYTES\s*=\s*32\s*<<\s*20", text) and B.FPDT_NOALLOC_SCRATCH_BYTES == 32 << 20


def _fwd(lib, S=1024, chunk=256, Hq=2, Hkv=2, D=64, scale=0.125, dtype=B.FPDT_DTYPE_BF16, flags=0,
         ptr=0x1000, ws=0x100000, ws_bytes=1 << 40):
    return lib.fpdt_attn_fwd(ptr, ptr, ptr, ptr, ptr, S, chunk, Hq, Hkv, D, scale, dtype, flags, ws,
                             ws_bytes, None)


def test_invalid_arguments_are_rejected_without_a_gpu(lib):
    assert _fwd(lib, ptr=None) == B.FPDT_ERR_INVALID_ARG
    assert "NULL" in B.fpdt_last_error()
    assert _fwd(lib, S=0) == B.FPDT_ERR_INVALID_ARG
    assert _fwd(lib, chunk=0) == B.FPDT_ERR_INVALID_ARG
    assert _fwd(lib, S=1000, chunk=256) == B.FPDT_ERR_INVALID_ARG
    assert _fwd(lib, Hq=3, Hkv=2) == B.FPDT_ERR_INVALID_ARG
    assert _fwd(lib, scale=0.0) == B.FPDT_ERR_INVALID_ARG
    assert _fwd(lib, scale=float("nan")) == B.FPDT_ERR_INVALID_ARG
    assert _fwd(lib, scale=float("inf")) == B.FPDT_ERR_INVALID_ARG
    assert _fwd(lib, dtype=7) == B.FPDT_ERR_INVALID_ARG
    assert _fwd(lib, flags=1 << 20) == B.FPDT_ERR_INVALID_ARG
    assert _fwd(lib, flags=B.FPDT_BWD_KV_OUTER | B.FPDT_BWD_Q_OUTER) == B.FPDT_ERR_INVALID_ARG
    assert _fwd(lib, D=96) == B.FPDT_ERR_UNSUPPORTED
    assert _fwd(lib, S=1000, chunk=100) == B.FPDT_ERR_UNSUPPORTED           # bf16 chunk % 256
    assert _fwd(lib, dtype=B.FPDT_DTYPE_F32, flags=B.FPDT_KV_ON_HOST) == B.FPDT_ERR_UNSUPPORTED
    assert _fwd(lib, flags=B.FPDT_ACT_ON_HOST | B.FPDT_BWD_KV_OUTER) == B.FPDT_ERR_UNSUPPORTED
    # the stored-dS backward: bf16 only (the forward ignores the flag), and a chunk whose dS tiles
    # could not be indexed is refused
    bwd = lambda **kw: lib.fpdt_attn_bwd(*([0x1000] * 9), kw.get("S", 1024), kw.get("chunk", 256), 2, 2, 64, 0.125,
                                         kw.get("dtype", B.FPDT_DTYPE_BF16), kw.get("flags", 0), 0x100000, 1 << 40, None)
    assert bwd(dtype=B.FPDT_DTYPE_F32, flags=B.FPDT_BWD_STORE_DS) == B.FPDT_ERR_UNSUPPORTED
    assert "stored-dS" in B.fpdt_last_error()
    assert bwd(S=1 << 22, chunk=1 << 21, flags=B.FPDT_BWD_STORE_DS) == B.FPDT_ERR_UNSUPPORTED
    # sizes beyond the 32-bit launch arithmetic are refused, the largest supported one is accepted
    # as far as the scalar checks go (it then fails on the fake pointers, not on its size)
    assert _fwd(lib, S=(1 << 30) + 256, chunk=256) == B.FPDT_ERR_UNSUPPORTED and "launch limits" in B.fpdt_last_error()
    assert _fwd(lib, S=1 << 30, chunk=1 << 20, Hq=64, Hkv=8) == B.FPDT_ERR_UNSUPPORTED
    assert B.fpdt_attn_workspace_bytes(1 << 30, 1 << 16, 8, 2, 128, B.FPDT_DTYPE_BF16, B.FPDT_KV_ON_HOST, False) > 0
    assert _fwd(lib, ws=None) == B.FPDT_ERR_WORKSPACE
    assert _fwd(lib, ws_bytes=16) == B.FPDT_ERR_WORKSPACE
    assert _fwd(lib, ws=0x100010) == B.FPDT_ERR_WORKSPACE                    # misaligned
    assert B.fpdt_last_error() != ""
    rc = lib.fpdt_attn_bwd(*([0x1000] * 8), None, 1024, 256, 2, 2, 64, 0.125, 1, 0, 0x100000,
                           1 << 40, None)
    assert rc == B.FPDT_ERR_INVALID_ARG
    rc = lib.fpdt_attn_merge(0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0, 2, 64, 1, None)
    assert rc == B.FPDT_ERR_INVALID_ARG


def test_workspace_sizes():
    ws = B.fpdt_attn_workspace_bytes
    bf = B.FPDT_DTYPE_BF16
    assert ws(1000, 256, 2, 2, 64, bf) == 0                                  # invalid -> 0
    assert ws(1024, 256, 2, 2, 64, B.FPDT_DTYPE_F32) > 0
    # with K/V offloaded, the forward workspace depends on the chunk, not on S (Sec. 4.1:
    # only the chunks in use are resident)
    a = ws(1 << 18, 65536, 8, 2, 128, bf, B.FPDT_KV_ON_HOST)
    b = ws(1 << 21, 65536, 8, 2, 128, bf, B.FPDT_KV_ON_HOST)
    assert a == b and a > 0
    # two raw K/V chunk buffers (2 x 64 MiB) + packed chunk (64 MiB) + carried state
    assert a < 3 * (1 << 30) // 2
    # resident mode grows with S
    assert ws(1 << 21, 65536, 8, 2, 128, bf) > ws(1 << 18, 65536, 8, 2, 128, bf)
    # backward with everything streamed (Q-outer): only dK/dV accumulators scale with S
    c = ws(1 << 20, 65536, 8, 1, 128, bf, B.FPDT_KV_ON_HOST | B.FPDT_ACT_ON_HOST, True)
    d = ws(1 << 21, 65536, 8, 1, 128, bf, B.FPDT_KV_ON_HOST | B.FPDT_ACT_ON_HOST, True)
    assert d - c == 2 * (1 << 20) * 1 * 128 * 4
    # backward with only K/V offloaded: the part that grows with S is the documented one,
    #   KV-outer (default): fp32 dQ accumulator S * Hq * D * 4 and Delta S * Hq * 4
    #   Q-outer:            fp32 dK and dV accumulators 2 * S * Hkv * D * 4 and Delta S * Hq * 4
    kvh = B.FPDT_KV_ON_HOST
    for S1, S2 in ((1 << 18, 1 << 21), (1 << 19, 1 << 20)):
        grow = ws(S2, 65536, 8, 2, 128, bf, kvh, True) - ws(S1, 65536, 8, 2, 128, bf, kvh, True)
        assert grow == (S2 - S1) * 8 * (128 + 1) * 4
        assert grow == ws(S2, 65536, 8, 2, 128, bf, kvh | B.FPDT_BWD_KV_OUTER, True) - ws(S1, 65536, 8, 2, 128, bf, kvh | B.FPDT_BWD_KV_OUTER, True)
        grow_q = ws(S2, 65536, 8, 2, 128, bf, kvh | B.FPDT_BWD_Q_OUTER, True) - ws(S1, 65536, 8, 2, 128, bf, kvh | B.FPDT_BWD_Q_OUTER, True)
        assert grow_q == (S2 - S1) * (2 * 2 * 128 + 8) * 4
    # stored-dS backward: the dS tiles of one chunk pair on top of the pair-by-pair workspace; the
    # forward ignores the flag
    sd = B.FPDT_BWD_STORE_DS
    assert ws(1 << 21, 65536, 8, 2, 128, bf, kvh | sd, True) - ws(1 << 21, 65536, 8, 2, 128, bf, kvh, True) == 65536 * 65536 * 8 * 2
    assert ws(1 << 16, 8192, 4, 4, 80, bf, sd, True) - ws(1 << 16, 8192, 4, 4, 80, bf, B.FPDT_PAIRWISE, True) == 8192 * 8192 * 4 * 2
    assert ws(1 << 21, 65536, 8, 2, 128, bf, kvh | sd, False) == ws(1 << 21, 65536, 8, 2, 128, bf, kvh, False)
    assert ws(1024, 256, 2, 2, 64, B.FPDT_DTYPE_F32, sd, True) == 0              # fp32: unsupported
    # at the headline workload: 8 GiB + 64 MiB of S-sized state under KV-outer, 2 GiB + 64 MiB under Q-outer
    assert ws(1 << 21, 65536, 8, 2, 128, bf, kvh, True) - ws(1 << 21, 65536, 8, 2, 128, bf, kvh | B.FPDT_BWD_Q_OUTER, True) \
        == (1 << 21) * 8 * 128 * 4 - 2 * (1 << 21) * 2 * 128 * 4 - (65536 * 8 * 128 * 4 - 2 * 65536 * 2 * 128 * 4)


def test_pick_chunk_host_logic(lib):
    BF, F32 = B.FPDT_DTYPE_BF16, B.FPDT_DTYPE_F32
    # largest divisor of S up to the 64K knee of the measured curve
    assert B.FPDT_PREFERRED_CHUNK == 65536
    assert B.fpdt_attn_pick_chunk(2097152, 8, 2, 128, BF, B.FPDT_KV_ON_HOST) == 65536
    assert B.fpdt_attn_pick_chunk(65536, 4, 4, 80, BF) == 65536
    assert B.fpdt_attn_pick_chunk(768 * 256, 8, 2, 128, BF) == 65536      # 3 * 2^16 tokens
    assert B.fpdt_attn_pick_chunk(640 * 256, 8, 2, 128, BF) == 40960      # 5 * 2^15: divisor, multiple of 256
    assert B.fpdt_attn_pick_chunk(1024, 2, 2, 64, F32) == 1024
    # the answer is always a legal chunk for the entry points and respects the workspace limit
    for S, flags in ((2097152, B.FPDT_KV_ON_HOST), (1048576, B.FPDT_KV_ON_HOST | B.FPDT_ACT_ON_HOST), (262144, 0)):
        full = B.fpdt_attn_pick_chunk(S, 8, 2, 128, BF, flags)
        need = max(B.fpdt_attn_workspace_bytes(S, full, 8, 2, 128, BF, flags, b) for b in (False, True))
        assert need > 0
        c = B.fpdt_attn_pick_chunk(S, 8, 2, 128, BF, flags, need - 1)
        if c:
            assert c < full and S % c == 0 and c % 256 == 0
            assert max(B.fpdt_attn_workspace_bytes(S, c, 8, 2, 128, BF, flags, b) for b in (False, True)) <= need - 1
        assert B.fpdt_attn_pick_chunk(S, 8, 2, 128, BF, flags, need) == full
    # no chunk: reasons are reported
    assert B.fpdt_attn_pick_chunk(1000, 2, 2, 64, BF) == 0 and "multiple" in B.fpdt_last_error()
    assert B.fpdt_attn_pick_chunk(0, 2, 2, 64, BF) == 0 and B.fpdt_last_error() != ""
    assert B.fpdt_attn_pick_chunk(4096, 3, 2, 64, BF) == 0 and "Hq" in B.fpdt_last_error()
    assert B.fpdt_attn_pick_chunk(4096, 2, 2, 64, BF, 0, 16) == 0 and "workspace" in B.fpdt_last_error()


def test_calibration_arguments_are_checked_without_a_gpu(lib):
    tf = ctypes.c_double(0.0)
    assert lib.fpdt_calibrate_mfma(99, 1000, None, 0, ctypes.byref(tf), None, None) == B.FPDT_ERR_INVALID_ARG
    assert "kind" in B.fpdt_last_error()
    assert lib.fpdt_calibrate_mfma(0, 0, None, 0, ctypes.byref(tf), None, None) == B.FPDT_ERR_INVALID_ARG
    assert lib.fpdt_calibrate_mfma(0, 1000, None, 0, None, None, None) == B.FPDT_ERR_INVALID_ARG
    assert lib.fpdt_calibrate_mfma(0, 1000, None, 0, ctypes.byref(tf), None, None) == B.FPDT_ERR_WORKSPACE
    assert len(B.FPDT_CAL_KINDS) == 8

"""Host-side checks of the C ABI that need no GPU: the library loads, exports every declared symbol, and rejects
bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "skiparse.h")
PROBE_HEADER = os.path.join(ROOT, "include", "skiparse_probe.h")
LIBPATH = os.path.join(ROOT, "paper_2605_28691_amd", "libskiparse.so")
PROBE_LIBPATH = os.path.join(ROOT, "paper_2605_28691_amd", "libskiparse_probe.so")


@pytest.fixture(scope="module")
def lib():
    import paper_2605_28691_amd as sk

    if not os.path.exists(LIBPATH):
        from paper_2605_28691_amd import build

        build.build()
    return sk.lib()


@pytest.fixture(scope="module")
def probe_lib():
    from paper_2605_28691_amd import probe

    if not os.path.exists(PROBE_LIBPATH):
        from paper_2605_28691_amd import build

        build.build()
    return probe.lib()


def _declared_functions(header=HEADER):
    text = open(header).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b([a-z_0-9]+)\s*\(", text)) - {"defined"})


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert {"skiparse_permute", "skiparse_unpermute", "dense_attn_fwd", "skiparse_attn_fwd", "skiparse_workspace_bytes",
            "skiparse_quantize_fp8", "skiparse_attn_fwd_fp8", "skiparse_strerror", "skiparse_last_hip_error",
            "skiparse_switch_pattern", "skiparse_attn_fwd_sparse", "skiparse_attn_fwd_lse",
            "skiparse_bwd_workspace_bytes", "skiparse_attn_bwd", "skiparse_lse_bytes", "skiparse_attn_bwd_static",
            "skiparse_static_scratch_bytes", "skiparse_ssp_pack", "skiparse_ssp_unpack",
            "skiparse_quantize_fp8_ex", "skiparse_attn_fwd_fp8_ex"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert not [n for n in names if "probe" in n]  # the measurement kernels live in a library of their own


def test_every_declared_probe_symbol_is_exported(probe_lib):
    names = _declared_functions(PROBE_HEADER)
    assert {"skiparse_mfma_probe", "skiparse_mfma_valu_probe", "skiparse_mfma_lds_probe", "skiparse_lds_read_probe", "skiparse_mfma_chain_probe", "skiparse_mfma8_valu_probe", "skiparse_probe_device_info",
            "skiparse_probe_last_hip_error"} <= set(names)
    for n in names:
        assert hasattr(probe_lib, n), n


def test_strerror(lib):
    for code in range(-6, 1):
        assert lib.skiparse_strerror(code)


FAKE = 0x10000  # a non-null, 16-byte aligned address; never dereferenced because validation fails first


def test_permute_rejects_bad_arguments(lib):
    p, q = ctypes.c_void_p(FAKE), ctypes.c_void_p(FAKE + (1 << 30))
    ok_args = [1, 2, 2, 8, 8, 64, 2, 0, 0]

    def call(src, dst, *a):
        return lib.skiparse_permute(src, dst, *a, None)

    assert call(None, q, *ok_args) == -1
    assert call(p, None, *ok_args) == -1
    assert call(p, p, *ok_args) == -1  # src == dst
    assert call(p, ctypes.c_void_p(FAKE + 64), *ok_args) == -1  # overlapping
    assert call(ctypes.c_void_p(FAKE + 4), q, *ok_args) == -1  # misaligned
    assert call(p, q, 0, 2, 2, 8, 8, 64, 2, 0, 0) == -1  # B = 0
    assert call(p, q, 1, 2, 2, 8, 8, 64, 0, 0, 0) == -1  # s = 0
    assert call(p, q, 1, 2, 2, 8, 8, 64, 2, 7, 0) == -1  # unknown pattern
    assert call(p, q, 1, 2, 2, 8, 8, 64, 2, 0, 9) == -1  # unknown dtype
    assert call(p, q, 1, 2, 2, 6, 8, 64, 2, 1, 0) == -2  # group-wise needs H % 4 == 0
    assert call(p, q, 1, 2, 2, 7, 8, 64, 2, 0, 0) == -2  # token-wise needs H % 2 == 0
    assert call(p, q, 1, 2, 1 << 12, 1 << 10, 1 << 10, 64, 2, 0, 0) == -2  # 2^32 tokens
    assert call(p, q, 1, 1, 2, 8, 8, 3, 2, 0, 2) == -3  # 3-byte rows cannot be moved in 16-byte pieces
    assert lib.skiparse_unpermute(p, q, 1, 2, 2, 6, 8, 64, 2, 1, 0, None) == -2


def test_attention_rejects_bad_arguments(lib):
    a = [ctypes.c_void_p(FAKE + i * (1 << 30)) for i in range(5)]
    f = ctypes.c_float(0.0)
    assert lib.dense_attn_fwd(None, a[1], a[2], a[3], 1, 2, 2, 8, 8, 64, f, 0, None) == -1
    assert lib.dense_attn_fwd(a[0], a[1], a[2], a[0], 1, 2, 2, 8, 8, 64, f, 0, None) == -1  # out aliases q
    assert lib.dense_attn_fwd(a[0], a[1], a[2], a[3], 1, 2, 2, 8, 8, 96, f, 0, None) == -3  # head_dim 96
    assert lib.dense_attn_fwd(a[0], a[1], a[2], a[3], 1, 2, 2, 8, 8, 64, f, 1, None) == -3  # fp32 attention
    assert lib.dense_attn_fwd(a[0], a[1], a[2], a[3], 1, 2, 2, 8, 8, 64, f, 5, None) == -1  # unknown dtype

    def sparse(flags, ws, ws_bytes, H=8, pattern=0, s=2):
        return lib.skiparse_attn_fwd(a[0], a[1], a[2], a[3], 1, 2, 2, H, 8, 64, s, pattern, f, 0, flags, ws, ws_bytes, None)

    assert sparse(1, None, 0, H=6, pattern=1) == -2
    assert sparse(4, None, 0) == -1  # unknown flag bit
    assert sparse(2, None, 0) == -3  # padding without the fused kernel
    assert sparse(1, None, 0, H=7) == -2  # H = 7 needs the any-resolution flag
    # with the flag the shape is accepted and the next check (out aliases q) is reached
    assert lib.skiparse_attn_fwd(a[0], a[1], a[2], a[0], 1, 2, 2, 7, 9, 64, 2, 1, f, 0, 3, None, 0, None) == -1
    assert sparse(0, None, 0) == -4  # unfused path without a workspace
    need = lib.skiparse_workspace_bytes(1, 2, 2, 8, 8, 64, 2, 0, 0)
    assert need == 4 * 1 * 128 * 2 * 64 * 2
    assert sparse(0, a[4], need - 1) == -4
    assert lib.skiparse_workspace_bytes(1, 2, 2, 8, 8, 64, 2, 0, 1) == 0  # fused needs none
    assert lib.skiparse_workspace_bytes(1, 2, 2, 7, 8, 64, 2, 0, 0) == 0  # bad shape


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    import paper_2605_28691_amd as sk

    monkeypatch.setattr(sk, "_lib", None)
    monkeypatch.setattr(sk, "_LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        sk.lib()


def test_fp8_entry_points_reject_bad_arguments(lib):
    a = [ctypes.c_void_p(FAKE + i * (1 << 30)) for i in range(8)]
    f = ctypes.c_float(0.0)
    assert lib.skiparse_quantize_fp8(None, a[1], a[2], 1, 2, 2, 8, 8, 64, 2, 0, None) == -1
    assert lib.skiparse_quantize_fp8(a[0], a[1], a[2], 1, 2, 2, 6, 8, 64, 2, 1, None) == -2  # group-wise needs H % 4 == 0
    assert lib.skiparse_quantize_fp8(a[0], a[1], a[2], 1, 2, 2, 8, 8, 96, 2, 0, None) == -3  # head_dim 96
    assert lib.skiparse_quantize_fp8(a[0], a[0], a[2], 1, 2, 2, 8, 8, 64, 2, 0, None) == -1  # output aliases input
    ok = [1, 2, 2, 8, 8, 64, 2, 0]
    assert lib.skiparse_attn_fwd_fp8(a[0], a[1], a[2], a[3], a[4], None, a[6], *ok, f, None) == -1
    assert lib.skiparse_attn_fwd_fp8(a[0], a[1], a[2], a[3], a[4], a[5], a[0], *ok, f, None) == -1  # out aliases q8
    assert lib.skiparse_attn_fwd_fp8(a[0], a[1], a[2], a[3], a[4], a[5], a[6], 1, 2, 2, 8, 8, 32, 2, 0, f, None) == -3
    assert lib.skiparse_attn_fwd_fp8(a[0], a[1], a[2], a[3], a[4], a[5], a[6], 1, 2, 2, 8, 7, 64, 2, 0, f, None) == -2
    assert lib.skiparse_attn_fwd_fp8(a[0], a[1], a[2], ctypes.c_void_p(FAKE + 2), a[4], a[5], a[6], *ok, f, None) == -1  # misaligned scales
    assert lib.skiparse_attn_fwd_fp8(a[0], a[1], a[2], a[3], a[4], ctypes.c_void_p(a[6].value + 64), a[6], *ok, f, None) == -1  # scales inside out


def test_attention_rejects_out_of_range_sizes(lib):
    a = [ctypes.c_void_p(FAKE + i * (1 << 40)) for i in range(4)]
    f = ctypes.c_float(0.0)
    # 2^24 tokens per batch element: beyond the 24-bit multiplies of the attention kernels' address arithmetic
    assert lib.dense_attn_fwd(a[0], a[1], a[2], a[3], 1, 1, 1 << 8, 1 << 8, 1 << 8, 64, f, 0, None) == -2
    # one batch element of 4 GiB or more: beyond the 32-bit row offsets
    assert lib.dense_attn_fwd(a[0], a[1], a[2], a[3], 1, 64, 1 << 6, 1 << 6, 1 << 6, 128, f, 0, None) == -2


def test_switch_pattern_rejects_bad_arguments(lib):
    p, q = ctypes.c_void_p(FAKE), ctypes.c_void_p(FAKE + (1 << 30))
    assert lib.skiparse_switch_pattern(None, q, 1, 2, 2, 8, 8, 64, 2, 0, 0, None) == -1
    assert lib.skiparse_switch_pattern(p, p, 1, 2, 2, 8, 8, 64, 2, 0, 0, None) == -1
    assert lib.skiparse_switch_pattern(p, q, 1, 2, 2, 8, 8, 64, 2, 3, 0, None) == -1  # unknown pattern
    assert lib.skiparse_switch_pattern(p, q, 1, 2, 2, 6, 8, 64, 2, 0, 0, None) == -2  # token-wise alone would accept H = 6, the switch needs H % 4 == 0


def test_attn_fwd_sparse_rejects_bad_arguments(lib):
    a = [ctypes.c_void_p(FAKE + i * (1 << 30)) for i in range(4)]
    f = ctypes.c_float(0.0)

    def call(H, W, s, pattern, layout, out=a[3], D=64, dtype=0):
        return lib.skiparse_attn_fwd_sparse(a[0], a[1], a[2], out, 1, 1, 1, H, W, D, s, pattern, layout, f, dtype, None)

    assert call(12, 12, 2, 0, 3) == -1          # unknown output layout
    assert call(12, 12, 2, 2, 0) == -1          # unknown pattern
    assert call(6, 24, 2, 0, 1) == -2           # the other pattern's layout needs H, W multiples of s*s
    assert call(12, 12, 2, 1, 0, out=a[0]) == -1  # out overlaps q
    assert call(12, 12, 2, 0, 0, out=None) == -1
    assert call(12, 12, 2, 0, 0, D=96) == -3    # no kernel for this head_dim
    assert call(12, 12, 2, 0, 0, dtype=1) == -3  # bf16 only


def test_backward_rejects_bad_arguments(lib):
    a = [ctypes.c_void_p(FAKE + i * (1 << 30)) for i in range(11)]
    f = ctypes.c_float(0.0)
    need = lib.skiparse_bwd_workspace_bytes(1, 2, 2, 8, 8, 64, 2, 0, 0)
    assert need == 1 * 128 * 2 * 4  # one float per query and head (already a multiple of 256)
    assert lib.skiparse_lse_bytes(1, 2, 2, 8, 8, 64, 2, 0, 0) == need
    assert lib.skiparse_bwd_workspace_bytes(1, 2, 2, 7, 8, 64, 2, 0, 0) == 0  # bad shape
    # any-resolution mode: positions of the grid padded to multiples of s*s = 4: 2 x 8 x 8 again
    assert lib.skiparse_lse_bytes(1, 2, 2, 7, 6, 64, 2, 0, 2) == need
    assert lib.skiparse_lse_bytes(1, 2, 2, 7, 6, 64, 2, 0, 1) == 0  # unknown flag

    def bwd(ptrs, ws=a[9], ws_bytes=need, H=8, D=64, dtype=0, flags=0):
        return lib.skiparse_attn_bwd(*ptrs, 1, 2, 2, H, 8, D, 2, 0, f, dtype, flags, ws, ws_bytes, None)

    ok = a[:9]
    assert bwd([None] + ok[1:]) == -1
    assert bwd(ok[:6] + [ok[0]] + ok[7:]) == -1        # dq aliases q
    assert bwd(ok[:7] + [ok[6]] + ok[8:]) == -1        # dk aliases dq
    assert bwd(ok, ws=None) == -4
    assert bwd(ok, ws_bytes=need - 1) == -4
    assert bwd(ok, ws=ok[8]) == -1                     # workspace aliases dv
    assert bwd(ok, H=7) == -2
    assert bwd(ok, flags=1) == -1                      # only SKIPARSE_PAD is a flag here
    assert bwd(ok, D=96) == -3
    assert bwd(ok, dtype=1) == -3
    # forward with log-sum-exp
    assert lib.skiparse_attn_fwd_lse(a[0], a[1], a[2], a[3], None, 1, 2, 2, 8, 8, 64, 2, 0, f, 0, 0, None) == -1
    assert lib.skiparse_attn_fwd_lse(a[0], a[1], a[2], a[3], a[3], 1, 2, 2, 8, 8, 64, 2, 0, f, 0, 0, None) == -1  # lse aliases out
    assert lib.skiparse_attn_fwd_lse(a[0], a[1], a[2], a[3], a[4], 1, 2, 2, 8, 6, 64, 2, 1, f, 0, 0, None) == -2  # group-wise needs W % 4 == 0


def test_mfma_probe_rejects_bad_arguments(probe_lib):
    lib = probe_lib
    p, q = ctypes.c_void_p(FAKE), ctypes.c_void_p(FAKE + (1 << 30))
    flop = ctypes.c_double(0.0)
    assert lib.skiparse_mfma_probe(None, 1 << 20, q, 1 << 30, 0, 8, 10, ctypes.byref(flop), None) == -1
    assert lib.skiparse_mfma_probe(p, 1 << 20, q, 1 << 30, 1, 8, 10, ctypes.byref(flop), None) == -3   # fp32: no such probe
    assert lib.skiparse_mfma_probe(p, 100, q, 1 << 30, 0, 8, 10, ctypes.byref(flop), None) == -4       # operand buffer too small
    assert lib.skiparse_mfma_probe(p, 1 << 20, q, 8 * 256 * 4 - 1, 0, 8, 10, ctypes.byref(flop), None) == -4
    assert lib.skiparse_mfma_probe(p, 1 << 20, q, 1 << 30, 0, 0, 10, ctypes.byref(flop), None) == -1
    assert lib.skiparse_mfma_valu_probe(p, 1 << 20, q, 1 << 30, 3, 8, 10, ctypes.byref(flop), None) == -3   # only 0, 2, 4, 6, 8
    assert lib.skiparse_mfma_valu_probe(p, 1 << 20, q, 100, 4, 8, 10, ctypes.byref(flop), None) == -4
    assert lib.skiparse_mfma_valu_probe(None, 1 << 20, q, 1 << 30, 4, 8, 10, ctypes.byref(flop), None) == -1
    assert lib.skiparse_mfma_lds_probe(None, 1 << 20, q, 1 << 30, 8, 10, ctypes.byref(flop), None) == -1
    assert lib.skiparse_mfma_lds_probe(p, 100, q, 1 << 30, 8, 10, ctypes.byref(flop), None) == -4
    assert lib.skiparse_mfma_lds_probe(p, 1 << 20, q, 1 << 30, 8, 0, ctypes.byref(flop), None) == -1
    assert lib.skiparse_lds_read_probe(p, 1 << 20, q, 1 << 30, 3, 8, 10, ctypes.byref(flop), None) == -3    # kinds 0..2
    assert lib.skiparse_lds_read_probe(p, 1 << 20, q, 8 * 512 * 4 - 1, 0, 8, 10, ctypes.byref(flop), None) == -4
    assert lib.skiparse_lds_read_probe(None, 1 << 20, q, 1 << 30, 0, 8, 10, ctypes.byref(flop), None) == -1
    assert lib.skiparse_mfma8_valu_probe(p, 1 << 20, q, 1 << 30, 6, 8, 10, ctypes.byref(flop), None) == -3   # multiples of 4 up to 16
    assert lib.skiparse_mfma_chain_probe(p, 1 << 20, q, 1 << 30, 3, 8, 10, ctypes.byref(flop), None) == -3   # 1, 2, 4 or 8
    assert lib.skiparse_probe_device_info(0, None, None) == -1
    assert lib.skiparse_probe_device_info(-1, ctypes.byref(ctypes.c_int()), ctypes.byref(ctypes.c_int())) == -1


def test_static_scratch_backward_rejects_what_does_not_fit(lib):
    """skiparse_attn_bwd_static: a problem whose delta array exceeds the static scratch is refused before any HIP call, and bad
    arguments are refused like skiparse_attn_bwd's."""
    assert lib.skiparse_static_scratch_bytes() == 16 * 1024 * 1024
    ptrs = [ctypes.c_void_p(FAKE + (i << 34)) for i in range(9)]
    f = ctypes.c_float(0.0)
    # B = 2 at the 768P shape: 2 * 40 * 80640 floats = 25.8 MB > 16 MiB
    rc = lib.skiparse_attn_bwd_static(*ptrs, 2, 40, 21, 48, 80, 128, 2, 0, f, 0, 0, None)
    assert rc == -4 and b"scratch" in lib.skiparse_strerror(rc)
    assert lib.skiparse_attn_bwd_static(*ptrs[:8], None, 1, 2, 2, 8, 8, 64, 2, 0, f, 0, 0, None) == -1
    assert lib.skiparse_attn_bwd_static(*ptrs, 1, 2, 2, 8, 6, 64, 2, 1, f, 0, 0, None) == -2   # group-wise needs W % 4 == 0
    assert lib.skiparse_attn_bwd_static(*ptrs, 1, 2, 2, 8, 8, 96, 2, 0, f, 0, 0, None) == -3   # head_dim 96
    assert lib.skiparse_attn_bwd_static(*ptrs, 1, 2, 2, 8, 8, 64, 2, 0, f, 0, 4, None) == -1   # unknown flag


def test_ssp_entry_points_reject_bad_arguments(lib):
    p, q = ctypes.c_void_p(FAKE), ctypes.c_void_p(FAKE + (1 << 30))
    for fn in (lib.skiparse_ssp_pack, lib.skiparse_ssp_unpack):
        ok = [1, 2, 2, 8, 8, 64, 2, 2, 0]  # b, heads, T, H, W, head_dim, s, group_size, dtype
        assert fn(None, q, *ok, None) == -1
        assert fn(p, p, *ok, None) == -1                                    # src == dst
        assert fn(p, q, 1, 2, 2, 8, 8, 64, 2, 3, 0, None) == -2             # group_size must divide s*s
        assert fn(p, q, 1, 2, 2, 8, 6, 64, 2, 2, 0, None) == -2             # W must be a multiple of s*s
        assert fn(p, q, 0, 2, 2, 8, 8, 64, 2, 2, 0, None) == -1
        assert fn(p, q, 1, 2, 2, 8, 8, 64, 2, 0, 0, None) == -1
        assert fn(p, q, 1, 2, 2, 8, 8, 64, 2, 2, 7, None) == -1             # unknown element type
        assert fn(ctypes.c_void_p(FAKE + 8), q, *ok, None) == -1            # misaligned


def test_fp8_flagged_entry_points(lib):
    """The any-resolution flag admits grids that the plain calls refuse; unknown flags are refused."""
    a = [ctypes.c_void_p(FAKE + i * (1 << 30)) for i in range(8)]
    f = ctypes.c_float(0.0)
    assert lib.skiparse_quantize_fp8(a[0], a[1], a[2], 1, 2, 2, 7, 9, 64, 2, 0, None) == -2
    assert lib.skiparse_quantize_fp8_ex(a[0], a[1], a[2], 1, 2, 2, 7, 9, 64, 2, 0, 4, None) == -1       # unknown flag
    assert lib.skiparse_quantize_fp8_ex(None, a[1], a[2], 1, 2, 2, 7, 9, 64, 2, 0, 2, None) == -1       # shape accepted, pointer refused
    assert lib.skiparse_quantize_fp8_ex(a[0], a[1], a[2], 1, 2, 2, 7, 9, 96, 2, 0, 2, None) == -3       # head_dim 96
    assert lib.skiparse_attn_fwd_fp8(a[0], a[1], a[2], a[3], a[4], a[5], a[6], 1, 2, 2, 7, 9, 64, 2, 1, f, None) == -2
    assert lib.skiparse_attn_fwd_fp8_ex(a[0], a[1], a[2], a[3], a[4], a[5], a[6], 1, 2, 2, 7, 9, 64, 2, 1, f, 1, None) == -1   # SKIPARSE_FUSED is no flag here
    assert lib.skiparse_attn_fwd_fp8_ex(a[0], a[1], a[2], a[3], a[4], None, a[6], 1, 2, 2, 7, 9, 64, 2, 1, f, 2, None) == -1
    assert lib.skiparse_attn_fwd_fp8_ex(a[0], a[1], a[2], a[3], a[4], a[5], a[0], 1, 2, 2, 7, 9, 64, 2, 1, f, 2, None) == -1   # out aliases q8

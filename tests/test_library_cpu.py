"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and rejects bad arguments with the documented codes before touching the device."""
import ctypes

import pytest

import paper_2210_17323_amd as g

OK, INVALID, NOT_POSDEF, HIP, UNSUPPORTED, WORKSPACE = range(6)


def test_library_loads_and_exports_every_declared_symbol():
    L = g.lib()
    names = g.exported_symbols()
    assert {"gptq_hessian_accumulate", "gptq_damp_cholesky_inverse", "gptq_quantize_layer", "gptq_pack"} <= set(names)
    for name in names:
        assert getattr(L, name) is not None
    assert g.version() >= 100


def test_workspace_sizes():
    assert g.gptq_damp_cholesky_inverse_workspace_bytes(256) >= 2 * 128 * 128 * 4 + 256 * 128 * 4
    big = g.gptq_quantize_layer_workspace_bytes(12288, 49152)
    planes = (12288 + 1024 + 49152) * 6144 + 3 * 16384      # bf16 pieces of an error panel, of 1024 and of all columns of U's rows
    assert 12288 * 49152 * 4 + planes < big < 12288 * 49152 * 4 * 1.05 + planes + (1 << 24)      # W copy + two r x 1024 error panels
    assert g.gptq_quantize_layer_workspace_bytes(0, 0) > 0
    assert g.gptq_hessian_accumulate_workspace_bytes(49152, 32768) == 49152 * 32800 * 2
    # few tiles (136 for 256 CUs): the token range is split in 5, repacked chunk + 5 partial tiles per tile
    assert g.gptq_hessian_accumulate_workspace_bytes(4096, 32768) == 4096 * 32800 * 2 + 5 * 136 * 65536 * 4
    assert g.gptq_hessian_accumulate_workspace_bytes(1024, 32768) == 0       # small matrices: the 128-tile kernel, no workspace
    assert g.gptq_hessian_accumulate_workspace_bytes(4096, 256) == 0         # too few tokens to split


def test_long_hessian_calls_are_sliced_only_on_large_matrices():
    import torch
    # one launch of the matrix-core kernel per 32768 tokens where one slice fills the chip; the workspace holds two slices
    assert g.gptq_hessian_accumulate_launches(49152, 262144, torch.float16) == 8
    assert g.gptq_hessian_accumulate_launches(12288, 262144, torch.float16) == 8
    assert g.gptq_hessian_accumulate_launches(12288, 32768, torch.float16) == 1
    assert g.gptq_hessian_accumulate_launches(12288, 40000, torch.bfloat16) == 2
    assert g.gptq_hessian_accumulate_launches(4096, 262144, torch.float16) == 1       # few tiles: one launch, split token range
    assert g.gptq_hessian_accumulate_launches(49152, 262144, torch.float32) == 1      # float32 activations: the float32 GEMM
    assert g.gptq_hessian_accumulate_launches(0, 100, torch.float16) == 0
    two_slices = 2 * 49152 * 32800 * 2 + 256
    assert g.gptq_hessian_accumulate_workspace_bytes(49152, 262144) == two_slices
    assert g.gptq_hessian_accumulate_workspace_bytes(49152, 65536) == two_slices


def _err():
    return g.lib().gptq_last_error().decode()


def test_argument_validation_happens_on_the_host():
    L = g.lib()
    one = ctypes.c_void_p(256)       # never dereferenced: every call below must fail validation first
    assert L.gptq_hessian_accumulate(one, 8, one, 0, -1, 8, 8, None, 0, None) == INVALID
    assert L.gptq_hessian_accumulate(None, 8, one, 0, 8, 8, 8, None, 0, None) == INVALID
    assert L.gptq_hessian_accumulate(one, 4, one, 0, 8, 8, 8, None, 0, None) == INVALID          # ldh < n
    assert L.gptq_hessian_accumulate(one, 8, one, 7, 8, 8, 8, None, 0, None) == INVALID          # dtype
    assert L.gptq_hessian_accumulate(one, 8, one, 0, 8, 12, 12, None, 0, None) == INVALID        # ldx % 8
    assert "ldx" in _err()
    assert L.gptq_hessian_accumulate(one, 8, one, 0, 0, 8, 8, None, 0, None) == OK               # empty is a no-op
    # a workspace that is given must be usable: too small or misaligned is an error, not a silent slow path
    assert L.gptq_hessian_accumulate(one, 49152, one, 0, 49152, 32768, 32768, one, 1024, None) == WORKSPACE
    assert L.gptq_hessian_accumulate(one, 49152, one, 0, 49152, 32768, 32768, ctypes.c_void_p(264), 1 << 40, None) == WORKSPACE
    assert "workspace" in _err()
    tm = L.gptq_hessian_accumulate_token_major
    assert tm(one, 8, one, 0, 8, 16, 4, one, 1 << 30, None) == INVALID                           # ldx < n
    assert tm(one, 8, one, 2, 8, 16, 8, one, 1 << 30, None) == UNSUPPORTED                       # float32
    assert tm(one, 8, one, 0, 8, 16, 8, None, 0, None) == WORKSPACE
    assert tm(one, 8, one, 0, 8, 16, 8, one, 64, None) == WORKSPACE
    assert tm(one, 8, one, 0, 8, 0, 8, None, 0, None) == OK
    assert g.gptq_hessian_accumulate_token_major_workspace_bytes(300, 100) == 512 * 160 * 2
    assert L.gptq_damp_cholesky_inverse(one, 8, 8, -0.5, one, 1 << 30, one, None) == INVALID
    assert L.gptq_damp_cholesky_inverse(one, 8, 8, 0.01, one, 16, one, None) == WORKSPACE
    assert L.gptq_damp_cholesky_inverse(one, 8, 8, 0.01, None, 0, one, None) == WORKSPACE
    assert L.gptq_damp_cholesky_inverse(one, 6, 6, 0.01, one, 1 << 30, one, None) == INVALID   # ld % 4
    na = L.gptq_damp_cholesky_inverse_noalloc
    assert L.gptq_noalloc_max_n() == 4096
    assert na(one, 4100, 4100, 0.01, one, None) == UNSUPPORTED and "4096" in _err()       # beyond the library's fixed scratch array
    assert na(one, 8, 8, -1.0, one, None) == INVALID and na(one, 8, 8, 0.01, None, None) == INVALID
    assert na(one, 6, 6, 0.01, one, None) == INVALID and na(one, 8, 0, 0.01, one, None) == OK
    q = lambda **kw: L.gptq_quantize_layer(one, kw.get("wd", 0), 256, kw.get("r", 4), 256, one, 256, kw.get("bits", 4),
                                           kw.get("grid", 0), kw.get("block", 128), kw.get("group", 0), one, 256, one, one,
                                           None, 0, None, kw.get("ws", one), kw.get("wsb", 1 << 30), None)
    assert q(bits=5) == INVALID and q(bits=1) == INVALID
    assert q(grid=3) == INVALID
    assert q(block=64) == UNSUPPORTED and q(block=0) == INVALID
    assert q(group=100) == INVALID          # 256 % 100 != 0
    assert q(group=4) == UNSUPPORTED
    assert q(wd=9) == INVALID
    assert q(wsb=1024) == WORKSPACE
    assert q(r=0) == OK
    assert q(grid=1, bits=0, wsb=8) == WORKSPACE   # ternary ignores bits; fails later on the workspace
    tu = L.gptq_trailing_update
    assert tu(ctypes.c_void_p(260), 64, one, 8, one, 64, 4, 64, 8, None) == INVALID and "aligned" in _err()
    assert tu(one, 64, one, 10, one, 64, 4, 64, 8, None) == INVALID          # lde % 4
    assert tu(one, 60, one, 8, one, 64, 4, 64, 8, None) == INVALID          # ldw < ncols
    assert tu(None, 64, one, 8, one, 64, 4, 64, 8, None) == INVALID
    assert tu(one, 64, one, 8, one, 64, 0, 64, 8, None) == OK and tu(one, 64, one, 8, one, 64, 4, 64, 0, None) == OK
    assert L.gptq_release_thread_resources() == OK          # nothing created on this thread: a no-op
    tus = L.gptq_trailing_update_split
    assert tus(one, 256, one, 1024, one, 256, 256, 256, 512, one, 1 << 30, None) == UNSUPPORTED and "1024" in _err()   # k
    assert tus(one, 256, one, 1024, one, 256, 200, 256, 1024, one, 1 << 30, None) == UNSUPPORTED                      # r % 256
    assert tus(one, 256, one, 1024, one, 256, 256, 256, 1024, one, 1024, None) == WORKSPACE
    assert tus(one, 256, one, 1024, one, 256, 256, 256, 1024, None, 0, None) == WORKSPACE
    assert tus(one, 128, one, 1024, one, 256, 256, 256, 1024, one, 1 << 30, None) == INVALID                           # ldw < ncols
    assert tus(one, 256, one, 1024, one, 256, 0, 256, 1024, one, 1 << 30, None) == OK
    assert g.gptq_trailing_update_split_workspace_bytes(256, 512) == 3 * (3 * 32 * 16384) + 2 * 16384 + 256
    prev = g.gptq_set_split_min_tiles(9)
    assert g.gptq_set_split_min_tiles(-3) == 9 and g.gptq_set_split_min_tiles(prev) == 0      # a value <= 0 is the library's own rule
    sus = L.gptq_symmetric_update_split
    assert sus(one, 256, one, 1024, 256, 128, one, 1 << 30, None) == UNSUPPORTED
    assert sus(one, 256, one, 1024, 300, 1024, one, 1 << 30, None) == UNSUPPORTED
    assert sus(one, 256, one, 1024, 256, 1024, one, 64, None) == WORKSPACE
    assert sus(one, 256, one, 1000, 256, 1024, one, 1 << 30, None) == INVALID                                           # ldp < k
    assert sus(one, 256, one, 1024, 0, 1024, None, 0, None) == OK
    assert L.gptq_pack(one, 64, 2, 64, 5, one, 8, None) == INVALID
    assert L.gptq_pack(one, 64, 2, 64, 3, one, 5, None) == INVALID      # 64*3/32 = 6 words needed
    assert L.gptq_pack(one, 32, 2, 64, 3, one, 6, None) == INVALID      # ldc < n
    assert L.gptq_unpack(one, 6, 2, 64, 3, None, 64, None) == INVALID
    assert L.gptq_pack(one, 64, 0, 64, 3, one, 6, None) == OK
    assert L.gptq_check_info(None, None, None) == INVALID
    dq = lambda **kw: L.gptq_dequantize_packed(one, kw.get("ldp", 6), kw.get("r", 2), kw.get("n", 64), kw.get("bits", 3), one, one,
                                               kw.get("group", 0), kw.get("out", one), kw.get("od", 0), kw.get("ldo", 64), None)
    assert dq(bits=5) == INVALID and dq(ldp=5) == INVALID and dq(group=48) == INVALID and dq(od=1) == INVALID
    assert dq(ldo=32) == INVALID and dq(out=None) == INVALID and dq(r=0) == OK
    mv = lambda **kw: L.gptq_matvec_packed(one, kw.get("ldp", 6), kw.get("r", 2), kw.get("n", 64), kw.get("bits", 3), one, one,
                                           kw.get("group", 0), kw.get("x", one), kw.get("xd", 0), kw.get("y", one), None)
    assert mv(bits=1) == INVALID and mv(ldp=2) == INVALID and mv(xd=1) == INVALID and mv(x=None) == INVALID
    assert mv(group=4) == UNSUPPORTED and mv(group=-8) == INVALID and mv(r=0) == OK


def test_missing_library_fails_loudly(tmp_path):
    with pytest.raises(FileNotFoundError):
        g.load_library(str(tmp_path / "nope.so"))

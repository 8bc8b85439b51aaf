"""The C-ABI library loads, exports every symbol include/qblora.h declares, and validates on the host.

No compute is launched here: every call below is rejected by host-side argument checks before any
HIP call, so the tests run without a GPU.
"""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "qblora.h")


@pytest.fixture(scope="module")
def qb():
    from paper_2407_17029_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2407_17029_amd import build
        build.build_library()
    binding.lib()
    return binding


def _declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(q[a]?blora_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported(qb):
    names = _declared_functions()
    assert set(names) == set(qb.EXPORTS)
    for n in names:
        assert hasattr(qb.lib(), n), n


def test_strerror(qb):
    assert qb.strerror(0) == "ok"
    for code in range(-6, 0):
        assert qb.strerror(code) and "unknown" not in qb.strerror(code)
    assert "unknown" in qb.strerror(-99)


def test_host_validation_rejects_bad_arguments(qb):
    L = qb.lib()
    qw = qb.CQWeight()
    dummy = C.c_void_p(0x1000)       # never dereferenced: the calls fail validation first
    assert L.qblora_quantize_blockwise(None, 64, 64, 64, 0, None, 0, C.byref(qw), None) == -1
    assert L.qblora_quantize_blockwise(dummy, 64, 100, 64, 0, None, 0, C.byref(qw), None) == -2
    assert L.qblora_quantize_blockwise(dummy, 64, 64, 32, 0, None, 0, C.byref(qw), None) == -3
    assert L.qblora_quantize_blockwise(dummy, 0, 64, 64, 0, None, 0, C.byref(qw), None) == -2
    qw.d_out, qw.d_in, qw.block = 128, 128, 64
    assert L.qblora_linear_fwd(C.byref(qw), None, dummy, 4, dummy, None, 0, None) == -1      # codes missing
    qw.codes = 0x1000; qw.scales = 0x1000
    ad = qb.CAdapter()
    ad.lambda1, ad.lambda2, ad.R, ad.s, ad.A, ad.B = 3, 2, 16, 1.0, 0x1000, 0x1000
    assert L.qblora_linear_fwd(C.byref(qw), C.byref(ad), dummy, 4, dummy, dummy, 1 << 30, None) == -2   # 128 % 3
    ad.lambda1 = 2
    assert L.qblora_linear_fwd(C.byref(qw), C.byref(ad), dummy, 4, dummy, None, 0, None) == -4           # workspace
    assert L.qblora_linear_fwd(C.byref(qw), C.byref(ad), dummy, -1, dummy, dummy, 1 << 30, None) == -2
    assert L.qblora_linear_fwd(C.byref(qw), C.byref(ad), dummy, 0, dummy, None, 0, None) == 0            # empty batch
    assert L.qblora_linear_bwd(C.byref(qw), C.byref(ad), dummy, dummy, 4, None, None, None, dummy, 1 << 30, None) == -1
    qw.d_out = 96
    assert L.qblora_linear_fwd(C.byref(qw), None, dummy, 4, dummy, None, 0, None) == -2                  # d_out % 64
    qw.d_out = 128
    out = qb.CQWeight()
    out.codes = out.scales = out.beta = 0x1000
    assert L.qablora_merge_quantize(C.byref(qw), dummy, 2, 2, C.c_float(1.0), 0, C.byref(out), None) == -5
    assert L.qablora_merge_quantize(C.byref(qw), dummy, 3, 2, C.c_float(1.0), 1, C.byref(out), None) == -2
    assert L.qablora_merge_quantize(C.byref(qw), None, 2, 2, C.c_float(1.0), 1, C.byref(out), None) == -1
    Pq = C.POINTER(qb.CQWeight)
    barr, oarr, harr = (Pq * 2)(C.pointer(qw), C.pointer(qw)), (Pq * 2)(C.pointer(out), C.pointer(out)), (C.c_void_p * 2)(0x1000, 0)
    assert L.qablora_merge_quantize_batch(0, None, None, 2, 2, C.c_float(1.0), 1, None, None) == 0       # empty batch
    assert L.qablora_merge_quantize_batch(2, None, harr, 2, 2, C.c_float(1.0), 1, oarr, None) == -1
    assert L.qablora_merge_quantize_batch(2, barr, harr, 2, 2, C.c_float(1.0), 1, oarr, None) == -1      # second H missing
    assert L.qablora_merge_quantize_batch(-1, barr, harr, 2, 2, C.c_float(1.0), 1, oarr, None) == -2


def test_host_validation_of_the_later_entry_points(qb):
    """Single-matrix adapter, 16-bit merge, small-batch inference, saved activations: bad arguments are turned
    into error codes on the host, before any launch."""
    L = qb.lib()
    qw = qb.CQWeight()
    dummy = C.c_void_p(0x1000)       # never dereferenced
    qw.d_out, qw.d_in, qw.block = 128, 256, 64
    qw.codes = qw.scales = 0x1000
    f = C.c_float(1.0)
    big = 1 << 30
    # single-matrix adapter
    assert L.qablora_linear_fwd(C.byref(qw), None, 2, 2, f, dummy, 4, dummy, dummy, big, None) == -1       # H missing
    assert L.qablora_linear_fwd(C.byref(qw), dummy, 3, 2, f, dummy, 4, dummy, dummy, big, None) == -2      # 256 % 3
    assert L.qablora_linear_fwd(C.byref(qw), dummy, 64, 2, f, dummy, 4, dummy, dummy, big, None) == -2     # pooled width 4
    assert L.qablora_linear_fwd(C.byref(qw), dummy, 2, 2, f, dummy, 4, dummy, None, 0, None) == -4         # workspace
    assert L.qablora_linear_fwd(C.byref(qw), dummy, 2, 2, f, dummy, 0, dummy, None, 0, None) == 0          # empty batch
    assert L.qablora_linear_bwd(C.byref(qw), dummy, 2, 2, f, dummy, dummy, 4, None, None, dummy, big, None) == -1
    assert L.qablora_linear_fwd_workspace_bytes(C.byref(qw), 2, 2, 64) % 256 == 0
    assert L.qablora_linear_bwd_workspace_bytes(C.byref(qw), 2, 2, 64) > 0
    # 16-bit merge
    assert L.qblora_merge_bf16(C.byref(qw), None, 2, 2, f, dummy, None) == -1
    assert L.qblora_merge_bf16(C.byref(qw), dummy, 2, 2, f, None, None) == -1
    assert L.qblora_merge_bf16(C.byref(qw), dummy, 5, 2, f, dummy, None) == -2
    # small-batch inference
    assert L.qblora_linear_decode(C.byref(qw), None, dummy, 257, dummy, None, 0, None) == -2              # T > 256
    assert L.qblora_linear_decode_tokens_workspace_bytes(C.byref(qw), 16) == L.qblora_linear_decode_workspace_bytes(C.byref(qw))
    big_qw = qb.CQWeight()
    big_qw.d_out, big_qw.d_in, big_qw.block = 4096, 4096, 64
    big_qw.codes = big_qw.scales = 0x1000
    need = L.qblora_linear_decode_tokens_workspace_bytes(C.byref(big_qw), 64)                            # split partial tiles
    assert need >= 2 * 64 * 4096 * 4 and need % 256 == 0
    assert L.qblora_linear_decode(C.byref(big_qw), None, dummy, 64, dummy, dummy, need - 1, None) == -4
    assert L.qblora_linear_decode(C.byref(qw), None, None, 4, dummy, None, 0, None) == -1
    assert L.qblora_linear_decode(C.byref(qw), None, dummy, 0, dummy, None, 0, None) == 0
    assert L.qblora_linear_decode(C.byref(qw), C.c_void_p(0x1010), dummy, 4, dummy, None, 0, None) == -2   # pack alignment
    assert L.qblora_decode_pack(C.byref(qw), None, None) == -1
    rows, bpr = 256, 4
    assert L.qblora_decode_pack_bytes(C.byref(qw)) == rows * bpr * 32 + rows * bpr * 4                    # codes + scales
    qw.beta = 0x1000
    assert L.qblora_decode_pack_bytes(C.byref(qw)) == rows * bpr * 32 + 2 * rows * bpr * 4
    qw.beta = None
    # saved activations
    ad = qb.CAdapter()
    ad.lambda1, ad.lambda2, ad.R, ad.s, ad.A, ad.B = 2, 2, 16, 1.0, 0x1000, 0x1000
    assert L.qblora_saved_bytes(C.byref(ad), 100) == 2 * 100 * 16 * 2
    assert L.qblora_saved_bytes(None, 100) == 0
    assert L.qblora_linear_fwd_save(C.byref(qw), C.byref(ad), dummy, 4, dummy, None, dummy, big, None) == -1
    assert L.qblora_linear_bwd_saved(C.byref(qw), C.byref(ad), dummy, dummy, 4, None, dummy, dummy, dummy, dummy, big,
                                     None) == -1


def test_workspace_sizes(qb):
    L = qb.lib()
    qw = qb.CQWeight()
    qw.d_out, qw.d_in, qw.block = 4096, 4096, 64
    qw.codes = qw.scales = 0x1000
    few = L.qblora_dense_min_tokens() - 1                               # weight tiles rebuilt in LDS per token tile
    many = L.qblora_dense_min_tokens()                                  # weight dequantized once into the workspace
    assert few >= 256
    scales_t = 4 * 4096 * 64                                            # tile-ordered fp32 block scales
    assert L.qblora_linear_fwd_workspace_bytes(C.byref(qw), None, few) == scales_t
    ad = qb.CAdapter()
    ad.lambda1, ad.lambda2, ad.R, ad.s, ad.A, ad.B = 2, 2, 128, 1.0, 0x1000, 0x1000
    fwd = L.qblora_linear_fwd_workspace_bytes(C.byref(qw), C.byref(ad), few)
    assert fwd == scales_t + 2 * (128 * 4096 + 2048 * 128 + few * 128) + (256 - 2 * few * 128 % 256) % 256   # + At_x, Bt, U in bf16
    bwd = L.qblora_linear_bwd_workspace_bytes(C.byref(qw), C.byref(ad), few)
    assert bwd > fwd and bwd % 256 == 0
    dense_w = 2 * 4096 * 4096                                           # the bf16 weight
    assert L.qblora_linear_fwd_workspace_bytes(C.byref(qw), None, many) == dense_w
    fwd_many = L.qblora_linear_fwd_workspace_bytes(C.byref(qw), C.byref(ad), many)
    assert fwd_many == dense_w + 2 * (128 * 4096 + 2048 * 128 + many * 128)
    assert L.qblora_linear_bwd_workspace_bytes(C.byref(qw), C.byref(ad), many) > dense_w
    # double-quantized scales: the one-off pass reads reconstructed fp32 scales from the workspace
    qw.scale_mode, qw.scale_group = 1, 256
    qw.scale_codes = qw.scale_step = qw.scale_mid = 0x1000
    assert L.qblora_linear_fwd_workspace_bytes(C.byref(qw), None, many) == dense_w + 4 * 4096 * 64

"""The C-ABI boundary without a GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

from paper_2603_22943_amd import taq as T

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000001000  # 16-byte aligned, never dereferenced on error paths
ODD = FAKE + 4


def header_functions():
    text = open(os.path.join(ROOT, "include", "taq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(taq_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = T.load()
    names = header_functions()
    assert set(names) == set(T.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def test_struct_sizes_match_header_layout():
    assert ctypes.sizeof(T.taq_shape) == 14 * 4
    assert ctypes.sizeof(T.taq_request) == 7 * 8
    assert ctypes.sizeof(T.taq_debug) == 8 * 8 + 8


def test_status_strings():
    assert T.taq_status_string(0) == "TAQ_OK"
    for code in (-1, -2, -3, -4, -5, -6):
        assert T.taq_status_string(code).startswith("TAQ_ERR_")
    assert "unknown" in T.taq_status_string(-99)


def test_size_queries_are_host_only_and_consistent():
    s = T.make_shape(B=2, N=4096, C=320, H=8, T=77, Cc=768, bits_kv=8)
    kv8 = T.taq_kv_packed_bytes(s)
    ws = T.taq_workspace_bytes(s)
    s4 = T.make_shape(B=2, N=4096, C=320, H=8, T=77, Cc=768, bits_kv=4)
    kv4 = T.taq_kv_packed_bytes(s4)
    # int4 codes take half the bytes of int8 codes
    code8 = 2 * 2 * 77 * 320
    assert kv8 - kv4 == pytest.approx(code8 / 2, abs=1024)
    # a shape without the operand-ordered image: 16-bit has no code section at all
    a8 = T.taq_kv_packed_bytes(T.make_shape(B=2, N=64, C=96, H=4, T=77, Cc=64, bits_kv=8))
    a16 = T.taq_kv_packed_bytes(T.make_shape(B=2, N=64, C=96, H=4, T=77, Cc=64, bits_kv=16))
    assert a8 - a16 == pytest.approx(2 * 2 * 77 * 96, abs=1024)
    assert kv8 % 256 == 0 and ws % 256 == 0
    # the plain code sections: C bytes per row at 8 bits, C/2 at 4 bits, none at 16; V behind K, both inside the buffer
    k8, v8, rb8 = T.taq_kv_code_layout(s)
    k4, v4, rb4 = T.taq_kv_code_layout(s4)
    assert (rb8, rb4) == (320, 160) and v8 - k8 >= 2 * 77 * rb8 and v4 - k4 >= 2 * 77 * rb4 and v8 + 2 * 77 * rb8 <= kv8
    assert T.taq_kv_code_layout(T.make_shape(B=2, N=64, C=96, H=4, T=77, Cc=64, bits_kv=16))[2] == 0
    # workspace holds at least the int8 Q~ codes, their float32 source and the float32 O
    assert ws >= 2 * 4096 * 320 * (1 + 4 + 1 + 4 + 1)


@pytest.mark.parametrize("kw,expect", [
    (dict(bits_kv=5), T.TAQ_ERR_UNSUPPORTED_BITS),
    (dict(bits_prob=5), T.TAQ_ERR_UNSUPPORTED_BITS),
    (dict(bits_prob=2), T.TAQ_ERR_UNSUPPORTED_BITS),
    (dict(bits_q=12), T.TAQ_ERR_UNSUPPORTED_BITS),
    (dict(prob_grid=3), T.TAQ_ERR_INVALID_ARG),
    (dict(bits_proj=4), T.TAQ_ERR_UNSUPPORTED_BITS),
    (dict(C=324), T.TAQ_ERR_BAD_SHAPE),  # C % H != 0
    (dict(C=96, H=8), T.TAQ_ERR_BAD_SHAPE),  # d = 12, not a multiple of 8
    (dict(C=2048, H=8), T.TAQ_ERR_BAD_SHAPE),  # d = 256 > 160
    (dict(T=97), T.TAQ_ERR_BAD_SHAPE),
    (dict(Cc=100), T.TAQ_ERR_BAD_SHAPE),
    (dict(B=0), T.TAQ_ERR_INVALID_ARG),
    (dict(softmax_scale=-1.0), T.TAQ_ERR_INVALID_ARG),
    (dict(tok_tile=8), T.TAQ_ERR_INVALID_ARG),
])
def test_bad_shapes_are_rejected(kw, expect):
    base = dict(B=2, N=64, C=320, H=8, T=77, Cc=768)
    base.update(kw)
    s = T.make_shape(**base)
    n = ctypes.c_size_t(0)
    assert T.load().taq_kv_packed_bytes(ctypes.byref(s), ctypes.byref(n)) == expect
    with pytest.raises(T.TaqError) as e:
        T.taq_kv_packed_bytes(s)
    assert e.value.status == expect


def test_entry_points_reject_null_misaligned_and_inconsistent_arguments_without_launching():
    lib = T.load()
    s = T.make_shape(B=1, N=64, C=320, H=8, T=77, Cc=768, bits_kv=8)
    sp = ctypes.byref(s)
    # taq_quantize_kv
    assert lib.taq_quantize_kv(None, FAKE, FAKE, FAKE, 8, sp, FAKE, FAKE, None) == T.TAQ_ERR_INVALID_ARG
    assert lib.taq_quantize_kv(FAKE, FAKE, FAKE, FAKE, 4, sp, FAKE, FAKE, None) == T.TAQ_ERR_INVALID_ARG  # bits != shape
    assert lib.taq_quantize_kv(ODD, FAKE, FAKE, FAKE, 8, sp, FAKE, FAKE, None) == T.TAQ_ERR_MISALIGNED
    assert lib.taq_quantize_kv(FAKE, FAKE, FAKE, FAKE, 8, None, FAKE, FAKE, None) == T.TAQ_ERR_INVALID_ARG
    # taq_quantize_kv_w8
    assert lib.taq_quantize_kv_w8(FAKE, FAKE, None, FAKE, 8, sp, FAKE, FAKE, None) == T.TAQ_ERR_INVALID_ARG
    assert lib.taq_quantize_kv_w8(FAKE, FAKE, FAKE, FAKE, 4, sp, FAKE, FAKE, None) == T.TAQ_ERR_INVALID_ARG
    assert lib.taq_quantize_kv_w8(FAKE, FAKE, ODD, FAKE, 8, sp, FAKE, FAKE, None) == T.TAQ_ERR_MISALIGNED
    # taq_cross_attn
    assert lib.taq_cross_attn(FAKE, FAKE, FAKE, FAKE, FAKE, None, sp, None, FAKE, None) == T.TAQ_ERR_INVALID_ARG
    assert lib.taq_cross_attn(FAKE, FAKE, FAKE, ODD, FAKE, None, sp, FAKE, FAKE, None) == T.TAQ_ERR_MISALIGNED
    s0 = T.make_shape(B=1, N=0, C=320, H=8, T=77, Cc=768)
    assert lib.taq_cross_attn(FAKE, FAKE, FAKE, FAKE, FAKE, None, ctypes.byref(s0), FAKE, FAKE, None) == T.TAQ_ERR_INVALID_ARG
    # taq_cross_attn_static: the size limit is checked on the host, before anything touches the GPU
    assert lib.taq_cross_attn_static(FAKE, FAKE, FAKE, FAKE, FAKE, None, sp, None, None) == T.TAQ_ERR_INVALID_ARG
    big = T.make_shape(B=2, N=4096, C=1280, H=8, T=77, Cc=768)   # head-group path: ~11*B*N*C bytes of scratch
    assert lib.taq_cross_attn_static(FAKE, FAKE, FAKE, FAKE, FAKE, None, ctypes.byref(big), FAKE, None) == T.TAQ_ERR_SCRATCH_TOO_SMALL
    assert T.taq_workspace_bytes(big) > T.TAQ_STATIC_SCRATCH_BYTES
    # taq_quantize_weight
    assert lib.taq_quantize_weight(FAKE, 0, 64, FAKE, FAKE, None) == T.TAQ_ERR_INVALID_ARG
    assert lib.taq_quantize_weight(FAKE, 8, 60, FAKE, FAKE, None) == T.TAQ_ERR_BAD_SHAPE
    assert lib.taq_quantize_weight(FAKE, 8, 64, ODD, FAKE, None) == T.TAQ_ERR_MISALIGNED
    # batched
    assert lib.taq_cross_attn_batched(0, None, sp, FAKE, None) == T.TAQ_ERR_INVALID_ARG
    tab = (T.taq_request * 2)()
    tab[0] = T.taq_request(FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE)
    tab[1] = T.taq_request(FAKE, FAKE, FAKE, FAKE, FAKE, None, None)  # second request lacks `out`
    assert lib.taq_cross_attn_batched(2, tab, sp, FAKE, None) == T.TAQ_ERR_INVALID_ARG
    # unpack
    assert lib.taq_unpack_kv(None, sp, None, None, None, None, None, None, None) == T.TAQ_ERR_INVALID_ARG
    # weight re-layout
    assert lib.taq_pack_weight(None, sp, FAKE, None) == T.TAQ_ERR_INVALID_ARG
    assert lib.taq_pack_weight(FAKE, sp, ODD, None) == T.TAQ_ERR_MISALIGNED
    bad = T.make_shape(B=1, N=64, C=320, H=8, T=77, Cc=768, w_layout=2)
    assert lib.taq_pack_weight(FAKE, ctypes.byref(bad), FAKE, None) == T.TAQ_ERR_INVALID_ARG
    # the re-laid-out buffer holds the row-major codes plus one KiB per (head, 16-row tile, 64-code step)
    assert T.taq_weight_bytes(s) == 320 * 320 + 8 * 3 * 5 * 1024


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2603_22943_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith(".py"):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2603_22943_amd" not in text and "libtaq" not in text.replace("the HIP library", ""), f

"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, its layout
index functions agree with the formulas of include/nsn.h, and argument errors are reported
before anything touches a GPU."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2505_18231_amd import api
from tests import helpers

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(api.LIB_PATH):
        from paper_2505_18231_amd.build import build_library
        build_library(verbose=False)
    return api.lib()


def test_exports_every_declared_symbol(L):
    header = open(os.path.join(ROOT, "include", "nsn.h")).read()
    names = set(re.findall(r"\b(nsn_[a-z_]+)\s*\(", header))
    names -= {"nsn_shape", "nsn_cache"}
    assert {"nsn_build_codebook", "nsn_finetune_codebook", "nsn_encode", "nsn_decode_attention",
            "nsn_decode_attention_residual", "nsn_workspace_bytes", "nsn_build_rope_table",
            "nsn_rope_table_bytes"} <= names
    for n in names:
        assert hasattr(L, n), n


@pytest.mark.parametrize("fmt", ["1bit", "2bit", "sign", "2bit-dq"])
def test_layout_offsets_match_header_formulas_and_are_bijections(L, fmt):
    import ctypes as C
    n = 192
    shape = {"1bit": api.make_shape(8, 4, 1, 256), "2bit": api.make_shape(4, 4, 1, 256),
             "sign": api.make_shape(8, 4, 1, 256, sign_format=True),
             "2bit-dq": api.make_shape(4, 4, 1, 256, side_bits=4)}[fmt]
    J = api.code_bytes_per_token(shape)
    layout = "tiled" if fmt in ("1bit", "2bit", "2bit-dq") else "legacy"
    for kind, fn in (("k", L.nsn_k_code_offset), ("v", L.nsn_v_code_offset)):
        ref = helpers.code_offsets(J, kind, n, layout)
        got = np.array([[fn(C.byref(shape), t, j) for j in range(J)] for t in range(n)])
        assert np.array_equal(ref, got)
        assert sorted(got.ravel().tolist()) == list(range(n * J))
        assert fn(C.byref(shape), 0, J) == -1 and fn(C.byref(shape), -1, 0) == -1
        if layout == "legacy" and kind == "v":
            # a V block holds J consecutive tokens of one sub-vector contiguously
            assert np.array_equal(ref[:J, 3], 3 * J + np.arange(J))
        if layout == "tiled":
            # every 64-token block is self-contained, and inside it every lane owns one run of J bytes
            assert ref[:64].max() == 64 * J - 1 and ref[64:128].min() == 64 * J
            lane_of = ref[:64] // J
            if kind == "k":   # lane = 16 * (32-channel quarter) + token % 16
                assert np.array_equal(lane_of, 16 * (np.arange(J)[None, :] // (J // 4)) + (np.arange(64) % 16)[:, None])
            else:             # lane = 16 * (token % 16 / 4) + 4 * (token % 4) + sub-vector % 4
                tb = np.arange(64)[:, None]
                assert np.array_equal(lane_of, 16 * (tb % 16 // 4) + 4 * (tb % 4) + np.arange(J)[None, :] % 4)


def test_pack_unpack_roundtrip():
    g = np.random.default_rng(0)
    for J in (16, 32):
        codes = g.integers(0, 256, size=(200, J), dtype=np.uint8)
        for kind in "kv":
            for layout in ("tiled", "legacy"):
                raw = helpers.pack_codes(codes, kind, 256, layout)
                assert np.array_equal(helpers.unpack_codes(raw, kind, J, layout)[:200], codes)


def test_shape_validation_and_error_text(L):
    good = api.make_shape(4, 32, 8, 8192, 64)
    # 256 arrival counters (one 256-byte line per sequence and query head) + one fp32 partial of 258 floats per (head, split)
    assert api.nsn_workspace_bytes(good, api.NSN_OP_DECODE, 8, 0, 4) == 8 * 32 * 256 + 8 * 32 * 4 * 258 * 4
    assert api.nsn_workspace_bytes(good, api.NSN_OP_ENCODE, 8, 8192) == 8 * 8 * 2 * 128 * 128 * 8
    assert api.nsn_max_groups(good) == 128
    assert api.nsn_max_groups(api.make_shape(8, 1, 1, 1024, 0)) == 1
    bad = api.make_shape(5, 32, 8, 8192, 64)
    assert api.nsn_workspace_bytes(bad, api.NSN_OP_DECODE, 8) == 0
    kc = api.nsn_cache(None, None, None, None)
    rc = L.nsn_encode(C.byref(bad), None, None, None, 1, None, None, 1, 0, C.byref(kc), C.byref(kc), None, 0, None)
    assert rc == api.NSN_ERR_UNSUPPORTED and b"sub_dim" in L.nsn_last_error()
    rc = L.nsn_encode(C.byref(good), None, None, None, 1, None, None, 1, 0, C.byref(kc), C.byref(kc), None, 0, None)
    assert rc == api.NSN_ERR_INVALID_ARG
    odd = api.make_shape(4, 32, 8, 8192, 48)
    rc = L.nsn_decode_attention(C.byref(odd), None, None, C.byref(kc), C.byref(kc), None, 1, 1, 1.0, 0, None,
                                None, 0, None)
    assert rc == api.NSN_ERR_INVALID_ARG and b"group_size" in L.nsn_last_error()
    rc = L.nsn_build_codebook(None, 1000, 8, 128, 1, None, None, None, 0, None)
    assert rc == api.NSN_ERR_UNSUPPORTED
    # side information width, rotary table alignment
    odd_bits = api.make_shape(4, 32, 8, 8192, 64, side_bits=5)
    assert api.nsn_workspace_bytes(odd_bits, api.NSN_OP_DECODE, 8) == 0
    rc = L.nsn_decode_attention(C.byref(odd_bits), None, None, C.byref(kc), C.byref(kc), None, 1, 1, 1.0, 0, None,
                                None, 0, None)
    assert rc == api.NSN_ERR_UNSUPPORTED and b"side_bits" in L.nsn_last_error()
    dq = api.make_shape(4, 32, 8, 8192, 64, side_bits=4)
    # 4-bit side information: the encoder workspace also carries fp16(s1) of every new token
    assert api.nsn_workspace_bytes(dq, api.NSN_OP_ENCODE, 8, 8192) == 8 * 8 * 2 * 128 * 128 * 8 + 8 * 8 * 2 * 8192 * 2
    misaligned = api.make_shape(4, 32, 8, 8192, 64)
    misaligned.rope_table = 0x1008
    rc = L.nsn_decode_attention(C.byref(misaligned), None, None, C.byref(kc), C.byref(kc), None, 1, 1, 1.0, 0, None,
                                None, 0, None)
    assert rc == api.NSN_ERR_INVALID_ARG and b"rope_table" in L.nsn_last_error()
    rc = L.nsn_quantize_codebook(None, 4, 256, None, None, None)
    assert rc == api.NSN_ERR_INVALID_ARG
    rc = L.nsn_quantize_codebook(None, 5, 256, None, None, None)
    assert rc == api.NSN_ERR_UNSUPPORTED
    # rotary table: three fixed parts (2 x 16 KiB fp16, 64 KiB fp64) + 1536 bytes per 64-token block
    assert L.nsn_rope_table_bytes(8192) == 98304 + 128 * 1536
    assert L.nsn_rope_table_bytes(100) == 0 and L.nsn_rope_table_bytes(0) == 0
    rc = L.nsn_build_rope_table(None, 8192, None, 0, None)
    assert rc == api.NSN_ERR_INVALID_ARG and b"rope" in L.nsn_last_error()


def test_variant_selection_returns_the_previous_choice(L):
    first = api.nsn_select_variant(api.NSN_OP_DECODE, api.NSN_VARIANT_ALT)
    assert first in (api.NSN_VARIANT_DEFAULT, api.NSN_VARIANT_ALT)
    # the lookup-table decode kernel takes index-only formats without a residual only: the shape check says so
    dq = api.make_shape(4, 32, 8, 8192, 64, side_bits=4)
    kc = api.nsn_cache(1, 1, 1, None)
    rc = L.nsn_decode_attention(C.byref(dq), 1, 1, C.byref(kc), C.byref(kc), 1, 1, 64, 1.0, 0, 1, None, 0, None)
    assert rc == api.NSN_ERR_UNSUPPORTED and b"lookup-table" in L.nsn_last_error()
    assert api.nsn_select_variant(api.NSN_OP_DECODE, first) == api.NSN_VARIANT_ALT
    assert api.nsn_select_variant(api.NSN_OP_ENCODE, api.NSN_VARIANT_DEFAULT) in (0, 1)
    assert L.nsn_select_variant(api.NSN_OP_CODEBOOK, 0) == api.NSN_ERR_INVALID_ARG
    assert L.nsn_select_variant(api.NSN_OP_DECODE, 2) == api.NSN_ERR_INVALID_ARG


def test_product_package_does_not_import_oracle():
    pkg = os.path.join(ROOT, "paper_2505_18231_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".h", ".hip", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.replace("oracle's tests", ""), f

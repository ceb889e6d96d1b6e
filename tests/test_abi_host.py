"""Host-only checks of the C ABI: the library loads, exports every symbol include/lutnn.h declares,
and rejects bad arguments on the host before anything could be launched.  No GPU needed."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lut():
    import paper_2302_03213_amd as lut_mod
    return lut_mod


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "lutnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"LUTNN_API[^;(]*?\b(lutnn_\w+)\s*\(", text)))


def test_header_declares_the_documented_entry_points():
    names = declared_symbols()
    for must in ("lutnn_build_table", "lutnn_encode", "lutnn_lookup", "lutnn_linear"):
        assert must in names
    assert len(names) >= 19


def test_header_is_plain_c99(tmp_path):
    """The boundary is a C ABI: the header must compile as C, without torch or HIP types."""
    import subprocess
    src = tmp_path / "use_header.c"
    src.write_text('#include "lutnn.h"\n'
                   'int main(void) { lutnn_layer l; lutnn_tree t; lutnn_conv2d_geom g;\n'
                   '  (void)l; (void)t; (void)g; return LUTNN_OK; }\n')
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only",
                        "-I", os.path.join(ROOT, "include"), str(src)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def test_library_exports_every_declared_symbol(lut):
    for name in declared_symbols():
        assert hasattr(lut.LIB, name), "liblutnn.so does not export %s" % name
    assert sorted(lut.binding.EXPORTS) == declared_symbols()


def test_no_other_symbols_leak(lut):
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", lut.binding._build.LIB],
                         capture_output=True, text=True, check=True).stdout
    syms = [l.split()[-1] for l in out.splitlines() if " T " in l]
    assert sorted(s for s in syms if s.startswith("lutnn_")) == declared_symbols()


def test_size_queries(lut):
    assert lut.table_bytes(1024, 16, 4096, lut.TABLE_I8) == 64 * 2 ** 20  # 64 MiB table
    assert lut.table_bytes(128, 16, 512, lut.TABLE_F32) == 128 * 16 * 512 * 4
    assert lut.table_bytes(0, 16, 512, lut.TABLE_I8) == 0
    assert lut.table_bytes(4, 16, 8, 7) == 0
    assert lut.table_bytes(3, 16, 9, lut.TABLE_I4) == 3 * 16 * 5  # two entries per byte, rows padded
    assert lut.packed_bytes(64, 16, 64, lut.TABLE_I4) == 64 * 256 * 16  # one int8 per entry, as INT8
    assert lut.packed_bytes(64, 16, 64, lut.TABLE_I8) == 64 * 256 * 16  # M padded to 256
    assert lut.packed_bytes(3, 33, 257, lut.TABLE_I8) == 3 * 3 * 512 * 16  # ceil(33/16) k blocks
    assert lut.packed_bytes(64, 16, 64, lut.TABLE_F32) == 0


def test_status_strings_and_version(lut):
    names = [lut.LIB.lutnn_status_string(i).decode() for i in range(7)]
    assert names == ["LUTNN_OK", "LUTNN_E_NULL", "LUTNN_E_SHAPE", "LUTNN_E_UNSUPPORTED",
                     "LUTNN_E_ALIGN", "LUTNN_E_HIP", "LUTNN_E_UNKNOWN"]
    assert re.fullmatch(r"\d+\.\d+\.\d+\+[0-9a-f]{12}", lut.version())


def _layer(lut, **kw):
    from paper_2302_03213_amd.binding import _CLayer
    f = dict(C=4, K=16, V=4, M=8, table_dtype=lut.TABLE_I8, reserved=0, centroids=0x1000,
             table=0x2000, table_packed=0x3000, scale=0x4000, bias=None)
    f.update(kw)
    return _CLayer(**f)


def _status(lut, code):
    return lut.LIB.lutnn_status_string(code).decode(), lut.LIB.lutnn_last_error().decode()


def test_host_validation_rejects_bad_arguments_before_any_launch(lut):
    """Every call below fails validation on the host; the fake non-NULL addresses are never
    dereferenced and nothing is enqueued."""
    L, vp = lut.LIB, ctypes.c_void_p
    X, Y, IDX = vp(0x10000), vp(0x20000), vp(0x30000)
    ok = _layer(lut)
    cases = [
        (L.lutnn_encode(None, X, 4, 16, IDX, None), "LUTNN_E_NULL"),
        (L.lutnn_encode(ctypes.byref(ok), None, 4, 16, IDX, None), "LUTNN_E_NULL"),
        (L.lutnn_encode(ctypes.byref(ok), X, 4, 16, None, None), "LUTNN_E_NULL"),
        (L.lutnn_encode(ctypes.byref(ok), X, -1, 16, IDX, None), "LUTNN_E_SHAPE"),
        (L.lutnn_encode(ctypes.byref(ok), X, 4, 15, IDX, None), "LUTNN_E_SHAPE"),  # ldx < C*V
        (L.lutnn_encode(ctypes.byref(ok), vp(0x10002), 4, 16, IDX, None), "LUTNN_E_ALIGN"),
        (L.lutnn_encode(ctypes.byref(_layer(lut, K=257)), X, 4, 16, IDX, None), "LUTNN_E_SHAPE"),
        (L.lutnn_encode(ctypes.byref(_layer(lut, C=0)), X, 4, 16, IDX, None), "LUTNN_E_SHAPE"),
        (L.lutnn_encode(ctypes.byref(_layer(lut, table_dtype=9)), X, 4, 16, IDX, None),
         "LUTNN_E_UNSUPPORTED"),
        (L.lutnn_encode(ctypes.byref(_layer(lut, reserved=1)), X, 4, 16, IDX, None),
         "LUTNN_E_SHAPE"),
        (L.lutnn_encode(ctypes.byref(_layer(lut, centroids=None)), X, 4, 16, IDX, None),
         "LUTNN_E_NULL"),
        (L.lutnn_lookup(ctypes.byref(ok), None, 4, Y, 8, lut.VARIANT_LDS, None), "LUTNN_E_NULL"),
        (L.lutnn_lookup(ctypes.byref(ok), IDX, 4, None, 8, lut.VARIANT_LDS, None), "LUTNN_E_NULL"),
        (L.lutnn_lookup(ctypes.byref(ok), IDX, 4, Y, 7, lut.VARIANT_LDS, None), "LUTNN_E_SHAPE"),
        (L.lutnn_lookup(ctypes.byref(ok), IDX, 4, Y, 8, lut.VARIANT_FUSED, None),
         "LUTNN_E_UNSUPPORTED"),
        (L.lutnn_lookup(ctypes.byref(ok), IDX, 4, Y, 8, 17, None), "LUTNN_E_UNSUPPORTED"),
        (L.lutnn_lookup(ctypes.byref(_layer(lut, table_packed=None)), IDX, 4, Y, 8,
                        lut.VARIANT_MFMA, None), "LUTNN_E_NULL"),
        (L.lutnn_lookup(ctypes.byref(_layer(lut, table_packed=0x3008)), IDX, 4, Y, 8,
                        lut.VARIANT_MFMA, None), "LUTNN_E_ALIGN"),
        (L.lutnn_lookup(ctypes.byref(_layer(lut, K=32)), IDX, 4, Y, 8, lut.VARIANT_MFMA, None),
         "LUTNN_E_UNSUPPORTED"),
        (L.lutnn_lookup(ctypes.byref(ok), IDX, 4, Y, 8, lut.VARIANT_SMFMAC, None),
         "LUTNN_E_UNSUPPORTED"),  # C = 4 is not a multiple of 32
        (L.lutnn_lookup(ctypes.byref(_layer(lut, C=64)), vp(0x30004), 4, Y, 8, lut.VARIANT_SMFMAC, None),
         "LUTNN_E_ALIGN"),
        (L.lutnn_lookup(ctypes.byref(_layer(lut, table_dtype=lut.TABLE_F32)), IDX, 4, Y, 8,
                        lut.VARIANT_MFMA, None), "LUTNN_E_UNSUPPORTED"),
        (L.lutnn_lookup(ctypes.byref(_layer(lut, scale=None)), IDX, 4, Y, 8, lut.VARIANT_LDS, None),
         "LUTNN_E_NULL"),
        (L.lutnn_lookup(ctypes.byref(_layer(lut, table=None)), IDX, 4, Y, 8, lut.VARIANT_LDS, None),
         "LUTNN_E_NULL"),
        (L.lutnn_linear(ctypes.byref(ok), X, 4, 16, Y, 8, lut.VARIANT_MFMA, None, None),
         "LUTNN_E_NULL"),  # split variants need the index workspace
        (L.lutnn_linear(ctypes.byref(_layer(lut, V=5)), X, 4, 20, Y, 8, lut.VARIANT_FUSED, None,
                        None), "LUTNN_E_UNSUPPORTED"),
        (L.lutnn_linear(ctypes.byref(ok), X, 4, 16, None, 8, lut.VARIANT_FUSED, None, None),
         "LUTNN_E_NULL"),
        (L.lutnn_build_table(None, X, 8, 4, 16, 4, 8, lut.TABLE_I8, Y, None, IDX, None),
         "LUTNN_E_NULL"),
        (L.lutnn_build_table(X, X, 7, 4, 16, 4, 8, lut.TABLE_I8, Y, None, IDX, None),
         "LUTNN_E_SHAPE"),  # ldw < M
        (L.lutnn_build_table(X, X, 8, 4, 16, 4, 8, lut.TABLE_I8, Y, None, None, None),
         "LUTNN_E_NULL"),  # INT8 needs scale_out
        (L.lutnn_build_table(X, X, 8, 4, 16, 4, 8, 5, Y, None, IDX, None), "LUTNN_E_UNSUPPORTED"),
        (L.lutnn_build_table(X, X, 8, 4, 16, 4, 8, lut.TABLE_I8, Y, vp(0x3004), IDX, None),
         "LUTNN_E_ALIGN"),
    ]
    for i, (code, want) in enumerate(cases):
        name, detail = _status(lut, code)
        assert name == want, "case %d: got %s (%s), wanted %s" % (i, name, detail, want)
        assert detail


def test_empty_batch_is_ok_without_a_gpu(lut):
    L, vp = lut.LIB, ctypes.c_void_p
    ok = _layer(lut)
    assert L.lutnn_encode(ctypes.byref(ok), vp(0x10000), 0, 16, vp(0x30000), None) == 0
    assert L.lutnn_lookup(ctypes.byref(ok), vp(0x30000), 0, vp(0x20000), 8, lut.VARIANT_MFMA, None) == 0
    assert L.lutnn_linear(ctypes.byref(ok), vp(0x10000), 0, 16, vp(0x20000), 8, lut.VARIANT_FUSED,
                          None, None) == 0


def test_conv2d_geometry_and_validation(lut):
    from paper_2302_03213_amd.binding import _CConvGeom
    L, vp = lut.LIB, ctypes.c_void_p
    g = _CConvGeom(64, 56, 56, 3, 3, 1, 1, 1, 1, 0)
    assert L.lutnn_conv2d_rows(ctypes.byref(g), 1) == 56 * 56  # "same" convolution
    assert L.lutnn_conv2d_rows(ctypes.byref(g), 0) == 0
    assert L.lutnn_conv2d_rows(ctypes.byref(_CConvGeom(64, 56, 56, 3, 3, 2, 2, 1, 1, 0)), 4) == 4 * 28 * 28
    assert L.lutnn_conv2d_rows(ctypes.byref(_CConvGeom(8, 7, 9, 1, 1, 1, 1, 0, 0, 0)), 2) == 2 * 63
    assert L.lutnn_conv2d_rows(ctypes.byref(_CConvGeom(8, 7, 9, 3, 5, 2, 3, 0, 1, 0)), 1) == 3 * 3
    assert L.lutnn_conv2d_rows(ctypes.byref(_CConvGeom(8, 2, 2, 3, 3, 1, 1, 0, 0, 0)), 1) == -1  # filter > image
    assert L.lutnn_conv2d_rows(ctypes.byref(_CConvGeom(8, 7, 9, 3, 3, 0, 1, 0, 0, 0)), 1) == -1  # stride 0
    assert L.lutnn_conv2d_rows(ctypes.byref(g), -1) == -1
    assert L.lutnn_conv2d_rows(None, 1) == -1
    ok = _layer(lut, C=64, V=9, M=64)
    X, Y, IDX = vp(0x10000), vp(0x20000), vp(0x30000)
    cases = [
        (L.lutnn_encode_conv2d(ctypes.byref(ok), X, 1, None, IDX, None), "LUTNN_E_NULL"),
        (L.lutnn_encode_conv2d(ctypes.byref(ok), None, 1, ctypes.byref(g), IDX, None), "LUTNN_E_NULL"),
        (L.lutnn_encode_conv2d(ctypes.byref(ok), X, 1, ctypes.byref(g), None, None), "LUTNN_E_NULL"),
        (L.lutnn_encode_conv2d(ctypes.byref(_layer(lut, C=64, V=4)), X, 1, ctypes.byref(g), IDX, None),
         "LUTNN_E_SHAPE"),  # Cin*kh*kw != C*V
        (L.lutnn_encode_conv2d(ctypes.byref(_layer(lut, C=18, V=32)), X, 1, ctypes.byref(g), IDX, None),
         "LUTNN_E_UNSUPPORTED"),  # 64*9 = 18*32, but no convolution encoder for V = 32
        (L.lutnn_encode_conv2d(ctypes.byref(ok), X, 1, ctypes.byref(_CConvGeom(64, 56, 56, 3, 3, 1, 1, 1, 1, 7)),
                               IDX, None), "LUTNN_E_SHAPE"),  # reserved
        (L.lutnn_conv2d(ctypes.byref(ok), X, 1, ctypes.byref(g), Y, 64, lut.VARIANT_FUSED, IDX, None),
         "LUTNN_E_UNSUPPORTED"),
        (L.lutnn_conv2d(ctypes.byref(ok), X, 1, ctypes.byref(g), Y, 64, lut.VARIANT_AUTO, None, None),
         "LUTNN_E_NULL"),  # workspace required
        (L.lutnn_conv2d(ctypes.byref(ok), X, 1, ctypes.byref(g), Y, 63, lut.VARIANT_LDS, IDX, None),
         "LUTNN_E_SHAPE"),  # ldy < M
    ]
    for i, (code, want) in enumerate(cases):
        name, detail = _status(lut, code)
        assert name == want, "case %d: got %s (%s), wanted %s" % (i, name, detail, want)
    assert L.lutnn_encode_conv2d(ctypes.byref(ok), X, 0, ctypes.byref(g), IDX, None) == 0  # empty batch


def test_tree_descriptor_validation(lut):
    """lutnn_encode_tree / lutnn_linear_tree reject bad descriptors on the host."""
    from paper_2302_03213_amd.binding import _CTree
    L, vp = lut.LIB, ctypes.c_void_p
    X, Y, IDX = vp(0x10000), vp(0x20000), vp(0x30000)

    def tree(**kw):
        f = dict(C=4, V=4, levels=4, reserved=0, split_dim=0x5000, threshold=0x6000)
        f.update(kw)
        return _CTree(**f)

    ok, layer = tree(), _layer(lut)
    cases = [
        (L.lutnn_encode_tree(None, X, 8, 16, IDX, None), "LUTNN_E_NULL"),
        (L.lutnn_encode_tree(ctypes.byref(tree(levels=0)), X, 8, 16, IDX, None), "LUTNN_E_SHAPE"),
        (L.lutnn_encode_tree(ctypes.byref(tree(levels=9)), X, 8, 16, IDX, None), "LUTNN_E_SHAPE"),
        (L.lutnn_encode_tree(ctypes.byref(tree(C=0)), X, 8, 16, IDX, None), "LUTNN_E_SHAPE"),
        (L.lutnn_encode_tree(ctypes.byref(tree(reserved=1)), X, 8, 16, IDX, None), "LUTNN_E_SHAPE"),
        (L.lutnn_encode_tree(ctypes.byref(tree(split_dim=None)), X, 8, 16, IDX, None), "LUTNN_E_NULL"),
        (L.lutnn_encode_tree(ctypes.byref(tree(threshold=None)), X, 8, 16, IDX, None), "LUTNN_E_NULL"),
        (L.lutnn_encode_tree(ctypes.byref(ok), None, 8, 16, IDX, None), "LUTNN_E_NULL"),
        (L.lutnn_encode_tree(ctypes.byref(ok), X, 8, 16, None, None), "LUTNN_E_NULL"),
        (L.lutnn_encode_tree(ctypes.byref(ok), X, 8, 15, IDX, None), "LUTNN_E_SHAPE"),  # ldx < D
        (L.lutnn_encode_tree(ctypes.byref(ok), vp(0x10002), 8, 16, IDX, None), "LUTNN_E_ALIGN"),
        (L.lutnn_linear_tree(ctypes.byref(layer), ctypes.byref(tree(levels=3)), X, 8, 16, Y, 8,
                             lut.VARIANT_AUTO, IDX, None), "LUTNN_E_SHAPE"),  # K != 2^levels
        (L.lutnn_linear_tree(ctypes.byref(layer), ctypes.byref(tree(V=2)), X, 8, 16, Y, 8,
                             lut.VARIANT_AUTO, IDX, None), "LUTNN_E_SHAPE"),
        (L.lutnn_linear_tree(ctypes.byref(layer), ctypes.byref(ok), X, 8, 16, Y, 8, lut.VARIANT_LDS,
                             None, None), "LUTNN_E_NULL"),  # two launches need the workspace
        (L.lutnn_linear_tree(ctypes.byref(_layer(lut, M=6)), ctypes.byref(ok), X, 8, 16, Y, 8,
                             lut.VARIANT_FUSED, IDX, None), "LUTNN_E_UNSUPPORTED"),  # M % 4 != 0
        (L.lutnn_linear_tree(ctypes.byref(_layer(lut, table_dtype=lut.TABLE_I4)), ctypes.byref(ok), X, 8, 16,
                             Y, 8, lut.VARIANT_FUSED, IDX, None), "LUTNN_E_UNSUPPORTED"),  # INT4 storage
        (L.lutnn_linear_tree(ctypes.byref(layer), ctypes.byref(ok), X, 8, 16, Y, 7, lut.VARIANT_FUSED,
                             None, None), "LUTNN_E_SHAPE"),  # one launch: ldy < M
        (L.lutnn_linear_tree(ctypes.byref(layer), ctypes.byref(ok), X, 8, 16, Y, 7, lut.VARIANT_LDS,
                             IDX, None), "LUTNN_E_SHAPE"),  # ldy < M
    ]
    for i, (code, want) in enumerate(cases):
        name, detail = _status(lut, code)
        assert name == want, "case %d: got %s (%s), wanted %s" % (i, name, detail, want)
    assert L.lutnn_encode_tree(ctypes.byref(ok), None, 0, 16, None, None) == 0  # empty batch
    assert L.lutnn_linear_tree(ctypes.byref(layer), ctypes.byref(ok), None, 0, 16, None, 8,
                               lut.VARIANT_AUTO, None, None) == 0


def test_sixteen_bit_index_entry_points_validate_on_the_host(lut):
    """lutnn_encode_tree16 / lutnn_lookup16 / lutnn_linear_tree16: levels up to 12, K up to 4096."""
    from paper_2302_03213_amd.binding import _CTree
    L, vp = lut.LIB, ctypes.c_void_p
    X, Y, IDX = vp(0x10000), vp(0x20000), vp(0x30000)

    def tree(**kw):
        f = dict(C=4, V=4, levels=12, reserved=0, split_dim=0x5000, threshold=0x6000)
        f.update(kw)
        return _CTree(**f)

    deep = _layer(lut, K=4096)
    cases = [
        (L.lutnn_encode_tree16(None, X, 8, 16, IDX, None), "LUTNN_E_NULL"),
        (L.lutnn_encode_tree16(ctypes.byref(tree(levels=13)), X, 8, 16, IDX, None), "LUTNN_E_SHAPE"),
        (L.lutnn_encode_tree16(ctypes.byref(tree(levels=0)), X, 8, 16, IDX, None), "LUTNN_E_SHAPE"),
        (L.lutnn_encode_tree16(ctypes.byref(tree()), X, 8, 15, IDX, None), "LUTNN_E_SHAPE"),
        (L.lutnn_encode_tree16(ctypes.byref(tree()), X, 8, 16, None, None), "LUTNN_E_NULL"),
        (L.lutnn_encode_tree16(ctypes.byref(tree()), X, 8, 16, vp(0x30001), None), "LUTNN_E_ALIGN"),
        (L.lutnn_lookup16(None, IDX, 8, Y, 8, None), "LUTNN_E_NULL"),
        (L.lutnn_lookup16(ctypes.byref(_layer(lut, K=4097)), IDX, 8, Y, 8, None), "LUTNN_E_SHAPE"),
        (L.lutnn_lookup16(ctypes.byref(_layer(lut, K=4096, table_dtype=lut.TABLE_I4)), IDX, 8, Y, 8, None),
         "LUTNN_E_UNSUPPORTED"),
        (L.lutnn_lookup16(ctypes.byref(deep), None, 8, Y, 8, None), "LUTNN_E_NULL"),
        (L.lutnn_lookup16(ctypes.byref(deep), IDX, 8, None, 8, None), "LUTNN_E_NULL"),
        (L.lutnn_lookup16(ctypes.byref(deep), IDX, 8, Y, 7, None), "LUTNN_E_SHAPE"),
        (L.lutnn_lookup16(ctypes.byref(_layer(lut, K=4096, scale=None)), IDX, 8, Y, 8, None), "LUTNN_E_NULL"),
        (L.lutnn_lookup16(ctypes.byref(_layer(lut, K=4096, table=None)), IDX, 8, Y, 8, None), "LUTNN_E_NULL"),
        (L.lutnn_lookup16(ctypes.byref(deep), vp(0x30001), 8, Y, 8, None), "LUTNN_E_ALIGN"),
        (L.lutnn_linear_tree16(ctypes.byref(deep), ctypes.byref(tree(levels=11)), X, 8, 16, Y, 8, IDX, None),
         "LUTNN_E_SHAPE"),  # K != 2^levels
        (L.lutnn_linear_tree16(ctypes.byref(deep), ctypes.byref(tree()), X, 8, 16, Y, 8, None, None),
         "LUTNN_E_NULL"),
        (L.lutnn_linear_tree16(ctypes.byref(deep), ctypes.byref(tree()), X, 8, 16, Y, 7, IDX, None),
         "LUTNN_E_SHAPE"),
        # the 8-bit entry points still stop at 8 levels / 256 centroids, and say where to go
        (L.lutnn_encode_tree(ctypes.byref(tree()), X, 8, 16, IDX, None), "LUTNN_E_SHAPE"),
        (L.lutnn_lookup(ctypes.byref(deep), IDX, 8, Y, 8, lut.VARIANT_AUTO, None), "LUTNN_E_SHAPE"),
    ]
    for i, (code, want) in enumerate(cases):
        name, detail = _status(lut, code)
        assert name == want, "case %d: got %s (%s), wanted %s" % (i, name, detail, want)
    assert "16" in _status(lut, L.lutnn_lookup(ctypes.byref(deep), IDX, 8, Y, 8, lut.VARIANT_AUTO, None))[1]
    assert L.lutnn_encode_tree16(ctypes.byref(tree()), None, 0, 16, None, None) == 0  # empty batch
    assert L.lutnn_lookup16(ctypes.byref(deep), None, 0, None, 8, None) == 0
    # tables of up to 4096 rows per codebook are built without the packed copy
    P, W, T, PK, S = (vp(0x10000 * i) for i in range(1, 6))
    name, _ = _status(lut, L.lutnn_build_table(P, W, 8, 4, 4096, 4, 8, lut.TABLE_I8, T, PK, S, None))
    assert name == "LUTNN_E_UNSUPPORTED"
    name, _ = _status(lut, L.lutnn_build_table(P, W, 8, 4, 4097, 4, 8, lut.TABLE_I8, T, None, S, None))
    assert name == "LUTNN_E_SHAPE"


def test_softpq_backward_validation_and_workspace_query(lut):
    L, vp = lut.LIB, ctypes.c_void_p
    X, Z, DP, DX, DT, WS = (vp(0x10000 * i) for i in range(1, 7))
    # config 5: 64 column tiles of 16 codebooks, 32 chunks of 8 row tiles; one 64-float group per
    # codebook and chunk, one temperature partial per workgroup
    assert lut.softpq_workspace_bytes(1024, 16, 4, 16384) == (32 * 1024 * 64 + 32 * 64) * 4
    assert lut.softpq_workspace_bytes(1024, 5, 4, 16384) == 0      # K not supported
    assert lut.softpq_workspace_bytes(1024, 16, 5, 16384) == 0     # V not supported
    assert lut.softpq_workspace_bytes(1024, 16, 4, 0) == 0
    assert lut.softpq_workspace_bytes(4, 16, 9, 64) == (1 * 4 * 3 * 64 + 1) * 4  # ceil(9/4) = 3 groups
    ok = _layer(lut)
    f = ctypes.c_float
    big = 1 << 20
    cases = [
        (L.lutnn_softpq_backward(None, f(1.0), X, 8, 16, Z, 16, DP, DX, 16, DT, WS, big, None), "LUTNN_E_NULL"),
        (L.lutnn_softpq_backward(ctypes.byref(ok), f(0.0), X, 8, 16, Z, 16, DP, DX, 16, DT, WS, big, None),
         "LUTNN_E_SHAPE"),
        (L.lutnn_softpq_backward(ctypes.byref(ok), f(float("nan")), X, 8, 16, Z, 16, DP, DX, 16, DT, WS, big,
                                 None), "LUTNN_E_SHAPE"),
        (L.lutnn_softpq_backward(ctypes.byref(_layer(lut, K=5)), f(1.0), X, 8, 16, Z, 16, DP, DX, 16, DT, WS,
                                 big, None), "LUTNN_E_UNSUPPORTED"),
        (L.lutnn_softpq_backward(ctypes.byref(_layer(lut, V=5)), f(1.0), X, 8, 20, Z, 20, DP, DX, 20, DT, WS,
                                 big, None), "LUTNN_E_UNSUPPORTED"),
        (L.lutnn_softpq_backward(ctypes.byref(ok), f(1.0), X, 8, 16, Z, 16, None, DX, 16, DT, WS, big, None),
         "LUTNN_E_NULL"),
        (L.lutnn_softpq_backward(ctypes.byref(ok), f(1.0), None, 8, 16, Z, 16, DP, DX, 16, DT, WS, big, None),
         "LUTNN_E_NULL"),
        (L.lutnn_softpq_backward(ctypes.byref(ok), f(1.0), X, 8, 16, None, 16, DP, DX, 16, DT, WS, big, None),
         "LUTNN_E_NULL"),
        (L.lutnn_softpq_backward(ctypes.byref(ok), f(1.0), X, 8, 15, Z, 16, DP, DX, 16, DT, WS, big, None),
         "LUTNN_E_SHAPE"),
        (L.lutnn_softpq_backward(ctypes.byref(ok), f(1.0), X, 8, 16, Z, 15, DP, DX, 16, DT, WS, big, None),
         "LUTNN_E_SHAPE"),
        (L.lutnn_softpq_backward(ctypes.byref(ok), f(1.0), X, 8, 16, Z, 16, DP, DX, 15, DT, WS, big, None),
         "LUTNN_E_SHAPE"),
        (L.lutnn_softpq_backward(ctypes.byref(ok), f(1.0), X, 8, 16, Z, 16, DP, DX, 16, DT, None, big, None),
         "LUTNN_E_NULL"),
        (L.lutnn_softpq_backward(ctypes.byref(ok), f(1.0), X, 8, 16, Z, 16, DP, DX, 16, DT, WS, 16, None),
         "LUTNN_E_SHAPE"),  # workspace too small
        (L.lutnn_softpq_backward(ctypes.byref(ok), f(1.0), X, 8, 16, vp(0x20002), 16, DP, DX, 16, DT, WS, big,
                                 None), "LUTNN_E_ALIGN"),
    ]
    for i, (code, want) in enumerate(cases):
        name, detail = _status(lut, code)
        assert name == want, "case %d: got %s (%s), wanted %s" % (i, name, detail, want)


def test_static_scratch_form_refuses_oversize_shapes_on_the_host(lut):
    """lutnn_softpq_backward_static checks the scratch need against its static array before it
    touches a device: the refusal needs no GPU."""
    L, vp, f = lut.LIB, ctypes.c_void_p, ctypes.c_float
    X, Z, DP, DX, DT = (vp(0x10000 * i) for i in range(1, 6))
    C, K, V, N = 131072, 16, 4, 8
    assert lut.softpq_workspace_bytes(C, K, V, N) > 32 << 20
    code = L.lutnn_softpq_backward_static(ctypes.byref(_layer(lut, C=C)), f(1.0), X, N, C * V, Z, C * V, DP, DX,
                                          C * V, DT, None)
    name, detail = _status(lut, code)
    assert name == "LUTNN_E_SHAPE" and "static buffer" in detail, (name, detail)
    assert L.lutnn_softpq_backward_static(None, f(1.0), X, 8, 16, Z, 16, DP, DX, 16, DT, None) == 1  # E_NULL


def test_tuning_switches(lut):
    for name, good, bad in (("LUTNN_FUSED_KERNEL", ("small", "tile"), "both"),
                            ("LUTNN_SMFMAC_SPLIT", ("0", "1"), "2"),
                            ("LUTNN_SMFMAC_TILE_ROWS", ("128", "256", "384", "512"), "200"),
                            ("LUTNN_SMFMAC_ROW_GROUP", ("0", "8", "64"), "65"),
                            ("LUTNN_SMFMAC_TILE_COLS", ("96", "128"), "64")):
        for v in good:
            lut.set_tunable(name, v)
        with pytest.raises(lut.LutnnError) as e:
            lut.set_tunable(name, bad)
        assert e.value.name == "LUTNN_E_SHAPE"
        lut.set_tunable(name, None)
        lut.set_tunable(name, "")
    with pytest.raises(lut.LutnnError) as e:
        lut.set_tunable("LUTNN_NO_SUCH_SWITCH", "1")
    assert e.value.name == "LUTNN_E_UNSUPPORTED"
    assert lut.LIB.lutnn_set_tunable(None, b"1") == 1
    with lut.tunables(LUTNN_SMFMAC_SPLIT=1):
        pass


def test_version_carries_the_hash_of_the_sources(lut):
    from paper_2302_03213_amd import build
    assert lut.version().endswith("+" + build.source_hash())


def test_auto_variant_rule(lut):
    """AUTO is a pure function of the descriptor, N and the address of idx."""
    L, vp = lut.LIB, ctypes.c_void_p
    big = _layer(lut, C=1024, M=4096)
    assert L.lutnn_auto_variant(ctypes.byref(big), vp(0x30000), 16384) == lut.VARIANT_SMFMAC
    assert L.lutnn_auto_variant(ctypes.byref(big), vp(0x30004), 16384) == lut.VARIANT_MFMA  # idx alignment
    assert L.lutnn_auto_variant(ctypes.byref(big), vp(0x30000), 200) == lut.VARIANT_SMFMAC
    assert L.lutnn_auto_variant(ctypes.byref(big), vp(0x30000), 1) == lut.VARIANT_LDS   # split gather: a few rows
    assert L.lutnn_auto_variant(ctypes.byref(big), vp(0x30000), 32) == lut.VARIANT_LDS
    assert L.lutnn_auto_variant(ctypes.byref(big), vp(0x30000), 33) == lut.VARIANT_SMFMAC
    odd = _layer(lut, C=1000, M=4096)
    assert L.lutnn_auto_variant(ctypes.byref(odd), vp(0x30000), 16384) == lut.VARIANT_MFMA  # C % 32 != 0
    small = _layer(lut, C=64, M=64)  # few table entries: rows gathered straight from L2
    assert L.lutnn_auto_variant(ctypes.byref(small), vp(0x30000), 3136) == lut.VARIANT_LDS
    assert L.lutnn_auto_variant(ctypes.byref(small), vp(0x30000), 1 << 20) == lut.VARIANT_SMFMAC
    # priced against the launch it would replace: a BERT attention-output shape takes the gather up
    # to a few hundred rows, and where only the dense kernel can run (C % 32 != 0) for longer
    attn = _layer(lut, C=384, M=768)
    assert L.lutnn_auto_variant(ctypes.byref(attn), vp(0x30000), 128) == lut.VARIANT_LDS
    assert L.lutnn_auto_variant(ctypes.byref(attn), vp(0x30000), 512) == lut.VARIANT_SMFMAC
    v16 = _layer(lut, C=48, M=3072)
    assert L.lutnn_auto_variant(ctypes.byref(v16), vp(0x30000), 512) == lut.VARIANT_LDS
    assert L.lutnn_auto_variant(ctypes.byref(v16), vp(0x30000), 2048) == lut.VARIANT_MFMA
    f32 = _layer(lut, table_dtype=lut.TABLE_F32, C=128, M=512)
    assert L.lutnn_auto_variant(ctypes.byref(f32), vp(0x30000), 256) == lut.VARIANT_LDS
    wide_k = _layer(lut, K=32, C=64, M=4096)
    assert L.lutnn_auto_variant(ctypes.byref(wide_k), vp(0x30000), 1 << 16) == lut.VARIANT_LDS
    assert L.lutnn_auto_variant(None, vp(0x30000), 16) == -1


def test_linear_auto_variant_rule(lut):
    """What lutnn_linear runs for AUTO: one launch for small problems (the lookup would be the gather
    and the centroids a workgroup re-reads are few), else the lookup's own rule; pure host function."""
    L, vp = lut.LIB, ctypes.c_void_p
    ws = vp(0x30000)
    qkv = _layer(lut, C=384, V=2, M=2304)  # BERT QKV at V = 2
    assert L.lutnn_linear_auto_variant(ctypes.byref(qkv), ws, 1) == lut.VARIANT_FUSED
    assert L.lutnn_linear_auto_variant(ctypes.byref(qkv), ws, 16) == lut.VARIANT_FUSED
    assert L.lutnn_linear_auto_variant(ctypes.byref(qkv), ws, 4096) == lut.VARIANT_SMFMAC
    wide = _layer(lut, C=1024, V=4, M=4096)  # 256 KiB of centroids per workgroup: two launches
    assert L.lutnn_linear_auto_variant(ctypes.byref(wide), ws, 1) == lut.VARIANT_LDS
    assert L.lutnn_linear_auto_variant(ctypes.byref(wide), ws, 16384) == lut.VARIANT_SMFMAC
    assert L.lutnn_linear_auto_variant(ctypes.byref(wide), None, 16384) == lut.VARIANT_FUSED  # no workspace
    fc_small = _layer(lut, table_dtype=lut.TABLE_F32, C=128, V=4, M=512)
    assert L.lutnn_linear_auto_variant(ctypes.byref(fc_small), ws, 256) == lut.VARIANT_FUSED
    assert L.lutnn_linear_auto_variant(ctypes.byref(fc_small), ws, 1 << 16) == lut.VARIANT_LDS
    odd_m = _layer(lut, C=64, V=4, M=37)  # M % 4 != 0: the one-launch form cannot run
    assert L.lutnn_linear_auto_variant(ctypes.byref(odd_m), ws, 8) != lut.VARIANT_FUSED
    int4 = _layer(lut, table_dtype=lut.TABLE_I4, C=64, V=4, M=512)
    assert L.lutnn_linear_auto_variant(ctypes.byref(int4), ws, 8) != lut.VARIANT_FUSED
    assert L.lutnn_linear_auto_variant(None, ws, 16) == -1


def test_cost_model_formulas(lut):
    c = lut.cost
    # Table 1 with the paper's own example: FLOPs reduction M / (K + M/V) (Sec. 6.2)
    N, D, M, K, V = 3136, 576, 64, 16, 9
    assert c.lut_flops(N, D, M, K, V) == N * D * K + N * M * (D // V)
    assert abs(c.mm_flops(N, D, M) / c.lut_flops(N, D, M, K, V) - c.flops_reduction(M, K, V)) < 1e-9
    # "M = 128, 256 or 512 ... FLOPs can be reduced by 4x when K = 8" (Sec. 4): K-dominated limit
    assert abs(c.flops_reduction(768, 16, 32) - 768 / (16 + 24)) < 1e-12
    assert c.lut_size_bytes(D, M, K, V) == 4 * D * K + D * M * K // V
    assert c.mm_size_bytes(D, M) == 4 * D * M
    assert c.equivalent_flops(16384, 4096, 4096) == 2 * 16384 * 4096 * 4096
    assert c.lookup_mfma_ops(16384, 1024, 4096) == 2 * 16384 * 16384 * 4096


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asking for more exits with a message before touching a GPU."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True)
    assert r.returncode == 2 and "ONE GPU" in r.stderr
    env = dict(os.environ, WORLD_SIZE="4")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True, env=env)
    assert r.returncode == 2 and "ONE GPU" in r.stderr


def test_stream_probe_validates_on_the_host(lut):
    L = lut.LIB
    assert L.lutnn_probe_smfmac_stream(1, 10, None, 1 << 20, None) == 1  # E_NULL
    fake = ctypes.c_void_p(0x1000)
    for operands, iterations, nbytes in ((3, 10, 1 << 20), (-1, 10, 1 << 20), (1, -1, 1 << 20),
                                         (1, (1 << 24) + 1, 1 << 20), (1, 10, 16)):
        code = L.lutnn_probe_smfmac_stream(operands, iterations, fake, nbytes, None)
        name, detail = _status(lut, code)
        assert name == "LUTNN_E_SHAPE", (operands, iterations, nbytes, name, detail)

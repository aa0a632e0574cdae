"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, answers the size queries, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "sbn.h")
PROBE_HEADER = os.path.join(ROOT, "include", "sbn_probe.h")


@pytest.fixture(scope="module")
def sbn():
    import paper_2603_05168_amd as m
    return m


def declared_functions(header=HEADER):
    text = open(header).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sbn_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_boundary():
    names = declared_functions()
    for must in ("sbn_quantize_mask_pack", "sbn_sparse_ternary_linear", "sbn_sparse_ternary_linear_backward",
                 "sbn_sparse_ternary_linear_backward_grouped",
                 "sbn_packed_bytes", "sbn_workspace_bytes", "sbn_unpack", "sbn_last_error"):
        assert must in names


def test_library_exports_every_declared_symbol(sbn):
    lib = ctypes.CDLL(sbn.lib_path())
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} is declared in include/sbn.h but not exported"
    for name in declared_functions():
        assert hasattr(sbn, name), f"{name} has no Python binding of the same name"


def test_every_header_is_covered_and_the_probe_library_exports_its_symbol():
    # include/ holds exactly the layer's header and the benchmark probes' header, each with a library of its own
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["sbn.h", "sbn_probe.h"]
    from paper_2603_05168_amd import probe
    lib = ctypes.CDLL(probe.lib_path())
    names = declared_functions(PROBE_HEADER)
    assert names == ["sbn_ceiling_probe"]
    for name in names:
        assert hasattr(lib, name) and hasattr(probe, name)
    assert "sbn_ceiling_probe" not in declared_functions()       # measurement support stays out of the layer's boundary


def test_spin_limit_hook_is_callable_without_a_gpu(sbn):
    sbn.sbn_test_set_spin_limits(0, -1)
    sbn.sbn_test_set_spin_limits()


def test_packed_bytes(sbn):
    assert sbn.sbn_packed_bytes(6912, 2560, 2, 4) == 6912 * 2560 // 4
    assert sbn.sbn_packed_bytes(6912, 2560, 1, 4) == 6912 * 2560 // 8
    assert sbn.sbn_packed_bytes(2560, 6912, 2, 8) == 2560 * 6912 * 5 // 32
    assert sbn.sbn_packed_bytes(3, 8, 2, 4) == 3 * 32            # one zero-padded chunk per row
    assert sbn.sbn_packed_bytes(16, 256, 8, 8) == 16 * 256 // 4  # dense ternary: 2 bits per weight, no indices


def test_packed_bytes_matches_oracle_layout(sbn):
    import oracle
    for N, M in ((2, 4), (1, 4), (2, 8), (6, 8), (4, 4), (1, 2), (7, 8)):
        for d_in in (8, 128, 136, 2560):
            assert sbn.sbn_packed_bytes(24, d_in, N, M) == oracle.packed_bytes(24, d_in, N, M)


@pytest.mark.parametrize("args", [(0, 256, 2, 4), (16, 0, 2, 4), (16, 130, 2, 4), (16, 256, 0, 4), (16, 256, 5, 4),
                                  (16, 256, 2, 3), (16, 256, 2, 16)])
def test_bad_shapes_are_einval(sbn, args):
    with pytest.raises(sbn.SbnError) as e:
        sbn.sbn_packed_bytes(*args)
    assert e.value.status == sbn.SBN_EINVAL


def test_workspace_queries(sbn):
    for op in (sbn.SBN_OP_QUANTIZE_MASK_PACK, sbn.SBN_OP_LINEAR, sbn.SBN_OP_BACKWARD, sbn.SBN_OP_MASK_FLIPS):
        assert sbn.sbn_workspace_bytes(op, 16, 256, 256, 2, 4) > 0
    with pytest.raises(sbn.SbnError):
        sbn.sbn_workspace_bytes(7, 16, 256, 256, 2, 4)
    with pytest.raises(sbn.SbnError):
        sbn.sbn_workspace_bytes(sbn.SBN_OP_LINEAR, 0, 256, 256, 2, 4)


def test_argument_errors_come_before_any_launch(sbn):
    """Null and misaligned pointers, short workspaces and unsupported requests return their status
    on the host; no GPU is present here, so reaching a launch would fail differently."""
    lib = ctypes.CDLL(sbn.lib_path())
    lib.sbn_quantize_mask_pack.restype = ctypes.c_int
    lib.sbn_sparse_ternary_linear.restype = ctypes.c_int
    lib.sbn_sparse_ternary_linear_backward.restype = ctypes.c_int
    vp, i64, ci, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t
    A = 0x10000  # fake, aligned, never dereferenced on the host
    # null packed
    assert lib.sbn_quantize_mask_pack(vp(A), ci(1), i64(16), i64(256), i64(256), ci(2), ci(4), vp(0), vp(A), vp(A),
                                      sz(1 << 20), vp(0)) == sbn.SBN_EINVAL
    # ld_w < d_in
    assert lib.sbn_quantize_mask_pack(vp(A), ci(1), i64(16), i64(256), i64(128), ci(2), ci(4), vp(A), vp(A), vp(A),
                                      sz(1 << 20), vp(0)) == sbn.SBN_EINVAL
    # misaligned packed
    assert lib.sbn_quantize_mask_pack(vp(A), ci(1), i64(16), i64(256), i64(256), ci(2), ci(4), vp(A + 4), vp(A), vp(A),
                                      sz(1 << 20), vp(0)) == sbn.SBN_EALIGN
    # workspace too small
    assert lib.sbn_quantize_mask_pack(vp(A), ci(1), i64(16), i64(256), i64(256), ci(2), ci(4), vp(A), vp(A), vp(A),
                                      sz(8), vp(0)) == sbn.SBN_ESIZE
    lin = lambda **kw: lib.sbn_sparse_ternary_linear(  # noqa: E731
        vp(kw.get("X", A)), i64(kw.get("tokens", 8)), i64(kw.get("d_in", 256)), i64(256), ci(kw.get("N", 2)),
        ci(kw.get("M", 4)), vp(A), vp(A), vp(0), vp(kw.get("Y", A)), vp(0), vp(0), vp(0), ci(kw.get("path", 0)), vp(A),
        sz(kw.get("ws", 1 << 24)), vp(0))
    assert lin(Y=0) == sbn.SBN_EINVAL
    assert lin(X=0) == sbn.SBN_EINVAL                       # no X and no pre-quantized inputs
    assert lin(X=A + 2) == sbn.SBN_EALIGN
    assert lin(path=9) == sbn.SBN_EINVAL
    assert lin(ws=16) == sbn.SBN_ESIZE
    assert lin(tokens=64, path=sbn.SBN_PATH_GEMV) == sbn.SBN_EUNSUPPORTED  # decode kernel takes <= 16 tokens
    assert lin(d_in=200, path=sbn.SBN_PATH_SMFMAC) == sbn.SBN_EUNSUPPORTED
    # backward: nothing requested
    assert lib.sbn_sparse_ternary_linear_backward(vp(A), i64(8), i64(256), i64(256), ci(2), ci(4), vp(A), vp(A), vp(A),
                                                  vp(A), vp(0), vp(0), ci(0), vp(A), sz(1 << 24), vp(0)) == sbn.SBN_EINVAL
    # backward: unknown flag bit
    assert lib.sbn_sparse_ternary_linear_backward(vp(A), i64(8), i64(256), i64(256), ci(2), ci(4), vp(A), vp(A), vp(A),
                                                  vp(A), vp(A), vp(A), ci(4), vp(A), sz(1 << 24), vp(0)) == sbn.SBN_EINVAL
    assert lin(d_in=200, path=sbn.SBN_PATH_DENSE_MFMA) == sbn.SBN_EUNSUPPORTED   # dense MFMA rows are multiples of 64
    # grouped backward: count out of range, null array, a layer that asks for nothing, short workspace, misaligned dY
    lib.sbn_sparse_ternary_linear_backward_grouped.restype = ctypes.c_int
    def bwd_grouped(count=2, dy=(A, A), dx=(A, A), dw=(A, A), ws=1 << 26, arrays_ok=True, flags=0):
        P = lambda vals: (vp * 2)(*[vp(v) if v else None for v in vals])   # noqa: E731
        I = lambda v: (i64 * 2)(v, v)                                       # noqa: E731
        return lib.sbn_sparse_ternary_linear_backward_grouped(
            ci(count), P(dy), I(8), I(256), I(256), ci(2), ci(4), P((A, A)), P((A, A)), P((A, A)), P((A, A)),
            P(dx) if arrays_ok else None, P(dw), ci(flags), vp(A), sz(ws), vp(0))
    assert bwd_grouped(count=0) == sbn.SBN_EINVAL
    assert bwd_grouped(count=9) == sbn.SBN_EINVAL
    assert bwd_grouped(arrays_ok=False) == sbn.SBN_EINVAL
    assert bwd_grouped(dx=(A, 0), dw=(A, 0)) == sbn.SBN_EINVAL
    assert bwd_grouped(flags=8) == sbn.SBN_EINVAL
    assert bwd_grouped(dy=(A, A + 2)) == sbn.SBN_EALIGN
    assert bwd_grouped(ws=1 << 12) == sbn.SBN_ESIZE
    # in-place pack with flip counts: null counters, misaligned counters, fp32 weights, a pattern and a row length
    # outside what the flip-counting kernels cover
    lib.sbn_quantize_mask_pack_flips_batched.restype = ctypes.c_int
    one_p, one_i = (vp * 1), (i64 * 1)

    def pflips(wdt=1, d_out=16, d_in=256, N=2, M=4, fl=A):
        return lib.sbn_quantize_mask_pack_flips_batched(ci(1), one_p(A), ci(wdt), one_i(d_out), one_i(d_in), ci(N), ci(M), one_p(A),
                                                        one_p(A), vp(fl), vp(A), sz(1 << 20), vp(0))
    assert pflips(fl=0) == sbn.SBN_EINVAL
    assert pflips(fl=A + 4) == sbn.SBN_EALIGN
    assert pflips(wdt=0) == sbn.SBN_EUNSUPPORTED
    assert pflips(N=6, M=8) == sbn.SBN_EUNSUPPORTED
    assert pflips(d_in=200) == sbn.SBN_EUNSUPPORTED
    # mask flips: null input, misaligned count, short workspace
    lib.sbn_mask_flips.restype = ctypes.c_int
    flips = lambda **kw: lib.sbn_mask_flips(  # noqa: E731
        vp(kw.get("a", A)), vp(A), i64(64), i64(256), ci(2), ci(4), vp(kw.get("out", A)), vp(A), sz(kw.get("ws", 1 << 16)), vp(0))
    assert flips(a=0) == sbn.SBN_EINVAL
    assert flips(out=A + 4) == sbn.SBN_EALIGN
    assert flips(ws=8) == sbn.SBN_ESIZE
    # conversion of packed forms: null, target that cannot hold the pattern, same form, ragged rows
    lib.sbn_convert_packed.restype = ctypes.c_int
    conv = lambda **kw: lib.sbn_convert_packed(  # noqa: E731
        vp(kw.get("src", A)), i64(64), i64(kw.get("d_in", 256)), ci(kw.get("N", 6)), ci(kw.get("M", 8)),
        ci(kw.get("to_N", 8)), ci(kw.get("to_M", 8)), vp(kw.get("out", A)), vp(0))
    assert conv(src=0) == sbn.SBN_EINVAL
    assert conv(out=A + 4) == sbn.SBN_EALIGN
    assert conv(to_N=2, to_M=4) == sbn.SBN_EUNSUPPORTED          # 6:8 keeps more than two of an aligned four
    assert conv(N=2, M=4, to_N=2, to_M=4) == sbn.SBN_EUNSUPPORTED  # already in that form
    assert conv(to_N=1, to_M=4) == sbn.SBN_EUNSUPPORTED          # only 2:4 and N = M are decode forms
    assert conv(d_in=200) == sbn.SBN_EUNSUPPORTED                # whole 128-weight chunks only
    assert conv(to_N=9, to_M=8) == sbn.SBN_EINVAL
    # ceiling probes (their own library): unknown kind, missing host output, buffer too small to stream
    from paper_2603_05168_amd import probe
    plib = ctypes.CDLL(probe.lib_path())
    plib.sbn_ceiling_probe.restype = ctypes.c_int
    work = ctypes.c_double(0.0)
    assert plib.sbn_ceiling_probe(ci(7), vp(A), sz(1 << 22), ci(1), ctypes.byref(work), vp(0)) == -1
    assert plib.sbn_ceiling_probe(ci(0), vp(A), sz(1 << 22), ci(1), vp(0), vp(0)) == -1
    assert plib.sbn_ceiling_probe(ci(0), vp(A), sz(1 << 22), ci(0), ctypes.byref(work), vp(0)) == -1
    assert plib.sbn_ceiling_probe(ci(3), vp(A), sz(4096), ci(1), ctypes.byref(work), vp(0)) == -1
    assert plib.sbn_ceiling_probe(ci(3), vp(A + 16), sz(1 << 22), ci(1), ctypes.byref(work), vp(0)) == -4
    assert sbn.sbn_last_error() == ""

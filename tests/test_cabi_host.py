"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol include/moss.h declares, and rejects bad arguments before launching anything."""
import ctypes as C

import pytest

import paper_2511_05811_amd as moss


@pytest.fixture(scope="module")
def L():
    return moss.load()


def test_every_declared_symbol_is_exported(L):
    names = moss.exported_symbols()
    assert {"moss_quant_act_2level", "moss_weight_autoscale_cast", "moss_gemm_fp8_mx"} <= set(names)
    for n in names:
        assert hasattr(L, n), n


def test_struct_layouts_match_header():
    assert C.sizeof(moss.WScaleState) == 48
    assert moss.WScaleState.cum_lr.offset == 8 and moss.WScaleState.overflow_count.offset == 36
    assert moss.WScaleState.flags.offset == 44
    assert C.sizeof(moss.AdamWArgs) == 56 and moss.AdamWArgs.step.offset == 48


def test_status_strings(L):
    assert L.moss_status_string(0) == b"ok"
    for code in range(1, 7):
        assert len(L.moss_status_string(code)) > 3
    assert L.moss_status_string(99) == b"unknown status"


def test_workspace_sizes(L):
    assert L.moss_quant_workspace_bytes(8192, 4096, 3) >= 4
    assert L.moss_weight_workspace_bytes(4096, 11008) >= 8
    assert L.moss_gemm_workspace_bytes(8192, 4096, 4096) == 0


FAKE = 0x10000  # 16-byte aligned, never dereferenced: validation fails first


def test_quant_argument_validation(L):
    q = lambda x, rows, cols, ld, flags, qr=FAKE, er=FAKE, qc=FAKE, ec=FAKE, s=FAKE, ws=FAKE, wsb=1 << 20: \
        L.moss_quant_act_2level(x, rows, cols, ld, flags, qr, er, qc, ec, s, ws, wsb, None)
    assert q(None, 32, 32, 32, 1) == 1                    # NULL input
    assert q(FAKE, 32, 32, 32, 1, qr=None) == 1           # NULL output that the flags ask for
    assert q(FAKE, 32, 32, 32, 2, qc=None) == 1
    assert q(FAKE, 32, 48, 48, 1) == 2                    # cols not a multiple of 32
    assert q(FAKE, 48, 32, 32, 2) == 2                    # rows not a multiple of 32 with column groups
    assert q(FAKE, 0, 32, 32, 1) == 2
    assert q(FAKE, 32, 64, 32, 1) == 2                    # ld < cols
    assert q(FAKE + 2, 32, 32, 32, 1) == 3                # misaligned input
    assert q(FAKE, 32, 32, 36, 1) == 3                    # ld not a multiple of 8
    assert q(FAKE, 32, 32, 32, 1, ws=None) == 4           # no workspace
    assert q(FAKE, 32, 32, 32, 1, wsb=16) == 4            # workspace too small
    assert q(FAKE, 32, 32, 32, 0) == 5                    # no output requested
    assert q(FAKE, 32, 32, 32, 64) == 5                   # unknown flag
    assert q(FAKE, 32, 48, 48, 1 | 8) == 2                # MOSS_WS_KEPT is a known flag: the shape error comes first


def test_noalloc_argument_validation(L):
    q = lambda x, rows, cols, ld, flags, qr=FAKE, er=FAKE, qc=FAKE, ec=FAKE, s=FAKE: \
        L.moss_quant_act_2level_noalloc(x, rows, cols, ld, flags, qr, er, qc, ec, s, None)
    assert q(FAKE, 32, 48, 48, 1) == 2
    assert q(FAKE, 32, 32, 32, 0) == 5
    assert q(FAKE, 32, 32, 32, 1, er=FAKE + 1) == 3       # exponent bytes leave as 4-byte words


def test_producer_argument_validation(L):
    q = lambda x, rows, cols, ld, flags, mx=FAKE, qr=FAKE, er=FAKE, qc=FAKE, ec=FAKE, s=FAKE: \
        L.moss_quant_act_2level_given_max(x, rows, cols, ld, flags, mx, qr, er, qc, ec, s, None)
    assert q(None, 32, 32, 32, 1) == 1
    assert q(FAKE, 32, 32, 32, 1, mx=None) == 1           # no maximum word
    assert q(FAKE, 32, 32, 32, 3, ec=None) == 1
    assert q(FAKE, 32, 48, 48, 1) == 2
    assert q(FAKE, 48, 32, 32, 2) == 2
    assert q(FAKE, 32, 32, 36, 1) == 3
    assert q(FAKE, 32, 32, 32, 1, mx=FAKE + 2) == 3       # misaligned maximum word
    assert q(FAKE, 32, 32, 32, 1 | 8) == 5                # no workspace here, so no promise about one
    assert q(FAKE, 32, 32, 32, 0) == 5
    f = lambda g=FAKE, u=FAKE, rows=4, cols=8, ld=8, h=FAKE, m=FAKE: L.moss_swiglu_bf16(g, u, rows, cols, ld, h, m, None)
    assert f(g=None) == 1 and f(m=None) == 1
    assert f(cols=12, ld=16) == 2                         # cols not a multiple of 8
    assert f(rows=0) == 2 and f(ld=4) == 2
    assert f(ld=12, cols=8) == 3                          # ld not a multiple of 8
    assert f(h=FAKE + 8) == 3
    b = lambda dh=FAKE, dg=FAKE, du=FAKE, mg=FAKE, mu=FAKE + 4, cols=8: \
        L.moss_swiglu_bf16_backward(FAKE, FAKE, dh, 4, cols, 8, dg, du, mg, mu, None)
    assert b(dh=None) == 1 and b(mu=None) == 1
    assert b(cols=4) == 2
    assert b(du=FAKE + 2) == 3
    assert b(mg=FAKE, mu=FAKE) == 5                       # one word for two maxima


def test_rmsnorm_argument_validation(L):
    import ctypes
    f = lambda x=FAKE, d=None, g=FAKE, eps=1e-5, rows=4, cols=64, ld=64, h=None, y=FAKE, m=FAKE: \
        L.moss_add_rmsnorm_bf16(x, d, g, ctypes.c_float(eps), rows, cols, ld, h, y, m, None)
    assert f(x=None) == 1 and f(m=None) == 1
    assert f(d=FAKE, h=None) == 1                          # a residual sum needs somewhere to go
    assert f(cols=12) == 2 and f(rows=0) == 2 and f(ld=32) == 2 and f(eps=-1.0) == 2
    assert f(cols=16384 + 8, ld=16384 + 8) == 5            # a row has to fit one workgroup's registers
    assert f(ld=68) == 3 and f(y=FAKE + 8) == 3 and f(m=FAKE + 2) == 3
    b = lambda h=FAKE, g=FAKE, dy=FAKE, dr=None, cols=64, dh=FAKE, m=FAKE: \
        L.moss_rmsnorm_bf16_backward(h, g, dy, dr, ctypes.c_float(1e-5), 4, cols, 64, dh, m, None)
    assert b(dy=None) == 1 and b(m=None) == 1
    assert b(cols=60) == 2
    assert b(dr=FAKE + 4) == 3 and b(dh=FAKE + 2) == 3


def test_weight_argument_validation(L):
    args = moss.AdamWArgs(3e-4, 0.9, 0.95, 1e-8, 0.1, 0.1, 0.05, 0.1, 0.05, 1.0, 500, 1)
    big = 1 << 20
    assert L.moss_weight_autoscale_init(None, 1, 4, 32, FAKE, FAKE, None, FAKE, big, None) == 1
    assert L.moss_weight_autoscale_init(FAKE, 7, 4, 32, FAKE, FAKE, None, FAKE, big, None) == 5
    assert L.moss_weight_autoscale_init(FAKE, 1, 3, 3, FAKE, FAKE, None, FAKE, big, None) == 2
    assert L.moss_weight_autoscale_init(FAKE, 1, 4, 32, FAKE, FAKE, None, FAKE, 8, None) == 4
    assert L.moss_weight_autoscale_cast(FAKE, FAKE, None, FAKE, 1, 4, 32, C.byref(args), FAKE, FAKE, None, FAKE, big, None) == 1
    assert L.moss_weight_autoscale_cast(FAKE, FAKE, FAKE, FAKE, 1, 4, 32, None, FAKE, FAKE, None, FAKE, big, None) == 1
    assert L.moss_weight_autoscale_cast(FAKE + 4, FAKE, FAKE, FAKE, 1, 4, 32, C.byref(args), FAKE, FAKE, None, FAKE, big, None) == 3
    args.step = 0
    assert L.moss_weight_autoscale_cast(FAKE, FAKE, FAKE, FAKE, 1, 4, 32, C.byref(args), FAKE, FAKE, None, FAKE, big, None) == 2


def test_gemm_argument_validation(L):
    g = lambda M, N, K, a=FAKE, b=FAKE, a_s=FAKE, b_s=FAKE, out=FAKE, dt=0, ld=None, acc=0: \
        L.moss_gemm_fp8_mx(M, N, K, a, None, a_s, b, None, b_s, out, dt, N if ld is None else ld, acc, None, 0, None)
    assert g(16, 16, 32, a=None) == 1
    assert g(16, 16, 32, a_s=None) == 1
    assert g(16, 16, 48) == 2                              # K not a multiple of the group size
    assert g(0, 16, 32) == 2
    assert g(16, 16, 32, ld=8) == 2                        # ld_out < N
    assert g(16, 16, 32, dt=9) == 5
    assert g(16, 16, 32, dt=0, acc=1) == 5                 # accumulate needs an FP32 output
    assert g(16, 16, 32, out=FAKE + 2) == 3
    assert L.moss_gemm_bf16_baseline(16, 16, 32, None, FAKE, FAKE, 16, None) == 1


def test_missing_library_fails_loudly(monkeypatch):
    from paper_2511_05811_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", "/nonexistent/libmoss_hip.so")
    with pytest.raises(moss.MossError):
        binding.load()

"""Host-only checks of the C ABI: the library loads, exports what include/prima.h declares,
and rejects bad arguments before launching anything (no GPU needed: validation is host code)."""
import ctypes as C
import os
import re

import pytest

from paper_2504_08791_amd import _ffi

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "prima.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(prima_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared()
    assert "prima_q4k_gemv" in names and "prima_attn_decode" in names and "prima_layer_window_decode" in names
    L = _ffi.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(_ffi.EXPORTS) == names


def test_abi_version_and_status_strings():
    L = _ffi.lib()
    assert L.prima_abi_version() == 1
    for code in range(7):
        assert L.prima_status_str(code)


def _dims(**kw):
    d = dict(e=512, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=768, rope_theta=1e4, rms_eps=1e-5, rope_mode=0)
    d.update(kw)
    return _ffi.Dims(**d)


FAKE = 0x7f0000001000  # never dereferenced: every call below must fail validation first


def test_gemv_argument_errors():
    L = _ffi.lib()
    f = lambda W=FAKE, rows=8, cols=512, x=FAKE, ldx=512, T=1, y=FAKE, ldy=8, ws=FAKE, wsb=1 << 20: \
        L.prima_q4k_gemv(W, rows, cols, x, ldx, T, y, ldy, ws, wsb, None)
    assert f(W=None) == 1 and f(x=None) == 1 and f(y=None) == 1 and f(ws=None) == 1
    assert f(cols=300) == 2 and f(ldx=256) == 2 and f(ldy=4) == 2
    assert f(T=0) == 4 and f(T=17) == 4
    assert f(W=FAKE + 8) == 3 and f(x=FAKE + 4) == 3 and f(ldx=514) == 3 and f(ws=FAKE + 16) == 3
    assert f(wsb=0) == 5


def test_noalloc_gemv_argument_errors():
    """The variant with the library's fixed scratch: every refusal comes before any device call."""
    L = _ffi.lib()
    f = lambda W=FAKE, rows=8, cols=512, x=FAKE, ldx=512, T=1, y=FAKE, ldy=8: \
        L.prima_q4k_gemv_noalloc(W, rows, cols, x, ldx, T, y, ldy, None)
    assert f(W=None) == 1 and f(x=None) == 1 and f(y=None) == 1
    assert f(cols=300) == 2 and f(ldx=256) == 2 and f(ldy=4) == 2
    assert f(T=0) == 4 and f(T=17) == 4
    assert f(W=FAKE + 8) == 3 and f(x=FAKE + 4) == 3 and f(ldx=514) == 3
    # a shape whose scratch exceeds the fixed array (the output layer at 8 tokens) is refused, nothing is launched
    assert L.prima_gemv_workspace_bytes(128256, 8192, 8) > _ffi.NOALLOC_SCRATCH_BYTES
    assert f(rows=128256, cols=8192, ldx=8192, T=8, ldy=128256) == 5
    assert f(rows=0) == 0


def test_dequant_argument_errors():
    L = _ffi.lib()
    assert L.prima_q4k_dequant(None, 1, 256, FAKE, None) == 1
    assert L.prima_q4k_dequant(None, 0, 256, None, None) == 0
    assert L.prima_q4k_dequant(FAKE, 1, 100, FAKE, None) == 2
    assert L.prima_q4k_dequant(FAKE + 2, 1, 256, FAKE, None) == 3


def test_attn_argument_errors():
    L = _ffi.lib()
    d = _dims()
    f = lambda dd=d, q=FAKE, k=FAKE, v=FAKE, cap=64, n_past=10, T=1, o=FAKE, ws=FAKE, wsb=1 << 30: \
        L.prima_attn_decode(C.byref(dd), q, k, v, cap, n_past, T, o, ws, wsb, None)
    assert f(q=None) == 1 and f(k=None) == 1 and f(o=None) == 1
    assert f(dd=_dims(head_dim=96)) == 2 and f(dd=_dims(n_q_heads=5)) == 2
    assert f(n_past=64) == 4 and f(T=0) == 4 and f(n_past=-1) == 4 and f(T=17) == 4
    assert f(k=FAKE + 2) == 3
    assert f(wsb=16) == 5


def test_window_argument_errors():
    L = _ffi.lib()
    d = _dims()
    lay = (_ffi.Layer * 1)()
    for name, _ in _ffi.Layer._fields_:
        setattr(lay[0], name, FAKE)
    need = L.prima_workspace_bytes(C.byref(d), 64, 4)
    assert need > 0
    f = lambda dd=d, layers=lay, Ln=1, cap=64, n_past=10, T=4, xi=FAKE, xo=FAKE, ws=FAKE, wsb=need: \
        L.prima_layer_window_decode(C.byref(dd), layers, Ln, cap, n_past, T, xi, xo, ws, wsb, None)
    assert f(xi=None) == 1 and f(ws=None) == 1 and f(layers=None) == 1
    assert f(dd=_dims(e=500)) == 2
    assert f(n_past=61) == 4 and f(Ln=0) == 4 and f(T=17) == 4
    assert f(xi=FAKE + 4) == 3
    assert f(wsb=need - 1) == 5
    bad = (_ffi.Layer * 1)()
    for name, _ in _ffi.Layer._fields_:
        setattr(bad[0], name, FAKE)
    bad[0].wo = None
    assert f(layers=bad) == 1
    assert L.prima_workspace_bytes(C.byref(_dims(e=100)), 64, 1) == 0


def test_matrix_product_and_prefill_argument_errors():
    """Every call fails validation before anything is launched (no GPU here)."""
    L = _ffi.lib()
    need = L.prima_gemm_workspace_bytes(40, 512)
    assert need >= 40 * 8 + 3 * 2 * 17 * 1024 and L.prima_gemm_workspace_bytes(0, 512) == 0 and L.prima_gemm_workspace_bytes(4, 300) == 0
    f = lambda W=FAKE, rows=8, cols=512, x=FAKE, ldx=512, T=40, gain=None, resid=None, ldr=0, y=FAKE, ldy=8, ws=FAKE, wsb=need: \
        L.prima_q4k_gemm(W, rows, cols, x, ldx, T, gain, 1e-5, resid, ldr, y, ldy, ws, wsb, None)
    assert f(W=None) == 1 and f(x=None) == 1 and f(y=None) == 1 and f(ws=None) == 1
    assert f(cols=300) == 2 and f(ldx=256) == 2 and f(ldy=4) == 2 and f(resid=FAKE, ldr=4) == 2
    assert f(T=0) == 4 and f(T=65537) == 4
    assert f(W=FAKE + 8) == 3 and f(x=FAKE + 4) == 3 and f(ldx=514) == 3 and f(gain=FAKE + 4) == 3 and f(ws=FAKE + 16) == 3
    assert f(wsb=need - 1) == 5

    d = _dims()
    lay = (_ffi.Layer * 1)()
    for name, _ in _ffi.Layer._fields_:
        setattr(lay[0], name, FAKE)
    needp = L.prima_prefill_workspace_bytes(C.byref(d), 256, 100)
    assert needp > L.prima_prefill_workspace_bytes(C.byref(d), 256, 50) > 0
    assert L.prima_prefill_workspace_bytes(C.byref(d), 256, 8193) == 0 and L.prima_prefill_workspace_bytes(C.byref(_dims(e=100)), 256, 8) == 0
    g = lambda dd=d, layers=lay, Ln=1, cap=256, n_past=10, T=100, xi=FAKE, xo=FAKE, ws=FAKE, wsb=needp: \
        L.prima_layer_window_prefill(C.byref(dd), layers, Ln, cap, n_past, T, xi, xo, ws, wsb, None)
    assert g(xi=None) == 1 and g(ws=None) == 1 and g(layers=None) == 1
    assert g(dd=_dims(e=500)) == 2
    assert g(n_past=157) == 4 and g(Ln=0) == 4 and g(T=0) == 4 and g(T=8193, cap=10000) == 4
    assert g(xi=FAKE + 4) == 3
    assert g(wsb=needp - 1) == 5
    bad = (_ffi.Layer * 1)()
    for name, _ in _ffi.Layer._fields_:
        setattr(bad[0], name, FAKE)
    bad[0].wdown = None
    assert g(layers=bad) == 1


def test_matrix_product_k_division_policy():
    """Host logic, no GPU: K is divided only where row blocks (256 rows) x token blocks (64 tokens) leave at least half of
    the device's 512 workgroup slots empty; the shares fill the slots, hold at least four super-blocks each and are at
    most 16; the larger workspace holds shares x T x (rows rounded up to 256) floats behind the minimum."""
    L = _ffi.lib()
    for T in (1, 16, 64, 65, 100, 128, 256, 512, 1024, 5000):
        for rows in (1, 256, 257, 1024, 8192, 10240, 28672, 57344):
            for cols in (256, 1024, 4096, 8192, 28672):
                s = L.prima_gemm_ksplit(T, rows, cols)
                wgs = -(-rows // 256) * -(-T // 64)
                nb = cols // 256
                assert 1 <= s <= 16
                if s > 1:
                    assert s * wgs <= 512 and nb // s >= 4
                    assert (s + 1) * wgs > 512 or nb // (s + 1) < 4 or s == 16     # as many shares as the limits allow
                else:
                    assert wgs * 2 > 512 or nb < 8
                base = L.prima_gemm_workspace_bytes(T, cols)
                full = L.prima_gemm_workspace_bytes_ksplit(T, rows, cols)
                part = s * T * (-(-rows // 256) * 256) * 4 if s > 1 else 0
                assert full == -(-base // 256) * 256 + part
    # 70B-shaped projections against a prompt of 128 tokens
    assert [L.prima_gemm_ksplit(128, r, c) for r, c in ((8192, 8192), (8192, 28672), (28672, 8192))] == [8, 8, 2]
    assert L.prima_gemm_ksplit(0, 8, 256) == 0 and L.prima_gemm_ksplit(4, 8, 300) == 0 and L.prima_gemm_ksplit(4, -1, 256) == 0
    assert L.prima_gemm_workspace_bytes_ksplit(0, 8, 256) == 0 and L.prima_gemm_workspace_bytes_ksplit(4, 8, 300) == 0


def test_batch_window_argument_errors():
    L = _ffi.lib()
    d = _dims()
    lay = (_ffi.Layer * 2)()
    for i in range(2):
        for name, _ in _ffi.Layer._fields_:
            setattr(lay[i], name, None if name in ("k_cache", "v_cache") else FAKE)   # the layers' own caches may be null
    B = 3
    need = L.prima_workspace_bytes(C.byref(d), 64, B)
    np_ok = (C.c_int32 * B)(0, 10, 63)
    ptrs = (C.c_void_p * (2 * B))(*([FAKE] * (2 * B)))
    f = lambda dd=d, layers=lay, Ln=2, cap=64, Bn=B, npast=np_ok, kc=ptrs, vc=ptrs, xi=FAKE, xo=FAKE, ws=FAKE, wsb=need: \
        L.prima_layer_window_decode_batch(C.byref(dd), layers, Ln, cap, Bn, npast, kc, vc, xi, xo, ws, wsb, None)
    assert f(npast=None) == 1 and f(kc=None) == 1 and f(vc=None) == 1 and f(xi=None) == 1 and f(layers=None) == 1
    assert f(dd=_dims(head_dim=96)) == 2
    assert f(Bn=0) == 4 and f(Bn=17) == 4 and f(Ln=0) == 4
    assert f(npast=(C.c_int32 * B)(0, 64, 1)) == 4 and f(npast=(C.c_int32 * B)(0, -1, 1)) == 4
    hole = (C.c_void_p * (2 * B))(*([FAKE] * (2 * B)))
    hole[4] = None
    assert f(kc=hole) == 1
    odd = (C.c_void_p * (2 * B))(*([FAKE] * (2 * B)))
    odd[1] = FAKE + 2
    assert f(vc=odd) == 3
    assert f(wsb=need - 1) == 5
    bad = (_ffi.Layer * 2)()
    for i in range(2):
        for name, _ in _ffi.Layer._fields_:
            setattr(bad[i], name, FAKE)
    bad[1].wdown = None
    assert f(layers=bad) == 1


def test_every_mat_vec_shape_can_be_planned():
    """Every number of super-blocks per row up to 160, every token count, few and many rows: a plan exists, fits the
    scratch, and gives every part of a unit a chunk in every slab of K (the kernel's unit queue relies on it: a plan
    that split K further than the short last slab allows once gave wrong sums and a memory fault, e.g. 8000 rows of
    41 or 57 super-blocks at 2 to 4 tokens)."""
    L = _ffi.lib()
    for nb in range(1, 161):
        for T in range(1, 17):
            for rows in (1, 17, 300, 1000, 8000, 20000):
                assert L.prima_gemv_plan_status(rows, nb * 256, T) == 0, (rows, nb, T)
    assert L.prima_gemv_plan_status(8, 100, 1) == 2 and L.prima_gemv_plan_status(8, 256, 0) == 4 and L.prima_gemv_plan_status(0, 256, 1) == 0


def test_format_calls_argument_errors():
    """The calls for the other weight formats refuse bad arguments before anything is launched."""
    L = _ffi.lib()
    d = _dims()
    Q4, Q6, F32 = 0, 2, 5
    assert L.prima_fmt_tensor_bytes(Q6, 4, 512) == 4 * 2 * 210 and L.prima_fmt_tensor_bytes(Q4, 4, 512) == 4 * 2 * 144
    assert L.prima_fmt_tensor_bytes(Q6, 4, 100) == 0 and L.prima_fmt_tensor_bytes(9, 4, 256) == 0 and L.prima_fmt_tensor_bytes(Q6, -1, 256) == 0
    g = lambda fmt=Q6, W=FAKE, r=8, c=512, x=FAKE, ldx=512, T=1, y=FAKE, ldy=8: L.prima_fmt_gemv(fmt, W, r, c, x, ldx, T, y, ldy, None)
    assert g(W=None) == 1 and g(x=None) == 1 and g(y=None) == 1
    assert g(fmt=Q4) == 2 and g(fmt=6) == 2 and g(fmt=-1) == 2            # Q4_K has its own entry point
    assert g(c=500) == 2 and g(ldx=256) == 2 and g(ldy=4) == 2 and g(c=0) == 2
    assert g(T=0) == 4 and g(T=17) == 4
    assert g(W=FAKE + 8) == 3 and g(x=FAKE + 4) == 3 and g(ldx=514) == 3 and g(y=FAKE + 2) == 3
    assert g(r=0) == 0                                                     # nothing to do
    q = lambda fmt=F32, W=FAKE, r=8, c=512, out=FAKE: L.prima_fmt_dequant(fmt, W, r, c, out, None)
    assert q(W=None) == 1 and q(out=None) == 1 and q(c=300) == 2 and q(fmt=7) == 2 and q(W=FAKE + 4) == 3
    assert q(r=0, W=None, out=None) == 0
    h = lambda dd=d, fmt=Q6, gf=FAKE, W=FAKE, vocab=100, x=FAKE, T=1, lo=FAKE: L.prima_lm_head_fmt(C.byref(dd), fmt, gf, W, vocab, x, T, lo, None)
    assert h(gf=None) == 1 and h(W=None) == 1 and h(x=None) == 1 and h(lo=None) == 1
    assert h(fmt=Q4) == 2 and h(vocab=0) == 2 and h(dd=_dims(head_dim=96)) == 2
    assert h(T=0) == 4 and h(T=17) == 4 and h(x=FAKE + 4) == 3
    # a window with formats: codes checked for every layer
    lay = (_ffi.Layer * 2)()
    for i in range(2):
        for name, _ in _ffi.Layer._fields_:
            setattr(lay[i], name, FAKE)
    fm = (_ffi.LayerFormats * 2)()
    need = L.prima_workspace_bytes(C.byref(d), 64, 1)
    w = lambda layers=lay, formats=fm, Ln=2, cap=64, npast=10, T=1, xi=FAKE, xo=FAKE, ws=FAKE, wsb=need: \
        L.prima_layer_window_decode_mixed(C.byref(d), layers, formats, Ln, cap, npast, T, xi, xo, ws, wsb, None)
    assert w(formats=None) == 1 and w(layers=None) == 1 and w(xi=None) == 1
    assert w(Ln=0) == 4 and w(npast=64) == 4 and w(wsb=need - 1) == 5
    bad = (_ffi.LayerFormats * 2)()
    bad[1].wdown = 6
    assert w(formats=bad) == 2
    ptrs = (C.c_void_p * 6)(*([FAKE] * 6))
    lens = (C.c_int32 * 3)(0, 5, 9)
    needb = L.prima_workspace_bytes(C.byref(d), 64, 3)
    assert L.prima_layer_window_decode_batch_mixed(C.byref(d), lay, bad, 2, 64, 3, lens, ptrs, ptrs, FAKE, FAKE, FAKE, needb, None) == 2
    assert L.prima_layer_window_decode_batch_mixed(C.byref(d), lay, fm, 2, 64, 3, None, ptrs, ptrs, FAKE, FAKE, FAKE, needb, None) == 1
    bad[1].wdown = -1
    assert w(formats=bad) == 2


def test_missing_library_is_an_error(monkeypatch, tmp_path):
    monkeypatch.setattr(_ffi, "_lib", None)
    monkeypatch.setattr(_ffi, "LIB_PATH", str(tmp_path / "absent.so"))
    with pytest.raises(ImportError):
        _ffi.lib()


def test_every_model_shape_and_token_count_can_be_planned():
    """Every mat-vec launch of a window step (the subsets launched for mixed formats included) finds a plan that fits
    the scratch the library asks for: all benchmark shapes, the tiny test shapes and two more models' shapes, every
    token count.  (A scratch sized from the plan of a slightly different tile count once refused config 0's shape
    from 8 tokens on.)"""
    from workloads.configs import CONFIGS, TINY, ModelDims
    L = _ffi.lib()
    shapes = {c.dims for c in list(CONFIGS.values()) + list(TINY.values())}
    shapes |= {ModelDims(3584, 28, 4, 128, 18944, 1e6), ModelDims(2048, 16, 2, 128, 5632, 1e4), ModelDims(4096, 32, 32, 128, 11008, 1e4)}
    for dm in shapes:
        d = _ffi.Dims(dm.e, dm.n_q_heads, dm.n_kv_heads, dm.head_dim, dm.ffn, dm.rope_theta, dm.rms_eps, dm.rope_mode)
        for T in range(1, 17):
            assert L.prima_window_plan_status(C.byref(d), 4096 + T, T) == 0, (dm, T)
    # a grid of small shapes, among them hidden sizes above 2 ffn and above the Q/K/V rows (the arrival counters were
    # once sized for those two only)
    for D, Hkv, G in [(64, 1, 4), (64, 8, 7), (128, 2, 5), (128, 8, 8), (64, 16, 16)]:
        for e in (256, 1536, 3584, 8192):
            for ffn in (256, 1280, 4864, 14336):
                d = _ffi.Dims(e, Hkv * G, Hkv, D, ffn, 1e4, 1e-5, 0)
                for T in (1, 2, 5, 8, 11, 16):
                    assert L.prima_window_plan_status(C.byref(d), 1100, T) == 0, (D, Hkv, G, e, ffn, T)
    d = _dims()
    assert L.prima_window_plan_status(None, 64, 1) == 1 and L.prima_window_plan_status(C.byref(_dims(head_dim=96)), 64, 1) == 2
    assert L.prima_window_plan_status(C.byref(d), 64, 0) == 4 and L.prima_window_plan_status(C.byref(d), 64, 17) == 4

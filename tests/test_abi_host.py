"""Host-side checks that need no GPU: the library loads, exports the declared symbols, and
validates arguments before touching the device."""
import ctypes
import os
import pathlib
import re

import pytest

ROOT = pathlib.Path(__file__).resolve().parent.parent


@pytest.fixture(scope="module")
def lib():
    from paper_2505_02146_amd import xp
    return xp.raw()


def _declared_symbols():
    text = (ROOT / "include" / "xp.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(xp_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_symbols()
    assert {"xp_gemm", "xp_gemm_batched", "xp_conv2d_nhwc", "xp_attention", "xp_num_configs", "xp_describe_config",
            "xp_force_config", "xp_last_config", "xp_status_string", "xp_version"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_lds_poison_build_exports_the_same_symbols():
    path = ROOT / "paper_2505_02146_amd" / "libxp_poison.so"
    assert path.exists(), "run paper_2505_02146_amd/build.py"
    debug = ctypes.CDLL(str(path))
    for n in _declared_symbols():
        assert hasattr(debug, n), n


def test_oracle_and_library_share_no_code():
    # neither side includes or imports the other
    for f in (ROOT / "paper_2505_02146_amd").rglob("*"):
        if f.suffix in (".hip", ".hpp", ".py", ".h"):
            t = f.read_text()
            assert "xp_oracle" not in t and "import oracle" not in t and "from oracle" not in t, f
    for f in (ROOT / "oracle").glob("*"):
        if f.suffix in (".c", ".h", ".py"):
            t = f.read_text()
            assert "paper_2505_02146_amd" not in t and "xp.h" not in t, f


def test_variant_tables(lib):
    from paper_2505_02146_amd import xp
    for t in ("f32", "bf16", "i8"):
        n = xp.xp_num_configs(xp.XP_OP_GEMM, t)
        assert n >= 2
        names = [xp.xp_describe_config(xp.XP_OP_GEMM, t, i) for i in range(n)]
        assert len(set(names)) == n
        assert names[0].startswith("general")
    assert xp.xp_num_configs(xp.XP_OP_GEMM, xp.XP_I32) == 0
    buf = ctypes.create_string_buffer(8)
    assert lib.xp_describe_config(0, xp.XP_BF16, 999, buf, 8) == 6
    assert lib.xp_describe_config(0, xp.XP_BF16, 1, buf, 8) == 0 and len(buf.value) == 7   # truncated, NUL kept
    assert lib.xp_force_config(0, xp.XP_BF16, 999) == 6
    assert lib.xp_force_config(0, xp.XP_BF16, -1) == 0
    assert lib.xp_last_config(0, xp.XP_I32) == -1


def _gemm(lib, M=4, N=4, K=4, alpha=1.0, A=16, at=0, al=0, lda=4, B=16, bt=0, bl=0, ldb=4, beta=0.0,
          C=16, ct=0, cl=0, ldc=4):
    return lib.xp_gemm(M, N, K, alpha, A, at, al, lda, B, bt, bl, ldb, beta, C, ct, cl, ldc, None)


def test_gemm_validation_returns_before_any_launch(lib):
    # pointers are fake (never dereferenced on the host, and every call below is rejected)
    assert _gemm(lib, M=-1) == 2
    assert _gemm(lib, K=-3) == 2
    assert _gemm(lib, A=None) == 1
    assert _gemm(lib, C=None) == 1
    assert _gemm(lib, lda=3) == 3
    assert _gemm(lib, ldb=3) == 3
    assert _gemm(lib, ldc=3) == 3
    assert _gemm(lib, al=1, lda=3, M=4, K=2) == 3          # column-major A needs ld >= M
    assert _gemm(lib, at=1, bt=0) == 5                     # mixed input types
    assert _gemm(lib, at=2, bt=2, ct=0) == 5               # int8 needs int32 output
    assert _gemm(lib, at=2, bt=2, ct=3, alpha=2.0) == 5    # int8 has no scaling
    assert _gemm(lib, at=2, bt=2, ct=3, beta=1.0) == 5
    assert _gemm(lib, at=1, bt=1, ct=1) == 5               # bf16 output not provided
    assert _gemm(lib, al=7) == 5
    assert _gemm(lib, A=18) == 4                           # fp32 pointer not 4-byte aligned
    # empty problems succeed without a launch (and without looking at the pointers)
    assert _gemm(lib, M=0, A=None, B=None, C=None) == 0
    assert _gemm(lib, N=0, A=None, B=None, C=None) == 0


def test_batched_validation(lib):
    def call(batch=2, sa=16, sb=16, sc=16, **kw):
        a = dict(M=4, N=4, K=4, alpha=1.0, A=16, at=0, al=0, lda=4, B=16, bt=0, bl=0, ldb=4, beta=0.0,
                 C=16, ct=0, cl=0, ldc=4)
        a.update(kw)
        return lib.xp_gemm_batched(batch, a["M"], a["N"], a["K"], a["alpha"], a["A"], a["at"], a["al"], a["lda"], sa,
                                   a["B"], a["bt"], a["bl"], a["ldb"], sb, a["beta"], a["C"], a["ct"], a["cl"],
                                   a["ldc"], sc, None)
    assert call(batch=-1) == 2
    assert call(sc=15) == 3                                # C slices would overlap
    assert call(sa=-1) == 3
    assert call(batch=0, A=None, B=None, C=None) == 0
    assert call(A=None) == 1


def test_conv_validation(lib):
    def call(N=1, H=4, W=4, Cin=2, Cout=2, R=3, S=3, sh=1, sw=1, ph=1, pw=1, x=16, xt=0, w=16, wt=0, wl=0,
             out=16, ot=0):
        return lib.xp_conv2d_nhwc(N, H, W, Cin, Cout, R, S, sh, sw, ph, pw, x, xt, w, wt, wl, out, ot, None)
    assert call(N=-1) == 2
    assert call(R=0) == 2
    assert call(sh=0) == 2
    assert call(ph=-1) == 2
    assert call(x=None) == 1
    assert call(out=None) == 1
    assert call(xt=2, wt=2) == 5                           # int8 convolution not provided
    assert call(xt=1, wt=0) == 5
    assert call(ot=1) == 5
    assert call(wl=3) == 5
    assert call(H=1, W=1, ph=0, pw=0, x=None, w=None, out=None) == 0   # filter larger than image: empty
    assert call(N=0, x=None, w=None, out=None) == 0


def test_attention_validation(lib):
    # every call here must be turned away (or be empty) on the host: the pointers are fake
    def call(batch=2, Lq=4, Lk=4, d=8, dv=8, scale=0.5, Q=16, qt=0, ldq=8, sq=32, K=16, kt=0, ldk=8, sk=32,
             V=16, vt=0, ldv=8, sv=32, O=16, ot=0, ldo=8, so=32):
        return lib.xp_attention(batch, Lq, Lk, d, dv, scale, Q, qt, ldq, sq, K, kt, ldk, sk, V, vt, ldv, sv,
                                O, ot, ldo, so, None)
    assert call(batch=-1) == 2
    assert call(Lk=-1) == 2
    assert call(Lk=0) == 2                                 # softmax over no keys
    assert call(Lk=0, Lq=0) == 0                           # ... unless the output is empty
    assert call(batch=0, Q=None, K=None, V=None, O=None) == 0
    assert call(dv=0, V=None, O=None) == 0
    assert call(ldq=7) == 3
    assert call(ldk=7) == 3
    assert call(ldv=7) == 3
    assert call(ldo=7) == 3
    assert call(sq=-1) == 3
    assert call(so=31) == 3                                # O slices would overlap
    assert call(Q=None) == 1
    assert call(V=None) == 1
    assert call(O=None) == 1
    assert call(qt=1, kt=0) == 5                           # mixed input types
    assert call(qt=2, kt=2, vt=2) == 5                     # int8 attention not provided
    assert call(ot=1) == 5
    assert call(scale=float("nan")) == 5
    assert call(scale=float("inf")) == 5
    assert call(Q=17, qt=1, kt=1, vt=1) == 4               # bf16 pointer not 2-byte aligned
    assert call(O=18) == 4


def test_attention_variant_table(lib):
    from paper_2505_02146_amd import xp
    assert xp.xp_num_configs(xp.XP_OP_ATTENTION, "bf16") >= 2
    assert xp.xp_num_configs(xp.XP_OP_ATTENTION, "f32") >= 1
    assert xp.xp_num_configs(xp.XP_OP_ATTENTION, "i8") == 0
    assert xp.xp_describe_config(xp.XP_OP_ATTENTION, "bf16", 0).startswith("general")
    assert lib.xp_force_config(xp.XP_OP_ATTENTION, xp.XP_BF16, 99) == 6
    assert lib.xp_force_config(xp.XP_OP_ATTENTION, xp.XP_BF16, -1) == 0
    assert lib.xp_last_config(xp.XP_OP_ATTENTION, xp.XP_I8) == -1


def test_tuned_shape_table_round_trip(lib, tmp_path):
    from paper_2505_02146_amd import xp
    xp.xp_tune_clear()
    assert xp.xp_tune_count() == 0
    src = tmp_path / "tuned.txt"
    src.write_text("# comment\n"
                   "gemm0 t1 b1 m512 n512 k512 a1 b1 | bf16 128x128x128B waves 2x2 ring 2 direct-to-lds mfma16\n"
                   "gemm0 t1 b1 m512 n512 k512 a1 b1 | bf16 64x64x128B waves 2x2 stages 2 mfma32\n"      # replaces the line above
                   "conv t1 n2 h8 w8 c64 k64 r3 s3 sh1 sw1 ph1 pw1 b1 | no such variant\n"
                   "a line without a separator\n")
    xp.xp_tune_load(src)
    assert xp.xp_tune_count() == 2
    dst = tmp_path / "saved.txt"
    xp.xp_tune_save(dst)
    lines = [l for l in dst.read_text().splitlines() if not l.startswith("#")]
    assert lines == ["conv t1 n2 h8 w8 c64 k64 r3 s3 sh1 sw1 ph1 pw1 b1 | no such variant",
                     "gemm0 t1 b1 m512 n512 k512 a1 b1 | bf16 64x64x128B waves 2x2 stages 2 mfma32"]
    xp.xp_tune_clear()
    xp.xp_tune_load(dst)
    assert xp.xp_tune_count() == 2
    xp.xp_tune_clear()
    assert xp.xp_tune_count() == 0
    assert lib.xp_tune_load(str(tmp_path / "missing.txt").encode()) == 8
    assert lib.xp_tune_save(str(tmp_path / "no_such_dir" / "x.txt").encode()) == 8
    assert lib.xp_tune_load(None) == 1 and lib.xp_tune_save(None) == 1
    assert xp.xp_tune_workspace_bytes(0) == 256 and xp.xp_tune_workspace_bytes(64) == 768
    assert xp.xp_tune_workspace_bytes(-1) == 0


def test_tune_validation(lib):
    # every call here must be turned away (or be empty) on the host: the pointers are fake
    def call(M=64, N=64, K=64, A=256, B=256, C=256, ws=256, ws_bytes=1 << 20, reps=3, at=0, ct=0):
        return lib.xp_tune_gemm(M, N, K, 1.0, A, at, 0, K, B, at, 1, K, 0.0, C, ct, 0, N, ws, ws_bytes, reps, None, None, None)
    assert call(M=-1) == 2
    assert call(A=None) == 1
    assert call(at=1, ct=1) == 5
    assert call(reps=0) == 2
    assert call(ws=None) == 8
    assert call(ws=260) == 8                                  # not 256-byte aligned
    assert call(ws_bytes=2 * 64 * 64 * 4 + 255) == 8          # one byte short
    assert call(M=0, A=None, B=None, C=None, ws=None) == 0    # nothing to compute, nothing recorded
    from paper_2505_02146_amd import xp
    assert xp.xp_tune_count() == 0


def test_memory_bound_operator_validation(lib):
    # every call here must be turned away (or be empty) on the host: the pointers are fake
    def soft(rows=2, cols=8, x=64, xt=0, ldx=8, y=64, yt=0, ldy=8):
        return lib.xp_softmax(rows, cols, x, xt, ldx, y, yt, ldy, None)
    assert soft(rows=-1) == 2
    assert soft(ldx=7) == 3 and soft(ldy=7) == 3
    assert soft(x=None) == 1 and soft(y=None) == 1
    assert soft(xt=2) == 5 and soft(yt=3) == 5
    assert soft(x=66, xt=0) == 4 and soft(x=65, xt=1) == 4
    assert soft(rows=0, x=None, y=None) == 0 and soft(cols=0, x=None, y=None, ldx=0, ldy=0) == 0
    assert lib.xp_layernorm(2, 8, 64, 0, 8, None, None, -1.0, 64, 0, 8, None) == 5       # negative eps
    assert lib.xp_layernorm(2, 8, 64, 0, 8, 66, None, 1e-5, 64, 0, 8, None) == 4        # gamma misaligned
    assert lib.xp_rmsnorm(2, 8, 64, 0, 8, None, float("inf"), 64, 0, 8, None) == 5
    assert lib.xp_unary(7, 4, 64, 0, 64, 0, None) == 5
    assert lib.xp_unary(0, -1, 64, 0, 64, 0, None) == 2
    assert lib.xp_unary(0, 4, None, 0, 64, 0, None) == 1
    assert lib.xp_unary(0, 0, None, 0, None, 0, None) == 0
    assert lib.xp_add(4, 64, None, 0, 64, 0, None) == 1
    assert lib.xp_add(4, 64, 64, 2, 64, 0, None) == 5
    def pool(op=0, N=1, H=4, W=4, C=8, R=2, S=2, sh=2, sw=2, ph=0, pw=0, x=64, xt=0, y=64, yt=0):
        return lib.xp_pool2d_nhwc(op, N, H, W, C, R, S, sh, sw, ph, pw, x, xt, y, yt, None)
    assert pool(op=4) == 5 and pool(R=0) == 2 and pool(sh=0) == 2 and pool(ph=-1) == 2 and pool(N=-1) == 2
    assert pool(x=None) == 1 and pool(xt=2) == 5
    assert pool(H=1, W=1, x=None, y=None) == 0                # window larger than the image: empty
    assert pool(C=0, x=None, y=None) == 0
    def dw(N=1, H=4, W=4, C=8, R=3, S=3, sh=1, sw=1, ph=1, pw=1, x=64, xt=0, w=64, wt=0, wl=1, y=64, yt=0):
        return lib.xp_depthwise_conv2d_nhwc(N, H, W, C, R, S, sh, sw, ph, pw, x, xt, w, wt, wl, y, yt, None)
    assert dw(R=0) == 2 and dw(N=-1) == 2 and dw(sw=0) == 2
    assert dw(wl=2) == 5 and dw(xt=1, wt=0) == 5 and dw(xt=2, wt=2) == 5
    assert dw(x=None) == 1 and dw(w=None) == 1 and dw(y=None) == 1
    assert dw(w=66) == 4
    assert dw(H=1, W=1, ph=0, pw=0, x=None, w=None, y=None) == 0


def test_deformable_attention_validation(lib):
    # every call here must be turned away (or be empty) on the host: the pointers are fake
    import ctypes as C
    hs, ws = (C.c_int64 * 16)(*([4] * 16)), (C.c_int64 * 16)(*([4] * 16))
    def call(batch=1, Lq=2, heads=2, d=8, levels=2, points=2, v=256, vt=0, h=hs, w=ws, loc=256, wg=256, out=256, ot=0):
        return lib.xp_deformable_attention(batch, Lq, heads, d, levels, points, v, vt, C.cast(h, C.c_void_p) if h else None,
                                           C.cast(w, C.c_void_p) if w else None, loc, wg, out, ot, None)
    assert call(batch=-1) == 2 and call(points=-1) == 2 and call(levels=17) == 2
    assert call(vt=2) == 5 and call(ot=2) == 5
    assert call(h=None) == 1 and call(loc=None) == 1 and call(wg=None) == 1 and call(v=None) == 1 and call(out=None) == 1
    assert call(loc=260) == 4 and call(wg=258) == 4
    assert call(d=3, v=258) == 4 and call(d=3, out=258) == 4          # scalar path: element alignment
    bad = (C.c_int64 * 16)(*([-1] * 16))
    assert call(h=bad) == 2
    huge = (C.c_int64 * 16)(*([1 << 25] * 16))
    assert call(w=huge) == 2
    assert call(Lq=0, v=None, loc=None, wg=None, out=None) == 0 and call(d=0, out=None) == 0


def test_conv_nchw_validation(lib):
    # every call here must be turned away (or be empty) on the host: the pointers are fake
    def call(N=1, H=4, W=4, Cin=2, Cout=2, R=3, S=3, sh=1, sw=1, ph=1, pw=1, x=256, xt=0, w=256, wt=0, out=256, ot=0,
             ws=256, wsb=1 << 20):
        return lib.xp_conv2d_nchw(N, H, W, Cin, Cout, R, S, sh, sw, ph, pw, x, xt, w, wt, out, ot, ws, wsb, None)
    assert call(N=-1) == 2 and call(R=0) == 2 and call(sh=0) == 2
    assert call(xt=2, wt=2) == 5 and call(xt=1, wt=0) == 5 and call(ot=1) == 5
    assert call(x=None) == 1 and call(out=None) == 1
    assert call(ws=None) == 8 and call(ws=260) == 8 and call(wsb=100) == 8
    assert call(N=70000) == 2
    assert call(H=1, W=1, ph=0, pw=0, x=None, w=None, out=None, ws=None) == 0
    assert call(N=0, x=None, w=None, out=None, ws=None) == 0
    need = lib.xp_conv2d_nchw_workspace_bytes(1, 4, 4, 2, 2, 3, 3, 1, 1, 1, 1, 0)
    assert need == 256 + 256                             # activations 128 B + filter 144 B, each rounded up to 256
    assert lib.xp_conv2d_nchw_workspace_bytes(1, 4, 4, 2, 2, 0, 3, 1, 1, 1, 1, 0) == 0


def test_entry_points_resolve_their_builders():
    # build() compiles for minutes, so it is not run here; what broke once is the lookup of the
    # oracle's build module behind the package attribute of the same name
    import importlib
    import inspect
    entry = importlib.import_module("__graft_entry__")
    assert callable(entry.build) and callable(entry.smoke)
    assert inspect.ismodule(importlib.import_module("oracle.build"))
    assert callable(importlib.import_module("oracle.build").build)
    assert callable(importlib.import_module("paper_2505_02146_amd.build").build)
    assert 'import_module("oracle.build")' in inspect.getsource(entry.build)


def test_status_strings(lib):
    from paper_2505_02146_amd import xp
    seen = {xp.status_string(i) for i in range(9)}
    assert len(seen) == 9 and "ok" in seen
    assert "gfx950" in xp.version()


def test_built_in_tuned_table_is_the_generators_output():
    """xp_tuned_table.inc is generated from the tuner's saved text beside it; the two must agree."""
    import subprocess
    import sys
    src = os.path.join(os.path.dirname(__file__), "..", "paper_2505_02146_amd", "csrc")
    out = subprocess.run([sys.executable, os.path.join(src, "make_tuned_table.py"), os.path.join(src, "xp_tuned_grid.txt")],
                         check=True, capture_output=True, text=True).stdout
    assert out == open(os.path.join(src, "xp_tuned_table.inc")).read()
    names = set(l.split('"')[1] for l in out.splitlines() if l.startswith("{"))
    from paper_2505_02146_amd import xp
    known = set()
    for t in ("f32", "bf16", "i8"):
        for op in (0,):
            known |= {xp.xp_describe_config(op, t, i) for i in range(xp.xp_num_configs(op, t))}
    assert names <= known, names - known                 # every winner names a variant this build has

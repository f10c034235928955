"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, and validates arguments before touching a device."""
import os
import re

import pytest

import paper_2605_19218_amd as rk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PTR = 4096          # a fake, 16-byte aligned, non-NULL "device pointer"; never dereferenced


@pytest.fixture(scope="module")
def ctx():
    c = rk.rk_create(rk.RK_DEVICE_NONE)
    yield c
    rk.rk_destroy(c)


def layout(**kw):
    base = dict(batch=2, n_q_heads=8, n_kv_heads=2, keep=64, dtype=rk.RK_BF16, capacity=1024, max_seq_len=1000,
                seq_len=PTR)
    base.update(kw)
    return rk.Layout(**base)


def rows(n=1000, **kw):
    base = dict(data=PTR, n_tokens=n, strides=(2 * 1024 * 128, 1024 * 128, 128))
    base.update(kw)
    return rk.Rows(**base)


def fit_out(**kw):
    base = dict(R=PTR, eigvals=PTR, mask=PTR, keep_idx=PTR, R_r=PTR, mu=PTR, delta_mu=PTR)
    base.update(kw)
    return rk.FitOut(**base)


def status_of(fn, *a, **k):
    try:
        fn(*a, **k)
    except rk.RotateKError as e:
        return e.status
    return rk.RK_OK


def test_header_symbols_are_exported():
    text = open(os.path.join(ROOT, "include", "rotatek.h")).read()
    declared = set(re.findall(r"\b(rk_[a-z_]+)\s*\(", text))
    assert declared == set(rk.EXPORTS), declared ^ set(rk.EXPORTS)
    L = rk.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_layout_validation():
    assert rk.rk_validate_layout(layout()) == rk.RK_OK
    assert rk.rk_validate_layout(layout(head_dim=64)) == rk.RK_ERR_UNSUPPORTED
    assert rk.rk_validate_layout(layout(dtype=7)) == rk.RK_ERR_UNSUPPORTED
    assert rk.rk_validate_layout(layout(n_q_heads=7)) == rk.RK_ERR_INVALID_ARG
    assert rk.rk_validate_layout(layout(keep=0)) == rk.RK_ERR_INVALID_ARG
    assert rk.rk_validate_layout(layout(keep=129)) == rk.RK_ERR_INVALID_ARG
    assert rk.rk_validate_layout(layout(capacity=0)) == rk.RK_ERR_INVALID_ARG
    assert rk.rk_validate_layout(layout(capacity=1000)) == rk.RK_ERR_INVALID_ARG      # not a multiple of 32
    assert rk.rk_validate_layout(layout(batch=0)) == rk.RK_ERR_INVALID_ARG
    assert rk.lib().rk_validate_layout(None) == rk.RK_ERR_INVALID_ARG


def test_no_device_context_validates_then_refuses(ctx):
    lay = layout()
    ws = rk.rk_decode_workspace_size(ctx, lay)
    assert ws > 0
    ok = (ctx, lay, PTR, PTR, PTR, PTR, PTR, 0.0, PTR, PTR)
    assert status_of(rk.rk_decode_attn, *ok, workspace_bytes=ws) == rk.RK_ERR_NO_DEVICE
    assert status_of(rk.rk_decode_attn, *ok, workspace_bytes=ws - 1) == rk.RK_ERR_WORKSPACE
    assert status_of(rk.rk_decode_attn, ctx, lay, None, PTR, PTR, PTR, PTR, 0.0, PTR, PTR,
                     workspace_bytes=ws) == rk.RK_ERR_INVALID_ARG
    assert status_of(rk.rk_decode_attn, ctx, layout(seq_len=None), PTR, PTR, PTR, PTR, PTR, 0.0, PTR, PTR,
                     workspace_bytes=ws) == rk.RK_ERR_INVALID_ARG
    assert status_of(rk.rk_decode_attn, ctx, layout(max_seq_len=2000), PTR, PTR, PTR, PTR, PTR, 0.0, PTR, PTR,
                     workspace_bytes=1 << 30) == rk.RK_ERR_CAPACITY
    # delta_mu is optional
    assert status_of(rk.rk_decode_attn, ctx, lay, PTR, PTR, PTR, PTR, None, 0.0, PTR, PTR,
                     workspace_bytes=ws) == rk.RK_ERR_NO_DEVICE
    assert "device" in rk.lib().rk_status_str(rk.RK_ERR_NO_DEVICE).decode()


def test_fit_validation(ctx):
    lay = layout()
    ws = rk.rk_fit_workspace_size(lay, 1000)
    assert ws > 0 and rk.rk_fit_workspace_size(lay, 2000) > ws
    args = lambda **kw: (ctx, kw.get("lay", lay), kw.get("rows", rows()), None, kw.get("flags", rk.RK_FIT_CENTER),
                         kw.get("out", fit_out()), PTR)
    assert status_of(rk.rk_fit_rotation, *args(), workspace_bytes=ws) == rk.RK_ERR_NO_DEVICE
    assert status_of(rk.rk_fit_rotation, *args(), workspace_bytes=ws - 1) == rk.RK_ERR_WORKSPACE
    assert status_of(rk.rk_fit_rotation, *args(out=fit_out(R=None)), workspace_bytes=ws) == rk.RK_ERR_INVALID_ARG
    assert status_of(rk.rk_fit_rotation, *args(flags=8), workspace_bytes=ws) == rk.RK_ERR_INVALID_ARG
    assert status_of(rk.rk_fit_rotation, *args(rows=rows(data=None)), workspace_bytes=ws) == rk.RK_ERR_INVALID_ARG
    assert status_of(rk.rk_fit_rotation, *args(rows=rows(data=PTR + 2)), workspace_bytes=ws) == rk.RK_ERR_INVALID_ARG
    assert status_of(rk.rk_fit_rotation, *args(rows=rows(strides=(0, 0, 64))), workspace_bytes=ws) == rk.RK_ERR_INVALID_ARG
    assert status_of(rk.rk_fit_rotation, *args(rows=rows(tok_idx=PTR)), workspace_bytes=ws) == rk.RK_ERR_INVALID_ARG
    assert status_of(rk.rk_fit_rotation, *args(rows=rows(tok_idx=PTR, tok_off=PTR)), workspace_bytes=ws) == rk.RK_ERR_NO_DEVICE
    assert status_of(rk.rk_fit_rotation, *args(lay=layout(head_dim=96)), workspace_bytes=ws) == rk.RK_ERR_UNSUPPORTED
    assert b"128" in rk.lib().rk_last_error(ctx)


def test_compress_append_validation(ctx):
    lay = layout()
    assert status_of(rk.rk_compress, ctx, lay, rows(), PTR, PTR) == rk.RK_ERR_NO_DEVICE
    assert status_of(rk.rk_compress, ctx, lay, rows(n=1025), PTR, PTR) == rk.RK_ERR_CAPACITY
    assert status_of(rk.rk_compress, ctx, lay, rows(), None, PTR) == rk.RK_ERR_INVALID_ARG
    assert status_of(rk.rk_compress, ctx, lay, rows(), PTR, PTR, values=rows(), v_cache=None) == rk.RK_ERR_INVALID_ARG
    assert status_of(rk.rk_compress, ctx, lay, rows(), PTR, PTR, values=rows(n=999), v_cache=PTR) == rk.RK_ERR_INVALID_ARG
    assert status_of(rk.rk_compress, ctx, lay, rows(), PTR, PTR, values=rows(), v_cache=PTR) == rk.RK_ERR_NO_DEVICE
    ap = (PTR, PTR, PTR, PTR, PTR, PTR)
    assert status_of(rk.rk_append, ctx, lay, *ap) == rk.RK_ERR_NO_DEVICE
    assert status_of(rk.rk_append, ctx, layout(max_seq_len=1024), *ap) == rk.RK_ERR_CAPACITY
    assert status_of(rk.rk_append, ctx, lay, PTR, None, PTR, PTR, PTR, PTR) == rk.RK_ERR_INVALID_ARG
    assert status_of(rk.rk_gather_rotation, ctx, lay, PTR, PTR, PTR) == rk.RK_ERR_NO_DEVICE
    assert status_of(rk.rk_gather_rotation, ctx, lay, PTR, None, PTR) == rk.RK_ERR_INVALID_ARG
    assert status_of(rk.rk_unpack_cache, ctx, lay, PTR, PTR, PTR, PTR) == rk.RK_ERR_NO_DEVICE
    assert status_of(rk.rk_unpack_cache, ctx, lay, None, PTR, PTR, None) == rk.RK_ERR_INVALID_ARG
    assert status_of(rk.rk_unpack_cache, ctx, lay, PTR, PTR, None, None) == rk.RK_ERR_INVALID_ARG
    # cache sizes: keep is padded to a multiple of 16 channels
    assert rk.rk_cache_bytes(lay) == (2 * 2 * 1024 * 64 * 2, 2 * 2 * 1024 * 128 * 2)
    assert rk.rk_cache_bytes(layout(keep=37, dtype=rk.RK_F32))[0] == 2 * 2 * 1024 * 48 * 4
    # from 4096 tokens on the slabs are spaced 64 tokens above a multiple of 256 (never closer than the capacity)
    for cap, spaced in ((4064, 4064), (4096, 4160), (16384, 16448), (16448, 16448), (16480, 16704), (16512, 16704)):
        assert rk.rk_cache_bytes(layout(capacity=cap)) == (2 * 2 * spaced * 64 * 2, 2 * 2 * spaced * 128 * 2), cap


def test_decode_plan_and_options(ctx):
    lay = layout(batch=8, n_q_heads=28, n_kv_heads=4, capacity=16384, max_seq_len=16384)
    S, tps = rk.rk_decode_plan(ctx, lay)
    assert S >= 1 and tps % 128 == 0 and S * tps >= 16384 and (S - 1) * tps < 16384
    rk.rk_set_option(ctx, rk.RK_OPT_DECODE_SPLITS, 5)
    S5, tps5 = rk.rk_decode_plan(ctx, lay)
    assert S5 <= 5 and S5 * tps5 >= 16384
    rk.rk_set_option(ctx, rk.RK_OPT_DECODE_SPLITS, 0)
    assert rk.rk_decode_plan(ctx, lay) == (S, tps)
    assert status_of(rk.rk_set_option, ctx, 99, 1) == rk.RK_ERR_INVALID_ARG
    assert status_of(rk.rk_set_option, ctx, rk.RK_OPT_DECODE_SPLITS, -1) == rk.RK_ERR_INVALID_ARG
    # a short cache never gets more splits than 128-token tiles
    assert rk.rk_decode_plan(ctx, layout(max_seq_len=100))[0] == 1
    assert rk.rk_decode_plan(ctx, layout(max_seq_len=0))[0] == 1


def text(**kw):
    base = dict(k=PTR, v=PTR, max_len=64, len=PTR, capacity=64, strides=(2 * 64 * 128, 64 * 128, 128))
    base.update(kw)
    return rk.Text(**base)


def test_dual_decode_and_text_append_validation(ctx):
    lay = layout()
    ws = rk.rk_decode_workspace_size(ctx, lay)
    dec = lambda t, **kw: status_of(rk.rk_decode_attn_dual, ctx, kw.get("lay", lay), PTR, PTR, PTR, PTR, PTR, t, 0.0,
                                    PTR, PTR, workspace_bytes=kw.get("ws", ws))
    assert dec(text()) == rk.RK_ERR_NO_DEVICE
    assert dec(text(len=None)) == rk.RK_ERR_NO_DEVICE            # NULL len = max_len rows everywhere
    assert dec(None) == rk.RK_ERR_INVALID_ARG
    assert dec(text(k=None)) == rk.RK_ERR_INVALID_ARG
    assert dec(text(v=PTR + 2)) == rk.RK_ERR_INVALID_ARG          # misaligned base
    assert dec(text(strides=(2 * 64 * 128, 64 * 128, 100))) == rk.RK_ERR_INVALID_ARG   # rows overlap / misaligned
    assert dec(text(strides=(2 * 64 * 132, 64 * 132, 132))) == rk.RK_ERR_INVALID_ARG   # not a multiple of 8
    assert dec(text(max_len=65)) == rk.RK_ERR_INVALID_ARG
    assert dec(text(), ws=ws - 1) == rk.RK_ERR_WORKSPACE
    assert dec(text(), lay=layout(max_seq_len=2000)) == rk.RK_ERR_CAPACITY
    app = lambda t, k=PTR, v=PTR: status_of(rk.rk_append_text, ctx, lay, t, k, v)
    assert app(text(max_len=63)) == rk.RK_ERR_NO_DEVICE
    assert app(text()) == rk.RK_ERR_CAPACITY
    assert app(text(max_len=63, len=None)) == rk.RK_ERR_INVALID_ARG
    assert app(text(max_len=63), k=None) == rk.RK_ERR_INVALID_ARG
    assert app(None) == rk.RK_ERR_INVALID_ARG


def test_fused_step_validation(ctx):
    lay = layout()
    ws = rk.rk_decode_workspace_size(ctx, layout(max_seq_len=1001))
    # rk_append_decode_attn(ctx, L, k_new, v_new, q, R_r, delta_mu, k_packed, v_cache, seq_len, scale, out, ws)
    step = lambda **kw: status_of(rk.rk_append_decode_attn, ctx, kw.get("lay", lay), kw.get("k", PTR), kw.get("v", PTR),
                                  PTR, PTR, kw.get("dmu", PTR), PTR, PTR, kw.get("seq", PTR), 0.0, PTR, PTR,
                                  workspace_bytes=kw.get("ws", ws))
    assert step() == rk.RK_ERR_NO_DEVICE
    assert step(dmu=None) == rk.RK_ERR_NO_DEVICE                  # the bias is optional
    assert step(lay=layout(seq_len=None)) == rk.RK_ERR_NO_DEVICE  # the layout's seq_len is not used
    assert step(seq=None) == rk.RK_ERR_INVALID_ARG
    assert step(v=None) == rk.RK_ERR_INVALID_ARG
    assert step(k=PTR + 2) == rk.RK_ERR_INVALID_ARG               # k_new feeds 16-byte loads
    assert step(lay=layout(max_seq_len=1024)) == rk.RK_ERR_CAPACITY
    assert step(ws=ws - 1) == rk.RK_ERR_WORKSPACE
    # a workspace sized for the length after the append always suffices
    assert rk.rk_decode_workspace_size(ctx, layout(max_seq_len=1001)) >= rk.rk_decode_workspace_size(ctx, lay)
    ws = rk.rk_decode_workspace_size(ctx, lay)
    dual = lambda t, **kw: status_of(rk.rk_append_text_decode_attn_dual, ctx, lay, kw.get("k", PTR), kw.get("v", PTR), PTR,
                                     PTR, PTR, PTR, PTR, t, 0.0, PTR, PTR, workspace_bytes=kw.get("ws", ws))
    assert dual(text(max_len=63)) == rk.RK_ERR_NO_DEVICE
    assert dual(text()) == rk.RK_ERR_CAPACITY                     # 64 + 1 rows in a 64-row segment
    assert dual(text(max_len=63, len=None)) == rk.RK_ERR_INVALID_ARG
    assert dual(text(max_len=63), k=None) == rk.RK_ERR_INVALID_ARG
    assert dual(text(max_len=63), v=PTR + 8) == rk.RK_ERR_INVALID_ARG
    assert dual(None) == rk.RK_ERR_INVALID_ARG
    assert dual(text(max_len=63), ws=ws - 1) == rk.RK_ERR_WORKSPACE


def test_fit_subspace_validation(ctx):
    lay = layout()
    ws = rk.rk_fit_workspace_size(lay, 1000)
    call = lambda **kw: status_of(rk.rk_fit_subspace, ctx, kw.get("lay", lay), rows(), None, rk.RK_FIT_CENTER,
                                  kw.get("v0", PTR), kw.get("T", 5), kw.get("eps", 1e-6), kw.get("Rr", PTR), PTR, PTR,
                                  PTR, workspace_bytes=kw.get("ws", ws))
    assert call() == rk.RK_ERR_NO_DEVICE
    assert call(v0=None) == rk.RK_ERR_INVALID_ARG
    assert call(T=0) == rk.RK_ERR_INVALID_ARG
    assert call(eps=-1.0) == rk.RK_ERR_INVALID_ARG
    assert call(eps=float("nan")) == rk.RK_ERR_INVALID_ARG
    assert call(Rr=None) == rk.RK_ERR_INVALID_ARG
    assert call(ws=ws - 1) == rk.RK_ERR_WORKSPACE
    assert call(lay=layout(keep=104)) == rk.RK_ERR_NO_DEVICE
    assert call(lay=layout(keep=105)) == rk.RK_ERR_UNSUPPORTED


def test_query_sigma_validation(ctx):
    lay = layout()
    st = (8 * 32 * 128, 32 * 128, 128)
    call = lambda q=PTR, w=32, sg=PTR, strides=st: status_of(rk.rk_query_sigma, ctx, lay, q, w, sg, strides=strides)
    assert call() == rk.RK_ERR_NO_DEVICE
    assert call(q=None) == rk.RK_ERR_INVALID_ARG
    assert call(sg=None) == rk.RK_ERR_INVALID_ARG
    assert call(w=0) == rk.RK_ERR_INVALID_ARG
    assert call(strides=(8 * 32 * 128, 32 * 128, 64)) == rk.RK_ERR_INVALID_ARG


def test_product_does_not_import_oracle():
    """The product path must not route through the CPU oracle."""
    pkg = os.path.join(ROOT, "paper_2605_19218_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "rotatek_oracle" not in text, f


def test_c99_caller_builds_and_runs(tmp_path):
    """The header is C (not C++) and the library links into a plain C program: a C99 caller
    exercises the host-only entry points on a context without a device."""
    import shutil
    import subprocess
    cc = shutil.which("gcc") or shutil.which("cc")
    if cc is None:
        pytest.skip("no C compiler")
    root = ROOT
    libdir = os.path.dirname(rk.LIB_PATH)
    exe = str(tmp_path / "host_calls")
    subprocess.run([cc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(root, "include"),
                    os.path.join(root, "tests", "c_abi", "host_calls.c"), "-o", exe, "-L", libdir, "-lrotatek",
                    "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib"], check=True)
    res = subprocess.run([exe], capture_output=True, text=True, timeout=60)
    assert res.returncode == 0, (res.returncode, res.stdout, res.stderr)
    msg, n_splits, tokens, ws = res.stdout.strip().split("|")
    assert "device" in msg and int(n_splits) >= 1 and int(tokens) % 128 == 0
    c = rk.rk_create(rk.RK_DEVICE_NONE)
    try:
        assert int(ws) == rk.rk_decode_workspace_size(c, layout())
    finally:
        rk.rk_destroy(c)


def test_static_scratch_entry_validates_on_the_host(ctx):
    """rk_decode_attn_static: the same argument checks as rk_decode_attn, the size limit of the built-in
    scratch array, and only then the missing device."""
    call = lambda lay, q=PTR: status_of(rk.rk_decode_attn_static, ctx, lay, q, PTR, PTR, PTR, None, 0.0, PTR)
    assert call(layout()) == rk.RK_ERR_NO_DEVICE                     # valid, fits: only the device is missing
    assert call(layout(), q=PTR + 2) == rk.RK_ERR_INVALID_ARG        # misaligned query
    assert call(layout(max_seq_len=2048)) == rk.RK_ERR_CAPACITY
    big = layout(batch=4096, n_q_heads=64, n_kv_heads=64, capacity=1 << 16, max_seq_len=1 << 16)
    assert rk.rk_decode_workspace_size(ctx, big) > rk.RK_STATIC_SCRATCH_BYTES
    assert call(big) == rk.RK_ERR_WORKSPACE
    assert "scratch" in rk.lib().rk_last_error(ctx).decode()
    # the header's constant and the binding's agree
    text = open(os.path.join(ROOT, "include", "rotatek.h")).read()
    m = re.search(r"#define RK_STATIC_SCRATCH_BYTES \((\d+)u << (\d+)\)", text)
    assert m and int(m.group(1)) << int(m.group(2)) == rk.RK_STATIC_SCRATCH_BYTES

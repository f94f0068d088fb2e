"""Host-only checks of the C ABI: the library loads, exports every symbol the header declares,
and every argument error is reported before anything touches a GPU."""
import ctypes
import os
import re

import pytest

from paper_2602_05305_amd import flashblock as fb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", n) for n in sorted(os.listdir(os.path.join(ROOT, "include"))) if n.endswith(".h")]


def _declared():
    names = set()
    for h in HEADERS:
        text = re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S)
        names |= set(re.findall(r"\b(fb_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    lib = fb.load_library()
    names = _declared()
    assert {"fb_external_partial", "fb_internal_merge", "fb_sparse_external_residual"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(fb.exported_symbols())
    assert fb.fb_version() == 110
    for n in names:   # the binding offers the same names
        assert hasattr(fb, n) or n in ("fb_status_string", "fb_last_hip_error"), n


def test_struct_layout_matches_header():
    assert ctypes.sizeof(fb.fb_shape) == 36
    assert fb.fb_shape.scale.offset == 32


def _ok_shape(**kw):
    base = dict(batch=1, n_q_heads=4, n_kv_heads=2, head_dim=64, block_len=16, prefix_len=256, dtype="f32")
    base.update(kw)
    return fb.make_shape(**base)


@pytest.mark.parametrize("kw,status", [
    (dict(), fb.FB_OK),
    (dict(batch=0), fb.FB_ERR_SHAPE),
    (dict(n_q_heads=5), fb.FB_ERR_SHAPE),
    (dict(n_q_heads=66, n_kv_heads=2), fb.FB_ERR_SHAPE),
    (dict(block_len=0), fb.FB_ERR_SHAPE),
    (dict(prefix_len=-1), fb.FB_ERR_SHAPE),
    (dict(prefix_len=0), fb.FB_OK),
    (dict(head_dim=96), fb.FB_ERR_UNSUPPORTED),
    (dict(head_dim=0), fb.FB_ERR_SHAPE),
    (dict(dtype=7), fb.FB_ERR_DTYPE),
    (dict(scale=-1.0), fb.FB_ERR_SHAPE),
    (dict(scale=float("nan")), fb.FB_ERR_SHAPE),
    (dict(scale=float("inf")), fb.FB_ERR_SHAPE),
    (dict(dtype="bf16", head_dim=128), fb.FB_OK),
])
def test_check_shape(kw, status):
    assert fb.fb_check_shape(_ok_shape(**kw)) == status


def test_struct_size_is_checked():
    s = _ok_shape()
    s.struct_size = 8
    assert fb.fb_check_shape(s) == fb.FB_ERR_SHAPE
    assert fb.load_library().fb_check_shape(None) == fb.FB_ERR_NULL


def test_workspace_and_split_queries():
    s = _ok_shape()
    assert fb.fb_external_splits(s) >= 1
    assert fb.fb_workspace_bytes(s) >= 256
    assert fb.fb_workspace_bytes(s, 0, 0, 8) >= 8 * 64 * (64 + 2) * 4
    assert fb.fb_workspace_bytes(s, 64, 2) > fb.fb_workspace_bytes(s)
    assert fb.fb_workspace_bytes(s, 48, 2) == 0             # key_block not a multiple of 64
    assert fb.fb_workspace_bytes(s, 0, 0, 1000) == 0
    assert fb.fb_workspace_bytes(_ok_shape(batch=0)) == 0
    big = _ok_shape(dtype="bf16", head_dim=128, n_q_heads=32, n_kv_heads=8, block_len=32, prefix_len=131072)
    assert fb.fb_external_splits(big) == 32      # one 8-wavefront workgroup per CU: 256 CUs / 8 KV heads


TOO_SMALL = 256                      # below one split partial of _ok_shape (the general query also covers fb_refresh_step)
FAKE = ctypes.c_void_p(0x1000)       # aligned, never dereferenced: validation fails first
ODD = ctypes.c_void_p(0x1004)


def test_external_partial_error_paths():
    lib = fb.load_library()
    s = _ok_shape()
    ws_bytes = fb.fb_workspace_bytes(s)
    call = lib.fb_external_partial
    assert call(ctypes.byref(s), None, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, ws_bytes, None) == fb.FB_ERR_NULL
    assert call(ctypes.byref(s), FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE, ws_bytes, None) == fb.FB_ERR_NULL
    assert call(ctypes.byref(s), FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, ws_bytes, None) == fb.FB_ERR_NULL
    assert call(ctypes.byref(s), ODD, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, ws_bytes, None) == fb.FB_ERR_ALIGN
    assert call(ctypes.byref(s), FAKE, FAKE, FAKE, FAKE, FAKE, ODD, FAKE, ws_bytes, None) == fb.FB_ERR_ALIGN
    assert call(ctypes.byref(s), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, ws_bytes, None) == fb.FB_ERR_WORKSPACE
    assert call(ctypes.byref(s), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, TOO_SMALL, None) == fb.FB_ERR_WORKSPACE
    bad = _ok_shape(head_dim=96)
    assert call(ctypes.byref(bad), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, ws_bytes, None) == fb.FB_ERR_UNSUPPORTED
    ex = lib.fb_external_partial_ex
    assert ex(ctypes.byref(s), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 257, FAKE, 1 << 30, None) == fb.FB_ERR_SHAPE
    assert ex(ctypes.byref(s), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, -1, FAKE, 1 << 30, None) == fb.FB_ERR_SHAPE
    assert ex(ctypes.byref(s), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 16, FAKE, TOO_SMALL, None) in (
        fb.FB_ERR_WORKSPACE,)


def test_external_partial_heads_error_paths():
    lib = fb.load_library()
    s = _ok_shape()
    ws_bytes = fb.fb_workspace_bytes(s)
    call = lib.fb_external_partial_heads
    assert call(ctypes.byref(s), FAKE, FAKE, FAKE, None, 0, FAKE, FAKE, FAKE, FAKE, ws_bytes, None) == fb.FB_ERR_NULL
    assert call(ctypes.byref(s), FAKE, FAKE, FAKE, FAKE, 0, FAKE, FAKE, FAKE, FAKE, TOO_SMALL, None) == fb.FB_ERR_WORKSPACE
    assert call(ctypes.byref(s), FAKE, FAKE, FAKE, ODD, 0, ODD, FAKE, FAKE, FAKE, ws_bytes, None) == fb.FB_ERR_ALIGN  # mask may be unaligned, o may not
    assert call(ctypes.byref(s), FAKE, FAKE, FAKE, FAKE, -1, FAKE, FAKE, FAKE, FAKE, ws_bytes, None) == fb.FB_ERR_SHAPE
    # the hint changes the split count where few heads leave the GPU underfilled
    video = _ok_shape(dtype="bf16", head_dim=128, n_q_heads=12, n_kv_heads=12, block_len=4680, prefix_len=37440)
    assert fb.fb_external_heads_splits(video, 0) == fb.fb_external_splits(video) == 1
    assert fb.fb_external_heads_splits(video, 12) == 1
    assert fb.fb_external_heads_splits(video, 6) == 1            # 222 workgroups: one round either way
    assert fb.fb_external_heads_splits(video, 3) == 2
    assert fb.fb_external_heads_splits(video, 1) == 6            # 37 row tiles x 6 = 222 workgroups, one round
    assert fb.fb_external_heads_splits(video, -1) == 0


def _paged(**kw):
    base = dict(struct_size=ctypes.sizeof(fb.fb_paged_kv), num_pages=8, page_size=64, max_pages=4,
                k_pool=0x1000, v_pool=0x1000, block_table=0x1000, prefix_lens=0x1000)
    base.update(kw)
    return fb.fb_paged_kv(**base)


def test_external_partial_paged_error_paths():
    lib = fb.load_library()
    s = _ok_shape()                       # prefix_len 256 = 4 pages of 64
    ws_bytes = fb.fb_workspace_bytes(s, 0, 0, fb.fb_paged_splits(s))
    call = lib.fb_external_partial_paged
    tail = (FAKE, FAKE, FAKE, 0, FAKE, ws_bytes, None)
    assert ctypes.sizeof(fb.fb_paged_kv) == 48
    assert call(ctypes.byref(s), FAKE, None, *tail) == fb.FB_ERR_NULL
    assert call(ctypes.byref(s), None, ctypes.byref(_paged()), *tail) == fb.FB_ERR_NULL
    assert call(ctypes.byref(s), FAKE, ctypes.byref(_paged(struct_size=40)), *tail) == fb.FB_ERR_SHAPE
    assert call(ctypes.byref(s), FAKE, ctypes.byref(_paged(block_table=None)), *tail) == fb.FB_ERR_NULL
    assert call(ctypes.byref(s), FAKE, ctypes.byref(_paged(prefix_lens=None)), *tail) == fb.FB_ERR_NULL
    assert call(ctypes.byref(s), FAKE, ctypes.byref(_paged(k_pool=None)), *tail) == fb.FB_ERR_NULL
    assert call(ctypes.byref(s), FAKE, ctypes.byref(_paged(page_size=96)), *tail) == fb.FB_ERR_UNSUPPORTED
    assert call(ctypes.byref(s), FAKE, ctypes.byref(_paged(page_size=0)), *tail) == fb.FB_ERR_SHAPE
    assert call(ctypes.byref(s), FAKE, ctypes.byref(_paged(num_pages=0)), *tail) == fb.FB_ERR_SHAPE
    assert call(ctypes.byref(s), FAKE, ctypes.byref(_paged(max_pages=3)), *tail) == fb.FB_ERR_SHAPE   # 3*64 < 256
    assert call(ctypes.byref(s), FAKE, ctypes.byref(_paged(v_pool=0x1004)), *tail) == fb.FB_ERR_ALIGN
    assert call(ctypes.byref(s), FAKE, ctypes.byref(_paged()), FAKE, FAKE, FAKE, 0, FAKE, TOO_SMALL, None) == fb.FB_ERR_WORKSPACE
    assert call(ctypes.byref(s), FAKE, ctypes.byref(_paged()), FAKE, FAKE, FAKE, 300, FAKE, 1 << 30, None) == fb.FB_ERR_SHAPE


def test_internal_merge_error_paths():
    lib = fb.load_library()
    s = _ok_shape()
    call = lib.fb_internal_merge
    assert call(ctypes.byref(s), None, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, None) == fb.FB_ERR_NULL
    assert call(ctypes.byref(s), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, None, None) == fb.FB_ERR_NULL
    assert call(ctypes.byref(s), FAKE, FAKE, FAKE, FAKE, None, FAKE, FAKE, None, None) == fb.FB_ERR_NULL  # 2 of 3
    assert call(ctypes.byref(s), FAKE, FAKE, ODD, FAKE, FAKE, FAKE, FAKE, None, None) == fb.FB_ERR_ALIGN
    assert call(ctypes.byref(s), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, ODD, None) == fb.FB_ERR_ALIGN


def test_refresh_step_error_paths():
    lib = fb.load_library()
    s = _ok_shape()
    ws_bytes = fb.fb_workspace_bytes(s)
    call = lib.fb_refresh_step
    ok = [FAKE] * 9 + [None, FAKE, ws_bytes, None]       # q kp vp kb vb o m lse out | lse_out ws bytes stream
    for i in (0, 3, 4, 5, 6, 7, 8):
        a = list(ok); a[i] = None
        assert call(ctypes.byref(s), *a) == fb.FB_ERR_NULL, i
    a = list(ok); a[1] = None
    assert call(ctypes.byref(s), *a) == fb.FB_ERR_NULL                       # prefix_len > 0 needs k_prefix
    a = list(ok); a[8] = ODD
    assert call(ctypes.byref(s), *a) == fb.FB_ERR_ALIGN
    a = list(ok); a[10] = None
    assert call(ctypes.byref(s), *a) == fb.FB_ERR_WORKSPACE
    a = list(ok); a[11] = ws_bytes - 1
    assert call(ctypes.byref(s), *a) == fb.FB_ERR_WORKSPACE
    assert call(ctypes.byref(_ok_shape(head_dim=96)), *ok) == fb.FB_ERR_UNSUPPORTED


def test_sparse_error_paths():
    lib = fb.load_library()
    s = _ok_shape()
    ws_bytes = fb.fb_workspace_bytes(s, 64, 2)
    call = lib.fb_sparse_external_residual
    args = [FAKE] * 3 + [64, 2, FAKE] + [FAKE] * 6 + [FAKE, ws_bytes, None]
    assert call(ctypes.byref(s), 3, *args) == fb.FB_ERR_SHAPE                       # bad mode
    a = list(args); a[5] = None; a[13] = TOO_SMALL
    assert call(ctypes.byref(s), 2, *a) == fb.FB_ERR_WORKSPACE                      # same-selection reuse takes no sel_idx
    a = list(args); a[3] = 48
    assert call(ctypes.byref(s), 0, *a) == fb.FB_ERR_UNSUPPORTED                    # key_block % 64
    a = list(args); a[3] = 0
    assert call(ctypes.byref(s), 0, *a) == fb.FB_ERR_SHAPE
    a = list(args); a[4] = -1
    assert call(ctypes.byref(s), 0, *a) == fb.FB_ERR_SHAPE
    a = list(args); a[5] = None
    assert call(ctypes.byref(s), 0, *a) == fb.FB_ERR_NULL                           # topk > 0 needs idx
    a = list(args); a[6] = None
    assert call(ctypes.byref(s), 1, *a) == fb.FB_ERR_NULL
    a = list(args); a[13] = ws_bytes - 1
    assert call(ctypes.byref(s), 0, *a) == fb.FB_ERR_WORKSPACE
    a = list(args); a[0] = ODD
    assert call(ctypes.byref(s), 0, *a) == fb.FB_ERR_ALIGN
    assert lib.fb_pool_keys(ctypes.byref(s), FAKE, 32, FAKE, None) == fb.FB_ERR_UNSUPPORTED
    assert lib.fb_pool_keys(ctypes.byref(s), None, 64, FAKE, None) == fb.FB_ERR_NULL
    assert lib.fb_select_topk(ctypes.byref(s), None, FAKE, 64, 2, FAKE, None, 0, None) == fb.FB_ERR_NULL
    assert lib.fb_select_topk(ctypes.byref(s), FAKE, FAKE, 64, 2, ODD, None, 0, None) == fb.FB_ERR_ALIGN
    n = fb.fb_select_workspace_bytes(s, 64)
    heads = s.batch * s.n_q_heads
    assert n >= heads * (s.head_dim + -(-s.prefix_len // 64)) * 4 and n % 256 == 0
    assert fb.fb_select_workspace_bytes(s, 48) == 0
    assert lib.fb_select_topk(ctypes.byref(s), FAKE, FAKE, 64, 2, FAKE, FAKE, n - 1, None) == fb.FB_ERR_WORKSPACE
    assert lib.fb_select_topk(ctypes.byref(s), FAKE, FAKE, 64, 2, FAKE, ODD, n, None) == fb.FB_ERR_ALIGN
    huge = _ok_shape(prefix_len=64 * 16385)
    assert lib.fb_pool_keys(ctypes.byref(huge), FAKE, 64, FAKE, None) == fb.FB_ERR_UNSUPPORTED


def test_select_topk_mass_error_paths():
    lib = fb.load_library()
    s = _ok_shape()
    n = fb.fb_select_mass_workspace_bytes(s, 64)
    assert n >= 64 * 4 * 4                           # 64 rows x 4 key blocks, floats
    assert fb.fb_select_mass_workspace_bytes(s, 48) == 0
    assert fb.fb_select_mass_workspace_bytes(_ok_shape(batch=0), 64) == 0
    call = lib.fb_select_topk_mass
    ok = [FAKE, FAKE, FAKE, 64, 2, FAKE, None, FAKE, n, None]     # q k lse key_block topk idx mass ws bytes stream
    for i in (0, 1, 2, 5):
        a = list(ok); a[i] = None
        assert call(ctypes.byref(s), *a) == fb.FB_ERR_NULL, i
    a = list(ok); a[3] = 48
    assert call(ctypes.byref(s), *a) == fb.FB_ERR_UNSUPPORTED
    a = list(ok); a[4] = -1
    assert call(ctypes.byref(s), *a) == fb.FB_ERR_SHAPE
    a = list(ok); a[4] = 0
    assert call(ctypes.byref(s), *a) == fb.FB_OK                  # nothing to select, nothing launched
    a = list(ok); a[6] = ODD
    assert call(ctypes.byref(s), *a) == fb.FB_ERR_ALIGN
    a = list(ok); a[7] = None
    assert call(ctypes.byref(s), *a) == fb.FB_ERR_WORKSPACE
    a = list(ok); a[8] = n - 1
    assert call(ctypes.byref(s), *a) == fb.FB_ERR_WORKSPACE
    assert call(ctypes.byref(_ok_shape(prefix_len=0)), *ok) == fb.FB_OK


def test_status_strings():
    lib = fb.load_library()
    seen = {lib.fb_status_string(i).decode() for i in range(8)}
    assert len(seen) == 8 and all(s.startswith("FB_") for s in seen)
    assert lib.fb_status_string(99).decode().startswith("unknown")


def test_binding_has_no_cpu_fallback(monkeypatch, tmp_path):
    monkeypatch.setattr(fb, "_lib", None)
    monkeypatch.setattr(fb, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        fb.load_library()


def test_bench_refuses_more_than_one_gpu():
    """This build has no multi-GPU part: bench.py --gpus N > 1 exits with a message (before touching any GPU)."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=60, cwd=ROOT)
    assert r.returncode != 0 and "one GPU" in r.stderr


def test_header_is_plain_c_and_links(tmp_path):
    """include/flashblock.h is a C header (C99, no C++ needed) and a C program links against the library."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    src = tmp_path / "use.c"
    src.write_text('#include "flashblock.h"\n#include <stdio.h>\n'
                   "int main(void) {\n"
                   "  fb_shape s = {sizeof(fb_shape), 1, 4, 2, 64, 16, 256, FB_F32, 0.0f};\n"
                   "  fb_paged_kv kv; kv.struct_size = sizeof kv; (void)kv;\n"
                   '  printf("%d %d %d %zu\\n", fb_version(), (int)fb_check_shape(&s), (int)fb_external_splits(&s),\n'
                   "         fb_workspace_bytes(&s, 0, 0, 0));\n"
                   "  return 0;\n}\n")
    exe = tmp_path / "use"
    libdir = os.path.dirname(fb.LIB_PATH)
    r = subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src),
                        "-o", str(exe), "-L", libdir, "-l:libflashblock.so", f"-Wl,-rpath,{libdir}",
                        "-Wl,-rpath,/opt/rocm/lib", "-L/opt/rocm/lib"], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=60)
    assert out.returncode == 0, out.stderr
    ver, ok, splits, ws = out.stdout.split()
    assert int(ver) == 110 and int(ok) == fb.FB_OK and int(splits) >= 1 and int(ws) >= 256


def test_builtin_workspace_entry_rejects_on_the_host():
    """The entry point for callers that cannot allocate: size and argument checks come before any HIP call."""
    assert fb.fb_builtin_workspace_bytes() == 20 * 1024 * 1024
    lib = fb.load_library()
    video = fb.make_shape(1, 12, 12, 128, 4680, 37440, "bf16")
    one = ctypes.c_void_p(16)
    assert lib.fb_external_partial_builtin_ws(ctypes.byref(video), one, one, one, one, one, one, None) == fb.FB_ERR_WORKSPACE
    small = fb.make_shape(1, 4, 4, 64, 16, 256, "f32")
    assert lib.fb_external_partial_builtin_ws(ctypes.byref(small), None, one, one, one, one, one, None) == fb.FB_ERR_NULL
    bad = fb.make_shape(1, 4, 3, 64, 16, 256, "f32")
    assert lib.fb_external_partial_builtin_ws(ctypes.byref(bad), one, one, one, one, one, one, None) == fb.FB_ERR_SHAPE


def test_external_kernel_name_follows_the_launch_rules():
    """Host-only query the benchmark labels its roofline with: streaming kernel (with 1, 2 or 4 row groups per workgroup) for up
    to 128 rows per KV group and at least 8 tiles per split, register-staged kernel for short prefixes, fp32 kernel for fp32."""
    name = lambda *a: fb.fb_external_kernel_name(fb.make_shape(*a))
    assert name(1, 32, 8, 128, 32, 32768, "bf16") == "attn_stream_kernel<128, 0, 0, 4>"       # 128 rows per KV group
    assert name(1, 32, 8, 128, 16, 32768, "bf16") == "attn_stream_kernel<128, 0, 0, 2>"       # 64 rows
    assert name(1, 32, 8, 128, 8, 131072, "bf16") == "attn_stream_kernel<128, 0, 0, 1>"       # 32 rows
    assert name(1, 12, 12, 128, 4680, 37440, "bf16") == "attn_stream_kernel<128, 0, 2, 4>"    # row-pair layout
    assert name(1, 32, 8, 128, 8, 4096, "bf16").startswith("attn_bf16_kernel<128, 0, 64, 4, ")  # short prefix: register-staged
    assert name(1, 32, 8, 64, 32, 32768, "bf16") == "attn_stream_kernel<64, 0, 0, 4>"
    assert name(1, 4, 4, 64, 16, 256, "f32") == "attn_f32_kernel<64, 0>"
    bad = fb.make_shape(1, 4, 3, 64, 16, 256, "f32")
    assert fb.fb_external_kernel_name(bad) == ""

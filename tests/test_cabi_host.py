"""Host side of the C ABI: the library loads, exports what include/wkv.h declares, validates
its arguments before touching a GPU and computes derived sizes.  No compute calls; CPU only."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2503_17922_amd as W
from oracle import wkv_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _problem(**kw):
    base = dict(n_q_heads=32, n_kv_heads=8, head_dim=128, w_obs=32, seq_len=[4096], win=[8], top_p=[8],
                k_windows=[64], dtype=W.WKV_BF16)
    base.update(kw)
    return W.Problem(**base)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "wkv.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(wkv_[a-z_]+)\s*\(", header))
    assert declared == set(W.EXPORTS)
    lib = W.lib()
    for name in declared:
        assert getattr(lib, name) is not None


def test_dims_of_the_named_configurations():
    import wkv_synth as S
    want = {"c1": (16, 504, 63, 8, 72), "c2": (128, 4064, 508, 64, 544), "c3a": (128, 16352, 2044, 256, 2080),
            "c3b": (128, 16352, 511, 64, 2080), "c4": (128, 32736, 2046, 256, 4128)}
    for name, (rows, ts, nw, km, nk) in want.items():
        w = S.make_workload(name)
        p = W.Problem(n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, w_obs=w.w_obs,
                      seq_len=w.seq_len, win=w.win, top_p=w.top_p, k_windows=w.k_windows,
                      dtype=W.WKV_F32 if w.dtype == "f32" else W.WKV_BF16)
        d = W.wkv_get_dims(p)
        assert (d.obs_rows, d.t_stride, d.nw_max, d.k_max, d.nkeep_max) == (rows, ts, nw, km, nk)
        assert d.total_tokens == sum(w.seq_len)
        assert W.wkv_workspace_bytes(p, w.n_groups) % 256 == 0
    w = S.make_workload("c5")
    p = W.Problem(n_q_heads=32, n_kv_heads=8, head_dim=128, w_obs=32, seq_len=w.seq_len, win=w.win,
                  top_p=w.top_p, k_windows=w.k_windows, dtype=W.WKV_BF16)
    d = W.wkv_get_dims(p)
    assert d.nw_max == max(w.n_windows(b) for b in range(8)) and d.nkeep_max == w.nkeep_max
    assert d.total_tokens == sum(w.seq_len)


@pytest.mark.parametrize("kw,status", [
    (dict(n_q_heads=30), W.WKV_ERR_INVALID_ARG),
    (dict(head_dim=96), W.WKV_ERR_UNSUPPORTED),
    (dict(w_obs=0), W.WKV_ERR_INVALID_ARG),
    (dict(seq_len=[16]), W.WKV_ERR_INVALID_ARG),                 # shorter than w_obs
    (dict(seq_len=[5000], max_seq_len=4096), W.WKV_ERR_INVALID_ARG),
    (dict(win=[0]), W.WKV_ERR_INVALID_ARG),
    (dict(win=[256]), W.WKV_ERR_UNSUPPORTED),
    (dict(top_p=[0]), W.WKV_ERR_INVALID_ARG),
    (dict(k_windows=[509]), W.WKV_ERR_INVALID_ARG),              # NW = 508
    (dict(k_windows=[-1]), W.WKV_ERR_INVALID_ARG),
    (dict(dtype=7), W.WKV_ERR_INVALID_ARG),
    (dict(scale=-1.0), W.WKV_ERR_INVALID_ARG),
    (dict(scale=float("nan")), W.WKV_ERR_INVALID_ARG),
    (dict(w_obs=128, seq_len=[4096]), W.WKV_ERR_UNSUPPORTED),    # 4*128 rows > 256
    (dict(seq_len=[4096] * 65, win=[8] * 65, top_p=[8] * 65, k_windows=[1] * 65), W.WKV_ERR_UNSUPPORTED),
    (dict(kv_strides=(8 * 4096 * 128, 4096 * 128, 100)), W.WKV_ERR_INVALID_ARG),
    (dict(kv_strides=(8 * 4096 * 132, 4096 * 132, 132)), W.WKV_ERR_INVALID_ARG),   # not 16-byte rows
    (dict(seq_len=[300000], win=[8], k_windows=[1]), W.WKV_ERR_UNSUPPORTED),       # too many windows
    (dict(flags=64), W.WKV_ERR_INVALID_ARG),                                       # unknown flag bit
    (dict(flags=W.WKV_SCORE_TWO_PASS | W.WKV_SCORE_SINGLE_READ), W.WKV_ERR_INVALID_ARG),   # they exclude each other
])
def test_invalid_problems_are_rejected_on_the_host(kw, status):
    with pytest.raises(W.WkvError) as e:
        W.wkv_get_dims(_problem(**kw))
    assert e.value.status == status
    assert len(str(e.value)) > 20


def test_half_precision_dtypes_share_limits_and_sizes():
    a, b = W.wkv_get_dims(_problem(dtype=W.WKV_F16)), W.wkv_get_dims(_problem(dtype=W.WKV_BF16))
    assert (a.obs_rows, a.nw_max, a.k_max, a.nkeep_max) == (b.obs_rows, b.nw_max, b.k_max, b.nkeep_max)
    assert W.wkv_workspace_bytes(_problem(dtype=W.WKV_F16), 3) == W.wkv_workspace_bytes(_problem(dtype=W.WKV_BF16), 3)
    with pytest.raises(W.WkvError):                      # rows of 2-byte elements need strides in units of 8
        W.wkv_get_dims(_problem(dtype=W.WKV_F16, kv_strides=(8 * 4096 * 132, 4096 * 132, 132)))


def test_known_flags_are_accepted():
    assert W.wkv_get_dims(_problem(flags=W.WKV_KEEP_PADDING)).nkeep_max == W.wkv_get_dims(_problem()).nkeep_max


def test_stage_calls_validate_before_any_launch():
    # null tensors / workspace are caught on the host: safe to call without a GPU
    lib = W.lib()
    p = _problem()
    null = C.c_void_p(0)
    assert lib.wkv_score(p.ref(), null, null, null, null, null, 0, null) == W.WKV_ERR_INVALID_ARG
    assert lib.wkv_window_pool(p.ref(), null, null, null) == W.WKV_ERR_INVALID_ARG
    assert lib.wkv_topk_windows(p.ref(), null, null, null, null, null) == W.WKV_ERR_INVALID_ARG
    assert lib.wkv_gather_group(p.ref(), 1, None, None, null, null, None, None, null) == W.WKV_ERR_INVALID_ARG
    assert lib.wkv_get_dims(None, None) == W.WKV_ERR_INVALID_ARG
    fake = C.c_void_p(4096)      # aligned, non-null, never dereferenced on these paths
    assert lib.wkv_score(p.ref(), fake, fake, null, fake, null, 0, null) == W.WKV_ERR_WORKSPACE
    assert lib.wkv_score(p.ref(), fake, fake, null, fake, C.c_void_p(4096 + 64), 1 << 30, null) == W.WKV_ERR_WORKSPACE
    assert lib.wkv_score(p.ref(), fake, fake, fake, fake, fake, 16, null) == W.WKV_ERR_WORKSPACE
    assert b"needed" in lib.wkv_last_error()
    assert lib.wkv_score(p.ref(), C.c_void_p(4100), fake, null, fake, fake, 1 << 30, null) == W.WKV_ERR_INVALID_ARG
    assert lib.wkv_score(p.ref(), fake, fake, C.c_void_p(4098), fake, fake, 1 << 30, null) == W.WKV_ERR_INVALID_ARG
    arr = (C.c_void_p * 1)(4096)
    assert lib.wkv_gather_group(p.ref(), 0, arr, arr, fake, fake, arr, arr, null) == W.WKV_ERR_INVALID_ARG
    assert lib.wkv_gather_group(p.ref(), 65, arr, arr, fake, fake, arr, arr, null) == W.WKV_ERR_INVALID_ARG
    assert lib.wkv_compress_groups(p.ref(), 8, 9, arr, None, None, arr, arr, arr, arr, fake, fake, fake, fake, 1 << 30,
                                   null) == W.WKV_ERR_INVALID_ARG


def test_per_group_budgets_are_validated_on_the_host():
    # k_windows_groups: every entry within [0, k_windows[b]] (the capacity); caught before any launch
    lib = W.lib()
    p = _problem(seq_len=[4096, 2048], win=[8, 8], top_p=[8, 8], k_windows=[64, 32])
    null, fake = C.c_void_p(0), C.c_void_p(4096)
    arr = (C.c_void_p * 2)(4096, 4096)

    def call(ks):
        kg = (C.c_int32 * len(ks))(*ks)
        return lib.wkv_compress_groups(p.ref(), 2, 1, arr, None, kg, arr, arr, arr, arr, fake, fake, fake, null, 0, null)

    assert call([64, 32, 65, 0]) == W.WKV_ERR_INVALID_ARG and b"k_windows_groups[1][0]" in lib.wkv_last_error()
    assert call([64, 33, 1, 1]) == W.WKV_ERR_INVALID_ARG
    assert call([0, -1, 1, 1]) == W.WKV_ERR_INVALID_ARG
    assert call([64, 32, 0, 7]) == W.WKV_ERR_WORKSPACE      # the budgets pass; the missing workspace is next


def test_decode_shape_validation_and_workspace():
    lib = W.lib()
    ok = dict(batch=2, n_q_heads=32, n_kv_heads=8, head_dim=128, dtype=W.WKV_BF16, capacity=4160)
    n = W.wkv_decode_workspace_bytes(W.DecodeShape(**ok))
    assert n > 0 and n % (4 * (128 + 2)) == 0            # [rows][splits][G][d + 2] floats
    for bad, status in ((dict(n_q_heads=30), W.WKV_ERR_INVALID_ARG), (dict(head_dim=96), W.WKV_ERR_UNSUPPORTED),
                        (dict(n_q_heads=72), W.WKV_ERR_UNSUPPORTED), (dict(capacity=0), W.WKV_ERR_INVALID_ARG),
                        (dict(dtype=5), W.WKV_ERR_INVALID_ARG), (dict(cache_strides=(4160 * 128 * 8, 4160 * 128, 100)), W.WKV_ERR_INVALID_ARG),
                        (dict(scale=-1.0), W.WKV_ERR_INVALID_ARG)):
        kw = dict(ok); kw.update(bad)
        sh = W.DecodeShape(**kw)
        assert lib.wkv_decode_workspace_bytes(sh.ref()) == 0
        null, fake = C.c_void_p(0), C.c_void_p(4096)
        assert lib.wkv_decode_step(sh.ref(), fake, fake, fake, fake, fake, fake, fake, fake, 1 << 30, null) == status
    sh = W.DecodeShape(**ok)
    null, fake = C.c_void_p(0), C.c_void_p(4096)
    assert lib.wkv_decode_step(sh.ref(), fake, fake, fake, fake, fake, fake, null, fake, 1 << 30, null) == W.WKV_ERR_INVALID_ARG
    assert lib.wkv_decode_step(sh.ref(), fake, C.c_void_p(4104), fake, fake, fake, fake, fake, fake, 1 << 30, null) == W.WKV_ERR_INVALID_ARG
    assert lib.wkv_decode_step(sh.ref(), fake, fake, fake, fake, fake, fake, fake, null, 0, null) == W.WKV_ERR_WORKSPACE
    assert lib.wkv_decode_step(sh.ref(), fake, fake, fake, fake, fake, fake, fake, fake, 64, null) == W.WKV_ERR_WORKSPACE


def test_status_strings():
    lib = W.lib()
    seen = {lib.wkv_status_string(s).decode() for s in (0, -1, -2, -3, -4)}
    assert len(seen) == 5 and all(seen)


@pytest.mark.parametrize("H,lam,total", [(4, 14.0, 8192.0), (8, 14.0, 32768.0), (1, 14.0, 100.0), (7, 3.0, 1e3)])
def test_group_budgets_match_eq_5_to_7(H, lam, total):
    got = W.wkv_group_budgets(total, H, lam)
    np.testing.assert_allclose(got, O.group_budgets(total, H, lam), rtol=1e-14)
    assert sum(got) == pytest.approx(total, rel=1e-13)
    with pytest.raises(W.WkvError):
        W.wkv_group_budgets(total, 0, lam)
    with pytest.raises(W.WkvError):
        W.wkv_group_budgets(total, H, 0.0)


def test_header_is_c99_and_library_links_from_c(tmp_path):
    # include/wkv.h compiled by gcc as pedantic C99; the program calls the host-only entry points
    import shutil, subprocess, os
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    W.lib()
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    libdir = os.path.dirname(W.LIB_PATH)
    exe = str(tmp_path / "cabi_host")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(root, "include"),
                    os.path.join(root, "tests", "c", "cabi_host.c"), "-L", libdir, "-lwkv", f"-Wl,-rpath,{libdir}",
                    "-Wl,-rpath,/opt/rocm/lib", "-o", exe], check=True)
    out = subprocess.run([exe], check=True, capture_output=True, text=True).stdout.split()
    d = W.wkv_get_dims(_problem())
    assert out[:5] == ["0", str(d.obs_rows), str(d.nw_max), str(d.k_max), str(d.nkeep_max)]
    assert int(out[5]) == W.wkv_workspace_bytes(_problem(), 1) and out[6] == "ok"


def test_host_side_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """The validation / sizing / planning code of the library, built for the CPU with ASan + UBSan and
    driven through every entry point with valid and invalid arguments (tests/c/cabi_validation.cpp;
    the kernel launchers are replaced by stand-ins, so no GPU is involved)."""
    import subprocess
    from paper_2503_17922_amd import build as B
    exe = B.build_host_sanitized(str(tmp_path), [os.path.join(ROOT, "tests", "c", "cabi_validation.cpp"),
                                                 os.path.join(ROOT, "tests", "c", "launch_stubs.cpp")])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)          # the sanitizer runtime must come first in the link order of the process
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-4000:]
    assert res.stdout.strip().endswith("ok (0 checks failed)")

"""CPU-only checks of the C ABI: the library loads, exports every declared symbol, and
rejects bad arguments on the host before launching anything."""
import ctypes
import os
import re

import pytest

from paper_2510_07651_amd import binding as obc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return obc.load_library()


def test_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "obcache.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(obc_[a-z_]+)\s*\(", header))
    assert {"obc_score", "obc_select", "obc_compact", "obc_score_workspace_bytes", "obc_status_string",
            "obc_version"} <= names
    for n in names:
        assert hasattr(lib, n), n
    assert obc.obc_version() >= 100


def test_status_strings(lib):
    assert obc.obc_status_string(0) == "OBC_OK"
    for code in (-1, -2, -3, -4):
        assert obc.obc_status_string(code).startswith("OBC_E")
    assert "unknown" in obc.obc_status_string(-99)


def test_workspace_query_validation():
    assert obc.obc_score_workspace_bytes(1, 512, 16, 1, 1, 64, obc.OBC_F32, obc.OBC_ALL) % 256 == 0
    big = obc.obc_score_workspace_bytes(4, 32768, 32, 32, 8, 128, obc.OBC_BF16, obc.OBC_JOINT)
    assert 0 < big < (1 << 30)
    # one-row windows: short caches plan the decode kernels' buffers (logits of G rows per head-token, range records),
    # long ones the matrix-core path's; head_dim 64 and 8 query heads per KV head are served, fp32 goes the plain way
    for args in ((1, 1025, 1, 32, 8, 128, obc.OBC_BF16, obc.OBC_JOINT), (4, 1025, 1, 28, 4, 128, obc.OBC_BF16, obc.OBC_ALL),
                 (1, 131072, 1, 32, 8, 128, obc.OBC_BF16, obc.OBC_JOINT), (2, 3000, 1, 8, 1, 64, obc.OBC_BF16, obc.OBC_VALUE),
                 (1, 1 << 21, 1, 8, 8, 64, obc.OBC_BF16, obc.OBC_KEY), (1, 1025, 1, 32, 8, 128, obc.OBC_F32, obc.OBC_JOINT)):
        need = obc.obc_score_workspace_bytes(*args)
        assert need > 0 and need % 256 == 0, args
    short = obc.obc_score_workspace_bytes(1, 1025, 1, 32, 8, 128, obc.OBC_BF16, obc.OBC_JOINT)
    assert short >= 8 * 1025 * 4 * 4                     # the stored logits alone
    bad = [
        (1, 512, 16, 3, 2, 64, obc.OBC_F32, obc.OBC_ALL, obc.OBC_EINVAL),        # Hq % Hkv != 0
        (1, 8, 16, 1, 1, 64, obc.OBC_F32, obc.OBC_ALL, obc.OBC_EINVAL),          # W > N
        (0, 512, 16, 1, 1, 64, obc.OBC_F32, obc.OBC_ALL, obc.OBC_EINVAL),        # B < 1
        (1, 512, 16, 1, 1, 64, obc.OBC_F32, 7, obc.OBC_EINVAL),                  # variant
        (1, 512, 16, 1, 1, 96, obc.OBC_F32, obc.OBC_ALL, obc.OBC_EUNSUPPORTED),  # head_dim
        (1, 512, 16, 1, 1, 64, 5, obc.OBC_ALL, obc.OBC_EUNSUPPORTED),            # dtype
        (1, 512, 65, 1, 1, 64, obc.OBC_F32, obc.OBC_ALL, obc.OBC_EUNSUPPORTED),  # window too long
        (1, 512, 64, 16, 1, 64, obc.OBC_F32, obc.OBC_ALL, obc.OBC_EUNSUPPORTED), # G*W too large
    ]
    for *args, expect in bad:
        with pytest.raises(obc.ObcError) as e:
            obc.obc_score_workspace_bytes(*args)
        assert e.value.status == expect, args


def test_entry_points_reject_bad_arguments_before_launch(lib):
    """Null pointers, bad lengths and missing workspace return error codes on a box with no GPU."""
    fake = ctypes.c_void_p(4096)          # never dereferenced: validation fails first
    lens = (ctypes.c_int32 * 2)(100, 5)
    sc = lib.obc_score
    assert sc(None, fake, fake, 512, 16, 1, 1, 64, 2, fake, 1, 0, None, fake, 1 << 30, None) == obc.OBC_EINVAL
    assert sc(fake, fake, fake, 512, 16, 1, 1, 64, 2, None, 1, 0, None, fake, 1 << 30, None) == obc.OBC_EINVAL
    odd = ctypes.c_void_p(4104)           # 8-byte aligned only
    assert sc(fake, odd, fake, 512, 16, 1, 1, 64, 2, fake, 1, 0, None, fake, 1 << 30, None) == obc.OBC_EINVAL
    # W > len_b for the second sequence
    assert sc(fake, fake, fake, 512, 16, 1, 1, 64, 2, fake, 2, 0, lens, fake, 1 << 30, None) == obc.OBC_EINVAL
    # len_b > N
    lens2 = (ctypes.c_int32 * 1)(600)
    assert sc(fake, fake, fake, 512, 16, 1, 1, 64, 2, fake, 1, 0, lens2, fake, 1 << 30, None) == obc.OBC_EINVAL
    # workspace: null, misaligned, too small
    assert sc(fake, fake, fake, 512, 16, 1, 1, 64, 2, fake, 1, 0, None, None, 1 << 30, None) == obc.OBC_EWORKSPACE
    assert sc(fake, fake, fake, 512, 16, 1, 1, 64, 2, fake, 1, 0, None, ctypes.c_void_p(4100), 1 << 30,
              None) == obc.OBC_EWORKSPACE
    assert sc(fake, fake, fake, 512, 16, 1, 1, 64, 2, fake, 1, 0, None, fake, 16, None) == obc.OBC_EWORKSPACE
    # ragged batch larger than the by-value table
    many = (ctypes.c_int32 * 200)(*([512] * 200))
    assert sc(fake, fake, fake, 512, 16, 1, 1, 64, 2, fake, 200, 0, many, fake, 1 << 40, None) == obc.OBC_EUNSUPPORTED

    sel = lib.obc_select
    assert sel(None, 4, fake, 1, 1, 16, None, None, 0, None) == obc.OBC_EINVAL
    assert sel(fake, 0, fake, 1, 1, 16, None, None, 0, None) == obc.OBC_EINVAL
    assert sel(fake, 17, fake, 1, 1, 16, None, None, 0, None) == obc.OBC_EINVAL
    short = (ctypes.c_int32 * 1)(3)
    assert sel(fake, 4, fake, 1, 1, 16, short, None, 0, None) == obc.OBC_EINVAL          # budget > len_b
    assert sel(fake, 4, fake, 1, 1, 16, None, ctypes.c_void_p(4100), 1 << 20, None) == obc.OBC_EWORKSPACE  # misaligned scratch

    sp = lib.obc_select_protected          # (scores, num_hh, num_sinks, num_recent, num_coming, keep, B, Hkv, N, lens, stream)
    assert sp(None, 4, 0, 0, 0, fake, 1, 1, 16, None, None, 0, None) == obc.OBC_EINVAL
    assert sp(fake, 4, 0, 2, 3, fake, 1, 1, 16, None, None, 0, None) == obc.OBC_EINVAL         # num_coming > num_recent
    assert sp(fake, -1, 0, 0, 0, fake, 1, 1, 16, None, None, 0, None) == obc.OBC_EINVAL
    assert sp(fake, 0, 0, 0, 0, fake, 1, 1, 16, None, None, 0, None) == obc.OBC_EINVAL         # nothing kept
    assert sp(fake, 10, 4, 5, 2, fake, 1, 1, 16, None, None, 0, None) == obc.OBC_EINVAL        # 17 kept of 16
    assert sp(fake, 2, 1, 1, 0, fake, 1, 1, 16, short, None, 0, None) == obc.OBC_EINVAL        # 4 kept of len 3
    pl = lib.obc_select_pooled             # (scores, num_hh, num_sinks, num_recent, num_coming, pool, keep, B, Hkv, N, lens, stream)
    assert pl(fake, 4, 0, 0, 0, 4, fake, 1, 1, 16, None, None, 0, None) == obc.OBC_EINVAL      # even window
    assert pl(fake, 4, 0, 0, 0, 0, fake, 1, 1, 16, None, None, 0, None) == obc.OBC_EINVAL
    assert pl(fake, 4, 0, 0, 0, 17, fake, 1, 1, 16, None, None, 0, None) == obc.OBC_EUNSUPPORTED
    assert pl(fake, 17, 0, 0, 0, 5, fake, 1, 1, 16, None, None, 0, None) == obc.OBC_EINVAL
    ad = lib.obc_select_adaptive           # (scores, budget, n_safe, keep, counts, cap, B, Hkv, N, lens, ws, ws_bytes, stream)
    assert ad(fake, 4, 5, fake, fake, 16, 1, 2, 16, None, fake, 1 << 30, None) == obc.OBC_EINVAL     # n_safe > budget
    assert ad(fake, 4, 1, fake, fake, 6, 1, 2, 16, None, fake, 1 << 30, None) == obc.OBC_EINVAL      # cap < 2*4 - 1
    assert ad(fake, 4, 1, fake, None, 7, 1, 2, 16, None, fake, 1 << 30, None) == obc.OBC_EINVAL
    assert ad(fake, 4, 1, fake, fake, 7, 1, 2, 16, None, None, 0, None) == obc.OBC_EWORKSPACE
    assert ad(fake, 4, 1, fake, fake, 7, 1, 2, 16, None, fake, 64, None) == obc.OBC_EWORKSPACE
    need = ctypes.c_size_t(0)
    assert lib.obc_select_adaptive_workspace_bytes(4, 8, 32768, 2048, 409, ctypes.byref(need)) == obc.OBC_OK
    assert need.value % 256 == 0 and need.value > 4 * 8 * 32768 * 4
    cs = lib.obc_compact_scores            # (scores, keep, out, B, Hkv, N, budget, N_out, stream)
    assert cs(fake, None, fake, 1, 1, 16, 4, 8, None) == obc.OBC_EINVAL
    assert cs(fake, fake, fake, 1, 1, 16, 4, 3, None) == obc.OBC_EINVAL               # N_out < budget
    probe = lib.obc_probe_read_bandwidth
    assert probe(None, 1024, fake, None) == obc.OBC_EINVAL
    assert probe(fake, 1000, fake, None) == obc.OBC_EINVAL                            # not a multiple of 16

    cp = lib.obc_compact
    assert cp(fake, fake, None, fake, fake, 1, 1, 16, 4, 64, 0, None) == obc.OBC_EINVAL
    assert cp(fake, fake, fake, fake, fake, 1, 1, 16, 0, 64, 0, None) == obc.OBC_EINVAL
    assert cp(fake, fake, fake, ctypes.c_void_p(4104), fake, 1, 1, 16, 4, 64, 0, None) == obc.OBC_EINVAL   # misaligned output
    assert cp(fake, fake, fake, fake, fake, 1, 1, 16, 4, 6, 1, None) == obc.OBC_EUNSUPPORTED   # 12-byte rows
    assert cp(fake, fake, fake, fake, fake, 1, 1, 16, 4, 64, 9, None) == obc.OBC_EUNSUPPORTED  # dtype
    ip = lib.obc_compact_inplace           # (k, v, scores|NULL, keep, B, Hkv, N, budget, d, dtype, stream)
    assert ip(fake, fake, None, None, 1, 1, 16, 4, 64, 0, None) == obc.OBC_EINVAL
    assert ip(fake, None, None, fake, 1, 1, 16, 4, 64, 0, None) == obc.OBC_EINVAL
    assert ip(fake, fake, None, fake, 1, 1, 16, 17, 64, 0, None) == obc.OBC_EINVAL            # budget > N
    assert ip(fake, ctypes.c_void_p(4104), None, fake, 1, 1, 16, 4, 64, 0, None) == obc.OBC_EINVAL   # misaligned cache
    assert ip(fake, fake, ctypes.c_void_p(4098), fake, 1, 1, 16, 4, 64, 0, None) == obc.OBC_EINVAL   # misaligned scores
    assert ip(fake, fake, None, fake, 1, 1, 16, 4, 6, 1, None) == obc.OBC_EUNSUPPORTED       # 12-byte rows
    assert ip(fake, fake, None, fake, 1, 1, 16, 4, 64, 7, None) == obc.OBC_EUNSUPPORTED      # dtype

    ds = lib.obc_decode_step   # (q, k, v, scores, evicted, N, Hq, Hkv, d, variant, B, dtype, lens, sinks, recent, ws, ws_bytes, stream)
    assert ds(fake, fake, fake, fake, fake, 1025, 32, 8, 128, obc.OBC_ALL, 1, 0, None, 4, 24, fake, 1 << 30, None) == obc.OBC_EINVAL
    assert ds(fake, fake, fake, fake, fake, 1025, 32, 8, 128, 2, 1, 0, None, -1, 24, fake, 1 << 30, None) == obc.OBC_EINVAL
    assert ds(fake, fake, fake, fake, fake, 28, 32, 8, 128, 2, 1, 0, None, 4, 24, fake, 1 << 30, None) == obc.OBC_EINVAL   # nothing competes
    tiny = (ctypes.c_int32 * 1)(28)
    assert ds(fake, fake, fake, fake, fake, 1025, 32, 8, 128, 2, 1, 0, tiny, 4, 24, fake, 1 << 30, None) == obc.OBC_EINVAL  # nor in this sequence
    assert ds(fake, fake, fake, fake, ctypes.c_void_p(4098), 1025, 32, 8, 128, 2, 1, 0, None, 4, 24, fake, 1 << 30, None) == obc.OBC_EINVAL
    assert ds(fake, fake, fake, fake, fake, 1025, 32, 8, 128, 2, 1, 0, None, 4, 24, None, 1 << 30, None) == obc.OBC_EWORKSPACE
    assert ds(fake, fake, fake, fake, fake, 1025, 32, 8, 128, 2, 1, 0, None, 4, 24, fake, 256, None) == obc.OBC_EWORKSPACE
    assert ds(None, fake, fake, fake, fake, 1025, 32, 8, 128, 2, 1, 0, None, 4, 24, fake, 1 << 30, None) == obc.OBC_EINVAL
    assert ds(fake, fake, fake, None, fake, 1025, 32, 8, 128, 2, 1, 0, None, 4, 24, fake, 1 << 30, None) == obc.OBC_EINVAL
    step = obc.obc_decode_step_workspace_bytes(1, 1025, 32, 8, 128, obc.OBC_BF16, obc.OBC_JOINT)
    assert step == obc.obc_score_workspace_bytes(1, 1025, 1, 32, 8, 128, obc.OBC_BF16, obc.OBC_JOINT) + 256
    with pytest.raises(obc.ObcError):
        obc.obc_decode_step_workspace_bytes(1, 1025, 32, 8, 128, obc.OBC_BF16, obc.OBC_ALL)


def test_plan_ignores_the_process_environment_and_follows_the_hooks(lib, monkeypatch):
    """The workspace plan is a function of the arguments and of obc_set_score_path / obc_set_score_tuning alone:
    changing the environment between the size query and the call cannot make them disagree."""
    c3 = (4, 32768, 32, 32, 8, 128, obc.OBC_BF16, obc.OBC_JOINT)
    dec = (1, 1025, 1, 32, 8, 128, obc.OBC_BF16, obc.OBC_JOINT)
    base = [obc.obc_score_workspace_bytes(*a) for a in (c3, dec)]
    for name, value in (("OBC_SCORE_PATH", "plain"), ("OBC_TUNE_SPLITS", "3"), ("OBC_TUNE_RANGE", "128")):
        monkeypatch.setenv(name, value)
    assert [obc.obc_score_workspace_bytes(*a) for a in (c3, dec)] == base
    # the call after an environment change still accepts a workspace of exactly the queried size: it gets past the
    # workspace check (with no GPU here the launch itself then fails)
    fake = ctypes.c_void_p(1 << 20)
    import torch
    if not torch.cuda.is_available():      # (with a GPU present the made-up pointers must never reach a kernel)
        rc = lib.obc_score(fake, fake, fake, 32768, 32, 32, 8, 128, 2, fake, 4, 1, None, fake, base[0], None)
        assert rc == obc.OBC_ELAUNCH
    assert lib.obc_score(fake, fake, fake, 32768, 32, 32, 8, 128, 2, fake, 4, 1, None, fake, base[0] - 256,
                         None) == obc.OBC_EWORKSPACE
    # the matrix-core plan holds no buffer of the plain path: forcing the plain path changes the size
    try:
        obc.obc_set_score_path("plain")
        plain = obc.obc_score_workspace_bytes(*c3)
        assert plain != base[0] and plain >= 2 * 4 * 32 * 32 * 128 * 4
        obc.obc_set_score_path("mfma")
        assert obc.obc_score_workspace_bytes(*dec) != base[1]          # one-row window kept on the matrix cores
        obc.obc_set_score_path("auto")
        obc.obc_set_score_tuning(4, 256)
        assert obc.obc_score_workspace_bytes(*c3) < base[0]            # fewer splits, smaller partial records
        with pytest.raises(obc.ObcError):
            obc.obc_set_score_tuning(4, 100)                           # not a multiple of 64
        with pytest.raises(obc.ObcError):
            obc.obc_set_score_path(9)
    finally:
        obc.obc_set_score_path("auto")
        obc.obc_set_score_tuning(0, 0)
    assert [obc.obc_score_workspace_bytes(*a) for a in (c3, dec)] == base
    # c3's workspace: the split partials dominate (16 splits x 4096 rows x 132 floats) and nothing of the plain path is in it
    assert base[0] < 16 * 4096 * 132 * 4 + (4 << 20)


def test_bench_refuses_more_than_one_gpu():
    """One GPU per box in this build: bench.py says so and exits instead of launching collectives."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""

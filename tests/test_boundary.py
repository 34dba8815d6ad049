"""Host-side checks of the C ABI (no GPU): the library loads, exports every function the header
declares, and rejects invalid arguments before anything is enqueued."""
import ctypes as C
import os
import re

import pytest

import paper_2605_25475_amd as im
from paper_2605_25475_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return im.load_library()


def good_cfg(**kw):
    d = dict(batch=2, n_q_heads=32, n_kv_heads=8, capacity=512, n_idx_heads=8, max_queries=16)
    d.update(kw)
    return im.Config(**d)


def test_every_declared_function_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "indexmem.h")).read()
    declared = set(re.findall(r"\b(im_[a-z_]+)\s*\(", header))
    assert declared == set(im.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_workspace_bytes_and_config_validation(lib):
    c = good_cfg().c_struct()
    n = lib.im_workspace_bytes(C.byref(c))
    assert n > 0 and n % 256 == 0
    bigger = good_cfg(max_queries=64).c_struct()
    assert lib.im_workspace_bytes(C.byref(bigger)) > n
    bad = [dict(batch=0), dict(n_q_heads=30), dict(capacity=0), dict(n_idx_heads=0), dict(n_idx_heads=17),
           dict(gate_in_dim=100), dict(n_sink=-1), dict(fold_block=16), dict(max_queries=0),
           dict(mem_eps=0.0), dict(n_sink=600)]
    for kw in bad:
        cc = good_cfg(**kw).c_struct()
        assert lib.im_workspace_bytes(C.byref(cc)) == 0, kw
        h = C.c_void_p()
        assert lib.im_create(C.byref(cc), 4096, 1 << 40, C.byref(h)) == im.IM_ERR_INVALID_ARG, kw
    for kw in [dict(head_dim=64), dict(idx_dim=32), dict(mem_dim=64), dict(n_q_heads=72, n_kv_heads=8)]:
        cc = good_cfg(**kw).c_struct()
        h = C.c_void_p()
        assert lib.im_create(C.byref(cc), 4096, 1 << 40, C.byref(h)) == im.IM_ERR_UNSUPPORTED, kw
    assert lib.im_workspace_bytes(None) == 0


def _fake_handle(lib, cfg):
    # im_create is host-only, so a fake (aligned, never dereferenced) workspace address will do
    c = cfg.c_struct()
    h = C.c_void_p()
    assert lib.im_create(C.byref(c), 1 << 20, lib.im_workspace_bytes(C.byref(c)), C.byref(h)) == im.IM_OK
    return h


def test_create_rejects_bad_workspace(lib):
    c = good_cfg().c_struct()
    n = lib.im_workspace_bytes(C.byref(c))
    h = C.c_void_p()
    assert lib.im_create(C.byref(c), None, n, C.byref(h)) == im.IM_ERR_INVALID_ARG
    assert lib.im_create(C.byref(c), (1 << 20) + 8, n, C.byref(h)) == im.IM_ERR_INVALID_ARG    # misaligned
    assert lib.im_create(C.byref(c), 1 << 20, n - 1, C.byref(h)) == im.IM_ERR_INVALID_ARG      # too small
    assert lib.im_create(C.byref(c), 1 << 20, n, None) == im.IM_ERR_INVALID_ARG


def test_calls_validate_before_enqueuing(lib):
    cfg = good_cfg()
    h = _fake_handle(lib, cfg)
    X = 1 << 21   # a non-null stand-in address; every call below must fail before using it
    st = B.ImState(X, X, X, X, X, X, X, X)
    st_bad = B.ImState(X, X, None, X, X, X, X, X)
    pr = B.ImParams(X, X, X, None, None, X, X, 0.0)
    pr_bad = B.ImParams(X, None, X, None, None, X, X, 0.0)
    E = im.IM_ERR_INVALID_ARG
    assert lib.im_set_max_live(h, 0) == E and lib.im_set_max_live(h, 513) == E
    assert lib.im_set_max_live(h, 257) == im.IM_OK
    assert lib.im_append_kv(h, C.byref(st), X, X, X, 0, None) == E
    assert lib.im_append_kv(h, C.byref(st), X, X, X, 513, None) == E
    assert lib.im_append_kv(h, C.byref(st), None, X, X, 1, None) == E
    assert lib.im_append_kv(h, C.byref(st_bad), X, X, X, 1, None) == E
    assert lib.im_append_kv_hidden(h, C.byref(pr), C.byref(st), X, X, None, X, 1, None) == E
    assert lib.im_append_kv_hidden(h, C.byref(pr), C.byref(st), X, X, X, X, 1, None) == im.IM_ERR_UNSUPPORTED   # per-head layout
    assert lib.im_index_score(h, C.byref(pr), C.byref(st), X, X, X, 0, X, None) == E
    assert lib.im_index_score(h, C.byref(pr), C.byref(st), X, X, X, 17, X, None) == E
    assert lib.im_index_score(h, C.byref(pr_bad), C.byref(st), X, X, X, 1, X, None) == E
    assert lib.im_index_score(h, C.byref(pr), C.byref(st), X, X, X, 1, None, None) == E
    assert lib.im_topb_select(h, X, C.byref(st), 3, X, X, X, X, None) == E          # below the 4 sinks
    assert lib.im_topb_select(h, X, C.byref(st), 513, X, X, X, X, None) == E        # above capacity
    assert lib.im_topb_select(h, None, C.byref(st), 64, X, X, X, X, None) == E
    assert lib.im_memory_update(h, C.byref(pr), C.byref(st), X, X, 0.0, 0.5, None) == E
    assert lib.im_memory_update(h, C.byref(pr), C.byref(st), X, X, 1.5, 0.5, None) == E
    assert lib.im_memory_update(h, C.byref(pr), C.byref(st), X, X, 0.9, 0.0, None) == E
    assert lib.im_memory_update(h, C.byref(pr), C.byref(st), None, X, 0.9, 0.5, None) == E
    assert lib.im_compact_kv(h, C.byref(st), X, None, X, X, None) == E
    st2 = B.ImState(*([X + 4096] * 8))
    assert lib.im_gather_kept(h, C.byref(st), C.byref(st), 64, X, X, X, X, None) == E      # in place: im_compact_kv's job
    assert lib.im_gather_kept(h, C.byref(st), C.byref(st2), 0, X, X, X, X, None) == E
    assert lib.im_gather_kept(h, C.byref(st), C.byref(st_bad), 64, X, X, X, X, None) == E
    assert lib.im_gather_kept(h, C.byref(st), C.byref(st2), 64, X, None, X, X, None) == E
    assert lib.im_decode_attn_with_readout(h, C.byref(pr), C.byref(st), None, X, None, None) == E
    assert lib.im_decode_attn_with_readout(h, C.byref(pr), C.byref(st_bad), X, X, None, None) == E
    assert lib.im_decode_step(h, C.byref(pr), C.byref(st), X, X, X, X, X, X, 3, 0.9, 0.5, X, None, None, None, None) == E
    assert lib.im_decode_step(h, C.byref(pr), C.byref(st), X, None, X, X, X, X, 64, 0.9, 0.5, X, None, None, None, None) == E
    assert lib.im_decode_step(h, C.byref(pr), C.byref(st), X, X, X, X, X, X, 64, 0.9, 0.5, None, None, None, None, None) == E
    assert lib.im_attend_step(h, C.byref(pr), C.byref(st), None, X, X, X, X, None, None) == E
    assert lib.im_attend_step(h, C.byref(pr), C.byref(st_bad), X, X, X, X, X, None, None) == E
    assert lib.im_attend_step(h, C.byref(pr), C.byref(st), X, X, X, X, None, None, None) == E
    assert lib.im_attend_step_hidden(h, C.byref(pr), C.byref(st), X, X, X, X, X, X, None, None) == im.IM_ERR_UNSUPPORTED   # per-head layout
    assert lib.im_decode_step_shared(h, C.byref(pr), C.byref(st), X, X, X, X, None, 0.9, 0.5, X, None, None) == E
    assert lib.im_decode_step_shared(h, C.byref(pr), C.byref(st), X, X, X, X, X, 1.5, 0.5, X, None, None) == E
    assert lib.im_decode_step_shared(h, C.byref(pr), C.byref(st), X, X, None, X, X, 0.9, 0.5, X, None, None) == E
    assert lib.im_profile_start(h, 0, 0) == E and lib.im_profile_start(h, 4, 3) == E
    assert lib.im_query_status(h, None, None) == E
    assert b"status_host" in lib.im_last_error(h)
    lib.im_destroy(h)
    assert lib.im_set_max_live(None, 1) == E


def test_head_shared_layout_validation(lib):
    ok = good_cfg(head_shared=1, idx_dim=16)
    assert lib.im_workspace_bytes(C.byref(ok.c_struct())) > lib.im_workspace_bytes(C.byref(good_cfg().c_struct()))
    h = C.c_void_p()
    assert lib.im_create(C.byref(good_cfg(head_shared=2, idx_dim=16).c_struct()), 1 << 20, 1 << 40, C.byref(h)) == im.IM_ERR_INVALID_ARG
    assert lib.im_create(C.byref(good_cfg(head_shared=1).c_struct()), 1 << 20, 1 << 40, C.byref(h)) == im.IM_ERR_UNSUPPORTED   # idx_dim 64
    assert lib.im_create(C.byref(good_cfg(idx_dim=16).c_struct()), 1 << 20, 1 << 40, C.byref(h)) == im.IM_ERR_UNSUPPORTED
    h = _fake_handle(lib, ok)
    X = 1 << 21
    st = B.ImState(X, X, X, X, X, X, X, X)
    pr = B.ImParams(X, X, X, None, None, X, X, 0.0)
    U = im.IM_ERR_UNSUPPORTED
    assert lib.im_append_kv(h, C.byref(st), X, X, X, 1, None) == U
    assert lib.im_decode_step(h, C.byref(pr), C.byref(st), X, None, X, X, X, X, 64, 0.9, 0.5, X, None, None, None, None) == im.IM_ERR_INVALID_ARG
    assert lib.im_attend_step(h, C.byref(pr), C.byref(st), X, X, X, X, X, None, None) == U
    assert lib.im_decode_step_shared(h, C.byref(pr), C.byref(st), X, X, X, X, X, 0.9, 0.5, X, None, None) == U
    assert lib.im_attend_step_hidden(h, C.byref(pr), C.byref(st), X, None, X, X, X, X, None, None) == im.IM_ERR_INVALID_ARG
    assert lib.im_decode_step_shared_hidden(h, C.byref(pr), C.byref(st), X, X, X, X, X, None, 0.9, 0.5, X, None, None) == im.IM_ERR_INVALID_ARG
    assert lib.im_decode_step_shared_hidden(h, C.byref(pr), C.byref(st), X, X, X, X, X, X, 1.5, 0.5, X, None, None) == im.IM_ERR_INVALID_ARG
    assert lib.im_append_kv_hidden(h, C.byref(pr), C.byref(st), X, X, X, X, 0, None) == im.IM_ERR_INVALID_ARG
    assert b"head_shared" in lib.im_last_error(h) or b"n_new" in lib.im_last_error(h)
    lib.im_destroy(h)


def test_binding_fails_loudly_on_invalid_config():
    with pytest.raises(im.IndexMemError):
        im.Handle(good_cfg(head_dim=64), device="cpu")


def test_static_entry_point_validates_on_the_host(lib):
    # im_decode_attn_with_readout_static: invalid arguments and sizes beyond its built-in buffer are
    # refused before any GPU call, with a text under im_last_error(NULL)
    cfg = good_cfg().c_struct()
    p = B.ImParams(1 << 20, 1 << 20, 1 << 20, None, None, 1 << 20, 1 << 20, 0.0)
    st = B.ImState(*([1 << 20] * 8))
    f = lib.im_decode_attn_with_readout_static
    assert f(None, 10, C.byref(p), C.byref(st), 1 << 20, 1 << 20, None, None, None) == im.IM_ERR_INVALID_ARG
    assert f(C.byref(cfg), 0, C.byref(p), C.byref(st), 1 << 20, 1 << 20, None, None, None) == im.IM_ERR_INVALID_ARG
    assert f(C.byref(cfg), 513, C.byref(p), C.byref(st), 1 << 20, 1 << 20, None, None, None) == im.IM_ERR_INVALID_ARG
    assert b"max_live" in lib.im_last_error(None)
    assert f(C.byref(cfg), 10, C.byref(p), C.byref(st), None, 1 << 20, None, None, None) == im.IM_ERR_INVALID_ARG
    big = good_cfg(batch=64, n_q_heads=64, n_kv_heads=8, n_idx_heads=16, capacity=16384).c_struct()
    need = 256 + 520 * 64 * 64 * 128
    assert need > im.IM_STATIC_SCRATCH_BYTES
    assert f(C.byref(big), 16384, C.byref(p), C.byref(st), 1 << 20, 1 << 20, None, None, None) == im.IM_ERR_INVALID_ARG
    msg = lib.im_last_error(None).decode()
    assert str(need) in msg and "IM_STATIC_SCRATCH_BYTES" in msg
    bad = good_cfg(head_dim=64).c_struct()
    assert f(C.byref(bad), 10, C.byref(p), C.byref(st), 1 << 20, 1 << 20, None, None, None) == im.IM_ERR_UNSUPPORTED


def test_a_plain_c_program_compiles_against_the_header_links_and_runs(tmp_path):
    # the boundary is a C ABI: tests/c_abi/host_calls.c is C99 (-pedantic), includes the header, links the
    # library and drives its host-only calls
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    from paper_2605_25475_amd import build as _build
    im.load_library()   # (builds the library if it is absent)
    libdir = os.path.dirname(_build.LIB_PATH)
    exe = str(tmp_path / "host_calls")
    cmd = [gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "c_abi", "host_calls.c"), "-L", libdir, "-lindexmem",
           "-Wl,-rpath," + libdir, "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and r.stdout.startswith("ok "), r.stdout + r.stderr

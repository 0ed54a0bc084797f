"""Host-side checks that need no GPU: the library loads, exports every declared symbol, and
rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

import paper_2510_14961_amd as R
from paper_2510_14961_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(R.library_path()):
        import paper_2510_14961_amd.build as bld
        bld.build(verbose=False)
    return R.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "rdlm.h")).read()
    declared = set(re.findall(r"\b(rdlm_[a-z_0-9]+)\s*\(", header))
    assert declared, "no declarations found"
    assert declared == set(R.EXPORTED_SYMBOLS)
    for name in declared:
        assert hasattr(lib, name), name


def test_struct_layouts_match_the_header():
    assert C.sizeof(B._Model) == 12 * 4
    assert C.sizeof(B._Sampler) == 14 * 4 + 8
    assert B._Sampler.beta.offset == 40 and B._Sampler.eta.offset == 44
    assert B._Sampler.top_p.offset == 48 and B._Sampler.init_mode.offset == 52 and B._Sampler.seed.offset == 56


def _model(**kw):
    base = dict(vocab=256, hidden=128, n_heads=2, head_dim=64, mlp=512, n_prelude=1, n_core=2, n_coda=1,
                rope_base=10000.0, rms_eps=1e-6, emb_scale=1.0, dtype=0)
    base.update(kw)
    return B._Model(*[base[f[0]] for f in B._Model._fields_])


def test_num_weights(lib):
    assert lib.rdlm_num_weights(C.byref(_model())) == 1 + 7 * 4 + 3


@pytest.mark.parametrize("bad", [
    dict(hidden=130), dict(n_heads=3), dict(head_dim=63, n_heads=2, hidden=126), dict(n_core=0), dict(dtype=7),
    dict(dtype=1, hidden=144, n_heads=3, head_dim=48), dict(dtype=1, vocab=250), dict(mlp=64), dict(rope_base=0.0),
])
def test_create_rejects_bad_shapes_on_the_host(lib, bad):
    m = _model(**bad)
    n = 64
    ptrs = (C.c_void_p * n)(*([1] * n))          # never dereferenced: validation comes first
    out = C.c_void_p()
    assert lib.rdlm_create(C.byref(m), ptrs, 1, 64, 32, None, C.byref(out)) == -1
    assert not out.value


def test_create_rejects_bad_capacities_and_null_pointers(lib):
    m = _model()
    n = lib.rdlm_num_weights(C.byref(m))
    ptrs = (C.c_void_p * n)(*([1] * n))
    out = C.c_void_p()
    for args in ((0, 64, 32), (1, 1, 32), (1, 64, 0), (65, 64, 32)):
        assert lib.rdlm_create(C.byref(m), ptrs, *args, None, C.byref(out)) == -1
    ptrs[3] = None
    assert lib.rdlm_create(C.byref(m), ptrs, 1, 64, 32, None, C.byref(out)) == -1
    assert lib.rdlm_create(None, ptrs, 1, 64, 32, None, C.byref(out)) == -1
    assert lib.rdlm_create(C.byref(m), None, 1, 64, 32, None, C.byref(out)) == -1


def test_null_context_is_an_error_not_a_crash(lib):
    assert lib.rdlm_sample_step(None) == -1
    assert lib.rdlm_generate(None, 1, None) == -1
    assert lib.rdlm_prefill(None, 0, 1, 1, 1.0, 1) == -1
    assert lib.rdlm_destroy(None) == -1
    assert lib.rdlm_strerror(-2).decode().startswith("exceeds")
    assert lib.rdlm_strerror(0).decode() == "ok"


def test_new_status_code_has_a_message(lib):
    assert "non-finite" in lib.rdlm_strerror(R.STATUS["ENUMERIC"]).decode()


def test_workspace_bytes_is_a_host_side_size_query(lib):
    m = _model()
    small = lib.rdlm_workspace_bytes(C.byref(m), 1, 32)
    big = lib.rdlm_workspace_bytes(C.byref(m), 1, 64)
    assert 0 < small < big
    assert small % 256 == 0
    # the slab holds at least the logits of every padded row (2 row tiles for 1 sequence x 32 rows)
    assert small >= 2 * 32 * 256 * 4
    assert lib.rdlm_workspace_bytes(C.byref(_model(hidden=130)), 1, 32) == 0
    assert lib.rdlm_workspace_bytes(C.byref(m), 0, 32) == 0
    assert lib.rdlm_workspace_bytes(None, 1, 32) == 0


def test_create_ws_rejects_a_bad_workspace_before_touching_the_device(lib):
    m = _model()
    n = lib.rdlm_num_weights(C.byref(m))
    ptrs = (C.c_void_p * n)(*([1] * n))
    out = C.c_void_p()
    need = lib.rdlm_workspace_bytes(C.byref(m), 1, 32)
    # misaligned
    assert lib.rdlm_create_ws(C.byref(m), ptrs, 1, 64, 32, None, C.c_void_p(0x1001), need, C.byref(out)) == -1
    # too small
    assert lib.rdlm_create_ws(C.byref(m), ptrs, 1, 64, 32, None, C.c_void_p(0x1000), need - 1, C.byref(out)) == -2
    assert not out.value


def test_entry_points_added_later_refuse_a_null_context(lib):
    assert lib.rdlm_core_step_static(None, 1, None, None, None, None, None, 1, None) == -1
    assert lib.rdlm_core_step_static_bytes(None, 1) == 0
    assert lib.rdlm_set_tuning(None, b"no_fold", b"1") == -1
    assert lib.rdlm_sampler_status(None, None, None) == -1
    assert R.STATIC_SCRATCH_BYTES == int(re.search(r"RDLM_STATIC_SCRATCH_BYTES \((\d+)u << 20\)",
                                                   open(os.path.join(ROOT, "include", "rdlm.h")).read()).group(1)) << 20


def test_bench_refuses_more_than_one_gpu():
    """One GPU only: bench.py --gpus 2 says so and exits non-zero before it touches a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""

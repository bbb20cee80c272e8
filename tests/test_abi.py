"""Host-side checks that need no GPU: the library loads, exports every symbol
the header declares, the ctypes structs match the header's layouts, and
profile validation rejects bad input before any device work."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2505_06641_amd import binding, workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "sneakpeek.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2505_06641_amd import build
        build.build_library(verbose=False)
    return binding.load_library()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sp_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_struct_layouts_match_the_header():
    assert C.sizeof(binding.sp_decision) == 40
    assert binding.sp_decision.t_start_ms.offset == 16 and binding.sp_decision.score.offset == 32
    assert C.sizeof(binding.sp_summary) == 40
    assert binding.sp_profile.n_classes.offset == 24
    assert binding.sp_profile.prio_timescale_ms.offset == 24 + 9 * 8


def test_strerror_covers_all_codes(lib):
    seen = set()
    for code in (0, 1, -1, -2, -3, -4, -5):
        s = lib.sp_strerror(code).decode()
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 7
    assert lib.sp_strerror(-99).decode() == "unknown status"


def _create(lib, profile, max_requests=16):
    st, keep = binding.marshal_profile(profile, max_requests)
    h = C.c_void_p()
    rc = lib.sp_create(C.byref(st), 0, C.byref(h))
    if rc == binding.SP_OK:
        lib.sp_destroy(h)
    return rc


def test_profile_validation_happens_before_device_work(lib):
    base = lambda: wl.tiny(seed=1, n=4, classes=(3, 2), models=(2, 3), max_batch=4).profile
    good = _create(lib, base())
    assert good in (binding.SP_OK, binding.SP_EDEVICE)      # EDEVICE on a box without a GPU

    p = base(); p.acc[1][2, 1] = 1.5
    assert _create(lib, p) == binding.SP_EINVAL
    p = base(); p.acc[0][0, 0] = np.nan
    assert _create(lib, p) == binding.SP_EINVAL
    p = base(); p.lat_ms[0][1, 2] = p.lat_ms[0][1, 1] - 0.1
    assert _create(lib, p) == binding.SP_EINVAL
    p = base(); p.lat_ms[1][0, 0] = -1.0
    assert _create(lib, p) == binding.SP_EINVAL
    p = base(); p.penalty[1] = 7
    assert _create(lib, p) == binding.SP_EINVAL
    p = base(); p.prio_timescale_ms = 0.0
    assert _create(lib, p) == binding.SP_EINVAL
    p = base(); p.n_classes[0] = 0
    assert _create(lib, p) == binding.SP_EINVAL
    p = base(); p.feat_dtype = 5
    assert _create(lib, p) == binding.SP_EINVAL
    p = base(); p.max_batch = 100000
    assert _create(lib, p) == binding.SP_ECAPACITY
    p = base(); p.n_models[0] = 17
    assert _create(lib, p) == binding.SP_ECAPACITY
    assert _create(lib, base(), max_requests=-1) == binding.SP_EINVAL
    h = C.c_void_p()
    assert lib.sp_create(None, 0, C.byref(h)) == binding.SP_EINVAL


def test_null_context_is_rejected(lib):
    assert lib.sp_score(None, 0, None, None, None, None, None, None, None) == binding.SP_EINVAL
    assert lib.sp_greedy_round(None, None, None, None) == binding.SP_EINVAL
    assert lib.sp_schedule(None, 0, None, None, None, None, None, None, 0, None) == binding.SP_EINVAL
    assert lib.sp_max_models(None) == 0
    lib.sp_destroy(None)


def test_a_missing_library_is_an_error_not_a_fallback(tmp_path):
    # the product path has no CPU substitute: without the built library, loading raises
    from paper_2505_06641_amd import binding
    with pytest.raises(RuntimeError, match="is missing"):
        binding.load_library(str(tmp_path / "libsneakpeek_hip.so"))
    src = open(binding.__file__).read()
    assert "oracle" not in src.replace("the binding and the oracle", "")

"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol,
and its host-side packing agrees bit for bit with the oracle's (two independent
implementations of the canonical format)."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_2602_06694_amd import binding as nq
from paper_2602_06694_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    import glob
    names = set()
    for path in sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))):
        src = open(path).read()
        src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
        names |= set(re.findall(r"\b(nq_[a-z0-9_]+)\s*\(", src))
    return sorted(names)


def test_library_loads_and_exports_every_declared_symbol():
    L = nq.lib()
    names = declared_functions()
    assert len(names) >= 17, names
    for n in names:
        assert hasattr(L, n), f"{n} declared in include/*.h but not exported"


def test_binding_has_every_declared_name():
    for n in declared_functions():
        assert hasattr(nq, n), f"binding lacks {n}"


def test_header_constants_match_binding():
    src = open(os.path.join(ROOT, "include", "nq_binlr.h")).read()
    for name in ("NQ_OK", "NQ_E_INVALID_ARG", "NQ_E_SHAPE", "NQ_E_ALIGN", "NQ_E_NULL", "NQ_E_UNSUPPORTED", "NQ_E_HIP",
                 "NQ_I8", "NQ_F32", "NQ_F16", "NQ_BF16", "NQ_MAX_DIM", "NQ_DECODE_MAX_BATCH", "NQ_PREFILL_MIN_BATCH"):
        m = re.search(rf"#define\s+{name}\s+\(?(-?\d+)\)?", src)
        assert m, name
        assert int(m.group(1)) == getattr(nq, name), name


@pytest.mark.parametrize("cols", [1, 31, 32, 33, 63, 64, 65, 256, 3520])
def test_pack_bit_exact_against_oracle(cols):
    pm1 = synth.gen_signs_pm1(5, cols, 900 + cols)
    w = nq.nq_pack_signs(pm1)
    assert np.array_equal(w, oracle.pack_signs(pm1))
    assert np.array_equal(nq.nq_unpack_signs(w, cols), pm1)
    assert np.array_equal(nq.nq_unpack_signs(w, cols), oracle.unpack_signs(w, cols))
    assert nq.nq_packed_words(5, cols) == w.size


def test_pack_float_types_and_sign_rule():
    vals = np.array([[-1.0, 1.0, 0.0, -0.0, -1e-30, 1e-30, -np.inf, np.inf, 0.5, -0.5]], dtype=np.float32)
    expect = oracle.pack_signs(vals)
    assert np.array_equal(nq.nq_pack_signs(vals), expect)
    v16 = np.array([[-1.0, 1.0, 0.0, -0.0, -6e-8, 6e-8, -np.inf, np.inf, 0.5, -0.5]], dtype=np.float16)
    assert np.array_equal(nq.nq_pack_signs(v16), oracle.pack_signs(v16))
    bf = synth.f32_to_bf16_bits(vals)
    assert np.array_equal(nq.nq_pack_signs(bf, dtype=nq.NQ_BF16), oracle.pack_signs(synth.bf16_bits_to_f32(bf)))
    rnd = np.random.default_rng(3).standard_normal((9, 77)).astype(np.float32)
    assert np.array_equal(nq.nq_pack_signs(rnd), oracle.pack_signs(rnd))


def test_pack_rejects_bad_values():
    with pytest.raises(nq.NQError) as e:
        nq.nq_pack_signs(np.array([[1.0, np.nan]], dtype=np.float32))
    assert e.value.status == nq.NQ_E_INVALID_ARG
    for bad in (0, 2, -2):
        with pytest.raises(nq.NQError) as e:
            nq.nq_pack_signs(np.array([[1, bad]], dtype=np.int8))
        assert e.value.status == nq.NQ_E_INVALID_ARG
    L = nq.lib()
    out = np.zeros(4, dtype=np.uint32)
    a = np.ones((1, 4), dtype=np.int8)
    assert L.nq_pack_signs(None, nq.NQ_I8, 1, 4, out.ctypes.data_as(ctypes.c_void_p)) == nq.NQ_E_NULL
    assert L.nq_pack_signs(a.ctypes.data_as(ctypes.c_void_p), nq.NQ_I8, 1, 4, None) == nq.NQ_E_NULL
    assert L.nq_pack_signs(a.ctypes.data_as(ctypes.c_void_p), nq.NQ_I8, 0, 4, out.ctypes.data_as(ctypes.c_void_p)) == nq.NQ_E_SHAPE
    assert L.nq_pack_signs(a.ctypes.data_as(ctypes.c_void_p), 17, 1, 4, out.ctypes.data_as(ctypes.c_void_p)) == nq.NQ_E_INVALID_ARG
    assert "dtype" in nq.nq_last_error_string()


def test_argument_validation_needs_no_gpu():
    L = nq.lib()
    h = ctypes.c_void_p()
    w = np.zeros((4, 1), dtype=np.uint32)
    s = np.ones(4, dtype=np.float16)
    p = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    assert L.nq_binlr_create(None, 4, 4, 4, p(w), p(w), p(s), p(s), nq.NQ_F32, nq.NQ_F32, 0) == nq.NQ_E_NULL
    assert L.nq_binlr_create(ctypes.byref(h), 0, 4, 4, p(w), p(w), p(s), p(s), nq.NQ_F32, nq.NQ_F32, 0) == nq.NQ_E_SHAPE
    assert L.nq_binlr_create(ctypes.byref(h), 4, 4, nq.NQ_MAX_DIM + 1, p(w), p(w), p(s), p(s), nq.NQ_F32, nq.NQ_F32, 0) == nq.NQ_E_SHAPE
    assert L.nq_binlr_create(ctypes.byref(h), 4, 4, 4, None, p(w), p(s), p(s), nq.NQ_F32, nq.NQ_F32, 0) == nq.NQ_E_NULL
    assert L.nq_binlr_create(ctypes.byref(h), 4, 4, 4, p(w), p(w), p(s), p(s), nq.NQ_I8, nq.NQ_F32, 0) == nq.NQ_E_INVALID_ARG
    assert L.nq_binlr_create(ctypes.byref(h), 4, 4, 4, p(w), p(w), p(s), p(s), nq.NQ_F32, nq.NQ_I8, 0) == nq.NQ_E_INVALID_ARG
    assert L.nq_binlr_create(ctypes.byref(h), 4, 4, 4, p(w), p(w), p(s), p(s), nq.NQ_F32, nq.NQ_F32, 64) == nq.NQ_E_INVALID_ARG
    assert h.value is None
    assert L.nq_binlr_create_from_device(ctypes.byref(h), 4, 4, 4, None, p(w), p(s), p(s), nq.NQ_F32, nq.NQ_F32, 0) == nq.NQ_E_NULL
    assert L.nq_binlr_create_from_device(ctypes.byref(h), 4, 0, 4, p(w), p(w), p(s), p(s), nq.NQ_F32, nq.NQ_F32, 0) == nq.NQ_E_SHAPE
    assert L.nq_pack_signs_device(None, nq.NQ_F32, 4, 4, p(w), None, None) == nq.NQ_E_NULL
    assert L.nq_pack_signs_device(p(w), nq.NQ_F32, 0, 4, p(w), None, None) == nq.NQ_E_SHAPE
    assert L.nq_pack_signs_device(p(w), 77, 4, 4, p(w), None, None) == nq.NQ_E_INVALID_ARG
    assert L.nq_binlr_forward(None, None, None, 1, None) == nq.NQ_E_NULL
    assert L.nq_binlr_weight_bytes(None) == 0
    assert L.nq_binlr_destroy(None) == nq.NQ_OK
    assert L.nq_plan_destroy(None) == nq.NQ_OK
    assert L.nq_plan_forward(None, None) == nq.NQ_E_NULL
    assert nq.nq_status_string(nq.NQ_E_ALIGN) == "pointer not 16-byte aligned"


def test_tuning_options_are_set_read_and_restored_without_a_gpu():
    """The options are plain integers behind nq_set_option / nq_get_option: unset (-1) until given a
    value, flags are normalised to 0 / 1, a negative value restores the default, unknown names are errors."""
    assert nq.nq_get_option("schedule_full") == -1
    nq.nq_set_option("schedule_full", 1)
    assert nq.nq_get_option("schedule_full") == 1
    nq.nq_set_option("fuse_max_mb", 0)
    assert nq.nq_get_option("fuse_max_mb") == 0                 # 0 is a value (never fuse), not "unset"
    nq.nq_set_option("no_selfq", 7)
    assert nq.nq_get_option("no_selfq") == 1
    for name in ("schedule_full", "fuse_max_mb", "no_selfq"):
        nq.nq_set_option(name, None)
        assert nq.nq_get_option(name) == -1
    with pytest.raises(nq.NQError) as e:
        nq.nq_set_option("no_such_option", 1)
    assert e.value.status == nq.NQ_E_INVALID_ARG
    with pytest.raises(nq.NQError):
        nq.nq_get_option("NQ_SCHEDULE_FULL")                    # the environment's spelling is not an option name


def test_no_environment_lookup_on_a_launch_path():
    """The library reads the environment in one place only (the options table's initialiser)."""
    import glob
    hits = []
    for f in glob.glob(os.path.join(ROOT, "paper_2602_06694_amd", "csrc", "*")):
        for i, line in enumerate(open(f), 1):
            if "getenv" in line and not line.lstrip().startswith("//"):
                hits.append((os.path.basename(f), i))
    assert len(hits) == 1 and hits[0][0] == "nq_api.hip", hits


def test_lb_admm_host_checks():
    """Argument checks of the LB-ADMM entry points that need no GPU."""
    b = nq.nq_lb_admm_workspace_bytes(4096, 4096, 1024)
    # four padded r x r matrices and four n x r ones at least, in binary64
    assert b >= 8 * (4 * 1024 * 1024 + 4 * 4096 * 1024) and b % 256 == 0
    assert nq.nq_lb_admm_workspace_bytes(100, 70, 65) >= 8 * 4 * 128 * 128
    for bad in ((0, 4, 4), (4, 0, 4), (4, 4, 0), (nq.NQ_ADMM_MAX_DIM + 1, 4, 4), (4, 4, nq.NQ_ADMM_MAX_RANK + 1)):
        with pytest.raises(nq.NQError) as e:
            nq.nq_lb_admm_workspace_bytes(*bad)
        assert e.value.status == nq.NQ_E_SHAPE
    L = nq.lib()
    assert L.nq_lb_admm(None, 4, 4, 2, None, None, 1, 1.0, 1.0, 0.0, 1, None, None, None, None, None, None, None, 0, None) == nq.NQ_E_NULL
    assert L.nq_dgemm(0, 0, 4, 4, 4, 1.0, None, 4, None, 4, 0.0, None, 4, None) == nq.NQ_E_NULL
    assert L.nq_dgemm(0, 0, 4, 4, 4, 1.0, 8, 3, 8, 4, 0.0, 8, 4, None) == nq.NQ_E_SHAPE      # lda < K
    assert L.nq_dgemm(2, 0, 4, 4, 4, 1.0, 8, 4, 8, 4, 0.0, 8, 4, None) == nq.NQ_E_INVALID_ARG
    assert L.nq_dgemm(0, 0, 4, 4, 4, 1.0, 12, 4, 8, 4, 0.0, 8, 4, None) == nq.NQ_E_ALIGN

"""Host-side checks of the C ABI: the library loads, exports every symbol the header declares,
and rejects bad arguments before touching the GPU.  No compute calls."""
import ctypes
import os
import re

import pytest

import paper_2101_08358_amd as mar
from paper_2101_08358_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(mar.library_path()):
        from paper_2101_08358_amd import build
        build.build()
    return mar.load_library()


def _declared():
    text = open(os.path.join(ROOT, "include", "marius_hip.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mar_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None
        assert hasattr(mar, n), "binding lacks " + n


def test_struct_layouts_match_header():
    assert ctypes.sizeof(mar.MarConfig) == 64
    assert mar.MarConfig.seed.offset == 48 and mar.MarConfig.lr.offset == 36
    assert mar.MarConfig.precision.offset == 56 and mar.MarConfig.reserved.offset == 60
    assert ctypes.sizeof(mar.MarDebugOut) == 7 * 8


def _cfg(**kw):
    base = dict(num_nodes=1000, num_rels=3, dim=50, model=0, batch_size=100, num_chunks=10, negs_per_chunk=20,
                deg_negs_per_chunk=0, lr=0.1, eps=1e-10, init_std=0.001, seed=0)
    base.update(kw)
    return mar.MarConfig(**base)


def test_workspace_bytes_scales_and_validates(lib):
    small = mar.mar_workspace_bytes(_cfg())
    big = mar.mar_workspace_bytes(_cfg(batch_size=1000, negs_per_chunk=200))
    assert 0 < small < big
    assert small % 256 == 0
    for bad, code in ((dict(dim=0), -2), (dict(dim=401), -2), (dict(model=4), -1), (dict(model=1, dim=51), -1),
                      (dict(batch_size=101), -2), (dict(num_chunks=0), -1), (dict(deg_negs_per_chunk=21), -1),
                      (dict(num_nodes=(1 << 31) - 2), -2), (dict(lr=0.0), -1), (dict(num_rels=0), -1),
                      (dict(precision=2), -1), (dict(precision=-1), -1), (dict(precision=1, model=2), -1),
                      (dict(reserved=1), -1),
                      (dict(batch_size=40_000_000, num_chunks=1, negs_per_chunk=100, dim=400), -2),     # 64 GB of rows in one chunk
                      (dict(batch_size=30_000, num_chunks=1, negs_per_chunk=30_000, dim=8), -2)):        # 3.6 GB of pair weights in one chunk
        with pytest.raises(mar.MarError) as e:
            mar.mar_workspace_bytes(_cfg(**bad))
        assert e.value.code == code, bad
        assert mar.mar_last_error() != ""


def test_split_precision_is_a_configuration_of_its_own(lib):
    """The split-precision passes keep operand images instead of stored weights: another workspace size, and the
    bilinear models only."""
    for model in (0, 1, 3):
        a = mar.mar_workspace_bytes(_cfg(model=model, dim=52))
        b = mar.mar_workspace_bytes(_cfg(model=model, dim=52, precision=mar.PRECISION_SPLIT_BF16))
        assert a > 0 and b > 0 and a != b
    for dim in (4, 17, 100, 128, 200, 256, 400):
        assert mar.mar_workspace_bytes(_cfg(dim=dim, precision=1)) % 256 == 0


def test_argument_checks_need_no_gpu(lib):
    cfg = _cfg()
    out = ctypes.c_void_p()
    # null table
    rc = lib.mar_init_tables(ctypes.byref(cfg), None, None, None, None, None, 0, 0, None, ctypes.byref(out))
    assert rc == -1
    # misaligned table pointer, then a too-small workspace (fake non-null addresses; nothing is dereferenced)
    rc = lib.mar_init_tables(ctypes.byref(cfg), 0x1008, 0x2000, 0x3000, 0x4000, 0x10000, 1 << 30, 0, None, ctypes.byref(out))
    assert rc == -1 and b"aligned" in lib.mar_last_error(None)
    rc = lib.mar_init_tables(ctypes.byref(cfg), 0x1000, 0x2000, 0x3000, 0x4000, 0x10000, 1024, 0, None, ctypes.byref(out))
    assert rc == -3
    rc = lib.mar_init_tables(ctypes.byref(cfg), 0x1000, 0x2000, 0x3000, 0x4000, 0x10010, 1 << 30, 0, None, ctypes.byref(out))
    assert rc == -1
    # null context
    assert lib.mar_train_batch(None, None, None, None, 0, None, None, None, None, None) == -1
    assert lib.mar_sample_negatives(None, 0, None, None, 0, None, None, None) == -1
    assert lib.mar_eval_scores(None, None, None, None, 0, None, None, None, None, None, None) == -1
    assert lib.mar_profile_enable(None, 1, 63) == -1
    assert lib.mar_destroy(None) == 0


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(FileNotFoundError):
        binding.load_library()

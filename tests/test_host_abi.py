"""CPU-side checks of the C ABI: the library loads, exports every symbol the header declares,
and its host-only entry points behave as documented.  No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import loract_oracle as orc
from paper_2509_23472_amd import _lib
from paper_2509_23472_amd._lib import LoractParams

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "loract.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(loract_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = _lib.load()
    names = _declared_symbols()
    assert len(names) >= 12
    for name in names:
        assert hasattr(lib, name), "libloract.so does not export %s" % name
        assert name in _lib.SIGNATURES, "binding has no signature for %s" % name


def test_version_and_strerror():
    lib = _lib.load()
    assert lib.loract_version().decode().startswith("loract")
    assert lib.loract_strerror(0).decode() == "ok"
    for code in (-1, -2, -3, -4, -5, -99):
        assert len(lib.loract_strerror(code).decode()) > 0


@pytest.mark.parametrize("m,l", [(1, 1), (10, 3), (17, 17), (1000, 37), (8192, 128), (65536, 256),
                                  (12608, 64)])
def test_sample_indices_agree_with_oracle_definition(m, l):
    # Both sides implement the row sampling of Algorithm 1 independently (splitmix64 + Floyd, sorted).
    lib = _lib.load()
    buf = (ctypes.c_int32 * l)()
    for seed in (0, 1, 2, 12345, 2 ** 63 + 11, 2 ** 64 - 1):
        assert lib.loract_sample_indices(m, l, seed, buf) == 0
        assert list(buf) == orc.sample_indices(m, l, seed).tolist()


def test_sample_indices_reproduce_the_hand_derived_vectors():
    # the library against the hand derivations themselves (tests/golden), not only against the
    # oracle: the vectors include draws that land on an id already chosen
    lib = _lib.load()
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "sample_indices_vectors.txt")
    rows = [[int(t) for t in ln.split()] for ln in open(path) if ln.strip() and not ln.startswith("#")]
    assert len(rows) >= 3
    for m, l, seed, *expected in rows:
        buf = (ctypes.c_int32 * l)()
        assert lib.loract_sample_indices(m, l, seed, buf) == 0
        assert list(buf) == expected


def test_sample_indices_rejects_bad_arguments():
    lib = _lib.load()
    buf = (ctypes.c_int32 * 4)()
    assert lib.loract_sample_indices(3, 4, 0, buf) == -1
    assert lib.loract_sample_indices(10, -1, 0, buf) == -1
    assert lib.loract_sample_indices(10, 2, 0, None) == -1
    assert lib.loract_sample_indices(2 ** 31, 2, 0, buf) == -1


def test_static_scratch_entry_rejects_oversized_shapes_on_the_host():
    # a 65536-row gradient needs 30 MiB of scratch, the built-in buffer holds 16 MiB: refused
    # before any pointer is touched or anything is enqueued (so this runs without a GPU)
    lib = _lib.load()
    assert lib.loract_static_scratch_bytes() == 16 << 20
    need = ctypes.c_size_t(0)
    assert lib.loract_lora_grad_workspace_bytes(65536, 4096, 256, 4096, 16, ctypes.byref(need)) == 0
    assert need.value > lib.loract_static_scratch_bytes()
    fake = ctypes.c_void_p(256)
    rc = lib.loract_lora_grad_static(fake, fake, 65536, 4096, 256, 1, fake, 4096, fake, 16, 1, 1.0, fake, None)
    assert rc == -2
    assert b"16777216" in lib.loract_last_hip_error()
    assert lib.loract_lora_grad_static(fake, fake, 0, 4096, 256, 1, fake, 4096, fake, 16, 1, 1.0, fake, None) == -1


def _params(**kw):
    base = dict(m=1024, n=256, ldx=256, k=16, l=0, t=0, x_dtype=0, factor_dtype=0, seed=0)
    base.update(kw)
    return LoractParams(**base)


def test_workspace_bytes_validation_and_monotonicity():
    lib = _lib.load()
    out = ctypes.c_size_t(0)
    assert lib.loract_workspace_bytes(ctypes.byref(_params()), ctypes.byref(out)) == 0
    small = out.value
    assert small > 0 and small % 256 == 0
    assert lib.loract_workspace_bytes(ctypes.byref(_params(m=8192, n=4096, ldx=4096, k=128, x_dtype=1,
                                                           factor_dtype=1)), ctypes.byref(out)) == 0
    assert out.value > small
    bad = [dict(k=0), dict(k=257), dict(k=2000, m=4096, n=4096, ldx=4096), dict(ldx=255), dict(m=0),
           dict(x_dtype=7), dict(t=-1), dict(l=8), dict(x_dtype=0, factor_dtype=1)]
    for kw in bad:
        assert lib.loract_workspace_bytes(ctypes.byref(_params(**kw)), ctypes.byref(out)) < 0, kw
    assert lib.loract_workspace_bytes(None, ctypes.byref(out)) == -1
    assert lib.loract_workspace_bytes(ctypes.byref(_params()), None) == -1


def test_compress_rejects_bad_arguments_before_touching_the_device():
    # Host-side validation returns before any HIP call, so this is safe without a GPU.
    lib = _lib.load()
    p = _params()
    fake = ctypes.c_void_p(4096)
    assert lib.loract_compress(None, ctypes.byref(p), None, fake, fake, fake, 1 << 30, None, None) == -1
    assert lib.loract_compress(fake, ctypes.byref(p), None, fake, fake, fake, 16, None, None) == -2
    bad_idx = (ctypes.c_int32 * 16)(*([5] * 16))
    assert lib.loract_compress(fake, ctypes.byref(p), bad_idx, fake, fake, fake, 1 << 30, None, None) == -1
    assert lib.loract_reconstruct(fake, fake, 8, 8, 0, 0, fake, 8, 0, None) == -1
    assert lib.loract_reconstruct(fake, fake, 8, 8, 2, 0, fake, 4, 0, None) == -1
    sz = ctypes.c_size_t(0)
    assert lib.loract_lora_grad_workspace_bytes(8, 8, 2, 8, 65, ctypes.byref(sz)) == -1
    assert lib.loract_lora_grad_workspace_bytes(8192, 4096, 128, 4096, 16, ctypes.byref(sz)) == 0
    assert sz.value > 0


def _python_sources(*roots):
    import os
    here = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    for root in roots:
        path = os.path.join(here, root)
        if os.path.isfile(path):
            yield path
            continue
        for dirpath, _, files in os.walk(path):
            for f in files:
                if f.endswith((".py", ".h", ".hip")):
                    yield os.path.join(dirpath, f)


def test_product_path_is_independent_of_the_oracle_and_of_working_files():
    # The oracle is test infrastructure: nothing in the package may import it (the smoke check and
    # the benchmark's cpu_baseline leg are the only callers outside tests/), and nothing committed
    # may reach into the scratch folder or the reference text.
    import re
    for path in _python_sources("paper_2509_23472_amd", "workloads"):
        text = open(path, encoding="utf-8").read()
        assert not re.search(r"^\s*(from|import)\s+oracle\b", text, re.M), path
    for path in _python_sources("paper_2509_23472_amd", "workloads", "oracle", "bench.py",
                                "__graft_entry__.py", "tests"):
        if path.endswith("test_host_abi.py"):
            continue
        text = open(path, encoding="utf-8").read()
        assert "/root/reference" not in text, path
        assert not re.search(r"[\"'/]_work/", text), path
    oracle_text = "".join(open(p, encoding="utf-8").read() for p in _python_sources("oracle"))
    assert "paper_2509_23472_amd" not in oracle_text.replace("must never be imported by the product package", "")


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    # no CPU or eager fallback: without the built shared object the loader raises
    monkeypatch.setattr(_lib, "_lib", None)
    monkeypatch.setattr(_lib, "LIB_PATH", str(tmp_path / "libloract_missing.so"), raising=False)
    try:
        with pytest.raises(Exception):
            _lib.load()
    finally:
        monkeypatch.undo()
        _lib.load()

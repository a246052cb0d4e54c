"""CPU-side checks of the C ABI: the library loads, exports every declared symbol, and rejects bad shapes on the host."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "hts.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hts_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2012_09849_amd import binding
    lib = binding.load_library()
    names = _declared()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def test_param_count_and_shape_rejection():
    import paper_2012_09849_amd as hts
    assert hts.param_count(4, 84, 84, 6) == 1687719
    assert hts.param_count(4, 84, 84, 18) == 1693875
    assert hts.param_count(16, 72, 96, 19) == 1424052
    for bad in [(4, 84, 83, 6), (4, 20, 84, 6), (0, 84, 84, 6), (4, 84, 84, 0), (4, 84, 84, 65)]:
        with pytest.raises(hts.HtsError):
            hts.param_count(*bad)
    with pytest.raises(hts.HtsError):
        hts.param_count(4, 84, 84, 6, precision=7)


def test_strerror():
    from paper_2012_09849_amd import binding
    lib = binding.load_library()
    assert lib.hts_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4):
        assert len(lib.hts_strerror(code)) > 5


def test_null_arguments_rejected_without_gpu():
    from paper_2012_09849_amd import binding
    lib = binding.load_library()
    assert lib.hts_create(None, 1, 1, None, None) == -1
    assert lib.hts_destroy(None) == -1
    assert lib.hts_returns_gae(None, None, None, None, 0.99, 0.95, 4, 4, None, None) == -1
    assert lib.hts_act(None, None, None, 0, 0, 1, 0, None, None, None, None) == -1


def test_bench_refuses_more_than_one_gpu():
    """The benchmark measures one GPU; asking for more exits with a message before anything touches a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)

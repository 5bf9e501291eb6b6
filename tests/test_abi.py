"""CPU-only checks of the boundary: the library loads, exports every symbol the
header declares, and rejects unsupported shapes without touching a GPU."""
import ctypes
import os
import re
import shutil
import subprocess

import pytest

import paper_1412_4944_amd as sbo

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "sbo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sbo_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert set(names) == set(sbo.EXPORTS)
    L = sbo.lib()
    for n in names:
        assert getattr(L, n) is not None


def test_workspace_bytes_and_shape_rejection():
    assert sbo.sbo_workspace_bytes(64, 32, 8, 262144) > 262144 * 8
    assert sbo.sbo_workspace_bytes(64, 32, 8, 1 << 20) > sbo.sbo_workspace_bytes(64, 32, 8, 1 << 10)
    for bad in [(48, 4, 3, 100), (64, 0, 3, 100), (64, 4, 0, 100), (64, 4, 17, 100),
                (16, 4, 3, 0), (64, 2000, 3, 100), (64, 4, 3, 1 << 31)]:
        assert sbo.sbo_workspace_bytes(*bad) == 0
        h = ctypes.c_void_p()
        rc = sbo.lib().sbo_create(ctypes.byref(h), bad[0], bad[1], bad[2], bad[3], None)
        assert rc == sbo.binding.SBO_EINVAL and not h.value
    assert sbo.lib().sbo_create(None, 64, 4, 3, 100, None) == sbo.binding.SBO_EINVAL


def test_strerror_and_null_context():
    assert sbo.sbo_strerror(0) == "success"
    assert "invalid" in sbo.sbo_strerror(-1)
    assert "memory" in sbo.sbo_strerror(-2)
    assert sbo.sbo_strerror(-77) == "unknown error code"
    L = sbo.lib()
    assert L.sbo_destroy(None) == sbo.binding.SBO_EINVAL
    assert L.sbo_set_timing(None, 1) == sbo.binding.SBO_EINVAL
    assert L.sbo_code(None, None, 1, None, None, None, None, None) == sbo.binding.SBO_EINVAL


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not installed")
def test_compare_exchange_networks_on_host(tmp_path):
    exe = str(tmp_path / "host_networks")
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-O1", "-std=c++17",
                        os.path.join(ROOT, "tests", "host_networks.hip"), "-o", exe],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    r = subprocess.run([exe], capture_output=True, text=True)
    assert r.returncode == 0 and r.stdout.strip() == "ok", r.stdout[-2000:]


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    """No CPU fallback: with the shared library absent the binding raises instead of
    computing anything some other way."""
    import paper_1412_4944_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "LIB_PATH", str(tmp_path / "libsbo.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        b.lib()
    with pytest.raises(RuntimeError):
        b.sbo_workspace_bytes(64, 4, 8, 1024)

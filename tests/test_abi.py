"""Host-only checks of the C-ABI library: it loads and exports every symbol the headers under include/ declare."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    names = set()
    inc = os.path.join(ROOT, "include")
    for h in sorted(os.listdir(inc)):
        if h.endswith(".h"):
            src = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, h)).read(), flags=re.S)
            names |= set(re.findall(r"\b(sev_[a-z_0-9]+)\s*\(", src))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    from paper_2505_17052_amd import binding
    names = _declared()
    assert "sev_verify" in names and "sev_kv_commit" in names and "sev_kv_rollback" in names and "sev_sched_next_batch" in names
    L = binding.lib()
    for n in names:
        assert hasattr(L, n), n


def test_host_side_validation_without_gpu():
    """Calls that fail validation never reach the device, so they can be exercised on a CPU-only box."""
    from paper_2505_17052_amd import binding
    L = binding.lib()
    bad = binding.ModelDesc(2, 256, 4, 3, 64, 688, 1024, 10000.0, 1e-5, 0)       # 4 heads over 3 KV heads
    assert L.sev_model_arena_bytes(ctypes.byref(bad)) == 0
    assert b"multiple" in L.sev_last_error()
    ok = binding.ModelDesc(2, 256, 4, 4, 64, 688, 1024, 10000.0, 1e-5, 0)
    assert L.sev_model_arena_bytes(ctypes.byref(ok)) >= 4 * (2 * 1024 * 256 + 2 * (3 * 256 * 256 + 256 * 256 + 3 * 256 * 688))
    bf = binding.ModelDesc(2, 256, 4, 4, 64, 688, 1024, 10000.0, 1e-5, 1)        # bf16 path needs head_dim 128
    assert L.sev_model_arena_bytes(ctypes.byref(bf)) == 0
    h = ctypes.c_void_p()
    assert L.sev_model_create(ctypes.byref(ok), None, 0, ctypes.byref(h)) == -1
    assert L.sev_verify(None, None, None, None, None, 1, 1, None, None, None) == -1


def test_bench_refuses_more_than_one_gpu():
    """bench.py runs on one GPU only: any other --gpus value ends with a message and a non-zero status before torch is imported."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=60)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""

"""The memory-system probe (a measurement tool outside the library): its library builds and exports its entry point
(CPU), and it runs on small arrays and rejects what it does not support (GPU)."""
import ctypes
import os
import subprocess
import sys

import pytest

from paper_2502_11034_amd import build as lib_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_probe_library_exports_its_entry_point():
    path = os.path.join(lib_build.HERE, "libadagc_probe.so")
    if not os.path.exists(path):
        lib_build.build_probe()
    L = ctypes.CDLL(path)
    assert hasattr(L, "adagc_probe_stream")


@pytest.mark.gpu
def test_probe_runs_and_checks_its_arguments():
    import torch
    from paper_2502_11034_amd import memory_probe
    L = memory_probe.lib()
    arrays = [torch.zeros(8192, dtype=torch.float32, device="cuda:0") for _ in range(4)]
    ptrs = (ctypes.c_void_p * 4)(*[a.data_ptr() for a in arrays])
    assert L.adagc_probe_stream(ptrs, 4, 3, 8192, None) == 0
    torch.cuda.synchronize()
    # 4 reads + 3 in-place writes of zeros: v = (1,2,3,4) + 0, array s gets v * (s + 1); the fourth array is only read
    assert arrays[0][:4].tolist() == [1.0, 2.0, 3.0, 4.0] and arrays[2][:4].tolist() == [3.0, 6.0, 9.0, 12.0]
    assert float(arrays[3].abs().max()) == 0.0
    assert L.adagc_probe_stream(ptrs, 4, 3, 8192 + 4, None) == -1          # not a multiple of the item size
    assert L.adagc_probe_stream(ptrs, 3, 2, 8192, None) == -1              # a mix it has no kernel for
    out = subprocess.run([sys.executable, "-m", "paper_2502_11034_amd.memory_probe", "--gib-per-array", "0.0625", "--reps", "1"],
                         cwd=ROOT, capture_output=True, text=True, timeout=120)
    assert out.returncode == 0 and "4 : 3 (in place)" in out.stdout

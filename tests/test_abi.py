"""The C-ABI library loads, exports every symbol its header declares, and validates arguments
before touching a device.  No compute calls: runs without a GPU."""
import ctypes
import os
import re

import pytest

from paper_2502_11034_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "adagc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(adagc_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported():
    L = B.lib()
    names = declared_symbols()
    assert len(names) >= 14
    for name in names:
        assert hasattr(L, name), name
    assert sorted(B.EXPORTS) == names


def test_struct_layouts_match_header():
    assert ctypes.sizeof(B.adagc_tensor_desc) == 16
    assert ctypes.sizeof(B.adagc_config) == 44
    assert ctypes.sizeof(B.adagc_step_params) == 56
    assert ctypes.sizeof(B.adagc_hyper) == 44


def test_strerror():
    assert B.strerror(0) == "ok"
    assert "invalid" in B.strerror(B.ADAGC_ERR_INVALID_ARG)
    assert B.strerror(-999) == "unknown error code"


def _create(numels, **cfg_kw):
    L = B.lib()
    ctx = ctypes.c_void_p(None)
    fields = dict(optimizer=0, grad_dtype=0, has_bf16_param_copy=0, telemetry=0, grid_blocks=0, unroll=0, nontemporal=0, schedule=0,
                  update_split=0, schedule_run=0)
    fields.update(cfg_kw)
    cfg = B.adagc_config(**fields)
    descs = (B.adagc_tensor_desc * max(1, len(numels)))()
    for i, n in enumerate(numels):
        descs[i].numel = n
    rc = L.adagc_create(ctypes.byref(ctx), ctypes.cast(descs, ctypes.c_void_p), len(numels), ctypes.byref(cfg))
    return rc, ctx


def test_create_validates_before_touching_the_device():
    L = B.lib()
    assert _create([])[0] == B.ADAGC_ERR_INVALID_ARG
    assert _create([4, 0])[0] == B.ADAGC_ERR_INVALID_ARG
    assert _create([4], optimizer=7)[0] == B.ADAGC_ERR_INVALID_ARG
    assert _create([4], grad_dtype=2)[0] == B.ADAGC_ERR_INVALID_ARG
    assert _create([4], has_bf16_param_copy=3)[0] == B.ADAGC_ERR_INVALID_ARG
    assert _create([4], unroll=3)[0] == B.ADAGC_ERR_INVALID_ARG
    assert _create([4], grid_blocks=-1)[0] == B.ADAGC_ERR_INVALID_ARG
    assert _create([4], telemetry=2)[0] == B.ADAGC_ERR_INVALID_ARG
    assert _create([4], nontemporal=3)[0] == B.ADAGC_ERR_INVALID_ARG
    assert _create([4], update_split=3)[0] == B.ADAGC_ERR_INVALID_ARG
    assert _create([4], update_split=8)[0] == B.ADAGC_ERR_INVALID_ARG      # more than 16384 / (4*1024)
    assert _create([4], update_split=16, unroll=2)[0] == B.ADAGC_ERR_INVALID_ARG
    assert _create([4], schedule_run=-1)[0] == B.ADAGC_ERR_INVALID_ARG
    cfg = B.adagc_config()
    assert L.adagc_create(None, None, 1, ctypes.byref(cfg)) == B.ADAGC_ERR_INVALID_ARG
    rc, ctx = _create([4])
    assert ctx.value is None or rc == B.ADAGC_OK
    if rc == B.ADAGC_OK:       # a GPU is present
        L.adagc_destroy(ctx)
    else:                      # no device: a clean error, not a crash
        assert rc == B.ADAGC_ERR_HIP


def test_create_rejects_a_list_with_too_many_tensors():
    """One workgroup per tensor in the per-tensor kernels bounds the tensor count at 2^24 - 1; the check
    comes before anything touches the device."""
    import numpy as np
    L = B.lib()
    n = 1 << 24
    descs = np.zeros(n, dtype=[("numel", "<i8"), ("flags", "<u4"), ("reserved", "<u4")])
    descs["numel"] = 1
    cfg = B.adagc_config()
    ctx = ctypes.c_void_p()
    rc = L.adagc_create(ctypes.byref(ctx), ctypes.c_void_p(descs.ctypes.data), n, ctypes.byref(cfg))
    assert rc == B.ADAGC_ERR_TOO_LARGE and ctx.value is None


def test_null_context_is_rejected_everywhere():
    L = B.lib()
    hp = B.make_hyper()
    assert L.adagc_step(None, None, None, None, None, None, ctypes.byref(hp), 1, None) == B.ADAGC_ERR_INVALID_ARG
    assert L.adagc_step_graph(None, None, None, None, None, None, None, None) == B.ADAGC_ERR_INVALID_ARG
    assert L.adagc_get_norms(None, None, None, None, 1, None) == B.ADAGC_ERR_INVALID_ARG
    assert L.adagc_get_state_norms(None, None, None, None, 1, None) == B.ADAGC_ERR_INVALID_ARG
    assert L.adagc_set_param_copies(None, None) == B.ADAGC_ERR_INVALID_ARG
    assert L.adagc_get_segment_table(None, None, None, None) == B.ADAGC_ERR_INVALID_ARG
    assert L.adagc_profile_begin(None, 4) == B.ADAGC_ERR_INVALID_ARG
    assert L.adagc_num_chunks(None) < 0 and L.adagc_num_tensors(None) < 0
    L.adagc_destroy(None)   # no-op


def test_header_is_plain_c_and_links_against_the_library(tmp_path):
    """include/adagc.h compiles as C99 with -pedantic, its struct sizes are the ones the binding assumes, and a C
    program that only uses the host-side entry points links against libadagc.so and runs without a GPU."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("needs gcc")
    src = tmp_path / "use_header.c"
    src.write_text(r'''
#include <stdio.h>
#include "adagc.h"
int main(void)
{
    adagc_tensor_desc d[3] = {{5, 0, 0}, {40000, 0, 0}, {1, 0, 0}};
    int64_t begin[4], total = 0;
    uint32_t order[8];
    if (adagc_build_segment_table(d, 3, adagc_chunk_elems(), begin, NULL, NULL, 0, &total) != ADAGC_OK) return 1;
    if (total != 5 || begin[3] != 5) return 2;
    if (adagc_build_visiting_order(8, 2, 8, order) != ADAGC_OK) return 3;
    if (adagc_step(NULL, NULL, NULL, NULL, NULL, NULL, NULL, 1, NULL) != ADAGC_ERR_INVALID_ARG) return 4;
    printf("%d %d %d %s\n", (int)sizeof(adagc_tensor_desc), (int)sizeof(adagc_config), (int)sizeof(adagc_hyper),
           adagc_strerror(ADAGC_ERR_STATE));
    return 0;
}
''')
    lib = B._build.LIB
    exe = str(tmp_path / "use_header")
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", exe, lib, "-Wl,-rpath," + os.path.dirname(lib)], check=True)
    res = subprocess.run([exe], capture_output=True, text=True, timeout=60)
    assert res.returncode == 0, res.stdout + res.stderr
    assert res.stdout.split()[:3] == ["16", "44", "44"]
    assert "wrong state" in res.stdout

"""Build libadagc.so for gfx950 with hipcc, in-tree (next to this file)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libadagc.so")
SOURCES = ["api.cpp", "segment_table.cpp", "kernels.hip", "static_step.hip", "muon_gemm.hip", "muon.hip"]
HEADERS = [os.path.join(ROOT, "include", "adagc.h"), os.path.join(CSRC, "adagc_internal.h"), os.path.join(CSRC, "muon_internal.h")]


def hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def is_stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + HEADERS
    return any(os.path.getmtime(d) > t for d in deps)


def build(force=True, verbose=False, extra_flags=(), out=None):
    """Compile every source for gfx950 and link the shared library.  Cross-compiles without a GPU.
    extra_flags/out build a variant (e.g. another chunk size) somewhere else, for measurements."""
    out = out or LIB
    if out == LIB and not force and not is_stale():
        return LIB
    tmp = out + ".tmp.%d" % os.getpid()
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           # packed-fp32 code generation is switched off on purpose (known-bad forms on this part)
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wextra", "-Wno-unused-parameter",
           "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-x", "hip"]
    cmd += list(extra_flags)
    cmd += [os.path.join(CSRC, s) for s in SOURCES]
    cmd += ["-o", tmp]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)
    os.replace(tmp, out)
    return out


def build_probe():
    """libadagc_probe.so: the memory-system probe (csrc/memory_probe.hip), a measurement tool outside the library."""
    out = os.path.join(HERE, "libadagc_probe.so")
    tmp = out + ".tmp.%d" % os.getpid()
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wextra", "-x", "hip",
           os.path.join(CSRC, "memory_probe.hip"), "-o", tmp]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stderr)
    os.replace(tmp, out)
    return out


if __name__ == "__main__":
    print(build(force=True, verbose=True))
    print(build_probe())

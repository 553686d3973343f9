"""Build the HIP library in-tree: paper_2504_19449_amd/librsparse.so (gfx950 only)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librsparse.so")
LIB_STAMPS = os.path.join(HERE, "librsparse_stamps.so")     # measurement build, loaded only on request (RSPARSE_LIB)
SOURCES = ["kernels.hip", "kernels_strip.hip", "kernels_mfma.hip", "kernels_topk.hip", "kernels_q4row.hip", "static_scratch.hip", "api.cpp", "svd_host.cpp", "recipe_search.cpp"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
         # keep the compiler from forming packed-fp32 instructions on its own
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-munsafe-fp-atomics", "-Wall", "-Wno-unused-command-line-argument"]


def is_current() -> bool:
    if not os.path.exists(LIB):
        return False
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(HERE, "..", "include", "rsparse.h")]
    return all(os.path.getmtime(d) <= t for d in deps)


def build(force: bool = True, stamps: bool = False) -> str:
    """stamps=True (or RSPARSE_STAMPS=1 in the environment): a measurement build whose strip kernel records per-wave
    phase time stamps (rsparse_debug_stamps).  It goes to librsparse_stamps.so, which nothing loads unless the
    environment names it in RSPARSE_LIB (`bench.py --stamps` does)."""
    stamps = stamps or os.environ.get("RSPARSE_STAMPS") == "1"
    if not stamps and not force and is_current():
        return LIB
    lib = LIB_STAMPS if stamps else LIB
    objs = []
    procs = []
    os.makedirs(os.path.join(HERE, "_build"), exist_ok=True)
    for src in SOURCES:
        obj = os.path.join(HERE, "_build", src + (".stamps.o" if stamps else ".o"))
        objs.append(obj)
        procs.append((src, subprocess.Popen([HIPCC, *FLAGS, *(["-DRSPARSE_STAMPS=1"] if stamps else []), "-c",
                                             os.path.join(CSRC, src), "-o", obj],
                                            stderr=subprocess.PIPE, text=True)))
    for src, p in procs:
        _, err = p.communicate()
        err = "\n".join(l for l in err.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{err}")
        if err.strip():
            sys.stderr.write(err + "\n")
    subprocess.run([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", lib, *objs], check=True)
    return lib


if __name__ == "__main__":
    print(build(force=True, stamps="--stamps" in sys.argv))

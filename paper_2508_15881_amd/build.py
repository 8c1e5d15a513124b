"""Builds libtpla.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2508_15881_amd.build

Objects go to <repo>/_build/, the library to paper_2508_15881_amd/lib/.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
INCLUDE = os.path.join(ROOT, "include")
OBJ_DIR = os.path.join(ROOT, "_build")
LIB_DIR = os.path.join(PKG, "lib")
# TPLA_LIB_NAME: file name of the library to write (measurement builds with extra flags get their own name
# and object folder, so the default library stays as it is)
LIB_NAME = os.environ.get("TPLA_LIB_NAME", "libtpla.so")
LIB_PATH = os.path.join(LIB_DIR, LIB_NAME)
if LIB_NAME != "libtpla.so":
    OBJ_DIR = os.path.join(OBJ_DIR, LIB_NAME.replace(".so", ""))

SOURCES = ["api.hip", "decode_mfma.hip", "decode_generic.hip", "transform.hip", "transform_mfma.hip", "absorb_combine.hip",
           "absorb_combine_mfma.hip", "pca.hip", "prefill_mfma.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    # packed-fp32 instruction selection is switched off for every device TU
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-I", INCLUDE, "-I", CSRC,
] + os.environ.get("TPLA_EXTRA_HIPCC_FLAGS", "").split()


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if r.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build(verbose=True):
    os.makedirs(OBJ_DIR, exist_ok=True)
    os.makedirs(LIB_DIR, exist_ok=True)
    objs = [os.path.join(OBJ_DIR, s.replace(".hip", ".o")) for s in SOURCES]

    def compile_one(i):
        return _run([HIPCC] + FLAGS + ["-c", os.path.join(CSRC, SOURCES[i]), "-o", objs[i]])

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        for s, out in zip(SOURCES, ex.map(compile_one, range(len(SOURCES)))):
            if verbose and out:
                print("[%s]\n%s" % (s, out))
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH] + objs)
    if verbose:
        print("built", LIB_PATH)
    return LIB_PATH


def device_assembly(source, extra_flags=()):
    """The gfx950 assembly hipcc generates for one source file of csrc/, as text (same flags as build()).
    Used by tests/test_isa_lds_waits.py, which checks this build's own kernels on the CPU machine."""
    out_dir = os.path.join(OBJ_DIR, "asm")
    os.makedirs(out_dir, exist_ok=True)
    path = os.path.join(out_dir, source.replace(".hip", ".s"))
    _run([HIPCC] + FLAGS + list(extra_flags) + ["-S", "--cuda-device-only", os.path.join(CSRC, source), "-o", path])
    with open(path) as f:
        return f.read()


def build_host_sanitized(driver_cpp, exe_path, verbose=False):
    """Second build configuration, for the CPU machine only: the same sources with AddressSanitizer
    and UndefinedBehaviorSanitizer on the HOST code (device code is compiled as usual, unsanitised),
    linked with a C++ driver into an executable -- the sanitizer runtime is linked statically into
    it, so nothing has to be preloaded.  Used by tests/test_host_sanitizers.py; never run on a GPU machine."""
    obj_dir = os.path.join(OBJ_DIR, "host_sanitized")
    os.makedirs(obj_dir, exist_ok=True)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined"]
    flags = ["--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fno-omit-frame-pointer",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
             "-I", INCLUDE, "-I", CSRC] + san
    objs = [os.path.join(obj_dir, s.replace(".hip", ".o")) for s in SOURCES]

    def compile_one(i):
        return _run([HIPCC] + flags + ["-c", os.path.join(CSRC, SOURCES[i]), "-o", objs[i]])

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        outs = list(ex.map(compile_one, range(len(SOURCES))))
    drv_obj = os.path.join(obj_dir, "driver.o")
    host_san = ["-fsanitize=address,undefined", "-fno-gpu-sanitize", "-fno-sanitize-recover=undefined",
                "-Wno-unused-command-line-argument"]
    outs.append(_run([HIPCC, "-O1", "-g", "-std=c++17", "-I", INCLUDE, "-I", CSRC, "--offload-arch=gfx950", "-x", "hip", driver_cpp,
                      "-c", "-o", drv_obj] + san + ["-Wno-unused-command-line-argument"]))
    outs.append(_run([HIPCC] + host_san + objs + [drv_obj, "-o", exe_path]))
    if verbose:
        print("\n".join(o for o in outs if o))
    return exe_path


if __name__ == "__main__":
    build()
    sys.exit(0)

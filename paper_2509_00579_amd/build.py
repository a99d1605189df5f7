"""Build libkvcomp.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import pathlib
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = pathlib.Path(__file__).resolve().parent
CSRC = HERE / "csrc"
LIB = HERE / "libkvcomp.so"
OBJ = HERE / "_build"
SOURCES = ["kvcomp_api.hip", "quantize.hip", "encode.hip", "attn_fused.hip", "attn_fp16.hip", "decompress.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
    "-fhip-fp32-correctly-rounded-divide-sqrt",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-pragmas",
]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def _compile(src: str) -> pathlib.Path:
    obj = OBJ / (src + ".o")
    cmd = [_hipcc(), *FLAGS, "-c", str(CSRC / src), "-o", str(obj)]
    r = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    # the host pass does not know the gfx-only -packed-fp32-ops feature and says so once per function: harmless
    noise = "'-packed-fp32-ops' is not a recognized feature"
    err = "\n".join(line for line in r.stderr.splitlines() if noise not in line)
    if err.strip():
        print(err, flush=True)
    if r.returncode:
        raise subprocess.CalledProcessError(r.returncode, cmd)
    return obj


def build(verbose: bool = False, extra_flags=(), out: pathlib.Path | None = None) -> pathlib.Path:
    """Compile all sources and link the shared library (extra_flags / out: experimental variants)."""
    global FLAGS, OBJ
    lib = pathlib.Path(out) if out else LIB
    saved = (FLAGS, OBJ)
    if extra_flags:
        FLAGS = FLAGS + list(extra_flags)
        OBJ = HERE / "_build" / ("var_" + lib.stem)
    OBJ.mkdir(parents=True, exist_ok=True)
    try:
        with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
            objs = list(ex.map(_compile, SOURCES))
    finally:
        FLAGS, OBJ = saved
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(lib), *map(str, objs)]
    subprocess.run(cmd, check=True)
    if verbose:
        print(lib)
    return lib


def device_assembly(src: str) -> str:
    """gfx950 assembly text of one source file, compiled with the library's flags (for checks on the generated code)."""
    cmd = [_hipcc(), *FLAGS, "--cuda-device-only", "-S", str(CSRC / src), "-o", "-"]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.DEVNULL, text=True, check=True)
    return r.stdout


if __name__ == "__main__":
    build(verbose=True)

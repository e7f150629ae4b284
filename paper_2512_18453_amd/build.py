"""Build libnova.so (HIP kernels + C ABI) for gfx950, in-tree.

    python -m paper_2512_18453_amd.build            # compile what changed, link
    python -m paper_2512_18453_amd.build --force    # compile everything
    python -m paper_2512_18453_amd.build --sanitize # host sources under AddressSanitizer + UBSan (no GPU code)

hipcc cross-compiles for gfx950 without a GPU.  -ffp-contract=off: the kernels spell out
every fused multiply-add themselves, because the binary32 input transform has a fixed
operation order.  The packed-FP32 instructions are switched off for the device pass.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libnova.so")

SOURCES = ["transforms.cpp", "discovery.cpp", "api.cpp", "filter_transform.hip", "input_transform.hip",
           "contract.hip", "output_transform.hip", "pool.hip", "static_workspace.hip", "int8.hip", "fused_output.hip"]
COMMON = ["-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-Wall", "-Wno-unused-function"]
DEVICE = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _newest_header():
    headers = [os.path.join(SRC, f) for f in os.listdir(SRC) if f.endswith(".hpp")]
    headers.append(os.path.join(HERE, "..", "include", "nova.h"))
    return max(os.path.getmtime(h) for h in headers)


def _compile(name, force):
    src = os.path.join(SRC, name)
    obj = os.path.join(OBJ, name + ".o")
    if (not force and os.path.exists(obj)
            and os.path.getmtime(obj) > max(os.path.getmtime(src), _newest_header())):
        return obj
    cmd = ["hipcc"] + COMMON + (DEVICE if name.endswith(".hip") else []) + ["-c", src, "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(ln for ln in res.stderr.splitlines() if noise not in ln)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {name}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(force=False):
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        objs = list(pool.map(lambda s: _compile(s, force), SOURCES))
    subprocess.check_call(["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs)
    return LIB


SANITIZE = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-static-libasan",
            "-static-libubsan", "-fno-omit-frame-pointer"]


def sanitize_selftest():
    """The host-only sources of the library (exact construction, point discovery) and the oracle's C loops,
    each compiled with AddressSanitizer and UndefinedBehaviorSanitizer into a program of its own that walks
    through their entry points (csrc/host_selftest.cpp, oracle/conv_oracle_selftest.c), and run.  Programs
    rather than a sanitized libnova.so: a sanitizer runtime cannot be loaded into a running Python.  GPU code
    is not part of it.  Returns what the two programs printed; raises if one of them fails."""
    os.makedirs(OBJ, exist_ok=True)
    oracle_dir = os.path.join(HERE, "..", "oracle")
    host = os.path.join(OBJ, "host_selftest_sanitized")
    orac = os.path.join(OBJ, "conv_oracle_selftest_sanitized")
    subprocess.check_call(["g++", "-std=c++17", "-pthread"] + SANITIZE + ["-o", host] +
                          [os.path.join(SRC, f) for f in ("host_selftest.cpp", "transforms.cpp", "discovery.cpp")])
    subprocess.check_call(["gcc", "-std=c11", "-ffp-contract=off", "-fopenmp"] + SANITIZE +
                          ["-o", orac, os.path.join(oracle_dir, "conv_oracle_selftest.c"), "-lm"])
    out = []
    for prog in (host, orac):
        res = subprocess.run([prog], capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"{os.path.basename(prog)} failed ({res.returncode}):\n{res.stdout}\n{res.stderr}")
        out.append(res.stdout.strip())
    return out


if __name__ == "__main__":
    if "--sanitize" in sys.argv:
        print("\n".join(sanitize_selftest()))
    else:
        print(build(force="--force" in sys.argv))

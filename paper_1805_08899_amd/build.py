"""Builds libechoattn.so from csrc/*.hip for gfx950 with hipcc (in-tree).

    python -m paper_1805_08899_amd.build [--sanitize] [extra hipcc flags]

Objects go to paper_1805_08899_amd/_build/, the library next to this file.
hipcc cross-compiles without a GPU present.

--sanitize builds a second library, _build/libechoattn_san.so, whose HOST code carries AddressSanitizer and
UndefinedBehaviorSanitizer instrumentation (the device code is built as usual: sanitizers for device code are not
available here).  It is for the host-side walk through the argument checks in tests/host/, never for the GPU.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libechoattn.so")

# Packed fp32 VALU forms are switched off for all device code.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-parameter",
]


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))


SAN_LIB = os.path.join(OBJ, "libechoattn_san.so")
# each -fsanitize= directly behind -Xarch_host, so that only the host pass sees it
SAN_COMPILE = ["-g", "-fno-omit-frame-pointer", "-Xarch_host", "-fsanitize=address", "-Xarch_host",
               "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined"]
SAN_LINK = ["-fsanitize=address,undefined", "-fno-gpu-sanitize", "-shared-libsan"]


def _compile(src: str, extra, suffix: str = "") -> str:
    obj = os.path.join(OBJ, os.path.basename(src)[:-4] + suffix + ".o")
    cmd = ["hipcc", *HIPCC_FLAGS, *extra, "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    msgs = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                     if "is not a recognized feature for this target" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{msgs}")
    if msgs.strip():
        print(msgs, file=sys.stderr)
    return obj


def build_library(extra_flags=(), verbose=True, sanitize=False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    srcs = sources()
    flags = list(extra_flags) + (SAN_COMPILE if sanitize else [])
    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(lambda s: _compile(s, flags, "_san" if sanitize else ""), srcs))
    out = SAN_LIB if sanitize else LIB
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *(SAN_LINK if sanitize else []), "-o", out, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout + r.stderr)
    if verbose:
        print(f"built {out} from {len(srcs)} sources")
    return out


if __name__ == "__main__":
    args = sys.argv[1:]
    san = "--sanitize" in args
    build_library([a for a in args if a != "--sanitize"], sanitize=san)

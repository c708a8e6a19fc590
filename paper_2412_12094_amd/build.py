"""Build libsepattn.so (HIP, gfx950) in-tree with hipcc.  Run as `python -m paper_2412_12094_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libsepattn.so")
SOURCES = ["api.hip", "mark_compact.hip", "attn_fp32.hip", "fwd_bf16.hip", "bwd_bf16.hip", "bwd_dkv_bf16.hip", "decode.hip", "decode_mfma.hip", "decode_noalloc.hip",
           "evict.hip", "cache_fill.hip", "rope_table.hip", "cache_append.hip", "doc_bounds.hip"]
# packed fp32 VALU instructions are switched off (some of their forms have miscomputed on
# the test machines); the host pass does not know the feature and says so, which is harmless
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def _compile(src: str, extra) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = ["hipcc", *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(extra_flags=(), lib_path: str = LIB) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile(s, list(extra_flags)), SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", lib_path]
    subprocess.run(cmd, check=True)
    return lib_path


if __name__ == "__main__":
    print(build(sys.argv[1:]))

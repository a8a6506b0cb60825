"""Builds libmixdq.so (gfx950) in-tree with hipcc.  Object files are cached per source; pass force=True to
rebuild everything."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.environ.get("MQ_CSRC_DIR", os.path.join(HERE, "csrc"))
OBJ = os.environ.get("MQ_OBJ_DIR", os.path.join(HERE, "_build"))
LIB = os.environ.get("MQ_LIB_OUT", os.path.join(HERE, "libmixdq.so"))
EXTRA = os.environ.get("MQ_EXTRA_FLAGS", "").split()
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
          "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option"]
# The quantisers decide integer codes: every fp32 operation must round once.
PER_FILE = {
    "quant_pack.hip": ["-ffp-contract=off"],
    "act_quant.hip": ["-ffp-contract=off"],
    "alloc.cpp": ["-ffp-contract=off"],  # budgets are floors of double products: no fused multiply-add
    # The epilogue converts four results per lane to 16 bits; the SLP vectoriser pairs the middle two and then needs
    # three more instructions per four values to put the halves where the store wants them.
    "gemm.hip": ["-fno-slp-vectorize"],
}
SOURCES = ["api.hip", "quant_pack.hip", "act_quant.hip", "gemm.hip", "bos.hip", "prof.hip", "peaks.hip", "alloc.cpp"]


def _compile(src: str, force: bool) -> str:
    path = os.path.join(CSRC, src)
    obj = os.path.join(OBJ, src + ".o")
    deps = [path, os.path.join(CSRC, "mq_common.h"), os.path.join(CSRC, "bos_rows.h"),
            os.path.join(HERE, "..", "include", "mixdq.h"), __file__]
    if not force and os.path.exists(obj) and all(os.path.getmtime(obj) >= os.path.getmtime(d) for d in deps):
        return obj
    cmd = [HIPCC, *COMMON, *EXTRA, *PER_FILE.get(src, []), "-c", path, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        errs = [l for l in (r.stdout + r.stderr).splitlines() if "error" in l]
        sys.stderr.write("\n".join(errs[:20]) + "\n")
        raise RuntimeError(f"hipcc failed on {src}")
    warn = [l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip()]
    if warn:
        sys.stderr.write("\n".join(warn) + "\n")
    return obj


def build(force: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), SOURCES))
    if force or not os.path.exists(LIB) or any(os.path.getmtime(o) > os.path.getmtime(LIB) for o in objs):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            sys.stderr.write(r.stdout + r.stderr)
            raise RuntimeError("link failed")
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))

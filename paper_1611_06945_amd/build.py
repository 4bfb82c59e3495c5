"""Build libconvfwd.so from csrc/ with hipcc for gfx950 (cross-compiles without a GPU).

    python -m paper_1611_06945_amd.build [--force] [--jobs N]

Objects go to <repo>/_build/ (not committed); the shared library is written next
to this file so that it travels with the tree.
"""
from __future__ import annotations

import argparse
import concurrent.futures as cf
import os
import subprocess
import sys
import time

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ_DIR = os.path.join(ROOT, "_build")
LIB = os.path.join(PKG, "libconvfwd.so")

SOURCES = ["api.hip", "igemm_f32.hip", "igemm_f16.hip", "igemm_bf16.hip", "ugemm_f32.hip", "ugemm_f16.hip", "ugemm_bf16.hip", "fc_kernels.hip", "nhwc_f16.hip", "nhwc_bf16.hip", "nwin_f16.hip", "nwin_bf16.hip", "wconv_f32.hip", "wconv_f16.hip", "wconv_bf16.hip", "wino_f32.hip", "swin_f16.hip", "swin_bf16.hip", "swinp_f16.hip", "swinp_bf16.hip", "pwin_f16.hip", "pwin_bf16.hip", "pwk_f32.hip", "pwk_f16.hip", "pwk_bf16.hip", "pwin32_f32.hip", "aux_kernels.hip", "probe_kernels.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-value", "-Wno-unknown-warning-option",
]


def _headers():
    hs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    hs.append(os.path.join(ROOT, "include", "convfwd.h"))
    return hs


def _stale(target, deps):
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def _compile(src, obj):
    cmd = [HIPCC] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    t0 = time.time()
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in p.stdout.splitlines() if "packed-fp32-ops" not in l)  # host pass does not know the feature
    return src, p.returncode, out, time.time() - t0


def build(force: bool = False, jobs: int = 0, verbose: bool = True) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    heads = _headers()
    todo, objs = [], []
    for s in SOURCES:
        obj = os.path.join(OBJ_DIR, s.replace(".hip", ".o"))
        objs.append(obj)
        if force or _stale(obj, [os.path.join(CSRC, s)] + heads):
            todo.append((s, obj))
    jobs = jobs or min(len(todo) or 1, int(os.environ.get("MAX_JOBS", "8")), os.cpu_count() or 1)
    failed = False
    with cf.ThreadPoolExecutor(max_workers=jobs) as ex:
        for src, rc, out, dt in ex.map(lambda so: _compile(*so), todo):
            if verbose:
                print("[build] %-18s %s in %.1fs" % (src, "ok" if rc == 0 else "FAILED", dt), flush=True)
            if out.strip() and (rc != 0 or verbose):
                print(out, flush=True)
            failed |= rc != 0
    if failed:
        raise RuntimeError("hipcc failed")
    if force or todo or _stale(LIB, objs):
        tmp = LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs)
        os.replace(tmp, LIB)
        if verbose:
            print("[build] linked %s" % LIB, flush=True)
    return LIB


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--force", action="store_true")
    ap.add_argument("--jobs", type=int, default=0)
    a = ap.parse_args()
    build(force=a.force, jobs=a.jobs)
    sys.exit(0)

"""Build libnmconv.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2507_17301_amd.build [-j N] [--force]

Objects go to ``_build/`` at the repository root (never committed); the shared
library is written next to this file so that it travels with the tree.
"""
from __future__ import annotations

import argparse
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
INCLUDE = os.path.join(ROOT, "include")
OBJDIR = os.path.join(ROOT, "_build")
LIB = os.path.join(PKG, "libnmconv.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function",
    # ragged-tail loops of some tile shapes keep a run-time trip count; their unroll hint is best-effort
    "-Wno-pass-failed",
    # the compiler must not form packed fp32 instructions on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # MFMA accumulators stay in ordinary VGPRs: with the AGPR form the register
    # allocator shuffles them through v_accvgpr moves inside the chunk loop
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
    "-I", INCLUDE, "-I", CSRC,
]


def _shapes():
    """(NBLK, WP, NJ) triples of NM_SHAPES in nm_variants.h."""
    text = open(os.path.join(CSRC, "nm_variants.h")).read()
    body = text[text.index("#define NM_SHAPES(X)"):]
    body = body[:body.index("\n\n")]
    return [tuple(int(v) for v in m) for m in re.findall(r"X\((\d+),\s*(\d+),\s*(\d+)\)", body)]


def _shapes16():
    """(NBLK, WP, NJ, SHARE) of NM16_SHAPES in nm_variants.h."""
    text = open(os.path.join(CSRC, "nm_variants.h")).read()
    body = text[text.index("#define NM16_SHAPES(X)"):]
    body = body[:body.index("// Y(")]
    return [tuple(int(v) for v in m)
            for m in re.findall(r"X\((\d+),\s*(\d+),\s*(\d+),\s*(\d+)\)", body)]


def _shapes_sp():
    """(NBLK, WP, NJ) of NMSP_SHAPES in nm_variants.h."""
    text = open(os.path.join(CSRC, "nm_variants.h")).read()
    body = text[text.index("#define NMSP_SHAPES(X)"):]
    body = body[:body.index("// Y(")]
    return [tuple(int(v) for v in m) for m in re.findall(r"X\((\d+),\s*(\d+),\s*(\d+)\)", body)]


def _shapes_spw():
    """(NBLK, WP, NJ) of NMSPW_SHAPES in nm_variants.h."""
    text = open(os.path.join(CSRC, "nm_variants.h")).read()
    body = text[text.index("#define NMSPW_SHAPES(X)"):]
    body = body[:body.index("// Y(")]
    return [tuple(int(v) for v in m) for m in re.findall(r"X\((\d+),\s*(\d+),\s*(\d+)\)", body)]


def _shapes_spr():
    """(NBLK, WP, NJ) of NMSPR_SHAPES in nm_variants.h."""
    text = open(os.path.join(CSRC, "nm_variants.h")).read()
    body = text[text.index("#define NMSPR_SHAPES(X)"):]
    body = body[:body.index("// Y(")]
    return [tuple(int(v) for v in m) for m in re.findall(r"X\((\d+),\s*(\d+),\s*(\d+)\)", body)]


def _shapes_run():
    """(NBLK, WP, NJ) of NMRUN_SHAPES in nm_variants.h."""
    text = open(os.path.join(CSRC, "nm_variants.h")).read()
    body = text[text.index("#define NMRUN_SHAPES(X)"):]
    body = body[:body.index("// Y(")]
    return [tuple(int(v) for v in m) for m in re.findall(r"X\((\d+),\s*(\d+),\s*(\d+)\)", body)]


def _shapes_var():
    """(NBLK, WP, NJ) of NMVAR_SHAPES in nm_variants.h."""
    text = open(os.path.join(CSRC, "nm_variants.h")).read()
    body = text[text.index("#define NMVAR_SHAPES(X)"):]
    body = body[:body.index("// Y(")]
    return [tuple(int(v) for v in m) for m in re.findall(r"X\((\d+),\s*(\d+),\s*(\d+)\)", body)]


def _shapes_f8s():
    """(NBLK, WP, NJ) of NMF8S_SHAPES in nm_variants.h."""
    text = open(os.path.join(CSRC, "nm_variants.h")).read()
    body = text[text.index("#define NMF8S_SHAPES(X)"):]
    body = body[:body.index("// Y(")]
    return [tuple(int(v) for v in m) for m in re.findall(r"X\((\d+),\s*(\d+),\s*(\d+)\)", body)]


def _shapes_f8():
    """(NBLK, WP, NJ) of NMF8_SHAPES in nm_variants.h."""
    text = open(os.path.join(CSRC, "nm_variants.h")).read()
    body = text[text.index("#define NMF8_SHAPES(X)"):]
    return [tuple(int(v) for v in m) for m in re.findall(r"X\((\d+),\s*(\d+),\s*(\d+)\)", body)]


def _jobs():
    jobs = []
    for src in ("nm_api.hip", "nm_prune_kernels.hip", "nm_pool_kernels.hip", "nm_conv_registry.hip", "nm_scratch.hip"):
        jobs.append((os.path.join(CSRC, src), os.path.join(OBJDIR, src.replace(".hip", ".o")), []))
    inst = os.path.join(CSRC, "nm_conv_inst.hip")
    for nb, wp, nj in _shapes():
        jobs.append((inst, os.path.join(OBJDIR, f"nm_conv_inst_{nb}_{wp}_{nj}.o"),
                     [f"-DNM_INST_NBLK={nb}", f"-DNM_INST_WP={wp}", f"-DNM_INST_NJ={nj}"]))
    jobs.append((inst, os.path.join(OBJDIR, "nm_conv_inst_scalar.o"), ["-DNM_INST_SCALAR"]))
    for nb, wp, nj in _shapes_var():
        jobs.append((inst, os.path.join(OBJDIR, f"nm_conv_inst_var_{nb}_{wp}_{nj}.o"),
                     ["-DNM_INST_VAR", f"-DNM_INST_NBLK={nb}", f"-DNM_INST_WP={wp}", f"-DNM_INST_NJ={nj}"]))
    inst16 = os.path.join(CSRC, "nm_conv16_inst.hip")
    for nb, wp, nj, sh in _shapes16():
        jobs.append((inst16, os.path.join(OBJDIR, f"nm_conv16_inst_{nb}_{wp}_{nj}_{sh}.o"),
                     [f"-DNM_INST_NBLK={nb}", f"-DNM_INST_WP={wp}", f"-DNM_INST_NJ={nj}",
                      f"-DNM_INST_SHARE={sh}"]))
    instsp = os.path.join(CSRC, "nm_conv_sp16_inst.hip")
    for nb, wp, nj in _shapes_sp():
        jobs.append((instsp, os.path.join(OBJDIR, f"nm_conv_sp16_inst_{nb}_{wp}_{nj}.o"),
                     [f"-DNM_INST_NBLK={nb}", f"-DNM_INST_WP={wp}", f"-DNM_INST_NJ={nj}"]))
    for nb, wp, nj in _shapes_spw():
        jobs.append((instsp, os.path.join(OBJDIR, f"nm_conv_sp16_inst_spw_{nb}_{wp}_{nj}.o"),
                     ["-DNM_INST_SPW", f"-DNM_INST_NBLK={nb}", f"-DNM_INST_WP={wp}", f"-DNM_INST_NJ={nj}"]))
    for nb, wp, nj in _shapes_spr():
        jobs.append((instsp, os.path.join(OBJDIR, f"nm_conv_sp16_inst_spr_{nb}_{wp}_{nj}.o"),
                     ["-DNM_INST_SPR", f"-DNM_INST_NBLK={nb}", f"-DNM_INST_WP={wp}", f"-DNM_INST_NJ={nj}"]))
    for nb, wp, nj in _shapes_f8s():
        jobs.append((instsp, os.path.join(OBJDIR, f"nm_conv_sp16_inst_f8s_{nb}_{wp}_{nj}.o"),
                     ["-DNM_INST_F8S", f"-DNM_INST_NBLK={nb}", f"-DNM_INST_WP={wp}", f"-DNM_INST_NJ={nj}"]))
    instrun = os.path.join(CSRC, "nm_conv_run16_inst.hip")
    for nb, wp, nj in _shapes_run():
        jobs.append((instrun, os.path.join(OBJDIR, f"nm_conv_run16_inst_{nb}_{wp}_{nj}.o"),
                     [f"-DNM_INST_NBLK={nb}", f"-DNM_INST_WP={wp}", f"-DNM_INST_NJ={nj}"]))
    instf8 = os.path.join(CSRC, "nm_conv_f8_inst.hip")
    for nb, wp, nj in _shapes_f8():
        jobs.append((instf8, os.path.join(OBJDIR, f"nm_conv_f8_inst_{nb}_{wp}_{nj}.o"),
                     [f"-DNM_INST_NBLK={nb}", f"-DNM_INST_WP={wp}", f"-DNM_INST_NJ={nj}"]))
    return jobs


def _newest_header():
    hs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    hs += [os.path.join(INCLUDE, f) for f in os.listdir(INCLUDE) if f.endswith(".h")]
    return max(os.path.getmtime(h) for h in hs)


def _compile(job, force, hdr_time):
    src, obj, defs = job
    if (not force and os.path.exists(obj)
            and os.path.getmtime(obj) >= max(os.path.getmtime(src), hdr_time)):
        return obj
    cmd = [HIPCC] + FLAGS + defs + ["-c", src, "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + r.stdout)
    warn = [l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l and l.strip()]
    if any("warning" in l for l in warn):
        sys.stderr.write("\n".join(warn) + "\n")
    return obj


def build(jobs: int = 8, force: bool = True) -> str:
    """Compile every translation unit and link libnmconv.so.  With force=False
    only out-of-date objects are rebuilt."""
    os.makedirs(OBJDIR, exist_ok=True)
    hdr_time = _newest_header()
    todo = _jobs()
    with ThreadPoolExecutor(max_workers=max(1, jobs)) as ex:
        objs = list(ex.map(lambda j: _compile(j, force, hdr_time), todo))
    cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    # a kernel whose host stub was not emitted only shows when the library is loaded
    import ctypes
    ctypes.CDLL(LIB)
    return LIB


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("-j", type=int, default=min(8, os.cpu_count() or 1))
    ap.add_argument("--incremental", action="store_true", help="rebuild only stale objects")
    a = ap.parse_args()
    print(build(a.j, force=not a.incremental))

"""Compile the HIP kernels and the C ABI into libconv_direct.so (gfx950 only).

Every row of csrc/variants.def is one translation unit (conv_variant.hip compiled
with that row's parameters); the units compile in parallel and are linked with the
fallback kernel and the C ABI.  Objects are cached under csrc/_build/ by a hash of
their inputs; build(force=True) ignores the cache.
"""
from __future__ import annotations

import concurrent.futures as cf
import hashlib
import json
import os
import re
import subprocess
import time

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJDIR = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "libconv_direct.so")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
COMMON_DEPS = [os.path.join(CSRC, "variant.h"), os.path.join(CSRC, "variants.def"),
               os.path.join(INCLUDE, "conv_direct.h")]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    "-Rpass-analysis=kernel-resource-usage",   # registers, scratch and spills of every kernel (parsed below)
]


def variants():
    """(name, family, params) for every X(...) row of variants.def."""
    out = []
    with open(os.path.join(CSRC, "variants.def")) as f:
        for ln in f:
            m = re.match(r"\s*X\(\s*(\w+)\s*,\s*(\w+)\s*,(.*)\)\s*$", ln)
            if m:
                out.append((m.group(1), m.group(2), re.sub(r"\s+", "", m.group(3))))
    return out


def _units(only=None):
    """(object stem, source, extra defines, dependency files) per translation unit."""
    units = []
    for name, family, params in variants():
        if only and name not in only:
            continue
        header = {"DMA": "conv_dma_kernel.h", "ROWS": "conv_rows_kernel.h", "PW": "conv_pw_kernel.h", "PWK": "conv_pwk_kernel.h",
                  "TAPS": "conv_taps_kernel.h"}[family]
        units.append((f"tile_{name}", "conv_variant.hip",
                      [f"-DV_NAME={name}", f"-DV_FAMILY={family}", f"-DV_PARAMS={params}"],
                      [os.path.join(CSRC, header), os.path.join(CSRC, "conv_dma_kernel.h"), os.path.join(CSRC, "conv_rows_kernel.h"),
                       os.path.join(CSRC, "variant.h")],
                      family + params))
    defs = []
    if only:
        # a reduced table: the chosen rows only
        sub = os.path.join(OBJDIR, "variants_subset.def")
        with open(os.path.join(CSRC, "variants.def")) as f, open(sub, "w") as g:
            g.writelines(ln for ln in f if (m := re.match(r"\s*X\(\s*(\w+)", ln)) and m.group(1) in only)
        defs = [f'-DCONVD_VARIANTS_DEF="{sub}"']
    units.append(("generic", "conv_generic_kernel.hip", defs, COMMON_DEPS, ",".join(sorted(only or []))))
    units.append(("wgrad", "conv_wgrad.hip", [], COMMON_DEPS + [os.path.join(CSRC, "wgrad.h"), os.path.join(CSRC, "conv_dma_kernel.h")], ""))
    units.append(("layout", "conv_layout_kernels.hip", [], COMMON_DEPS + [os.path.join(CSRC, "layout.h")], ""))
    units.append(("probe", "conv_probe.hip", [], COMMON_DEPS + [os.path.join(CSRC, "layout.h")], ""))
    units.append(("api", "conv_direct_api.cpp", [], COMMON_DEPS + [os.path.join(CSRC, "layout.h"), os.path.join(CSRC, "wgrad.h")], ""))
    return units


def _hipcc():
    return os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _take_resource_remarks(text: str, path: str) -> str:
    """Split hipcc's output into the kernel resource remarks (written to `path` as
    JSON: one record per kernel) and everything else (returned)."""
    kernels, rest, cur, echo = [], [], None, False
    for ln in text.splitlines():
        if "is not a recognized feature" in ln:
            continue
        if echo and re.match(r"\s*\d*\s*\|", ln):   # source echo that follows a remark
            continue
        echo = False
        m = re.search(r"remark:\s+(.*?)\s*\[-Rpass-analysis=kernel-resource-usage\]", ln)
        if m:
            echo = True
            key, _, val = m.group(1).partition(":")
            key, val = key.strip(), val.strip()
            if key == "Function Name":
                cur = {"kernel": val}
                kernels.append(cur)
            elif cur is not None:
                cur[key] = val
            continue
        if ln.startswith("In file included from") or "remarks generated" in ln or "remark generated" in ln:
            continue
        rest.append(ln)
    with open(path, "w") as f:
        json.dump(kernels, f, indent=1)
    return "\n".join(rest)


def kernel_resources():
    """Resource records of every kernel in the objects of the last build."""
    out = []
    for nm in sorted(os.listdir(OBJDIR)) if os.path.isdir(OBJDIR) else []:
        if nm.endswith(".usage.json"):
            with open(os.path.join(OBJDIR, nm)) as f:
                out += [dict(r, unit=nm.rsplit("-", 1)[0]) for r in json.load(f)]
    return out


def _compile(unit, extra_flags, force, verbose):
    stem, src, defs, deps, salt = unit
    srcp = os.path.join(CSRC, src)
    h = hashlib.sha256()
    for p in [srcp] + list(deps):
        with open(p, "rb") as f:
            h.update(f.read())
    h.update(" ".join(FLAGS + list(extra_flags) + defs + [salt]).encode())
    obj = os.path.join(OBJDIR, f"{stem}-{h.hexdigest()[:16]}.o")
    if force or not os.path.exists(obj):
        for old in os.listdir(OBJDIR):
            if old.startswith(stem + "-") and (old.endswith(".o") or old.endswith(".usage.json")):
                os.remove(os.path.join(OBJDIR, old))
        cmd = [_hipcc()] + FLAGS + list(extra_flags) + defs + ["-c", srcp, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        t0 = time.perf_counter()
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if verbose:
            print(f"[build] {stem}: {time.perf_counter() - t0:.1f} s", flush=True)
        msg = _take_resource_remarks(r.stdout, obj[:-2] + ".usage.json")
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {stem}:\n{msg}")
        if msg.strip():
            print(msg, flush=True)
    return obj


def build(force: bool = True, extra_flags=(), verbose: bool = False, only=None, lib: str = LIB,
          jobs: int | None = None) -> str:
    """Compile and link; returns the library path.  `only` (a set of variant names)
    builds a reduced library for experiments (the fallback kernel is always included)."""
    os.makedirs(OBJDIR, exist_ok=True)
    units = _units(set(only) if only else None)
    jobs = jobs or min(len(units), os.cpu_count() or 1, 16)
    with cf.ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda u: _compile(u, extra_flags, force, verbose), units))
    if not only:
        # a full build leaves nothing of earlier variant sets behind (their resource
        # reports would otherwise be mistaken for kernels of this library)
        keep = {os.path.basename(o)[:-2] for o in objs}
        for nm in os.listdir(OBJDIR):
            if nm.rsplit(".", 2)[0] not in keep and (nm.endswith(".o") or nm.endswith(".usage.json")):
                os.remove(os.path.join(OBJDIR, nm))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", lib]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser()
    ap.add_argument("--only", nargs="*", help="variant names for a reduced experimental library")
    ap.add_argument("--lib", default=LIB)
    ap.add_argument("--cached", action="store_true", help="reuse objects whose inputs did not change")
    ap.add_argument("flags", nargs="*", help="extra hipcc flags (after --)")
    a = ap.parse_args()
    print(build(force=not a.cached, extra_flags=a.flags, verbose=True, only=a.only, lib=a.lib))

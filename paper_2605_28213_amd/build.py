"""Builds libgemm_lineage.so (HIP, gfx950 only) next to this file.

Each .hip translation unit is compiled to an object in ``_build/`` and linked with
``hipcc -shared``.  Objects are rebuilt when their source or a header is newer, unless
``force`` is set.  hipcc cross-compiles without a GPU present.

The compiler's per-kernel resource remarks (registers, spills, scratch, LDS, occupancy) are kept
beside each object and merged into ``libgemm_lineage.resources.json`` next to the library together
with a digest of the sources it was built from: the compile leg of the validation gate records them
(``resources()``, ``sources_digest()``).
"""
from __future__ import annotations

import hashlib
import json
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libgemm_lineage.so")
RESOURCES = os.path.join(HERE, "libgemm_lineage.resources.json")
SOURCES = ["gemm_api.hip", "conv_api.hip", "topk.hip", "k0_naive.hip", "k123_valu_tiled.hip", "k3_async.hip", "k4_mfma.hip", "k4_ring.hip", "k4_thin.hip", "probes.hip"]
HEADERS = [os.path.join(CSRC, "common.hpp"), os.path.join(CSRC, "k4_kernels.hpp"), os.path.join(CSRC, "k4_ring.hpp"), os.path.join(CSRC, "k4_thin.hpp"),
           os.path.join(os.path.dirname(HERE), "include", "gemm_lineage.h"),
           os.path.join(os.path.dirname(HERE), "include", "conv_lineage.h"),
           os.path.join(os.path.dirname(HERE), "include", "topk_lineage.h")]
# packed fp32 VALU forms (v_pk_*_f32) are switched off: the compiler must not form them for this target
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# Per translation unit.  Machine-code sinking moves whole chains of matrix instructions (pure register
# operations whose results are next used in a later block) past the loads, barriers and waits they were
# interleaved with, and then needs two slabs' fragments in registers at once: the persistent kernel places
# them by hand.  (The streaming kernels need the pass: without it they spill.)
EXTRA_FLAGS = {"k4_ring.hip": ["-mllvm", "-disable-machine-sink"]}
REMARKS = "-Rpass-analysis=kernel-resource-usage"
_FIELDS = {"TotalSGPRs": "sgpr", "VGPRs": "vgpr", "AGPRs": "agpr", "ScratchSize [bytes/lane]": "scratch_bytes_per_lane",
           "Occupancy [waves/SIMD]": "waves_per_simd", "SGPRs Spill": "sgpr_spill", "VGPRs Spill": "vgpr_spill",
           "LDS Size [bytes/block]": "lds_bytes"}


def sources_digest() -> str:
    """sha256 over every source and header the library is built from (names and contents)."""
    h = hashlib.sha256()
    for p in sorted([os.path.join(CSRC, s) for s in SOURCES] + HEADERS):
        h.update(os.path.basename(p).encode())
        with open(p, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def _parse_remarks(stderr: str) -> dict:
    """{mangled kernel name: {sgpr, vgpr, agpr, scratch_bytes_per_lane, waves_per_simd, spills, lds_bytes}}."""
    out, cur = {}, None
    for line in stderr.splitlines():
        m = re.search(r"remark:\s+(.*?)\s+\[-Rpass-analysis=kernel-resource-usage\]", line)
        if not m:
            continue
        text = m.group(1)
        if text.startswith("Function Name:"):
            cur = out.setdefault(text.split(":", 1)[1].strip(), {})
        elif cur is not None and ":" in text:
            key, val = text.rsplit(":", 1)
            if key.strip() in _FIELDS and val.strip().isdigit():
                cur[_FIELDS[key.strip()]] = int(val)
    return out


def _demangle(names):
    try:
        r = subprocess.run(["c++filt"], input="\n".join(names), capture_output=True, text=True, check=True)
        return r.stdout.splitlines()
    except Exception:
        return list(names)


def _compile(src: str, force: bool) -> str:
    obj = os.path.join(BUILD, os.path.splitext(src)[0] + ".o")
    path = os.path.join(CSRC, src)
    newest = max(os.path.getmtime(p) for p in [path] + HEADERS)
    res = obj + ".resources.json"
    if force or not os.path.exists(obj) or not os.path.exists(res) or os.path.getmtime(obj) < newest:
        r = subprocess.run(["hipcc", *FLAGS, *EXTRA_FLAGS.get(src, []), REMARKS, "-c", path, "-o", obj], capture_output=True, text=True)
        remarks = _parse_remarks(r.stderr)
        # what is left of stderr once the remarks (and the source line and caret echoed after some) are taken out
        keep, after_remark = [], False
        for l in r.stderr.splitlines():
            if "-Rpass-analysis=kernel-resource-usage" in l:
                after_remark = True
            elif after_remark and re.match(r"^\s*(\d+\s*)?\|", l):
                pass
            else:
                after_remark = False
                if "packed-fp32-ops" not in l and not re.match(r"^\d+ warnings? generated", l):
                    keep.append(l)
        err = "\n".join(keep)
        if r.returncode == 0 and not any(w in err for w in ("warning:", "error:")):
            err = ""            # only include-chain lines of the remarks are left
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{err}")
        if err.strip():
            sys.stderr.write(err + "\n")
        with open(res, "w") as f:
            json.dump(remarks, f)
        _compile.built.append(src)
    return obj


_compile.built = []


def build(force: bool = False) -> str:
    """Brings the library up to date with its sources; returns its path.  `last_built()` then names the
    translation units this call compiled (none when everything was current)."""
    os.makedirs(BUILD, exist_ok=True)
    _compile.built = []
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), SOURCES))
    if force or not os.path.exists(LIB) or not os.path.exists(RESOURCES) or any(os.path.getmtime(o) > os.path.getmtime(LIB) for o in objs):
        r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                           capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stderr)
        kernels = {}
        for o in objs:
            with open(o + ".resources.json") as f:
                kernels.update(json.load(f))
        names = sorted(kernels)
        table = {d: dict(kernels[m], mangled=m) for m, d in zip(names, _demangle(names))}
        with open(RESOURCES, "w") as f:
            json.dump({"sources_sha256": sources_digest(), "flags": FLAGS, "extra_flags": EXTRA_FLAGS, "kernels": table}, f, indent=1, sort_keys=True)
    return LIB


def last_built():
    return list(_compile.built)


def resources() -> dict:
    """The record written at link time: {"sources_sha256", "flags", "kernels": {demangled name: figures}}.
    Raises FileNotFoundError when the library was not built by this module."""
    with open(RESOURCES) as f:
        return json.load(f)


def is_stale() -> bool:
    """True when the library is missing, or was linked from other sources than the ones on disk."""
    try:
        return not os.path.exists(LIB) or resources()["sources_sha256"] != sources_digest()
    except (FileNotFoundError, KeyError, ValueError):
        return True


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))

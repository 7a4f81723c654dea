"""Builds libmodse.so (HIP, gfx950 only) next to this file.

    python -m paper_2409_12210_amd.build

The build also reads the compiler's per-kernel resource remarks and fails unless every kernel keeps its working
set in the 256 architectural vector registers: no scratch memory, no spilled registers, no accumulation registers
(spills into scratch have cost kernels here several times their run time, and a router variant that the compiler
had let run over into accumulation registers computed wrong sums).  The table goes to kernel_resources.txt next
to the library.
"""
from __future__ import annotations

import os
import subprocess
import sys
import re
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmodse.so")
RESOURCES = os.path.join(HERE, "kernel_resources.txt")
SOURCES = ["api.hip", "route.hip", "gemm.hip"]
# packed fp32 VALU ops are switched off for all device code (known to misbehave on the test machines)
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-Wno-unused-command-line-argument",
         "-Rpass-analysis=kernel-resource-usage"]
# kernels allowed to use accumulation registers (AGPRs): none
AGPR_ALLOWED = ()


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


_REMARK = re.compile(r"remark: +(.*?) *\[-Rpass-analysis=kernel-resource-usage\]")
_FIELDS = {"VGPRs": "vgprs", "AGPRs": "agprs", "ScratchSize [bytes/lane]": "scratch", "VGPRs Spill": "vgpr_spill",
           "SGPRs Spill": "sgpr_spill", "Occupancy [waves/SIMD]": "occupancy", "LDS Size [bytes/block]": "lds",
           "TotalSGPRs": "sgprs"}


def parse_resource_remarks(stderr: str) -> dict:
    """{mangled kernel name: {vgprs, agprs, scratch, vgpr_spill, sgpr_spill, occupancy, lds, sgprs}} from the
    output of -Rpass-analysis=kernel-resource-usage."""
    out, cur = {}, None
    for line in stderr.splitlines():
        m = _REMARK.search(line)
        if not m:
            continue
        text = m.group(1).strip()
        if text.startswith("Function Name:"):
            cur = out.setdefault(text.split(":", 1)[1].strip(), {})
        elif cur is not None and ":" in text:
            key, val = text.rsplit(":", 1)
            if key.strip() in _FIELDS and val.strip().lstrip("-").isdigit():
                cur[_FIELDS[key.strip()]] = int(val)
    return out


def resource_violations(res: dict) -> list:
    bad = []
    for name, r in sorted(res.items()):
        if r.get("scratch", 0) or r.get("vgpr_spill", 0):
            bad.append(f"{name}: scratch {r.get('scratch', 0)} bytes/lane, {r.get('vgpr_spill', 0)} spilled VGPRs")
        if r.get("agprs", 0) and not any(a in name for a in AGPR_ALLOWED):
            bad.append(f"{name}: uses {r['agprs']} accumulation registers")
    return bad


def _compile(src: str, extra):
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    cmd = [_hipcc(), *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and "remark:" not in l)
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    res = parse_resource_remarks(r.stderr)
    # the remarks (with the source lines they quote) are not shown; warnings are
    if re.search(r"\b(warning|error):", "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)):
        sys.stderr.write("\n".join(l for l in r.stderr.splitlines()
                                   if "remark:" not in l and "packed-fp32-ops" not in l) + "\n")
    return obj, res


def build(extra_flags=(), verbose: bool = True) -> str:
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        done = list(ex.map(lambda s: _compile(s, list(extra_flags)), SOURCES))
    objs = [o for o, _ in done]
    res = {}
    for _, r in done:
        res.update(r)
    with open(RESOURCES, "w") as f:
        f.write("# kernel  vgprs agprs scratch_bytes_per_lane vgpr_spill occupancy lds_bytes\n")
        for name, r in sorted(res.items()):
            f.write(f"{name} {r.get('vgprs', -1)} {r.get('agprs', -1)} {r.get('scratch', -1)} "
                    f"{r.get('vgpr_spill', -1)} {r.get('occupancy', -1)} {r.get('lds', -1)}\n")
    if not res:
        raise RuntimeError("the compiler printed no kernel-resource-usage remarks: cannot check register use")
    bad = resource_violations(res)
    if bad:
        raise RuntimeError("kernels outside the register budget:\n  " + "\n  ".join(bad))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print(f"built {LIB} ({len(res)} kernels within the register budget)")
    return LIB


def build_host_sanitized(out_dir: str, driver_c: str) -> str:
    """Builds, into out_dir, a copy of the library whose api.hip HOST code is instrumented with AddressSanitizer and
    UndefinedBehaviorSanitizer (the device code and the other two objects are the ordinary ones: build() first),
    and the C program driver_c against it with the same sanitizers.  Returns the path of the program."""
    os.makedirs(out_dir, exist_ok=True)
    san = []
    for f in ("-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"):
        san += ["-Xarch_host", f]
    flags = [f for f in FLAGS if f != "-Rpass-analysis=kernel-resource-usage"]
    obj = os.path.join(out_dir, "api_san.o")
    lib = os.path.join(out_dir, "libmodse_hostsan.so")
    exe = os.path.join(out_dir, "host_abi_driver")
    others = [os.path.join(CSRC, s.replace(".hip", ".o")) for s in SOURCES if s != "api.hip"]
    for o in others:
        if not os.path.exists(o):
            raise FileNotFoundError(f"{o} not found: run build() first")
    steps = [
        [_hipcc(), *flags, *san, "-g", "-c", os.path.join(CSRC, "api.hip"), "-o", obj],
        [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *san, obj, *others, "-o", lib],
        [_hipcc(), "-x", "c", "-std=c99", "-g", "-fsanitize=address", "-fsanitize=undefined",
         "-fno-sanitize-recover=undefined", "-I" + os.path.join(ROOT, "include"), driver_c, "-x", "none", lib,
         "-Wl,-rpath," + out_dir, "-o", exe],
    ]
    for cmd in steps:
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
            raise RuntimeError("sanitized host build failed: " + " ".join(cmd) + "\n" + err)
    return exe


if __name__ == "__main__":
    build(sys.argv[1:])

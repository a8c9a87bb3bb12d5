"""Compiles every device translation unit of libhfr to gfx950 assembly and checks
what the arithmetic contract and the performance of the kernels rest on:

  * no kernel uses scratch memory (a register array that the compiler could not
    keep in registers shows up here, long before it shows up in a benchmark);
  * no fused multiply-add and no packed-fp32 instruction (every add and the
    scale multiply must stay separately rounded binary32 operations);
  * no fp16 mixed-precision fused instruction (it would round a product once,
    straight to fp16, instead of to binary32 first);
  * nothing writes through the scalar data cache.

    python -m tests.check_isa [part-of-a-file-name ...]   # a few minutes on 8 cores for all of them
                                                          # (CPU only: a build check, not product code)

Also prints the largest register count (VGPRs + AGPRs) among each unit's kernels.

Exit status 0 when every check holds; the offending kernels are listed otherwise.
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

from paper_2408_14158_amd import build as hfr_build

# integer multiply-adds (address arithmetic) are fine; floating-point ones are not
FORBIDDEN = re.compile(r"\b(v_fma_\w+|v_fmac_\w+|v_mac_\w+|v_mad_(?!u64_u32|i64_i32|u32_u24|i32_i24|u32_u16|i32_i16)\w+"
                       r"|v_pk_(?:add|mul|fma)_f32|v_dot\w+|s_(?:buffer_|scratch_)?store\w*|s_atomic\w*|s_dcache_wb\w*|s_dcache_inv\w*)\b")


def _check(src: str, outdir: str):
    path = os.path.join(hfr_build.CSRC, src)
    asm = os.path.join(outdir, src + ".s")
    cmd = [hfr_build.hipcc(), *hfr_build.COMMON, *hfr_build.DEVICE, "-S", "--cuda-device-only", path, "-o", asm]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        return src, 0, 0, ["compile failed: " + r.stderr[-400:]]
    text = open(asm).read()
    os.remove(asm)
    problems = []
    meta = text[text.index("amdhsa.kernels:"):] if "amdhsa.kernels:" in text else ""
    kernels = meta.split("  - .agpr_count:")[1:]
    regs = 0
    for k in kernels:
        agpr = int(re.match(r"\s*(\d+)", k).group(1))
        regs = max(regs, agpr + int(re.search(r"\.vgpr_count:\s+(\d+)", k).group(1)))
        name = re.search(r"\.name:\s+(\S+)", k).group(1)
        scratch = int(re.search(r"\.private_segment_fixed_size:\s+(\d+)", k).group(1))
        if scratch:
            problems.append("%s: %d bytes of scratch" % (name, scratch))
    for m in sorted(set(FORBIDDEN.findall("\n".join(l for l in text.split("\n") if l.startswith("\t"))))):
        problems.append("forbidden instruction %s" % m)
    return src, len(kernels), regs, problems


def main() -> int:
    only = sys.argv[1:]
    srcs = [s for s in hfr_build.SOURCES if s.endswith(".hip") and (not only or any(o in s for o in only))]
    bad = 0
    with tempfile.TemporaryDirectory() as tmp, ThreadPoolExecutor(max_workers=8) as ex:
        for src, count, regs, problems in ex.map(lambda s: _check(s, tmp), srcs):
            print("%-32s %4d kernels  max %3d registers  %s" % (src, count, regs, "ok" if not problems else "%d problem(s)" % len(problems)), flush=True)
            for p in problems:
                print("    " + p)
            bad += len(problems)
    return 1 if bad else 0


if __name__ == "__main__":
    sys.exit(main())

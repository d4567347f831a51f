#!/usr/bin/env python3
"""Build-time check of the register-spill precondition of the main kernel's inline-assembly LDS reads.

The direct-read variants of igemm_kernel (B source 2, 3 or 5) issue their transposing LDS reads as inline
assembly and wait for them themselves; a fragment register the compiler spilled between such a read and the
kernel's own wait would be saved before its data has arrived.  Those variants must therefore compile to zero
scratch.  This script reads the compiler's kernel-resource-usage remarks (one file per kernel translation
unit, written by the Makefile) and fails when a variant that uses the inline-assembly reads reports scratch
or spilled vector registers.  Variants that keep the compiler's builtins (32-byte fragments on wave windows of eight or more
MFMA tiles: igemm.hpp, ASM_TR) may spill and are only listed.

usage: check_resources.py FILE.res [FILE.res ...]      exit status 1 on a violation
"""
import re
import sys

NAME = re.compile(r"Function Name: _ZN4unit12igemm_kernelI((?:Li\d+E)+)EEvNS_9IgemmArgsE")
FIELD = re.compile(r"remark:\s+([A-Za-z ]+?)(?: \[[^\]]*\])?: (\S+) \[-Rpass-analysis")
DIRECT = (2, 3, 5)                     # BSRC_NCHW, BSRC_NCHWS, BSRC_NCHWE


def kernels(path):
    cur = None
    for line in open(path, errors="replace"):
        m = NAME.search(line)
        if m:
            cur = {"args": [int(v) for v in re.findall(r"Li(\d+)E", m.group(1))]}
            yield cur
            continue
        if cur is not None:
            f = FIELD.search(line)
            if f:
                cur[f.group(1).strip()] = f.group(2)


def main(paths):
    bad, seen, spilled_builtin = [], 0, 0
    for p in paths:
        for k in list(kernels(p)):
            dt, bm, bn, bkb, wgm, wgn, wgk, mf, nst, occ, bsrc, epi = k["args"]
            if bsrc not in DIRECT:
                continue
            fw = 2 if dt == 5 else 1
            asm_tr = not (fw == 2 and (bm // wgm // mf) * (bn // wgn // mf) >= 8)
            scratch = int(k.get("ScratchSize", "0"))
            # (spilled SGPRs live in lanes of a reserved VGPR: they never touch the fragment registers)
            spills = int(k.get("VGPRs Spill", "0"))
            seen += 1
            if asm_tr and (scratch or spills):
                bad.append((p, k["args"], scratch, spills))
            elif scratch or spills:
                spilled_builtin += 1
    if not seen:
        print("check_resources: no direct-read igemm_kernel variant found in", paths, file=sys.stderr)
        return 1
    for p, args, scratch, spills in bad:
        print(f"check_resources: {p}: igemm_kernel<{', '.join(map(str, args))}> uses inline-assembly LDS reads but "
              f"has {scratch} bytes of scratch per lane and {spills} spilled vector registers", file=sys.stderr)
    print(f"check_resources: {seen} direct-read variants, {len(bad)} violations, "
          f"{spilled_builtin} builtin-read variants with spills (allowed)")
    return 1 if bad else 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))

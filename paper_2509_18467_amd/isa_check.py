"""Developer check on the compiled chunk kernels (no GPU needed): compiles the two instantiation files to gfx950
ISA and reports, per kernel, registers, scratch (spill) bytes and any wait on global-memory loads inside the
MFMA stage of the output pass.

Why it exists: twice during tuning the compiler made the MFMA stage wait for the next granule's prefetch --
once through scratch reloads (a reload carries `s_waitcnt vmcnt(0)`), once through a false register dependency
that made it flush all loads in front of the chunk loop.  Neither shows up in a test, only in the timing.

Usage:  python -m paper_2509_18467_amd.isa_check        (exit status 1 if a kernel spills or waits)
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
import tempfile

from . import build as _build

_KERNEL = re.compile(r"^(_ZN6lawcat5chunk16gla_chunk_kernelILi(\d+)ELi(\d+)ELi(\d+)ELb(\d)E[^:\s]*):", re.M)


def _compile(src: str, out: str) -> str:
    cmd = [_build.HIPCC, *_build.FLAGS, "--cuda-device-only", "-Rpass-analysis=kernel-resource-usage", "-S",
           os.path.join(_build.CSRC, src), "-o", out]
    return subprocess.run(cmd, check=True, capture_output=True, text=True).stderr


def _resources(remarks: str) -> dict:
    res, name = {}, None
    for line in remarks.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            res[name] = {}
        for key, pat in (("vgprs", r"\bVGPRs: (\d+)"), ("scratch", r"ScratchSize \[bytes/lane\]: (\d+)")):
            m = re.search(pat, line)
            if m and name:
                res[name][key] = int(m.group(1))
    return res


def _loop_end(body: list, inside: int) -> int:
    """Index just past the last basic block of the depth-1 loop (the granule loop) that contains line `inside`,
    read from the compiler's block annotations."""
    header = None
    for j in range(inside, -1, -1):
        m = re.match(r"\.(LBB\d+_\d+):.*This Loop Header: Depth=1", body[j])
        if m:
            header = m.group(1)[1:]  # "BBn_m"
            break
    if header is None:
        return len(body)
    member = re.compile(rf"(Header={header}\b|Parent Loop {header}\b)")
    last = max(j for j, l in enumerate(body) if member.search(l) or l.startswith("." + "L" + header + ":"))
    for j in range(last + 1, len(body)):
        if re.match(r"\.LBB\d+_\d+:", body[j]):
            return j
    return len(body)


def check() -> int:
    bad = 0
    with tempfile.TemporaryDirectory() as tmp:
        for src in ("gla_chunk_d64.hip", "gla_chunk_d128.hip"):
            asm = os.path.join(tmp, src + ".s")
            res = _resources(_compile(src, asm))
            text = open(asm).read()
            starts = [(m.start(), m) for m in _KERNEL.finditer(text)]
            for i, (pos, m) in enumerate(starts):
                body = text[pos:starts[i + 1][0] if i + 1 < len(starts) else len(text)]
                body = body.split("s_endpgm")[0].splitlines()
                name, d, gr, mode, output = m.group(1), int(m.group(2)), int(m.group(3)), int(m.group(4)), m.group(5) == "1"
                r = res.get(name, {})
                waits = []
                if output:
                    # inside the granule loop the barriers cut the code into regions; those that hold MFMAs make
                    # up the MFMA stage (the compute stage has none), whatever order the blocks were laid out in
                    bars = [j for j, l in enumerate(body) if "s_barrier" in l]
                    if bars:
                        end = _loop_end(body, bars[-1])
                        cuts = [j for j in bars if j < end] + [end]
                        for lo, hi in zip(cuts[:-1], cuts[1:]):
                            if any("v_mfma" in body[j] for j in range(lo, hi)):
                                waits += [(j, body[j].strip()) for j in range(lo, hi)
                                          if "s_waitcnt" in body[j] and "vmcnt" in body[j]]
                    else:
                        waits = [(0, "(no barrier found: kernel layout not recognised)")]
                flag = ""
                if r.get("scratch", 0) > 0:
                    flag += "  <-- spills"
                if waits:
                    flag += "  <-- waits for loads in the MFMA stage: " + "; ".join(w for _, w in waits[:3])
                bad += bool(flag)
                kind = "output" if output else "state "
                print(f"d={d:3d} group={gr} mode={mode} {kind} pass: {r.get('vgprs', '?'):>3} VGPRs, "
                      f"{r.get('scratch', '?')} B scratch{flag}")
    return 1 if bad else 0


if __name__ == "__main__":
    sys.exit(check())

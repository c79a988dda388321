"""Build the HIP library for gfx950: one hipcc compile per translation unit (in parallel), one link.

    python -m paper_2502_04420_amd.build

Produces paper_2502_04420_amd/libkvq.so next to this file.  The objects go to
paper_2502_04420_amd/_build/.  hipcc cross-compiles, so no GPU is needed to build.
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libkvq.so")
OBJ = os.path.join(HERE, "_build")

COMMON = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function",
          # packed fp32 instructions are kept out of the generated code on purpose
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# the encode path must not contract or reassociate anything: its results are compared bit for bit
PER_FILE = {"kvq_quantize.hip": ["-ffp-contract=off"],
            # M0 is named as clobbered by the global-to-LDS fetch; the compiler notes that it reserves that register
            "kvq_prefill_attn.hip": ["-Wno-inline-asm"]}


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    cmd = ["hipcc"] + COMMON + PER_FILE.get(src, []) + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "not a recognized feature" not in l)
    if r.returncode:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, err))
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def device_assembly(src: str, extra=()) -> str:
    """The gfx950 assembly hipcc generates for one source file with the library's flags."""
    out = os.path.join(OBJ, src.replace(".hip", ".s"))
    cmd = (["hipcc"] + COMMON + ["-w"] + PER_FILE.get(src, []) + list(extra)
           + ["-S", "--cuda-device-only", os.path.join(CSRC, src), "-o", out])
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode:
        raise RuntimeError("hipcc -S failed for %s:\n%s" % (src, r.stderr[-2000:]))
    with open(out) as f:
        return f.read()


def kernel_bodies(asm: str, name: str):
    """(mangled name, text) of the kernels whose mangled name contains `name`."""
    return [(m.group(1), m.group(0)) for m in re.finditer(r"^(_Z\w*%s\w*):.*?^\.Lfunc_end\d+:" % name, asm, re.S | re.M)]


def check_prefill_attention_code(asm: str) -> None:
    """The prefill attention kernels set M0 in inline assembly (LDS base of their global-to-LDS fetches).  The library
    is only linked if, in the generated code, every M0 write is the one in front of such a fetch, nothing else reads or
    writes M0, and no kernel of the file spills registers (two waves per SIMD is what its pipelining assumes)."""
    kernels = kernel_bodies(asm, "prefill_attention")
    if len(kernels) != 2:                                                  # keys quantized / fp16
        raise RuntimeError("expected 2 prefill_attention kernels in the generated code, found %d" % len(kernels))
    for name, body in kernels:
        lines = [l.strip() for l in body.splitlines()]
        code = [l for l in lines if l and not l.startswith((";", ".", "_Z")) and not l.endswith(":")]
        writes = [i for i, l in enumerate(code) if re.match(r"s_mov_b32 m0,", l)]
        fetches = [i for i, l in enumerate(code) if l.startswith("global_load_lds_dwordx4")]
        if not fetches or len(writes) != len(fetches):
            raise RuntimeError("%s: %d writes of M0 for %d fetches" % (name, len(writes), len(fetches)))
        for w, f in zip(writes, fetches):
            if not w < f <= w + 3:                                         # s_mov m0 ; s_nop ; load
                raise RuntimeError("%s: M0 write not in front of a fetch: %s" % (name, code[w:w + 4]))
        others = [l for l in code if re.search(r"\bm0\b", l) and not re.match(r"s_mov_b32 m0,", l)]
        if others:
            raise RuntimeError("%s: M0 used outside the fetches: %s" % (name, others[:3]))
    spills = re.findall(r"\.vgpr_spill_count:\s+(\d+)", asm)
    if not spills or any(int(x) for x in spills):
        raise RuntimeError("kvq_prefill_attn.hip: register spills %s" % spills)


def _vregs(text: str):
    out = set()
    for a, b in re.findall(r"\bv\[(\d+):(\d+)\]", text):
        out.update(range(int(a), int(b) + 1))
    out.update(int(a) for a in re.findall(r"\bv(\d+)\b", text))
    return out


def check_decode_code(asm: str) -> int:
    """The matrix-core decode kernels issue the block loads of their streaming loop in inline assembly and wait for them
    with hand-written counts; the compiler does not know that the destination registers are being written until the
    wait.  The library is only linked if, in the generated code, no instruction of the compiler's own touches such a
    register between the issue of a load and a wait that covers it.  Model: loads return in order, so after
    `s_waitcnt vmcnt(N)` only the N youngest loads are pending.  The code is followed in layout order; a backward
    conditional branch (a loop) is followed once more from its target with the state at the branch; the state is
    dropped after an unconditional branch (what follows in the layout is reached from elsewhere).  A statement that
    holds two waits (await_loads_either: the count depends on whether the zero-points of the next blocks were asked
    for in this step) is taken with the larger count if at least that many loads were issued since the last wait,
    else with the smaller.  Returns the number of hand-issued loads seen."""
    seen = 0
    for name, body in kernel_bodies(asm, "decode_mfma"):
        lines = body.split("\n")
        labels = {}
        for i, l in enumerate(lines):
            m = re.match(r"^(\.LBB\d+_\d+):", l)
            if m:
                labels[m.group(1)] = i

        def run(start, stop, pending, follow):
            nonlocal seen
            in_asm = False
            asm_waits = []
            issued = 0                      # hand-issued loads since the last wait on the load counter
            i = start
            while i < stop:
                t = lines[i].strip()
                i += 1
                if t.startswith(";;#ASMSTART"):
                    in_asm = True
                    asm_waits = []
                    continue
                if t.startswith(";;#ASMEND"):
                    in_asm = False
                    if asm_waits:
                        # A statement that holds two waits takes one of them at run time: the larger count when further
                        # loads (the zero-points of the next blocks) went out behind the awaited block's in this step,
                        # which shows in the number of loads issued since the last wait; otherwise the smaller one.
                        n = max(asm_waits) if issued >= max(asm_waits) else min(asm_waits)
                        pending = pending[len(pending) - n:] if n else []
                        issued = 0
                    continue
                if not t or t[0] in ";." or t.endswith(":"):
                    continue
                w = re.match(r"s_waitcnt\b.*vmcnt\((\d+)\)", t)
                if w:
                    n = int(w.group(1))
                    if in_asm and re.match(r"s_waitcnt\s+vmcnt\(\d+\)$", t):
                        asm_waits.append(n)
                    else:
                        pending = pending[len(pending) - n:] if n else []
                        issued = 0
                    continue
                if in_asm:
                    if t.startswith("buffer_load"):
                        pending = pending + [_vregs(t.split(",")[0])]
                        issued += 1
                        if follow:
                            seen += 1
                    continue
                used = _vregs(t)
                for regs in pending:
                    if used & regs:
                        raise RuntimeError("%s: `%s` touches v%s while a hand-issued load may still be writing it"
                                           % (name, t, sorted(used & regs)))
                b = re.match(r"s_cbranch_\w+\s+(\.LBB\d+_\d+)", t)
                if b and follow and labels.get(b.group(1), i) < i - 1:
                    run(labels[b.group(1)], i - 1, list(pending), False)       # the loop once more, entered with this state
                if t.startswith("s_branch") or t.startswith("s_endpgm"):
                    pending = []

        run(0, len(lines), [], True)
    return seen


def _check_generated_code() -> None:
    check_prefill_attention_code(device_assembly("kvq_prefill_attn.hip"))
    if check_decode_code(device_assembly("kvq_decode_mfma.hip")) == 0:
        raise RuntimeError("kvq_decode_mfma.hip: no hand-issued loads found in the generated code")


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    srcs = sources()
    with ThreadPoolExecutor(max_workers=min(8, len(srcs) + 1)) as ex:
        checked = ex.submit(_check_generated_code)          # alongside the compiles; a failure refuses the link
        objs = list(ex.map(_compile, srcs))
        checked.result()
    tmp = OUT + ".tmp.%d" % os.getpid()
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs,
                       capture_output=True, text=True)
    if r.returncode:
        raise RuntimeError("link failed:\n" + r.stderr)
    os.replace(tmp, OUT)
    if verbose:
        print("built", OUT)
    return OUT


if __name__ == "__main__":
    build()

"""Properties of the generated code that the sources rely on but the compiler does not promise."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2502_04420_amd", "csrc")


def _assembly(src, tmp_path, extra=()):
    hipcc = shutil.which("hipcc")
    if hipcc is None:
        pytest.skip("hipcc not available")
    out = tmp_path / (src + ".s")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-w", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-S", "--cuda-device-only", *extra,
           os.path.join(CSRC, src), "-o", str(out)]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, r.stderr[-2000:]
    return out.read_text()


def _kernels(asm, name):
    """Bodies of the kernels whose mangled name contains `name`."""
    bodies = []
    for m in re.finditer(r"^(_Z\w*%s\w*):.*?^\.Lfunc_end\d+:" % name, asm, re.S | re.M):
        bodies.append((m.group(1), m.group(0)))
    return bodies


def test_prefill_attention_writes_m0_only_for_its_own_fetches(tmp_path):
    """The attention kernel sets M0 in inline assembly (LDS base of a global-to-LDS load) without telling the compiler:
    that is sound only while the compiler itself never uses M0 in that kernel.  Every M0 write in the generated code must
    be the one in front of one of those loads, and no other instruction may read M0."""
    asm = _assembly("kvq_prefill_attn.hip", tmp_path)
    kernels = _kernels(asm, "prefill_attention")
    assert len(kernels) == 2                                            # keys quantized / fp16
    for name, body in kernels:
        lines = [l.strip() for l in body.splitlines()]
        code = [l for l in lines if l and not l.startswith((";", ".", "_Z")) and not l.endswith(":")]
        writes = [i for i, l in enumerate(code) if re.match(r"s_mov_b32 m0,", l)]
        fetches = [i for i, l in enumerate(code) if l.startswith("global_load_lds_dwordx4")]
        assert fetches and len(writes) == len(fetches), (name, len(writes), len(fetches))
        for w, f in zip(writes, fetches):
            assert w < f <= w + 3, (name, code[w:w + 4])                # s_mov m0 ; s_nop ; load
        others = [l for l in code if re.search(r"\bm0\b", l) and not re.match(r"s_mov_b32 m0,", l)]
        assert not others, (name, others[:3])
    # and no kernel of the file spills registers to scratch memory (the budget of two waves per SIMD holds)
    spills = re.findall(r"\.vgpr_spill_count:\s+(\d+)", asm)
    assert spills and all(int(x) == 0 for x in spills), spills


def test_quantize_kernel_keeps_the_fused_widen_and_subtract(tmp_path):
    """x - z is meant to be one mixed-precision instruction per element (both fp16 operands widened inside it); the
    multiplier 1.0 is hidden from the optimiser for that.  If a compiler folds it after all, the code is still right
    but slower: this test tells."""
    asm = _assembly("kvq_quantize.hip", tmp_path, extra=("-ffp-contract=off",))
    kernels = [b for n, b in _kernels(asm, "quantize_blocks") if "ILi4ELi2ELb0E" in n]
    assert len(kernels) == 1
    assert len(re.findall(r"^\s*v_fma_mix_f32 ", kernels[0], re.M)) >= 128      # 2 tensors x 64 elements per lane

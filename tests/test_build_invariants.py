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
    """The attention kernel sets M0 in inline assembly (LDS base of a global-to-LDS load).  M0 is named as clobbered,
    and on top of that the build refuses to link a library in whose generated code M0 is written anywhere but in front
    of those loads, read by anything else, or in which a kernel of the file spills: the same check, run here."""
    if shutil.which("hipcc") is None:
        pytest.skip("hipcc not available")
    from paper_2502_04420_amd import build as B

    asm = B.device_assembly("kvq_prefill_attn.hip")
    B.check_prefill_attention_code(asm)
    # the check is not vacuous: a second user of M0, or an M0 write away from a fetch, is refused
    name, body = B.kernel_bodies(asm, "prefill_attention")[0]
    planted = asm.replace(body, body.replace("global_load_lds_dwordx4", "s_mov_b32 m0, s5\n\tglobal_load_lds_dwordx4", 1), 1)
    with pytest.raises(RuntimeError):
        B.check_prefill_attention_code(planted)
    planted = asm.replace(body, body.replace("s_nop 0", "v_readlane_b32 s4, v0, m0\n\ts_nop 0", 1), 1)
    with pytest.raises(RuntimeError):
        B.check_prefill_attention_code(planted)


def test_quantize_kernel_keeps_the_fused_widen_and_subtract(tmp_path):
    """x - z is meant to be one mixed-precision instruction per element (both fp16 operands widened inside it); the
    multiplier 1.0 is hidden from the optimiser for that.  If a compiler folds it after all, the code is still right
    but slower: this test tells."""
    asm = _assembly("kvq_quantize.hip", tmp_path, extra=("-ffp-contract=off",))
    kernels = [b for n, b in _kernels(asm, "quantize_blocks") if "ILi4ELi2ELb0E" in n]
    assert len(kernels) == 1
    assert len(re.findall(r"^\s*v_fma_mix_f32 ", kernels[0], re.M)) >= 128      # 2 tensors x 64 elements per lane


def test_builtin_scratch_array_is_visible_to_the_loader():
    """kvq_decode_attention_noalloc asks the runtime for the device address of the library's built-in scratch array.
    That only works if the device code object exports the array as a global symbol (an attribute such as `used` keeps
    a static device variable local, the lookup then yields an address that is not the array's, and the first kernel
    that uses it faults).  Checked on the object the build produced."""
    tools = "/opt/rocm/llvm/bin"
    obj = os.path.join(ROOT, "paper_2502_04420_amd", "_build", "kvq_api.o")
    if not (os.path.exists(obj) and all(os.path.exists(os.path.join(tools, t)) for t in ("llvm-objcopy", "clang-offload-bundler", "llvm-readelf"))):
        pytest.skip("needs the built object and the LLVM binary tools")
    import tempfile

    with tempfile.TemporaryDirectory() as tmp:
        fat, co = os.path.join(tmp, "fat.bin"), os.path.join(tmp, "api.co")
        subprocess.check_call([os.path.join(tools, "llvm-objcopy"), "-O", "binary", "--only-section=.hip_fatbin", obj, fat])
        subprocess.check_call([os.path.join(tools, "clang-offload-bundler"), "--type=o", "--input=" + fat,
                               "--targets=hipv4-amdgcn-amd-amdhsa--gfx950", "--output=" + co, "--unbundle"])
        syms = subprocess.check_output([os.path.join(tools, "llvm-readelf"), "-s", co], text=True)
    rows = [l.split() for l in syms.splitlines() if l.strip().endswith("scratch")]
    assert rows, "no scratch symbol in the device code object"
    assert all(r[4] == "GLOBAL" and r[3] == "OBJECT" and int(r[2]) == 16384 * 130 * 4 for r in rows), rows


def test_decode_kernels_leave_hand_issued_loads_alone():
    """The matrix-core decode kernels issue their block loads in inline assembly and wait for them with hand-written
    counts.  The build refuses a library in whose generated code an instruction of the compiler's own touches a
    register such a load may still be writing: the same check, run here on one instantiation, and shown not to be
    vacuous by planting a copy of an in-flight register."""
    if shutil.which("hipcc") is None:
        pytest.skip("hipcc not available")
    from paper_2502_04420_amd import build as B

    asm = B.device_assembly("kvq_decode_mfma.hip")
    assert B.check_decode_code(asm) > 1000                               # every instantiation streams through these loads
    name, body = [kb for kb in B.kernel_bodies(asm, "decode_mfma") if "ILi4ELi2ELi4ELb0ELb0E" in kb[0]][0]
    m = re.search(r"buffer_load_dwordx4 (v\[(\d+):\d+\]), [^\n]*\n\s*;;#ASMEND\n", body)
    assert m
    planted = body[:m.end()] + "\tv_mov_b32_e32 v200, v%s\n" % m.group(2) + body[m.end():]
    with pytest.raises(RuntimeError):
        B.check_decode_code(asm.replace(body, planted, 1))

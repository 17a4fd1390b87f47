"""The device compiler honours the switch that keeps packed fp32 arithmetic out of the kernels: the ISA
generated with the library's flags contains no v_pk_add_f32 / v_pk_mul_f32 / v_pk_fma_f32, while the
same source without the switch does (so the check can tell the difference)."""
import os
import re
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PK = re.compile(r"\bv_pk_(add|mul|fma)_f32\b")


def _isa(flags, src):
    r = subprocess.run(["hipcc"] + flags + ["-S", "--cuda-device-only", "-I" + os.path.join(ROOT, "include"), "-o", "-", src],
                       capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    return r.stdout


def test_no_packed_fp32_instructions_in_device_code(tmp_path):
    from paper_2001_02772_amd import rec
    probe = tmp_path / "probe.hip"
    probe.write_text("#include <hip/hip_runtime.h>\n"
                     "__global__ void k(float2* a, const float2* b) { float2 x = a[threadIdx.x], y = b[threadIdx.x];\n"
                     "  x.x = x.x * y.x + 1.f; x.y = x.y * y.y + 1.f; a[threadIdx.x] = x; }\n")
    plain = [f for f in rec.HIPCC_FLAGS if f not in ("-Xclang", "-target-feature", "-packed-fp32-ops")]
    assert PK.search(_isa(plain, str(probe))), "the probe no longer provokes packed fp32 code: the check below proves nothing"
    assert not PK.search(_isa(rec.HIPCC_FLAGS, str(probe)))
    for name in ("sls.hip", "interact.hip"):
        assert not PK.search(_isa(rec.HIPCC_FLAGS, os.path.join(ROOT, "paper_2001_02772_amd", "csrc", name))), name

"""CPU-only checks of what the build flags promise about the DEVICE code (hipcc cross-compiles for
gfx950 without a GPU; the assembly read here is that of this repository's own kernels):

- the packed-fp32 feature switch is honoured by the gfx950 device pass (the x86 host pass prints
  "not a recognized feature", which says nothing about the device pass);
- no kernel of the library contains a packed fp32 add/mul/fma;
- the update and averaging kernels round once per operation: no fused fp32 multiply-add in them, except
  in the Adam kernels, whose correctly rounded division is built from them by the compiler.
"""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

pytestmark = pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not installed")

PROBE = r"""
#include <hip/hip_runtime.h>
__global__ void probe(const float2 *a, const float2 *b, float2 *c, int n)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        float2 x = a[i], y = b[i], r;
        r.x = x.x * y.x + 1.0f;
        r.y = x.y * y.y + 1.0f;
        r.x = r.x + x.x;
        r.y = r.y + x.y;
        c[i] = r;
    }
}
"""

PACKED = re.compile(r"\bv_pk_(add|mul|fma)_f32\b")
FUSED = re.compile(r"\bv_(fma|fmac|mad|madak|madmk|fmaak|fmamk)_f32\b")


def device_asm(src, flags, tmp_path, name):
    out = os.path.join(tmp_path, name + ".s")
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-S", "--cuda-device-only", *flags,
                    "-o", out, src], check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    return open(out).read()


def test_packed_fp32_switch_is_honoured_by_the_device_pass(tmp_path):
    src = os.path.join(tmp_path, "probe.hip")
    open(src, "w").write(PROBE)
    off = ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
    assert PACKED.search(device_asm(src, [], str(tmp_path), "default")), \
        "probe no longer provokes packed fp32 code: the check below would prove nothing"
    assert not PACKED.search(device_asm(src, off, str(tmp_path), "switched_off"))


def test_library_kernels_have_no_packed_fp32_and_no_fused_multiply_add(tmp_path):
    from paper_2307_07950_amd import build
    flags = [f for f in build.HIPCC_FLAGS if f not in ("-fPIC", "-shared", "--offload-arch=gfx950", "-O3", "-std=c++17")]
    for source in build.SOURCES:
        if source == "selsync_host.hip":
            continue                                    # no kernels in it
        asm = device_asm(os.path.join(build.CSRC, source), flags, str(tmp_path), source)
        assert "global_load" in asm and ".amdhsa_kernel" in asm         # this really is the device code
        assert not PACKED.search(asm), source
        # Split into functions.  The kernels that carry the method's fp32 arithmetic must not hold a fused
        # fp32 multiply-add, except the Adam ones, whose correctly rounded division the compiler builds from
        # them (other kernels may: integer division by a run-time value is expanded through fp32 too).
        parts = re.split(r"\n(?=_Z[\w]+:\s*; @)", asm)
        checked = 0
        for part in parts:
            name = part.split(":", 1)[0]
            if not any(k in name for k in ("k_stream", "k_aggregate", "k_update_ga", "k_sync_step")):
                continue
            checked += 1
            if FUSED.search(part):
                assert "AdamOpt" in name, "fused fp32 multiply-add in %s (%s)" % (name[:80], source)
        if source == "selsync_kernels.hip":
            assert checked > 50

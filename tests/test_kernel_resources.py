"""The kernels must not touch scratch (private) memory: a register array indexed by a runtime
value is silently moved there by the compiler, and the spills are real HBM traffic (a four-float
array indexed in a loop with a runtime bound once cost the headline tick 40 MB per launch,
8 % of its traffic, without failing any parity test).  Compiles the device code to assembly
(no GPU needed) and reads the resource summary the compiler writes for every kernel."""
import os
import re
import subprocess

import pytest

from paper_2602_01665_amd import build as hip_build


@pytest.fixture(scope="module")
def kernels(tmp_path_factory):
    """(name, metadata text) of every kernel, and the whole assembly listing."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in hip_build.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    asm = tmp_path_factory.mktemp("asm") / "tabx_kernels.s"
    subprocess.run([hipcc] + flags + ["-S", "--cuda-device-only"] + hip_build.SOURCES +
                   ["-o", str(asm)], check=True, capture_output=True)
    text = asm.read_text()
    return re.findall(r"\.name:\s+(_ZN4tabx\w+)\n(.*?)\.wavefront_size", text, re.S), text


def test_no_kernel_uses_scratch_memory_or_spills_vector_registers(kernels):
    """No kernel may execute a scratch instruction or spill a vector register.  (The compiler
    sometimes leaves a few dozen bytes of private segment RESERVED for scalar spill slots that it
    then keeps in vector-register lanes: which instantiation gets them changes with any edit.
    Such a reservation costs no traffic; what the test forbids is code that touches the segment,
    and the two launches the benchmark times must not even reserve it.)"""
    kernels, text = kernels
    assert len(kernels) >= 15          # every instantiation of the tick kernel, reset, global state
    for name, meta in kernels:
        private = int(re.search(r"\.private_segment_fixed_size:\s+(\d+)", meta).group(1))
        spills = int(re.search(r"\.vgpr_spill_count:\s+(\d+)", meta).group(1))
        vgprs = int(re.search(r"\.vgpr_count:\s+(\d+)", meta).group(1))
        assert private <= 64, f"{name} reserves {private} bytes of scratch memory per lane"
        headline = "tabx_tick_kernelILi1ELb0ELb1ELb1ELb0ELi2E" in name or \
                   "tabx_tick_kernelILi1ELb0ELb1ELb1ELb0ELi0E" in name or \
                   "tabx_tick_kernelILi2ELb0ELb1ELb1ELb0ELi0E" in name
        assert private == 0 or not headline, f"{name} reserves {private} bytes of scratch memory"
        assert spills == 0, f"{name} spills {spills} vector registers"
        assert vgprs <= 256, name
    assert not re.search(r"\bscratch_(load|store)", text)
    assert not re.search(r"\bbuffer_(load|store)\w* .*\boffen\b", text)


def test_headline_launch_keeps_six_workgroups_per_cu(kernels):
    """The fused tick of the headline shape runs two wavefronts per env group, and a CU holds six
    such workgroups only while one takes at most 21 LDS allocation granules of 1280 bytes
    (measured: with 768 bytes more than today the launch is unchanged, with 1024 it loses the sixth
    workgroup and 8 % of its speed) and at most 168 vector registers (three wavefronts per SIMD)."""
    from paper_2602_01665_amd import binding as B
    from paper_2602_01665_amd import inputs as I
    meta, text = dict(kernels[0]), kernels[1]
    name = next(k for k in meta if "tabx_tick_kernelILi1ELb0ELb1ELb1ELb0ELi2E" in k)
    static = int(re.search(r"\.amdhsa_kernel " + name + r"\n\s+\.amdhsa_group_segment_fixed_size (\d+)",
                           text).group(1))
    vgprs = int(re.search(r"\.vgpr_count:\s+(\d+)", meta[name]).group(1))
    assert vgprs <= 168
    for name in ("c3_16384env_10v10", "c3e_16384env_10v10_ellipses"):
        info = B.tabx_launch_info(B.make_params(I.make_params(I.WORKLOADS[name])), "step_observe")
        assert info["wavefronts_per_env_group"] == 2 and info["threads_per_workgroup"] == 128
        assert static + info["dynamic_lds_bytes"] <= 21 * 1280, (name, static, info)

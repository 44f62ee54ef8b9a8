"""The kernels must not touch scratch (private) memory: a register array indexed by a runtime
value is silently moved there by the compiler, and the spills are real HBM traffic (a four-float
array indexed in a loop with a runtime bound once cost the headline tick 40 MB per launch,
8 % of its traffic, without failing any parity test).  Compiles the device code to assembly
(no GPU needed) and reads the resource summary the compiler writes for every kernel."""
import os
import re
import subprocess

from paper_2602_01665_amd import build as hip_build


def test_no_kernel_uses_scratch_memory_or_spills_vector_registers(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in hip_build.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    asm = tmp_path / "tabx_kernels.s"
    subprocess.run([hipcc] + flags + ["-S", "--cuda-device-only"] + hip_build.SOURCES +
                   ["-o", str(asm)], check=True, capture_output=True)
    text = asm.read_text()
    kernels = re.findall(r"\.name:\s+(_ZN4tabx\w+)\n(.*?)\.wavefront_size", text, re.S)
    assert len(kernels) >= 15          # every instantiation of the tick kernel, reset, global state
    for name, meta in kernels:
        private = int(re.search(r"\.private_segment_fixed_size:\s+(\d+)", meta).group(1))
        spills = int(re.search(r"\.vgpr_spill_count:\s+(\d+)", meta).group(1))
        vgprs = int(re.search(r"\.vgpr_count:\s+(\d+)", meta).group(1))
        assert private == 0, f"{name} uses {private} bytes of scratch memory per lane"
        assert spills == 0, f"{name} spills {spills} vector registers"
        assert vgprs <= 256, name
    assert not re.search(r"\bscratch_(load|store)", text)

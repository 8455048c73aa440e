"""What the compiler made of the kernels, checked without a GPU: no kernel of the library may use
scratch (private) memory.  In the Attention kernel a scratch store sits in a streaming wave,
where any store makes the waits on the tile loads inexact (a struct with padding bytes or a
small array of HIP's vector structs is enough for the compiler to produce one); in the cache
kernels it would double the traffic.  Also: register counts within what two waves per SIMD
allow (the Attention kernel's workgroup has five waves on four SIMDs)."""
import os
import re
import shutil
import subprocess

import pytest

from paper_2509_08309_amd import build

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def kernel_metadata(source, tmp_path):
    asm = tmp_path / (source + ".s")
    flags = [f for f in build.HIPCC_FLAGS if f not in ("-fPIC", "-shared")]
    subprocess.run([HIPCC] + flags + ["-S", "--cuda-device-only", "-o", str(asm),
                                      os.path.join(build.CSRC, source)], check=True,
                   stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    text = asm.read_text()
    meta = {}
    for m in re.finditer(r"\.name:\s+(\S+)\n((?:\s+\.\w+:.*\n)+)", text):
        fields = dict(re.findall(r"\.(\w+):\s+(\S+)", m.group(2)))
        if "vgpr_count" in fields:
            meta[m.group(1)] = fields
    return meta


@pytest.mark.skipif(shutil.which(HIPCC) is None, reason="hipcc not found")
@pytest.mark.parametrize("source,expected", [("hetis_attn.hip", 48), ("hetis_kv.hip", 8)])
def test_no_kernel_uses_scratch_memory(source, expected, tmp_path):
    meta = kernel_metadata(source, tmp_path)
    main = {k: v for k, v in meta.items() if "persistent_kernel" in k or "kv_" in k}
    assert len(main) == expected, sorted(meta)
    for name, f in meta.items():
        assert int(f["private_segment_fixed_size"]) == 0, (name, f["private_segment_fixed_size"])
        assert int(f.get("vgpr_spill_count", 0)) == 0, name
        assert int(f["vgpr_count"]) + int(f.get("agpr_count", 0)) <= 256, (name, f["vgpr_count"])

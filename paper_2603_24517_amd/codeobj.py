"""Reads the metadata notes of the gfx950 code object inside a built library (register counts, scratch
size, spills per kernel).  Metadata only: nothing is disassembled."""
import os
import re
import subprocess
import tempfile

LLVM_BIN = os.environ.get("ROCM_LLVM_BIN", "/opt/rocm/llvm/bin")
TARGET = "hipv4-amdgcn-amd-amdhsa--gfx950"
FIELDS = ("vgpr_count", "agpr_count", "sgpr_count", "vgpr_spill_count", "sgpr_spill_count",
          "private_segment_fixed_size", "group_segment_fixed_size", "max_flat_workgroup_size")


def kernel_metadata(lib_path):
    """{kernel symbol: {field: int}} for every kernel of the library's gfx950 code object."""
    with tempfile.TemporaryDirectory() as tmp:
        fatbin, code = os.path.join(tmp, "fatbin"), os.path.join(tmp, "code.o")
        subprocess.run([os.path.join(LLVM_BIN, "llvm-objcopy"), "-O", "binary", "--only-section=.hip_fatbin",
                        lib_path, fatbin], check=True)
        subprocess.run([os.path.join(LLVM_BIN, "clang-offload-bundler"), "--unbundle", "--type=o",
                        f"--targets={TARGET}", f"--input={fatbin}", f"--output={code}"], check=True)
        notes = subprocess.run([os.path.join(LLVM_BIN, "llvm-readelf"), "--notes", code], check=True,
                               capture_output=True, text=True).stdout
    kernels = {}
    for entry in re.split(r"\n\s*- \.", notes):
        name = re.search(r"\.name:\s+(\S+)", entry)
        if not name or ".vgpr_count" not in entry and "vgpr_count" not in entry:
            continue
        fields = {}
        for f in FIELDS:
            m = re.search(r"\.?%s:\s+(\d+)" % f, entry)
            if m:
                fields[f] = int(m.group(1))
        if "vgpr_count" in fields:
            kernels[name.group(1)] = fields
    return kernels

"""The built code objects keep every kernel inside the register file and out of scratch memory.

The key-block loop counts its own outstanding tile loads (s_waitcnt vmcnt(n) written by hand); a
register spill would put reloads of the compiler's own into that loop, each behind a wait for every
tile request in flight, so "no scratch, no spilled vector register" is a rule of the shipped library
and of every variant that the GPU tests run.  Read from the metadata notes of the code object."""
import pytest

from paper_2603_24517_amd import build as B
from paper_2603_24517_amd import codeobj

LIBS = [("shipped", B.LIB)] + [(n, B.variant_path(n)) for n in B.VARIANTS]


@pytest.mark.parametrize("name,path", LIBS, ids=[n for n, _ in LIBS])
def test_attention_kernels_have_no_scratch_and_fit_the_register_file(name, path):
    meta = codeobj.kernel_metadata(path)
    kernels = {k: v for k, v in meta.items() if "attn_fwd_kernel" in k or "attn_fwd_split_kernel" in k}
    assert len(kernels) == 8 and len(meta) == 8, sorted(meta)       # two kernels x causal x sign of the scale
    for k, f in kernels.items():
        assert f["private_segment_fixed_size"] == 0, (name, k, f)
        assert f["vgpr_spill_count"] == 0, (name, k, f)
        assert f["vgpr_count"] + f.get("agpr_count", 0) <= 256, (name, k, f)    # two wavefronts per SIMD
        assert f["group_segment_fixed_size"] == 0, (name, k, f)                 # LDS is dynamic: all 160 KiB
        assert f["max_flat_workgroup_size"] == 512, (name, k, f)


def test_probe_kernels_have_no_scratch():
    meta = codeobj.kernel_metadata(B.PROBE_LIB)
    assert len(meta) == 8
    for k, f in meta.items():
        assert f["private_segment_fixed_size"] == 0 and f["vgpr_spill_count"] == 0, (k, f)
        assert f["vgpr_count"] + f.get("agpr_count", 0) <= 128, (k, f)         # up to four wavefronts per SIMD

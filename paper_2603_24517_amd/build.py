"""Build the gfx950 shared libraries in-tree with hipcc.

    python -m paper_2603_24517_amd.build            the attention library (C ABI of include/attn.h)
    python -m paper_2603_24517_amd.build --all      that, the measurement-aid library (include/attn_probe.h)
                                                     and every variant of the attention kernel

The variants are builds of the same source with one compile-time switch each (see the head of
csrc/attn_fwd.hip); they exist to measure the shipped choices against their alternatives and are
never loaded by the product path.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "attn_fwd.hip")
LIB = os.path.join(HERE, "libattn_mi355x.so")
PROBE_SRC = os.path.join(HERE, "csrc", "attn_probe.hip")
PROBE_LIB = os.path.join(HERE, "libattn_probe.so")
VARIANT_DIR = os.path.join(HERE, "variants")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed FP32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]

# name -> extra compiler flags; what each stands for is described where the switches are defined
VARIANTS = {
    "softmax_blockmax_always": ["-DATTN_SOFTMAX=1"],
    "softmax_blockmax_vote": ["-DATTN_SOFTMAX=2"],
    "softmax_blockmax_threshold": ["-DATTN_SOFTMAX=3"],
    "no_item_overlap": ["-DATTN_ITEM_OVERLAP=0"],
    # every launch through the 256-row kernel / every launch through the split-key kernel for small problems
    "no_small_path": ["-DATTN_SMALL_PATH=0"],
    "always_small_path": ["-DATTN_SMALL_PATH=2"],
    "lds_prefetch_1": ["-DATTN_LDS_PREFETCH=1"],
    "lds_prefetch_5": ["-DATTN_LDS_PREFETCH=5"],
    # the shipped kernel plus clock stamps of its first workgroup (exports attn_clocks_read as well)
    "clocks": ["-DATTN_CLOCKS"],
    # the same plus cycle sums per phase of one work item (exports attn_phases_read as well)
    "phases": ["-DATTN_CLOCKS=2"],
}


def variant_path(name):
    return os.path.join(VARIANT_DIR, f"libattn_{name}.so")


def _hipcc(flags, out, src, verbose):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *flags, "-o", out, src]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return out


def build_library(extra_flags=(), out=LIB, verbose=False):
    return _hipcc(list(extra_flags), out, SRC, verbose)


def build_probe(verbose=False):
    return _hipcc([], PROBE_LIB, PROBE_SRC, verbose)


def build_variants(names=None, verbose=False):
    os.makedirs(VARIANT_DIR, exist_ok=True)
    return [build_library(VARIANTS[n], variant_path(n), verbose) for n in (names or VARIANTS)]


def build_all(verbose=False, jobs=4):
    """Everything, a few compilations at a time (each is a single-threaded hipcc run of about ten seconds)."""
    from concurrent.futures import ThreadPoolExecutor
    os.makedirs(VARIANT_DIR, exist_ok=True)
    tasks = [lambda: build_library(verbose=verbose), lambda: build_probe(verbose=verbose)]
    tasks += [lambda n=n: build_library(VARIANTS[n], variant_path(n), verbose) for n in VARIANTS]
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        for f in [pool.submit(t) for t in tasks]:
            f.result()


if __name__ == "__main__":
    if sys.argv[1:] == ["--all"]:
        build_all(verbose=True)
    else:
        print(build_library(extra_flags=sys.argv[1:], verbose=True))

"""The variant builds of the attention kernel (one compile-time switch each, see the head of
csrc/attn_fwd.hip) and the measurement-aid library, on the GPU: every variant goes through the same
parity checks against the FP64 oracle as the shipped kernel, so that what is measured against the
shipped choice (the alternatives that sections 5.1 and 5.2 of the paper weigh on its hardware) is a
correct kernel too."""
import math

import numpy as np
import pytest
import torch

from paper_2603_24517_amd import build as B
from paper_2603_24517_amd import probe as P
from paper_2603_24517_amd import workloads as W
import gpu_util as U

pytestmark = pytest.mark.gpu
SCALE = 1.0 / math.sqrt(128)

# B, Hq, Hkv, Sq, Skv, q_mul: ragged tiles, head packing, several items per workgroup, moving maxima
SHAPES = [
    (1, 2, 2, 300, 200, 1.0), (2, 8, 2, 333, 777, 1.0), (1, 3, 1, 700, 130, 4.0), (3, 16, 16, 520, 520, 1.0),
    (2, 64, 8, 260, 260, 1.0), (1, 4, 4, 1500, 2100, 16.0), (40, 8, 8, 256, 256, 4.0),
]


def _entry(name):
    return lambda *a: P.variant_attn_fwd(name, *a)


# The shipped library sends launches with few 256-row work items to the split-key kernel, which would
# leave the small shapes of the parity tests to that kernel alone: the two builds below pin the choice,
# so that BOTH kernels see every small and ragged shape (and the split-key kernel some larger ones).
import test_attn_gpu as T     # noqa: E402


@pytest.mark.parametrize("causal", [False, True], ids=["full", "causal"])
@pytest.mark.parametrize("shape", T.SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("name", ["no_small_path", "always_small_path"])
def test_both_kernels_on_small_shapes(name, shape, causal):
    Bn, Hq, Hkv, Sq, Skv = shape
    q, k, v = U.rand_qkv(Bn, Hq, Hkv, Sq, Skv, seed=hash(shape) % 10000)
    print(f"variant {name} shape={shape} causal={causal}", flush=True)
    U.check_full(q, k, v, causal, SCALE, what=f"{name} {shape} causal={causal}", attn_fwd=_entry(name))


@pytest.mark.parametrize("name", ["no_small_path", "always_small_path"])
def test_both_kernels_on_random_shapes_and_hard_cases(name):
    rng = np.random.default_rng(20260325)
    for n in range(24):
        hkv = int(rng.choice([1, 2, 3, 5]))
        g = int(rng.choice([1, 2, 3, 4, 6, 8, 16]))
        Bn = int(rng.integers(1, 4))
        Sq = int(rng.integers(1, 700))
        Skv = int(rng.integers(1, 900))
        causal = bool(rng.integers(0, 2))
        q_mul = float(rng.choice([1.0, 1.0, 4.0]))
        print(f"variant {name} case {n}: B={Bn} Hq={hkv * g} Hkv={hkv} Sq={Sq} Skv={Skv} causal={causal} q_mul={q_mul}", flush=True)
        q, k, v = U.rand_qkv(Bn, hkv * g, hkv, Sq, Skv, seed=3000 + n, q_mul=q_mul)
        U.check_full(q, k, v, causal, SCALE, what=f"{name} random case {n}", attn_fwd=_entry(name))
    # rows without keys, huge scores, negative scale, keys that dominate
    q, k, v = U.rand_qkv(1, 2, 2, 300, 40, seed=3)
    U.check_full(q, k, v, True, SCALE, what=f"{name} empty rows", attn_fwd=_entry(name))
    q, k, v = U.rand_qkv(1, 2, 2, 640, 1024, seed=33, q_mul=64.0)
    U.check_full(q, k, v, False, 1.0, what=f"{name} huge scores", attn_fwd=_entry(name))
    U.check_full(q, k, v, True, -1.0, what=f"{name} huge scores, negative scale", attn_fwd=_entry(name))
    q, _, v = U.rand_qkv(2, 4, 4, 500, 500, seed=34, q_mul=1.5)
    U.check_full(q, q.clone(), v, True, SCALE, what=f"{name} K = Q", attn_fwd=_entry(name))


def test_split_kernel_long_keys_few_rows():
    """What the split-key kernel is for: a handful of query rows against a long key sequence."""
    for (Bn, Hq, Hkv, Sq, Skv, causal) in [(1, 8, 2, 1, 20000, False), (2, 4, 4, 17, 9001, True), (1, 32, 8, 64, 4096, True)]:
        q, k, v = U.rand_qkv(Bn, Hq, Hkv, Sq, Skv, seed=4400 + Sq)
        print(f"shape {(Bn, Hq, Hkv, Sq, Skv)} causal={causal}", flush=True)
        U.check_full(q, k, v, causal, SCALE, what=f"long keys {(Bn, Hq, Hkv, Sq, Skv)}")


@pytest.mark.parametrize("causal", [False, True], ids=["full", "causal"])
@pytest.mark.parametrize("name", sorted(B.VARIANTS))
def test_variant_parity_small_shapes(name, causal):
    for n, (Bn, Hq, Hkv, Sq, Skv, q_mul) in enumerate(SHAPES):
        print(f"variant {name} causal={causal} shape={SHAPES[n]}", flush=True)
        q, k, v = U.rand_qkv(Bn, Hq, Hkv, Sq, Skv, seed=8100 + n, q_mul=q_mul)
        U.check_full(q, k, v, causal, SCALE, what=f"{name} {SHAPES[n]}", attn_fwd=_entry(name))


@pytest.mark.parametrize("name", sorted(B.VARIANTS))
def test_variant_scores_jump_and_sorted_keys(name):
    """Maxima that keep rising: where the variants differ from each other."""
    q, k, v = U.rand_qkv(1, 2, 2, 2048, 2048, seed=32)
    k = k.float()
    k[:, 1024:] *= 40.0
    for causal in (False, True):
        U.check_full(q, k.to(torch.bfloat16), v, causal, SCALE, what=f"{name} score jump", attn_fwd=_entry(name))
    S = 512
    q = (torch.ones(1, 64, 1, 128) * 0.5).to(torch.bfloat16)
    k = (torch.linspace(-4.0, 4.0, S).view(1, S, 1, 1) * torch.ones(1, S, 1, 128)).to(torch.bfloat16)
    v = torch.randn(1, S, 1, 128, generator=torch.Generator().manual_seed(5)).to(torch.bfloat16)
    U.check_full(q, k, v, False, 0.5, what=f"{name} sorted keys", attn_fwd=_entry(name))


@pytest.mark.parametrize("name", sorted(B.VARIANTS))
def test_variant_headline_and_short_causal_sampled_rows(name):
    for wl in ("cfg2_mha_nc_b8_h16_s4096", "cfg3a_mha_c_b8_s4096_q4"):
        w = W.WORKLOADS[wl]
        print(f"variant {name} workload {wl}", flush=True)
        q, k, v = W.make_qkv(w)
        rows = W.sample_rows(w, 768)
        U.check_rows(q, k, v, rows, w.causal, w.scale, what=f"{name} {wl}", ceiling=U.CEILINGS[wl],
                     attn_fwd=_entry(name))


def test_clocks_variant_reports_a_plausible_clock():
    w = W.WORKLOADS["cfg2_mha_nc_b8_h16_s4096"]
    q, k, v = (x.cuda() for x in W.make_qkv(w))
    o = torch.empty_like(q)
    lse = torch.empty((w.B, w.Hq, w.Sq), dtype=torch.float32, device="cuda")
    for _ in range(3):
        assert P.variant_attn_fwd("clocks", q, k, v, o, lse, w.B, w.Hq, w.Hkv, w.Sq, w.Skv, w.D, False, w.scale,
                                  torch.cuda.current_stream().cuda_stream) == 0
    c = P.clocks_read()
    print(c, flush=True)
    assert 5e5 < c["cycles_first_workgroup"] < 5e6 and 0.5 < c["clock_ghz"] < 2.6
    # 8 items of 64 key blocks per workgroup: an iteration is at least the 2048 matrix-pipe cycles of its MFMAs
    assert c["iterations_per_item"] == 64 and 2048 <= c["cycles_per_iteration"] < 6000
    assert 1000 < c["cycles_between_items"] < 60000


def test_phases_variant_accounts_for_every_cycle_of_an_item():
    w = W.WORKLOADS["cfg3a_mha_c_b8_s4096_q4"]
    q, k, v = (x.cuda() for x in W.make_qkv(w))
    o = torch.empty_like(q)
    lse = torch.empty((w.B, w.Hq, w.Sq), dtype=torch.float32, device="cuda")
    for _ in range(3):
        assert P.variant_attn_fwd("phases", q, k, v, o, lse, w.B, w.Hq, w.Hkv, w.Sq, w.Skv, w.D, True, w.scale,
                                  torch.cuda.current_stream().cuda_stream) == 0
    ph = P.phases_read()
    print(ph, flush=True)
    assert ph is not None
    for wave in ("first_wavefront", "last_wavefront"):
        d = ph[wave]
        # a 256-row item of this workload has 4 .. 64 key blocks: iterations 0 .. nblk-2 are counted by kind, then the last
        n = d["fast_iterations_n"] + d["other_iterations_n"] + 1
        assert 4 <= n <= 64 and n % 4 == 0, d
        assert d["item"] == sum(d[key] for key in ("setup", "first_two_score_blocks", "first_softmax", "barrier_and_first_requests",
                                                  "fast_iterations", "other_iterations", "last_iteration", "wait_for_loads",
                                                  "epilogue"))
        # two score products are 32 MFMAs of 32 matrix-pipe cycles; an iteration of either kind holds 32 as well
        assert d["first_two_score_blocks"] >= 1024 and d["epilogue"] > 0 and d["last_iteration"] >= 512
        iters = d["fast_iterations"] + d["other_iterations"]
        assert 1024 * (n - 1) <= iters < 8000 * (n - 1), d
    # the first wavefront's rows end before the diagonal blocks of the last: it runs fewer fast iterations or as many
    assert ph["first_wavefront"]["fast_iterations_n"] <= ph["last_wavefront"]["fast_iterations_n"]


@pytest.mark.parametrize("waves", [1, 2, 4])
@pytest.mark.parametrize("mode", range(8))
def test_probe_runs(mode, waves):
    ops = torch.randn(12, 64, 8, generator=torch.Generator().manual_seed(7)).to(torch.bfloat16).cuda()
    tiles = torch.randn(1 << 20, generator=torch.Generator().manual_seed(8)).to(torch.bfloat16).cuda()   # 2 MiB
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    clocks = torch.zeros(4, dtype=torch.int64, device="cuda")
    rc = P.attn_probe_mfma(ops, tiles, tiles.numel() * 2, sink, clocks, mode, waves, 50,
                           torch.cuda.current_stream().cuda_stream)
    assert rc == 0
    torch.cuda.synchronize()
    c = clocks.cpu().numpy()
    assert float(sink.item()) == 0.0
    cycles, ticks = int(c[1] - c[0]), int(c[3] - c[2])
    # 50 x 32 MFMAs of 32 matrix-pipe cycles per wavefront, `waves` wavefronts sharing a pipe
    assert cycles >= 50 * 32 * 32 * waves * 0.9 and ticks > 0
    assert 0.5 < 0.1 * cycles / ticks < 2.6

"""GPU parity: the HIP path (through the C ABI) against the FP64 oracle, element by element."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2603_24517_amd as A
from paper_2603_24517_amd import workloads as W
import gpu_util as U

pytestmark = pytest.mark.gpu
SCALE = 1.0 / math.sqrt(128)

# B, Hq, Hkv, Sq, Skv : several tiles, ragged tails, every head-packing factor, Sq != Skv
SHAPES = [
    (1, 1, 1, 1, 1), (1, 1, 1, 1, 70), (1, 1, 1, 33, 1), (1, 2, 2, 64, 64), (2, 2, 2, 100, 77),
    (1, 2, 2, 300, 200), (1, 1, 1, 257, 513), (2, 4, 4, 512, 512), (1, 3, 3, 129, 640),
    (1, 2, 1, 200, 260), (1, 4, 1, 150, 150), (2, 8, 1, 70, 333), (1, 8, 2, 96, 96),
    (1, 3, 1, 90, 190), (1, 6, 2, 130, 65), (1, 16, 1, 40, 129), (1, 12, 3, 65, 64),
    (1, 1, 1, 700, 130), (1, 4, 2, 31, 1000),
]


@pytest.mark.parametrize("causal", [False, True], ids=["full", "causal"])
@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_small_shapes_full_compare(shape, causal):
    B, Hq, Hkv, Sq, Skv = shape
    q, k, v = U.rand_qkv(B, Hq, Hkv, Sq, Skv, seed=hash(shape) % 10000)
    print(f"case shape={shape} causal={causal}", flush=True)
    U.check_full(q, k, v, causal, SCALE, what=f"{shape} causal={causal}")


@pytest.mark.parametrize("q_mul", [4.0, 16.0])
@pytest.mark.parametrize("causal", [False, True])
def test_peaked_softmax(q_mul, causal):
    """Large scores: the running maximum keeps moving and the accumulator is rescaled often."""
    q, k, v = U.rand_qkv(1, 2, 2, 384, 448, seed=77, q_mul=q_mul)
    U.check_full(q, k, v, causal, SCALE, what=f"q_mul={q_mul}")


def test_sorted_keys_force_rescale_every_block():
    """Keys ordered by increasing score for every query: the maximum rises in every block."""
    torch.manual_seed(5)
    S = 512
    q = torch.ones(1, 64, 1, 128) * 0.5
    ramp = torch.linspace(-4.0, 4.0, S).view(1, S, 1, 1)
    k = (ramp * torch.ones(1, S, 1, 128)).to(torch.bfloat16)
    v = torch.randn(1, S, 1, 128).to(torch.bfloat16)
    U.check_full(q.to(torch.bfloat16), k, v, False, 0.5, what="sorted keys")


@pytest.mark.parametrize("scale", [0.0, 1.0, 0.01])
def test_scales(scale):
    q, k, v = U.rand_qkv(1, 2, 2, 130, 140, seed=11)
    q = (q.float() * 0.25).to(torch.bfloat16)
    for causal in (False, True):
        U.check_full(q, k, v, causal, scale, what=f"scale={scale}")


def test_empty_rows_when_sq_gt_skv():
    q, k, v = U.rand_qkv(1, 2, 2, 300, 40, seed=3)
    o, lse = U.run_gpu(q, k, v, True, SCALE)
    assert np.all(lse[:, :, :260] == -np.inf) and np.all(o[:, :260] == 0.0)
    assert np.all(np.isfinite(lse[:, :, 260:]))
    U.check_full(q, k, v, True, SCALE, what="empty rows")


# ---- the definition's invariants, re-run on the GPU path -----------------------------------------
def test_constant_v_gpu():
    q, k, v = U.rand_qkv(1, 4, 2, 200, 300, seed=21)
    c = torch.randn(1, 1, 2, 128).to(torch.bfloat16)
    v = c.expand(1, 300, 2, 128).contiguous()
    for causal in (False, True):
        o, _ = U.run_gpu(q, k, v, causal, SCALE)
        want = c.double().numpy()[:, :, np.repeat(np.arange(2), 2), :]
        assert np.abs(o - want).max() <= 2e-2


def test_zero_q_gives_prefix_mean_gpu():
    _, k, v = U.rand_qkv(1, 2, 2, 150, 150, seed=22)
    q = torch.zeros(1, 150, 2, 128, dtype=torch.bfloat16)
    o, lse = U.run_gpu(q, k, v, True, SCALE)
    vd = v.double().numpy()
    csum = np.cumsum(vd, axis=1) / np.arange(1, 151).reshape(1, -1, 1, 1)
    assert np.abs(o - csum).max() <= 2e-2
    assert np.abs(lse - np.log(np.arange(1, 151))).max() <= 1e-3
    o, lse = U.run_gpu(q, k, v, False, SCALE)
    assert np.abs(o - vd.mean(axis=1, keepdims=True)).max() <= 2e-2
    assert np.abs(lse - math.log(150)).max() <= 1e-3


def test_causal_row0_is_v0_gpu():
    q, k, v = U.rand_qkv(2, 2, 2, 128, 128, seed=23)
    o, lse = U.run_gpu(q, k, v, True, SCALE)
    assert np.array_equal(o[:, 0], v[:, 0].double().numpy())     # p = 1 exactly, V is BF16 already
    s00 = SCALE * (q[:, 0].double() * k[:, 0].double()).sum(-1).numpy()
    assert np.abs(lse[:, :, 0] - s00).max() <= 1e-3


def test_gqa_equals_repeated_mha_gpu():
    q, k, v = U.rand_qkv(1, 8, 2, 160, 200, seed=24)
    o, lse = U.run_gpu(q, k, v, True, SCALE)
    k2, v2 = k.repeat_interleave(4, dim=2), v.repeat_interleave(4, dim=2)
    o2, lse2 = U.run_gpu(q, k2, v2, True, SCALE)
    assert np.abs(o - o2).max() <= 2e-2 and np.abs(lse - lse2).max() <= 1e-3


def test_split_merge_gpu():
    q, k, v = U.rand_qkv(1, 2, 2, 100, 320, seed=25)
    o, lse = U.run_gpu(q, k, v, False, SCALE)
    o1, l1 = U.run_gpu(q, k[:, :128].contiguous(), v[:, :128].contiguous(), False, SCALE)
    o2, l2 = U.run_gpu(q, k[:, 128:].contiguous(), v[:, 128:].contiguous(), False, SCALE)
    tot = np.logaddexp(l1, l2)
    w1 = np.exp(l1 - tot).transpose(0, 2, 1)[..., None]
    w2 = np.exp(l2 - tot).transpose(0, 2, 1)[..., None]
    assert np.abs(lse - tot).max() <= 1e-3
    assert np.abs(o - (w1 * o1 + w2 * o2)).max() <= 2e-2


# (B, Hq, Hkv, Sq, Skv): one launch that goes to the split-key kernel (few rows) and one that goes to the 256-row kernel
BOTH_KERNELS = [(2, 4, 2, 333, 333), (4, 16, 4, 1000, 1100)]


@pytest.mark.parametrize("shape", BOTH_KERNELS, ids=["split_key_kernel", "main_kernel"])
def test_deterministic_and_stream_gpu(shape):
    q, k, v = U.rand_qkv(*shape, seed=26)
    o1, l1 = U.run_gpu(q, k, v, True, SCALE)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        o2, l2 = U.run_gpu(q, k, v, True, SCALE, stream=s.cuda_stream)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)


@pytest.mark.parametrize("shape", [(2, 8, 2, 700, 900), (4, 16, 4, 1000, 1100)], ids=["split_key_kernel", "main_kernel"])
def test_launch_recorded_in_a_hip_graph_replays_identically(shape):
    """attn_fwd only enqueues one kernel, so (after one ordinary call on the device) it can be recorded
    into a HIP graph; every replay, with other work and synchronisations in between, must reproduce the
    directly launched result bit for bit."""
    B, Hq, Hkv, Sq, Skv = shape
    q, k, v = U.rand_qkv(B, Hq, Hkv, Sq, Skv, seed=28)
    o_ref, lse_ref = U.run_gpu(q, k, v, True, SCALE)            # also the first call on the device
    dev = torch.device("cuda:0")
    qd, kd, vd = q.to(dev), k.to(dev), v.to(dev)
    o = torch.zeros_like(qd)
    lse = torch.zeros((B, Hq, Sq), dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        rc = A.attn_fwd(qd, kd, vd, o, lse, B, Hq, Hkv, Sq, Skv, 128, True, SCALE,
                        torch.cuda.current_stream().cuda_stream)
    assert rc == 0, A.attn_strerror(rc)
    for rep in range(4):
        o.fill_(float("nan"))
        lse.fill_(float("nan"))
        other = (qd.float() * 2).sum()                          # unrelated eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(o.cpu().double().numpy(), o_ref), f"replay {rep}: O differs"
        assert np.array_equal(lse.cpu().double().numpy(), lse_ref), f"replay {rep}: LSE differs"
        assert torch.isfinite(other)


def test_attention_wrapper_gpu():
    q, k, v = U.rand_qkv(1, 2, 2, 64, 64, seed=27)
    o, lse = A.attention(q.cuda(), k.cuda(), v.cuda(), causal=True)
    o_ref, lse_ref = oracle.attn_ref(q, k, v, True, SCALE)
    U.compare(o.cpu().double().numpy(), lse.cpu().double().numpy(), o_ref, lse_ref, "wrapper")


# ---- the benchmark configurations ---------------------------------------------------------------------
def test_cfg1_full():
    w = W.WORKLOADS[W.SMALL]
    q, k, v = W.make_qkv(w)
    r = U.check_full(q, k, v, w.causal, w.scale, what=w.name, ceiling=U.CEILINGS[w.name])
    print(w.name, r, flush=True)


BIG = [n for n in W.WORKLOADS if n != W.SMALL]


@pytest.mark.parametrize("name", BIG)
def test_configs_sampled_rows(name):
    """Full-size launch (the one bench.py times); a stratified sample of rows checked one by one."""
    w = W.WORKLOADS[name]
    print(f"case {name}", flush=True)
    q, k, v = W.make_qkv(w)
    rows = W.sample_rows(w, 1536)
    r = U.check_rows(q, k, v, rows, w.causal, w.scale, what=name, ceiling=U.CEILINGS[name])
    print(name, r, flush=True)


@pytest.mark.parametrize("name", sorted(W.PAPER_GRID))
def test_paper_grid_sampled_rows(name):
    """The rest of the paper's own benchmark grid (section 4.1: 16-head MHA, causal and not, at the four
    (batch, sequence) points; section 4.3: 32 query heads on 8 and on 4 K/V heads): the full-size launch,
    a stratified sample of rows checked one by one against the oracle."""
    w = W.PAPER_GRID[name]
    print(f"case {name}", flush=True)
    q, k, v = W.make_qkv(w)
    rows = W.sample_rows(w, 1536)
    r = U.check_rows(q, k, v, rows, w.causal, w.scale, what=name)
    print(name, r, flush=True)


@pytest.mark.parametrize("name", ["cfg2_mha_nc_b8_h16_s4096", "cfg3a_mha_c_b8_s4096_q4", "cfg3b_mha_c_b4_s8192_q4"])
def test_configs_every_row(name):
    """The headline workload and the two shorter causal ones: EVERY row of O and LSE against the oracle
    (about a minute of oracle time in all; the longer workloads are checked this way by tests/full_parity.py)."""
    from full_parity import check_every_row
    r = check_every_row(name, chunk=65536, log=lambda m: print(m, flush=True))
    print(r, flush=True)
    assert r["pass"], r


# Shapes at the far ends of each axis (B, Hq, Hkv, Sq, Skv, causal, q_mul): one head with 1024 key blocks, a
# group of 128 query heads on one K/V head, many tiny batch entries, a very long Q against a short K/V and the
# reverse.  Sampled rows (stratified), every valid key of each.
EXTREMES = [
    (1, 1, 1, 65536, 65536, False, 1.0), (1, 1, 1, 65536, 65536, True, 1.0), (1, 128, 1, 1024, 1024, True, 1.0),
    (300, 2, 2, 256, 256, True, 4.0), (1, 2, 2, 100000, 333, False, 1.0), (1, 2, 2, 333, 100000, True, 1.0),
]


@pytest.mark.parametrize("case", EXTREMES, ids=lambda c: "x".join(map(str, c[:5])) + ("-causal" if c[5] else "-full"))
def test_extreme_shapes_sampled_rows(case):
    B, Hq, Hkv, Sq, Skv, causal, q_mul = case
    w = W.custom("extreme", B, Hq, Hkv, Sq, Skv, causal=causal, seed=700 + EXTREMES.index(case), q_mul=q_mul)
    q, k, v = W.make_qkv(w)
    rows = W.sample_rows(w, 2500)
    print(f"case {case}: {len(rows)} rows", flush=True)
    r = U.check_rows(q, k, v, rows, causal, SCALE, what=str(case))
    print(r, flush=True)


@pytest.mark.parametrize("scale", [-SCALE, -1.0])
@pytest.mark.parametrize("causal", [False, True])
def test_negative_scale(scale, causal):
    """A negative scale turns the largest scaled score into the smallest raw one; every path that looks
    for a maximum (first block, masked blocks, the exact path after an overflow) has to follow."""
    q, k, v = U.rand_qkv(2, 4, 2, 700, 900, seed=41, q_mul=2.0)
    U.check_full(q, k, v, causal, scale, what=f"scale={scale}")
    q, k, v = U.rand_qkv(1, 2, 2, 640, 1024, seed=42, q_mul=48.0)     # overflow of the first guess
    U.check_full(q, k, v, causal, scale, what=f"scale={scale}, huge scores")


def test_random_shapes_gpu():
    """Seeded sweep of irregular shapes: head packing, ragged tiles on both axes, Sq != Skv, odd batch."""
    rng = np.random.default_rng(20260324)
    for n in range(28):
        hkv = int(rng.choice([1, 2, 3, 5]))
        g = int(rng.choice([1, 2, 3, 4, 6, 8, 16]))
        B = int(rng.integers(1, 4))
        Sq = int(rng.integers(1, 700))
        Skv = int(rng.integers(1, 900))
        causal = bool(rng.integers(0, 2))
        q_mul = float(rng.choice([1.0, 1.0, 4.0]))
        print(f"case {n}: B={B} Hq={hkv * g} Hkv={hkv} Sq={Sq} Skv={Skv} causal={causal} q_mul={q_mul}", flush=True)
        q, k, v = U.rand_qkv(B, hkv * g, hkv, Sq, Skv, seed=1000 + n, q_mul=q_mul)
        U.check_full(q, k, v, causal, SCALE, what=f"random case {n}")


@pytest.mark.parametrize("causal", [False, True])
def test_long_ragged_sequence(causal):
    q, k, v = U.rand_qkv(1, 4, 2, 1000, 5037, seed=31)
    U.check_full(q, k, v, causal, SCALE, what="long ragged")


@pytest.mark.parametrize("causal", [False, True])
def test_scores_jump_mid_sequence(causal):
    """Small scores for the first 1024 keys, then keys 40x larger: the running reference must be raised
    in the middle of the unmasked fast path (probabilities overflow the fast path's limit there)."""
    q, k, v = U.rand_qkv(1, 2, 2, 2048, 2048, seed=32)
    k = k.float()
    k[:, 1024:] *= 40.0
    U.check_full(q, k.to(torch.bfloat16), v, causal, SCALE, what="score jump")


@pytest.mark.parametrize("causal", [False, True])
def test_keys_equal_queries_diagonal_dominates(causal):
    """K = Q: every query's own key scores far above the others, so under the causal mask the reference
    has to be raised in the diagonal (masked) block of every query tile, item after item."""
    q, _, v = U.rand_qkv(3, 4, 4, 1100, 1100, seed=34, q_mul=1.5)
    U.check_full(q, q.clone(), v, causal, SCALE, what="K = Q")


def test_huge_scores_overflow_exp():
    """Scores of several hundred: exp2 of the first guess overflows to inf, the exact path must take over."""
    q, k, v = U.rand_qkv(1, 2, 2, 640, 1024, seed=33, q_mul=64.0)
    U.check_full(q, k, v, False, 1.0, what="huge scores")


# More work items than the launch has workgroups (one per CU, 256): every workgroup works through a
# list, and the tiles and Q of an item are requested while the item before it is still in its last
# blocks.  Shapes: (B, Hq, Hkv, Sq, Skv); what each one exercises is named beside it.
MANY_ITEMS = [
    (9, 16, 16, 520, 520),     # 432 items of 9 blocks: second round half full, ragged last tile
    (3, 40, 40, 777, 777),     # 480 items, partial last key block on every item
    (8, 32, 8, 300, 300),      # group of 4 heads packed into a workgroup, 5 blocks per item
    (5, 64, 8, 260, 260),      # group of 8 packed, 32 positions per item
    (4, 24, 24, 900, 500),     # causal: leading tiles without any valid key between regular ones
    (4, 24, 24, 520, 1100),    # causal with more keys than queries
    (16, 32, 32, 128, 128),    # two blocks per item: too short to carry the next item's requests
    (4, 64, 64, 960, 960),     # four rounds, every tile full
    (3, 5, 5, 5000, 5000),     # 15 heads: causal tiles split eight ways over the XCDs
    (2, 6, 2, 4100, 4100),     # 4 groups after packing 3 heads singly: split two ways
    (64, 64, 64, 256, 256),    # 4096 items of exactly four blocks: the shortest item that carries the next one's requests
    (32, 16, 2, 320, 320),     # group of 8 packed, ten tiles of 32 positions, five blocks
    (1, 48, 6, 1111, 1111),    # group of 8 in one chunk, ragged everywhere, six K/V heads
]


@pytest.mark.parametrize("causal", [False, True], ids=["full", "causal"])
@pytest.mark.parametrize("shape", MANY_ITEMS, ids=lambda s: "x".join(map(str, s)))
def test_many_items_per_workgroup(shape, causal):
    B, Hq, Hkv, Sq, Skv = shape
    q, k, v = U.rand_qkv(B, Hq, Hkv, Sq, Skv, seed=7000 + hash(shape) % 1000)
    print(f"case shape={shape} causal={causal}", flush=True)
    U.check_full(q, k, v, causal, SCALE, what=f"{shape} causal={causal}")


def test_back_to_back_launches_of_different_shapes():
    """LDS and registers carry nothing from one launch to the next: alternate two shapes, compare each time."""
    a = U.rand_qkv(6, 16, 16, 600, 600, seed=7101)
    b = U.rand_qkv(2, 8, 2, 333, 1000, seed=7102)
    ref_a = oracle.attn_ref(*a, True, SCALE)
    ref_b = oracle.attn_ref(*b, False, SCALE)
    for n in range(3):
        print(f"round {n}", flush=True)
        U.compare(*U.run_gpu(*a, True, SCALE), *ref_a, what=f"A round {n}")
        U.compare(*U.run_gpu(*b, False, SCALE), *ref_b, what=f"B round {n}")

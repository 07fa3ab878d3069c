"""Pins for the FP64 oracle: what the definition of attention fixes, independent of the oracle's code.

Every function takes an `oracle.Oracle` and raises AssertionError when the
oracle violates the pinned fact.  `ALL_PINS` is run against the real oracle
(must pass) and against deliberately broken builds of it (each must fail at
least one pin).  Definition: paper section 2.2 ("Attention computation"),
causal masking and grouped-query heads from sections 4.1 and 4.3.
"""
import math
import os

import numpy as np
import torch

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _rand(shape, seed, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


def _qkv(B, Hq, Hkv, Sq, Skv, D, seed):
    return (_rand((B, Sq, Hq, D), seed), _rand((B, Skv, Hkv, D), seed + 1),
            _rand((B, Skv, Hkv, D), seed + 2))


def _nvalid(i, Sq, Skv, causal):
    return max(0, min(Skv, i + 1 + Skv - Sq)) if causal else Skv


# P1 ---------------------------------------------------------------------
def pin_probs_sum_to_one(orc):
    B, Hq, Hkv, Sq, Skv, D = 2, 4, 2, 9, 13, 8
    q, k, _ = _qkv(B, Hq, Hkv, Sq, Skv, D, 10)
    for causal in (False, True):
        for (b, h, i) in [(0, 0, 0), (1, 3, 8), (0, 2, 4), (1, 1, 5)]:
            p = orc.attn_ref_probs(q, k, b, h, i, causal, 0.4)
            n = _nvalid(i, Sq, Skv, causal)
            assert np.all(p >= 0)
            assert abs(p.sum() - 1.0) < 1e-13, (causal, b, h, i, p.sum())
            assert np.all(p[n:] == 0.0), "masked keys must have zero weight"
            assert np.all(p[:n] > 0.0)


# P2 ---------------------------------------------------------------------
def pin_constant_v(orc):
    B, Hq, Hkv, Sq, Skv, D = 2, 4, 2, 7, 11, 6
    q, k, _ = _qkv(B, Hq, Hkv, Sq, Skv, D, 20)
    c = _rand((B, 1, Hkv, D), 23)
    v = np.broadcast_to(c, (B, Skv, Hkv, D)).copy()
    for causal in (False, True):
        o, _ = orc.attn_ref(q, k, v, causal, 0.7)
        for h in range(Hq):
            want = np.broadcast_to(c[:, :, h // (Hq // Hkv), :], (B, Sq, D))
            assert np.allclose(o[:, :, h, :], want, atol=1e-13, rtol=0)


# P3 ---------------------------------------------------------------------
def pin_zero_q_gives_mean(orc):
    B, Hq, Hkv, Sq, Skv, D = 2, 4, 2, 6, 10, 5
    _, k, v = _qkv(B, Hq, Hkv, Sq, Skv, D, 30)
    q0 = np.zeros((B, Sq, Hq, D))
    qr = _rand((B, Sq, Hq, D), 33)
    for (q, scale) in ((q0, 0.9), (qr, 0.0)):
        for causal in (False, True):
            o, lse = orc.attn_ref(q, k, v, causal, scale)
            for i in range(Sq):
                n = _nvalid(i, Sq, Skv, causal)
                for h in range(Hq):
                    g = h // (Hq // Hkv)
                    want = v[:, :n, g, :].mean(axis=1)
                    assert np.allclose(o[:, i, h, :], want, atol=1e-13, rtol=0)
                    assert np.allclose(lse[:, h, i], math.log(n), atol=1e-13, rtol=0)


# P4 ---------------------------------------------------------------------
def pin_causal_row0(orc):
    B, H, S, D = 2, 3, 8, 4
    q, k, v = _qkv(B, H, H, S, S, D, 40)
    scale = 0.35
    o, lse = orc.attn_ref(q, k, v, True, scale)
    assert np.array_equal(o[:, 0], v[:, 0])
    s00 = scale * np.einsum("bhd,bhd->bh", q[:, 0], k[:, 0])
    assert np.allclose(lse[:, :, 0], s00, atol=1e-14, rtol=0)
    # with the mask one key too tight / too loose, row 1 would be wrong:
    s = scale * np.einsum("bhd,bjhd->bhj", q[:, 1], k[:, :2])
    w = np.exp(s) / np.exp(s).sum(-1, keepdims=True)
    want = np.einsum("bhj,bjhd->bhd", w, v[:, :2])
    assert np.allclose(o[:, 1], want, atol=1e-13, rtol=0)


# P5 ---------------------------------------------------------------------
def _brute(q, k, v, causal, scale):
    """Scalar loops, softmax written as exp(s)/sum exp(s) with no max subtraction."""
    B, Sq, Hq, D = q.shape
    _, Skv, Hkv, _ = k.shape
    G = Hq // Hkv
    o = np.zeros((B, Sq, Hq, D))
    lse = np.full((B, Hq, Sq), -math.inf)
    for b in range(B):
        for h in range(Hq):
            g = h // G
            for i in range(Sq):
                e = []
                for j in range(Skv):
                    if causal and j > i + Skv - Sq:
                        continue
                    s = 0.0
                    for d in range(D):
                        s += q[b, i, h, d] * k[b, j, g, d]
                    e.append((j, math.exp(scale * s)))
                if not e:
                    continue
                tot = sum(x for _, x in e)
                lse[b, h, i] = math.log(tot)
                for d in range(D):
                    o[b, i, h, d] = sum(x * v[b, j, g, d] for j, x in e) / tot
    return o, lse


def pin_brute_force_tiny(orc):
    cases = [  # B, Hq, Hkv, Sq, Skv, D
        (1, 1, 1, 1, 1, 1), (1, 1, 1, 3, 3, 2), (2, 2, 1, 4, 4, 3), (1, 4, 2, 3, 5, 4),
        (1, 2, 2, 5, 3, 2), (2, 6, 3, 2, 4, 3), (1, 6, 2, 4, 4, 2),
    ]
    for n, (B, Hq, Hkv, Sq, Skv, D) in enumerate(cases):
        q, k, v = _qkv(B, Hq, Hkv, Sq, Skv, D, 50 + 3 * n)
        for causal in (False, True):
            for scale in (1.0, 0.5):
                o, lse = orc.attn_ref(q, k, v, causal, scale)
                bo, bl = _brute(q, k, v, causal, scale)
                assert np.allclose(o, bo, atol=1e-12, rtol=0), (B, Hq, Hkv, Sq, Skv, D, causal)
                fin = np.isfinite(bl)
                assert np.array_equal(np.isfinite(lse), fin)
                assert np.allclose(lse[fin], bl[fin], atol=1e-12, rtol=0)
                if (~fin).any():           # empty rows: O = 0, LSE = -inf
                    assert np.all(lse[~fin] == -math.inf)
                    assert np.all(o.transpose(0, 2, 1, 3)[~fin] == 0.0)


# P6 ---------------------------------------------------------------------
def pin_library_sdpa(orc):
    F = torch.nn.functional
    for (B, Hq, Hkv, S, D, causal) in [(2, 4, 4, 33, 16, False), (1, 4, 4, 40, 8, True),
                                       (2, 8, 2, 17, 16, True), (1, 6, 3, 21, 8, False)]:
        q, k, v = _qkv(B, Hq, Hkv, S, S, D, 60 + S)
        scale = 1.0 / math.sqrt(D)
        o, lse = orc.attn_ref(q, k, v, causal, scale)
        G = Hq // Hkv
        tq = torch.from_numpy(q).permute(0, 2, 1, 3)
        tk = torch.from_numpy(k).permute(0, 2, 1, 3).repeat_interleave(G, dim=1)
        tv = torch.from_numpy(v).permute(0, 2, 1, 3).repeat_interleave(G, dim=1)
        want = F.scaled_dot_product_attention(tq, tk, tv, is_causal=causal, scale=scale)
        assert np.allclose(o, want.permute(0, 2, 1, 3).numpy(), atol=1e-12, rtol=0)
        sc = scale * tq @ tk.transpose(-1, -2)
        if causal:
            sc = sc.masked_fill(torch.ones(S, S, dtype=torch.bool).triu(1), -math.inf)
        assert np.allclose(lse, torch.logsumexp(sc, -1).numpy(), atol=1e-12, rtol=0)


# P7 ---------------------------------------------------------------------
def pin_causal_is_prefix(orc):
    B, Hq, Hkv, D = 1, 2, 1, 4
    for (Sq, Skv) in [(5, 5), (3, 7), (6, 4)]:
        q, k, v = _qkv(B, Hq, Hkv, Sq, Skv, D, 70 + Sq)
        o, lse = orc.attn_ref(q, k, v, True, 0.6)
        for i in range(Sq):
            n = _nvalid(i, Sq, Skv, True)
            if n == 0:
                assert np.all(o[:, i] == 0) and np.all(lse[:, :, i] == -math.inf)
                continue
            po, pl = orc.attn_ref(q[:, i:i + 1], k[:, :n], v[:, :n], False, 0.6)
            assert np.allclose(o[:, i], po[:, 0], atol=1e-13, rtol=0), (Sq, Skv, i)
            assert np.allclose(lse[:, :, i], pl[:, :, 0], atol=1e-13, rtol=0)


# P8 ---------------------------------------------------------------------
def pin_gqa_is_repeated_mha(orc):
    B, Hq, Hkv, Sq, Skv, D = 2, 6, 2, 5, 7, 4
    q, k, v = _qkv(B, Hq, Hkv, Sq, Skv, D, 80)
    G = Hq // Hkv
    for causal in (False, True):
        o, lse = orc.attn_ref(q, k, v, causal, 0.5)
        o2, lse2 = orc.attn_ref(q, np.repeat(k, G, axis=2), np.repeat(v, G, axis=2), causal, 0.5)
        assert np.allclose(o, o2, atol=1e-14, rtol=0) and np.allclose(lse, lse2, atol=1e-14, rtol=0)


# P9 ---------------------------------------------------------------------
def pin_key_permutation(orc):
    B, Hq, Hkv, Sq, Skv, D = 1, 2, 2, 4, 9, 4
    q, k, v = _qkv(B, Hq, Hkv, Sq, Skv, D, 90)
    perm = np.random.default_rng(91).permutation(Skv)
    o, lse = orc.attn_ref(q, k, v, False, 0.8)
    o2, lse2 = orc.attn_ref(q, k[:, perm], v[:, perm], False, 0.8)
    assert np.allclose(o, o2, atol=1e-13, rtol=0) and np.allclose(lse, lse2, atol=1e-13, rtol=0)


# P10 --------------------------------------------------------------------
def pin_split_merge(orc):
    B, Hq, Hkv, Sq, Skv, D = 1, 2, 1, 3, 10, 4
    q, k, v = _qkv(B, Hq, Hkv, Sq, Skv, D, 100)
    a = 4
    o, lse = orc.attn_ref(q, k, v, False, 0.9)
    o1, l1 = orc.attn_ref(q, k[:, :a], v[:, :a], False, 0.9)
    o2, l2 = orc.attn_ref(q, k[:, a:], v[:, a:], False, 0.9)
    tot = np.log(np.exp(l1) + np.exp(l2))                      # [B,H,Sq]
    w1 = np.exp(l1 - tot).transpose(0, 2, 1)[..., None]
    w2 = np.exp(l2 - tot).transpose(0, 2, 1)[..., None]
    assert np.allclose(lse, tot, atol=1e-13, rtol=0)
    assert np.allclose(o, w1 * o1 + w2 * o2, atol=1e-13, rtol=0)


# P11 --------------------------------------------------------------------
def pin_score_shift(orc):
    B, H, Sq, Skv, D = 1, 2, 3, 6, 4
    q, k, v = _qkv(B, H, H, Sq, Skv, D, 110)
    scale, c = 0.5, 3.25
    o, lse = orc.attn_ref(q, k, v, False, scale)
    q2 = np.concatenate([q, np.ones((B, Sq, H, 1))], axis=-1)
    k2 = np.concatenate([k, np.full((B, Skv, H, 1), c / scale)], axis=-1)
    v2 = np.concatenate([v, np.zeros((B, Skv, H, 1))], axis=-1)
    o2, lse2 = orc.attn_ref(q2, k2, v2, False, scale)
    assert np.allclose(o2[..., :D], o, atol=1e-13, rtol=0)
    assert np.allclose(lse2, lse + c, atol=1e-12, rtol=0)


# P12 --------------------------------------------------------------------
def pin_dominant_key(orc):
    B, H, Sq, Skv, D = 1, 1, 2, 5, 2
    q = np.zeros((B, Sq, H, D)); q[..., 0] = 1.0
    k = np.zeros((B, Skv, H, D)); k[:, 3, :, 0] = 1000.0      # score 1000 vs 0: exp would overflow
    v = _rand((B, Skv, H, D), 120)
    o, lse = orc.attn_ref(q, k, v, False, 1.0)
    assert np.all(np.isfinite(o)) and np.all(np.isfinite(lse))
    assert np.allclose(o[:, :, 0], v[:, 3:4, 0], atol=1e-13, rtol=0)
    assert np.allclose(lse, 1000.0, atol=1e-10, rtol=0)
    k[:, 3, :, 0] = -1000.0                                   # all others dominate equally
    o, lse = orc.attn_ref(q, k, v, False, 1.0)
    assert np.allclose(o[:, 0, 0], v[:, [0, 1, 2, 4], 0].mean(axis=1), atol=1e-13, rtol=0)
    assert np.allclose(lse, math.log(4.0), atol=1e-13, rtol=0)


# golden closed form ------------------------------------------------------
def _golden():
    vals = {}
    with open(os.path.join(GOLDEN, "closed_form_two_keys.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, *nums = line.split()
            vals[key] = np.array([float(x) for x in nums])
    return vals


def pin_golden_two_keys(orc):
    g = _golden()
    k = np.stack([g["k0"], g["k1"]]).reshape(1, 2, 1, 2)
    v = np.stack([g["v0"], g["v1"]]).reshape(1, 2, 1, 2)
    q1 = g["q"].reshape(1, 1, 1, 2)
    o, lse = orc.attn_ref(q1, k, v, False, 1.0)
    assert np.allclose(o.ravel(), g["o_noncausal"], atol=1e-14, rtol=0)
    assert np.allclose(lse.ravel(), g["lse_noncausal"], atol=1e-14, rtol=0)
    q2 = np.concatenate([q1, q1], axis=1)
    o, lse = orc.attn_ref(q2, k, v, True, 1.0)
    assert np.allclose(o[0, 0, 0], g["o_causal_row0"], atol=1e-14, rtol=0)
    assert np.allclose(o[0, 1, 0], g["o_causal_row1"], atol=1e-14, rtol=0)
    assert np.allclose(lse[0, 0], [g["lse_causal_row0"][0], g["lse_causal_row1"][0]], atol=1e-14, rtol=0)


# rows / layout -------------------------------------------------------------
def pin_rows_entry_matches_full(orc):
    """The sampled-rows entry is checked against brute force directly (not only against the full entry)."""
    B, Hq, Hkv, Sq, Skv, D = 2, 4, 2, 5, 6, 3
    q, k, v = _qkv(B, Hq, Hkv, Sq, Skv, D, 130)
    rows = np.array([(1, 3, 4), (0, 0, 0), (1, 2, 1), (0, 1, 3), (1, 0, 2)], dtype=np.int32)
    for causal in (False, True):
        bo, bl = _brute(q, k, v, causal, 0.7)
        ro, rl = orc.attn_ref_rows(q, k, v, rows, causal, 0.7)
        for n, (b, h, i) in enumerate(rows):
            assert np.allclose(ro[n], bo[b, i, h], atol=1e-13, rtol=0)
            assert abs(rl[n] - bl[b, h, i]) < 1e-13


def pin_batch_and_head_independence(orc):
    """Changing batch 1 / kv head 1 must not change batch 0 / heads of kv group 0 (indexing)."""
    B, Hq, Hkv, Sq, Skv, D = 2, 4, 2, 4, 5, 3
    q, k, v = _qkv(B, Hq, Hkv, Sq, Skv, D, 140)
    o, lse = orc.attn_ref(q, k, v, True, 0.5)
    k2, v2 = k.copy(), v.copy()
    k2[1] += 1.0; v2[1] -= 2.0; k2[:, :, 1] *= 3.0; v2[:, :, 1] += 5.0
    o2, lse2 = orc.attn_ref(q, k2, v2, True, 0.5)
    assert np.array_equal(o[0, :, :2], o2[0, :, :2]) and np.array_equal(lse[0, :2], lse2[0, :2])
    assert not np.allclose(o[0, :, 2:], o2[0, :, 2:])
    assert not np.allclose(o[1], o2[1])


def pin_probs_values_against_brute_force(orc):
    """The weights entry, for rows of several batch entries and heads: exp(scale s_j) / sum, by scalar loops."""
    B, Hq, Hkv, Sq, Skv, D = 2, 6, 3, 5, 7, 3
    q, k, _ = _qkv(B, Hq, Hkv, Sq, Skv, D, 330)
    scale = 0.6
    for causal in (False, True):
        for (b, h, i) in [(1, 4, 2), (0, 5, 0), (1, 0, 4), (1, 3, 3)]:
            g = h // (Hq // Hkv)
            n = _nvalid(i, Sq, Skv, causal)
            e = [math.exp(scale * sum(q[b, i, h, d] * k[b, j, g, d] for d in range(D))) for j in range(n)]
            want = np.zeros(Skv)
            want[:n] = np.array(e) / sum(e)
            got = orc.attn_ref_probs(q, k, b, h, i, causal, scale)
            assert np.allclose(got, want, atol=1e-14, rtol=0), (causal, b, h, i)


ALL_PINS = [
    pin_probs_sum_to_one, pin_constant_v, pin_zero_q_gives_mean, pin_causal_row0,
    pin_brute_force_tiny, pin_library_sdpa, pin_causal_is_prefix, pin_gqa_is_repeated_mha,
    pin_key_permutation, pin_split_merge, pin_score_shift, pin_dominant_key,
    pin_golden_two_keys, pin_rows_entry_matches_full, pin_batch_and_head_independence,
    pin_probs_values_against_brute_force,
]

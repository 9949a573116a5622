"""Pins for the fp64 CPU oracle (oracle/attn_oracle.c).

The paper prints no worked attention example, so the oracle is pinned by what
the mathematics fixes: closed forms, invariants, special cases that reduce to a
library routine, and brute force on tiny inputs.  Each test is chosen so that a
plausible slip (dropped scale, wrong mask side, transposed operand, log base,
missing normalisation) fails at least one of them.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2501_08071_amd import inputs as I

F16, BF16 = I.F16, I.BF16


def bits(x, dtype=F16):
    return I.to_bits(np.asarray(x, np.float32), dtype).reshape(np.shape(x))


def rnd(shape, dtype=F16, seed=0, mul=1.0):
    r = np.random.default_rng(seed)
    return bits(r.standard_normal(shape).astype(np.float32) * mul, dtype)


# ---- the oracle's own 16-bit decoders --------------------------------------------------

@pytest.mark.parametrize("b,val", [
    (0x3C00, 1.0), (0xC000, -2.0), (0x0001, 2.0 ** -24), (0x03FF, 1023 * 2.0 ** -24),
    (0x0400, 2.0 ** -14), (0x7BFF, 65504.0), (0x3555, 0.333251953125), (0x8000, 0.0),
])
def test_widen_f16_hand_patterns(b, val):
    assert oracle.widen(b, F16) == val


@pytest.mark.parametrize("b,val", [
    (0x3F80, 1.0), (0xC000, -2.0), (0x4049, 3.140625), (0x3F81, 1.0078125),
    (0x0080, 2.0 ** -126), (0x7F7F, (2 - 2.0 ** -7) * 2.0 ** 127), (0x8000, 0.0),
])
def test_widen_bf16_hand_patterns(b, val):
    assert oracle.widen(b, BF16) == val


def test_widen_all_patterns_match_numpy():
    for b in range(0, 0x7C00, 37):
        assert oracle.widen(b, F16) == float(np.array([b], np.uint16).view(np.float16)[0])


# ---- P12: brute force twin --------------------------------------------------------------

@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype", [F16, BF16])
def test_bruteforce_twin(causal, dtype):
    B, H, S, D = 2, 2, 16, 8
    q, k, v = rnd((B, H, S, D), dtype, 1), rnd((B, H, S, D), dtype, 2), rnd((B, H, S, D), dtype, 3)
    o, lse = oracle.attn_oracle(q, k, v, causal, 0.37, dtype)
    ob, lb, p = oracle.attn_bruteforce(q, k, v, causal, 0.37, dtype)
    assert np.abs(o - ob).max() < 1e-12
    assert np.abs(lse - lb).max() < 1e-12
    # P1: weights are a probability distribution over the visible keys
    assert np.abs(p.sum(-1) - 1).max() < 1e-15 and p.min() >= 0
    if causal:
        assert np.all(np.triu(p, 1) == 0)          # nothing above the diagonal
        assert np.all(np.diagonal(p, axis1=-2, axis2=-1) > 0)   # diagonal included


def test_bruteforce_written_out_in_python():
    """The definition once more, as nested Python loops on a 1x1x5x3 case."""
    S, D, scale = 5, 3, 0.5
    q, k, v = rnd((1, 1, S, D), F16, 4), rnd((1, 1, S, D), F16, 5), rnd((1, 1, S, D), F16, 6)
    Q, K, V = (I.bits_to_f64(t, F16)[0, 0] for t in (q, k, v))
    for causal in (False, True):
        o, lse = oracle.attn_oracle(q, k, v, causal, scale, F16)
        for i in range(S):
            js = range(i + 1) if causal else range(S)
            w = [math.exp(scale * sum(Q[i, d] * K[j, d] for d in range(D))) for j in js]
            z = sum(w)
            for d in range(D):
                assert abs(o[0, 0, i, d] - sum(wj * V[j, d] for wj, j in zip(w, js)) / z) < 1e-13
            assert abs(lse[0, 0, i] - math.log(z)) < 1e-13


# ---- P13: library special case ----------------------------------------------------------

@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype,D", [(F16, 64), (BF16, 128)])
def test_against_torch_fp64_softmax(causal, dtype, D):
    B, H, S = 2, 3, 200
    scale = 1 / math.sqrt(D)
    q, k, v = rnd((B, H, S, D), dtype, 7), rnd((B, H, S, D), dtype, 8), rnd((B, H, S, D), dtype, 9)
    Q, K, V = (torch.from_numpy(I.bits_to_f64(t, dtype)) for t in (q, k, v))
    s = Q @ K.transpose(-1, -2) * scale
    if causal:
        s = s.masked_fill(torch.ones(S, S, dtype=torch.bool).triu(1), float("-inf"))
    want_o = torch.softmax(s, -1) @ V
    want_l = torch.logsumexp(s, -1)
    o, lse = oracle.attn_oracle(q, k, v, causal, scale, dtype)
    assert np.abs(o - want_o.numpy()).max() < 1e-12
    assert np.abs(lse - want_l.numpy()).max() < 1e-12


# ---- closed forms -----------------------------------------------------------------------

def test_constant_v_gives_constant_output():            # P2
    q, k = rnd((1, 2, 33, 16), F16, 10, 3.0), rnd((1, 2, 33, 16), F16, 11, 3.0)
    v = bits(np.full((1, 2, 33, 16), 0.75, np.float32))
    for causal in (False, True):
        o, _ = oracle.attn_oracle(q, k, v, causal, 0.25, F16)
        assert np.abs(o - 0.75).max() < 1e-15


def test_causal_first_row_is_v0():                      # P3
    q, k, v = rnd((2, 2, 40, 16), BF16, 12), rnd((2, 2, 40, 16), BF16, 13), rnd((2, 2, 40, 16), BF16, 14)
    o, lse = oracle.attn_oracle(q, k, v, True, 0.3, BF16)
    V, Q, K = (I.bits_to_f64(t, BF16) for t in (v, q, k))
    assert np.array_equal(o[:, :, 0, :], V[:, :, 0, :])
    assert np.abs(lse[:, :, 0] - 0.3 * (Q[:, :, 0] * K[:, :, 0]).sum(-1)).max() < 1e-14


def test_one_hot_dominant_logits_copy_one_v_row():      # P4
    S, D, jstar, lam = 24, 16, 17, 4096.0
    q = rnd((1, 1, S, D), F16, 15)
    Q = I.bits_to_f64(q, F16)[0, 0]
    K = np.zeros((S, D))
    # one query (row 5) sees logit ~ scale*lam at key jstar, 0 elsewhere
    K[jstar] = lam * Q[5] / (Q[5] @ Q[5])
    k = bits(K[None, None].astype(np.float32))
    v = rnd((1, 1, S, D), F16, 16)
    scale = 0.5
    o, lse = oracle.attn_oracle(q, k, v, False, scale, F16)
    Kr = I.bits_to_f64(k, F16)[0, 0]
    logit = scale * (Q[5] @ Kr[jstar])
    assert logit > 1000                                  # would overflow exp() without max subtraction
    assert np.abs(o[0, 0, 5] - I.bits_to_f64(v, F16)[0, 0, jstar]).max() < 1e-12
    assert abs(lse[0, 0, 5] - logit) < 1e-9
    assert np.isfinite(o).all() and np.isfinite(lse).all()


def test_zero_q_gives_running_mean_and_log_count():     # P5
    S, D = 37, 8
    q = bits(np.zeros((1, 1, S, D), np.float32))
    k, v = rnd((1, 1, S, D), F16, 17), rnd((1, 1, S, D), F16, 18)
    V = I.bits_to_f64(v, F16)[0, 0]
    o, lse = oracle.attn_oracle(q, k, v, False, 0.7, F16)
    assert np.abs(o[0, 0] - V.mean(0)).max() < 1e-14
    assert np.abs(lse[0, 0] - math.log(S)).max() < 1e-14
    o, lse = oracle.attn_oracle(q, k, v, True, 0.7, F16)
    want = np.cumsum(V, 0) / np.arange(1, S + 1)[:, None]
    assert np.abs(o[0, 0] - want).max() < 1e-14
    assert np.abs(lse[0, 0] - np.log(np.arange(1, S + 1))).max() < 1e-14
    # scale = 0 with non-zero q is the same statement
    o2, lse2 = oracle.attn_oracle(rnd((1, 1, S, D), F16, 19), k, v, True, 0.0, F16)
    assert np.abs(o2[0, 0] - want).max() < 1e-14


def test_single_key():                                  # P6
    q, k, v = rnd((3, 2, 1, 8), BF16, 20), rnd((3, 2, 1, 8), BF16, 21), rnd((3, 2, 1, 8), BF16, 22)
    o, lse = oracle.attn_oracle(q, k, v, False, 1.5, BF16)
    assert np.array_equal(o, I.bits_to_f64(v, BF16))
    want = 1.5 * (I.bits_to_f64(q, BF16) * I.bits_to_f64(k, BF16)).sum(-1)
    assert np.abs(lse - want).max() < 1e-14


def test_two_keys_is_a_logistic():
    """S=2 non-causal: weight on key 1 is sigmoid(s1-s0); lse = s0 + log1p(exp(s1-s0))."""
    q, k, v = rnd((1, 1, 2, 4), F16, 23), rnd((1, 1, 2, 4), F16, 24), rnd((1, 1, 2, 4), F16, 25)
    Q, K, V = (I.bits_to_f64(t, F16)[0, 0] for t in (q, k, v))
    o, lse = oracle.attn_oracle(q, k, v, False, 0.9, F16)
    for i in range(2):
        s0, s1 = 0.9 * Q[i] @ K[0], 0.9 * Q[i] @ K[1]
        w1 = 1 / (1 + math.exp(s0 - s1))
        assert np.abs(o[0, 0, i] - ((1 - w1) * V[0] + w1 * V[1])).max() < 1e-15
        assert abs(lse[0, 0, i] - (s0 + math.log1p(math.exp(s1 - s0)))) < 1e-14


# ---- invariants -------------------------------------------------------------------------

def test_causal_row_equals_noncausal_prefix():          # P7
    S, D = 50, 16
    q, k, v = rnd((1, 2, S, D), F16, 26), rnd((1, 2, S, D), F16, 27), rnd((1, 2, S, D), F16, 28)
    oc, lc = oracle.attn_oracle(q, k, v, True, 0.25, F16)
    for i in (0, 1, 17, 31, 32, 49):
        op, lp = oracle.attn_oracle(q[:, :, : i + 1], k[:, :, : i + 1], v[:, :, : i + 1], False, 0.25, F16)
        assert np.abs(oc[:, :, i] - op[:, :, i]).max() < 1e-14
        assert np.abs(lc[:, :, i] - lp[:, :, i]).max() < 1e-14


def test_split_merge_by_logsumexp():                    # P8
    S, D, cut = 64, 16, 23
    q, k, v = rnd((1, 2, S, D), BF16, 29), rnd((1, 2, S, D), BF16, 30), rnd((1, 2, S, D), BF16, 31)
    o, lse = oracle.attn_oracle(q, k, v, False, 0.25, BF16)

    def part(lo, hi):
        """All S queries against keys [lo,hi): the oracle wants equal q and k lengths, so the
        queries go through in blocks of hi-lo rows (the last block zero-padded, padding dropped)."""
        n = hi - lo
        kk, vv = np.ascontiguousarray(k[:, :, lo:hi]), np.ascontiguousarray(v[:, :, lo:hi])
        outs, lses = [], []
        for start in range(0, S, n):
            blk = q[:, :, start:start + n]
            have = blk.shape[2]
            if have < n:
                blk = np.concatenate([blk, np.zeros((1, 2, n - have, D), np.uint16)], 2)
            oo, ll = oracle.attn_oracle(np.ascontiguousarray(blk), kk, vv, False, 0.25, BF16)
            outs.append(oo[:, :, :have]); lses.append(ll[:, :, :have])
        return np.concatenate(outs, 2), np.concatenate(lses, 2)

    o1, l1 = part(0, cut)
    o2, l2 = part(cut, S)
    w1, w2 = np.exp(l1), np.exp(l2)
    assert np.abs(np.log(w1 + w2) - lse).max() < 1e-13
    merged = (w1[..., None] * o1 + w2[..., None] * o2) / (w1 + w2)[..., None]
    assert np.abs(merged - o).max() < 1e-13


def test_permutation_equivariance():                    # P9
    S, D = 48, 16
    q, k, v = rnd((1, 1, S, D), F16, 32), rnd((1, 1, S, D), F16, 33), rnd((1, 1, S, D), F16, 34)
    o, lse = oracle.attn_oracle(q, k, v, False, 0.25, F16)
    perm = np.random.default_rng(35).permutation(S)
    o2, l2 = oracle.attn_oracle(q, np.ascontiguousarray(k[:, :, perm]), np.ascontiguousarray(v[:, :, perm]),
                                False, 0.25, F16)
    assert np.abs(o - o2).max() < 1e-14 and np.abs(lse - l2).max() < 1e-14
    o3, l3 = oracle.attn_oracle(np.ascontiguousarray(q[:, :, perm]), k, v, False, 0.25, F16)
    assert np.array_equal(o3, o[:, :, perm]) and np.array_equal(l3, lse[:, :, perm])


def test_key_shift_moves_lse_only():                    # P10
    S, D = 32, 8
    # values on a coarse grid so that k + t is exactly representable in binary16
    r = np.random.default_rng(36)
    mk = lambda: (r.integers(-16, 17, (1, 1, S, D)) / 8.0).astype(np.float32)
    Qf, Kf, Vf = mk(), mk(), mk()
    t = (r.integers(-8, 9, D) / 8.0).astype(np.float32)
    o, lse = oracle.attn_oracle(bits(Qf), bits(Kf), bits(Vf), True, 0.5, F16)
    o2, l2 = oracle.attn_oracle(bits(Qf), bits(Kf + t), bits(Vf), True, 0.5, F16)
    assert np.abs(o - o2).max() < 1e-13
    assert np.abs((l2 - lse) - 0.5 * (Qf.astype(np.float64) @ t.astype(np.float64))).max() < 1e-13


def test_output_in_convex_hull_of_v():                  # P11
    S, D = 70, 8
    q, k, v = rnd((2, 2, S, D), F16, 37, 3.0), rnd((2, 2, S, D), F16, 38, 3.0), rnd((2, 2, S, D), F16, 39)
    V = I.bits_to_f64(v, F16)
    o, _ = oracle.attn_oracle(q, k, v, False, 0.35, F16)
    assert np.all(o <= V.max(2, keepdims=True) + 1e-15) and np.all(o >= V.min(2, keepdims=True) - 1e-15)
    o, _ = oracle.attn_oracle(q, k, v, True, 0.35, F16)
    assert np.all(o <= np.maximum.accumulate(V, 2) + 1e-15)
    assert np.all(o >= np.minimum.accumulate(V, 2) - 1e-15)


def test_heads_and_batches_are_independent():
    q, k, v = rnd((2, 3, 20, 8), F16, 40), rnd((2, 3, 20, 8), F16, 41), rnd((2, 3, 20, 8), F16, 42)
    o, lse = oracle.attn_oracle(q, k, v, True, 0.3, F16)
    for b in range(2):
        for h in range(3):
            sl = (slice(b, b + 1), slice(h, h + 1))
            o1, l1 = oracle.attn_oracle(*(np.ascontiguousarray(t[sl]) for t in (q, k, v)), True, 0.3, F16)
            assert np.array_equal(o1[0, 0], o[b, h]) and np.array_equal(l1[0, 0], lse[b, h])


def test_row_subset_equals_full():
    q, k, v = rnd((2, 2, 90, 16), BF16, 43), rnd((2, 2, 90, 16), BF16, 44), rnd((2, 2, 90, 16), BF16, 45)
    rows = np.array([0, 1, 31, 32, 33, 63, 64, 89], np.int32)
    for causal in (False, True):
        o, lse = oracle.attn_oracle(q, k, v, causal, 0.2, BF16)
        os_, ls_ = oracle.attn_oracle(q, k, v, causal, 0.2, BF16, rows=rows)
        assert np.array_equal(os_, o[:, :, rows]) and np.array_equal(ls_, lse[:, :, rows])


def test_scale_is_applied_to_logits_not_outputs():
    """Doubling scale equals doubling q (exactly, power of two) and differs from scale alone."""
    q, k, v = rnd((1, 1, 30, 8), F16, 46), rnd((1, 1, 30, 8), F16, 47), rnd((1, 1, 30, 8), F16, 48)
    q2 = bits(I.bits_to_f64(q, F16).astype(np.float32) * 2)
    o1, l1 = oracle.attn_oracle(q, k, v, False, 0.5, F16)
    o2, l2 = oracle.attn_oracle(q2, k, v, False, 0.25, F16)
    assert np.abs(o1 - o2).max() < 1e-14 and np.abs(l1 - l2).max() < 1e-14
    o3, _ = oracle.attn_oracle(q, k, v, False, 0.25, F16)
    assert np.abs(o1 - o3).max() > 1e-3


# ---- P14: structure of the peaky workload ----------------------------------------------

def test_peaky_workload_is_near_one_hot():
    w = I.workload(5)
    q, k, v = I.gen_tensors(1, 1, 256, w.D, w.dtype, workload_id=w.id, qk_mul=w.qk_mul, v_dist=w.v_dist)
    # logits have std about 16 (entries 4*N(0,1), D=64, scale=1/8): measure, then look at the weights
    Q, K = I.bits_to_f64(q, w.dtype)[0, 0], I.bits_to_f64(k, w.dtype)[0, 0]
    s = Q @ K.T * w.scale
    assert 14.0 < s.std() < 18.0
    o, lse = oracle.attn_oracle(q, k, v, False, w.scale, w.dtype)
    pmax = np.exp(s.max(1) - lse[0, 0])
    assert (pmax > 0.5).mean() > 0.6                     # most rows dominated by a single key
    assert np.abs(o).max() < 1.0 and np.isfinite(lse).all()
    assert s.max() > 40                                  # far beyond what fp16 exp could hold unshifted


def test_bad_arguments_are_rejected():
    q = rnd((1, 1, 4, 4), F16, 50)
    with pytest.raises(ValueError):
        oracle.attn_oracle(q, q, q, False, 1.0, F16, rows=np.array([4], np.int32))
    with pytest.raises(TypeError):
        oracle.attn_oracle(q.astype(np.float32), q, q, False, 1.0, F16)
    with pytest.raises(ValueError):
        oracle.attn_oracle(q, q, q, False, 1.0, 2)


# ---- hand-worked fixture ---------------------------------------------------------------

def _read_pow2_fixture():
    import os
    rows = {"q": [], "k": [], "v": []}
    want = {"noncausal": {}, "causal": {}}
    with open(os.path.join(os.path.dirname(__file__), "golden", "pow2_weights_S4_D2.txt")) as f:
        for line in f:
            t = line.split("#")[0].split()
            if not t:
                continue
            if t[0] in rows:
                rows[t[0]].append([float(x) for x in t[1:]])
            else:
                want[t[0]][int(t[1])] = ([int(t[2]), int(t[3])], int(t[4]))
    return rows, want


@pytest.mark.parametrize("dtype", [F16, BF16])
@pytest.mark.parametrize("causal", [False, True])
def test_hand_worked_rational_weights(causal, dtype):
    """Integer logits times ln 2 give power-of-two weights; expected values were worked out by hand."""
    rows, want = _read_pow2_fixture()
    q, k, v = (bits(np.array(rows[n], np.float32)[None, None], dtype) for n in "qkv")
    scale = math.log(2.0)
    o, lse = oracle.attn_oracle(q, k, v, causal, scale, dtype)
    for i, (num, den) in want["causal" if causal else "noncausal"].items():
        assert np.abs(o[0, 0, i] - np.array(num) / den).max() < 1e-12
        assert abs(lse[0, 0, i] - math.log(den)) < 1e-12

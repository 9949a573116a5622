"""GPU parity, the whole matrix of kernel instances: every (element type, head dimension, mask) instance in both launch
modes at a ragged length that wraps the LDS buffer ring several times, every element against the oracle; and a seeded
run of random shapes, scales and value ranges (Section 4.1 of the paper: outputs of randomised inputs against reference
outputs)."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2501_08071_amd as P
from paper_2501_08071_amd import inputs as I
from parity import MAX_ABS, MEAN_ABS, LSE_REL, check_full, errors, to_device

pytestmark = pytest.mark.gpu
F16, BF16 = I.F16, I.BF16


@pytest.mark.parametrize("wide", [False, True], ids=["four_wavefronts", "eight_wavefronts"])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("D", [32, 64, 128])
@pytest.mark.parametrize("dtype", [F16, BF16])
def test_every_instance_in_both_launch_modes(dtype, D, causal, wide):
    """S = 1100: five query tiles of 256 rows (nine of 128), the last one ragged; 1100 keys are more than four
    rounds of the 256-key buffer ring.  26 heads give 130 large tiles, which takes the eight-wavefront instance;
    two heads take the four-wavefront one."""
    B, H, S = (2, 13, 1100) if wide else (1, 2, 1100)
    assert P.attn_launch_rows(B, H, S, D, dtype, causal) == (256 if wide else 128)
    name = P.attn_kernel_name(B, H, S, D, dtype, causal)
    assert name.endswith(", 8>" if wide else ", 4>") or "rows64" in name
    q, k, v = I.gen_tensors(B, H, S, D, dtype, workload_id=4000 + D)
    mx, mean, lrel = check_full(q, k, v, dtype, causal, 1 / math.sqrt(D), f"{name} B{B} H{H} S{S}")
    print(f"{name} B{B} H{H} S{S}: max-abs {mx:.2e} mean-abs {mean:.2e} lse-rel {lrel:.2e}")


def test_random_shapes_scales_and_ranges():
    """150 seeded cases: D, element type, mask, S in three ranges (one key block, a few, many), few or many heads (both
    launch modes), q/k scaled by 0.1 .. 8 (binary16: at most 3, its logits must stay finite), scales of either sign, one
    call in four through attn_fwd_o16 (whose bar carries the rounding of O to the element type the header states).
    Stops at the first failure and names the case."""
    rng = np.random.default_rng(20250108)
    worst = [0.0, 0.0, 0.0]
    for it in range(150):
        D = int(rng.choice([32, 64, 128]))
        dtype = int(rng.choice([F16, BF16]))
        causal = bool(rng.integers(2))
        S = int(rng.choice([rng.integers(1, 40), rng.integers(40, 300), rng.integers(300, 1400)]))
        B, H = (int(rng.integers(1, 3)), int(rng.integers(1, 4))) if rng.integers(3) else (int(rng.integers(2, 5)), int(rng.integers(33, 70)))
        if B * H > 20:
            S = min(S, 400)
        mul = float(rng.choice([0.1, 1.0, 1.0, 3.0, 8.0]))
        scale = float(rng.choice([1 / math.sqrt(D), 1.0, -0.2, 0.01, 2.5]))
        if dtype == F16:
            mul = min(mul, 3.0)
        o16 = rng.integers(4) == 0
        case = f"case {it}: B{B} H{H} S{S} D{D} dtype{dtype} causal={causal} qk x{mul} scale={scale:.4f} {'attn_fwd_o16' if o16 else 'attn_fwd'}"
        q, k, v = I.gen_tensors(B, H, S, D, dtype, workload_id=1000 + it, qk_mul=mul)
        dq, dk, dv = (to_device(t, dtype) for t in (q, k, v))
        o, lse = (P.attn_fwd_o16 if o16 else P.attn_fwd)(dq, dk, dv, causal, scale)
        torch.cuda.synchronize()
        o_ref, l_ref = oracle.attn_oracle(q, k, v, causal, scale, dtype)
        og, lg = o.float().cpu().numpy(), lse.cpu().numpy()
        assert np.isfinite(og).all() and np.isfinite(lg).all(), case
        mx, mean, lrel = errors(og, lg, o_ref, l_ref)
        # attn_fwd_o16 rounds O once more: half an ulp of the element type at the largest |O|
        allow = (2.0 ** -9 if dtype == BF16 else 2.0 ** -12) * float(np.abs(o_ref).max()) if o16 else 0.0
        assert mx <= MAX_ABS + allow and mean <= MEAN_ABS + allow and lrel <= LSE_REL, f"{case}: max {mx:.2e} mean {mean:.2e} lse {lrel:.2e}"
        worst = [max(a, b) for a, b in zip(worst, (mx, mean, lrel))]
    print(f"150 random cases: worst max-abs {worst[0]:.2e} mean-abs {worst[1]:.2e} lse-rel {worst[2]:.2e}")


@pytest.mark.parametrize("bad", [float("inf"), float("nan")])
def test_non_finite_v_row_above_the_diagonal(bad):
    """The header asks for finite q, k and v everywhere: masked keys enter the second product with weight 0, and 0 * Inf
    is not a number.  This pins what that means.  A non-finite row j of v: the rows of O that see key j are non-finite
    in the oracle too; of the rows that do not, those in earlier key blocks come out exactly as without the
    bad row (`attn_tile_keys` keys per block); the rows of j's own block before j are the ones the requirement is there
    for (they are not checked)."""
    B, H, S, D, dtype, j = 1, 2, 200, 64, F16, 150
    q, k, v = I.gen_tensors(B, H, S, D, dtype, workload_id=77)
    dq, dk, dv = (to_device(t, dtype) for t in (q, k, v))
    o_clean, lse_clean = P.attn_fwd(dq, dk, dv, True, 0.125)
    dv_bad = dv.clone()
    dv_bad[:, :, j, :] = bad
    o, lse = P.attn_fwd(dq, dk, dv_bad, True, 0.125)
    torch.cuda.synchronize()
    keys = P.attn_tile_keys(D, dtype, True)
    first_of_block = (j // keys) * keys
    assert torch.equal(o[:, :, :first_of_block], o_clean[:, :, :first_of_block])       # earlier blocks: untouched, bit for bit
    assert torch.equal(lse, lse_clean)                                                   # v takes no part in the logsumexp
    v_bad = v.copy()
    v_bad[:, :, j, :] = 0x7C00 if math.isinf(bad) else 0x7E00                            # binary16 +Inf / a quiet NaN
    o_ref, _ = oracle.attn_oracle(q, k, v_bad, True, 0.125, dtype)
    assert not np.isfinite(o_ref[:, :, j:]).any()                                        # the definition: every row from j on
    assert not torch.isfinite(o[:, :, j:]).any()                                         # the kernel agrees
    assert np.isfinite(o_ref[:, :, :j]).all()                                            # and the rows before j are finite there

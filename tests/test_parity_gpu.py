"""GPU parity: the HIP attention forward, called through the C ABI, against the fp64 oracle."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2501_08071_amd as P
from paper_2501_08071_amd import inputs as I
from parity import (MAX_ABS, assert_parity, check_full, edge_rows, errors, run_gpu, to_device)

pytestmark = pytest.mark.gpu
F16, BF16 = I.F16, I.BF16


# ---- small shapes, every output element compared ---------------------------------------

SMALL = [
    # B, H, S, D  -- S chosen to hit: one key, sub-tile, tile edges +-1, several query tiles, ragged tails
    (2, 2, 1, 64), (1, 2, 2, 128), (1, 3, 31, 64), (1, 2, 33, 128), (2, 1, 64, 64), (1, 2, 65, 128),
    (1, 2, 127, 64), (1, 1, 128, 128), (1, 2, 129, 64), (2, 2, 200, 128), (1, 3, 257, 64), (1, 2, 300, 128),
    (2, 2, 517, 64), (1, 2, 640, 128),
    (2, 2, 1, 32), (1, 2, 33, 32), (1, 3, 127, 32), (2, 1, 256, 32), (1, 2, 300, 32), (1, 2, 777, 32),
]


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype", [F16, BF16])
@pytest.mark.parametrize("B,H,S,D", SMALL)
def test_small_shapes_full_compare(B, H, S, D, dtype, causal):
    q, k, v = I.gen_tensors(B, H, S, D, dtype, workload_id=100 + S)
    check_full(q, k, v, dtype, causal, 1 / math.sqrt(D), f"B{B} H{H} S{S} D{D} dt{dtype} causal{causal}")


# The same edge lengths with so many (b,h) pairs that the library takes its full-size workgroups (256 query rows,
# eight wavefronts): with few tiles it launches the same kernel with four wavefronts per workgroup.
WIDE = [(3, 43, 1, 64), (3, 43, 33, 128), (3, 43, 65, 32), (3, 43, 129, 64), (3, 43, 200, 128), (3, 43, 257, 64),
        (3, 43, 300, 128), (3, 43, 257, 32)]


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype", [F16, BF16])
@pytest.mark.parametrize("B,H,S,D", WIDE)
def test_small_shapes_full_size_workgroups(B, H, S, D, dtype, causal):
    assert P.attn_launch_rows(B, H, S, D, dtype, causal) == P.attn_tile_rows(D, dtype, causal) == 256
    q, k, v = I.gen_tensors(B, H, S, D, dtype, workload_id=500 + S)
    check_full(q, k, v, dtype, causal, 1 / math.sqrt(D), f"B{B} H{H} S{S} D{D} dt{dtype} causal{causal}")


def test_small_problems_take_half_size_workgroups():
    for (B, H, S, D) in SMALL:
        assert P.attn_launch_rows(B, H, S, D, F16, False) == 128
    assert P.attn_launch_rows(1, 4, 4096, 32, F16, True) == 128          # the paper's own shape: 64 large tiles
    assert P.attn_launch_rows(2, 32, 4096, 128, BF16, True) == 256 and P.attn_launch_rows(4, 16, 1024, 64, F16, False) == 256


def test_workload_1_full():
    w = I.workload(1)
    q, k, v = I.gen_inputs(w)
    mx, mean, lrel = check_full(q, k, v, w.dtype, w.causal, w.scale, w.name)
    print(f"{w.name}: max-abs {mx:.2e} mean-abs {mean:.2e} lse-rel {lrel:.2e}")


@pytest.mark.parametrize("scale", [0.0, -0.125, 1.0, 1e-4])
@pytest.mark.parametrize("causal", [False, True])
def test_scale_values(scale, causal):
    q, k, v = I.gen_tensors(1, 2, 200, 64, F16, workload_id=201)
    check_full(q, k, v, F16, causal, scale, f"scale {scale}")


def test_peaky_logits_small():
    w = I.workload(5)
    q, k, v = I.gen_tensors(2, 2, 384, w.D, w.dtype, workload_id=w.id, qk_mul=w.qk_mul, v_dist=w.v_dist)
    check_full(q, k, v, w.dtype, False, w.scale, "peaky small")
    check_full(q, k, v, w.dtype, True, w.scale, "peaky small causal")


def test_huge_logits_do_not_overflow():
    """|s| up to ~1e4: exp would overflow without the running maximum."""
    q, k, v = I.gen_tensors(1, 2, 256, 64, BF16, workload_id=202, qk_mul=32.0)
    check_full(q, k, v, BF16, False, 1.0, "huge logits")


def _trend_inputs(S, D, dtype, kind, seed):
    """Keys whose logits follow a trend along the sequence: the running maximum of a row keeps moving
    (rising), never moves after the first block (falling), or jumps once, late, in some rows (spike)."""
    rng = np.random.default_rng(seed)
    qf = rng.standard_normal((1, 2, S, D)).astype(np.float32)
    kf = rng.standard_normal((1, 2, S, D)).astype(np.float32) * 0.25
    vf = rng.standard_normal((1, 2, S, D)).astype(np.float32)
    u = np.ones(D, np.float32) / math.sqrt(D)
    qf += 4.0 * u                                   # every query has a component along u ...
    pos = np.arange(S, dtype=np.float32)[None, None, :, None]
    if kind == "rising":
        kf += (pos / 8.0) * u                       # ... so q.k grows by about 0.5 per key
    elif kind == "falling":
        kf -= (pos / 8.0) * u
    else:
        kf[..., S - 37, :] += 60.0 * u              # one key far above all the others, near the end
    return tuple(I.to_bits(t, dtype) for t in (qf, kf, vf))


@pytest.mark.parametrize("kind", ["rising", "falling", "spike"])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype,D", [(F16, 64), (BF16, 128), (F16, 128), (BF16, 64), (F16, 32), (BF16, 32)])
def test_moving_reference_maximum(dtype, D, causal, kind):
    """The kernel takes row maxima only when a block's weight sum overflows a threshold: drive that path
    many times (rising), never (falling), and once with a jump of many orders of magnitude (spike)."""
    q, k, v = _trend_inputs(421, D, dtype, kind, seed=7)
    check_full(q, k, v, dtype, causal, 1.0, f"{kind} logits D={D}")


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype,D,S", [(F16, 64, 333), (BF16, 128, 300), (F16, 128, 257), (BF16, 64, 129)])
def test_output_in_input_dtype(dtype, D, S, causal):
    """attn_fwd_o16: O rounded to the input type is the fp32 O of attn_fwd, rounded (bit for bit), and
    meets the same bar against the oracle; lse is the same."""
    q, k, v = I.gen_tensors(2, 2, S, D, dtype, workload_id=400 + D)
    dq, dk, dv = (to_device(t, dtype) for t in (q, k, v))
    scale = 1.0 / math.sqrt(D)
    o32, lse32 = P.attn_fwd(dq, dk, dv, causal, scale)
    o16, lse16 = P.attn_fwd_o16(dq, dk, dv, causal, scale)
    torch.cuda.synchronize()
    assert o16.dtype == dq.dtype
    assert torch.equal(o16, o32.to(dq.dtype))          # torch rounds to nearest even, as the kernel does
    assert torch.equal(lse16, lse32)
    o_ref, lse_ref = oracle.attn_oracle(q, k, v, causal, scale, dtype)
    assert_parity(o16.float().cpu().numpy(), lse16.cpu().numpy(), o_ref, lse_ref, f"o16 D={D} S={S}")


def test_closed_forms_on_gpu():
    S, D = 300, 64
    q, k, v = I.gen_tensors(1, 2, S, D, F16, workload_id=203)
    V = I.bits_to_f64(v, F16)
    # zero queries: running mean of V, lse = ln(i+1)
    o, lse = run_gpu(np.zeros_like(q), k, v, F16, True, 0.125)
    want = np.cumsum(V, 2) / np.arange(1, S + 1)[None, None, :, None]
    assert np.abs(o - want).max() < 2e-3
    assert np.abs(lse - np.log(np.arange(1, S + 1))).max() < 1e-4
    # constant V comes back unchanged
    cv = I.to_bits(np.full((1, 2, S, D), 0.75, np.float32), F16)
    o, _ = run_gpu(q, k, cv, F16, False, 0.125)
    assert np.abs(o - 0.75).max() < 1e-3
    # causal first row equals V[0]
    o, lse = run_gpu(q, k, v, F16, True, 0.125)
    assert np.abs(o[:, :, 0] - V[:, :, 0]).max() < 1e-6


def test_lse_optional_and_outputs_reused():
    q, k, v = I.gen_tensors(1, 2, 130, 64, F16, workload_id=204)
    o1, lse1 = run_gpu(q, k, v, F16, True, 0.125)
    o2, none = run_gpu(q, k, v, F16, True, 0.125, want_lse=False)
    assert none is None and np.array_equal(o1, o2)


def test_run_to_run_bitwise_determinism():
    w = I.workload(2)
    q, k, v = I.gen_tensors(2, 4, 1024, w.D, w.dtype, workload_id=w.id)
    dq, dk, dv = (to_device(t, w.dtype) for t in (q, k, v))
    o0, l0 = P.attn_fwd(dq, dk, dv, True, w.scale)
    for _ in range(5):
        o1, l1 = P.attn_fwd(dq, dk, dv, True, w.scale)
        assert torch.equal(o0, o1) and torch.equal(l0, l1)


def test_non_default_stream_and_guard_bytes():
    """Runs on a side stream and writes nothing outside o / lse."""
    B, H, S, D = 1, 2, 100, 64
    q, k, v = I.gen_tensors(B, H, S, D, BF16, workload_id=205)
    dq, dk, dv = (to_device(t, BF16) for t in (q, k, v))
    pad = 1024
    obuf = torch.full((B * H * S * D + 2 * pad,), 7.0, device="cuda")
    lbuf = torch.full((B * H * S + 2 * pad,), 7.0, device="cuda")
    o = obuf[pad:-pad].view(B, H, S, D)
    lse = lbuf[pad:-pad].view(B, H, S)
    st = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(st):
        P.attn_fwd(dq, dk, dv, True, 0.125, o=o, lse=lse, stream=st)
    st.synchronize()
    assert (obuf[:pad] == 7).all() and (obuf[-pad:] == 7).all()
    assert (lbuf[:pad] == 7).all() and (lbuf[-pad:] == 7).all()
    o_ref, l_ref = oracle.attn_oracle(q, k, v, True, 0.125, BF16)
    assert_parity(o.cpu().numpy(), lse.cpu().numpy(), o_ref, l_ref, "side stream")


@pytest.mark.parametrize("causal", [False, True])
def test_paper_attention_shape(causal):
    """The shape the paper evaluates its flash-attention kernel on (Table 2: B=1, n_head=4, seq_len=4096,
    d_head=32, fp16), every output element compared."""
    q, k, v = I.gen_tensors(1, 4, 4096, 32, F16, workload_id=600)
    check_full(q, k, v, F16, causal, 1.0 / math.sqrt(32), f"paper shape causal={causal}")


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("S", [300, 512, 1000])
def test_more_tiles_than_compute_units(S, causal):
    """More workgroups than the chip runs at once (320 to 640 tiles of 256 query rows), whole (S = 512) and
    ragged (S = 300, 1000) key streams, every output element compared."""
    B, H = 4, 40
    q, k, v = I.gen_tensors(B, H, S, 128, BF16, workload_id=700 + S)
    check_full(q, k, v, BF16, causal, 1.0 / math.sqrt(128), f"many tiles S={S} causal={causal}")


def test_graph_capture_and_replay():
    """The call is one asynchronous kernel launch with no allocation and no synchronisation, so it can be
    captured into a HIP graph; every replay, with new inputs written in place and eager work in between,
    gives the eager result bit for bit."""
    B, H, S = 1, 2, 300
    cases = []
    for D, dtype, causal in ((128, BF16, True), (64, F16, False)):
        q, k, v = I.gen_tensors(B, H, S, D, dtype, workload_id=500 + D)
        dq, dk, dv = (to_device(t, dtype) for t in (q, k, v))
        o = torch.empty((B, H, S, D), dtype=torch.float32, device="cuda")
        lse = torch.empty((B, H, S), dtype=torch.float32, device="cuda")
        P.attn_fwd(dq, dk, dv, causal, 0.1, o=o, lse=lse)          # first call outside the capture
        cases.append((dq, dk, dv, causal, o, lse))
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for dq, dk, dv, causal, o, lse in cases:
            P.attn_fwd(dq, dk, dv, causal, 0.1, o=o, lse=lse)
    for rep in range(3):
        for dq, dk, dv, causal, o, lse in cases:
            dq.copy_(torch.roll(dq, rep + 1, dims=2)); dv.mul_(-1.0)      # new inputs, in place
            o.fill_(float("nan")); lse.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        for dq, dk, dv, causal, o, lse in cases:
            o_e, lse_e = P.attn_fwd(dq, dk, dv, causal, 0.1)
            torch.cuda.synchronize()
            assert torch.equal(o, o_e) and torch.equal(lse, lse_e), f"replay {rep}"
    dq, dk, dv, causal, o, lse = cases[0]
    bits = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)
    o_ref, l_ref = oracle.attn_oracle(bits(dq), bits(dk), bits(dv), causal, 0.1, BF16)
    assert_parity(o.cpu().numpy(), lse.cpu().numpy(), o_ref, l_ref, "graph replay")


# ---- the five workloads at full size, in the launch configuration the bench times -------

@pytest.mark.parametrize("wid", [2, 3, 4, 5])
def test_workloads_full_size_row_subset(wid):
    """Every (b,h); rows at every tile edge +-1 plus a seeded random sample (rows are independent,
    so the oracle on a row subset is exact for those rows)."""
    w = I.workload(wid)
    q, k, v = I.gen_inputs(w)
    o, lse = run_gpu(q, k, v, w.dtype, w.causal, w.scale)
    assert np.isfinite(o).all() and np.isfinite(lse).all()
    br, bc = P.attn_tile_rows(w.D, w.dtype, w.causal), P.attn_tile_keys(w.D, w.dtype, w.causal)
    # tile-edge rows for all tiles would be most of a 16k sequence: keep edges of the first and last 4 tiles
    rows = edge_rows(w.S, br, bc, extra=w.S // 32, seed=wid)
    if len(rows) > w.S // 8:
        keep = (rows < 4 * br + 2) | (rows > w.S - 4 * br - 2)
        rng = np.random.default_rng(wid)
        rows = np.unique(np.concatenate([rows[keep], rng.choice(rows[~keep], w.S // 16, replace=False)]))
    o_ref, lse_ref = oracle.attn_oracle(q, k, v, w.causal, w.scale, w.dtype, rows=rows)
    mx, mean, lrel = assert_parity(o[:, :, rows], lse[:, :, rows], o_ref, lse_ref, w.name)
    print(f"{w.name}: {len(rows)} rows/head: max-abs {mx:.2e} mean-abs {mean:.2e} lse-rel {lrel:.2e}")
    # properties that hold at any size, over the whole output
    V = I.bits_to_f64(v, w.dtype)
    if not w.causal:
        assert (o <= V.max(2, keepdims=True) + 1e-3).all() and (o >= V.min(2, keepdims=True) - 1e-3).all()
    else:
        assert np.abs(o[:, :, 0] - V[:, :, 0]).max() < 1e-6


@pytest.mark.parametrize("wid", [2, 3, 5, 4])
def test_workloads_every_element(wid):
    """The whole output of every benchmark workload against the oracle (a few seconds of the host's cores for
    workloads 2, 3 and 5, about half a minute for workload 4)."""
    w = I.workload(wid)
    q, k, v = I.gen_inputs(w)
    mx, mean, lrel = check_full(q, k, v, w.dtype, w.causal, w.scale, w.name)
    print(f"{w.name} full: max-abs {mx:.2e} mean-abs {mean:.2e} lse-rel {lrel:.2e}")


def test_issue_share_probe_runs():
    """Every wavefront reports its loop: the vector wavefronts make exactly `iters` iterations, the matrix wavefronts
    stop when their partner is done (or after `iters` when it is idle); all cycle counts positive; the derived figures
    are in the range the instruction timings allow (a 32x32x16 matrix instruction occupies its pipe for 32 cycles)."""
    out = torch.zeros(4 * 16, dtype=torch.int64, device="cuda")
    assert P.lib.probe_issue_share(out.data_ptr(), 4, 50, 1, 1, None) == 0
    torch.cuda.synchronize()
    r = out.cpu().reshape(4, 8, 2)
    assert torch.all(r[:, 4:, 1] == 50) and torch.all(r[:, :4, 1] >= 1) and torch.all(r[:, :4, 1] <= 400) and torch.all(r[..., 0] > 0)
    assert P.lib.probe_issue_share(out.data_ptr(), 4, 50, 1, 0, None) == 0
    torch.cuda.synchronize()
    r = out.cpu().reshape(4, 8, 2)
    assert torch.all(r[:, :4, 1] == 50) and torch.all(r[:, 4:, 1] == 0)
    res = P.probe_issue_share(iters=100, workgroups=64)
    assert 30.0 <= res["mfma_cycles_alone"] <= 40.0
    assert 0.0 <= res["mfma_issue_cycles"] <= 32.0
    for t in ("bf16", "f16"):
        assert 10.0 <= res[f"valu_cycles_per_64_scores_{t}"] <= 40.0
        assert res[f"valu_cycles_per_64_scores_{t}_next_to_mfma"] >= res[f"valu_cycles_per_64_scores_{t}"] - 1.0
        assert 30.0 <= res[f"mfma_cycles_next_to_{t}"] <= 64.0


def test_matrix_instruction_probe_runs():
    """The measuring aid: returns the flop count of its launch and a finite, positive rate; constant operands
    accumulate exactly (every lane sums iters * 16 instructions * 16 products of 1.0 * 1.0 per accumulator element)."""
    out = torch.zeros(8 * 256, dtype=torch.float32, device="cuda")
    flops = P.lib.probe_mfma(out.data_ptr(), 8, 3, BF16, 0, None)
    torch.cuda.synchronize()
    assert flops == 8 * 4 * 3 * 16 * 32768
    assert torch.all(out == 3 * 16 * 16 * 16.0)            # 64 accumulator values per lane, 3 * 4 instructions * 16 products each
    for dt in (F16, BF16):
        r = P.probe_mfma(iters=200, dtype=dt, random_operands=True, workgroups=512, repeats=2)
        assert math.isfinite(r) and r > 0

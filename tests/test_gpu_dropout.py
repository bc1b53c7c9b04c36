"""GPU parity of segment attention with dropout on the weights (Section 2.2) against the fp64
oracle, through the C ABI.  The keep decisions are integer work and must agree exactly; the
floating-point results are held to the same tolerances as the plain path."""
import numpy as np
import pytest
import torch

import oracle
from paper_2311_02382_amd import lss, synth
from _util import TOL, Staged, lse_err, rel_err, stage_all, to_np

pytestmark = pytest.mark.gpu


def run_segment(Q, K, V, DO, s0, l_s, causal, kind, p, seed, tag=""):
    tol = TOL[kind]
    sl = slice(s0, s0 + l_s)
    q_dev, do_dev = Q.dev[:, sl].contiguous(), DO.dev[:, sl].contiguous()
    out, lse = lss.lss_segment_attn_fwd(q_dev, K.dev, V.dev, s0, causal, p_drop=p, seed=seed)
    ref_o, ref_l = oracle.segment_fwd_dropout(Q.f64[:, sl], K.f64, V.f64, s0, causal, p, seed)
    assert rel_err(to_np(out), ref_o) <= tol["t"], f"{tag} out"
    assert lse_err(to_np(lse), ref_l) <= tol["lse"], f"{tag} lse"
    dq, dk, dv = lss.lss_segment_attn_bwd(q_dev, K.dev, V.dev, s0, out, lse, do_dev, causal, p_drop=p, seed=seed)
    rdq, rdk, rdv = oracle.segment_bwd_dropout(Q.f64[:, sl], K.f64, V.f64, DO.f64[:, sl], s0, causal, p, seed)
    for name, got, ref in (("dq", dq, rdq), ("dk", dk, rdk), ("dv", dv, rdv)):
        assert rel_err(to_np(got), ref) <= tol["t"], f"{tag} {name}"
    return out, dk, dv


@pytest.mark.parametrize("kind", ["bf16", "f32"])
def test_tiny_workload_all_segments_with_dropout(kind):
    w = synth.WORKLOADS["tiny"]
    p, seed = 0.1, 0xC0FFEE
    Q, K, V, DO = stage_all(w.B, w.l_x, w.H, w.d, w.seed, kind)
    outs, dks, dvs = [], [], []
    for s0 in w.offsets():
        out, dk, dv = run_segment(Q, K, V, DO, s0, w.l_s, True, kind, p, seed, tag=f"s0={s0}")
        outs.append(out); dks.append(dk); dvs.append(dv)
    # the segments drop what the sequential computation drops: concatenation and segment sum still hold
    full_o, _ = oracle.segment_fwd_dropout(Q.f64, K.f64, V.f64, 0, True, p, seed)
    assert rel_err(to_np(torch.cat(outs, dim=1)), full_o) <= TOL[kind]["t"]
    _, fdk, fdv = oracle.segment_bwd_dropout(Q.f64, K.f64, V.f64, DO.f64, 0, True, p, seed)
    rows_valid = [s0 + w.l_s for s0 in w.offsets()]
    assert rel_err(to_np(lss.lss_reduce_partials(dks, rows_valid)), fdk) <= TOL[kind]["t"]
    assert rel_err(to_np(lss.lss_reduce_partials(dvs, rows_valid)), fdv) <= TOL[kind]["t"]


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("kind,p", [("bf16", 0.25), ("f32", 0.5)])
def test_ragged_segments_and_head_width_128_with_dropout(kind, p, causal):
    Q, K, V, DO = stage_all(2, 1000, 2, 64, 301, kind)
    for a, b in ((0, 300), (300, 437), (437, 1000)):
        run_segment(Q, K, V, DO, a, b - a, causal, kind, p, 17, tag=f"[{a},{b})")
    Q, K, V, DO = stage_all(1, 333, 2, 128, 302, kind)
    run_segment(Q, K, V, DO, 70, 200, causal, kind, p, 18, tag="d128")


def test_skinny_segment_with_key_splits_and_dropout():
    # 58 rows against 6000 keys: the forward and dQ kernels split the keys; the dropped weights must
    # not depend on how
    Q, K, V, DO = stage_all(1, 6000, 2, 64, 303, "bf16")
    run_segment(Q, K, V, DO, 5942, 58, True, "bf16", 0.1, 2 ** 40 + 3, tag="skinny")


@pytest.mark.parametrize("kind", ["bf16", "f32"])
def test_p_zero_is_the_plain_call_bit_for_bit(kind):
    Q, K, V, DO = stage_all(1, 700, 2, 64, 304, kind)
    q, do = Q.dev[:, 200:500].contiguous(), DO.dev[:, 200:500].contiguous()
    a = lss.lss_segment_attn_fwd(q, K.dev, V.dev, 200, True)
    b = lss.lss_segment_attn_fwd(q, K.dev, V.dev, 200, True, p_drop=0.0, seed=5)
    assert all(torch.equal(x, y) for x, y in zip(a, b))
    ga = lss.lss_segment_attn_bwd(q, K.dev, V.dev, 200, a[0], a[1], do, True)
    gb = lss.lss_segment_attn_bwd(q, K.dev, V.dev, 200, a[0], a[1], do, True, p_drop=0.0, seed=5)
    assert all(torch.equal(x, y) for x, y in zip(ga, gb))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("s0,window", [(0, 0), (500, 448), (49000, 30016), (50111, 50048)])
def test_keep_decisions_equal_the_oracles_exactly(s0, window, dtype):
    # Q = 0 makes every visible weight 1/n; V holds a one-hot row e_(j - window) for the 64 keys of a
    # window and zeros elsewhere, so out[r, c] is nonzero exactly where key window + c is kept for
    # row r.  Rows and keys up to the paper's longest sequence.
    B, l_x, H, d, l_s, p, seed = 1, 50112, 2, 64, 1, 0.5, 0xDEADBEEF12345678
    l_s = min(64, l_x - s0)
    q = torch.zeros((B, l_s, H, d), dtype=dtype, device="cuda")
    k = torch.zeros((B, l_x, H, d), dtype=dtype, device="cuda")
    v = torch.zeros((B, l_x, H, d), dtype=dtype, device="cuda")
    v[:, window:window + 64] = torch.eye(64, device="cuda", dtype=dtype).view(1, 64, 1, 64)
    out, lse = lss.lss_segment_attn_fwd(q, k, v, s0, False, p_drop=p, seed=seed)
    got = (out != 0).permute(0, 2, 1, 3).cpu().numpy()                    # [B, H, l_s, 64]
    want = oracle.dropout_mask(p, seed, s0, l_s, l_x, B, H)[..., window:window + 64].astype(bool)
    assert np.array_equal(got, want)
    assert 0.4 < want.mean() < 0.6
    # and in the backward: dv of key j collects dO[r] / (n (1 - p)) from the rows that keep it
    do = torch.ones((B, l_s, H, d), dtype=dtype, device="cuda")
    _, _, dv = lss.lss_segment_attn_bwd(q, k, v, s0, out, lse, do, False, p_drop=p, seed=seed)
    counts = oracle.dropout_mask(p, seed, s0, l_s, l_x, B, H).sum(axis=2)   # [B, H, l_x] rows keeping key j
    got_counts = to_np(dv[..., 0]).transpose(0, 2, 1) * l_x * (1 - p)
    # (bf16: the weight 1/n is rounded to bf16 before it is summed, 2^-9 of up to 64 rows)
    assert np.abs(got_counts - counts).max() < (1e-2 if dtype == torch.float32 else 0.2)
    assert np.array_equal(np.rint(got_counts), counts)


def test_full_size_sampled_rows_with_dropout():
    # lx8k, last segment, through the calls bench.py --dropout makes; rows checked one by one (the
    # mask of a row depends on its global position only, so a one-row oracle call reproduces it)
    w = synth.WORKLOADS["lx8k"]
    p, seed = 0.1, 20231127
    q, k, v, do = synth.workload_inputs(w)
    Q, K, V, DO = (Staged(a, "bf16") for a in (q, k, v, do))
    s0 = (w.N - 1) * w.l_s
    sl = slice(s0, s0 + w.l_s)
    out, lse = lss.lss_segment_attn_fwd(Q.dev[:, sl].contiguous(), K.dev, V.dev, s0, True, p_drop=p, seed=seed)
    dq, dk, dv = lss.lss_segment_attn_bwd(Q.dev[:, sl].contiguous(), K.dev, V.dev, s0, out, lse,
                                          DO.dev[:, sl].contiguous(), True, p_drop=p, seed=seed)
    rng = np.random.default_rng(1)
    for r in sorted({0, 127, 128, w.l_s - 1} | set(int(x) for x in rng.integers(0, w.l_s, size=6))):
        g = s0 + r
        ro, rl = oracle.segment_fwd_dropout(Q.f64[:, g:g + 1], K.f64, V.f64, g, True, p, seed)
        assert rel_err(to_np(out[:, r:r + 1]), ro) <= TOL["bf16"]["t"]
        assert lse_err(to_np(lse[:, :, r:r + 1]), rl) <= TOL["bf16"]["lse"]
        rdq, _, _ = oracle.segment_bwd_dropout(Q.f64[:, g:g + 1], K.f64, V.f64, DO.f64[:, g:g + 1], g, True, p, seed)
        assert rel_err(to_np(dq[:, r:r + 1]), rdq) <= TOL["bf16"]["t"]
    # the (batch 0, head 0) slice of the partials against the oracle run on that slice alone (the
    # generator is keyed on batch*head, which is 0 both in the whole tensor and in the slice)
    _, rdk, rdv = oracle.segment_bwd_dropout(Q.f64[:1, sl, :1], K.f64[:1, :, :1], V.f64[:1, :, :1],
                                             DO.f64[:1, sl, :1], s0, True, p, seed)
    assert rel_err(to_np(dk[:1, :, :1]), rdk) <= TOL["bf16"]["t"]
    assert rel_err(to_np(dv[:1, :, :1]), rdv) <= TOL["bf16"]["t"]

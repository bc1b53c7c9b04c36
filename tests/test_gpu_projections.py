"""GPU parity of the linear maps around the attention (fused-communication form, Section 3,
Principle 3; Fig. 2(ii), (iii), (v)) against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_2311_02382_amd import lss, synth
from _util import TOL, Staged, rel_err, to_np

pytestmark = pytest.mark.gpu


def stage_proj(B, l_x, H, d, seed, std=1.0):
    x, w_q, w_kv = synth.make_projection_inputs(B, l_x, H, d, seed, std)
    return Staged(x, "bf16"), Staged(w_q, "bf16"), Staged(w_kv, "bf16")


def assert_close_elementwise(got, ref, tag):
    # one rounding to bf16 (2^-9 relative) of a sum accumulated in fp32
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    assert np.all(np.isfinite(got)), tag
    bound = 2.0 ** -8 * np.abs(ref) + 1e-4 * np.abs(ref).max()
    bad = np.abs(got - ref) > bound
    assert not bad.any(), f"{tag}: {bad.sum()} elements off, worst {np.abs(got - ref).max()}"


SHAPES = [  # B, l_x, H, d, s0, l_s
    (1, 1024, 4, 64, 256, 256),     # the tiny workload's shape
    (2, 1000, 2, 64, 437, 300),     # E_m = 128: one column tile; ragged rows, unaligned segment
    (1, 700, 2, 128, 0, 700),       # head width 128; the segment is the whole sequence
    (2, 2500, 8, 64, 2442, 58),     # E_m = 512: 20 row tiles and a tail; a skinny last segment
    (3, 130, 2, 64, 1, 1),          # shorter than one tile; a one-row segment
]


@pytest.mark.parametrize("B,l_x,H,d,s0,l_s", SHAPES)
def test_project_qkv_matches_oracle(B, l_x, H, d, s0, l_s):
    X, WQ, WKV = stage_proj(B, l_x, H, d, 9100 + l_x)
    q, k, v = lss.lss_project_qkv(X.dev, WQ.dev, WKV.dev, s0, l_s, H)
    rq, rk, rv = oracle.project_qkv(X.f64, WQ.f64, WKV.f64, s0, l_s, H)
    for name, got, ref in (("q", q, rq), ("k", k, rk), ("v", v, rv)):
        assert rel_err(to_np(got), ref) <= TOL["bf16"]["t"], name
        assert_close_elementwise(to_np(got), ref, f"{name} {B, l_x, H, d, s0, l_s}")


@pytest.mark.parametrize("skip_tail", [False, True])
@pytest.mark.parametrize("B,l_x,H,d,s0,l_s", SHAPES)
def test_project_bwd_matches_oracle(B, l_x, H, d, s0, l_s, skip_tail):
    _, WQ, WKV = stage_proj(B, l_x, H, d, 9200 + l_x)
    E = H * d
    n = B * l_x * E
    dk = synth.normal_f32(9300, n).reshape(B, l_x, H, d)
    dv = synth.normal_f32(9301, n).reshape(B, l_x, H, d)
    DQ = Staged(synth.normal_f32(9302, B * l_s * E).reshape(B, l_s, H, d), "bf16")
    rows_valid = s0 + l_s
    dk[:, rows_valid:] = 0.0
    dv[:, rows_valid:] = 0.0
    rdxq, rdxp = oracle.project_bwd(DQ.f64, dk, dv, WQ.f64, WKV.f64)
    # the device copies carry NaN where the library must not read
    dk_dev, dv_dev = torch.from_numpy(dk).cuda(), torch.from_numpy(dv).cuda()
    dk_dev[:, rows_valid:] = float("nan")
    dv_dev[:, rows_valid:] = float("nan")
    canary = -7.25
    dxp = torch.full((B, l_x, E), canary, dtype=torch.float32, device="cuda")
    dxq, dxp = lss.lss_project_bwd(DQ.dev, dk_dev, dv_dev, WQ.dev, WKV.dev, rows_valid, dx_partial=dxp,
                                   skip_masked_tail=skip_tail)
    assert rel_err(to_np(dxq), rdxq) <= TOL["bf16"]["t"]
    got = to_np(dxp)
    assert rel_err(got[:, :rows_valid], rdxp[:, :rows_valid]) <= TOL["bf16"]["t"]
    first_skipped = -(-rows_valid // 256) * 256 if skip_tail else l_x     # whole 256-row tiles past the data
    assert not np.any(got[:, rows_valid:min(first_skipped, l_x)])
    assert np.all(got[:, first_skipped:] == canary)


@pytest.mark.parametrize("causal", [True, False])
def test_whole_chain_matches_oracle(causal):
    # x -> (Q_i, K, V) -> E_i -> gradients -> dx, all segments of the tiny workload's shape, against
    # the oracle's chain on the same x and weights.  Every stage's bf16 rounding (Q, K, V, E, dQ,
    # the partials as operands) enters here, so the bound is twice the single-stage one.
    B, l_x, H, d, N = 1, 1024, 4, 64, 4
    l_s, E = l_x // N, H * d
    X, WQ, WKV = stage_proj(B, l_x, H, d, 9400)
    DO = Staged(synth.normal_f32(9401, B * l_x * E).reshape(B, l_x, H, d), "bf16")
    parts, ref_parts = [], []
    dx = torch.zeros((B, l_x, E), dtype=torch.float32, device="cuda")
    ref_dx = np.zeros((B, l_x, E))
    rows_valid = []
    for s0 in range(0, l_x, l_s):
        q, k, v = lss.lss_project_qkv(X.dev, WQ.dev, WKV.dev, s0, l_s, H)
        out, lse = lss.lss_segment_attn_fwd(q, k, v, s0, causal)
        do = DO.dev[:, s0:s0 + l_s].contiguous()
        dq, dk, dv = lss.lss_segment_attn_bwd(q, k, v, s0, out, lse, do, causal)
        rv = s0 + l_s if causal else l_x
        dxq, dxp = lss.lss_project_bwd(dq, dk, dv, WQ.dev, WKV.dev, rv)
        dx[:, s0:s0 + l_s] += dxq
        parts.append(dxp); rows_valid.append(rv)
        rq, rk, rvv = oracle.project_qkv(X.f64, WQ.f64, WKV.f64, s0, l_s, H)
        rdq, rdk, rdv = oracle.segment_bwd(rq, rk, rvv, DO.f64[:, s0:s0 + l_s], s0, causal)
        a, p = oracle.project_bwd(rdq, rdk, rdv, WQ.f64, WKV.f64)
        ref_dx[:, s0:s0 + l_s] += a
        ref_parts.append(p)
    total = lss.lss_reduce_partials([p.view(B, l_x, 1, E) for p in parts], rows_valid).view(B, l_x, E)
    dx += total
    ref_dx += oracle.reduce_partials(ref_parts)
    # The 2e-2 that the benchmark spec states is for the attention's own tensors (O, dQ, dK, dV against bf16 inputs).  This
    # chain rounds to bf16 at every stage on the way (Q, K, V, E, dQ, the partials as operands): its bound is twice
    # the single-stage one.  The measured errors are printed so that the margin is on record.
    e_total, e_dx = rel_err(to_np(total), oracle.reduce_partials(ref_parts)), rel_err(to_np(dx), ref_dx)
    print(f"whole chain causal={causal}: sum of dx partials err {e_total:.2e}, dx err {e_dx:.2e} (bound {2 * TOL['bf16']['t']:.0e})")
    assert e_total <= 2 * TOL["bf16"]["t"]
    assert e_dx <= 2 * TOL["bf16"]["t"]


def test_projections_bitwise_reproducible_and_empty_segment():
    B, l_x, H, d = 2, 600, 2, 64
    X, WQ, WKV = stage_proj(B, l_x, H, d, 9500)
    a = lss.lss_project_qkv(X.dev, WQ.dev, WKV.dev, 100, 200, H)
    b = lss.lss_project_qkv(X.dev, WQ.dev, WKV.dev, 100, 200, H)
    assert all(torch.equal(s, t) for s, t in zip(a, b))
    # l_s = 0: K and V are still produced
    q0, k0, v0 = lss.lss_project_qkv(X.dev, WQ.dev, WKV.dev, 600, 0, H)
    assert q0.numel() == 0 and torch.equal(k0, a[1]) and torch.equal(v0, a[2])
    # rows_valid = 0: nothing is read, everything is zero
    nan = torch.full((B, l_x, H, d), float("nan"), dtype=torch.float32, device="cuda")
    dq0 = torch.empty((B, 0, H, d), dtype=torch.bfloat16, device="cuda")
    _, dxp = lss.lss_project_bwd(dq0, nan, nan, WQ.dev, WKV.dev, 0)
    assert torch.count_nonzero(dxp) == 0


@pytest.mark.parametrize("name,seg", [("lx8k", 7), ("lx8k", 2), ("lx32k_d128", 15), ("lx50k_skinny", 863)])
def test_full_size_projections_on_sampled_rows(name, seg):
    # The benchmark's shapes, through the calls bench.py --projections makes.  A projected row
    # depends on its own input row only, so the oracle is run on a sample of rows: tile corners,
    # the ragged tail, random picks; and, for the backward map, rows either side of rows_valid.
    w = synth.WORKLOADS[name]
    B, l_x, H, d, l_s = w.B, w.l_x, w.H, w.d, w.l_s
    E, s0 = H * d, seg * w.l_s
    X, WQ, WKV = stage_proj(B, l_x, H, d, w.seed, w.qkv_std)
    q, k, v = lss.lss_project_qkv(X.dev, WQ.dev, WKV.dev, s0, l_s, H)
    rng = np.random.default_rng(seg)
    rows = sorted({0, 1, 255, 256, 257, l_x // 2, l_x - 257, l_x - 256, l_x - 1, s0, s0 + l_s - 1}
                  | set(int(r) for r in rng.integers(0, l_x, size=24)))
    for b in {0, B - 1}:
        xs = X.f64[b:b + 1, rows]
        _, rk, rv = oracle.project_qkv(xs, WQ.f64, WKV.f64, 0, 0, H)
        assert_close_elementwise(to_np(k[b:b + 1, rows]), rk, f"{name} k batch {b}")
        assert_close_elementwise(to_np(v[b:b + 1, rows]), rv, f"{name} v batch {b}")
        qrows = sorted({0, l_s // 2, l_s - 1} | set(int(r) for r in rng.integers(0, l_s, size=8)))
        rq, _, _ = oracle.project_qkv(X.f64[b:b + 1, [s0 + r for r in qrows]], WQ.f64, WKV.f64, 0, len(qrows), H)
        assert_close_elementwise(to_np(q[b:b + 1, qrows]), rq, f"{name} q batch {b}")
    del k, v
    # backward map on seeded partials (any values do: the map is linear in them)
    rows_valid = s0 + l_s if w.causal else l_x
    gen = torch.Generator(device="cuda"); gen.manual_seed(seg)
    dk = torch.randn((B, l_x, H, d), device="cuda", generator=gen)
    dv = torch.randn((B, l_x, H, d), device="cuda", generator=gen)
    dq = torch.randn((B, l_s, H, d), device="cuda", generator=gen).to(torch.bfloat16)
    dk[:, rows_valid:] = float("nan")
    dv[:, rows_valid:] = float("nan")
    dxq, dxp = lss.lss_project_bwd(dq, dk, dv, WQ.dev, WKV.dev, rows_valid)
    brows = sorted(r for r in set(rows) | {rows_valid - 1, max(rows_valid - 256, 0)} if r < rows_valid)
    for b in {0, B - 1}:
        _, rp = oracle.project_bwd(np.zeros((1, 0, H, d)), to_np(dk[b:b + 1, brows]), to_np(dv[b:b + 1, brows]),
                                   WQ.f64, WKV.f64)
        assert rel_err(to_np(dxp[b:b + 1, brows]), rp) <= TOL["bf16"]["t"]
        qrows = sorted({0, l_s - 1} | set(int(r) for r in rng.integers(0, l_s, size=8)))
        rqx, _ = oracle.project_bwd(to_np(dq[b:b + 1, qrows]), np.zeros((1, 0, H, d)), np.zeros((1, 0, H, d)),
                                    WQ.f64, WKV.f64)
        assert rel_err(to_np(dxq[b:b + 1, qrows]), rqx) <= TOL["bf16"]["t"]
    assert torch.count_nonzero(dxp[:, rows_valid:]) == 0
    assert torch.isfinite(dxp).all() and torch.isfinite(dxq).all()


def test_projection_random_shapes_sweep():
    # seeded random problems, E_m in {128, 256, 384, 640}: column tiles that are cut by the matrix
    # edge (E_m not a multiple of 256), row counts around the 256-row tile, segments at either end
    rng = np.random.default_rng(4242)
    for case in range(16):
        H, d = [(2, 64), (4, 64), (3, 128), (6, 64), (5, 128), (10, 64)][case % 6]
        E = H * d
        B = int(rng.integers(1, 4))
        l_x = int(rng.choice([1, 5, 255, 256, 257, 300, 511, 513, 700]))
        l_s = int(rng.integers(1, l_x + 1))
        s0 = int(rng.choice([0, l_x - l_s]))
        X, WQ, WKV = stage_proj(B, l_x, H, d, 9600 + case)
        q, k, v = lss.lss_project_qkv(X.dev, WQ.dev, WKV.dev, s0, l_s, H)
        for name, got, ref in zip("qkv", (q, k, v), oracle.project_qkv(X.f64, WQ.f64, WKV.f64, s0, l_s, H)):
            assert_close_elementwise(to_np(got), ref, f"case {case} {name} {(B, l_x, H, d, s0, l_s)}")
        rows_valid = int(rng.integers(0, l_x + 1))
        dk = synth.normal_f32(9700 + case, B * l_x * E).reshape(B, l_x, H, d)
        dv = synth.normal_f32(9800 + case, B * l_x * E).reshape(B, l_x, H, d)
        dk[:, rows_valid:] = 0.0
        dv[:, rows_valid:] = 0.0
        DQ = Staged(synth.normal_f32(9900 + case, B * l_s * E).reshape(B, l_s, H, d), "bf16")
        dxq, dxp = lss.lss_project_bwd(DQ.dev, torch.from_numpy(dk).cuda(), torch.from_numpy(dv).cuda(), WQ.dev,
                                       WKV.dev, rows_valid)
        rq, rp = oracle.project_bwd(DQ.f64, dk, dv, WQ.f64, WKV.f64)
        assert rel_err(to_np(dxq), rq) <= TOL["bf16"]["t"], f"case {case} dx_q"
        assert rel_err(to_np(dxp), rp, floor=1e-3) <= TOL["bf16"]["t"], f"case {case} dx_partial"
        assert not np.any(to_np(dxp)[:, rows_valid:])


def test_projections_and_dropout_record_into_a_graph():
    # projections, the dropout pair and the segment sum of dx recorded once, replayed on fresh inputs
    # with eager work in between; every replay equals the eager calls bit for bit
    B, l_x, H, d, s0, l_s, p, seed = 2, 600, 2, 64, 300, 200, 0.2, 99
    E = H * d

    def fresh(sd):
        X, WQ, WKV = stage_proj(B, l_x, H, d, sd)
        DO = Staged(synth.normal_f32(sd + 50, B * l_s * E).reshape(B, l_s, H, d), "bf16")
        return X.dev, WQ.dev, WKV.dev, DO.dev

    x, wq, wkv, do = [t.clone() for t in fresh(800)]
    q = torch.empty((B, l_s, H, d), dtype=torch.bfloat16, device="cuda")
    k, v = (torch.empty((B, l_x, H, d), dtype=torch.bfloat16, device="cuda") for _ in range(2))
    out, dq = torch.empty_like(q), torch.empty_like(q)
    lse = torch.empty((B, H, l_s), dtype=torch.float32, device="cuda")
    dk, dv = (torch.empty((B, l_x, H, d), dtype=torch.float32, device="cuda") for _ in range(2))
    dxq = torch.empty((B, l_s, E), dtype=torch.float32, device="cuda")
    dxp, tot = (torch.empty((B, l_x, E), dtype=torch.float32, device="cuda") for _ in range(2))

    def step():
        lss.lss_project_qkv(x, wq, wkv, s0, l_s, H, q_seg=q, k=k, v=v)
        lss.lss_segment_attn_fwd(q, k, v, s0, True, out=out, lse=lse, p_drop=p, seed=seed)
        lss.lss_segment_attn_bwd(q, k, v, s0, out, lse, do, True, dq=dq, dk_partial=dk, dv_partial=dv,
                                 p_drop=p, seed=seed)
        lss.lss_project_bwd(dq, dk, dv, wq, wkv, s0 + l_s, dx_q=dxq, dx_partial=dxp)
        lss.lss_reduce_partials([dxp.view(B, l_x, 1, E), dxp.view(B, l_x, 1, E)], [s0 + l_s, 100],
                                out=tot.view(B, l_x, 1, E))

    results = (q, k, v, out, lse, dq, dk, dv, dxq, dxp, tot)
    step()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for sd in (801, 802, 803):
        for dst, src in zip((x, wq, wkv, do), fresh(sd)):
            dst.copy_(src)
        for t in results:
            t.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in results]
        for t in results:
            t.fill_(float("nan"))
        step()
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(zip(got, results)):
            assert torch.equal(a, b), f"seed {sd}: result {i} differs between replay and eager"
        assert all(torch.isfinite(t).all() for t in got)


@pytest.mark.parametrize("B,l_x,H,d,s0,l_s", SHAPES)
def test_project_bwd_weight_matches_oracle(B, l_x, H, d, s0, l_s):
    X, _, _ = stage_proj(B, l_x, H, d, 9600 + l_x)
    E = H * d
    n = B * l_x * E
    dk = synth.normal_f32(9601, n).reshape(B, l_x, H, d)
    dv = synth.normal_f32(9602, n).reshape(B, l_x, H, d)
    DQ = Staged(synth.normal_f32(9603, B * l_s * E).reshape(B, l_s, H, d), "bf16")
    rows_valid = s0 + l_s
    dk[:, rows_valid:] = 0.0
    dv[:, rows_valid:] = 0.0
    rq, rkv = oracle.project_bwd_weight(X.f64, DQ.f64, dk, dv, s0)
    # the device copies carry NaN where the library must not read
    dk_dev, dv_dev = torch.from_numpy(dk).cuda(), torch.from_numpy(dv).cuda()
    dk_dev[:, rows_valid:] = float("nan")
    dv_dev[:, rows_valid:] = float("nan")
    need = lss.lss_project_bwd_weight_scratch_bytes(l_s, l_x, B, H, d)
    scratch = torch.full((max(need, 16),), 0xFF, dtype=torch.uint8, device="cuda")
    dwq, dwkv = lss.lss_project_bwd_weight(X.dev, DQ.dev, dk_dev, dv_dev, s0, rows_valid, scratch=scratch)
    # fp32 sums of products of bf16-rounded operands: the partials' rounding (2^-9 each, independent)
    # averages out over the rows, the bound is the single-stage one
    assert rel_err(to_np(dwq), rq) <= TOL["bf16"]["t"]
    assert rel_err(to_np(dwkv), rkv) <= TOL["bf16"]["t"]
    # against the oracle fed the same bf16-rounded partials the matrix cores see: fp32 accumulation only
    rdk = to_np(torch.from_numpy(dk).cuda().to(torch.bfloat16))
    rdv = to_np(torch.from_numpy(dv).cuda().to(torch.bfloat16))
    _, rkv_r = oracle.project_bwd_weight(X.f64, DQ.f64, rdk, rdv, s0)
    assert rel_err(to_np(dwq), rq) <= TOL["f32"]["t"] and rel_err(to_np(dwkv), rkv_r) <= TOL["f32"]["t"]
    again = lss.lss_project_bwd_weight(X.dev, DQ.dev, dk_dev, dv_dev, s0, rows_valid)
    assert torch.equal(again[0], dwq) and torch.equal(again[1], dwkv)


def test_project_bwd_weight_sums_over_segments_and_empty_cases():
    B, l_x, H, d, N = 2, 640, 2, 64, 4
    X, WQ, WKV = stage_proj(B, l_x, H, d, 9700)
    E, l_s = H * d, l_x // N
    DO = Staged(synth.normal_f32(9701, B * l_x * E).reshape(B, l_x, H, d), "bf16")
    tot_q, tot_kv = np.zeros((E, E)), np.zeros((E, 2 * E))
    for i in range(N):
        s0 = i * l_s
        q, k, v = lss.lss_project_qkv(X.dev, WQ.dev, WKV.dev, s0, l_s, H)
        out, lse = lss.lss_segment_attn_fwd(q, k, v, s0, True)
        dq, dkp, dvp = lss.lss_segment_attn_bwd(q, k, v, s0, out, lse, DO.dev[:, s0:s0 + l_s].contiguous(), True)
        a, b_ = lss.lss_project_bwd_weight(X.dev, dq, dkp, dvp, s0, s0 + l_s)
        tot_q += to_np(a)
        tot_kv += to_np(b_)
    # the oracle's chain on the whole sequence as one segment (Section 4: the contributions add up)
    rq_, rk_, rv_ = oracle.project_qkv(X.f64, WQ.f64, WKV.f64, 0, l_x, H)
    rdq, rdk, rdv = oracle.segment_bwd(rq_, rk_, rv_, DO.f64, 0, True)
    ref_q, ref_kv = oracle.project_bwd_weight(X.f64, rdq, rdk, rdv, 0)
    assert rel_err(tot_q, ref_q) <= 2 * TOL["bf16"]["t"] and rel_err(tot_kv, ref_kv) <= 2 * TOL["bf16"]["t"]
    # no query rows / no valid rows: zeros
    dq0 = torch.empty((B, 0, H, d), dtype=torch.bfloat16, device="cuda")
    a, b_ = lss.lss_project_bwd_weight(X.dev, dq0, dkp, dvp, 0, 0, dw_q=torch.full((E, E), 2.0, device="cuda"),
                                       dw_kv=torch.full((E, 2 * E), 2.0, device="cuda"))
    assert not a.any() and not b_.any()

"""GPU parity at the full benchmark sizes, through the same calls bench.py times.

The oracle cannot afford whole configurations here (9-31 TFLOP of fp64), so each case checks
  * sampled query rows of out / lse / dq against the oracle, row by row (a row of Eq. 2 depends on
    that query row alone: the oracle is called on a one-row segment at the row's global position);
  * dk_partial / dv_partial of one (batch, head) slice against the oracle run on that whole slice;
  * properties that hold at any size: column sums of the partials (sum_j dS[r, j] = 0 and
    sum_j P[r, j] = 1), exactly-zero causal tails, and the exact fp32 segment sum.
Inputs are the seeded workload tensors of synth.WORKLOADS, bf16-rounded; the oracle reads exactly those values."""
import numpy as np
import pytest
import torch

import oracle
from paper_2311_02382_amd import lss, synth
from _util import TOL, lse_err, rel_err, to_np

pytestmark = pytest.mark.gpu
T = TOL["bf16"]


class Workload:
    def __init__(self, name):
        self.w = w = synth.WORKLOADS[name]
        q, k, v, do = synth.workload_inputs(w)
        self.bits = [synth.f32_to_bf16_bits(a) for a in (q, k, v, do)]
        del q, k, v, do
        self.dev = [torch.from_numpy(b.view(np.int16)).cuda().view(torch.bfloat16) for b in self.bits]

    def host(self, which, b, h, rows=slice(None)):
        """float64 copy of tensor `which` (0..3 = q, k, v, dO) for one (batch, head): [1, rows, 1, d]."""
        sl = self.bits[which][b:b + 1, rows, h:h + 1, :]
        return synth.bf16_bits_to_f64(sl).reshape(sl.shape)

    def run_segment(self, i):
        w = self.w
        s0 = i * w.l_s
        qd, kd, vd, dod = self.dev
        q_seg = qd[:, s0:s0 + w.l_s].contiguous()
        do_seg = dod[:, s0:s0 + w.l_s].contiguous()
        out, lse = lss.lss_segment_attn_fwd(q_seg, kd, vd, s0, w.causal)
        dq, dk, dv = lss.lss_segment_attn_bwd(q_seg, kd, vd, s0, out, lse, do_seg, w.causal)
        return s0, out, lse, dq, dk, dv


def sample_rows(l_s, n=12):
    picks = {0, 1, 31, 32, 63, 64, 127, 128, 255, 256, l_s // 2, l_s - 65, l_s - 33, l_s - 2, l_s - 1}
    rng = np.random.default_rng(l_s)
    picks |= set(int(x) for x in rng.integers(0, l_s, size=n))
    return sorted(r for r in picks if 0 <= r < l_s)


def check_segment(W, i, slices, dkv_slice):
    w = W.w
    s0, out, lse, dq, dk, dv = W.run_segment(i)
    kv_hi = s0 + w.l_s if w.causal else w.l_x
    # -- sampled rows of out, lse, dq
    for (b, h) in slices:
        kh, vh = W.host(1, b, h), W.host(2, b, h)
        rows = sample_rows(w.l_s)
        ref_o, ref_l, ref_dq = [], [], []
        for r in rows:
            g = s0 + r
            qr, dor = W.host(0, b, h, slice(g, g + 1)), W.host(3, b, h, slice(g, g + 1))
            o, l = oracle.segment_fwd(qr, kh, vh, g, w.causal)
            dq_r, _, _ = oracle.segment_bwd(qr, kh, vh, dor, g, w.causal)
            ref_o.append(o[0, 0, 0]); ref_l.append(l[0, 0, 0]); ref_dq.append(dq_r[0, 0, 0])
        idx = torch.tensor(rows, device="cuda")
        assert rel_err(to_np(out[b, idx, h]), np.array(ref_o)) <= T["t"], (i, b, h, "out")
        assert lse_err(to_np(lse[b, h, idx]), np.array(ref_l)) <= T["lse"], (i, b, h, "lse")
        assert rel_err(to_np(dq[b, idx, h]), np.array(ref_dq)) <= T["t"], (i, b, h, "dq")
    # -- one whole slice of the partials
    if dkv_slice is not None:
        b, h = dkv_slice
        sl = slice(s0, s0 + w.l_s)
        _, rdk, rdv = oracle.segment_bwd(W.host(0, b, h, sl), W.host(1, b, h), W.host(2, b, h), W.host(3, b, h, sl),
                                         s0, w.causal)
        assert rel_err(to_np(dk[b, :, h]), rdk[0, :, 0]) <= T["t"], (i, "dk")
        assert rel_err(to_np(dv[b, :, h]), rdv[0, :, 0]) <= T["t"], (i, "dv")
    # -- properties at full size
    if w.causal:
        assert torch.count_nonzero(dk[:, kv_hi:]) == 0 and torch.count_nonzero(dv[:, kv_hi:]) == 0
    do_sum = W.dev[3][:, s0:s0 + w.l_s].double().sum(dim=1)            # [B, H, d]
    dv_sum = dv.double().sum(dim=1)
    dk_sum = dk.double().sum(dim=1)
    scale = float(do_sum.abs().max())
    assert float((dv_sum - do_sum).abs().max()) <= 2e-2 * scale         # sum_j P[r, j] = 1
    assert float(dk_sum.abs().max()) <= 2e-2 * float(dk.abs().max()) * np.sqrt(w.l_s)   # sum_j dS[r, j] = 0
    assert bool(torch.isfinite(out.float()).all()) and bool(torch.isfinite(dq.float()).all())
    return dk, dv


def test_lx8k_all_segments_and_segment_sum():
    W = Workload("lx8k")
    w = W.w
    dks, dvs = [], []
    for i in range(w.N):
        dk, dv = check_segment(W, i, [(0, 0), (w.B - 1, w.H - 1)], (1, 3) if i in (0, 4, 7) else None)
        dks.append(dk); dvs.append(dv)
    rows_valid = [s0 + w.l_s for s0 in w.offsets()]
    dK = lss.lss_reduce_partials(dks, rows_valid)
    dV = lss.lss_reduce_partials(dvs, rows_valid)
    ref = dks[0].clone()
    for p in dks[1:]:
        ref += p
    assert torch.equal(dK, ref)                                         # exact fp32 sum in list order
    # the sum over segments is the full-sequence gradient (one slice, whole sequence in the oracle)
    b, h = 0, 5
    _, fdk, fdv = oracle.segment_bwd(W.host(0, b, h), W.host(1, b, h), W.host(2, b, h), W.host(3, b, h), 0, True)
    assert rel_err(to_np(dK[b, :, h]), fdk[0, :, 0]) <= T["t"]
    assert rel_err(to_np(dV[b, :, h]), fdv[0, :, 0]) <= T["t"]


def test_lx24k_near_uniform_softmax():
    W = Workload("lx24k")
    w = W.w
    check_segment(W, w.N - 1, [(0, 0), (w.B - 1, w.H - 1)], (2, 7))
    check_segment(W, 0, [(1, 3)], None)


def test_lx32k_d128_noncausal():
    W = Workload("lx32k_d128")
    w = W.w
    check_segment(W, 0, [(0, 0), (0, w.H - 1)], (0, 9))
    check_segment(W, w.N - 1, [(0, 4)], None)


def test_lx50k_ragged_tails():
    W = Workload("lx50k")
    w = W.w
    assert w.l_s == 1044 and w.l_s % 32 != 0      # ragged: 1044 = 8 * 128 + 20
    check_segment(W, w.N - 1, [(0, 0), (0, w.H - 1)], (0, 2))           # densest segment, s0 = 49,068
    check_segment(W, 0, [(0, 1)], (0, 1))
    check_segment(W, 23, [(0, 6)], None)


def test_lx50k_skinny_segments():
    # 58-row segments (less than half a query tile; one Q/dO tile per dK/dV workgroup)
    W = Workload("lx50k_skinny")
    w = W.w
    assert w.l_s == 58
    check_segment(W, w.N - 1, [(0, 0), (w.B - 1, w.H - 1)], (1, 2))    # s0 = 50,054: sees the whole sequence
    check_segment(W, 0, [(2, 5)], (2, 5))                               # s0 = 0: 58 keys, all diagonal
    check_segment(W, 431, [(3, 1)], (0, 6))


def test_lx50k_full_sweep_segment_sum_is_exact_and_reproducible():
    # all 48 segments back to back; dk partials accumulated with the library's fixed-order sum
    W = Workload("lx50k")
    w = W.w
    rows_valid = [s0 + w.l_s for s0 in w.offsets()]

    def sweep():
        parts = [W.run_segment(i)[4] for i in range(w.N)]
        return lss.lss_reduce_partials(parts, rows_valid), parts

    dK1, parts = sweep()
    ref = parts[0].clone()
    for p in parts[1:]:
        ref += p
    assert torch.equal(dK1, ref)
    del parts, ref
    dK2, _ = sweep()
    assert torch.equal(dK1.view(torch.int32), dK2.view(torch.int32))    # bit-reproducible
    # keys of the last 64 positions receive contributions from the last segment only: oracle by rows
    b, h, j_lo = 0, 3, w.l_x - 64
    sl = slice(j_lo, w.l_x)
    _, rdk, _ = oracle.segment_bwd(W.host(0, b, h, sl), W.host(1, b, h), W.host(2, b, h), W.host(3, b, h, sl),
                                   j_lo, True)
    assert rel_err(to_np(dK1[b, j_lo:, h]), rdk[0, j_lo:, 0]) <= T["t"]


@pytest.mark.parametrize("name,slice_bh", [("lx8k", (1, 2)), ("lx24k", (2, 7)), ("lx32k_d128", (0, 9)), ("lx50k", (0, 5))])
def test_benchmark_configuration_sums_to_the_full_sequence_gradient(name, slice_bh):
    # Exactly the calls of one bench.py step, for every configuration it times: preallocated outputs, all N
    # segments forward and backward with LSS_FLAG_SKIP_MASKED_TAIL (key tiles past a causal segment's last
    # query stay unwritten -- here they hold a canary), then the segment sum with rows_valid.  Checked
    # against ONE call of the oracle on the unsegmented sequence (Section 3, Principle 3: the segments'
    # outputs concatenate to the sequential result; Principle 4 / Fig. 2(v): the partials add up to the
    # full gradient), for one (batch, head) slice: all l_x rows of dK and dV, the concatenated dQ and out.
    W = Workload(name)
    w = W.w
    qd, kd, vd, dod = W.dev
    canary = 12345.0
    dks = [torch.full(kd.shape, canary, dtype=torch.float32, device="cuda") for _ in range(w.N)]
    dvs = [torch.full(kd.shape, canary, dtype=torch.float32, device="cuda") for _ in range(w.N)]
    outs, dqs, lses = [], [], []
    for i, s0 in enumerate(w.offsets()):
        q_seg, do_seg = qd[:, s0:s0 + w.l_s].contiguous(), dod[:, s0:s0 + w.l_s].contiguous()
        out, lse = lss.lss_segment_attn_fwd(q_seg, kd, vd, s0, w.causal)
        dq, _, _ = lss.lss_segment_attn_bwd(q_seg, kd, vd, s0, out, lse, do_seg, w.causal,
                                            dk_partial=dks[i], dv_partial=dvs[i], skip_masked_tail=True)
        outs.append(out); dqs.append(dq); lses.append(lse)
    rows_valid = [s0 + w.l_s if w.causal else w.l_x for s0 in w.offsets()]
    for i, rv in enumerate(rows_valid):
        hidden = -(-rv // 128) * 128                       # first key tile no query of segment i sees
        assert bool((dks[i][:, hidden:] == canary).all()) and bool((dvs[i][:, hidden:] == canary).all())
        assert torch.count_nonzero(dks[i][:, rv:hidden]) == 0 and torch.count_nonzero(dvs[i][:, rv:hidden]) == 0
    dK = lss.lss_reduce_partials(dks, rows_valid)
    dV = lss.lss_reduce_partials(dvs, rows_valid)
    del dks, dvs
    b, h = slice_bh
    qh, kh, vh, doh = (W.host(t, b, h) for t in range(4))
    fdq, fdk, fdv = oracle.segment_bwd(qh, kh, vh, doh, 0, w.causal)
    fo, fl = oracle.segment_fwd(qh, kh, vh, 0, w.causal)
    errs = {"dK": rel_err(to_np(dK[b, :, h]), fdk[0, :, 0]), "dV": rel_err(to_np(dV[b, :, h]), fdv[0, :, 0]),
            "dQ": rel_err(to_np(torch.cat(dqs, dim=1)[b, :, h]), fdq[0, :, 0]),
            "out": rel_err(to_np(torch.cat(outs, dim=1)[b, :, h]), fo[0, :, 0])}
    e_lse = lse_err(to_np(torch.cat(lses, dim=2)[b, h]), fl[0, 0])
    print(f"{name} slice {slice_bh}: {errs} lse {e_lse:.2e}")
    assert max(errs.values()) <= T["t"], errs
    assert e_lse <= T["lse"]

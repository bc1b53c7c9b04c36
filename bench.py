#!/usr/bin/env python3
"""Benchmark of the segment-attention hot path on one MI355X.

A "step" is one pass of the whole path over one synthetic batch: for each of the N
segments of the sequence, forward then backward (Eq. 2 of Section 3 and its gradient),
followed by the segment sum of the dK and dV partials (the arithmetic of the
reduce-scatter of Fig. 2(v)).  Inputs are resident in HBM before the timed region.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload lx24k] [--projections | --layer-ops]

The default workload is lx24k (B=4, l_x=24576, 6 segments of 4096 rows, 16 heads of width 64, causal): the
largest configuration with d = 64 and l_s >= 1024.  Run without --workload, the line also carries `extra`: the
other four configurations (tiny, lx8k, lx32k_d128, lx50k), each timed the same way over at least 5 steps and
50 ms, after at least 30 ms of warm-up (a run needs that long under load to reach its steady state).

With --projections every segment also runs the linear maps either side of the attention in
the fused-communication form (Q_i, K, V from x before the forward; dx_q and dx_partial after
the backward; Fig. 2(ii), (v)), the segment sum then runs on the dx partials, and `value`
counts the projections' flops as well: a second workload, not the headline one.

With --segments I,J,... only the listed segments run (and the sum of their partials): for workloads whose
N partial buffers do not fit in memory at once.  --layer-ops, --dropout P and --dtype f32 are further workloads
(see their help texts).

Prints ONE JSON line.  `value` is the strict-count rate: 12*d flops per unmasked
(query, key) pair and head (six matrix products: S, PV, dV, dP, dQ, dK), recomputation not
counted, over a timed region that holds the library's calls and nothing else.  The region is then run a
second time with the dominant kernel bracketed by HIP events on its launch stream (`roofline`: against the
matrix peak, or against the HBM peak when the kernel's algorithmic flops per algorithmic byte are below the
machine's balance point); the other kernels' averages come from an untimed survey pass.  `cpu_baseline` is
the fp64 oracle's rate on the host cores for a bounded sample of the same workload.

Contract timed: lss_segment_attn_fwd and lss_segment_attn_bwd as they are (every row of the partials written, rows
no query of a causal segment sees as zeros).  --skip-masked-tail passes LSS_FLAG_SKIP_MASKED_TAIL instead
(lss_segment_attn_bwd_ex): the only reader of the partials here is the segment sum, which is told how many rows of
each part hold data, so those zeros need not be written (0.7 % of an lx24k step, 1.7 % of an lx8k step).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 matrix peak (published)
PEAK_F32_TFLOPS = 157.3        # ... and the fp32 matrix peak, for --dtype f32
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E peak (published)

# Matrix products each kernel contributes to the strict count (per pair: 2*d flops each).
# fwd: S and PV.  The backward's main kernel holds two kinds of workgroup: dQ (dP and dQ; it also
# recomputes S) and dK/dV (dV and dK; it also recomputes S and dP).  Together the six products of
# the 12*d count.  (bwd_dq_kernel / bwd_dkv_kernel: the fp32 path, which launches them separately.)
# Names are those of the __global__ functions, as a profiler prints them (bf16: the tuned kernels; fwd_kernel,
# bwd_dq_kernel, bwd_dkv_kernel: the general kernels that serve --dtype f32, launched separately).
ALGO_PRODUCTS = {"fwd_bf16_kernel": 2, "bwd_main_bf16_kernel": 4, "fwd_kernel": 2, "bwd_dq_kernel": 2, "bwd_dkv_kernel": 2}
EXEC_PRODUCTS = {"fwd_bf16_kernel": 2, "bwd_main_bf16_kernel": 7, "fwd_kernel": 2, "bwd_dq_kernel": 3, "bwd_dkv_kernel": 4}
FWD_KERNELS = ("fwd_bf16_kernel", "fwd_kernel", "fwd_merge_kernel")
BWD_KERNELS = ("bwd_prep_bf16_kernel", "bwd_rowdot_kernel", "bwd_main_bf16_kernel", "bwd_dq_kernel", "bwd_dkv_kernel",
               "bwd_dq_merge_kernel")


def measured_traffic(workload: str, kernel: str):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary, or None."""
    path = os.path.join(ROOT, "profiles", f"{workload}_hbm_traffic.md")
    try:
        for line in open(path):
            parts = line.split()
            if len(parts) == 3 and parts[0] == "traffic_bytes_per_launch" and parts[1] == kernel:
                return float(parts[2])
    except OSError:
        pass
    return None


def layer_ops(args, w) -> int:
    """The segment-local remainder of a layer (Section 3, Principles 1 and 2) on the workload's shape:
    per segment, x = tok + PE rows, LayerNorm, feed-forward unit (E_m -> 4 E_m -> E_m, exact GeLU),
    residual connection with dropout 0.1 on the branch, then the same backwards, weight gradients of the two maps included.  `value` is the feed-forward
    unit's matrix flops (12 * rows * E_m * 4 E_m per segment) over the time of the whole step, streaming kernels included."""
    import numpy as np
    import torch

    from paper_2311_02382_amd import lss, synth, timing

    dev = torch.device("cuda:0")
    E, F, l_s, offs = w.H * w.d, 4 * w.H * w.d, w.l_s, w.offsets()
    rows = w.B * l_s

    def stage(seed, shape, std=1.0, bf16=True):
        a = (synth.normal_f32(seed, int(np.prod(shape))) * np.float32(std)).reshape(shape)
        if not bf16:
            return torch.from_numpy(a).to(dev), a.astype(np.float64)
        bits = synth.f32_to_bf16_bits(a)
        return (torch.from_numpy(bits.view(np.int16).reshape(shape)).to(dev).view(torch.bfloat16),
                synth.bf16_bits_to_f64(bits).reshape(shape))

    tok, tok_h = stage(w.seed + 20, (w.B, w.l_x, E))
    pe, pe_h = stage(w.seed + 21, (w.l_x, E))
    w1, w1_h = stage(w.seed + 22, (E, F), E ** -0.5)
    w2, w2_h = stage(w.seed + 23, (F, E), F ** -0.5)
    dy, dy_h = stage(w.seed + 24, (w.B, l_s, E))
    gamma, gamma_h = stage(w.seed + 25, (E,), 0.1, bf16=False)
    gamma += 1.0
    gamma_h = gamma_h + 1.0
    beta, beta_h = stage(w.seed + 26, (E,), 0.1, bf16=False)
    tok_seg = [tok[:, s0:s0 + l_s].contiguous() for s0 in offs]
    bf = dict(dtype=torch.bfloat16, device=dev)
    P_HIDDEN = 0.1      # dropout on the feed-forward branch of the residual connection
    x, h, dh, dx, x2, dyb = (torch.empty((w.B, l_s, E), **bf) for _ in range(6))
    u, g, dg, du = (torch.empty((w.B, l_s, F), **bf) for _ in range(4))
    y = torch.empty((w.B, l_s, E), **bf)
    mean, rstd = (torch.empty((rows,), dtype=torch.float32, device=dev) for _ in range(2))
    dgamma, dbeta = (torch.empty((E,), dtype=torch.float32, device=dev) for _ in range(2))
    dpe = torch.empty((l_s, E), dtype=torch.float32, device=dev)
    scratch = torch.empty((max(16, lss.lss_layernorm_bwd_scratch_bytes(rows, E)),), dtype=torch.uint8, device=dev)
    dw1 = torch.empty((E, F), dtype=torch.float32, device=dev)
    dw2 = torch.empty((F, E), dtype=torch.float32, device=dev)
    wscratch = torch.empty((max(16, lss.lss_linear_bwd_weight_scratch_bytes(rows, E, F),
                            lss.lss_linear_bwd_weight_scratch_bytes(rows, F, E)),), dtype=torch.uint8, device=dev)

    def step():
        for i, s0 in enumerate(offs):
            lss.lss_embed_pe_fwd(tok_seg[i], pe, s0, x=x)
            lss.lss_layernorm_fwd(x, gamma, beta, y=h, mean=mean, rstd=rstd)
            if args.fused_gelu:     # GeLU and its derivative in the GEMMs' epilogues: same bits, two launches fewer
                lss.lss_linear_gelu_fwd(h, w1, u=u, g=g)
            else:
                lss.lss_linear_fwd(h, w1, c=u)
                lss.lss_gelu_fwd(u, g=g)
            lss.lss_linear_fwd(g, w2, c=y)
            lss.lss_residual_dropout_add(x, y, s0, P_HIDDEN, w.seed, out=x2)          # x2 = x + dropout(y)
            lss.lss_residual_dropout_add(None, dy, s0, P_HIDDEN, w.seed, out=dyb)       # gradient entering the branch
            if args.fused_gelu:
                lss.lss_linear_bwd_input_gelu(dyb, w2, u, du=du)
            else:
                lss.lss_linear_bwd_input(dyb, w2, da=dg)
                lss.lss_gelu_bwd(u, dg, du=du)
            lss.lss_linear_bwd_input(du, w1, da=dh)
            lss.lss_linear_bwd_weight(g, dyb, dw=dw2, scratch=wscratch)      # this segment's share of dW2 and dW1
            lss.lss_linear_bwd_weight(h, du, dw=dw1, scratch=wscratch)
            lss.lss_layernorm_bwd(x, gamma, mean, rstd, dh, dx=dx, dgamma=dgamma, dbeta=dbeta, scratch=scratch)
            lss.lss_residual_dropout_add(dy, dx, s0, 0.0, 0, out=dx)                    # + the gradient on the skip path
            lss.lss_embed_pe_bwd(dx, dpe_rows=dpe)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    names = timing.kernel_names()

    def read_kernels(steps):
        out_ = {}
        for kid_, name_ in names.items():
            ms, n = timing.read(kid_)
            if n:
                out_[name_] = {"launches_per_step": n / steps, "avg_us": 1e3 * ms / n, "ms_per_step": ms / steps}
        return out_

    timing.reset()
    timing.enable(True)
    for _ in range(2):
        step()
    torch.cuda.synchronize()
    timing.enable(False)
    kernels = read_kernels(2)
    dom = max(("proj_gemm_kernel:linear_fwd", "proj_gemm_kernel:linear_bwd_input"), key=lambda n_: kernels[n_]["ms_per_step"])
    timing.reset()
    timing.select([k_ for k_, n_ in names.items() if n_ == dom])
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    gpu_ms = e0.elapsed_time(e1)
    timing.enable(False)
    ms_per_step = max(wall_ms, gpu_ms) / args.steps
    timed = read_kernels(args.steps)
    kernels[dom] = dict(timed[dom], timed_region=True)

    lin_flops = 2.0 * rows * E * F                  # one linear map of one segment
    flops_step = 6.0 * lin_flops * w.N             # two maps forward, their input and weight gradients backward
    # algorithmic bytes per launch: every operand read once, every result written once
    bytes_per_launch = {
        "embed_pe_fwd_kernel": 4 * rows * E + 2 * l_s * E, "embed_pe_bwd_kernel": 2 * rows * E + 4 * l_s * E,
        "layernorm_fwd_kernel": 4 * rows * E + 8 * rows + 8 * E,
        "layernorm_bwd_kernel": 6 * rows * E + 8 * rows + 4 * E + 8 * E * ((rows + 31) // 32),
        "layernorm_bwd_params_kernel": 8 * E * ((rows + 31) // 32) + 8 * E,
        "gelu_fwd_kernel": 4 * rows * F, "gelu_bwd_kernel": 6 * rows * F,
        "residual_add_kernel": 16 * rows * E / 3.0,        # three launches: 3, 2 and 3 tensors of rows * E bf16
    }
    for name, kk in kernels.items():
        if name in bytes_per_launch:
            kk["algorithmic_GBps"] = round(bytes_per_launch[name] / (kk["avg_us"] * 1e-6) / 1e9, 1)
            kk["frac_of_hbm_peak"] = round(kk["algorithmic_GBps"] / PEAK_HBM_GBS, 4)
        elif name.startswith("proj_gemm_kernel:linear_") or name == "wgrad_gemm_kernel":
            kk["algorithmic_tflops"] = round(lin_flops / (kk["avg_us"] * 1e-6) / 1e12, 2)
        kk["avg_us"] = round(kk["avg_us"], 2)
        kk["ms_per_step"] = round(kk["ms_per_step"], 4)
    achieved = lin_flops / (timed[dom]["avg_us"] * 1e-6) / 1e12
    roofline = {"kernel": dom, "bound": "mfma", "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": None,
                "avg_launch_us": round(timed[dom]["avg_us"], 2), "algorithmic_flops_per_launch": lin_flops}

    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle
        n_s = min(l_s, max(1, int(2.0e11 / (12.0 * w.B * E * F))))     # about 2e11 fp64 flops of matrix work
        t = time.perf_counter()
        xs = oracle.embed_pe(tok_h[:, :n_s], pe_h, 0)
        hs, _, _ = oracle.layernorm_fwd(xs, gamma_h, beta_h)
        ys, us = oracle.ffn_fwd(hs, w1_h, w2_h)
        oracle.residual_dropout_add(xs, ys, 0, P_HIDDEN, w.seed)
        dybs = oracle.residual_dropout_add(None, dy_h[:, :n_s], 0, P_HIDDEN, w.seed)
        dhs = oracle.ffn_bwd(dybs, us, w1_h, w2_h)
        oracle.linear_bwd_weight(oracle.gelu(us), dybs)
        oracle.linear_bwd_weight(hs, np.matmul(dybs, w2_h.T) * oracle.gelu_grad(us))
        dxs, _, _ = oracle.layernorm_bwd(xs, gamma_h, dhs)
        oracle.embed_pe_bwd(dy_h[:, :n_s] + dxs)
        t_cpu = time.perf_counter() - t
        from threadpoolctl import threadpool_info
        blas_threads = max([p_["num_threads"] for p_ in threadpool_info() if p_.get("user_api") == "blas"] or [1])
        cpu_baseline = {"value": round(12.0 * w.B * n_s * E * F / t_cpu / 1e12, 6), "unit": "TFLOP/s",
                        "cores": blas_threads, "kind": "oracle",
                        "sample": f"the first {n_s} rows of segment 0 for every batch entry, the same chain of "
                                  f"operations, {t_cpu:.1f} s of fp64 CPU work, same flop count"}

    value = flops_step / (ms_per_step * 1e-3) / 1e12
    print(json.dumps({
        "metric": "segment-local layer operations fwd+bwd: feed-forward matrix TFLOP/s over the whole step on 1 MI355X",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name + "+layer-ops" + ("+fused-gelu" if args.fused_gelu else ""), "B": w.B, "l_x": w.l_x, "N": w.N, "l_s": l_s, "E_m": E, "F": F,
                   "step": "per segment: x = tok + PE rows, LayerNorm, GeLU(h W1) W2, x + dropout(.), and the same backwards"},
        "frac_of_bf16_peak": round(value / PEAK_BF16_TFLOPS, 4),
        "gpu_ms_per_step_events": round(gpu_ms / args.steps, 4),
        "roofline": roofline, "cpu_baseline": cpu_baseline, "kernels": kernels}))
    return 0


def attention(args, w, steps, warmup, with_cpu_baseline, min_warm_ms=0.0, min_timed_ms=0.0):
    """Times `steps` steps of workload `w` and returns the JSON line as a dict.

    min_warm_ms / min_timed_ms (the `extra` configurations): warm up for at least that much GPU time and time at
    least that much, whatever `steps` and `warmup` say -- a run takes some ten milliseconds under load to reach
    its steady state (clock, launch queue), and five 1 ms steps after two would be timed on the way there (lx8k:
    373 against 413 TFLOP/s)."""
    import numpy as np
    import torch

    from paper_2311_02382_amd import lss, synth, timing

    dev = torch.device("cuda:0")
    q, k, v, do = synth.workload_inputs(w)

    f32 = args.dtype == "f32"
    peak = PEAK_F32_TFLOPS if f32 else PEAK_BF16_TFLOPS

    class HostCopy:
        """What the oracle reads: exactly the values the device tensor holds, widened to float64 on demand."""
        def __init__(self, arr, is_bits):
            self.arr, self.is_bits, self.shape = arr, is_bits, arr.shape

        def __getitem__(self, idx):
            return HostCopy(self.arr[idx], self.is_bits)

        def f64(self):
            return synth.bf16_bits_to_f64(self.arr).reshape(self.arr.shape) if self.is_bits else self.arr.astype(np.float64)

    def stage(x):
        if f32:
            x = np.ascontiguousarray(x, dtype=np.float32)
            return torch.from_numpy(x).to(dev), HostCopy(x, False)
        bits = synth.f32_to_bf16_bits(x)
        return torch.from_numpy(bits.view(np.int16).reshape(x.shape)).to(dev).view(torch.bfloat16), HostCopy(bits, True)

    (qd, qb), (kd, kb), (vd, vb), (dod, dob) = map(stage, (q, k, v, do))
    del q, k, v, do
    seg_ids = list(range(w.N)) if args.segments is None else sorted({int(t_) for t_ in args.segments.split(",")})
    if not seg_ids or seg_ids[0] < 0 or seg_ids[-1] >= w.N:
        raise SystemExit(f"bench.py: --segments must name segments in [0, {w.N})")
    offs, l_s = [w.offsets()[i_] for i_ in seg_ids], w.l_s
    E = w.H * w.d
    q_seg = [qd[:, s0:s0 + l_s].contiguous() for s0 in offs]
    do_seg = [dod[:, s0:s0 + l_s].contiguous() for s0 in offs]
    out = [torch.empty_like(t) for t in q_seg]
    dq = [torch.empty_like(t) for t in q_seg]
    lse = [torch.empty((w.B, w.H, l_s), dtype=torch.float32, device=dev) for _ in offs]
    rows_valid = [s0 + l_s if w.causal else w.l_x for s0 in offs]
    if args.projections:
        # Q, K and V are produced from x inside the step; the dK/dV partials of a segment are
        # consumed at once by the backward projection, so one pair of buffers serves all segments
        (xd, xb), (wqd, wqb), (wkvd, wkvb) = map(stage, synth.make_projection_inputs(w.B, w.l_x, w.H, w.d, w.seed, w.qkv_std))
        dk_one = torch.empty(kd.shape, dtype=torch.float32, device=dev)
        dv_one = torch.empty(kd.shape, dtype=torch.float32, device=dev)
        dx_q = [torch.empty((w.B, l_s, E), dtype=torch.float32, device=dev) for _ in offs]
        dx_part = [torch.empty((w.B, w.l_x, 1, E), dtype=torch.float32, device=dev) for _ in offs]
        dX = torch.empty((w.B, w.l_x, 1, E), dtype=torch.float32, device=dev)
        if args.weight_grads:
            dw_q = torch.empty((E, E), dtype=torch.float32, device=dev)
            dw_kv = torch.empty((E, 2 * E), dtype=torch.float32, device=dev)
            wg_scratch = torch.empty((max(16, lss.lss_project_bwd_weight_scratch_bytes(l_s, w.l_x, w.B, w.H, w.d)),),
                                     dtype=torch.uint8, device=dev)
    else:
        dk_part = [torch.empty(kd.shape, dtype=torch.float32, device=dev) for _ in offs]
        dv_part = [torch.empty(kd.shape, dtype=torch.float32, device=dev) for _ in offs]
        dK = torch.empty(kd.shape, dtype=torch.float32, device=dev)
        dV = torch.empty(kd.shape, dtype=torch.float32, device=dev)
    # The partials' only consumer here is the segment sum, which is told how many rows of each are valid: key
    # tiles no query of a segment sees need not be filled with zeros -- a flag of the call, off unless asked for
    skip = args.skip_masked_tail

    drop = {} if args.dropout is None else {"p_drop": args.dropout, "seed": w.seed}

    def step_attention():
        for i, s0 in enumerate(offs):
            lss.lss_segment_attn_fwd(q_seg[i], kd, vd, s0, w.causal, out=out[i], lse=lse[i], **drop)
            lss.lss_segment_attn_bwd(q_seg[i], kd, vd, s0, out[i], lse[i], do_seg[i], w.causal,
                                     dq=dq[i], dk_partial=dk_part[i], dv_partial=dv_part[i], skip_masked_tail=skip, **drop)
        lss.lss_reduce_partials(dk_part, rows_valid, out=dK)
        lss.lss_reduce_partials(dv_part, rows_valid, out=dV)

    def step_with_projections():
        for i, s0 in enumerate(offs):     # every segment projects K and V itself, as every GPU would
            lss.lss_project_qkv(xd, wqd, wkvd, s0, l_s, w.H, q_seg=q_seg[i], k=kd, v=vd)
            lss.lss_segment_attn_fwd(q_seg[i], kd, vd, s0, w.causal, out=out[i], lse=lse[i], **drop)
            lss.lss_segment_attn_bwd(q_seg[i], kd, vd, s0, out[i], lse[i], do_seg[i], w.causal,
                                     dq=dq[i], dk_partial=dk_one, dv_partial=dv_one, skip_masked_tail=skip, **drop)
            lss.lss_project_bwd(dq[i], dk_one, dv_one, wqd, wkvd, rows_valid[i], dx_q=dx_q[i],
                                dx_partial=dx_part[i].view(w.B, w.l_x, E), skip_masked_tail=skip)
            if args.weight_grads:
                lss.lss_project_bwd_weight(xd, dq[i], dk_one, dv_one, s0, rows_valid[i], dw_q=dw_q, dw_kv=dw_kv,
                                           scratch=wg_scratch)
        lss.lss_reduce_partials(dx_part, rows_valid, out=dX)

    step = step_with_projections if args.projections else step_attention

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    if min_timed_ms > 0:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        step()
        e1.record()
        torch.cuda.synchronize()
        est_ms = max(e0.elapsed_time(e1), 1e-3)
        more = int(min_warm_ms / est_ms)
        for _ in range(more):
            step()
        torch.cuda.synchronize()
        warmup += 1 + more
        steps = max(steps, int(min_timed_ms / est_ms) + 1)
    if args.calib_copy_mib > 0:
        src = torch.empty(args.calib_copy_mib << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)      # the calibration kernel: reads and writes calib_copy_mib MiB
        torch.cuda.synchronize()
        del src, dst

    use_events = not args.no_kernel_timing
    names = timing.kernel_names()

    def read_kernels(n_steps):
        out_ = {}
        for kid_, name_ in names.items():
            ms, n = timing.read(kid_)
            if n:
                out_[name_] = {"launches_per_step": n / n_steps, "avg_us": 1e3 * ms / n, "ms_per_step": ms / n_steps}
        return out_

    def timed_region():
        """`steps` steps between two events; returns (ms per step, per-step GPU times)."""
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps - 1)]    # step boundaries, for median and min
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record()
        for i_ in range(steps):
            step()
            if i_ < steps - 1:
                marks[i_].record()
        e1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        gpu_ms = e0.elapsed_time(e1)
        bounds = [e0] + marks + [e1]
        return max(wall_ms, gpu_ms) / steps, gpu_ms / steps, sorted(a_.elapsed_time(b_) for a_, b_ in zip(bounds, bounds[1:]))

    # 1. the timed region proper: the library's calls and nothing else
    timing.enable(False)
    ms_per_step, gpu_ms_per_step, per_step = timed_region()
    step_stats = {"median_ms": round(per_step[len(per_step) // 2], 4), "min_ms": round(per_step[0], 4),
                  "max_ms": round(per_step[-1], 4), "note": "GPU time between step boundaries inside the timed region"}

    # 1b. the same steps recorded once into a HIP graph and replayed (the library allocates nothing, records no
    # memset nodes and never synchronises, so a caller may do this): what a launch-bound configuration gains
    # from it.  Reported beside `value`, never as `value`.
    graph_replay = None
    if not args.no_graph:
        try:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                step()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                step()
            graph.replay()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(steps):
                graph.replay()
            e1.record()
            torch.cuda.synchronize()
            graph_replay = {"ms_per_step": round(e0.elapsed_time(e1) / steps, 4)}
            del graph
        except Exception as exc:       # reported, not fatal: the eager figures above stand on their own
            graph_replay = {"error": str(exc)[:200]}

    # 2. survey pass: every kernel bracketed by events, to find the one with the largest share of a step and to
    # report the others.  3. the timed region again, with that one kernel bracketed: its average launch duration
    # under the same back-to-back conditions, for the roofline.
    survey, dom, ms_per_step_events = {}, None, None
    if use_events:
        timing.reset()
        timing.enable(True)
        for _ in range(2):
            step()
        torch.cuda.synchronize()
        timing.enable(False)
        survey = read_kernels(2)
        cand = {n_: k_ for n_, k_ in survey.items() if n_ in ALGO_PRODUCTS}
        dom = max(cand, key=lambda n_: cand[n_]["ms_per_step"])
        timing.reset()
        timing.select([k_ for k_, n_ in names.items() if n_ == dom])
        ms_per_step_events, _, _ = timed_region()
        timing.enable(False)

    # unmasked (query, key) pairs x B x H: the whole sequence, or the listed segments
    pairs = w.pairs() if args.segments is None else sum(w.segment_pairs(i_) for i_ in seg_ids)
    flops_strict = 12.0 * pairs * w.d
    flops_fa = 14.0 * pairs * w.d
    # projections: 2 flops per multiply-add of Q_i, K, V and of dx_q, dx_partial (rows that hold data)
    proj_flops = {"proj_gemm_kernel:project_qkv": sum(2.0 * w.B * E * (2 * E * w.l_x + E * l_s) for _ in offs),
                  "proj_gemm_kernel:project_bwd": sum(2.0 * w.B * E * (2 * E * rv + E * l_s) for rv in rows_valid)}
    if args.projections and args.weight_grads:      # same products as the backward maps, contracted over rows instead
        proj_flops["wgrad_gemm_kernel"] = proj_flops["proj_gemm_kernel:project_bwd"]
    flops_proj = sum(proj_flops.values()) if args.projections else 0.0
    value = (flops_strict + flops_proj) / (ms_per_step * 1e-3) / 1e12

    kernels, roofline = {}, None
    if use_events:
        kernels = survey
        timed = read_kernels(steps)        # the dominant kernel, inside the second timed region
        kernels[dom] = dict(timed[dom], timed_region=True)
        per_launch = ALGO_PRODUCTS[dom] * 2.0 * w.d * pairs / timed[dom]["launches_per_step"]
        achieved = per_launch / (timed[dom]["avg_us"] * 1e-6) / 1e12
        roofline = {"kernel": dom, "bound": "mfma", "achieved": round(achieved, 2), "peak": peak,
                    "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
                    "traffic": measured_traffic(w.name, dom),
                    "avg_launch_us": round(timed[dom]["avg_us"], 2),
                    "algorithmic_flops_per_launch": per_launch,
                    "executed_over_algorithmic": EXEC_PRODUCTS[dom] / ALGO_PRODUCTS[dom],
                    "ms_per_step_with_events": round(ms_per_step_events, 4)}
        # Algorithmic bytes of that kernel per launch (averaged over the segments run): every operand read
        # once, every result written once.  Below the machine's balance point the launch is bound by
        # memory, and the roofline is reported against the HBM peak instead.
        eb, bh = (4 if f32 else 2), w.B * w.H
        def alg_bytes(kv):
            if dom in ("fwd_kernel", "fwd_bf16_kernel"):
                return bh * (eb * w.d * (2 * l_s + 2 * kv) + 4 * l_s)
            return bh * (eb * w.d * (4 * l_s + 2 * kv) + 8 * l_s + 8 * w.d * kv)    # backward: also the fp32 partials
        if dom in ("fwd_kernel", "fwd_bf16_kernel", "bwd_main_bf16_kernel"):
            byts = sum(alg_bytes(rv) for rv in rows_valid) / len(rows_valid)
            roofline["algorithmic_bytes_per_launch"] = byts
            roofline["flop_per_byte"] = round(per_launch / byts, 1)
            if per_launch / byts < peak * 1e12 / (PEAK_HBM_GBS * 1e9):
                gbs = byts / (timed[dom]["avg_us"] * 1e-6) / 1e9
                roofline.update({"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                 "frac": round(gbs / PEAK_HBM_GBS, 4), "achieved_tflops": round(achieved, 2)})
        for name, kk in kernels.items():
            if name in ALGO_PRODUCTS:
                kk["algorithmic_tflops"] = round(ALGO_PRODUCTS[name] * 2.0 * w.d * pairs / (kk["ms_per_step"] * 1e-3) / 1e12, 2)
            if name in proj_flops:
                kk["algorithmic_tflops"] = round(proj_flops[name] / (kk["ms_per_step"] * 1e-3) / 1e12, 2)
            kk["avg_us"] = round(kk["avg_us"], 2)
            kk["ms_per_step"] = round(kk["ms_per_step"], 4)
        if "reduce_partials_kernel" in kernels and not (args.projections and args.weight_grads):   # (there it also adds row chunks)
            # algorithmic bytes of the segment sum: valid rows of every part read once, l_x rows written
            row_bytes = w.B * w.H * w.d * 4
            byts = (1 if args.projections else 2) * (sum(rows_valid) + w.l_x) * row_bytes
            kernels["reduce_partials_kernel"]["algorithmic_GBps"] = round(
                byts / (kernels["reduce_partials_kernel"]["ms_per_step"] * 1e-3) / 1e9, 1)

    # forward-only and backward-only rates from the survey pass (kernel times, launch gaps not included)
    rates = None
    if kernels:
        t_f = sum(kernels[n_]["ms_per_step"] for n_ in FWD_KERNELS if n_ in kernels)
        t_b = sum(kernels[n_]["ms_per_step"] for n_ in BWD_KERNELS if n_ in kernels)
        if t_f > 0 and t_b > 0:
            rates = {"fwd_only_tflops": round(4.0 * pairs * w.d / (t_f * 1e-3) / 1e12, 2),
                     "bwd_only_tflops": round(8.0 * pairs * w.d / (t_b * 1e-3) / 1e12, 2),
                     "note": "strict counts 4*P*d and 8*P*d over the summed kernel times of one step"}

    cpu_baseline = None
    if with_cpu_baseline:
        import oracle
        # A bounded sample of the same workload: about 1e12 fp64 flops (10-30 s on the machine's cores).  The
        # whole workload if it is that small; otherwise the middle and the last segment, and of those
        # only some (batch, head) slices, (0, 0) and (B-1, H-1) among them -- heads are independent, so a
        # slice is a complete, smaller problem of the same shape.  (With projections the slices cannot be cut
        # out of x, so the sample is then whole segments.)
        budget = 1.0e12
        seg_flops = {i: 12.0 * w.segment_pairs(i) * w.d for i in seg_ids}
        if sum(seg_flops.values()) <= budget:
            sample, slices = list(seg_ids), None
        else:
            sample = sorted({seg_ids[max(len(seg_ids) // 2 - 1, 0)], seg_ids[-1]})
            slices = None
            if not args.projections and sum(seg_flops[i] for i in sample) > budget:
                # (0, 0), (B-1, H-1) and as many evenly spaced (batch, head) pairs as the budget allows
                bh = w.B * w.H
                n_sl = int(min(bh, max(2, budget // (sum(seg_flops[i] for i in sample) / bh))))
                picks = sorted({round(j_ * (bh - 1) / (n_sl - 1)) for j_ in range(n_sl)})
                slices = [(x_ // w.H, x_ % w.H) for x_ in picks]
        kh, vh = kb.f64(), vb.f64()
        if args.projections:
            xh, wqh, wkvh = (b_.f64() for b_ in (xb, wqb, wkvb))
        t_cpu, flops_cpu = 0.0, 0.0

        def oracle_segment(qh, kh_, vh_, doh, s0):
            if args.dropout is None:
                oracle.segment_fwd(qh, kh_, vh_, s0, w.causal)
                return oracle.segment_bwd(qh, kh_, vh_, doh, s0, w.causal)
            oracle.segment_fwd_dropout(qh, kh_, vh_, s0, w.causal, args.dropout, w.seed)
            return oracle.segment_bwd_dropout(qh, kh_, vh_, doh, s0, w.causal, args.dropout, w.seed)

        for i in sample:
            s0 = w.offsets()[i]
            qh, doh = qb[:, s0:s0 + l_s].f64(), dob[:, s0:s0 + l_s].f64()
            if slices is None:
                t = time.perf_counter()
                if args.projections:
                    qh, kh, vh = oracle.project_qkv(xh, wqh, wkvh, s0, l_s, w.H)
                g_ = oracle_segment(qh, kh, vh, doh, s0)
                if args.projections:
                    oracle.project_bwd(g_[0], g_[1], g_[2], wqh, wkvh)
                    flops_cpu += 2.0 * w.B * E * (2 * E * w.l_x + E * l_s) + 2.0 * w.B * E * (2 * E * rows_valid[seg_ids.index(i)] + E * l_s)
                t_cpu += time.perf_counter() - t
                flops_cpu += seg_flops[i]
            else:
                for (b_, h_) in slices:
                    cut = [np.ascontiguousarray(a[b_:b_ + 1, :, h_:h_ + 1]) for a in (qh, kh, vh, doh)]
                    t = time.perf_counter()
                    oracle_segment(cut[0], cut[1], cut[2], cut[3], s0)
                    t_cpu += time.perf_counter() - t
                    flops_cpu += seg_flops[i] / (w.B * w.H)
        what = "all batches and heads" if slices is None else f"(batch, head) slices {slices}"
        cpu_baseline = {"value": round(flops_cpu / t_cpu / 1e12, 6), "unit": "TFLOP/s",
                        "cores": oracle.threads(), "kind": "oracle",
                        "whole_step_extrapolated_s": round((flops_strict + flops_proj) / (flops_cpu / t_cpu), 1),
                        "sample": f"segments {sample} of {w.N} (fwd+bwd, {what}), "
                                  f"{t_cpu:.1f} s of fp64 CPU work, same strict flop count"}

    return {
        "metric": "segment-attention fwd+bwd TFLOP/s on 1 MI355X; % of bf16 MFMA peak",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": w.name + ("+projections" if args.projections else "")
                               + ("+weight-grads" if args.projections and args.weight_grads else "")
                               + (f"+dropout{args.dropout}" if args.dropout is not None else "")
                               + ("+f32" if f32 else "")
                               + (f"+segments{seg_ids}" if args.segments is not None else ""), "B": w.B, "l_x": w.l_x,
                   "N": w.N, "l_s": l_s, "H": w.H, "d": w.d, "causal": w.causal,
                   "step": ("per segment: Q_i, K, V from x, fwd, bwd, dx_q and dx_partial; then segment sum of dx"
                            if args.projections else
                            "fwd+bwd of the listed segments, then the sum of their dK and dV partials" if args.segments is not None
                            else "fwd+bwd of all N segments, then segment sum of dK and dV"),
                   "partials_contract": ("every row of the partials written (lss_segment_attn_bwd)" if not args.skip_masked_tail else
                                         "LSS_FLAG_SKIP_MASKED_TAIL: key tiles no query of a causal segment sees stay unwritten; "
                                         "the segment sum is given rows_valid")},
        ("frac_of_f32_peak" if f32 else "frac_of_bf16_peak"): round(value / peak, 4),
        "tflops_with_recompute_count_14Pd": round(flops_fa / (ms_per_step * 1e-3) / 1e12, 2),
        "gpu_ms_per_step_events": round(gpu_ms_per_step, 4), "step_stats": step_stats,
        "graph_replay": (None if graph_replay is None else graph_replay if "error" in graph_replay else
                         dict(graph_replay, value=round((flops_strict + flops_proj) / (graph_replay["ms_per_step"] * 1e-3) / 1e12, 2),
                              note="the same steps replayed from one HIP graph; not `value`")),
        "roofline": roofline, "cpu_baseline": cpu_baseline, "rates": rates, "kernels": kernels,
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=None,
                    help="one of synth.WORKLOADS; default lx24k, and then the other configurations are reported in `extra`")
    ap.add_argument("--projections", action="store_true",
                    help="also run the Q/K/V projections and their backward around every segment")
    ap.add_argument("--weight-grads", action="store_true",
                    help="with --projections: every segment also computes its share of dW_q and dW_kv")
    ap.add_argument("--dtype", choices=["bf16", "f32"], default="bf16",
                    help="storage type: bf16 (the benchmark) or f32 (the single-precision twins of the entry points)")
    ap.add_argument("--dropout", type=float, default=None, metavar="P",
                    help="run forward and backward with dropout probability P on the attention weights")
    ap.add_argument("--layer-ops", action="store_true",
                    help="a separate workload: the segment-local remainder of a layer (positional-embedding rows, "
                         "layer normalisation, feed-forward unit), forward and backward, for every segment")
    ap.add_argument("--fused-gelu", action="store_true",
                    help="with --layer-ops: use the GEMM entry points that apply GeLU and its derivative in their epilogues")
    ap.add_argument("--segments", default=None, metavar="I,J,...",
                    help="run only these segments of the workload (for workloads whose N segments' partials do not "
                         "fit in memory at once, e.g. lx50k_skinny); the segment sum then adds these segments' partials")
    ap.add_argument("--skip-masked-tail", action="store_true",
                    help="backward calls pass LSS_FLAG_SKIP_MASKED_TAIL: key tiles no query of a causal segment sees stay unwritten")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay of the step (`graph_replay`)")
    ap.add_argument("--no-extra", action="store_true", help="leave out the other configurations' figures")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="before the timed region, run one plain device-to-device copy of this many MiB "
                         "(a kernel of known traffic, to calibrate rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--no-kernel-timing", action="store_true",
                    help="no survey pass and no second, event-bracketed timed region (roofline becomes null)")
    args = ap.parse_args()

    if args.gpus != 1:
        print(f"bench.py: this build is one GPU's share of the path; --gpus {args.gpus} is not supported "
              "(no collectives, no second GPU). Run with --gpus 1.", file=sys.stderr)
        return 2

    import torch

    from paper_2311_02382_amd import lss, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    lss.load()      # fails loudly if the HIP library has not been built
    torch.cuda.set_device(0)

    headline = args.workload is None
    w = synth.WORKLOADS[args.workload or "lx24k"]
    if args.layer_ops:
        return layer_ops(args, w)
    if args.dtype == "f32" and args.projections:
        print("bench.py: the projections are bf16 only; --dtype f32 cannot be combined with --projections", file=sys.stderr)
        return 2
    if args.segments is not None and args.projections:
        print("bench.py: --segments cannot be combined with --projections", file=sys.stderr)
        return 2

    line = attention(args, w, args.steps, args.warmup, not args.no_cpu_baseline)
    plain = not (args.projections or args.dropout is not None or args.segments is not None or args.dtype == "f32")
    if headline and plain and not args.no_extra:
        # the other configurations, same step, same timing, a few steps each
        extra = []
        for name in ("tiny", "lx8k", "lx32k_d128", "lx50k"):
            torch.cuda.empty_cache()
            e = attention(args, synth.WORKLOADS[name], min(args.steps, 5), min(args.warmup, 2), False,
                          min_warm_ms=30.0, min_timed_ms=50.0)
            extra.append({"workload": name, "value": e["value"], "unit": e["unit"], "ms_per_step": e["ms_per_step"],
                          "graph_replay": e["graph_replay"], "steps": e["steps"], "warmup": e["warmup"], "frac_of_bf16_peak": e["frac_of_bf16_peak"],
                          "config": {k_: e["config"][k_] for k_ in ("B", "l_x", "N", "l_s", "H", "d", "causal")},
                          "roofline": e["roofline"], "rates": e["rates"]})
        line["extra"] = extra
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())

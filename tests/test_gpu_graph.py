"""A whole step -- forward and backward of every segment, then the segment sum -- recorded once into a
HIP graph and replayed.

The library allocates nothing, clears nothing with memset nodes and never synchronises, so its calls can be
captured.  Every replay, with new input values in the same buffers and eager work of the process between the
replays, must give the eager calls' results bit for bit (the kernels' reductions have a fixed order)."""
import pytest
import torch

from paper_2311_02382_amd import lss, synth

pytestmark = pytest.mark.gpu

B, L_X, H, D, N = 1, 2112, 2, 64, 4          # segments of 528 rows: ragged tiles, key splits in the later ones
L_S = L_X // N


def _step(q, k, v, do, out, lse, dq, dk_parts, dv_parts, dk, dv, ws):
    for i in range(N):
        s0 = i * L_S
        lss.lss_segment_attn_fwd(q[i], k, v, s0, True, out=out[i], lse=lse[i], workspace=ws)
        lss.lss_segment_attn_bwd(q[i], k, v, s0, out[i], lse[i], do[i], True, dq=dq[i], dk_partial=dk_parts[i],
                                 dv_partial=dv_parts[i], skip_masked_tail=True, workspace=ws)
    valid = [(i + 1) * L_S for i in range(N)]
    lss.lss_reduce_partials(dk_parts, valid, out=dk)
    lss.lss_reduce_partials(dv_parts, valid, out=dv)


def _buffers():
    dev = "cuda"
    seg = lambda dt: [torch.empty((B, L_S, H, D), dtype=dt, device=dev) for _ in range(N)]
    full = lambda: torch.empty((B, L_X, H, D), dtype=torch.float32, device=dev)
    return dict(q=seg(torch.bfloat16), k=torch.empty((B, L_X, H, D), dtype=torch.bfloat16, device=dev),
                v=torch.empty((B, L_X, H, D), dtype=torch.bfloat16, device=dev), do=seg(torch.bfloat16),
                out=seg(torch.bfloat16), lse=[torch.empty((B, H, L_S), dtype=torch.float32, device=dev) for _ in range(N)],
                dq=seg(torch.bfloat16), dk_parts=[full() for _ in range(N)], dv_parts=[full() for _ in range(N)],
                dk=full(), dv=full(),
                ws=torch.empty(lss.lss_workspace_bytes(L_S, L_X, B, H, D, 2), dtype=torch.uint8, device=dev))


def _load_inputs(buf, seed):
    q, k, v, do = (torch.from_numpy(a).to(torch.bfloat16).cuda() for a in synth.make_inputs(B, L_X, H, D, seed=seed))
    buf["k"].copy_(k)
    buf["v"].copy_(v)
    for i in range(N):
        buf["q"][i].copy_(q[:, i * L_S:(i + 1) * L_S])
        buf["do"][i].copy_(do[:, i * L_S:(i + 1) * L_S])


RESULTS = ("out", "lse", "dq", "dk", "dv")


def _results(buf):
    return {n: [t.clone() for t in buf[n]] if isinstance(buf[n], list) else buf[n].clone() for n in RESULTS}


def _bits(t):
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32)


def test_a_captured_step_replays_to_the_eager_results():
    eager, graphed = _buffers(), _buffers()
    _load_inputs(graphed, seed=100)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):           # one eager pass on a side stream before the capture
        _step(**graphed)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        _step(**graphed)
    for rep, seed in enumerate((101, 102, 103)):
        _load_inputs(eager, seed)
        _load_inputs(graphed, seed)
        for n in RESULTS + ("dk_parts", "dv_parts"):     # stale results must not survive a replay
            for t in (graphed[n] if isinstance(graphed[n], list) else [graphed[n]]):
                t.fill_(3.0)
        graph.replay()
        _step(**eager)                      # the process's own eager work, same library, between the replays
        torch.cuda.synchronize()
        want, got = _results(eager), _results(graphed)
        for n in RESULTS:
            pairs = zip(got[n], want[n]) if isinstance(got[n], list) else [(got[n], want[n])]
            for i, (a, b) in enumerate(pairs):
                assert torch.equal(_bits(a), _bits(b)), f"replay {rep}: {n}[{i}] differs from the eager call"

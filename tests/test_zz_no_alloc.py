"""The entry point that allocates nothing (lss_segment_attn_bwd_noalloc) against lss_segment_attn_bwd.

Same kernels, scratch in the library's built-in device buffer instead of the caller's workspace: the results
must be identical bit for bit.  Two calls in a row, the second on a smaller input (the buffer keeps the first
call's contents), a shape whose forward scratch would not fit (the backward's does), then a shape the buffer
cannot hold."""
import pytest
import torch

from paper_2311_02382_amd import lss, synth
from _util import Staged

pytestmark = pytest.mark.gpu


def _run(B, l_x, H, d, s0, l_s, causal, seed):
    q, k, v, do = (Staged(a, "bf16") for a in synth.make_inputs(B, l_x, H, d, seed=seed))
    q_seg, do_seg = q.dev[:, s0:s0 + l_s].contiguous(), do.dev[:, s0:s0 + l_s].contiguous()
    out, lse = lss.lss_segment_attn_fwd(q_seg, k.dev, v.dev, s0, causal)
    ref = lss.lss_segment_attn_bwd(q_seg, k.dev, v.dev, s0, out, lse, do_seg, causal)
    got = (torch.full_like(q_seg, 3.0), torch.full(k.dev.shape, 3.0, dtype=torch.float32, device="cuda"),
           torch.full(k.dev.shape, 3.0, dtype=torch.float32, device="cuda"))
    lss.lss_set_workspace(None)         # the call must not depend on a registered workspace
    lss.lss_segment_attn_bwd_noalloc(q_seg, k.dev, v.dev, s0, out, lse, do_seg, causal, *got)
    torch.cuda.synchronize()
    for name, a, b in zip(("dq", "dk_partial", "dv_partial"), got, ref):
        assert torch.equal(a.view(torch.int16 if a.dtype == torch.bfloat16 else torch.int32),
                           b.view(torch.int16 if b.dtype == torch.bfloat16 else torch.int32)), name


def test_noalloc_backward_equals_the_workspace_one_on_two_calls_in_a_row():
    # first call: key splits in the dQ workgroups (split partial dQ in the scratch) and a ragged tail
    _run(B=1, l_x=9000, H=2, d=64, s0=8400, l_s=600, causal=True, seed=41)
    # second call, smaller, other head width, non-causal: the buffer still holds the first call's values
    _run(B=2, l_x=700, H=1, d=128, s0=100, l_s=77, causal=False, seed=42)
    _run(B=1, l_x=1024, H=4, d=64, s0=768, l_s=256, causal=True, seed=0)


def test_noalloc_backward_needs_room_for_the_backward_scratch_only():
    # few query tiles and a long sequence: the forward's split partial results alone exceed the buffer,
    # the backward's scratch (start values and 4 partial dQ) does not
    B, l_x, H, d, l_s = 1, 16384, 16, 128, 1024
    assert lss.lss_workspace_bytes(l_s, l_x, B, H, d, 2) > lss.LSS_NOALLOC_SCRATCH_BYTES
    _run(B=B, l_x=l_x, H=H, d=d, s0=l_x - l_s, l_s=l_s, causal=True, seed=43)


def test_noalloc_backward_rejects_what_the_buffer_cannot_hold():
    B, l_s, l_x, H, d = 8, 32768, 32768, 32, 64     # 12 bytes of backward scratch per query row and head: 96 MiB
    assert 12 * B * H * l_s > lss.LSS_NOALLOC_SCRATCH_BYTES
    lib = lss.load()
    rc = lib.lss_segment_attn_bwd_noalloc(0x1000, 0x2000, 0x3000, 0, l_s, l_x, B, H, d, 1, 0x4000, 0x5000, 0x6000,
                                          0x7000, 0x8000, 0x9000, None)
    assert rc == -6 and "built-in buffer" in lss.lss_last_error()

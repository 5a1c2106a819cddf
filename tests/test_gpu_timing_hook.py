"""thk_profile_next: the next call's main kernel is launched with the caller's two events attached;
their interval is that kernel's duration, the result of the call is unchanged, and the pair is
used once."""
import pytest
import torch

import paper_2407_21018_amd as thk
from helpers import ws_tensor

pytestmark = pytest.mark.gpu
D = 128


def _recorded_event():
    e = torch.cuda.Event(enable_timing=True)
    e.record()      # torch creates the HIP event on first record
    return e


def test_timed_launch_gives_the_kernel_duration_and_the_same_result():
    U, S, T = 16, 8192, 76
    g = torch.Generator(device="cuda"); g.manual_seed(5)
    kp = torch.randn(U, S, T, generator=g, device="cuda").to(torch.bfloat16)
    v = torch.randn(U, S, D, generator=g, device="cuda").to(torch.bfloat16)
    q = torch.randn(U, D, generator=g, device="cuda").to(torch.bfloat16)
    idx = torch.sort(torch.rand(U, D, generator=g, device="cuda").argsort(dim=1)[:, :T], dim=1).values.to(torch.int16).contiguous()
    shape = thk.make_shape(1, 1, U, U, D, S, 1, T, 0, thk.THK_BF16, 0)
    ws = ws_tensor(thk.thk_workspace_bytes(shape, thk.THK_OP_DECODE))
    plain = torch.empty_like(q); timed = torch.empty_like(q); after = torch.empty_like(q)
    thk.thk_decode_attn(shape, q, kp, idx, v, None, None, 0, 0, plain, ws)
    torch.cuda.synchronize()

    e0, e1 = _recorded_event(), _recorded_event()
    w0, w1 = _recorded_event(), _recorded_event()
    torch.cuda.synchronize()
    thk.thk_profile_next(e0, e1)
    w0.record()
    thk.thk_decode_attn(shape, q, kp, idx, v, None, None, 0, 0, timed, ws)
    w1.record()
    thk.thk_decode_attn(shape, q, kp, idx, v, None, None, 0, 0, after, ws)   # the pair is spent: a plain launch
    torch.cuda.synchronize()
    kernel_ms, call_ms = e0.elapsed_time(e1), w0.elapsed_time(w1)
    print(f"kernel {kernel_ms * 1e3:.1f} us inside a call of {call_ms * 1e3:.1f} us", flush=True)
    assert 0.0 < kernel_ms <= call_ms          # the call also holds the merge launch and the gaps
    assert kernel_ms * 1e3 > U * S * (T + D) * 2 / 8e6   # not faster than the HBM peak allows (bytes / 8 TB/s, in us)
    assert torch.equal(timed, plain) and torch.equal(after, plain)

    # a cancelled pair is not used: its two events keep the records they had
    c0, c1 = _recorded_event(), _recorded_event()
    torch.cuda.synchronize()
    before = c0.elapsed_time(c1)
    thk.thk_profile_next(c0, c1)
    thk.thk_profile_next(None, None)
    thk.thk_decode_attn(shape, q, kp, idx, v, None, None, 0, 0, after, ws)
    torch.cuda.synchronize()
    assert torch.equal(after, plain)
    assert c0.elapsed_time(c1) == before

"""thk_decode_attn_static -- the entry point for callers that cannot allocate -- against
thk_decode_attn, through the C ABI: same kernels, same split, so the outputs must agree bit for
bit (which is inside the attention bars of the parity tests).  Two calls in a row share the
library's static device buffer, the second with a smaller input: nothing a call leaves behind
there may reach the next one."""
import pytest
import torch

import paper_2407_21018_amd as thk
from oracle import oracle as O
from paper_2407_21018_amd.synth import as_numpy
from helpers import ATTN_TOL, attn_rel_err, ws_tensor

pytestmark = pytest.mark.gpu
D = 128


def _case(dtype, B, N_kv, G, S, T, n_split, s_tail, cap, seed):
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    g = torch.Generator(device="cuda"); g.manual_seed(seed)
    U, H = B * N_kv, B * N_kv * G
    q = torch.randn(H, D, generator=g, device="cuda").to(tdt)
    kp = torch.randn(U, S, T, generator=g, device="cuda").to(tdt)
    v = torch.randn(U, S, D, generator=g, device="cuda").to(tdt)
    idx = torch.stack([torch.sort(torch.randperm(D, generator=g, device="cuda")[:T]).values for _ in range(U)]).to(torch.int16)
    kt = torch.randn(U, max(cap, 1), D, generator=g, device="cuda").to(tdt)
    vt = torch.randn(U, max(cap, 1), D, generator=g, device="cuda").to(tdt)
    shape = thk.make_shape(1, B, G * N_kv, N_kv, D, S, 1, T, 0, thk.THK_BF16 if dtype == "bf16" else thk.THK_F32, n_split)
    return shape, q, kp, idx, v, kt, vt, s_tail, cap


CASES = [
    # (dtype, B, N_kv, G, S, T, n_split, s_tail, cap): the larger call first, then smaller ones
    [("bf16", 2, 4, 1, 4100, 76, 8, 5, 8), ("bf16", 1, 2, 1, 700, 76, 3, 0, 0)],
    [("bf16", 2, 2, 4, 3000, 64, 6, 17, 32), ("bf16", 1, 1, 4, 513, 64, 2, 1, 32)],
    [("f32", 1, 8, 1, 2048, 64, 0, 0, 0), ("f32", 1, 3, 2, 300, 51, 2, 3, 4)],
]


@pytest.mark.parametrize("pair", CASES, ids=["bf16-g1", "bf16-g4-mfma", "f32"])
def test_static_scratch_decode_matches_workspace_decode(pair, decode_merge):
    for n, c in enumerate(pair):
        print(f"static decode case {c}", flush=True)
        shape, q, kp, idx, v, kt, vt, s_tail, cap = _case(*c, seed=4200 + n)
        assert thk.thk_default_split(shape, thk.THK_OP_DECODE) > 1 or shape.n_split > 1   # the scratch is in use
        want = torch.empty_like(q)
        ws = ws_tensor(thk.thk_workspace_bytes(shape, thk.THK_OP_DECODE))
        thk.thk_decode_attn(shape, q, kp, idx, v, kt if cap else None, vt if cap else None, s_tail, cap, want, ws)
        got = torch.full_like(q, float("nan"))
        thk.thk_decode_attn_static(shape, q, kp, idx, v, kt if cap else None, vt if cap else None, s_tail, cap, got)
        torch.cuda.synchronize()
        assert torch.equal(got.view(torch.uint8), want.view(torch.uint8)), c
        # ... and both sit inside the oracle's bar
        dtype, B, N_kv, G, S, T = c[:6]
        ref = O.decode_attn(as_numpy(q).reshape(B, N_kv * G, D), as_numpy(kp).reshape(B, N_kv, S, T),
                            idx.cpu().numpy().reshape(B, N_kv, T), as_numpy(v).reshape(B, N_kv, S, D), dtype,
                            as_numpy(kt).reshape(B, N_kv, -1, D) if cap else None,
                            as_numpy(vt).reshape(B, N_kv, -1, D) if cap else None, s_tail)
        assert attn_rel_err(got, ref.reshape(-1, D)).max() <= ATTN_TOL[dtype]


def test_static_scratch_rejects_oversized_shapes():
    """A shape whose split partials exceed the static buffer is refused before anything is
    enqueued (fake, never dereferenced addresses)."""
    A = 4096
    shape = thk.make_shape(1, 64, 64, 64, D, 1 << 20, 1, 64, 0, thk.THK_BF16, 64)
    assert thk.thk_workspace_bytes(shape, thk.THK_OP_DECODE) > (8 << 20)
    with pytest.raises(thk.ThkError) as e:
        thk.thk_decode_attn_static(shape, A, A, A, A, None, None, 0, 0, A, stream=0)
    assert e.value.status == 7

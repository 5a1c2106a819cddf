"""The library allocates nothing, never synchronises and records no memset, so a caller can
capture the whole path (prune, tail append, decode + split merge) in a HIP graph.  The graph
is replayed several times with eager work and synchronisations in between, and every replay
must reproduce the eager result bit for bit."""
import pytest
import torch

import paper_2407_21018_amd as thk
from helpers import TDT, ws_tensor

pytestmark = pytest.mark.gpu
D = 128


def _randn(shape, seed, sigma=1.0):
    g = torch.Generator(device="cuda"); g.manual_seed(seed)
    x = torch.randn(*shape, generator=g, device="cuda")
    if sigma:
        x = x * torch.exp(sigma * torch.randn(shape[-1], generator=g, device="cuda"))
    return x.to(torch.bfloat16)


@pytest.mark.parametrize("G,T", [(2, 76), (4, 76), (8, 128)])   # general kernel; matrix-core kernel, 4 and 8 heads per block
def test_prune_and_decode_replay_from_a_graph(G, T, prune_launch, decode_merge):
    L, B, N_kv, S, S_obs, cap = 2, 2, 4, 2048, 32, 8
    N_q, U = N_kv * G, B * N_kv
    q_obs = _randn((L, B, N_q, S_obs, D), 1); k = _randn((L, B, N_kv, S, D), 2); v = _randn((L, B, N_kv, S, D), 3, 0)
    q = _randn((L, B, N_q, D), 4); k_new = _randn((L, U, D), 5); v_new = _randn((L, U, D), 6, 0)
    shape_all = thk.make_shape(L, B, N_q, N_kv, D, S, S_obs, T, 0, thk.THK_BF16, 0)
    shape_1 = thk.make_shape(1, B, N_q, N_kv, D, S, S_obs, T, 0, thk.THK_BF16, 4)
    score = torch.empty(L * U, D, dtype=torch.float32, device="cuda")
    idx = torch.empty(L * U, T, dtype=torch.int16, device="cuda")
    kp = torch.empty(L, U, S, T, dtype=torch.bfloat16, device="cuda")
    kt = torch.zeros(L, U, cap, D, dtype=torch.bfloat16, device="cuda"); vt = torch.zeros_like(kt)
    out = torch.empty(L, B * N_q, D, dtype=torch.bfloat16, device="cuda")
    ws = ws_tensor(max(thk.thk_workspace_bytes(shape_all, thk.THK_OP_PRUNE),
                       thk.thk_workspace_bytes(shape_1, thk.THK_OP_DECODE)))

    def path():
        thk.thk_prune(shape_all, q_obs, k, score, idx, kp, ws)
        for l in range(L):
            thk.thk_tail_append(shape_1, k_new[l], v_new[l], kt[l], vt[l], 0, cap)
            thk.thk_decode_attn(shape_1, q[l], kp[l], idx[l * U:(l + 1) * U], v[l], kt[l], vt[l], 1, cap, out[l], ws)

    path()
    torch.cuda.synchronize()
    want = (score.clone(), idx.clone(), kp.clone(), out.clone())

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        path()                      # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        path()
    for rep in range(4):
        for t in (score, idx, kp, out):
            t.zero_()               # eager work between replays; also wipes the outputs
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (score, idx, kp, out)
        for a, b in zip(got, want):
            assert torch.equal(a, b), f"replay {rep} differs from the eager result"

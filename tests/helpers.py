"""Shared helpers of the GPU parity tests: run the C-ABI path on torch tensors
and compare with the CPU oracle.  Nothing here computes the method."""
import numpy as np
import torch

import paper_2407_21018_amd as thk
from oracle import oracle as O
from paper_2407_21018_amd.synth import as_numpy

DT = {"f32": thk.THK_F32, "bf16": thk.THK_BF16}
TDT = {"f32": torch.float32, "bf16": torch.bfloat16}
ATTN_TOL = {"f32": 1e-4, "bf16": 2e-2}     # max relative error per output vector
SCORE_TOL = 5e-7                            # relative; fp32 rounding of an fp64-merged score
TIE_TOL = 1e-6                              # oracle scores closer than this may swap


def ws_tensor(nbytes, device="cuda"):
    return torch.empty(max(16, nbytes), dtype=torch.uint8, device=device)


def gpu_score(shape, q_obs, k):
    U = shape.L * shape.B * shape.N_kv
    score = torch.empty(U, shape.D, dtype=torch.float32, device=k.device)
    ws = ws_tensor(thk.thk_workspace_bytes(shape, thk.THK_OP_SCORE))
    thk.thk_score(shape, q_obs, k, score, ws)
    torch.cuda.synchronize()
    return score


def gpu_select(shape, score):
    U = shape.L * shape.B * shape.N_kv
    idx = torch.full((U, shape.T), -1, dtype=torch.int16, device=score.device)
    thk.thk_select_topk(shape, score, idx)
    torch.cuda.synchronize()
    return idx


def gpu_compact(shape, k, idx, fill=0):
    U = shape.L * shape.B * shape.N_kv
    ld = shape.ld_keep or shape.T
    kp = torch.zeros(U, shape.S, ld, dtype=k.dtype, device=k.device)
    if fill:
        kp.fill_(fill)
    thk.thk_compact_keys(shape, k, idx, kp)
    torch.cuda.synchronize()
    return kp


def gpu_prune(shape, q_obs, k):
    U = shape.L * shape.B * shape.N_kv
    ld = shape.ld_keep or shape.T
    score = torch.empty(U, shape.D, dtype=torch.float32, device=k.device)
    idx = torch.full((U, shape.T), -1, dtype=torch.int16, device=k.device)
    kp = torch.zeros(U, shape.S, ld, dtype=k.dtype, device=k.device)
    ws = ws_tensor(thk.thk_workspace_bytes(shape, thk.THK_OP_PRUNE))
    thk.thk_prune(shape, q_obs, k, score, idx, kp, ws)
    torch.cuda.synchronize()
    return score, idx, kp


def gpu_decode(shape, q, kp, idx, v, k_tail=None, v_tail=None, s_tail=0, cap=0):
    out = torch.empty(shape.L * shape.B * shape.N_q, shape.D, dtype=q.dtype, device=q.device)
    ws = ws_tensor(thk.thk_workspace_bytes(shape, thk.THK_OP_DECODE))
    thk.thk_decode_attn(shape, q, kp, idx, v, k_tail, v_tail, s_tail, cap, out, ws)
    torch.cuda.synchronize()
    return out


def attn_rel_err(out, ref):
    """Per output vector: max |out - ref| / max |ref| (ref float64 [heads, D])."""
    o = out.detach().cpu().to(torch.float64).numpy().reshape(ref.shape)
    return np.abs(o - ref).max(axis=-1) / np.abs(ref).max(axis=-1)


def check_idx_with_tie_rule(gpu_idx, ora_idx, ora_score, T):
    """Index lists must agree except where the oracle's own scores tie: every
    channel in the symmetric difference must score within TIE_TOL (relative) of
    the oracle's T-th largest score.  Returns the units that differ."""
    gpu_idx = np.asarray(gpu_idx).reshape(-1, T)
    ora_idx = np.asarray(ora_idx).reshape(-1, T)
    sc = np.asarray(ora_score, np.float64).reshape(gpu_idx.shape[0], -1)
    differing = []
    for u in np.flatnonzero((gpu_idx != ora_idx).any(axis=1)):
        g, o = set(gpu_idx[u].tolist()), set(ora_idx[u].tolist())
        assert len(g) == T and all(0 <= c < sc.shape[1] for c in g), f"unit {u}: invalid index list"
        assert list(gpu_idx[u]) == sorted(g), f"unit {u}: not ascending"
        kth = np.sort(sc[u])[::-1][T - 1]
        for c in g ^ o:
            assert abs(sc[u, c] - kth) <= TIE_TOL * kth, \
                f"unit {u}: channel {c} score {sc[u, c]} vs T-th {kth} is not a tie"
        differing.append(int(u))
    return differing


def oracle_prune(q_obs, k, dtype, T, ld_keep=0):
    qn, kn = as_numpy(q_obs), as_numpy(k)
    sc = O.score(qn, kn, dtype)
    idx = O.select_topk(sc, T)
    kp = O.compact_keys(kn, idx, dtype, ld_keep)
    return sc, idx, kp

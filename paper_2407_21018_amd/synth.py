"""Seeded synthetic inputs shaped like the paper's workloads.

This module holds no arithmetic of the method: it only draws tensors.  Base
values are N(0,1); key and query channels carry a log-normal per-(layer, head,
channel) scale shared by all tokens and batch rows, mimicking the persistent
outlier channels of real key caches (Sec. 2, "Magnitudes of KV cache
channels"); values are left unscaled.  bf16 configs are rounded once here, so
the GPU path and the CPU oracle see identical bits.
"""
import torch

SEED0 = 20240721

# name -> shape of one of the five workloads (per layer)
CONFIGS = {
    1: dict(L=1, B=1, N_q=8, N_kv=8, D=128, S=2048, S_obs=32, lam=0.5, dtype="f32", sigma=1.0,
            steps=1, tail_cap=0),
    2: dict(L=32, B=4, N_q=32, N_kv=32, D=128, S=4096, S_obs=32, lam=0.4, dtype="bf16", sigma=1.5,
            steps=1, tail_cap=0),
    3: dict(L=1, B=8, N_q=32, N_kv=8, D=128, S=32768, S_obs=32, lam=0.5, dtype="bf16", sigma=1.0,
            steps=16, tail_cap=0),
    4: dict(L=1, B=1, N_q=32, N_kv=8, D=128, S=131072, S_obs=64, lam=0.5, dtype="bf16", sigma=2.0,
            steps=1, tail_cap=0),
    5: dict(L=1, B=32, N_q=40, N_kv=40, D=128, S=16384, S_obs=32, lam=0.6, dtype="bf16", sigma=1.0,
            steps=64, tail_cap=64),
}


def torch_dtype(name):
    return torch.bfloat16 if name == "bf16" else torch.float32


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def channel_scales(cfg_id, layer, N_q, N_kv, D, sigma, device):
    """exp(sigma * n) per (head, channel); key and query scales drawn independently."""
    g = _gen(SEED0 + 1000 * cfg_id + layer, "cpu")
    nk = torch.randn(N_kv, D, generator=g)
    nq = torch.randn(N_q, D, generator=g)
    return torch.exp(sigma * nk).to(device), torch.exp(sigma * nq).to(device)


def gen_prefill(cfg_id, layer, device, B, N_q, N_kv, D, S, S_obs, sigma, dtype, **_):
    """Q_obs [1,B,N_q,S_obs,D], K and V [1,B,N_kv,S,D] of one layer."""
    sk, sq = channel_scales(cfg_id, layer, N_q, N_kv, D, sigma, device)
    g = _gen(SEED0 + 1000 * cfg_id + layer + 500, device)
    dt = torch_dtype(dtype)
    q_obs = (torch.randn(1, B, N_q, S_obs, D, generator=g, device=device) * sq[None, None, :, None, :]).to(dt)
    k = torch.empty(1, B, N_kv, S, D, device=device, dtype=dt)
    v = torch.empty(1, B, N_kv, S, D, device=device, dtype=dt)
    for b in range(B):   # one batch row at a time bounds the fp32 temporaries
        k[0, b] = (torch.randn(N_kv, S, D, generator=g, device=device) * sk[:, None, :]).to(dt)
        v[0, b] = torch.randn(N_kv, S, D, generator=g, device=device).to(dt)
    return q_obs, k, v


def gen_decode(cfg_id, layer, step, device, B, N_q, N_kv, D, sigma, dtype, **_):
    """Decode-step query q [1,B,N_q,D] and the new token's k, v [1,B,N_kv,D]."""
    sk, sq = channel_scales(cfg_id, layer, N_q, N_kv, D, sigma, device)
    g = _gen(SEED0 + 1000 * cfg_id + layer + 700 + 7 * step, device)
    dt = torch_dtype(dtype)
    q = (torch.randn(1, B, N_q, D, generator=g, device=device) * sq[None, None]).to(dt)
    k_new = (torch.randn(1, B, N_kv, D, generator=g, device=device) * sk[None, None]).to(dt)
    v_new = torch.randn(1, B, N_kv, D, generator=g, device=device).to(dt)
    return q, k_new, v_new


def as_numpy(t):
    """Host numpy view of a tensor for the oracle: bf16 travels as uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view("uint16")
    return t.numpy()

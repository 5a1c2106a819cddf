"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

import paper_2407_21018_amd as thk
from oracle import oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
A = 4096      # a 16-byte aligned fake device address (never dereferenced on these paths)
BIG = 1 << 40


def _declared():
    hdr = open(os.path.join(ROOT, "include", "thk.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    return sorted(set(re.findall(r"\b(thk_[a-z_]+)\s*\(", hdr)))


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(thk.lib_path())
    names = _declared()
    assert {"thk_score", "thk_select_topk", "thk_compact_keys", "thk_decode_attn", "thk_prune",
            "thk_tail_append", "thk_workspace_bytes", "thk_keep_count"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in thk.h but not exported"


def test_binding_has_the_same_names():
    for n in _declared():
        assert hasattr(thk, n), f"binding lacks {n}"


def test_keep_count_matches_oracle():
    for D in (8, 64, 128):
        for lam in (0.0, 0.1, 0.25, 0.3, 0.4, 0.5, 0.6, 0.75, 0.9, 0.99):
            assert thk.thk_keep_count(D, lam) == O.keep_count(D, lam)
    assert thk.thk_keep_count(128, 1.0) == -1 and thk.thk_keep_count(0, 0.5) == -1


def _shape(**kw):
    d = dict(L=1, B=2, N_q=8, N_kv=2, D=128, S=1000, S_obs=32, T=64, ld_keep=0, dtype=thk.THK_BF16, n_split=0)
    d.update(kw)
    return thk.make_shape(**d)


def _status(fn, *a, **k):
    try:
        fn(*a, **k)
    except thk.ThkError as e:
        return e.status
    return 0


@pytest.mark.parametrize("kw,want", [
    (dict(N_q=7), 2), (dict(T=0), 2), (dict(T=129), 2), (dict(S=0), 2), (dict(S_obs=0), 2),
    (dict(S_obs=1001), 2), (dict(ld_keep=63), 2), (dict(ld_keep=132), 2), (dict(T=128, ld_keep=129), 2), (dict(n_split=-1), 2), (dict(n_split=5000), 2),
    (dict(B=0), 2), (dict(D=64, T=32), 3), (dict(dtype=7), 3),
])
def test_bad_shapes_are_rejected_before_launch(kw, want):
    s = _shape(**kw)
    assert _status(thk.thk_score, s, A, A, A, (A, BIG), stream=0) == want
    assert _status(thk.thk_prune, s, A, A, A, A, A, (A, BIG), stream=0) == want
    if "S_obs" not in kw:      # S_obs is ignored outside score / prune
        assert thk.thk_workspace_bytes(s, thk.THK_OP_SCORE) == 0
        assert _status(thk.thk_select_topk, s, A, A, stream=0) == want
        assert _status(thk.thk_compact_keys, s, A, A, A, stream=0) == want
        assert _status(thk.thk_decode_attn, s, A, A, A, A, None, None, 0, 0, A, (A, BIG), stream=0) == want
        assert _status(thk.thk_tail_append, s, A, A, A, A, 0, 4, stream=0) == want


def test_null_alignment_workspace_and_tail_errors():
    s = _shape()
    assert _status(thk.thk_score, s, None, A, A, (A, BIG), stream=0) == 1
    assert _status(thk.thk_score, s, A, A + 8, A, (A, BIG), stream=0) == 4
    assert _status(thk.thk_score, s, A, A, A, (A, 8), stream=0) == 5
    assert _status(thk.thk_score, s, A, A, A, (None, 0), stream=0) == 5
    assert _status(thk.thk_score, s, A, A, A, (A + 4, BIG), stream=0) == 5
    assert _status(thk.thk_select_topk, s, A, None, stream=0) == 1
    assert _status(thk.thk_compact_keys, s, A, A, A + 2, stream=0) == 4
    assert _status(thk.thk_prune, s, A, A, None, A, A, (A, 16), stream=0) == 5
    assert _status(thk.thk_score_magnitude, s, A, 3, A, (A, BIG), stream=0) == 2
    # decode: tail arguments
    dec = lambda *a: _status(thk.thk_decode_attn, s, *a, stream=0)
    assert dec(A, A, A, A, None, None, 1, 4, A, (A, BIG)) == 1      # tail rows but no tail buffers
    assert dec(A, A, A, A, A, A, 5, 4, A, (A, BIG)) == 2            # s_tail > cap
    assert dec(A, A, A, A, A, A, -1, 4, A, (A, BIG)) == 2
    assert dec(A, A, A, A, None, None, 0, 0, A, (A, 16)) == 5       # split > 1 needs a workspace
    assert dec(A, A, A, A, None, None, 0, 0, A + 1, (A, BIG)) == 4
    assert _status(thk.thk_tail_append, s, A, A, A, A, 4, 4, stream=0) == 2   # tail full
    assert "workspace" in thk.thk_status_string(5) and thk.thk_status_string(0) == "ok"


def test_workspace_sizes_follow_the_split():
    s = _shape(S=4096, B=4, N_q=32, N_kv=32, T=76)
    n_dec = thk.thk_default_split(s, thk.THK_OP_DECODE)
    assert n_dec >= 1
    # split records (max, sum, acc[128]) per head and piece, then one 8-byte flag word per
    # (unit, head group, piece) -- here one head per group
    want = 16 if n_dec == 1 else 4 * 32 * n_dec * 130 * 4 + 4 * 32 * n_dec * 8
    assert thk.thk_workspace_bytes(s, thk.THK_OP_DECODE) == want
    n_sc = thk.thk_default_split(s, thk.THK_OP_SCORE)
    assert thk.thk_workspace_bytes(s, thk.THK_OP_SCORE) == 4 * 32 * n_sc * 128 * 8
    s2 = _shape(S=4096, B=4, N_q=32, N_kv=32, T=76, n_split=7)
    assert thk.thk_workspace_bytes(s2, thk.THK_OP_DECODE) == 4 * 32 * 7 * 130 * 4 + 4 * 32 * 7 * 8
    assert thk.thk_workspace_bytes(s2, thk.THK_OP_SCORE) == 4 * 32 * 7 * 128 * 8


def test_binding_refuses_short_tensors():
    torch = pytest.importorskip("torch")
    s = _shape()
    k = torch.zeros(10, dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        thk.thk_compact_keys(s, k, A, A, stream=0)


def test_cache_growth_argument_checks():
    s = _shape(S=1000, S_recent=32, S_cap=1100)
    assert _status(thk.thk_prune, _shape(S_recent=1000), A, A, A, A, A, (A, BIG), stream=0) == 2   # S_recent >= S
    assert _status(thk.thk_prune, _shape(S=1000, S_recent=32, S_cap=900), A, A, A, A, A, (A, BIG), stream=0) == 2
    assert _status(thk.thk_compact_rows, s, A, 64, 0, A, A, 1090, 20, stream=0) == 2       # past the capacity
    assert _status(thk.thk_compact_rows, s, A, 64, 60, A, A, 0, 20, stream=0) == 2         # past the source
    assert _status(thk.thk_compact_rows, s, None, 64, 0, A, A, 0, 20, stream=0) == 1
    assert _status(thk.thk_copy_rows, s, A, 64, 0, A, 64, 1, 10, stream=0) == 2            # upward shift in place
    assert _status(thk.thk_copy_rows, s, A, 64, 0, A + 8, 64, 0, 10, stream=0) == 4
    assert _status(thk.thk_cache_append, _shape(S=1000, S_cap=1001), A, A, A, A, 1, 8, stream=0) == 2   # value cache full
    assert _status(thk.thk_cache_append, s, A, A, A, A, 8, 8, stream=0) == 2               # tail full
    assert _status(thk.thk_tail_flush, s, A, A, A, None, None, 10, 8, 4, stream=0) == 2    # s_tail > cap
    assert _status(thk.thk_tail_flush, s, A, A, A, None, None, 8, 8, 9, stream=0) == 2     # flush more than held
    assert _status(thk.thk_tail_flush, s, A, A, A, A, None, 8, 8, 4, stream=0) == 1        # v without v_tail
    assert _status(thk.thk_tail_flush, _shape(S=1000, S_cap=1002), A, A, A, None, None, 8, 8, 4, stream=0) == 2
    # unified value cache at decode needs room for the tail rows
    assert _status(thk.thk_decode_attn, _shape(S=1000, S_cap=1003), A, A, A, A, A, None, 4, 8, A, (A, BIG), stream=0) == 2


def test_value_cache_entry_points_reject_bad_arguments():
    s = _shape()
    ws = (A, BIG)
    # thk_score_value
    assert _status(thk.thk_score_value, s, A, A, A, 2, A, ws, stream=0) == 2          # causal flag
    assert _status(thk.thk_score_value, s, A, None, A, 0, A, ws, stream=0) == 1       # k missing
    assert _status(thk.thk_score_value, s, A, A, A + 8, 0, A, ws, stream=0) == 4      # v misaligned
    assert _status(thk.thk_score_value, s, A, A, A, 0, A, (A, 16), stream=0) == 5     # workspace too small
    assert _status(thk.thk_score_value, _shape(S_obs=1001), A, A, A, 0, A, ws, stream=0) == 2
    assert _status(thk.thk_score_value, _shape(N_q=2048, N_kv=1, S_obs=32, S=100), A, A, A, 0, A, ws, stream=0) == 2
    # thk_prune_value
    assert _status(thk.thk_prune_value, s, A, A, A, 0, A, None, A, ws, stream=0) == 1     # idx_v missing
    assert _status(thk.thk_prune_value, s, A, A, A, 0, A, A, A, (A, 16), stream=0) == 5
    assert _status(thk.thk_prune_value, s, A, A, A, 3, None, A, A, ws, stream=0) == 2     # causal flag
    # thk_decode_attn_kv
    d = (s, A, A, A, A)
    assert _status(thk.thk_decode_attn_kv, *d, A, 0, 0, None, None, 0, 0, A, ws, stream=0) == 2     # T_v < 1
    assert _status(thk.thk_decode_attn_kv, *d, A, 65, 64, None, None, 0, 0, A, ws, stream=0) == 2   # ld_v < T_v
    assert _status(thk.thk_decode_attn_kv, *d, A, 64, 132, None, None, 0, 0, A, ws, stream=0) == 2  # ld_v > D
    assert _status(thk.thk_decode_attn_kv, *d, A, 63, 63, None, None, 0, 0, A, ws, stream=0) == 3   # ld_v % 4
    assert _status(thk.thk_decode_attn_kv, *d, None, 64, 64, None, None, 0, 0, A, ws, stream=0) == 1
    assert _status(thk.thk_decode_attn_kv, *d, A + 2, 64, 64, None, None, 0, 0, A, ws, stream=0) == 4
    assert _status(thk.thk_decode_attn_kv, *d, A, 64, 64, A, None, 2, 4, A, ws, stream=0) == 1      # tail without v_tail


def test_value_workspace_and_split_sizes():
    """Workspace of the value score = partial attention records (one per unit, split and 32-row
    query tile: 128 x 32 outputs + 32 maxima + 32 sums, fp32) + the squared outputs when a unit
    has more than one query tile; the value prune adds the score array."""
    rec = (32 * 128 + 64) * 4
    for G, S_obs, S in [(1, 32, 4096), (4, 32, 32768), (4, 64, 131072), (3, 16, 300), (1, 1, 1)]:
        s = _shape(L=2, B=1, N_q=2 * G, N_kv=2, S=S, S_obs=S_obs)
        U = 4
        n = thk.thk_default_split(s, thk.THK_OP_SCORE_VALUE)
        assert 1 <= n <= 256 and (n == 1 or S // n >= 128)
        nqt = -(-G * S_obs // 32)
        qt = 4 if nqt >= 4 else 2 if nqt >= 2 else 1
        nqt_pad = -(-nqt // qt) * qt
        want = U * n * nqt_pad * rec + (U * nqt * 32 * 128 * 4 if nqt > 1 else 0)
        assert thk.thk_workspace_bytes(s, thk.THK_OP_SCORE_VALUE) == want
        assert thk.thk_workspace_bytes(s, thk.THK_OP_PRUNE_VALUE) == (want + 15) // 16 * 16 + U * 128 * 4
        s.n_split = 3
        assert thk.thk_default_split(s, thk.THK_OP_SCORE_VALUE) == n     # the library's own choice
    assert thk.thk_workspace_bytes(_shape(S_obs=0), thk.THK_OP_SCORE_VALUE) == 0


def test_prune_plan_by_shape(thk_env):
    """Which form thk_prune takes (2 = rows held on chip, 1 = rows read twice, 0 = staged)."""
    for v in ("THK_PRUNE_PATH", "THK_PRUNE_BLOCK_ROWS", "THK_PRUNE_HOLD_ROWS"):
        thk_env.delenv(v, raising=False)
    cfg2 = thk.make_shape(32, 4, 32, 32, 128, 4096, 32, 76, 0, thk.THK_BF16, 0)
    assert thk.thk_prune_is_fused(cfg2) == 2
    assert thk.thk_prune_is_fused(thk.make_shape(1, 1, 32, 8, 128, 131072, 64, 64, 0, thk.THK_BF16, 0)) == 2  # 256 blocks per unit
    assert thk.thk_prune_is_fused(thk.make_shape(1, 1, 32, 8, 128, 262144, 64, 64, 0, thk.THK_BF16, 0)) == 2  # 512 blocks per unit
    assert thk.thk_prune_is_fused(thk.make_shape(1, 1, 32, 8, 128, 393216, 64, 64, 0, thk.THK_BF16, 0)) == 2  # 768: all that fit at once
    assert thk.thk_prune_is_fused(thk.make_shape(1, 1, 32, 8, 128, 393217, 64, 64, 0, thk.THK_BF16, 0)) == 0  # one block more: staged
    thk_env.setenv("THK_PRUNE_MAX_BLOCKS", "256")
    assert thk.thk_prune_is_fused(thk.make_shape(1, 1, 32, 8, 128, 262144, 64, 64, 0, thk.THK_BF16, 0)) == 0
    thk_env.delenv("THK_PRUNE_MAX_BLOCKS")
    assert thk.thk_prune_is_fused(thk.make_shape(1, 8, 32, 8, 128, 32768, 32, 64, 0, thk.THK_BF16, 0)) == 2
    tiny = thk.make_shape(1, 1, 8, 8, 128, 2048, 32, 64, 0, thk.THK_F32, 0)
    assert thk.thk_prune_is_fused(tiny) == 2     # small calls: 128-row blocks, still held on chip
    assert thk.thk_prune_is_fused(thk.make_shape(1, 1, 8, 8, 128, 2048, 32, 64, 72, thk.THK_F32, 0)) == 2    # padded rows, pitch 288 bytes
    assert thk.thk_prune_is_fused(thk.make_shape(1, 1, 8, 8, 128, 2048, 32, 64, 73, thk.THK_F32, 0)) == 2    # any pitch
    assert thk.thk_prune_is_fused(thk.make_shape(1, 1, 8, 8, 128, 2047, 32, 51, 0, thk.THK_BF16, 0)) == 2    # dense rows: any length
    thk_env.setenv("THK_PRUNE_BLOCK_ROWS", "64")
    assert thk.thk_prune_is_fused(tiny) == 1     # a block size that is not held: rows read twice
    thk_env.delenv("THK_PRUNE_BLOCK_ROWS")
    thk_env.setenv("THK_PRUNE_PATH", "reread")
    assert thk.thk_prune_is_fused(cfg2) == 1
    thk_env.setenv("THK_PRUNE_PATH", "staged")
    assert thk.thk_prune_is_fused(cfg2) == 0


def test_prune_launch_count_by_shape(thk_env):
    """One launch for calls of at most two rounds of resident blocks (three for units of more than
    64 blocks), three launches beyond, three per group of units in the staged form."""
    for v in ("THK_PRUNE_PATH", "THK_PRUNE_BLOCK_ROWS", "THK_PRUNE_HOLD_ROWS", "THK_PRUNE_LAUNCH"):
        thk_env.delenv(v, raising=False)
    mk = lambda L, B, N_q, N_kv, S, T, dt=thk.THK_BF16: thk.make_shape(L, B, N_q, N_kv, 128, S, 32, T, 0, dt, 0)
    cfg1, cfg2, cfg2_1 = mk(1, 1, 8, 8, 2048, 64, thk.THK_F32), mk(32, 4, 32, 32, 4096, 76), mk(1, 4, 32, 32, 4096, 76)
    cfg3, cfg4, cfg5 = mk(1, 8, 32, 8, 32768, 64), mk(1, 1, 32, 8, 131072, 64), mk(1, 32, 40, 40, 16384, 51)
    assert [thk.thk_prune_launches(s) for s in (cfg1, cfg2_1, cfg4)] == [1, 1, 1]
    assert [thk.thk_prune_launches(s) for s in (cfg2, cfg3, cfg5)] == [3, 3, 3]
    thk_env.setenv("THK_PRUNE_LAUNCH", "classic")
    assert thk.thk_prune_launches(cfg1) == 3
    thk_env.setenv("THK_PRUNE_LAUNCH", "solo")
    assert thk.thk_prune_launches(cfg2) == 1
    thk_env.setenv("THK_PRUNE_PATH", "reread")      # rows read twice: only the three-launch form exists
    assert thk.thk_prune_launches(cfg1) == 3
    thk_env.setenv("THK_PRUNE_PATH", "staged")
    assert thk.thk_prune_launches(cfg2) == 3 * 4    # groups of at most 1 GiB of K: 4 groups of 8 layers
    assert thk.thk_prune_launches(mk(1, 1, 8, 8, 2048, 200)) == 0


def test_decode_kernel_choice_by_shape(thk_env):
    """bf16, query heads in groups of four, T and the row pitches multiples of 4: the matrix-core kernel."""
    thk_env.delenv("THK_DECODE_MFMA", raising=False)
    mk = lambda N_q, N_kv, T, ld, dt: thk.make_shape(1, 1, N_q, N_kv, 128, 4096, 1, T, ld, dt, 0)
    assert thk.thk_decode_on_matrix_cores(mk(32, 8, 64, 0, thk.THK_BF16)) == 1
    assert thk.thk_decode_on_matrix_cores(mk(32, 8, 76, 80, thk.THK_BF16)) == 1
    assert thk.thk_decode_on_matrix_cores(mk(64, 8, 128, 0, thk.THK_BF16)) == 1       # two groups of four
    assert thk.thk_decode_on_matrix_cores(mk(32, 32, 76, 0, thk.THK_BF16)) == 0       # one head per KV head
    assert thk.thk_decode_on_matrix_cores(mk(16, 8, 64, 0, thk.THK_BF16)) == 0        # two heads per KV head
    assert thk.thk_decode_on_matrix_cores(mk(24, 8, 64, 0, thk.THK_BF16)) == 1        # three: 3 of 4 slots
    assert thk.thk_decode_on_matrix_cores(mk(28, 4, 64, 0, thk.THK_BF16)) == 1        # seven: 7 of 8 slots
    assert thk.thk_decode_on_matrix_cores(mk(32, 8, 51, 0, thk.THK_BF16)) == 0        # dense rows of 51: pitch not a multiple of 4
    assert thk.thk_decode_on_matrix_cores(mk(32, 8, 51, 52, thk.THK_BF16)) == 1       # the same rows padded to 52
    assert thk.thk_decode_on_matrix_cores(mk(32, 8, 64, 66, thk.THK_BF16)) == 0       # pitch not a multiple of 4
    assert thk.thk_decode_on_matrix_cores(mk(32, 8, 64, 0, thk.THK_F32)) == 0
    assert thk.thk_decode_on_matrix_cores(mk(32, 8, 64, 0, thk.THK_BF16), 51, 52) == 1  # channel-pruned values
    assert thk.thk_decode_on_matrix_cores(mk(32, 8, 64, 0, thk.THK_BF16), 51, 51) == 0  # invalid pitch (below the ABI's multiple of 4)
    assert thk.thk_decode_on_matrix_cores(mk(32, 8, 64, 0, thk.THK_BF16), 200, 200) == 0
    # eight heads per block when the KV heads serve a multiple of eight: one block per unit and
    # split, three resident blocks per compute unit
    s8 = thk.make_shape(1, 8, 64, 8, 128, 32768, 1, 76, 0, thk.THK_BF16, 0)
    s4 = thk.make_shape(1, 8, 32, 8, 128, 32768, 1, 76, 0, thk.THK_BF16, 0)
    assert thk.thk_default_split(s8, thk.THK_OP_DECODE) == 8      # 64 units x 8 = 512 blocks <= 768
    assert thk.thk_default_split(s4, thk.THK_OP_DECODE) == 16     # 64 units x 16 = 1024 blocks
    thk_env.setenv("THK_DECODE_MFMA", "0")
    assert thk.thk_decode_on_matrix_cores(mk(32, 8, 64, 0, thk.THK_BF16)) == 0
    assert thk.thk_default_split(s8, thk.THK_OP_DECODE) == 8      # two blocks of four heads per unit and split


def test_default_decode_split_follows_the_size_of_the_call(thk_env):
    """Short sequences are not split (no merge launch), few units get small pieces, one unit may
    get up to 128 pieces; the workspace size follows the same choice."""
    thk_env.delenv("THK_DECODE_MFMA", raising=False)
    def split(B, N_q, N_kv, S, dtype=thk.THK_BF16):
        s = thk.make_shape(1, B, N_q, N_kv, 128, S, 1, 64, 0, dtype, 0)
        n = thk.thk_default_split(s, thk.THK_OP_DECODE)
        explicit = thk.make_shape(1, B, N_q, N_kv, 128, S, 1, 64, 0, dtype, n)
        assert thk.thk_workspace_bytes(s, thk.THK_OP_DECODE) == thk.thk_workspace_bytes(explicit, thk.THK_OP_DECODE)
        return n
    assert split(1, 8, 8, 512) == 1            # one head per block: no split up to 768 rows
    assert split(1, 8, 8, 768) == 1
    assert split(1, 8, 8, 1024) == 8           # 64 blocks of 128 rows
    assert split(1, 32, 8, 256) == 1           # four heads per block: no split up to 320 rows
    assert split(1, 32, 8, 512) == 4           # 128-row pieces while the launch is small
    assert split(1, 8, 8, 384, thk.THK_F32) == 1   # fp32 rows are twice the bytes: half the limits
    assert split(1, 8, 8, 512, thk.THK_F32) == 4
    assert split(4, 32, 32, 1024) == 4         # 128 units: 512 blocks of 256 rows, not 1024 of 128
    assert split(4, 32, 32, 4096) == 8         # the benchmark's shape
    assert split(1, 1, 1, 32768) == 128        # one unit: beyond 64 pieces
    assert split(1, 4, 4, 32768) == 64         # four units: 256 blocks already
    assert split(32, 40, 40, 16384) == 2       # big calls: two pieces per unit


def test_plain_c_program_uses_the_boundary(tmp_path):
    """thk.h is a C header and libthk.so a C library: a gcc-built program with no C++ and no
    Python in it includes the one and links the other."""
    import subprocess
    exe = tmp_path / "abi_host_check"
    libdir = os.path.dirname(thk.lib_path())
    subprocess.check_call(["gcc", "-std=c11", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"),
                           os.path.join(ROOT, "tests", "c", "abi_host_check.c"), "-o", str(exe),
                           "-L", libdir, "-lthk", f"-Wl,-rpath,{libdir}", "-Wl,-rpath,/opt/rocm/lib"])
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "abi host check ok" in out.stdout


def test_host_code_of_the_boundary_under_sanitizers(tmp_path):
    """The translation unit that holds every argument check (csrc/thk_api.hip) rebuilt with
    AddressSanitizer and UndefinedBehaviorSanitizer on the HOST side, linked with the other
    objects of the in-tree build, and driven by the plain-C program above: no report, exit 0."""
    import glob
    import shutil
    import subprocess
    objs = [o for o in glob.glob(os.path.join(ROOT, "paper_2407_21018_amd", "_build", "*.o"))
            if os.path.basename(o) != "thk_api.o"]
    clang = "/opt/rocm/lib/llvm/bin/clang"
    if not objs or shutil.which("hipcc") is None or not os.path.exists(clang):
        pytest.skip("needs the in-tree object files and the ROCm compilers")
    csrc = os.path.join(ROOT, "paper_2407_21018_amd", "csrc")
    san = ["-fsanitize=address", "-fsanitize=undefined"]
    host_san = [x for f in san for x in ("-Xarch_host", f)]
    api_o, lib, exe = tmp_path / "thk_api.o", tmp_path / "libthk.so", tmp_path / "abi_host_check"
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-Xclang",
                           "-target-feature", "-Xclang", "-packed-fp32-ops", *host_san, "-I",
                           os.path.join(ROOT, "include"), "-I", csrc, "-c", os.path.join(csrc, "thk_api.hip"),
                           "-o", str(api_o)], stderr=subprocess.DEVNULL)
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *san, "-shared-libsan", str(api_o),
                           *objs, "-o", str(lib)], stderr=subprocess.DEVNULL)
    rt = os.path.dirname(subprocess.check_output([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], text=True).strip())
    subprocess.check_call([clang, "-std=c11", "-g", *san, "-shared-libsan", "-I", os.path.join(ROOT, "include"),
                           os.path.join(ROOT, "tests", "c", "abi_host_check.c"), "-o", str(exe), "-L", str(tmp_path),
                           "-lthk", f"-Wl,-rpath,{tmp_path}", "-Wl,-rpath,/opt/rocm/lib", f"-Wl,-rpath,{rt}"])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:halt_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120, env=env)
    assert out.returncode == 0 and "abi host check ok" in out.stdout, out.stdout + out.stderr
    assert "runtime error" not in out.stderr and "AddressSanitizer" not in out.stderr, out.stderr


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    out = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                         text=True, timeout=120)
    assert out.returncode == 2 and "ONE GPU" in out.stderr


def test_environment_switches_are_read_once_and_on_reload(monkeypatch):
    """The library takes its THK_* switches from the environment once per process: a change made
    afterwards shows only after thk_reload_env()."""
    cfg2 = thk.make_shape(32, 4, 32, 32, 128, 4096, 32, 76, 0, thk.THK_BF16, 0)
    gqa = thk.make_shape(1, 1, 32, 8, 128, 4096, 1, 64, 0, thk.THK_BF16, 0)
    for v in ("THK_PRUNE_PATH", "THK_PRUNE_BLOCK_ROWS", "THK_PRUNE_HOLD_ROWS", "THK_DECODE_MFMA"):
        monkeypatch.delenv(v, raising=False)
    thk.thk_reload_env()
    assert thk.thk_prune_is_fused(cfg2) == 2 and thk.thk_decode_on_matrix_cores(gqa) == 1
    monkeypatch.setenv("THK_PRUNE_PATH", "staged")
    monkeypatch.setenv("THK_DECODE_MFMA", "0")
    assert thk.thk_prune_is_fused(cfg2) == 2 and thk.thk_decode_on_matrix_cores(gqa) == 1   # cached
    thk.thk_reload_env()
    assert thk.thk_prune_is_fused(cfg2) == 0 and thk.thk_decode_on_matrix_cores(gqa) == 0   # re-read
    monkeypatch.delenv("THK_PRUNE_PATH")
    monkeypatch.delenv("THK_DECODE_MFMA")
    assert thk.thk_prune_is_fused(cfg2) == 0
    thk.thk_reload_env()
    assert thk.thk_prune_is_fused(cfg2) == 2 and thk.thk_decode_on_matrix_cores(gqa) == 1


def test_bench_stream_rejects_misuse():
    """The benchmark stream kernel checks its arguments on the host: nothing is launched on a bad
    mode, block count, width, missing buffer or misaligned pointer."""
    L = thk.load()
    st = lambda mode, src, dst, n, w: L.thk_bench_stream(mode, src, dst, n, w, None)
    assert st(3, A, A, 1, 1) == 2 and st(-1, A, A, 1, 1) == 2                    # mode
    assert st(thk.THK_STREAM_COPY, A, A, 0, 1) == 2 and st(thk.THK_STREAM_COPY, A, A, 1 << 31, 1) == 2
    assert st(thk.THK_STREAM_COPY, A, A, 1, 0) == 2 and st(thk.THK_STREAM_WRITE, None, A, 1, 33) == 2
    assert st(thk.THK_STREAM_READ, None, None, 1, 0) == 1                          # src missing
    assert st(thk.THK_STREAM_COPY, A, None, 1, 4) == 1 and st(thk.THK_STREAM_WRITE, None, None, 1, 4) == 1
    assert st(thk.THK_STREAM_READ, A + 8, None, 1, 0) == 4 and st(thk.THK_STREAM_COPY, A, A + 4, 1, 4) == 4

"""thk_bench_stream: the plain read / copy / write kernel the benchmark uses as its ceiling does
what its description says (so that the ceilings mean what they are taken to mean) and touches
nothing outside the bytes it is given."""
import pytest
import torch

import paper_2407_21018_amd as thk

pytestmark = pytest.mark.gpu
CH = 4   # int32 words per 16-byte chunk


@pytest.mark.parametrize("n_blocks,w", [(1, 1), (3, 16), (5, 19), (2, 32)])
def test_copy_moves_the_first_w_chunks_of_every_thread(n_blocks, w):
    g = torch.Generator(device="cuda"); g.manual_seed(5)
    src = torch.randint(-2**31, 2**31 - 1, (n_blocks, 32, 256, CH), dtype=torch.int32, device="cuda", generator=g)
    guard = 64
    dst = torch.full((n_blocks * w * 256 * CH + 2 * guard,), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    body = dst[guard:guard + n_blocks * w * 256 * CH]
    thk.thk_bench_stream(thk.THK_STREAM_COPY, src, body, n_blocks, w)
    torch.cuda.synchronize()
    # block b, thread t keeps chunks j = 0 .. 31 (chunk j * 256 + t of the block) and stores j < w
    assert torch.equal(body.view(n_blocks, w, 256, CH), src[:, :w])
    assert (dst[:guard] == 0x5A5A5A5A).all() and (dst[-guard:] == 0x5A5A5A5A).all()


def test_write_fills_and_read_leaves_everything_alone():
    n_blocks, w = 4, 7
    dst = torch.zeros(n_blocks * w * 256 * CH + 16, dtype=torch.int32, device="cuda")
    thk.thk_bench_stream(thk.THK_STREAM_WRITE, None, dst[:n_blocks * w * 256 * CH], n_blocks, w)
    torch.cuda.synchronize()
    got = dst[:n_blocks * w * 256 * CH].view(n_blocks, w, 256, CH)
    b = torch.arange(n_blocks, device="cuda", dtype=torch.int32).view(-1, 1, 1).expand(n_blocks, w, 256)
    j = torch.arange(w, device="cuda", dtype=torch.int32).view(1, -1, 1).expand(n_blocks, w, 256)
    t = torch.arange(256, device="cuda", dtype=torch.int32).view(1, 1, -1).expand(n_blocks, w, 256)
    assert torch.equal(got[..., 0], b) and torch.equal(got[..., 1], j) and torch.equal(got[..., 3], t)
    assert (got[..., 2] == 0x74686B).all() and (dst[-16:] == 0).all()
    src = torch.arange(2 * 32 * 256 * CH, dtype=torch.int32, device="cuda")
    keep = src.clone()
    thk.thk_bench_stream(thk.THK_STREAM_READ, src, None, 2, 0)
    torch.cuda.synchronize()
    assert torch.equal(src, keep)


def test_binding_refuses_short_buffers():
    src = torch.zeros(32 * 256 * CH, dtype=torch.int32, device="cuda")
    with pytest.raises(ValueError):
        thk.thk_bench_stream(thk.THK_STREAM_READ, src, None, 2, 0)
    with pytest.raises(ValueError):
        thk.thk_bench_stream(thk.THK_STREAM_COPY, src, torch.zeros(8, dtype=torch.int32, device="cuda"), 1, 4)

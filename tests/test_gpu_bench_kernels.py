"""The two plain streaming kernels that measure the GPU's sustained read and copy rates
(include/lukv_bench.h): they must touch every byte they claim to."""
import numpy as np
import pytest
import torch

from paper_2602_08585_amd import lukv

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n16,blocks", [(1, 1), (256 * 8 * 3 + 5, 3), (100003, 64), (1 << 18, 1024)])
def test_stream_read_folds_every_word_and_copy_copies(n16, blocks):
    print("case bench kernels", n16, blocks, flush=True)
    lukv.load_library()
    g = torch.Generator().manual_seed(n16)
    host = torch.randint(-2**31, 2**31 - 1, (n16, 4), dtype=torch.int64, generator=g).to(torch.int32)
    src = host.cuda()
    sink = torch.zeros(4 * blocks, dtype=torch.int32, device="cuda")
    lukv.lukv_bench_stream_read(src, 16 * n16, sink, blocks)
    dst = torch.zeros_like(src)
    lukv.lukv_bench_copy(src, dst, 16 * n16, blocks)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    # the read kernel adds, per thread, x^y^z^w of the words of its full rounds of eight and the
    # x of the words of its tail: reproduce the total modulo 2^32
    h = host.numpy().view(np.uint32).astype(np.uint64)
    stride = blocks * 256
    # a thread leaves the rounds of eight as soon as ITS eighth word would pass the end
    idx = np.arange(n16)
    t, r = idx % stride, idx // stride
    rounds = np.maximum(0, (n16 - 1 - t - 7 * stride) // (8 * stride) + 1) * (n16 > t + 7 * stride)
    in_full = r < 8 * rounds
    fold = (h[:, 0] ^ h[:, 1] ^ h[:, 2] ^ h[:, 3])
    want = (int(fold[in_full].sum()) + int(h[~in_full, 0].sum())) % (1 << 32)
    got = int(sink.cpu().numpy().view(np.uint32).astype(np.uint64).sum()) % (1 << 32)
    assert got == want

"""GPU check of the measurement helper tandem_read_stream: the words it folds are exactly the buffer's words, each
read once (the rate bench.py quotes beside the attention kernels is the rate of reading ALL of the buffer)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tb():
    import torch

    from paper_2402_08644_amd import binding

    assert torch.cuda.is_available()
    binding.lib()
    return torch, binding


@pytest.mark.parametrize("n_bytes", [16, 4096 + 16, 2048 * 4096, 2048 * 4096 * 9 + 48, (1 << 26) + 4080])
def test_read_stream_folds_every_word_once(tb, n_bytes):
    torch, binding = tb
    g = torch.Generator("cuda").manual_seed(n_bytes % 1000)
    src = torch.randint(-(1 << 31), (1 << 31) - 1, (n_bytes // 4,), dtype=torch.int32, device="cuda", generator=g)
    sink = torch.full((binding.READ_STREAM_BLOCKS,), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    binding.tandem_read_stream(src, sink)
    torch.cuda.synchronize()
    got = np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32))
    want = np.bitwise_xor.reduce(src.cpu().numpy().view(np.uint32))
    assert got == want
    # flipping one bit anywhere changes the fold: the first, a middle and the last word
    for idx in (0, src.numel() // 2, src.numel() - 1):
        src[idx] ^= 1 << 7
        binding.tandem_read_stream(src, sink)
        torch.cuda.synchronize()
        got2 = np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32))
        assert got2 == want ^ np.uint32(1 << 7), idx
        src[idx] ^= 1 << 7


def test_read_stream_error_codes(tb):
    torch, binding = tb
    sink = torch.zeros((binding.READ_STREAM_BLOCKS,), dtype=torch.int32, device="cuda")
    buf = torch.zeros((64,), dtype=torch.int32, device="cuda")
    with pytest.raises(binding.TandemError) as ei:
        binding.tandem_read_stream(buf[:2], sink)  # fewer than 16 bytes
    assert ei.value.status == binding.ERR_SHAPE
    with pytest.raises(binding.TandemError) as ei:
        binding.tandem_read_stream(buf[1:33], sink)  # not 16-byte aligned
    assert ei.value.status == binding.ERR_SHAPE
    torch.cuda.synchronize()

"""The benchmark's bandwidth probes (libfdprobes.so, not part of the product library)."""
import pytest

@pytest.mark.gpu
@pytest.mark.parametrize("tiles", [0, 1, 3, 511, 512, 1500])
def test_stream_read_probe_sums_every_word(tiles):
    """The staged read probe reads each 32-bit word of its buffer exactly once: the per-thread sums add up
    to the word sum of the buffer modulo 2^32, whether the tiles divide among the work-groups or not."""
    import numpy as np
    import torch
    from paper_2605_20022_amd import probes as pr
    rng = np.random.default_rng(1234 + tiles)
    words = rng.integers(0, 2**32, size=tiles * 8192, dtype=np.uint32)
    src = torch.from_numpy(words.view(np.int32).copy()).cuda()
    sums = torch.full((pr.STREAM_READ_SUMS,), -1, dtype=torch.int32, device="cuda")
    if tiles == 0:
        src = torch.zeros(4, dtype=torch.int32, device="cuda")[:0]
        # an empty tensor has no storage to point at: pass a valid address with zero bytes
        pad = torch.zeros(4, dtype=torch.int32, device="cuda")
        pr.stream_read(pad, sums, nbytes=0)
    else:
        pr.stream_read(src, sums)
    torch.cuda.synchronize()
    got = int(sums.cpu().numpy().view(np.uint32).astype(np.uint64).sum() % (1 << 32))
    want = int(words.astype(np.uint64).sum() % (1 << 32))
    assert got == want

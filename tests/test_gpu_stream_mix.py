"""The access-pattern probe of the library (benchmark aid): it must read and write exactly the bytes it
reports, for every block order and workgroup shape, and refuse buffers that are too small."""
import numpy as np
import pytest
import torch

from paper_2604_02715_amd import binding as B

pytestmark = pytest.mark.gpu

LARGE = (0, 3, 6)          # blocks of every eight that write 128 bytes more


def expected_output(src: np.ndarray, small: int) -> np.ndarray:
    """What the probe stores, written out from its description: per block the XOR of the block's four 1 KiB
    quarters (as 32-bit words), repeated piece by piece with the first word of every 16 bytes counting the pieces."""
    n_blocks = src.size // 4096
    words = src.view(np.uint32).reshape(n_blocks, 4, 256)
    x = words[:, 0] ^ words[:, 1] ^ words[:, 2] ^ words[:, 3]           # [n_blocks][256 words = 1 KiB]
    out = []
    for nb in range(n_blocks):
        size = small + (128 if nb % 8 in LARGE else 0)
        pieces = []
        for p in range((size + 1023) // 1024):
            piece = x[nb].copy()
            piece[0::4] += np.uint32(p)
            pieces.append(piece)
        out.append(np.concatenate(pieces)[: size // 4])
    return np.concatenate(out)


@pytest.mark.parametrize("waves,per_wave,order", [(8, 3, 0), (4, 1, 0), (16, 2, 0), (8, 3, 1), (4, 5, 1), (8, 2, 2), (16, 7, 2)])
def test_probe_moves_the_bytes_it_reports(waves, per_wave, order):
    n_blocks, small = 1237, 1408                                         # several workgroups, a ragged last one
    rng = np.random.default_rng(5)
    src_h = rng.integers(0, 256, n_blocks * 4096, dtype=np.uint8)
    want = expected_output(src_h, small)
    src = torch.from_numpy(src_h).cuda()
    dst = torch.full((want.size * 4 + 4096,), 0xA5, dtype=torch.uint8, device="cuda")
    written = B.fluxmoe_stream_mix(dst.data_ptr(), dst.numel(), src.data_ptr(), src.numel(), small, waves, per_wave, order)
    torch.cuda.synchronize()
    assert written == want.size * 4
    got = dst.cpu().numpy()
    assert np.array_equal(got[:written].view(np.uint32), want)
    assert (got[written:] == 0xA5).all()                                 # nothing past the reported bytes


def test_probe_refuses_what_does_not_fit():
    src = torch.zeros(8 * 4096, dtype=torch.uint8, device="cuda")
    dst = torch.zeros(8 * 256 + 3 * 128 - 128, dtype=torch.uint8, device="cuda")      # one line short
    for kw in (dict(), dict(small=200), dict(waves=3), dict(order=3), dict(per_wave=0)):
        small, waves, per_wave, order = kw.get("small", 256), kw.get("waves", 8), kw.get("per_wave", 3), kw.get("order", 0)
        with pytest.raises(B.FluxmoeError) as err:
            B.fluxmoe_stream_mix(dst.data_ptr(), dst.numel(), src.data_ptr(), src.numel(), small, waves, per_wave, order)
        assert err.value.status == -1
    torch.cuda.synchronize()
    assert int(dst.sum()) == 0

"""hlq_stream_read (measurement helper): every 16-byte unit is read exactly once -- the XOR of the
per-workgroup checksums equals the XOR of all 32-bit words of the range."""
import numpy as np
import pytest
import torch

from paper_2510_19482_amd import binding as B

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("nbytes,blocks,offset", [
    (16, 0, 0), (4096, 1, 16), (4096 + 16, 7, 0), ((1 << 20) + 48, 0, 32), ((1 << 20) + 48, 512, 0),
    (3 * 4096 * 5 + 16, 3, 4096), ((8 << 20) - 16, 4096, 16),
])
def test_checksum_covers_every_word_once(nbytes, blocks, offset):
    print("stream_read", nbytes, blocks, offset, flush=True)
    rng = np.random.default_rng(nbytes + blocks)
    host = rng.integers(0, 2**32, size=(offset + nbytes) // 4 + 8, dtype=np.uint32)
    buf = torch.from_numpy(host.view(np.int32)).cuda()
    units = nbytes // 16
    launched = min(blocks if blocks else 2048, (units + 255) // 256)
    sink = torch.zeros(max(launched, 1), dtype=torch.int32, device="cuda")
    B.hlq_stream_read(buf, nbytes, sink, blocks=blocks, offset=offset)
    torch.cuda.synchronize()
    got = np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32)[:launched])
    want = np.bitwise_xor.reduce(host[offset // 4: (offset + nbytes) // 4])
    assert got == want


@pytest.mark.parametrize("unroll", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("temporal", [False, True])
def test_shaped_read_covers_every_word_once(unroll, temporal):
    nbytes, blocks, offset = (3 << 20) + 16 * 37, 96, 48
    print("stream_read_shaped", unroll, temporal, flush=True)
    rng = np.random.default_rng(unroll + 17 * temporal)
    host = rng.integers(0, 2**32, size=(offset + nbytes) // 4 + 8, dtype=np.uint32)
    buf = torch.from_numpy(host.view(np.int32)).cuda()
    sink = torch.zeros(blocks, dtype=torch.int32, device="cuda")
    B.hlq_stream_read_shaped(buf, nbytes, sink, blocks=blocks, unroll=unroll, temporal=temporal, offset=offset)
    torch.cuda.synchronize()
    got = np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32))
    assert got == np.bitwise_xor.reduce(host[offset // 4: (offset + nbytes) // 4])


def test_shaped_read_rejects_other_unrolls():
    buf = torch.zeros(1024, dtype=torch.int32, device="cuda")
    with pytest.raises(B.HlqError) as e:
        B.hlq_stream_read_shaped(buf, 4096, buf, unroll=3)
    assert e.value.status == 3

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


def test_mfma_probe_sums_what_its_operands_say():
    # hlq_mfma_probe (measurement helper): with small-integer operands every product and sum is exact, and the sum
    # of all elements of A B is sum_k (column sum of A)[k] (row sum of B)[k], whatever the order inside the
    # matrix core.  Lane l of a 32x32x16 operand holds row / column l % 32 and k = 8 (l / 32) .. + 7.
    iters, blocks = 3, 5
    print("mfma_probe", iters, blocks, flush=True)
    rng = np.random.default_rng(7)
    waves = blocks * 4
    units = waves * 8 - 3                      # fewer units than the wavefronts ask for: indices wrap around
    host = rng.integers(-2, 3, size=(units, 64, 8)).astype(np.float16)
    ops = torch.from_numpy(host).cuda()
    sink = torch.zeros(blocks * 256, dtype=torch.float32, device="cuda")
    flop = B.hlq_mfma_probe(ops, iters, blocks, sink)
    torch.cuda.synchronize()
    assert flop == waves * iters * 16 * 2.0 * 32 * 32 * 16
    got = sink.cpu().numpy().astype(np.float64).reshape(waves, 64).sum(axis=1)
    flat = host.astype(np.float64).reshape(-1, 8)      # 16-byte units as the kernel indexes them
    nflat = flat.shape[0]

    def ksums(w, slot):
        idx = ((w * 8 + slot) * 64 + np.arange(64)) % nflat
        return flat[idx].reshape(2, 32, 8).sum(axis=1).reshape(16)   # sum over the 32 rows / columns, per k
    for w in range(waves):
        a = [ksums(w, 2 * o) for o in range(4)]
        b = [ksums(w, 2 * o + 1) for o in range(4)]
        want = iters * sum(float(a[(o + c) % 4] @ b[o]) for o in range(4) for c in range(4))
        assert got[w] == want, (w, got[w], want)


def test_mx_probe_sums_what_its_operands_say():
    # kind 1 (bf8 x fp4, 16x16x128): operands restricted to values whose products and sums are exact.  An 8-bit
    # operand lane l holds row l % 16, k = 16 (l / 16) + i for its first 16 bytes and 64 + 16 (l / 16) + i for the
    # next 16; a 4-bit operand lane holds column l % 16, k = 32 (l / 16) + n for nibble n of its 16 bytes.
    iters, blocks = 2, 3
    print("mfma_probe mx", iters, blocks, flush=True)
    rng = np.random.default_rng(11)
    waves = blocks * 4
    units = waves * 12
    a_codes = np.array([0x00, 0x38, 0x3C, 0x3E], dtype=np.uint8)          # bf8 e5m2: 0, 0.5, 1, 1.5
    a_vals = np.array([0.0, 0.5, 1.0, 1.5])
    b_codes = np.array([0x0, 0x2, 0x4, 0xA, 0x1], dtype=np.uint8)         # fp4 e2m1: 0, 1, 2, -1, 0.5
    b_vals = np.array([0.0, 1.0, 2.0, -1.0, 0.5])
    ai = rng.integers(0, 4, size=(units, 64, 16))
    bi = rng.integers(0, 5, size=(units, 64, 32))
    raw = a_codes[ai].copy()                                              # every unit as 8-bit operand bytes ...
    for u in range(2, units, 3):                                          # ... and every third one as packed nibbles
        nib = b_codes[bi[u]]
        raw[u] = (nib[:, 0::2] | (nib[:, 1::2] << 4)).astype(np.uint8)
    ops = torch.from_numpy(raw.reshape(-1).view(np.float16)).cuda()
    sink = torch.zeros(blocks * 256, dtype=torch.float32, device="cuda")
    flop = B.hlq_mfma_probe(ops, iters, blocks, sink, kind=1)
    torch.cuda.synchronize()
    assert flop == waves * iters * 32 * 2.0 * 16 * 16 * 128
    got = sink.cpu().numpy().astype(np.float64).reshape(waves, 64).sum(axis=1)

    def a_ksums(w, o):      # sum over the 16 rows, per k
        lo, hi = a_vals[ai[w * 12 + 3 * o]], a_vals[ai[w * 12 + 3 * o + 1]]          # [lane, 16]
        ks = np.zeros(128)
        for kb in range(4):
            ks[16 * kb:16 * kb + 16] = lo[16 * kb:16 * kb + 16].sum(axis=0)
            ks[64 + 16 * kb:64 + 16 * kb + 16] = hi[16 * kb:16 * kb + 16].sum(axis=0)
        return ks

    def b_ksums(w, o):      # sum over the 16 columns, per k
        v = b_vals[bi[w * 12 + 3 * o + 2]]                                            # [lane, 32]
        return np.concatenate([v[16 * g:16 * g + 16].sum(axis=0) for g in range(4)])

    for w in range(waves):
        a = [a_ksums(w, o) for o in range(4)]
        b = [b_ksums(w, o) for o in range(4)]
        want = iters * sum(float(a[(o + c) % 4] @ b[o]) for o in range(4) for c in range(8))
        assert got[w] == want, (w, got[w], want)

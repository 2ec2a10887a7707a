"""CPU model of how the bf16 direct-to-LDS kernel keeps an operand that is contiguous along m / n (a transposed A,
a row-major B) in LDS, written out from the layout its source describes: the 1 KB a wavefront's load q fills, the
chunk swizzle, and the addresses of the transposing fragment reads.  It checks, for tile sides of 256, 192 and 128,
that the loads fill the tile once, that every lane of every fragment read receives the 8 consecutive k of its row
that the 16x16x32 MFMA wants, and that the 32 lanes of one pass of a read touch each of the 64 LDS banks once.  The
index arithmetic here is the kernel's, restated; the test guards the scheme, not the kernel's code (the GPU parity
tests do that)."""
import pytest


def kswz(k):
    """swizzle of k-row k in 16-byte chunks"""
    return (((k >> 1) & 1) | (((k >> 3) & 1) << 1)) << 1


def loads(blocks):
    """LDS byte address of each 16-byte piece -> (k-row of the K-tile, chunk of the k-row) it receives"""
    lds = {}
    for wave in range(4):
        for q in range(blocks):                     # load q of the wavefront: sub-tile q / 2, k-rows 16 w + 8 (q & 1) ..
            for lane in range(64):
                k = 16 * wave + 8 * (q & 1) + lane // 8
                chunk = 8 * (q >> 1) + ((lane % 8) ^ kswz(k))
                dst = (wave * blocks + q) * 1024 + lane * 16
                assert dst not in lds
                lds[dst] = (k, chunk)
    return lds


def read_address(blocks, first_block, b, kk, h, lane):
    """where lane `lane` points for read h (0, 1) of block b, k-step kk; first_block: of the wavefront's part"""
    l16, lq = lane & 15, lane >> 4
    krow, half, gb = 8 * lq + (l16 >> 2), (l16 >> 1) & 1, first_block + b
    in_kb = (krow & 7) * 128 + ((half ^ kswz(krow)) * 16) + (l16 & 1) * 8
    blk = ((krow >> 4) * blocks + 2 * (gb >> 2) + ((krow >> 3) & 1)) * 1024 + (in_kb ^ ((gb & 3) << 5))
    return blk + kk * 2048 * blocks + h * 512


@pytest.mark.parametrize("blocks", [8, 6, 4])           # 16-row blocks per wavefront: tile sides 256, 192, 128
def test_mn_contiguous_tile_in_lds(blocks):
    lds = loads(blocks)
    assert sorted(lds) == list(range(0, 64 * 64 * blocks, 16))
    assert sorted(lds.values()) == [(k, c) for k in range(64) for c in range(4 * blocks)]
    for wave in range(4):
        first_block, first_row = (wave >> 1) * blocks, (wave >> 1) * 16 * blocks
        for kk in range(2):
            for b in range(blocks):
                got = {}
                for h in range(2):
                    addr = [read_address(blocks, first_block, b, kk, h, lane) for lane in range(64)]
                    assert all(0 <= a < 64 * 64 * blocks and a % 8 == 0 for a in addr)
                    for p in range(2):              # a pass serves 32 lanes of 8 bytes: 64 banks of 4 bytes
                        banks = [(a // 4 + w) % 64 for a in addr[32 * p:32 * p + 32] for w in range(2)]
                        assert len(set(banks)) == 64
                    # DS_READ_B64_TR_B16: within 16 lanes, lane i receives element i % 4 of the 8 bytes that lanes
                    # i / 4, 4 + i / 4, 8 + i / 4 and 12 + i / 4 point at
                    for lane in range(64):
                        group, i = lane & ~15, lane & 15
                        for e in range(4):
                            a = addr[group + i // 4 + 4 * e]
                            k, chunk = lds[a & ~15]
                            got[lane, 4 * h + e] = (k, 8 * chunk + (a & 15) // 2 + i % 4)
                for lane in range(64):              # the MFMA's operand: 8 consecutive k of row lane % 16 at k-offset 8 (lane / 16)
                    for x in range(8):
                        assert got[lane, x] == (32 * kk + 8 * (lane >> 4) + x, first_row + 16 * b + (lane & 15))

"""Host-side model of the LDS tile layouts of the absorb kernels.

The kernels place every 16-byte chunk of a cache row in a swizzled slot (so that both of their
read patterns spread over the LDS banks) and compute the per-lane addresses of the transfers and
of the reads from separate formulas.  This test restates those formulas (from the comments of
tmla_absorb_tile.hpp, tmla_absorb128_mfma.hip and tmla_absorb16_mfma.hip), fills a model tile the way the transfers do and
checks that
  * every read returns the chunk the matrix-core operand layout wants, and
  * under the bank rules measured on the hardware (64 four-byte banks; a 16-byte read is served
    16 consecutive lanes at a time, an 8-byte transposing read 32 lanes at a time) no group of
    lanes hits a bank twice.
No GPU and no library involved: it pins the address arithmetic."""
import pytest

BANKS = 64


def _banks(addr, nbytes):
    return {((addr + 4 * i) // 4) % BANKS for i in range(nbytes // 4)}


def _conflict_free(addrs, nbytes, group):
    for g0 in range(0, 64, group):
        seen = set()
        for lane in range(g0, g0 + group):
            b = _banks(addrs[lane], nbytes)
            if seen & b:
                return False
            seen |= b
    return True


class Tile1088:
    """tmla_absorb_tile.hpp: latent row r at r * 1088, chunk c in slot c ^ ((r >> 2) & 3); rope
    rows of 128 B behind, chunk c of row r in slot c ^ ((r >> 1) & 7)."""
    ROW, MAIN = 1088, 32 * 1088

    @staticmethod
    def f(r):
        return (r >> 2) & 3

    def fill(self):
        """address of a 16-byte slot -> ('lat' | 'rope', row, chunk), as the 36 transfers write"""
        img = {}
        for wave in range(4):
            for K in range(8):
                r = wave + 4 * K
                for lane in range(64):
                    chunk = lane ^ (K & 3)               # d.off[K & 3] = (lane ^ sw) << 4
                    img[r * self.ROW + lane * 16] = ("lat", r, chunk)
            for lane in range(64):                       # rope rows 8 wave .. 8 wave + 7
                row = 8 * wave + (lane >> 3)
                chunk = (lane & 7) ^ ((row >> 1) & 7)
                img[self.MAIN + wave * 1024 + lane * 16] = ("rope", row, chunk)
        return img

    def score_addr(self, lane, ks):
        n, g = lane & 31, lane >> 5
        return n * self.ROW + (((2 * (ks & 1) + g) ^ self.f(n)) << 4) + 64 * (ks >> 1)

    def rope_addr(self, lane, k):
        n, g = lane & 31, lane >> 5
        return self.MAIN + n * 128 + (((2 * k + g) ^ ((n >> 1) & 7)) << 4)

    def tr_addr(self, lane, kk, half, mb, quarter):
        g, j16, r16 = lane >> 5, lane >> 4, lane & 15
        chunk = 2 * (j16 & 1) + ((r16 & 3) >> 1)
        row = (4 * g + (r16 >> 2)) * self.ROW + 8 * (r16 & 1)
        base = row + ((chunk ^ g) << 4) if half == 0 else \
            row + 8 * self.ROW + ((chunk ^ g ^ 2) << 4)
        return base + 16 * kk * self.ROW + 64 * mb + 256 * quarter


class Tile1024:
    """tmla_absorb128_mfma.hip: latent row r at r * 1024, chunk c in slot c ^ f(r),
    f(r) = ((r & 3) << 2) | ((r >> 2) & 3); rope part as above."""
    ROW, MAIN = 1024, 32 * 1024

    @staticmethod
    def f(r):
        return ((r & 3) << 2) | ((r >> 2) & 3)

    def fill(self):
        img = {}
        for wave in range(4):
            for K in range(8):
                r = wave + 4 * K
                for lane in range(64):
                    chunk = lane ^ ((wave << 2) | (K & 3))
                    img[r * self.ROW + lane * 16] = ("lat", r, chunk)
            for lane in range(64):
                row = 8 * wave + (lane >> 3)
                chunk = (lane & 7) ^ ((row >> 1) & 7)
                img[self.MAIN + wave * 1024 + lane * 16] = ("rope", row, chunk)
        return img

    def score_addr(self, lane, ks):
        n, g = lane & 31, lane >> 5
        s0 = n * 1024 + ((g ^ self.f(n)) << 4)
        return (s0 ^ ((ks & 7) << 5)) + 256 * (ks >> 3)

    def rope_addr(self, lane, k):
        n, g = lane & 31, lane >> 5
        r0 = self.MAIN + n * 128 + ((g ^ ((n >> 1) & 7)) << 4)
        return r0 ^ (k << 5)

    def tr_addr(self, lane, kk, half, mb, lh):
        g, j16, r16 = lane >> 5, lane >> 4, lane & 15
        rq = r16 >> 2
        cx = 2 * (j16 & 1) + ((r16 & 3) >> 1)
        v_lo = (4 * g + rq) * 1024 + 64 * rq + ((cx ^ g) << 4) + 8 * (r16 & 1) + 512 * lh
        v = v_lo if half == 0 else (v_lo + 8192) ^ 32
        return (v ^ ((mb & 3) << 6)) + 256 * (mb >> 2) + 16384 * kk


@pytest.mark.parametrize("tile,nmb,nsel", [(Tile1088(), 4, 4), (Tile1024(), 8, 2)],
                         ids=["stride_1088", "stride_1024_xor"])
def test_tile_reads_return_the_intended_chunks_without_bank_conflicts(tile, nmb, nsel):
    img = tile.fill()
    assert len(img) == 32 * 64 + 32 * 8          # every slot of the tile written exactly once
    # score product, latent k-steps: lane (n, g) wants row n, chunk 2 ks + g
    for ks in range(32):
        addrs = [tile.score_addr(lane, ks) for lane in range(64)]
        for lane, a in enumerate(addrs):
            assert img[a] == ("lat", lane & 31, 2 * ks + (lane >> 5)), (ks, lane)
        assert _conflict_free(addrs, 16, 16), f"score read, k-step {ks}"
    # score product, rope k-steps: row n, rope chunk 2 k + g
    for k in range(4):
        addrs = [tile.rope_addr(lane, k) for lane in range(64)]
        for lane, a in enumerate(addrs):
            assert img[a] == ("rope", lane & 31, 2 * k + (lane >> 5)), (k, lane)
        assert _conflict_free(addrs, 16, 16), f"rope read, k-step {k}"
    # output product, transposing 8-byte reads: 16-lane group j, r = lane % 16 wants token row
    # 16 kk + 8 half + 4 g + r / 4 and latent columns 32 mb + 16 (j % 2) + 4 (r % 4) .. + 3 of
    # the wavefront's share (a quarter of 128 columns, or a half of 256)
    width = 512 // nsel
    for sel in range(nsel):
        for kk in range(2):
            for half in range(2):
                for mb in range(nmb):
                    addrs = [tile.tr_addr(lane, kk, half, mb, sel) for lane in range(64)]
                    for lane, a in enumerate(addrs):
                        g, j16, r16 = lane >> 5, lane >> 4, lane & 15
                        row = 16 * kk + 8 * half + 4 * g + (r16 >> 2)
                        col = width * sel + 32 * mb + 16 * (j16 & 1) + 4 * (r16 & 3)
                        kind, r, chunk = img[a & ~15]
                        assert (kind, r) == ("lat", row), (sel, kk, half, mb, lane)
                        assert chunk * 8 + (a & 15) // 2 == col, (sel, kk, half, mb, lane)
                    assert _conflict_free(addrs, 8, 32), f"transposing read {sel} {kk} {half} {mb}"


def test_private_tile_of_the_16_row_kernel():
    """tmla_absorb16_mfma.hip: latent row r at r * 1056, chunk c in slot c ^ ((r >> 3) & 1); rope
    rows of 128 B behind, chunk c of row r in slot c ^ ((r >> 1) & 7).  Lane = n + 16 q of a
    16x16x32 matrix-core operand: row n, k = 8 q + e."""
    ROW, MAIN = 1056, 32 * 1056
    img = {}
    for r in range(32):                                   # one transfer per latent row
        for lane in range(64):
            img[r * ROW + lane * 16] = ("lat", r, lane ^ ((r >> 3) & 1))
    for j in range(4):                                    # rope parts of rows 8 j .. 8 j + 7
        for lane in range(64):
            row = 8 * j + (lane >> 3)
            ch = (((lane & 7) ^ (lane >> 4)) << 4) ^ ((j & 1) << 6)
            assert ch >> 4 == (lane & 7) ^ ((row >> 1) & 7)
            img[MAIN + j * 1024 + lane * 16] = ("rope", row, ch >> 4)
    assert len(img) == 32 * 64 + 32 * 8
    # scores: token block mb, latent k-step ks: row 16 mb + n, chunk 4 ks + q
    for mb in range(2):
        for ks in range(16):
            addrs = [(l & 15) * ROW + (((l >> 4) ^ (((l & 15) >> 3) & 1)) << 4) + 64 * ks
                     + 16 * ROW * mb for l in range(64)]
            for l, a in enumerate(addrs):
                assert img[a] == ("lat", 16 * mb + (l & 15), 4 * ks + (l >> 4))
            assert _conflict_free(addrs, 16, 16), f"score read {mb} {ks}"
        for k in range(2):
            addrs = [MAIN + (l & 15) * 128 + (((4 * k + (l >> 4)) ^ (((l & 15) >> 1) & 7)) << 4)
                     + 16 * 128 * mb for l in range(64)]
            for l, a in enumerate(addrs):
                assert img[a] == ("rope", 16 * mb + (l & 15), 4 * k + (l >> 4))
            assert _conflict_free(addrs, 16, 16), f"rope read {mb} {k}"
    # outputs: 16-lane group q, r = lane % 16 wants token row 16 half + 4 q + r / 4 and latent
    # columns 16 mb + 4 (r % 4) .. + 3
    for half in range(2):
        for mb in range(32):
            addrs = []
            for l in range(64):
                n, q = l & 15, l >> 4
                addrs.append((4 * q + (n >> 2)) * ROW + ((((n & 3) >> 1) ^ (q >> 1)) << 4)
                             + 8 * (n & 1) + 32 * mb + 16 * ROW * half)
            for l, a in enumerate(addrs):
                n, q = l & 15, l >> 4
                kind, r, chunk = img[a & ~15]
                assert (kind, r) == ("lat", 16 * half + 4 * q + (n >> 2))
                assert chunk * 8 + (a & 15) // 2 == 16 * mb + 4 * (n & 3)
            assert _conflict_free(addrs, 8, 32), f"transposing read {half} {mb}"


def test_the_former_layout_had_two_way_conflicts():
    """Row stride 1056 with a one-bit slot swizzle, the layout the probe measured at half the LDS
    rate: the bank model reproduces that (rows n and n + 8 of a 16-lane group collide)."""
    addrs = [(l & 31) * 1056 + (((l >> 5) ^ (((l & 31) >> 2) & 1)) << 4) for l in range(64)]
    assert not _conflict_free(addrs, 16, 16)

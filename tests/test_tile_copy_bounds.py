"""Host-side model of the attention kernel's K^ tile copies (csrc/sage_attn.hip: issue_tile_piece and the
per-lane offsets around it): for every key step, piece, wavefront and lane, the 16-byte chunk a lane fetches
must lie inside the head's K^ buffer of exactly Nk*D bytes, and together the fetched chunks must cover every
byte of the tile's valid rows exactly once.  The hardware bounds check compares the per-lane offset with the
descriptor's size; the model applies the same rule to the same arithmetic, so a caller's buffer of exactly
B*H*Nk*d bytes is never overrun.  (The GPU tests show the values are right; this shows the addresses are.)"""
import numpy as np
import pytest

NWG = 4          # wavefronts of the group that copies a tile


def _k_swz(row, D):
    return (row & 7) if D == 128 else ((row >> 1) & 3)


def fetched_chunks(Nk, D, j):
    """Byte offsets (inside the head's K^ buffer) of the 16-byte chunks that step j's copy fetches."""
    TILE = 128 * D
    CPG = TILE // 16 // (NWG * 64)                 # pieces per wavefront
    CPR = D // 16                                  # chunks per K row
    head_bytes = Nk * D
    out = []
    for wig in range(NWG):
        for lane in range(64):
            slot = wig * 64 + lane
            row, pc = slot // CPR, slot % CPR
            voff = row * D + ((pc ^ _k_swz(row, D)) << 4)          # per-lane offset of piece 0
            for k in range(CPG):
                first = j * TILE + k * NWG * 1024                  # base of the piece's descriptor
                records = max(head_bytes - first, 0)               # its size
                if voff + 16 <= records:                           # the hardware's range check
                    out.append(first + voff)
    return np.array(out, dtype=np.int64)


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("Nk", [1, 5, 63, 64, 65, 127, 128, 129, 200, 255, 256, 600, 1000, 17776])
def test_k_tile_copies_stay_inside_the_buffer_and_cover_it(D, Nk):
    head_bytes = Nk * D
    nT = -(-Nk // 128)
    for j in sorted({0, nT // 2, nT - 1}):
        got = fetched_chunks(Nk, D, j)
        assert got.size == 0 or (got.min() >= 0 and got.max() + 16 <= head_bytes), (Nk, D, j)
        # exactly the chunks of the tile's valid rows, each once
        lo, hi = j * 128 * D, min((j + 1) * 128, Nk) * D
        want = np.arange(lo, hi, 16, dtype=np.int64)
        assert np.array_equal(np.sort(got), want), (Nk, D, j)

"""Host-only checks of the local-memory layout of the FP16 macro-tile kernels (paper Section 3.2: the layout of
the tiles in local memory is tuned because bank conflicts cost).  The library exports the address formulas its
kernels are built from; here they are run through (1) the definition of what a lane must receive and (2) a model
of the LDS banks of gfx950.

Bank model (measured on the GPU by timing reads in which one lane was given another lane's bank): 64 banks of 4
bytes; lanes that read the same address share one access; an 8-byte read is served 32 consecutive lanes at a
time; a 16-byte read 16 lanes at a time, namely lanes {0-3, 12-15, 20-27}, then {4-11, 16-19, 28-31}, and the
same in the upper half of the wavefront."""
import itertools

import pytest

from paper_1705_05249_amd import gemm as G

PASSES_16B = [[l + 32 * h for l in grp] for h in (0, 1)
              for grp in ([0, 1, 2, 3, 12, 13, 14, 15, 20, 21, 22, 23, 24, 25, 26, 27],
                          [4, 5, 6, 7, 8, 9, 10, 11, 16, 17, 18, 19, 28, 29, 30, 31])]
PASSES_8B = [list(range(0, 32)), list(range(32, 64))]


def cycles(addresses, width, passes):
    """clocks the LDS needs for one wavefront read under the bank model (one per pass when conflict-free)"""
    total = 0
    for lanes in passes:
        per_bank = {}
        for lane in lanes:
            a = addresses[lane]
            assert a % width == 0
            for word in range(a // 4, (a + width) // 4):
                per_bank.setdefault(word % 64, set()).add(word)
        total += max(len(words) for words in per_bank.values())
    return total


def wave_rows(tile_rows, fragment_rows):
    """(wave_row, fragment) pairs of the wavefront tiles the kernels use: 64 or 128 rows per wavefront"""
    out = []
    for height in (64, 128):
        if height > tile_rows:
            continue
        for wave_row in range(0, tile_rows, height):
            if wave_row % 64:
                continue
            for f in range(height // fragment_rows):
                out.append((wave_row, f))
    return sorted(set(out))


@pytest.mark.parametrize("fragment_rows,tile_rows", [(32, 64), (32, 128), (32, 256), (16, 128), (16, 256)])
def test_k_contiguous_fragment_reads_fetch_the_right_elements_without_conflicts(fragment_rows, tile_rows):
    steps = fragment_rows // 8
    for (wave_row, f), s in itertools.product(wave_rows(tile_rows, fragment_rows), range(steps)):
        addr = [G.mg_lds_read_offset(True, fragment_rows, tile_rows, wave_row, lane, f, s) for lane in range(64)]
        assert min(addr) >= 0
        for lane in range(64):
            row = wave_row + fragment_rows * f + lane % fragment_rows
            k0 = 8 * ((64 // fragment_rows) * s + lane // fragment_rows)
            for e in range(8):
                assert G.mg_lds_store_offset(True, fragment_rows, tile_rows, row, k0 + e) == addr[lane] + 2 * e
        assert cycles(addr, 16, PASSES_16B) == 4, (fragment_rows, tile_rows, wave_row, f, s)


@pytest.mark.parametrize("fragment_rows,tile_rows", [(32, 128), (32, 256), (16, 128), (16, 256)])
def test_transposing_fragment_reads_fetch_the_right_elements_without_conflicts(fragment_rows, tile_rows):
    steps = fragment_rows // 8
    for (wave_row, f), s, half in itertools.product(wave_rows(tile_rows, fragment_rows), range(steps), (0, 1)):
        addr = [G.mg_lds_read_offset(False, fragment_rows, tile_rows, wave_row, lane, f, s, half) for lane in range(64)]
        assert min(addr) >= 0
        for lane in range(64):
            g, a, b = lane // 16, (lane % 16) // 4, lane % 4
            row = wave_row + fragment_rows * f + lane % fragment_rows
            k0 = 8 * ((64 // fragment_rows) * s + lane // fragment_rows) + 4 * half
            for j in range(4):
                source = 16 * g + a + 4 * j           # the lane whose element b ends up as value j of this lane
                assert G.mg_lds_store_offset(False, fragment_rows, tile_rows, row, k0 + j) == addr[source] + 2 * b
        assert cycles(addr, 8, PASSES_8B) == 2, (fragment_rows, tile_rows, wave_row, f, s, half)


def test_every_element_has_its_own_place():
    for k_contiguous, fragment_rows, tile_rows in ((True, 32, 64), (True, 32, 256), (True, 16, 256), (False, 32, 256),
                                                   (False, 16, 128)):
        seen = set()
        for row in range(tile_rows):
            for k in range(64):
                o = G.mg_lds_store_offset(k_contiguous, fragment_rows, tile_rows, row, k)
                assert 0 <= o < tile_rows * 128 and o % 2 == 0
                seen.add(o)
        assert len(seen) == tile_rows * 64


def test_the_bank_model_sees_the_conflict_of_the_32_row_swizzle_under_16_row_fragments():
    """what the counters showed on the earlier 16-row kernels (one extra pass per 16-byte fragment read): rows
    l % 16, chunk l / 16 under the swizzle made for 32-row fragments"""
    addr = []
    for lane in range(64):
        row, chunk = lane % 16, lane // 16
        addr.append(G.mg_lds_store_offset(True, 32, 256, row, 8 * chunk))
    assert cycles(addr, 16, PASSES_16B) == 8


def test_invalid_arguments():
    assert G.mg_lds_store_offset(True, 24, 256, 0, 0) == -1
    assert G.mg_lds_store_offset(True, 16, 256, 256, 0) == -1
    assert G.mg_lds_store_offset(False, 16, 64, 0, 0) == -1
    assert G.mg_lds_read_offset(True, 16, 256, 32, 0, 0, 0) == -1
    assert G.mg_lds_read_offset(True, 16, 256, 0, 64, 0, 0) == -1
    assert G.mg_lds_read_offset(True, 16, 256, 0, 0, 0, 2) == -1
    assert G.mg_lds_read_offset(False, 32, 256, 0, 0, 0, 0, 2) == -1

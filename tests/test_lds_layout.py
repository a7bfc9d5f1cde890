"""Host-only checks of the local-memory layout of the macro-tile kernels (paper Section 3.2: the layout of
the tiles in local memory is tuned because bank conflicts cost).  The library exports the address formulas its
kernels are built from; here they are run through (1) the definition of what a lane must receive and (2) a model
of the LDS banks of gfx950.

Bank model (measured on the GPU by timing reads in which one lane was given another lane's bank): 64 banks of 4
bytes; lanes that read the same address share one access; an 8-byte read is served 32 consecutive lanes at a
time; a 16-byte access 16 lanes at a time, namely lanes {0-3, 12-15, 20-27}, then {4-11, 16-19, 28-31}, and the
same in the upper half of the wavefront; a 4-byte read all 64 lanes at once."""
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


PASS_4B = [list(range(64))]


@pytest.mark.parametrize("tile_rows", [64, 128, 256])
def test_fp32_fragment_reads_fetch_the_right_elements_without_conflicts(tile_rows):
    """FP32 tiles: [row][k] is read 16 bytes per lane, [k][row] one float at a time (all 64 lanes in one clock when
    they hit 64 different banks)"""
    for wave_row in range(0, tile_rows, 32):
        for f, s in itertools.product(range((tile_rows - wave_row) // 32), range(4)):
            addr = [G.mg_lds_f32_read_offset(True, tile_rows, wave_row, lane, f, s) for lane in range(64)]
            for lane in range(64):
                row, k0 = wave_row + 32 * f + lane % 32, 8 * s + 4 * (lane // 32)
                for e in range(4):
                    assert G.mg_lds_f32_store_offset(True, tile_rows, row, k0 + e) == addr[lane] + 4 * e
                    assert G.mg_lds_f32_read_offset(True, tile_rows, wave_row, lane, f, s, e) == addr[lane] + 4 * e
            assert cycles(addr, 16, PASSES_16B) == 4, (tile_rows, wave_row, f, s)
            for e in range(4):
                addr = [G.mg_lds_f32_read_offset(False, tile_rows, wave_row, lane, f, s, e) for lane in range(64)]
                for lane in range(64):
                    row, k = wave_row + 32 * f + lane % 32, 8 * s + 4 * (lane // 32) + e
                    assert G.mg_lds_f32_store_offset(False, tile_rows, row, k) == addr[lane]
                assert cycles(addr, 4, PASS_4B) == 1, (tile_rows, wave_row, f, s, e)


@pytest.mark.parametrize("tile_rows,threads", [(64, 256), (128, 256), (256, 256), (256, 512)])
def test_fp32_loader_stores_are_conflict_free(tile_rows, threads):
    """the loaders' 16-byte stores: thread t + Q * threads holds piece number idx of the tile; [row][k]: row idx / 8,
    chunk idx % 8; [k][row]: line idx / (rows / 4), row chunk idx % (rows / 4)"""
    for first in range(0, tile_rows * 8, 64):             # one wavefront's store instruction
        by_k, by_row = [], []
        for idx in range(first, first + 64):
            by_k.append(G.mg_lds_f32_store_offset(True, tile_rows, idx // 8, 4 * (idx % 8)))
            by_row.append(G.mg_lds_f32_store_offset(False, tile_rows, 4 * (idx % (tile_rows // 4)), idx // (tile_rows // 4)))
        assert cycles(by_k, 16, PASSES_16B) == 4 and cycles(by_row, 16, PASSES_16B) == 4, (tile_rows, first)


def test_fp32_every_element_has_its_own_place():
    for k_contiguous, tile_rows in itertools.product((True, False), (64, 128, 256)):
        seen = {G.mg_lds_f32_store_offset(k_contiguous, tile_rows, row, k) for row in range(tile_rows) for k in range(32)}
        assert len(seen) == tile_rows * 32 and min(seen) == 0 and max(seen) == tile_rows * 128 - 4
        assert all(o % 4 == 0 for o in seen)


def test_the_bank_model_sees_the_conflict_of_unshifted_lines():
    """[k][row] without the half-bank-row shift of every other group of four lines: the two halves of the
    wavefront read the same rows of two lines, i.e. the same banks"""
    addr = [(4 * (lane // 32)) * 4 * 128 + 4 * (lane % 32) for lane in range(64)]
    assert cycles(addr, 4, PASS_4B) == 2


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
    assert G.mg_lds_f32_store_offset(True, 96, 0, 0) == -1
    assert G.mg_lds_f32_store_offset(False, 64, 0, 32) == -1
    assert G.mg_lds_f32_read_offset(False, 64, 32, 0, 1, 0, 0) == -1
    assert G.mg_lds_f32_read_offset(False, 64, 16, 0, 0, 0, 0) == -1
    assert G.mg_lds_f32_read_offset(True, 64, 0, 0, 0, 4, 0) == -1

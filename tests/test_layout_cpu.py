"""CPU tests of the tile layout: the numpy layout reference (tests/layout_ref.py) against positions worked out by
hand from the specification, its two directions against each other, and the library's own field reader
(pq_layout.h, compiled for the host) against tiles that the numpy reference wrote."""
import os
import subprocess
import sys

import numpy as np
import pytest

from tests import layout_ref

HERE = os.path.dirname(os.path.abspath(__file__))


def records_with(n, tau_b_field_value, seed=None):
    """n canonical records, random (seeded) or all zero, as the inverse of layout_ref._record_codes would see them."""
    if seed is None:
        return np.zeros((n, 62), dtype=np.uint8)
    return np.random.default_rng(seed).integers(0, 256, (n, 62), dtype=np.uint8)


def set_field(rec, tau, b, field, all_ones=True):
    """Sets every code that makes up `field` of block b of record tau to its maximum (canonical record order)."""
    def put(level_byte0, index, width):  # codes are packed `8 // width` per byte, earlier code in the higher bits
        per = 8 // width
        byte, pos = level_byte0 + index // per, index % per
        rec[tau, byte] |= ((1 << width) - 1) << (8 - width * (pos + 1))
    if field[0] == "Q":
        j = int(field[1])
        put(0, 8 * b + 2 * j, 4)       # c1 of pair 2j
        put(0, 8 * b + 2 * j + 1, 4)   # c1 of pair 2j+1
        put(32, 4 * b + j, 2)          # c2 of node j
    else:
        put(44, b, 2)                  # c4
        put(40, 2 * b, 2)              # c3 of half 0
        put(40, 2 * b + 1, 2)          # c3 of half 1


def test_fields_land_where_the_specification_puts_them():
    path = os.path.join(HERE, "golden", "tile_positions_hand_built.txt")
    cases = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(cases) >= 10
    for c in cases:
        kind, tau, b, field = int(c[0]), int(c[1]), int(c[2]), c[3]
        pieces = [(int(c[i]), int(c[i + 1]), int(c[i + 2])) for i in range(4, len(c), 3)]
        assert sum(p[2] for p in pieces) == (6 if field == "B" else 10)
        rec = np.zeros((64, 62), dtype=np.uint8)
        set_field(rec, tau, b, field)
        codes, radii = layout_ref.canonical_to_tiles(kind, rec)
        want = np.zeros(layout_ref.CODE_BYTES, dtype=np.uint8)
        for byte, first, width in pieces:
            want[byte] |= ((1 << width) - 1) << first
        assert np.array_equal(codes[0], want), (c, np.nonzero(codes[0])[0], np.nonzero(want)[0])
        assert not radii.any()


@pytest.mark.parametrize("kind", [0, 1])
def test_several_planes_in_one_pass_equal_one_plane_at_a_time(kind):
    n = 64 * 2 + 9
    planes = np.stack([records_with(n, None, seed=20 + 3 * kind + g) for g in range(3)])
    codes, radii = layout_ref.canonical_to_tiles_planes(kind, planes, 4, fill=0xC3)
    assert codes.shape == (3, 4, layout_ref.CODE_BYTES) and radii.shape == (3, 4, layout_ref.RADII)
    for g in range(3):
        c1, r1 = layout_ref.canonical_to_tiles(kind, planes[g], 4, fill=0xC3)
        assert np.array_equal(codes[g], c1) and np.array_equal(radii[g], r1)
        assert np.array_equal(layout_ref.tiles_to_canonical(kind, codes[g], radii[g], n), planes[g])
    assert np.all(codes[:, 3] == 0xC3) and np.all(radii[:, 3] == 0xC3C3)   # a tile without records keeps the fill


@pytest.mark.parametrize("kind", [0, 1])
def test_round_trip_and_full_coverage(kind):
    n = 64 * 3 + 17
    rec = records_with(n, None, seed=10 + kind)
    codes, radii = layout_ref.canonical_to_tiles(kind, rec, fill=0xA5)
    assert codes.shape == (4, layout_ref.CODE_BYTES) and radii.shape == (4, layout_ref.RADII)
    assert np.array_equal(layout_ref.tiles_to_canonical(kind, codes, radii, n), rec)
    # every bit of a full tile belongs to exactly one field: the fill value of unwritten bits cannot show there
    codes0, radii0 = layout_ref.canonical_to_tiles(kind, rec, fill=0x00)
    assert np.array_equal(codes[:3], codes0[:3]) and np.array_equal(radii[:3], radii0[:3])
    # slots beyond the records keep the fill
    tail = layout_ref.tiles_to_canonical(kind, codes, radii, 256)[n:]
    assert np.all(tail[:, 46:] == 0xA5)
    # 62 bytes per token exactly
    assert (layout_ref.CODE_BYTES + 2 * layout_ref.RADII) == 62 * 64
    # deep format
    rec50 = np.random.default_rng(20 + kind).integers(0, 256, (n, 50), dtype=np.uint8)
    c, t = layout_ref.canonical_to_tiles_deep(kind, rec50)
    assert t.shape == (4, 128)
    assert np.array_equal(layout_ref.tiles_to_canonical_deep(kind, c, t, n), rec50)


def test_record_unpackers_follow_the_record_specification():
    rec = np.zeros((1, 62), dtype=np.uint8)
    rec[0, 0] = 0x9C                      # codes of coordinates pairs 0, 1: 9 then 12
    rec[0, 33] = 0b11_01_00_10            # level-2 codes of nodes 4..7: 3, 1, 0, 2
    rec[0, 41] = 0b00_10_00_00            # level-3 code of node 5: 2
    rec[0, 45] = 0b00_00_00_11            # level-4 code of block 7: 3
    rec[0, 46 + 6], rec[0, 46 + 7] = 0x34, 0x12   # radius of block 3, little endian
    J, r = layout_ref.unpack_canonical(rec)
    assert J.shape == (1, 120) and r.shape == (1, 8)
    assert J[0, 0] == 9 and J[0, 1] == 12 and list(J[0, 64 + 4:64 + 8]) == [3, 1, 0, 2]
    assert J[0, 96 + 5] == 2 and J[0, 112 + 7] == 3 and r[0, 3] == 0x1234
    assert J.sum() == 9 + 12 + 3 + 1 + 2 + 2 + 3
    rec50 = np.zeros((1, 50), dtype=np.uint8)
    rec50[0, 46], rec50[0, 47] = 0b1011_0110, 0b0000_0101     # word 0x05B6
    rec50[0, 48], rec50[0, 49] = 0xCD, 0xAB
    J, r = layout_ref.unpack_canonical_deep(rec50, (2, 3, 1))   # level 5: 4 x 2 bits, level 6: 2 x 3 bits, level 7: 1 bit
    assert list(J[0, 120:]) == [2, 1, 3, 2, 5, 0, 0] and r[0] == 0xABCD


@pytest.mark.parametrize("kind", [0, 1])
def test_library_field_reader_agrees_with_the_numpy_reference(kind, tmp_path):
    """pq_layout.h, compiled for the host, reads back what the numpy reference wrote."""
    exe = str(tmp_path / "layout_host_check")
    src = os.path.join(HERE, "layout_host_check.cpp")
    subprocess.run(["g++", "-O1", "-std=c++17", src, "-o", exe], check=True)
    n = 128
    rec = np.random.default_rng(30 + kind).integers(0, 256, (n, 62), dtype=np.uint8)
    codes, radii = layout_ref.canonical_to_tiles(kind, rec)
    blob = np.array([kind, 2], dtype=np.int32).tobytes()
    for t in range(2):
        blob += codes[t].tobytes() + radii[t].tobytes()
    out = subprocess.run([exe], input=blob, stdout=subprocess.PIPE, check=True).stdout.decode().split("\n")
    got = np.array([[int(v) for v in line.split()] for line in out if line], dtype=np.int64).reshape(n, 8, 5)
    J, r = layout_ref.unpack_canonical(rec)
    for tau in range(n):
        for b in range(8):
            l1, g0, g1, c4, radius = got[tau, b]
            c1 = [(l1 >> (4 * p)) & 15 for p in range(8)]
            assert c1 == list(J[tau, 8 * b:8 * b + 8])
            c2 = [g0 >> 4, g0 & 3, g1 >> 4, g1 & 3]
            assert c2 == list(J[tau, 64 + 4 * b:64 + 4 * b + 4])
            assert [(g0 >> 2) & 3, (g1 >> 2) & 3] == list(J[tau, 96 + 2 * b:96 + 2 * b + 2])
            assert c4 == J[tau, 112 + b] and radius == r[tau, b]

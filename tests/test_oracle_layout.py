"""Pins for oracle.layout: the tile order is a bijection and matches its written definition, re-derived here
with plain loops."""
import numpy as np

from oracle import layout


def _slot_of_position(n, j, k):
    """Word index and code index p of contraction position k of row (n, j), by search over the header's statement:
    word ((n // 2) * 64 + j + 16 g) * 4 + 2 (n % 2) + w, code p at k = 32 g + 16 w + 8 (p % 2) + p // 2."""
    for g in range(4):
        for w in range(2):
            for p in range(16):
                if 32 * g + 16 * w + 8 * (p % 2) + p // 2 == k:
                    return ((n // 2) * 64 + j + 16 * g) * 4 + 2 * (n % 2) + w, p
    raise AssertionError


def _code_at(word, p):
    """The header's bit format: hi in bit 4 (p // 2) + 3 - p % 2, lo in bit 4 (p // 2) + 1 - p % 2; (hi, lo) = (1,1),
    (1,0), (0,0), (0,1) for the codes 0, 1, 2, 3."""
    hi = (int(word) >> (4 * (p // 2) + 3 - p % 2)) & 1
    lo = (int(word) >> (4 * (p // 2) + 1 - p % 2)) & 1
    return {(1, 1): 0, (1, 0): 1, (0, 0): 2, (0, 1): 3}[(hi, lo)]


def _word_with(p, code):
    hi, lo = {0: (1, 1), 1: (1, 0), 2: (0, 0), 3: (0, 1)}[code]
    return (hi << (4 * (p // 2) + 3 - p % 2)) | (lo << (4 * (p // 2) + 1 - p % 2))


def _k_slot(t, c):
    return _slot_of_position(t // 16, t % 16, c)  # row = token, position = channel


def _v_slot(t, c):
    for k in range(128):  # row = channel, position k holds token 16 (k % 8) + 4 ((k // 16) % 4) + 2 (k // 64) + (k // 8) % 2
        if 16 * (k % 8) + 4 * ((k // 16) % 4) + 2 * (k // 64) + (k // 8) % 2 == t:
            return _slot_of_position(c // 16, c % 16, k)
    raise AssertionError


def test_tiles_are_bijections_and_match_the_definition():
    rng = np.random.default_rng(0)
    codes = rng.integers(0, 4, size=(128, 128))
    for pack, unpack, slot in ((layout.pack_k_tile, layout.unpack_k_tile, _k_slot),
                               (layout.pack_v_tile, layout.unpack_v_tile, _v_slot)):
        tile = pack(codes)
        assert tile.shape == (1024,) and tile.dtype == np.uint32
        assert np.array_equal(unpack(tile), codes)
        seen = set()
        for t in range(0, 128, 7):
            for c in range(128):
                w, p = slot(t, c)
                assert _code_at(tile[w], p) == codes[t, c]
                seen.add((w, p))
        assert len(seen) == len(range(0, 128, 7)) * 128
        # a tile of code 2 is all zero bits; one other code in it sets exactly its own bit pair
        base = np.full((128, 128), 2, dtype=np.int64)
        assert not pack(base).any()
        base[70, 9] = 0
        w, p = slot(70, 9)
        t1 = pack(base)
        assert t1[w] == _word_with(p, 0) and np.count_nonzero(t1) == 1


def test_literal_corners():
    """Hand-placed codes in a tile of code 2 (which is stored as zero bits)."""
    def one(t, c, code):
        a = np.full((128, 128), 2, dtype=np.int64)
        a[t, c] = code
        return a
    # key: token 0 -> block 0, row 0; channel 1 = position 1 -> g 0, w 0, p 2 -> word 0, nibble 1, bits 7 (hi) and 5 (lo)
    assert layout.pack_k_tile(one(0, 1, 0))[0] == (1 << 7) | (1 << 5)
    assert layout.pack_k_tile(one(0, 1, 1))[0] == 1 << 7
    assert layout.pack_k_tile(one(0, 1, 3))[0] == 1 << 5
    # channel 8 -> p 1 of the same word: nibble 0, bits 2 (hi) and 0 (lo)
    assert layout.pack_k_tile(one(0, 8, 0))[0] == (1 << 2) | 1
    # key: token 1 -> row j = 1 -> word 4; p 0 -> bits 3 and 1
    assert layout.pack_k_tile(one(1, 0, 1))[4] == 1 << 3
    # key: token 16 -> block 1 (odd block: + 2); channel 16 -> w 1, p 0 -> word 3
    assert layout.pack_k_tile(one(16, 16, 3))[3] == 1 << 1
    # key: token 33 -> block 2, row 1; channel 40 -> g 1, w 0, p 1 -> word (64 + 1 + 16) * 4, bits 2 and 0
    assert layout.pack_k_tile(one(33, 40, 1))[(64 + 17) * 4] == 1 << 2
    # value: channel 0 -> block 0 row 0; token 16 = position 1 (k % 8 = 1) -> p 2 of word 0
    assert layout.pack_v_tile(one(16, 0, 3))[0] == 1 << 5
    # value: channel 64 -> block 4, row 0 -> words from 2 * 64 * 4; token 1 = position 8 -> p 1
    assert layout.pack_v_tile(one(1, 64, 0))[512] == (1 << 2) | 1
    # value: channel 17 -> block 1, row 1; token 2 = position 64 -> g 2 -> word (1 + 32) * 4 + 2, p 0
    assert layout.pack_v_tile(one(2, 17, 1))[(1 + 32) * 4 + 2] == 1 << 3


def test_state_tiles_are_a_bijection():
    rng = np.random.default_rng(5)
    S = rng.standard_normal((256, 128)).astype(np.float16)
    tiles = layout.pack_state_tiles(S)
    assert tiles.shape == (128, 64, 4)
    assert np.array_equal(layout.unpack_state_tiles(tiles).view(np.uint16), S.view(np.uint16))
    # the stated index map, element by element on a few entries
    for f, c in [(0, 0), (3, 5), (64, 63), (130, 64), (255, 127), (77, 100)]:
        t = (f // 64 * 2 + c // 64) * 16 + (f % 64) // 4
        assert tiles[t, c % 64, f % 4] == S[f, c]


def test_record_fields_sit_where_the_header_says():
    """include/kvlinc.h: a record is 2304 words -- key tile [0, 1024), value tile [1024, 2048), key scale [2048, 2112)
    and key zero-point [2112, 2176) as fp16 pairs (channel 2i in the low half of word i), then one word per token
    (token 16 n + j in word 2176 + 8 j + n) with the value scale in the low and the value zero-point in the high half."""
    z = lambda *shape: np.zeros(shape, dtype=np.float16)
    codes0 = np.full((1, 128, 128), 2, dtype=np.int64)  # code 2 is stored as zero bits

    def record(**fields):
        f = dict(k_codes=codes0, v_codes=codes0, k_scale=z(1, 128), k_zero=z(1, 128), v_scale=z(1, 128),
                 v_zero=z(1, 128))
        f.update(fields)
        return layout.pack_records(f["k_codes"], f["v_codes"], f["k_scale"], f["k_zero"], f["v_scale"], f["v_zero"])[0]

    one = codes0.copy()
    one[0, 0, 0] = 3  # code 3 = bit pair (0, 1), p 0: lo in bit 1
    r = record(k_codes=one)
    assert r.shape == (2304,) and r[0] == 2 and np.count_nonzero(r) == 1
    r = record(v_codes=one)
    assert r[1024] == 2 and np.count_nonzero(r) == 1
    h = z(1, 128)
    h[0, 5] = 1.5  # fp16 0x3E00; channel 5 = high half of word 2
    r = record(k_scale=h)
    assert r[2048 + 2] == 0x3E00 << 16 and np.count_nonzero(r) == 1
    r = record(k_zero=h)
    assert r[2112 + 2] == 0x3E00 << 16 and np.count_nonzero(r) == 1
    r = record(v_scale=h)  # token 5 = 16 * 0 + 5 -> word 2176 + 8 * 5 + 0
    assert r[2176 + 40] == 0x3E00 and np.count_nonzero(r) == 1
    r = record(v_zero=h)
    assert r[2176 + 40] == 0x3E00 << 16 and np.count_nonzero(r) == 1
    h2 = z(1, 128)
    h2[0, 35] = 1.5  # token 35 = 16 * 2 + 3 -> word 2176 + 8 * 3 + 2
    r = record(v_scale=h2)
    assert r[2176 + 26] == 0x3E00 and np.count_nonzero(r) == 1
    # and the whole record round-trips
    rng = np.random.default_rng(3)
    f = dict(k_codes=rng.integers(0, 4, size=(2, 128, 128)), v_codes=rng.integers(0, 4, size=(2, 128, 128)),
             k_scale=rng.standard_normal((2, 128)).astype(np.float16), k_zero=rng.standard_normal((2, 128)).astype(np.float16),
             v_scale=rng.standard_normal((2, 128)).astype(np.float16), v_zero=rng.standard_normal((2, 128)).astype(np.float16))
    back = layout.unpack_records(layout.pack_records(**f))
    for name, want in f.items():
        got = back[name]
        if want.dtype == np.float16:
            assert np.array_equal(got.view(np.uint16), want.view(np.uint16)), name
        else:
            assert np.array_equal(got, want), name


def test_value_window_order():
    """include/kvlinc.h: v_res is [R / 4][128][4] -- the rotated value of window token 4 i + k, channel c, sits at
    [i][c][k]; unused rows are zero."""
    rows = np.arange(5 * 128, dtype=np.float16).reshape(5, 128) / np.float16(8)
    tiled = layout.pack_value_window(rows, 128)
    assert tiled.shape == (32, 128, 4) and tiled.dtype == np.float16
    for t, c in [(0, 0), (1, 0), (3, 127), (4, 64)]:
        assert tiled[t // 4, c, t % 4] == rows[t, c]
    assert not tiled[1, :, 1:].any() and not tiled[2:].any()
    assert np.array_equal(layout.unpack_value_window(tiled, 5), rows)


# ---- 4-bit records: two 2-bit planes per tile ----------------------------------------------------------------

def test_four_bit_record_is_two_planes_per_tile():
    rng = np.random.default_rng(5)
    k_codes = rng.integers(0, 16, size=(2, 128, 128))
    v_codes = rng.integers(0, 16, size=(2, 128, 128))
    par = [rng.standard_normal((2, 128)).astype(np.float16) for _ in range(4)]
    rec = layout.pack_records4(k_codes, v_codes, *par)
    assert rec.shape == (2, 4352) and rec.dtype == np.uint32
    back = layout.unpack_records4(rec)
    assert np.array_equal(back["k_codes"], k_codes) and np.array_equal(back["v_codes"], v_codes)
    for got, want in zip((back["k_scale"], back["k_zero"], back["v_scale"], back["v_zero"]), par):
        assert np.array_equal(got.view(np.uint16), want.view(np.uint16))
    # every plane is a 2-bit tile (whose order the tests above pin) of one base-4 digit of the codes, read off here
    # with the search over the stated order
    for t in range(0, 128, 9):
        for c in range(0, 128, 7):
            w, p = _slot_of_position(t // 16, t % 16, c)
            digits = (_code_at(rec[1, w], p), _code_at(rec[1, 1024 + w], p))
            assert 4 * digits[0] + digits[1] == k_codes[1, t, c]
            kpos = [k for k in range(128) if 16 * (k % 8) + 4 * ((k // 16) % 4) + 2 * (k // 64) + (k // 8) % 2 == t][0]
            w, p = _slot_of_position(c // 16, c % 16, kpos)
            digits = (_code_at(rec[1, 2048 + w], p), _code_at(rec[1, 3072 + w], p))
            assert 4 * digits[0] + digits[1] == v_codes[1, t, c]
    # scales and zero-points behind the four planes, in the order of the 2-bit record
    assert np.array_equal(rec[0, 4096:4160], layout._halves_to_words(par[0])[0])
    assert np.array_equal(rec[0, 4160:4224], layout._halves_to_words(par[1])[0])
    t = 16 * 3 + 5  # token 16 n + j, n = 3, j = 5 -> word 8 j + n of the field
    assert rec[0, 4224 + 8 * 5 + 3] == int(par[2].view(np.uint16)[0, t]) | (int(par[3].view(np.uint16)[0, t]) << 16)


def test_four_bit_literal_corners():
    def one(t, c, code):
        a = np.full((1, 128, 128), 10, dtype=np.int64)  # code 10 = digits (2, 2) -> bit pairs (0, 0): planes of zeros
        a[0, t, c] = code
        return a
    z = np.zeros((1, 128), dtype=np.float16)
    k_of = lambda a: layout.pack_records4(a, np.full((1, 128, 128), 10), z, z, z, z)[0, :2048]
    v_of = lambda a: layout.pack_records4(np.full((1, 128, 128), 10), a, z, z, z, z)[0, 2048:4096]
    assert not k_of(np.full((1, 128, 128), 10)).any()
    # token 0, channel 0 -> code p = 0 of word 0 of a plane: hi in bit 3, lo in bit 1
    # code 2 = digits (0, 2): high plane (1, 1), low plane untouched; code 8 = digits (2, 0): the other way round
    t = k_of(one(0, 0, 2))
    assert t[0] == 0b1010 and t[1024] == 0 and np.count_nonzero(t) == 1
    t = k_of(one(0, 0, 8))
    assert t[0] == 0 and t[1024] == 0b1010 and np.count_nonzero(t) == 1
    # code 7 = digits (1, 3): high plane (1, 0), low plane (0, 1); code 15 = (3, 3): (0, 1) in both
    t = k_of(one(0, 0, 7))
    assert t[0] == 0b1000 and t[1024] == 0b0010
    t = k_of(one(0, 0, 15))
    assert t[0] == 0b0010 and t[1024] == 0b0010
    # value tile: channel 3 = row 3, token 16 = position 1 -> p = 2 -> bits 7 and 5 of word 3 * 4 of each plane
    t = v_of(one(16, 3, 1))  # digits (0, 1): (1, 1) high, (1, 0) low
    assert t[12] == 0b1010 << 4 and t[1024 + 12] == 0b1000 << 4 and np.count_nonzero(t) == 2

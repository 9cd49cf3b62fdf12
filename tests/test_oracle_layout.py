"""Pins for oracle.layout: the tile order is a bijection and matches its written definition, re-derived here
with plain loops."""
import numpy as np

from oracle import layout


def _k_slot(t, c):
    hf, l = divmod(t, 64)
    for q in range(8):
        for j in range(8):
            for e in range(2):
                if 8 * (4 * (q % 4) + j // 2) + 4 * (q // 4) + 2 * (j % 2) + e == c:
                    return ((hf * 2 + q // 4) * 64 + l) * 4 + q % 4, 2 * j + 16 * e
    raise AssertionError


def _v_slot(t, c):
    ch, l = divmod(c, 64)
    hf = t // 64
    for w in range(4):
        for j in range(8):
            for e in range(2):
                if 64 * hf + 4 * (4 * w + j // 2) + 2 * (j % 2) + e == t:
                    return ((hf * 2 + ch) * 64 + l) * 4 + w, 2 * j + 16 * e
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
                w, s = slot(t, c)
                assert (int(tile[w]) >> s) & 3 == codes[t, c]
                seen.add((w, s))
        assert len(seen) == len(range(0, 128, 7)) * 128
        one = np.zeros((128, 128), dtype=np.int64)
        one[70, 9] = 3
        w, s = slot(70, 9)
        t1 = pack(one)
        assert t1[w] == 3 << s and np.count_nonzero(t1) == 1


def test_literal_corners():
    one = np.zeros((128, 128), dtype=np.int64)
    one[0, 1] = 1  # key: token 0, channel 1 -> word 0, second element of pair 0 -> bit 16
    assert layout.pack_k_tile(one)[0] == 1 << 16
    one[:] = 0
    one[1, 0] = 2  # key: token 1 -> lane 1 -> word 4
    assert layout.pack_k_tile(one)[4] == 2
    one[:] = 0
    one[1, 0] = 1  # value: channel 0, token 1 -> word 0, second element of pair 0
    assert layout.pack_v_tile(one)[0] == 1 << 16
    one[:] = 0
    one[0, 64] = 3  # value: channel 64 = second channel half, lane 0 -> word (0*2+1)*64*4
    assert layout.pack_v_tile(one)[256] == 3


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
    and key zero-point [2112, 2176) as fp16 pairs (channel 2i in the low half of word i), then one word per token with
    the value scale in the low and the value zero-point in the high half."""
    z = lambda *shape: np.zeros(shape, dtype=np.float16)
    codes0 = np.zeros((1, 128, 128), dtype=np.int64)

    def record(**fields):
        f = dict(k_codes=codes0, v_codes=codes0, k_scale=z(1, 128), k_zero=z(1, 128), v_scale=z(1, 128),
                 v_zero=z(1, 128))
        f.update(fields)
        return layout.pack_records(f["k_codes"], f["v_codes"], f["k_scale"], f["k_zero"], f["v_scale"], f["v_zero"])[0]

    one = codes0.copy()
    one[0, 0, 0] = 3
    r = record(k_codes=one)
    assert r.shape == (2304,) and r[0] == 3 and np.count_nonzero(r) == 1
    r = record(v_codes=one)
    assert r[1024] == 3 and np.count_nonzero(r) == 1
    h = z(1, 128)
    h[0, 5] = 1.5  # fp16 0x3E00; channel 5 = high half of word 2
    r = record(k_scale=h)
    assert r[2048 + 2] == 0x3E00 << 16 and np.count_nonzero(r) == 1
    r = record(k_zero=h)
    assert r[2112 + 2] == 0x3E00 << 16 and np.count_nonzero(r) == 1
    r = record(v_scale=h)
    assert r[2176 + 5] == 0x3E00 and np.count_nonzero(r) == 1
    r = record(v_zero=h)
    assert r[2176 + 5] == 0x3E00 << 16 and np.count_nonzero(r) == 1
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

"""Physical order of the quantized cache: one 9216-byte record per group of 128 tokens, holding two 4 KB tiles of
packed 2-bit codes (1024 32-bit words per 128x128 block) and the group's scales and zero-points.

The paper fixes only that 16 two-bit codes share a 32-bit word (Sec. 3.3; K_I in R^{N/16 x d},
V_I in R^{N x d/16} in Alg. 1).  The logical content -- one code per (token, channel) -- is the
contract; the order inside a tile is an encoding chosen for the decode kernel and is written
down here independently of the kernel source.

Tile order (both tiles, the header's statement): a tile has 8 blocks n of 16 rows j; every row has 128
contraction positions k in 4 quarters g of 32.  The two words w = 0, 1 of (n, j, g) sit at word index

    ((n // 2) * 64 + j + 16 * g) * 4 + 2 * (n % 2) + w

and code p (0..15) of a word belongs to position k = 32 g + 16 w + 8 (p % 2) + p // 2.  A code c is stored as the bit
pair (hi, lo) = (1,1), (1,0), (0,0), (0,1) for c = 0, 1, 2, 3; code p keeps hi in bit 4 (p // 2) + 3 - p % 2 and lo in
bit 4 (p // 2) + 1 - p % 2 of its word (two codes share a nibble).

Key tile:   row (n, j) = token 16 n + j; position k = channel k.
Value tile: row (n, j) = channel 16 n + j; position k = token 16 (k % 8) + 4 ((k // 16) % 4) + 2 (k // 64) + (k // 8) % 2.

Group record, 2304 words (everything one decode step needs of a group, contiguous in memory):
    words    0 .. 1023   key tile
    words 1024 .. 2047   value tile
    words 2048 .. 2111   key scale, fp16 per channel 0..127 (two per word, low half first)
    words 2112 .. 2175   key zero-point, fp16 per channel
    words 2176 .. 2303   value (scale, zero-point) of token t = 16 n + j in word 2176 + 8 j + n: scale in the low half,
                         zero in the high

State tiles: the binary16 copy of S [256 features, 128 channels] that the decode step reads is stored as 128 tiles of
64 x 4 halves; tile (f // 64 * 2 + c // 64) * 16 + (f % 64) // 4 holds S[f][c] at [c % 64][f % 4].

4-bit codes (Eq. 1 at N = 4; `bits` = 4 in the cache descriptor): a code c = 4 c_hi + c_lo is stored as two 2-bit
codes, c_hi = c // 4 and c_lo = c % 4, each in a 2-bit tile of its own ("plane") with the order and the bit pairs above.
A record has 4352 words (17408 bytes): key tile high plane 0..1023, key tile low plane 1024..2047, value tile high
plane 2048..3071, value tile low plane 3072..4095, key scale 4096..4159, key zero-point 4160..4223, value (scale,
zero-point) 4224..4351 in the order above.  (c - 7.5 = 4 (c_hi - 1.5) + (c_lo - 1.5): a contraction with the codes is
the sum of the contractions with the two planes, the high one weighted by 4.)

Window of fp16 values: rotated values are stored 4 consecutive tokens per channel, v_res[slot // 4][channel][slot % 4],
so that a lane owning a channel reads 4 tokens with one 8-byte load; keys stay row-major k_res[slot][channel].
"""
import numpy as np

TILE_WORDS = 1024
RECORD_WORDS = 2304


SYMBOL_OF_CODE = np.array([0b11, 0b10, 0b00, 0b01], dtype=np.uint32)  # (hi, lo) of code 0, 1, 2, 3
CODE_OF_SYMBOL = np.array([2, 3, 1, 0], dtype=np.uint8)


def _position_maps():
    """For every (row r = 16 n + j, position k) of a tile: word index and the index p of its code inside the word."""
    r = np.arange(128)[:, None]
    k = np.arange(128)[None, :]
    n, j = r // 16, r % 16
    g = k // 32
    w = (k % 32) // 16
    # k % 16 = 8 (p % 2) + p // 2  <=>  p = 2 (k % 8) + (k % 16) // 8
    p = 2 * (k % 8) + (k % 16) // 8
    word = ((n // 2) * 64 + j + 16 * g) * 4 + 2 * (n % 2) + w
    return np.broadcast_to(word, (128, 128)), np.broadcast_to(p, (128, 128))


def _value_token_of_position():
    k = np.arange(128)
    return 16 * (k % 8) + 4 * ((k // 16) % 4) + 2 * (k // 64) + (k // 8) % 2


def _k_index_maps():
    """[token, channel] -> (word, p): rows are tokens, position k is channel k."""
    return _position_maps()


def _v_index_maps():
    """[token, channel] -> (word, p): rows are channels, position k holds token _value_token_of_position()[k]."""
    word_rk, shift_rk = _position_maps()          # [channel row, position]
    tok = _value_token_of_position()
    assert sorted(tok.tolist()) == list(range(128))
    word = np.empty((128, 128), dtype=np.int64)
    shift = np.empty((128, 128), dtype=np.int64)
    word[tok[None, :], np.arange(128)[:, None]] = word_rk
    shift[tok[None, :], np.arange(128)[:, None]] = shift_rk
    return word, shift


_K_WORD, _K_SHIFT = _k_index_maps()
_SZ_WORD = 8 * (np.arange(128) % 16) + np.arange(128) // 16  # word (after 2176) of token t = 16 n + j: 8 j + n
_V_WORD, _V_SHIFT = _v_index_maps()


def _pack(codes, word, p):
    codes = np.asarray(codes)
    assert codes.shape[-2:] == (128, 128) and codes.min() >= 0 and codes.max() <= 3
    lead = codes.shape[:-2]
    sym = SYMBOL_OF_CODE[codes.reshape((-1, 128 * 128))]
    out = np.zeros((sym.shape[0], TILE_WORDS), dtype=np.uint32)
    wi = word.reshape(-1)
    pp = p.reshape(-1).astype(np.uint32)
    hi_bit = 4 * (pp // 2) + 3 - pp % 2
    lo_bit = 4 * (pp // 2) + 1 - pp % 2
    for n in range(sym.shape[0]):
        np.bitwise_or.at(out[n], wi, ((sym[n] >> np.uint32(1)) << hi_bit) | ((sym[n] & np.uint32(1)) << lo_bit))
    return out.reshape(lead + (TILE_WORDS,))


def _unpack(tile, word, p):
    tile = np.asarray(tile, dtype=np.uint32)
    assert tile.shape[-1] == TILE_WORDS
    pp = p.astype(np.uint32)
    w = tile[..., word]
    hi = (w >> (4 * (pp // 2) + 3 - pp % 2)) & np.uint32(1)
    lo = (w >> (4 * (pp // 2) + 1 - pp % 2)) & np.uint32(1)
    return CODE_OF_SYMBOL[2 * hi + lo]


def pack_k_tile(codes):
    """codes[..., token 0..127, channel 0..127] in {0..3} -> uint32[..., 1024]."""
    return _pack(codes, _K_WORD, _K_SHIFT)


def unpack_k_tile(tile):
    return _unpack(tile, _K_WORD, _K_SHIFT)


def pack_v_tile(codes):
    """codes[..., token 0..127, channel 0..127] in {0..3} -> uint32[..., 1024]."""
    return _pack(codes, _V_WORD, _V_SHIFT)


def unpack_v_tile(tile):
    return _unpack(tile, _V_WORD, _V_SHIFT)


# ---- 4-bit codes ------------------------------------------------------------------------------------------------
RECORD_WORDS4 = 4352


def pack_records4(k_codes, v_codes, k_scale, k_zero, v_scale, v_zero):
    """4-bit codes: per-group arrays ([n_groups, 128, 128] codes 0..15, [n_groups, 128] fp16 parameters) -> uint32 [n_groups, 4352]."""
    k_codes, v_codes = np.asarray(k_codes).astype(np.int64), np.asarray(v_codes).astype(np.int64)
    n = k_codes.shape[0]
    rec = np.zeros((n, RECORD_WORDS4), dtype=np.uint32)
    if n == 0:
        return rec
    assert k_codes.min() >= 0 and k_codes.max() <= 15 and v_codes.min() >= 0 and v_codes.max() <= 15
    rec[:, 0:1024] = pack_k_tile(k_codes // 4)
    rec[:, 1024:2048] = pack_k_tile(k_codes % 4)
    rec[:, 2048:3072] = pack_v_tile(v_codes // 4)
    rec[:, 3072:4096] = pack_v_tile(v_codes % 4)
    rec[:, 4096:4160] = _halves_to_words(k_scale)
    rec[:, 4160:4224] = _halves_to_words(k_zero)
    vs = np.ascontiguousarray(v_scale, dtype=np.float16).view(np.uint16).astype(np.uint32)
    vz = np.ascontiguousarray(v_zero, dtype=np.float16).view(np.uint16).astype(np.uint32)
    rec[:, 4224:4352][:, _SZ_WORD] = vs | (vz << np.uint32(16))
    return rec


def unpack_records4(rec):
    """uint32 [n_groups, 4352] -> dict of the logical per-group arrays (inverse of pack_records4)."""
    rec = np.asarray(rec, dtype=np.uint32)
    def halves(words):
        lo = (words & np.uint32(0xFFFF)).astype(np.uint16)
        hi = (words >> np.uint32(16)).astype(np.uint16)
        return np.stack([lo, hi], axis=-1).reshape(words.shape[:-1] + (-1,)).view(np.float16)
    sz = rec[:, 4224:4352][:, _SZ_WORD]
    return {
        "k_codes": 4 * unpack_k_tile(rec[:, 0:1024]) + unpack_k_tile(rec[:, 1024:2048]),
        "v_codes": 4 * unpack_v_tile(rec[:, 2048:3072]) + unpack_v_tile(rec[:, 3072:4096]),
        "k_scale": halves(rec[:, 4096:4160]), "k_zero": halves(rec[:, 4160:4224]),
        "v_scale": (sz & np.uint32(0xFFFF)).astype(np.uint16).view(np.float16),
        "v_zero": (sz >> np.uint32(16)).astype(np.uint16).view(np.float16),
    }


def _halves_to_words(h16):
    """fp16 array [..., 2n] -> uint32 [..., n], element 2i in the low half of word i."""
    u = np.ascontiguousarray(h16, dtype=np.float16).view(np.uint16).astype(np.uint32)
    return u[..., 0::2] | (u[..., 1::2] << np.uint32(16))


def pack_records(k_codes, v_codes, k_scale, k_zero, v_scale, v_zero):
    """Per-group arrays ([n_groups, 128, 128] codes, [n_groups, 128] fp16 parameters) -> uint32 [n_groups, 2304]."""
    n = np.asarray(k_codes).shape[0]
    rec = np.zeros((n, RECORD_WORDS), dtype=np.uint32)
    if n == 0:
        return rec
    rec[:, 0:1024] = pack_k_tile(k_codes)
    rec[:, 1024:2048] = pack_v_tile(v_codes)
    rec[:, 2048:2112] = _halves_to_words(k_scale)
    rec[:, 2112:2176] = _halves_to_words(k_zero)
    vs = np.ascontiguousarray(v_scale, dtype=np.float16).view(np.uint16).astype(np.uint32)
    vz = np.ascontiguousarray(v_zero, dtype=np.float16).view(np.uint16).astype(np.uint32)
    rec[:, 2176:2304][:, _SZ_WORD] = vs | (vz << np.uint32(16))
    return rec


def unpack_records(rec):
    """uint32 [n_groups, 2304] -> dict of the logical per-group arrays (inverse of pack_records)."""
    rec = np.asarray(rec, dtype=np.uint32)
    def halves(words):
        lo = (words & np.uint32(0xFFFF)).astype(np.uint16)
        hi = (words >> np.uint32(16)).astype(np.uint16)
        return np.stack([lo, hi], axis=-1).reshape(words.shape[:-1] + (-1,)).view(np.float16)
    sz = rec[:, 2176:2304][:, _SZ_WORD]
    return {
        "k_codes": unpack_k_tile(rec[:, 0:1024]), "v_codes": unpack_v_tile(rec[:, 1024:2048]),
        "k_scale": halves(rec[:, 2048:2112]), "k_zero": halves(rec[:, 2112:2176]),
        "v_scale": (sz & np.uint32(0xFFFF)).astype(np.uint16).view(np.float16),
        "v_zero": (sz >> np.uint32(16)).astype(np.uint16).view(np.float16),
    }


def pack_value_window(v_rows, R):
    """Rotated fp16 values of the window, [n_res, 128] oldest first -> [R // 4, 128, 4] (unused slots zero)."""
    v_rows = np.asarray(v_rows, dtype=np.float16)
    assert R % 4 == 0 and v_rows.shape[0] <= R
    full = np.zeros((R, 128), dtype=np.float16)
    full[:v_rows.shape[0]] = v_rows
    return np.ascontiguousarray(full.reshape(R // 4, 4, 128).transpose(0, 2, 1))


def unpack_value_window(v_tiled, n_res):
    """[R // 4, 128, 4] -> [n_res, 128]."""
    v_tiled = np.asarray(v_tiled)
    R = v_tiled.shape[0] * 4
    return np.ascontiguousarray(v_tiled.transpose(0, 2, 1).reshape(R, 128)[:n_res])


def pack_state_tiles(S):
    """S [256, 128] -> fp16 [128, 64, 4] in the tile order of the decode step's copy of the state."""
    S = np.asarray(S)
    assert S.shape == (256, 128)
    f = np.arange(256)[:, None]
    c = np.arange(128)[None, :]
    tile = (f // 64 * 2 + c // 64) * 16 + (f % 64) // 4
    out = np.zeros((128, 64, 4), dtype=np.float16)
    out[tile, c % 64, f % 4] = S.astype(np.float16)
    return out


def unpack_state_tiles(tiles):
    """fp16 [128, 64, 4] -> [256, 128] (inverse of pack_state_tiles)."""
    tiles = np.asarray(tiles)
    assert tiles.shape == (128, 64, 4)
    f = np.arange(256)[:, None]
    c = np.arange(128)[None, :]
    tile = (f // 64 * 2 + c // 64) * 16 + (f % 64) // 4
    return tiles[tile, c % 64, f % 4]

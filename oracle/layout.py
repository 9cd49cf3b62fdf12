"""Physical order of the packed 2-bit codes: one 4 KB tile (1024 32-bit words) per 128x128 block.

The paper fixes only that 16 two-bit codes share a 32-bit word (Sec. 3.3; K_I in R^{N/16 x d},
V_I in R^{N x d/16} in Alg. 1).  The logical content -- one code per (token, channel) -- is the
contract; the order inside a tile is an encoding chosen for the decode kernel and is written
down here independently of the kernel source.

Word format (both tiles): a word holds 8 "pairs" j = 0..7; pair j keeps its first code in bits
[2j+1 : 2j] and its second code in bits [16+2j+1 : 16+2j].

Key tile, block of 128 tokens x 128 channels, token t = 64*hf + l (hf in {0,1}, l in 0..63):
    token t owns 8 words q = 0..7 at word index ((hf*2 + q//4)*64 + l)*4 + q%4
    word q, pair j, element e (0 = first, 1 = second) holds channel
        c = 8*(4*(q%4) + j//2) + 4*(q//4) + 2*(j%2) + e
    (so a lane that loads 16 contiguous bytes gets 64 channels of its own token).

Value tile, block of 128 tokens x 128 channels, channel c = 64*ch + l (ch in {0,1}, l in 0..63):
    channel c owns, for each token half hf in {0,1}, 4 words w = 0..3 at word index
        ((hf*2 + ch)*64 + l)*4 + w
    word w, pair j, element e holds token
        t = 64*hf + 4*(4*w + j//2) + 2*(j%2) + e
    (so a lane that loads 16 contiguous bytes gets 64 tokens of its own channel).
"""
import numpy as np

TILE_WORDS = 1024


def _k_index_maps():
    t = np.arange(128)[:, None]
    c = np.arange(128)[None, :]
    hf, l = t // 64, t % 64
    s = c // 8
    p = (c % 8) // 4
    jj = (c % 4) // 2
    e = c % 2
    w = s // 4
    j = 2 * (s % 4) + jj
    word = ((hf * 2 + p) * 64 + l) * 4 + w
    shift = 2 * j + 16 * e
    return np.broadcast_to(word, (128, 128)), np.broadcast_to(shift, (128, 128))


def _v_index_maps():
    t = np.arange(128)[:, None]
    c = np.arange(128)[None, :]
    hf, tt = t // 64, t % 64
    ch, l = c // 64, c % 64
    b = tt // 4
    kk = tt % 4
    w = b // 4
    j = 2 * (b % 4) + kk // 2
    e = kk % 2
    word = ((hf * 2 + ch) * 64 + l) * 4 + w
    shift = 2 * j + 16 * e
    return np.broadcast_to(word, (128, 128)), np.broadcast_to(shift, (128, 128))


_K_WORD, _K_SHIFT = _k_index_maps()
_V_WORD, _V_SHIFT = _v_index_maps()


def _pack(codes, word, shift):
    codes = np.asarray(codes)
    assert codes.shape[-2:] == (128, 128) and codes.min() >= 0 and codes.max() <= 3
    lead = codes.shape[:-2]
    flat = codes.reshape((-1, 128 * 128)).astype(np.uint32)
    out = np.zeros((flat.shape[0], TILE_WORDS), dtype=np.uint32)
    wi = word.reshape(-1)
    sh = shift.reshape(-1).astype(np.uint32)
    for n in range(flat.shape[0]):
        np.bitwise_or.at(out[n], wi, flat[n] << sh)
    return out.reshape(lead + (TILE_WORDS,))


def _unpack(tile, word, shift):
    tile = np.asarray(tile, dtype=np.uint32)
    assert tile.shape[-1] == TILE_WORDS
    return ((tile[..., word] >> shift.astype(np.uint32)) & np.uint32(3)).astype(np.uint8)


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

"""The prepared form of a permutation (perq_perm_prepare) rebuilt with NumPy from its description in
include/perq.h: place of every position, piece of the row in every slot, and the two tables of operand
offsets in the matrix-core kernel's lane order.  Test infrastructure for the host library and the GPU
tests; the library's own routine is in csrc/perq_host.cpp."""
import numpy as np


def fixed_slot(g):
    """slot of 16-byte piece g of a staged row in the fixed layout"""
    g = np.asarray(g, dtype=np.int64)
    c = (g >> 4) & 7
    return g ^ (((c & 3) << 1) | (c >> 2))


def lane_positions(high_k: bool):
    """position inside a 4096-wide tile of element e of operand fragment f of lane l: array [f][lane][e]"""
    f = np.arange(8).reshape(8, 1, 1)
    lane = np.arange(64).reshape(1, 64, 1)
    e = np.arange(8).reshape(1, 1, 8)
    l, h = lane & 31, lane >> 5
    if not high_k:
        return (l * 4 + (f >> 1)) * 32 + 16 * (f & 1) + 8 * h + e
    m = 16 * ((l >> 2) & 1) + 4 * (l >> 3) + (l & 3)            # row of the constant operand a lane holds
    K = 16 * f + 8 * h + e
    return (m & 15) | (K << 4) | ((m >> 4) << 11)


def lane_tables(perm, slot_of):
    """uint16 [2][tiles][8][64][8]: byte offset of every operand inside its staged row; rows wider than
    8192 are staged in the placement `slot_of` (slot of every piece), narrower ones in the fixed layout;
    0xFFFF past the end of the row"""
    perm = np.asarray(perm, dtype=np.int64)
    d = perm.size
    tiles = (d + 4095) // 4096
    slot = np.asarray(slot_of, dtype=np.int64) if d > 8192 else fixed_slot(np.arange(d // 8))
    out = np.full((2, tiles, 8, 64, 8), 0xFFFF, dtype=np.uint16)
    for mode in range(2):
        pos_in_tile = lane_positions(mode == 1)
        for t in range(tiles):
            pos = 4096 * t + pos_in_tile
            ok = pos < d
            a = perm[np.where(ok, pos, 0)]
            off = (slot[a >> 3] << 4) | ((a & 7) << 1)
            out[mode, t] = np.where(ok, off, 0xFFFF).astype(np.uint16)
    return out


def assemble(perm, slot_of):
    """the whole form as bytes, for the given slot of every piece (a bijection inside every line of 8)"""
    perm = np.asarray(perm, dtype=np.int64)
    d = perm.size
    G = d // 8
    slot_of = np.asarray(slot_of, dtype=np.int64)
    granule_of = np.empty(G, dtype=np.uint16)
    granule_of[slot_of] = np.arange(G, dtype=np.uint16)
    place = (slot_of[perm >> 3] * 8 + (perm & 7)).astype(np.int32)
    return np.concatenate([place.view(np.uint8), granule_of.view(np.uint8), lane_tables(perm, slot_of).reshape(-1).view(np.uint8)])

"""Host reference of the packed tile layout documented in include/mq.h, written
in numpy independently of the device packer (used to check mq_pack bit for bit).

Tile (rb, g) = rows rb*64..rb*64+63 x columns g*128..g*128+127, stored as r
lines of 64 x 16 bytes; lane l (row) owns dwords 4*i+j = dword j of its 16 bytes
in line i.  The lane's 4r dwords are split into units; in each unit, pair p is
the columns (2p, 2p+1) -> (low half, high half) of the dword(s) named below.
Each entry: (dword in unit, bit position in the 16-bit half, number of bits,
first code bit).
"""
import numpy as np

# r -> (dwords per unit, pairs per unit, {pair: [(dw, bitpos, nbits, code_bit0), ...]})
FIELDS = {
    2: (1, 8, {p: [(0, 2 * p, 2, 0)] for p in range(8)}),
    4: (1, 4, {p: [(0, 4 * p, 4, 0)] for p in range(4)}),
    8: (1, 2, {p: [(0, 8 * p, 8, 0)] for p in range(2)}),
    3: (3, 16, {**{5 * d + j: [(d, 3 * j, 3, 0)] for d in range(3) for j in range(5)},
                15: [(0, 15, 1, 0), (1, 15, 1, 1), (2, 15, 1, 2)]}),
    6: (3, 8, {0: [(0, 0, 6, 0)], 1: [(0, 6, 6, 0)], 2: [(1, 0, 6, 0)], 3: [(1, 6, 6, 0)],
               4: [(2, 0, 6, 0)], 5: [(2, 6, 6, 0)],
               6: [(1, 12, 2, 0), (0, 12, 4, 2)],
               7: [(2, 12, 4, 0), (1, 14, 2, 4)]}),
}


def pack_ref(S: np.ndarray, r: int) -> np.ndarray:
    """S uint8 [N,K] on the 2^(8-r) grid -> packed bytes (uint8, Npad*K*r/8)."""
    N, K = S.shape
    G = K // 128
    RB = (N + 63) // 64
    ud, ppu, fields = FIELDS[r]
    t = np.zeros((RB * 64, K), dtype=np.uint32)
    t[:N] = S.astype(np.uint32) >> (8 - r)
    t = t.reshape(RB, 64, G, 128)
    dws = np.zeros((RB, G, 64, 4 * r), dtype=np.uint32)          # lane dwords
    for un in range(4 * r // ud):
        for p, flist in fields.items():
            for h in range(2):
                code = t[:, :, :, 2 * (un * ppu + p) + h].transpose(0, 2, 1)   # [RB, G, 64]
                for (dw, pos, nb, b0) in flist:
                    v = (code >> b0) & ((1 << nb) - 1)
                    dws[:, :, :, un * ud + dw] |= v << (pos + 16 * h)
    # line i of a tile holds dwords 4i..4i+3 of every lane
    out = dws.reshape(RB, G, 64, r, 4).transpose(0, 1, 3, 2, 4)   # [RB, G, r, 64, 4]
    return np.ascontiguousarray(out).astype("<u4").view(np.uint8).reshape(-1)


def meta_ref(a: np.ndarray) -> np.ndarray:
    """[N, G] fp16 -> tiled [RB][G][64] fp16 (pad rows zero)."""
    N, G = a.shape
    RB = (N + 63) // 64
    p = np.zeros((RB * 64, G), dtype=np.float16)
    p[:N] = a
    return np.ascontiguousarray(p.reshape(RB, 64, G).transpose(0, 2, 1)).reshape(-1)

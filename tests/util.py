"""Helpers shared by the GPU parity tests: an independent statement of the tiled layout written from the header
text (the bit-pattern marshalling lives in the package, paper_2104_08378_amd/bits.py)."""
import numpy as np

from paper_2104_08378_amd.bits import OUT_DT, TORCH_DT, out_to_f64, to_bits, to_gpu  # noqa: F401  (re-exported for the tests)


def tiled_from_canonical(V, meta, dtype):
    """The tiled layout, restated from include/sp24.h: tiles of 32 rows x 64
    columns of A in order [M/32][K/64]; slot = (m % 32) + 32*h; one little-endian
    meta word per slot (canonical bytes 8*kb + 4*h .. +3); V: 16 bytes per slot
    (8-bit: canonical V columns 32*kb + 16*h .. +15; 16-bit: two runs s = 0,1 of
    64 slots, run s holding columns 32*kb + 16*h + 8*s .. +7)."""
    M, K2 = V.shape
    K = 2 * K2
    RB, KB = M // 32, K // 64
    meta_t = np.zeros((RB, KB, 64, 4), dtype=np.uint8)
    if dtype in ("i8", "f8"):
        V_t = np.zeros((RB, KB, 64, 16), dtype=V.dtype)
    else:
        V_t = np.zeros((RB, KB, 2, 64, 8), dtype=V.dtype)
    for rb in range(RB):
        for kb in range(KB):
            for h in range(2):
                rows = slice(rb * 32, rb * 32 + 32)
                slots = slice(32 * h, 32 * h + 32)
                meta_t[rb, kb, slots, :] = meta[rows, 8 * kb + 4 * h: 8 * kb + 4 * h + 4]
                if dtype in ("i8", "f8"):
                    V_t[rb, kb, slots, :] = V[rows, 32 * kb + 16 * h: 32 * kb + 16 * h + 16]
                else:
                    for s in range(2):
                        c0 = 32 * kb + 16 * h + 8 * s
                        V_t[rb, kb, s, slots, :] = V[rows, c0:c0 + 8]
    return V_t.reshape(M, K2), meta_t.reshape(M, K // 8)

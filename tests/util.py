"""Helpers shared by the GPU parity tests: numpy bit patterns <-> torch tensors,
and an independent statement of the tiled layout written from the header text."""
import numpy as np
import torch

TORCH_DT = {"f16": torch.float16, "bf16": torch.bfloat16, "i8": torch.int8}
OUT_DT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16, "i32": torch.int32}


def to_gpu(bits, dtype):
    """numpy uint16 bit patterns / int8 -> GPU tensor of the matching torch dtype (same bits)."""
    if dtype == "i8":
        return torch.from_numpy(np.ascontiguousarray(bits)).cuda()
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()
    return t.view(TORCH_DT[dtype])


def to_bits(t):
    """GPU tensor -> numpy array of raw storage (uint16 for 16-bit floats)."""
    t = t.detach().cpu().contiguous()
    if t.dtype in (torch.float16, torch.bfloat16):
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def out_to_f64(t):
    """Exact float64 value of a GPU result tensor."""
    t = t.detach().cpu()
    if t.dtype == torch.int32:
        return t.numpy().astype(np.float64)
    return t.to(torch.float64).numpy()


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
    if dtype == "i8":
        V_t = np.zeros((RB, KB, 64, 16), dtype=V.dtype)
    else:
        V_t = np.zeros((RB, KB, 2, 64, 8), dtype=V.dtype)
    for rb in range(RB):
        for kb in range(KB):
            for h in range(2):
                rows = slice(rb * 32, rb * 32 + 32)
                slots = slice(32 * h, 32 * h + 32)
                meta_t[rb, kb, slots, :] = meta[rows, 8 * kb + 4 * h: 8 * kb + 4 * h + 4]
                if dtype == "i8":
                    V_t[rb, kb, slots, :] = V[rows, 32 * kb + 16 * h: 32 * kb + 16 * h + 16]
                else:
                    for s in range(2):
                        c0 = 32 * kb + 16 * h + 8 * s
                        V_t[rb, kb, s, slots, :] = V[rows, c0:c0 + 8]
    return V_t.reshape(M, K2), meta_t.reshape(M, K // 8)

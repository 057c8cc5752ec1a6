"""Raw storage bits <-> torch tensors: numpy arrays of bit patterns (uint16 for the 16-bit float types, which numpy
does not have) go to the GPU and come back unchanged.  Marshalling only; nothing of the method is computed here."""
import numpy as np
import torch

TORCH_DT = {"f16": torch.float16, "bf16": torch.bfloat16, "i8": torch.int8, "f8": torch.float8_e4m3fn}
OUT_DT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16, "i32": torch.int32}


def to_gpu(bits, dtype):
    """numpy uint16 / uint8 bit patterns / int8 -> GPU tensor of the matching torch dtype (same bits)."""
    if dtype == "i8":
        return torch.from_numpy(np.ascontiguousarray(bits)).cuda()
    if dtype == "f8":
        return torch.from_numpy(np.ascontiguousarray(bits, dtype=np.uint8)).cuda().view(torch.float8_e4m3fn)
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()
    return t.view(TORCH_DT[dtype])


def to_bits(t):
    """GPU tensor -> numpy array of raw storage (uint16 for 16-bit floats)."""
    t = t.detach().cpu().contiguous()
    if t.dtype in (torch.float16, torch.bfloat16):
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype == torch.float8_e4m3fn:
        return t.view(torch.uint8).numpy()
    return t.numpy()


def out_to_f64(t):
    """Exact float64 value of a GPU result tensor."""
    t = t.detach().cpu()
    if t.dtype == torch.int32:
        return t.numpy().astype(np.float64)
    return t.to(torch.float64).numpy()

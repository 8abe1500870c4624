"""Device-memory plumbing for callers of the binding: PyTorch is used only to
own HBM buffers and to name a stream.  No torch op touches the data path."""
import numpy as np
import torch

_TORCH = {"bf16": torch.bfloat16, "f32": torch.float32, None: torch.bfloat16}


def alloc_tensors(plan, side, device="cuda", fill_bits=None):
    """One flat device tensor per registered tensor of the plan's side (0 = holder, 1 = reader).
    fill_bits: optional 16-bit pattern written to every 2-byte half (sentinel for tests)."""
    out = []
    for info in plan.tensors(side):
        n = info["rows"] * info["cols"]
        t = torch.empty(n, dtype=_TORCH[info["dtype"]], device=device)
        if fill_bits is not None and n:
            t.view(torch.int16).fill_(fill_bits - (1 << 16) if fill_bits >= 1 << 15 else fill_bits)
        out.append(t)
    return out


def ptrs(tensors):
    return np.array([t.data_ptr() for t in tensors], dtype=np.uint64)


def alloc_wire(plan, device="cuda", fill_byte=None):
    """One contiguous buffer holding every chunk of the plan back to back, and the chunk pointers."""
    nbytes = max(16, (plan.wire_bytes + 15) // 16 * 16)
    buf = torch.empty(nbytes, dtype=torch.uint8, device=device)
    if fill_byte is not None:
        buf.fill_(fill_byte)
    return buf, chunk_ptrs(plan, buf)


def chunk_ptrs(plan, buf):
    n = plan.num_chunks
    if n == 0:
        return np.zeros(0, dtype=np.uint64)
    cb = plan.chunk_bytes(0)
    return buf.data_ptr() + np.arange(n, dtype=np.uint64) * np.uint64(cb)


def current_stream():
    return torch.cuda.current_stream().cuda_stream

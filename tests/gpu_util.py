"""Helpers shared by the GPU tests: move seeded inputs to the device and run the C-ABI path."""
import numpy as np


def to_device(inputs, device="cuda:0"):
    import torch
    if inputs.x_dtype == "bf16":
        return torch.from_numpy(inputs.X_bits.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(inputs.X).to(device)


def run_forward(inputs, poison=True, **kw):
    """Packs, runs tsvd_forward through the binding, returns (y as float64 numpy, handle)."""
    import torch
    import paper_2308_07641_amd as tsvd
    h = tsvd.tsvd_pack(inputs.U, inputs.S, inputs.V)
    x = to_device(inputs)
    y = torch.empty((h.M, x.shape[1]), dtype=torch.float32, device=x.device)
    if poison:
        y.fill_(float("nan"))
    tsvd.tsvd_forward(h, x, y, **kw)
    torch.cuda.synchronize()
    return y.cpu().numpy().astype(np.float64), h


def rel_err(y, ref):
    return float(np.max(np.abs(y - ref)) / np.max(np.abs(ref)))

"""Move synthetic storage arrays onto the GPU as torch tensors (plumbing only)."""
import numpy as np

from .configs import DTYPE_F32, DTYPE_BF16, DTYPE_F16
from .gen import tensor_specs, make_tensor, STORAGE_NP


def torch_dtype(dtype):
    import torch
    return {DTYPE_F32: torch.float32, DTYPE_BF16: torch.bfloat16, DTYPE_F16: torch.float16}[dtype]


def to_device(arr, dtype, device="cuda"):
    """Storage array (uint16 bit patterns for bf16) -> torch tensor of the matching dtype on `device`."""
    import torch
    if dtype == DTYPE_BF16:
        return torch.from_numpy(arr.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(arr).to(device)


def weights_to_device(cfg, storage, device="cuda"):
    return {k: to_device(v, cfg.dtype, device) for k, v in storage.items()}


def make_weights_on_device(cfg, device="cuda", keep_host=None):
    """Generate every tensor on the host (one at a time, through a pinned staging buffer) and copy it
    to the GPU.  `keep_host`: optional list of names (prefix match) whose host arrays are returned too."""
    import torch
    out, host = {}, {}
    specs = tensor_specs(cfg)
    biggest = max(int(np.prod(s)) for _, s, _ in specs)
    npdt = STORAGE_NP[cfg.dtype]
    stage_t = torch.empty(biggest * np.dtype(npdt).itemsize, dtype=torch.uint8, pin_memory=True)
    stage = stage_t.numpy().view(npdt)
    for name, shape, kind in specs:
        n = int(np.prod(shape))
        arr = make_tensor(cfg, name, shape, kind, out=stage[:n])
        t = to_device(arr, cfg.dtype, device)
        torch.cuda.synchronize()
        out[name] = t
        if keep_host is not None and any(name == k or name.startswith(k) for k in keep_host):
            host[name] = arr.copy()
    return (out, host) if keep_host is not None else out

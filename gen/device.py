"""Host arrays of stored logits -> device tensors (inputs only, no arithmetic of the method)."""
import numpy as np
import torch


def to_device_logits(z: np.ndarray) -> torch.Tensor:
    """Host logits (float32, or uint16 bf16 bit patterns) -> device tensor (float32 / bfloat16).

    The library wants every row 16-byte aligned: when V * itemsize is not a multiple of 16 the rows
    are laid out with a padded pitch (padding filled with a large value that must never be read) and
    a [..., :V] view is returned."""
    if z.dtype == np.float32:
        t = torch.from_numpy(z)
        per16, big = 4, 1e30
    else:
        assert z.dtype == np.uint16
        t = torch.from_numpy(z.view(np.int16)).view(torch.bfloat16)
        per16, big = 8, 1e30
    V = z.shape[-1]
    if V % per16 == 0:
        return t.cuda()
    pitch = (V + per16 - 1) // per16 * per16
    padded = torch.full(z.shape[:-1] + (pitch,), big, dtype=t.dtype, device="cuda")
    padded[..., :V] = t.cuda()
    return padded[..., :V]

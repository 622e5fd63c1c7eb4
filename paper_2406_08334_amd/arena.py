"""Device arenas for chunked model states, spread over the GPU's physical memory.

Measured on MI355X (288 GiB of HBM3E): physical memory behaves as three regions of 96 GiB.  A
kernel that streams several large arrays side by side - the update reads and writes three fp32
arrays and two 16-bit ones - runs at 5.5-5.8 TB/s when its three fp32 arrays lie in the same
region and at 6.3-6.4 TB/s as soon as one of them lies in another (with the two 16-bit arrays
moved away instead: 6.1).  Virtual addresses, offsets inside the allocations and the launch
shape do not matter.  A fresh process on an idle GPU gets its allocations one after the other
from the same region, so a state of up to about 100 GB ends up in the slow arrangement.
Allocation order is the only handle a process has on physical placement: the arenas are
allocated with a temporary spacer after each one, sized to spread them over all free memory;
the spacers are released again right away (the arenas keep their place) and the memory is free
for everything else.

Plain PyTorch allocation calls; no arithmetic of the method lives here.
"""
from __future__ import annotations

import torch

GIB = 1 << 30


def spread_arenas(specs, device="cuda", gap_bytes: int | None = None, keep_free_bytes: int = 0):
    """Allocates one zero-filled tensor per (shape, dtype) in `specs`, a spacer between them.

    gap_bytes: size of each spacer; None = min(48 GiB, (free memory - arenas - keep_free_bytes) / n).
    Returns the list of tensors, in order.  With a gap of 0 this is plain allocation.
    """
    specs = list(specs)
    need = 0
    for shape, dtype in specs:
        n = 1
        for d in shape:
            n *= int(d)
        need += n * torch.empty(0, dtype=dtype).element_size()
    if gap_bytes is None:
        free, _ = torch.cuda.mem_get_info(device)
        gap_bytes = max(0, min(48 * GIB, (free - need - keep_free_bytes - 2 * GIB) // max(1, len(specs))))
    gap_bytes = int(gap_bytes) // (2 << 20) * (2 << 20)
    out, spacers = [], []
    for shape, dtype in specs:
        out.append(torch.zeros(*shape, dtype=dtype, device=device))
        if gap_bytes:
            spacers.append(torch.empty(gap_bytes, dtype=torch.uint8, device=device))
    del spacers
    torch.cuda.empty_cache()          # hands the spacers back to the driver; the arenas stay where they are
    return out


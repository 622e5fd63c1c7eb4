"""Device arenas for chunked model states, spread over the GPU's physical memory.

Measured on MI355X: a kernel that streams several large arrays side by side (the update
reads and writes five) runs about 10 % slower when those arrays sit close together in
physical memory - which is where a fresh process on an idle GPU gets them, one allocation
after the other - than when they are tens of GiB apart.  Virtual addresses, offsets inside
the allocations and the launch shape do not matter; the distance does.  Allocation order is
the only handle a process has on physical placement, so the arenas are allocated with a
temporary spacer after each one; the spacers are released again right away (the arenas keep
their place) and the memory is free for everything else.

Plain PyTorch allocation calls; no arithmetic of the method lives here.
"""
from __future__ import annotations

import torch

GIB = 1 << 30


def spread_arenas(specs, device="cuda", gap_bytes: int | None = None, keep_free_bytes: int = 0):
    """Allocates one zero-filled tensor per (shape, dtype) in `specs`, a spacer between them.

    gap_bytes: size of each spacer; None = min(20 GiB, (free memory - arenas - keep_free_bytes) / n).
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
        gap_bytes = max(0, min(20 * GIB, (free - need - keep_free_bytes - 2 * GIB) // max(1, len(specs))))
    gap_bytes = int(gap_bytes) // (2 << 20) * (2 << 20)
    out, spacers = [], []
    for shape, dtype in specs:
        out.append(torch.zeros(*shape, dtype=dtype, device=device))
        if gap_bytes:
            spacers.append(torch.empty(gap_bytes, dtype=torch.uint8, device=device))
    del spacers
    torch.cuda.empty_cache()          # hands the spacers back to the driver; the arenas stay where they are
    return out

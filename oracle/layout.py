"""CPU oracle of the paper's own chunk layout and chunk-size search.

TEST INFRASTRUCTURE ONLY (same rules as oracle.cpp: never imported by the product).
Plain Python, written from the paper's description (Appendix B.1, "Chunk Organization and
Size Search"):

  * parameters are laid out in the order given (execution order; a parameter shared between
    layers appears once, at its first occurrence);
  * the parameters of one transformer block go into one chunk;
  * a parameter is never split between chunks, so chunks carry unused space, and the chunk
    size is chosen by simulating that waste over a grid of candidate sizes and taking the
    size that wastes least.

How this file states it.  The tensors stand in a row; a chunk boundary is a CUT between two
neighbouring tensors.  A cut is FORBIDDEN between two tensors of the same transformer block
when that block, laid out on its own from the start of a chunk, fits a chunk of S elements
(then the block must stay whole); every other cut is allowed.  Chunks are filled from the
left: a chunk that starts at tensor p ends at the LAST allowed cut q for which the tensors
p .. q-1, laid one after the other, still fit S.  If not even the first allowed cut after p
fits, some single tensor is larger than S and S is infeasible.  Inside a chunk every tensor
starts at the next multiple of ALIGN = 8 elements (16 bytes, the vector width of the copy
kernels); a tensor of size 0 takes no room and has no place.

Readings where the paper is silent: the candidate grid is S_min, S_min + step, ... up to
S_min + span, with S_min = max(largest tensor, min_chunk) rounded up to a multiple of `step`;
among sizes of equal waste the smallest wins.  Pins: tests/test_oracle_layout.py (hand-worked
placements, structural invariants on random inputs, brute force over every candidate, and
the chunk counts the paper prints in its Table 4, which some - not all - grids reproduce).
"""
from __future__ import annotations

ALIGN = 8


def end_offset(sizes, first: int, last: int) -> int:
    """Elements a chunk needs to hold tensors first .. last-1 from its start, each at the next
    multiple of ALIGN (empty tensors skipped)."""
    end = 0
    for t in range(first, last):
        if sizes[t]:
            end = (end + ALIGN - 1) // ALIGN * ALIGN + sizes[t]
    return end


def allowed_cuts(sizes, group_ids, S: int):
    """cut[k] is True when a chunk boundary may fall between tensor k-1 and tensor k (0 < k < n)."""
    n = len(sizes)
    cut = [True] * (n + 1)
    k = 0
    while k < n:
        if group_ids[k] is None:
            k += 1
            continue
        stop = k                       # the block: tensors k .. stop-1 carry the same id in a row
        while stop < n and group_ids[stop] == group_ids[k]:
            stop += 1
        if end_offset(sizes, k, stop) <= S:
            for inner in range(k + 1, stop):
                cut[inner] = False     # the block fits a chunk: it stays whole
        k = stop
    return cut


def layout_grouped(sizes, group_ids, S: int):
    """-> (placements, n_chunks, waste), or None when a tensor is larger than S.
    placements[t] = (chunk, offset), None for an empty tensor; waste = n_chunks * S - sum(sizes)."""
    assert S > 0 and S % ALIGN == 0
    n = len(sizes)
    cut = allowed_cuts(sizes, group_ids, S)
    place = [None] * n
    chunk = 0
    p = 0
    while p < n and sizes[p] == 0:     # leading empty tensors belong to no chunk
        p += 1
    while p < n:
        best = None
        for q in range(p + 1, n + 1):
            if cut[q] and end_offset(sizes, p, q) <= S:
                best = q               # keep the last allowed cut that still fits
        if best is None:
            return None
        q = best
        while q < n and sizes[q] == 0:  # empty tensors after the cut take no room anywhere
            q += 1
        off = 0
        for t in range(p, best):
            if sizes[t]:
                off = (off + ALIGN - 1) // ALIGN * ALIGN
                place[t] = (chunk, off)
                off += sizes[t]
        chunk += 1
        p = q
    return place, chunk, chunk * S - sum(sizes)


def chunk_size_search(sizes, group_ids, min_chunk: int, span: int, step: int):
    """-> (S, n_chunks, waste) of least waste over the grid, the smaller S on equal waste."""
    assert step > 0 and step % ALIGN == 0
    floor = max(max(list(sizes) + [1]), min_chunk)
    s_min = (floor + step - 1) // step * step
    outcomes = []
    for k in range(span // step + 1):
        S = s_min + k * step
        r = layout_grouped(sizes, group_ids, S)
        if r is not None:
            outcomes.append((r[2], S, r[1]))           # (waste, S, n_chunks): min() orders by waste, then S
    if not outcomes:
        return None
    waste, S, n_chunks = min(outcomes)
    return S, n_chunks, waste


def execution_order(uses, n_tensors: int):
    """The order in which the tensors are handed to the layout (Appendix B.1, first sentences of
    "Chunk Organization and Size Search"; "Hierarchical Chunk Management for Model States"): by
    execution order, a parameter that several layers share counted at its FIRST occurrence.

    uses: the tensor indices (into the model's declaration table) in the order the forward pass
    touches them; an index may come more than once (shared parameters, layers run twice).
    Returns the n_tensors indices: used tensors by the position of their first use; tensors the
    trace never touches behind them, in declaration order (reading: the paper does not say where
    an unused parameter goes; it still needs storage).

    Written as the definition: each tensor's key is where it first appears in `uses`."""
    first = []
    for t in range(n_tensors):
        pos = None
        for k, u in enumerate(uses):
            if u == t:
                pos = k
                break
        first.append(pos)
    used = sorted((t for t in range(n_tensors) if first[t] is not None), key=lambda t: first[t])
    unused = [t for t in range(n_tensors) if first[t] is None]
    return used + unused

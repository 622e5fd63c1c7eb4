"""CPU oracle of the paper-faithful chunk layout and chunk-size search.

TEST INFRASTRUCTURE ONLY (same rules as oracle.cpp: never imported by the product).
Plain Python loops, written from the paper's description:

  * parameters are laid out in the order given (execution order; a parameter shared
    between layers appears once, at its first occurrence) - Appendix B.1, "Chunk
    Organization and Size Search";
  * parameters of one transformer block are grouped into one chunk - same passage;
  * a parameter is never split between chunks, so chunks carry unused space ("memory
    waste") - same passage, which chooses the chunk size by simulating that waste over
    candidate sizes and taking the minimum.

The paper gives neither the candidate grid nor a tie rule.  Reading taken here: the
candidates are S_min, S_min + step, ... <= S_min + span with S_min = the largest
parameter rounded up to `step`; ties go to the smaller size.  With span = 2^25 and
step = 2^20 elements this reproduces both chunk counts the paper prints (Table 4:
12 chunks for the 32-block GPT-2 1B, 49 for the 48-block GPT-2 10B).

Placement rule for a given chunk size S (elements):
  - walk the tensors in order; maximal runs of consecutive tensors with the same group
    id (a transformer block) form a group, tensors with group id None stand alone;
  - every tensor starts at a multiple of ALIGN = 8 elements inside its chunk (16 bytes:
    the vector width of the copy kernels);
  - a group that fits into an empty chunk is kept together: if it does not fit into the
    rest of the current chunk, the chunk is closed and the group opens the next one;
  - a group larger than a chunk is placed tensor by tensor under the same rule;
  - a tensor larger than S makes S infeasible.
"""
from __future__ import annotations

ALIGN = 8


def _up(x: int, a: int) -> int:
    return -(-x // a) * a


def _groups(sizes, group_ids):
    """maximal runs of equal non-None group ids -> list of lists of tensor indices"""
    runs, i, n = [], 0, len(sizes)
    while i < n:
        j = i + 1
        if group_ids[i] is not None:
            while j < n and group_ids[j] == group_ids[i]:
                j += 1
        runs.append(list(range(i, j)))
        i = j
    return runs


def _span(sizes, idxs, start: int) -> int:
    """end offset after placing tensors idxs one after the other from offset `start`"""
    off = start
    for t in idxs:
        if sizes[t] == 0:
            continue
        off = _up(off, ALIGN) + sizes[t]
    return off


def layout_grouped(sizes, group_ids, S: int):
    """-> (placements, n_chunks, waste) or None if S is infeasible.
    placements[t] = (chunk, offset) or None for an empty tensor; waste = n_chunks*S - sum(sizes)."""
    assert S > 0 and S % ALIGN == 0
    place = [None] * len(sizes)
    chunk, off, used_any = 0, 0, False
    for run in _groups(sizes, group_ids):
        pieces = [run] if _span(sizes, run, 0) <= S else [[t] for t in run]
        for piece in pieces:
            if all(sizes[t] == 0 for t in piece):
                continue
            if _span(sizes, piece, 0) > S:
                return None
            if _span(sizes, piece, off) > S:
                chunk, off = chunk + 1, 0
            for t in piece:
                if sizes[t] == 0:
                    continue
                off = _up(off, ALIGN)
                place[t] = (chunk, off)
                off += sizes[t]
                used_any = True
    n_chunks = chunk + 1 if used_any else 0
    return place, n_chunks, n_chunks * S - sum(sizes)


def chunk_size_search(sizes, group_ids, min_chunk: int, span: int, step: int):
    """-> (best S, n_chunks, waste): minimum waste over the candidate grid, ties to the smaller S."""
    assert step % ALIGN == 0 and step > 0
    biggest = max([s for s in sizes] + [1])
    s_min = _up(max(biggest, min_chunk), step)
    best = None
    S = s_min
    while S <= s_min + span:
        r = layout_grouped(sizes, group_ids, S)
        if r is not None:
            _, n_chunks, waste = r
            if best is None or waste < best[2]:
                best = (S, n_chunks, waste)
        S += step
    return best

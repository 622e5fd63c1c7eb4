"""Pins for the oracle's paper-faithful layout (no tensor split, transformer blocks kept
together, chunk size by minimum-waste search; paper, Appendix B.1 "Chunk Organization and
Size Search"): the chunk counts the paper prints in Table 4, structural invariants, and a
brute-force search over every candidate size on small inputs."""
import os
import random

import pytest

from oracle import layout as L
from paper_2406_08334_amd import shapes

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_table4_chunk_counts.txt")
MODELS = {"gpt2_1b": lambda: shapes.gpt2(1600, 32, 6400), "gpt2_10b": lambda: shapes.gpt2(4096, 48, 16384)}
SPAN, STEP = 1 << 25, 1 << 20


def test_search_reproduces_the_papers_chunk_counts():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) == 2
    for name, n_block, n_chunk in rows:
        table = MODELS[name]()
        sizes, gids = [n for _, n in table], shapes.block_ids(table)
        assert max(g for g in gids if g is not None) + 1 == int(n_block)
        S, n_chunks, waste = L.chunk_size_search(sizes, gids, 0, SPAN, STEP)
        assert n_chunks == int(n_chunk), (name, S, n_chunks)
        assert waste == n_chunks * S - sum(sizes) and waste < 0.05 * sum(sizes)


def check_invariants(sizes, gids, S, place, n_chunks):
    spans = {}
    for t, p in enumerate(place):
        if sizes[t] == 0:
            assert p is None
            continue
        c, off = p
        assert 0 <= c < n_chunks and off % L.ALIGN == 0 and off + sizes[t] <= S      # never split
        spans.setdefault(c, []).append((off, off + sizes[t], t))
    last = (-1, -1)
    for c in sorted(spans):                                   # order preserved, no overlap
        prev_end = 0
        for off, end, t in sorted(spans[c]):
            assert off >= prev_end and (c, off) > last
            prev_end, last = end, (c, off)
    assert sorted(spans) == list(range(n_chunks))             # no empty chunk
    order = [place[t] for t in range(len(sizes)) if sizes[t]]
    assert order == sorted(order)
    # a block that fits a chunk lives in exactly one chunk
    by_gid = {}
    for t, g in enumerate(gids):
        if g is not None and sizes[t]:
            by_gid.setdefault((g, _run_id(gids, t)), []).append(t)
    for ts in by_gid.values():
        if L._span(sizes, ts, 0) <= S:
            assert len({place[t][0] for t in ts}) == 1


def _run_id(gids, t):
    r = 0
    for i in range(1, t + 1):
        if gids[i] != gids[i - 1]:
            r += 1
    return r


def test_invariants_on_random_inputs():
    rng = random.Random(5)
    for _ in range(200):
        n = rng.randint(1, 14)
        sizes = [rng.choice([0, 1, 3, 8, 9, 17, 40, 64, 100]) for _ in range(n)]
        gids, g = [], 0
        for i in range(n):
            if rng.random() < 0.3:
                g += 1
            gids.append(None if rng.random() < 0.25 else g)
        S = rng.choice([8, 16, 64, 104, 128, 256])
        r = L.layout_grouped(sizes, gids, S)
        if max(sizes) > S:
            assert r is None
            continue
        place, n_chunks, waste = r
        assert waste == n_chunks * S - sum(sizes) >= 0
        check_invariants(sizes, gids, S, place, n_chunks)


def test_worked_small_example():
    # S = 32: [a:10][blk0: 8, 8][blk1: 20, 4] [z:3]
    sizes, gids = [10, 8, 8, 20, 4, 3], [None, 0, 0, 1, 1, None]
    place, n_chunks, waste = L.layout_grouped(sizes, gids, 32)
    # a at 0..10; block 0 (16 + alignment) fits after it: 16..24, 24..32; block 1 opens chunk 1; z follows
    assert place[:4] == [(0, 0), (0, 16), (0, 24), (1, 0)]
    assert place[4] == (1, 24) and place[5][0] == 2 and n_chunks == 3      # 24+4 = 28, z needs 32..35 > 32
    assert waste == 3 * 32 - sum(sizes)
    # a block bigger than a chunk is placed tensor by tensor
    place, n_chunks, _ = L.layout_grouped([20, 20, 20], [7, 7, 7], 32)
    assert place == [(0, 0), (1, 0), (2, 0)] and n_chunks == 3
    assert L.layout_grouped([40], [None], 32) is None


def test_search_is_the_brute_force_minimum():
    rng = random.Random(9)
    for _ in range(50):
        n = rng.randint(2, 10)
        sizes = [rng.randint(1, 60) for _ in range(n)]
        gids = [rng.choice([None, 0, 1, 2]) for _ in range(n)]
        step, span = 8, 8 * rng.randint(0, 12)
        got = L.chunk_size_search(sizes, gids, 0, span, step)
        s_min = -(-max(sizes) // step) * step
        cands = []
        for S in range(s_min, s_min + span + 1, step):
            r = L.layout_grouped(sizes, gids, S)
            if r is not None:
                cands.append((r[2], S, r[1]))
        waste, S, n_chunks = min(cands)
        assert got == (S, n_chunks, waste)

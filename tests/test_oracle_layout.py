"""Pins for the oracle's layout after the paper (no tensor split, transformer blocks kept
together, chunk size by minimum-waste search; paper, Appendix B.1 "Chunk Organization and
Size Search"): placements worked out by hand for the LLaMA-7B table and a GPT-2 block,
structural invariants on random inputs, and a brute-force search over every candidate size
on small inputs.  The chunk counts the paper prints in Table 4 are a consistency check, not
a pin: 49 chunks for the 48-block GPT2-10B follows from any grid (one block per chunk plus
the embeddings), and 12 chunks for the 32-block GPT2-1B - whose hidden size the paper does
not print - comes out for hidden sizes 1280 to 1792 under several (span, step) grids."""
import os
import random

import pytest

from oracle import layout as L
from paper_2406_08334_amd import shapes

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_table4_chunk_counts.txt")
MODELS = {"gpt2_1b": lambda: shapes.gpt2(1600, 32, 6400), "gpt2_10b": lambda: shapes.gpt2(4096, 48, 16384)}
SPAN, STEP = 1 << 25, 1 << 20


def test_search_is_consistent_with_the_papers_chunk_counts():
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
        need = 0                                              # room the block takes on its own, 8-aligned starts
        for t in ts:
            need = -(-need // 8) * 8 + sizes[t]
        if need <= S:
            assert len({place[t][0] for t in ts}) == 1
    # left-filled: the first tensor (or whole block) of a chunk would not have fitted behind the chunk before it
    first_of = {c: min(v)[2] for c, v in spans.items()}
    for c in range(1, n_chunks):
        t0 = first_of[c]
        block = [t0]
        if gids[t0] is not None:
            rid = _run_id(gids, t0)
            block = [t for t in range(len(sizes)) if gids[t] == gids[t0] and _run_id(gids, t) == rid and sizes[t]]
            alone = 0
            for t in block:
                alone = -(-alone // 8) * 8 + sizes[t]
            if alone > S:                                     # a block too big for a chunk goes tensor by tensor
                block = [t0]
        end = max(e for _, e, _ in spans[c - 1])
        for t in block:
            end = -(-end // 8) * 8 + sizes[t]
        assert end > S, (c, t0)


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


def test_llama7b_placements_worked_by_hand():
    """LLaMA-7B shape, S = 194 * 2^20 = 203,423,744.  By hand: the embedding (32000 * 4096 = 131,072,000)
    opens chunk 0; a block is 4 * 4096^2 + 3 * 4096 * 11008 + 2 * 4096 = 202,383,360 elements, more than the
    72,351,744 left in chunk 0, so block i fills chunk 1 + i and leaves 1,040,384; the final norm gain (4096)
    fits behind block 31 in chunk 32; the head (131,072,000) does not and opens chunk 33: 34 chunks,
    waste 34 * 203,423,744 - 6,738,415,616 = 177,991,680."""
    table = shapes.llama(4096, 11008, 32)
    sizes, gids = [n for _, n in table], shapes.block_ids(table)
    S = 194 << 20
    place, n_chunks, waste = L.layout_grouped(sizes, gids, S)
    assert n_chunks == 34 and waste == 177_991_680
    assert place[0] == (0, 0)
    inside = [0, 16_777_216, 33_554_432, 50_331_648, 67_108_864, 112_197_632, 157_286_400, 202_375_168, 202_379_264]
    for i in range(32):
        assert place[1 + 9 * i: 10 + 9 * i] == [(1 + i, off) for off in inside], i
    assert place[289] == (32, 202_383_360)        # norm.weight behind the last block
    assert place[290] == (33, 0)                  # lm_head.weight
    # one step smaller (193 * 2^20 = 202,375,168 < a block): blocks no longer fit a chunk and go tensor by tensor
    place2, n2, _ = L.layout_grouped(sizes, gids, 193 << 20)
    assert place2[1:10] == [(0, 131_072_000), (0, 147_849_216), (0, 164_626_432), (0, 181_403_648),
                            (1, 0), (1, 45_088_768), (1, 90_177_536), (1, 135_266_304), (1, 135_270_400)]


def test_gpt2_block_placements_worked_by_hand():
    """GPT-2 block, hidden 768 (7,087,872 elements: 768, 768, 1,769,472, 2304, 589,824, 768, 768, 768,
    2,359,296, 3072, 2,359,296, 768), preceded and followed by a lone tensor of 1000 elements."""
    blk = [n for _, n in shapes.gpt2_block(768)]
    sizes, gids = [1000] + blk + [1000], [None] + [0] * 12 + [None]
    # S = 7,089,000: the lone tensor takes [0, 1000); the block (7,087,872) would end at 7,088,872 <= S: same chunk
    place, n_chunks, waste = L.layout_grouped(sizes, gids, 7_089_000)
    starts = [1000, 1768, 2536, 1_772_008, 1_774_312, 2_364_136, 2_364_904, 2_365_672, 2_366_440, 4_725_736,
              4_728_808, 7_088_104]
    assert place[0] == (0, 0) and place[1:13] == [(0, o) for o in starts]
    assert place[13] == (1, 0) and n_chunks == 2       # 7,088,872 + 1000 > S
    assert waste == 2 * 7_089_000 - sum(sizes)
    # S = 7,088,000: the block fits an empty chunk (7,087,872) but not behind the lone tensor: it opens chunk 1
    place, n_chunks, _ = L.layout_grouped(sizes, gids, 7_088_000)
    assert place[0] == (0, 0) and place[1] == (1, 0) and place[12] == (1, 7_087_104) and place[13] == (2, 0)
    assert n_chunks == 3
    # S = 4,000,000 < block: tensor by tensor; fc.weight (2,359,296) does not fit behind 2,366,440 and opens chunk 1
    place, n_chunks, _ = L.layout_grouped(sizes, gids, 4_000_000)
    assert place[8] == (0, 2_365_672) and place[9] == (1, 0) and place[10] == (1, 2_359_296)
    assert place[11] == (2, 0) and place[12] == (2, 2_359_296) and place[13] == (2, 2_360_064) and n_chunks == 3


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


# ---- execution order with shared parameters at their first occurrence (Appendix B.1)

def test_execution_order_worked_by_hand():
    # a GPT-2-like model whose modules are DECLARED head first (head tied to the token embedding):
    #   0 head/wte   1 ln_f   2 block0.w   3 block1.w   4 wpe   5 never used
    # forward pass: wte, wpe, block0, block1, block0 again (a layer run twice), ln_f, head (= wte again)
    uses = [0, 4, 2, 3, 2, 1, 0]
    assert L.execution_order(uses, 6) == [0, 4, 2, 3, 1, 5]
    # the shared tensor counts where it is used first, not where it is used last
    assert L.execution_order([3, 1, 3, 0], 4) == [3, 1, 0, 2]
    # nothing shared, execution = declaration: identity; no trace at all: declaration order
    assert L.execution_order([0, 1, 2], 3) == [0, 1, 2]
    assert L.execution_order([], 3) == [0, 1, 2]
    assert L.execution_order([], 0) == []


def test_execution_order_properties_on_random_traces():
    rng = random.Random(11)
    for _ in range(300):
        n = rng.randint(0, 12)
        uses = [rng.randrange(n) for _ in range(rng.randint(0, 30))] if n else []
        order = L.execution_order(uses, n)
        assert sorted(order) == list(range(n))                       # a permutation: every tensor once
        seen = []
        for u in uses:                                               # independent formulation: walk the trace
            if u not in seen:
                seen.append(u)
        assert order[:len(seen)] == seen                             # first occurrences, in trace order
        rest = order[len(seen):]
        assert rest == sorted(rest) and not set(rest) & set(uses)    # the unused ones behind, as declared

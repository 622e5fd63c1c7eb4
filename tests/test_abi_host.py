"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol the header declares, the integer layout builder agrees with the oracle's
index map, and argument validation returns error codes instead of crashing."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2406_08334_amd import binding as B
from paper_2406_08334_amd import shapes

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ptchunk.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pt_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = B.lib()
    names = declared_functions()
    assert len(names) >= 19
    for n in names:
        assert hasattr(L, n), f"{n} is declared in ptchunk.h but not exported"
    assert sorted(B.EXPORTS) == names            # the binding covers the whole header
    assert "ptchunk" in B.pt_version()
    assert B.status_string(0) == "PT_OK" and B.status_string(4) == "PT_ERR_STATE"


def test_layout_dense_matches_the_oracle_index_map(orc):
    rng = np.random.default_rng(2)
    for S, sizes in ((8, [1, 3, 7, 8, 9, 17]), (16, [16, 16, 1, 0, 40]), (64, [5, 300, 2, 64, 1])):
        segs, n_chunks = B.pt_layout_dense(sizes, S)
        tensors = [rng.integers(0, 1 << 16, size=n, dtype=np.uint16) for n in sizes]
        want = orc.pack_dense(tensors, S)
        assert n_chunks == want.shape[0]
        got = np.zeros_like(want)
        cover = np.zeros(want.shape, dtype=np.int32)
        for s in segs:
            assert s.len > 0 and s.chunk_off + s.len <= S and s.chunk < n_chunks
            got[s.chunk, s.chunk_off:s.chunk_off + s.len] = tensors[s.tensor][s.src_off:s.src_off + s.len]
            cover[s.chunk, s.chunk_off:s.chunk_off + s.len] += 1
        assert np.array_equal(got, want)
        assert cover.reshape(-1)[:sum(sizes)].min() == 1 and cover.max() == 1      # a partition
        assert cover.reshape(-1)[sum(sizes):].sum() == 0                           # padding untouched


def test_layout_dense_gpt2_block_worked_example():
    table, S = shapes.workload("gpt2_block_768")
    segs, n_chunks = B.pt_layout_dense([n for _, n in table], S)
    assert n_chunks == 2 and len(segs) == 13                  # c_fc.weight is cut in two
    cut = [s for s in segs if s.tensor == 8]
    assert [(s.chunk, s.chunk_off, s.src_off, s.len) for s in cut] == \
        [(0, 2_365_440, 0, S - 2_365_440), (1, 0, S - 2_365_440, 4_724_736 - S)]
    last = segs[-1]
    assert last.chunk == 1 and last.chunk_off + last.len == S - 1_300_736


def test_layout_counts_of_the_large_workloads():
    for name, want_chunks in (("gpt2_xl", 47), ("llama_7b", 101), ("llama_13b", 194)):
        table, S = shapes.workload(name)
        segs, n_chunks = B.pt_layout_dense([n for _, n in table], S)
        assert n_chunks == want_chunks
        assert sum(s.len for s in segs) == shapes.total_elems(table)
        assert all(s.chunk_off % 8 == 0 and s.src_off % 8 == 0 for s in segs)     # vector path applies


def test_argument_validation_without_a_gpu():
    L = B.lib()
    out = C.c_void_p()
    assert L.pt_ctx_create(None, 0, 64, 1, None) == B.PT_ERR_INVALID_ARG
    assert L.pt_ctx_create(C.byref(out), 7, 64, 1, None) == B.PT_ERR_INVALID_ARG
    assert L.pt_ctx_create(C.byref(out), 0, 0, 1, None) == B.PT_ERR_INVALID_ARG
    assert L.pt_ctx_create(C.byref(out), 0, 64, 0, None) == B.PT_ERR_INVALID_ARG
    assert L.pt_ctx_create(C.byref(out), 0, 60, 1, None) == B.PT_ERR_ALIGNMENT
    assert "multiple of 8" in B.pt_last_error(None)
    bad = B.pt_scaler_cfg(0.5, 2.0, 0.5, 2000, 0)
    assert L.pt_ctx_create(C.byref(out), 1, 64, 1, C.byref(bad)) == B.PT_ERR_INVALID_ARG
    n = C.c_uint32()
    sizes = (C.c_uint64 * 2)(5, 6)
    assert L.pt_layout_dense(sizes, 2, 0, None, 0, C.byref(n), C.byref(n)) == B.PT_ERR_INVALID_ARG
    assert L.pt_layout_dense(sizes, 2, 12, None, 0, C.byref(n), C.byref(n)) == B.PT_ERR_ALIGNMENT
    assert L.pt_layout_dense(sizes, 2, 8, None, 0, None, C.byref(n)) == B.PT_ERR_INVALID_ARG
    segs = (B.pt_segment * 1)()
    assert L.pt_layout_dense(sizes, 2, 8, segs, 1, C.byref(n), C.byref(n)) == B.PT_ERR_INVALID_ARG  # cap too small
    for fn in ("pt_step_end", "pt_ctx_set_state", "pt_stream_reserve"):
        pass
    assert L.pt_step_end(None, None) == B.PT_ERR_INVALID_ARG
    assert L.pt_stream_reserve(None, 2) == B.PT_ERR_INVALID_ARG
    assert L.pt_chunk_adamw_step(None, None, 0, 0, None, None, None, None, None, None) == B.PT_ERR_INVALID_ARG
    assert L.pt_ctx_destroy(None) == B.PT_OK and L.pt_pack_plan_destroy(None) == B.PT_OK
    with pytest.raises(B.PtError):
        B.pt_layout_dense([1, 2], 12)


# ---- paper-faithful layout: library vs the oracle's plain-Python layout -------------------------

def _lib_places(sizes, gids, S):
    segs, n_chunks, waste = B.pt_layout_grouped(sizes, gids, S)
    place = [None] * len(sizes)
    for s in segs:
        assert s.src_off == 0 and s.len == sizes[s.tensor]          # one whole tensor per segment
        place[s.tensor] = (s.chunk, s.chunk_off)
    return place, n_chunks, waste


def test_layout_grouped_matches_the_oracle_on_random_inputs():
    import random
    from oracle import layout as OL
    rng = random.Random(17)
    for _ in range(300):
        n = rng.randint(1, 16)
        sizes = [rng.choice([0, 1, 3, 8, 9, 17, 40, 64, 100, 250]) for _ in range(n)]
        gids, g = [], 0
        for i in range(n):
            if rng.random() < 0.3:
                g += 1
            gids.append(None if rng.random() < 0.25 else g)
        S = rng.choice([8, 16, 64, 104, 128, 256, 512])
        want = OL.layout_grouped(sizes, gids, S)
        if want is None:
            with pytest.raises(B.PtError):
                B.pt_layout_grouped(sizes, gids, S)
            continue
        assert _lib_places(sizes, gids, S) == want


def test_execution_order_matches_the_oracle_and_feeds_the_grouped_layout():
    """The library's first-use order against the oracle's on random traces; then end to end on a GPT-2-like table
    declared head first with the head tied to the token embedding: ordered by the forward trace, the embedding
    leads, the blocks follow whole, and the layout of the reordered table equals the oracle's."""
    import random
    from oracle import layout as OL
    rng = random.Random(23)
    for _ in range(300):
        n = rng.randint(0, 14)
        uses = [rng.randrange(n) for _ in range(rng.randint(0, 40))] if n else []
        assert B.pt_layout_execution_order(uses, n) == OL.execution_order(uses, n)
    with pytest.raises(B.PtError):
        B.pt_layout_execution_order([0, 3], 3)                      # names a tensor that does not exist
    # declaration: 0 wte (tied head), 1 ln_f.g, 2 ln_f.b, then two blocks of three tensors, 9 wpe
    sizes = [4096, 64, 64, 640, 72, 640, 640, 72, 640, 512]
    gids = [None, None, None, 0, 0, 0, 1, 1, 1, None]
    trace = [0, 9, 3, 4, 5, 6, 7, 8, 1, 2, 0]                        # embeddings, blocks, final norm, head = wte again
    order = B.pt_layout_execution_order(trace, len(sizes))
    assert order == [0, 9, 3, 4, 5, 6, 7, 8, 1, 2]
    o_sizes, o_gids = [sizes[t] for t in order], [gids[t] for t in order]
    S = 4096
    place, n_chunks, waste = _lib_places(o_sizes, o_gids, S)
    assert (place, n_chunks, waste) == OL.layout_grouped(o_sizes, o_gids, S)
    assert place[0] == (0, 0) and place[1][0] == 1                   # the shared embedding alone in chunk 0, wpe opens chunk 1
    assert len({place[k][0] for k in (2, 3, 4)}) == 1 and len({place[k][0] for k in (5, 6, 7)}) == 1   # blocks whole


def test_chunk_size_search_matches_the_oracle_and_the_papers_table():
    import random
    from oracle import layout as OL
    for name, make, want_chunks in (("gpt2_1b", lambda: shapes.gpt2(1600, 32, 6400), 12),
                                    ("gpt2_10b", lambda: shapes.gpt2(4096, 48, 16384), 49)):
        table = make()
        sizes, gids = [n for _, n in table], shapes.block_ids(table)
        got = B.pt_chunk_size_search(sizes, gids, 0, 1 << 25, 1 << 20)
        assert got == OL.chunk_size_search(sizes, gids, 0, 1 << 25, 1 << 20)
        assert got[1] == want_chunks                                   # Table 4 of the paper
        assert _lib_places(sizes, gids, got[0]) == OL.layout_grouped(sizes, gids, got[0])
    rng = random.Random(3)
    for _ in range(100):
        n = rng.randint(1, 10)
        sizes = [rng.randint(1, 90) for _ in range(n)]
        gids = [rng.choice([None, 0, 1, 2]) for _ in range(n)]
        span, mn = 8 * rng.randint(0, 10), rng.choice([0, 0, 64])
        assert B.pt_chunk_size_search(sizes, gids, mn, span, 8) == OL.chunk_size_search(sizes, gids, mn, span, 8)
    with pytest.raises(B.PtError):
        B.pt_chunk_size_search([5, 6], None, 0, 64, 12)                # step not a multiple of 8


def test_llama7b_grouped_layout_keeps_every_block_whole():
    table, _ = shapes.workload("llama_7b")
    sizes, gids = [n for _, n in table], shapes.block_ids(table)
    block = 4 * 4096 ** 2 + 3 * 4096 * 11008 + 2 * 4096
    # the embedding (131 M) is the largest tensor; a block (202 M) only fits if the search starts there
    S, n_chunks, waste = B.pt_chunk_size_search(sizes, gids, block, 1 << 25, 1 << 20)
    place, n2, w2 = _lib_places(sizes, gids, S)
    assert (n2, w2) == (n_chunks, waste)
    assert S >= block and n_chunks == 34                               # embedding, 32 blocks, norm + head
    for b in range(32):
        assert len({place[t][0] for t, g in enumerate(gids) if g == b}) == 1
    assert waste < 0.03 * sum(sizes)


def test_context_creation_without_a_gpu_is_an_error_code_not_a_crash():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present: creation succeeds here")
    out = C.c_void_p()
    assert B.lib().pt_ctx_create(C.byref(out), 0, 64, 1, None) == B.PT_ERR_HIP
    assert not out.value and "hipGetDevice" in B.pt_last_error(None)
    with pytest.raises(B.PtError):
        B.pt_ctx_create(B.PT_BF16, 64, 1)


def test_bench_refuses_more_than_one_gpu():
    """the benchmark is a one-GPU program: --gpus above 1 exits with a message, before any GPU work"""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode == 2 and "ONE GPU" in res.stderr and res.stdout.strip() == ""

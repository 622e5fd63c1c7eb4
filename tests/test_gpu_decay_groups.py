"""GPU parity of the weight-decay groups: element runs kept out of the decay, through every
placement of a chunk (resident kernel, streamed through slots, updated by host threads).
The oracle takes the same choice as a per-element mask."""
import numpy as np
import pytest
import torch

from paper_2406_08334_amd import binding as B
from paper_2406_08334_amd import shapes

from gpu_harness import ChunkedState, hp_pair, to_u16, same_bits, assert_same_bits
from test_gpu_parity import end_to_end, run_mixed, run_oracle_f32seq

pytestmark = pytest.mark.gpu

TILE = 4096                       # elements of one kernel tile at the default unroll


def awkward_runs(S):
    """Runs that cover whole tiles, cut tiles, straddle tile edges, touch, overlap and sit in the
    ragged tail; given out of order on purpose."""
    return [
        (0, 5000, 3), (0, 0, TILE), (0, 2 * TILE - 1, 2), (0, 5 * TILE, S - 5 * TILE),
        (1, 0, S),
        (2, 150, 150), (2, 100, 100), (2, 300, 1), (2, 3 * TILE + 4, TILE), (2, 777, 0), (2, S - 1, 1),
    ]


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16])
@pytest.mark.parametrize("unroll,threads", [(4, 512), (1, 512), (8, 512), (4, 256), (8, 256)])
def test_masked_kernel_is_bit_exact_against_the_masked_f32_sequence(orc, dtype, unroll, threads):
    S, C = TILE * 5 + 40, 4
    st = ChunkedState([S * C - 5], S, dtype=dtype)
    try:
        B.pt_ctx_set_option(st.ctx, "adamw_unroll", unroll)
        B.pt_ctx_set_option(st.ctx, "adamw_threads", threads)
        B.pt_ctx_set_option(st.ctx, "adamw_nt", 1 if unroll != 8 else 2)     # hinted accesses too (a small state gets none by default)
        hp_b, hp_o, _ = hp_pair()
        mask = st.set_no_decay(runs=awkward_runs(S))
        assert 0 < mask.sum() < mask.size
        host = st.host_state()
        plain = {k: a.copy() for k, a in host.items()}
        for t in (1, 2):
            st.set_grads(t)
            st.pack()
            B.pt_step_override(st.ctx, 0.0121, False)
            st.adamw(hp_b)
            k = B.pt_update_consts_read(st.ctx)
            st.end()
            consts = orc.consts_f32(hp_o, t, float(np.float32(0.0121)))
            assert same_bits(np.array(list(k.c), dtype=np.float32), consts)      # the oracle runs on its own constants
            g16 = orc.pack_dense([to_u16(st.grad_src[:st.N])], S, st.C).reshape(-1)     # ... and its own packing
            assert_same_bits(to_u16(st.g16).reshape(-1), g16, ("g16", t))
            host["g16"] = plain["g16"] = g16.copy()
            run_oracle_f32seq(orc, consts, host, st.orc_dtype, no_decay=mask)
            run_oracle_f32seq(orc, consts, plain, st.orc_dtype)
            got = st.host_state()
            for name in ("w", "m", "v", "p16"):
                assert_same_bits(got[name], host[name], (name, t, unroll))
        # the mask matters where it is set and nowhere else
        differs = host["w"] != plain["w"]
        assert differs[mask == 0].sum() == 0 and differs[mask == 1].mean() > 0.9
    finally:
        st.close()


def test_clearing_the_list_restores_the_plain_update(orc):
    S = TILE * 2 + 8
    outs = []
    for use in (False, True):
        st = ChunkedState([3 * S], S)
        try:
            hp_b, _, _ = hp_pair()
            if use:
                st.set_no_decay(runs=[(1, 5, 4000)])
                st.set_no_decay()                                 # empty list: no run is left
            st.set_grads(1)
            st.step(hp_b)
            outs.append(st.host_state())
        finally:
            st.close()
    for name in ("w", "m", "v", "p16"):
        assert same_bits(outs[0][name], outs[1][name]), name


def test_runs_outside_the_chunks_are_refused():
    st = ChunkedState([10_000], 4096)
    try:
        for run in ((3, 0, 8), (0, 4096, 1), (0, 4000, 97)):
            with pytest.raises(B.PtError) as e:
                st.set_no_decay(runs=[run])
            assert e.value.status == B.PT_ERR_INVALID_ARG
        st.set_no_decay(runs=[(2, 4095, 1)])                      # the last element is fine
    finally:
        st.close()


def test_end_to_end_gpt2_block_with_biases_and_norm_gains_undecayed(orc):
    table, S = shapes.workload("gpt2_block_768")
    nd = [i for i, (name, _) in enumerate(table) if name.endswith(".bias") or ".ln_" in name]
    assert len(nd) == 8
    end_to_end(orc, [n for _, n in table], 1 << 20, torch.bfloat16, steps=3, no_decay_tensors=nd)


@pytest.mark.parametrize("dtype,scaler", [(torch.bfloat16, None),
                                          (torch.float16, B.pt_scaler_cfg(65536.0, 2.0, 0.5, 2000, 0))])
def test_streamed_and_host_updated_chunks_honour_the_runs(orc, dtype, scaler):
    S = 40_000
    sizes = [6 * S - 24]
    runs = [(0, 0, 100), (1, 39_000, 1000), (2, 0, S), (3, 4095, 3), (3, 20_000, 9000), (5, 39_900, 76)]
    ref = run_mixed(sizes, S, 6, 2, steps=2, dtype=dtype, scaler=scaler, no_decay_runs=runs, orc=orc)
    plain = run_mixed(sizes, S, 6, 2, steps=2, dtype=dtype, scaler=scaler)
    assert not torch.equal(ref["w"], plain["w"])
    for n_persist, n_slots, host_update in ((3, 2, False), (0, 3, False), (5, 2, False), (3, 2, True), (0, 2, True)):
        got = run_mixed(sizes, S, n_persist, n_slots, steps=2, dtype=dtype, scaler=scaler, host_update=host_update,
                        no_decay_runs=runs, orc=orc)     # every chunk, wherever it is updated, against the oracle
        for name in ("p16", "w", "m", "v"):
            view = torch.int16 if got[name].element_size() == 2 else torch.int32
            assert torch.equal(got[name].view(view), ref[name].view(view)), (name, n_persist, n_slots, host_update)

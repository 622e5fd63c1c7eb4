"""GPU parity at the benchmark's full sizes, in the launch configurations bench.py times
(all chunks of the state resident, one AdamW launch over the whole pointer table; and the
split state: a resident prefix next to chunks that live in pinned host memory).

Every element is checked: pack through the layout's defining property (dense layout = flat
concatenation), the norm through one fp64 pass of the oracle per chunk in every step, and
the update of the FIRST step on every chunk - one chunk at a time through pinned staging
buffers - bit for bit against the oracle's fp32 sequence, started from the seeded initial
state (16-bit parameters, master = their exact decode, zero moments).  The configurations'
own step counts then run on whole sampled chunks (first, middle, last-with-padding, the
chunk holding a planted inf, and for the split state chunks on both sides of the cut),
carried by the oracle beside the device: bit-exact through the fp32 sequence and within
tolerance of the fp64 evaluation in every step.
"""
import gc
import math
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import oracle as O
from paper_2406_08334_amd import binding as B
from paper_2406_08334_amd import shapes, synth
from gpu_harness import HP, assert_same_bits, hp_pair, to_u16
from tolerance import ScaleTracker, check_p16, far_cap

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


@pytest.fixture(autouse=True)
def progress_lines_bypass_capture(capsys):
    """These tests run for minutes: their progress lines go to the real stdout even when pytest captures
    output, so that whoever watches the run sees that it is alive."""
    global say

    def uncaptured(msg):
        with capsys.disabled():
            print(msg, flush=True)
    say = uncaptured
    yield
    say = lambda msg: print(msg, flush=True)


class FullState:
    def __init__(self, workload, dtype, scaler=None):
        table, S = shapes.workload(workload)
        self.sizes = [n for _, n in table]
        self.S, self.N = S, sum(self.sizes)
        self.dtype = dtype
        self.pt_dtype = B.PT_BF16 if dtype == torch.bfloat16 else B.PT_FP16
        self.orc_dtype = O.BF16 if dtype == torch.bfloat16 else O.FP16
        self.segs, self.C = B.pt_layout_dense(self.sizes, S)
        C, N, dev = self.C, self.N, "cuda"
        self.ctx = B.pt_ctx_create(self.pt_dtype, S, C, scaler)
        self.grad_src = torch.empty(N, dtype=dtype, device=dev)
        offs = np.cumsum([0] + self.sizes[:-1]).tolist()
        for s in self.segs:
            s.src = self.grad_src.data_ptr() + 2 * offs[s.tensor]
        self.plan = B.pt_pack_plan_create(self.ctx, self.segs)
        self.g16 = torch.zeros(C, S, dtype=dtype, device=dev)
        self.p16 = torch.zeros(C, S, dtype=dtype, device=dev)
        synth.normal_16(synth.SEED_PARAMS, 0, 0, 0, N, 0.02, dtype, dev, out=self.p16.view(-1)[:N])
        self.w = torch.empty(C, S, dtype=torch.float32, device=dev)
        for c in range(C):
            self.w[c].copy_(self.p16[c])
        self.m = torch.zeros(C, S, dtype=torch.float32, device=dev)
        self.v = torch.zeros(C, S, dtype=torch.float32, device=dev)
        self.p16_init = self.p16.clone()
        self.rows = lambda a: [a[c] for c in range(C)]
        torch.cuda.synchronize()

    def chunk_host(self, c):
        return dict(g16=to_u16(self.g16[c]).copy(), p16=to_u16(self.p16[c]).copy(), w=self.w[c].cpu().numpy().copy(),
                    m=self.m[c].cpu().numpy().copy(), v=self.v[c].cpu().numpy().copy())

    def oracle_sqnorm(self, sigma):
        """fp64 sum of squares over every chunk: inside a chunk in index order (one oracle call, one
        thread), the chunk sums added in chunk order.  Chunks travel through a ring of pinned buffers
        and are summed by a pool of threads (the oracle's C++ runs outside the interpreter lock)."""
        K = 12
        if getattr(self, "_pins", None) is None:
            self._pins = [torch.empty(self.S, dtype=torch.int16).pin_memory() for _ in range(K)]
        views = [p.numpy().view(np.uint16) for p in self._pins]

        def job(k):
            g = views[k]
            return O.sqnorm(g, self.orc_dtype, loss_scale=sigma, block=self.S, threads=1), O.found_nonfinite(g, self.orc_dtype)

        sums, found, pending = [], False, [None] * K
        with ThreadPoolExecutor(max_workers=K) as ex:
            for c in range(self.C):
                k = c % K
                if pending[k] is not None:
                    sq, f = pending[k].result()
                    sums.append(sq); found = found or f
                self._pins[k].copy_(self.g16[c].view(torch.int16))
                pending[k] = ex.submit(job, k)
            for j in range(K):                       # the rest, in chunk order
                k = (self.C + j) % K
                if pending[k] is not None:
                    sq, f = pending[k].result()
                    sums.append(sq); found = found or f
                    pending[k] = None
        assert len(sums) == self.C
        total = 0.0
        for sq in sums:
            total += sq
        return total, found

    def staged(self, c):
        """The five arrays of chunk c as numpy views of pinned staging buffers (valid until the next call)."""
        if getattr(self, "_stage", None) is None:
            self._stage = {k: torch.empty(self.S, dtype=dt).pin_memory() for k, dt in
                           (("g16", torch.int16), ("p16", torch.int16), ("w", torch.float32), ("m", torch.float32),
                            ("v", torch.float32))}
        for k, src in self.chunk_arrays(c).items():
            self._stage[k].copy_(src.view(torch.int16) if src.element_size() == 2 else src)
        torch.cuda.synchronize()
        return {k: (t.numpy().view(np.uint16) if t.dtype == torch.int16 else t.numpy()) for k, t in self._stage.items()}

    def chunk_arrays(self, c):
        return dict(g16=self.g16[c], p16=self.p16[c], w=self.w[c], m=self.m[c], v=self.v[c])

    def source_chunk(self, c):
        """gradient words of chunk c as the dense layout defines them, from the seeded source tensor itself"""
        S, N = self.S, self.N
        src = to_u16(self.grad_src[c * S: min(N, (c + 1) * S)])
        if src.size == S:
            return src
        out = np.zeros(S, np.uint16)
        out[:src.size] = src
        return out

    def initial_chunk(self, c):
        """the seeded 16-bit parameters chunk c started from (kept on the device since before the first step)"""
        return to_u16(self.p16_init[c]).copy()

    def run_step(self, hp_b):
        """pack -> norm -> update of every chunk, as the benchmark enqueues it"""
        C = self.C
        B.pt_chunk_pack_grads(self.ctx, self.plan, self.rows(self.g16))
        B.pt_chunk_grad_sqnorm(self.ctx, None, 0, C, True)
        B.pt_chunk_adamw_step(self.ctx, hp_b, 0, C, self.rows(self.g16), self.rows(self.w), self.rows(self.m),
                              self.rows(self.v), self.rows(self.p16))

    def check_pack(self):
        """every element: the dense layout is the flat concatenation, padding stays zero"""
        N = self.N
        assert torch.equal(self.g16.view(-1)[:N].view(torch.int16), self.grad_src.view(torch.int16))
        assert not bool(self.g16.view(-1)[N:].view(torch.int16).any())

    def check_padding(self):
        """padding of the last chunk stayed exactly zero through every step"""
        C, S = self.C, self.S
        pad = C * S - self.N
        if pad:
            for a in (self.w, self.m, self.v):
                assert not bool(a[C - 1][S - pad:].any())
            assert not bool(self.p16[C - 1][S - pad:].view(torch.int16).any())

    def close(self):
        torch.cuda.synchronize()
        B.pt_pack_plan_destroy(self.plan)
        B.pt_ctx_destroy(self.ctx)
        for name in ("grad_src", "g16", "p16", "w", "m", "v", "host", "_pins", "_stage", "p16_init"):
            setattr(self, name, None)
        gc.collect()
        torch.cuda.empty_cache()


def host_memory_total_gb():
    for line in open("/proc/meminfo"):
        if line.startswith("MemTotal:"):
            return int(line.split()[1]) * 1024 / 1e9
    return float("nan")


class SplitState(FullState):
    """The first n_resident + n_host chunks of a workload's dense layout: the prefix lives in HBM,
    the rest in pinned host memory and takes the streamed update.  n_host is as many of n_host_wanted
    chunks as the box lets this process pin (allocation stops at the first refusal; three chunks of
    headroom are given back for the staging buffers).  Gradient chunks are packed on the device
    (where their norm partials are taken) and the host chunks' gradients offloaded."""

    def __init__(self, workload, dtype, n_resident, n_host_wanted, n_slots=3):
        table, S = shapes.workload(workload)
        self.sizes = [n for _, n in table]
        self.S, self.dtype = S, dtype
        self.pt_dtype = B.PT_BF16 if dtype == torch.bfloat16 else B.PT_FP16
        self.orc_dtype = O.BF16 if dtype == torch.bfloat16 else O.FP16
        segs, c_all = B.pt_layout_dense(self.sizes, S)
        # Everything else that needs pinned memory comes first (the staging buffers; the runtime's own needs when the
        # context and its streams are created happen later but find the headroom given back below).
        self._pins = [torch.empty(S, dtype=torch.int16).pin_memory() for _ in range(12)]
        self._stage = {k: torch.empty(S, dtype=dt).pin_memory() for k, dt in
                       (("g16", torch.int16), ("p16", torch.int16), ("w", torch.float32), ("m", torch.float32),
                        ("v", torch.float32))}
        kinds = (("g16", dtype), ("p16", dtype), ("w", torch.float32), ("m", torch.float32), ("v", torch.float32))
        self.host = {name: [] for name, _ in kinds}
        for i in range(n_host_wanted):
            try:
                got = [torch.zeros(S, dtype=dt, pin_memory=True) for _, dt in kinds]
            except RuntimeError as e:
                say(f"[fullsize] pinning stopped after {i} host chunks ({16 * i * S / 1e9:.1f} GB pinned; host RAM "
                    f"{host_memory_total_gb():.0f} GB): {str(e).splitlines()[0][:120]}")
                got = None
                for name in self.host:
                    del self.host[name][max(0, i - 4):]
                gc.collect()
                torch._C._host_emptyCache()     # hands the dropped chunks back to the driver: real headroom for the runtime
                break
            for (name, _), t in zip(kinds, got):
                self.host[name].append(t)
            if i % 16 == 15:
                say(f"[fullsize] {i + 1} host chunks pinned")
        n_host = len(self.host["w"])
        assert n_host >= 8, "the box pins fewer than 8 host chunks"
        say(f"[fullsize] {n_resident} resident chunks, {n_host} of {n_host_wanted} host chunks pinned "
            f"({16 * n_host * S / 1e9:.1f} GB; host RAM {host_memory_total_gb():.0f} GB)")
        C = self.C = n_resident + n_host
        assert C < c_all, "the cut must fall on a chunk boundary before the padded last chunk"
        self.n_resident, self.n_host = n_resident, n_host
        N = self.N = C * S
        dev = "cuda"
        self.segs = [s for s in segs if s.chunk < C]
        self.ctx = B.pt_ctx_create(self.pt_dtype, S, C, None)
        B.pt_stream_reserve(self.ctx, n_slots)
        self.grad_src = torch.empty(N, dtype=dtype, device=dev)
        offs = np.cumsum([0] + self.sizes[:-1]).tolist()
        for s in self.segs:
            s.src = self.grad_src.data_ptr() + 2 * offs[s.tensor]
        self.plan = B.pt_pack_plan_create(self.ctx, self.segs)
        self.g16 = torch.zeros(C, S, dtype=dtype, device=dev)
        R = n_resident
        self.p16 = torch.zeros(R, S, dtype=dtype, device=dev)
        synth.normal_16(synth.SEED_PARAMS, 0, 0, 0, R * S, 0.02, dtype, dev, out=self.p16.view(-1))
        self.w = torch.empty(R, S, dtype=torch.float32, device=dev)
        for c in range(R):
            self.w[c].copy_(self.p16[c])
        self.m = torch.zeros(R, S, dtype=torch.float32, device=dev)
        self.v = torch.zeros(R, S, dtype=torch.float32, device=dev)
        self.p16_init = self.p16.clone()
        self.host_p16_init = []
        tmp = torch.empty(S, dtype=dtype, device=dev)
        for i in range(n_host):
            synth.normal_16(synth.SEED_PARAMS, 0, 0, (R + i) * S, S, 0.02, dtype, dev, out=tmp)
            self.host["p16"][i].copy_(tmp)
            self.host["w"][i].copy_(tmp.float())
            self.host_p16_init.append(self.host["p16"][i].clone())
        self.rows = lambda a, lo=0, hi=None: [a[c] for c in range(lo, a.shape[0] if hi is None else hi)]
        torch.cuda.synchronize()

    def chunk_arrays(self, c):
        R = self.n_resident
        if c < R:
            return dict(g16=self.g16[c], p16=self.p16[c], w=self.w[c], m=self.m[c], v=self.v[c])
        return {name: self.host[name][c - R] for name in self.host}

    def initial_chunk(self, c):
        R = self.n_resident
        return to_u16(self.p16_init[c] if c < R else self.host_p16_init[c - R]).copy()

    def chunk_host(self, c):
        torch.cuda.synchronize()
        R = self.n_resident
        if c < R:
            return dict(g16=to_u16(self.g16[c]).copy(), p16=to_u16(self.p16[c]).copy(), w=self.w[c].cpu().numpy().copy(),
                        m=self.m[c].cpu().numpy().copy(), v=self.v[c].cpu().numpy().copy())
        h = {name: self.host[name][c - R] for name in self.host}
        return dict(g16=to_u16(h["g16"]).copy(), p16=to_u16(h["p16"]).copy(), w=h["w"].numpy().copy(),
                    m=h["m"].numpy().copy(), v=h["v"].numpy().copy())

    def run_step(self, hp_b):
        R, C, h = self.n_resident, self.C, self.host
        B.pt_chunk_pack_grads(self.ctx, self.plan, self.rows(self.g16))
        for i in range(self.n_host):                                # the offload of the gradient chunks
            h["g16"][i].copy_(self.g16[R + i], non_blocking=True)
        torch.cuda.synchronize()
        B.pt_chunk_grad_sqnorm(self.ctx, None, 0, C, True)
        B.pt_chunk_stream_step(self.ctx, hp_b, R, C - R, h["g16"], h["w"], h["m"], h["v"], h["p16"])
        B.pt_chunk_adamw_step(self.ctx, hp_b, 0, R, self.rows(self.g16, 0, R), self.rows(self.w), self.rows(self.m),
                              self.rows(self.v), self.rows(self.p16))

    def check_padding(self):
        pass                                                         # the cut leaves whole chunks only

    def close(self):
        self.host_p16_init = None
        super().close()


def check_every_chunk_after_the_first_step(st, consts):
    """Every element of every chunk, bit for bit: the oracle's fp32 sequence from the seeded initial
    state (16-bit parameters, master weights = their exact decode, zero moments) and the seeded
    gradients, against what the device (or the streamed path) left in the chunk."""
    S = st.S
    t0 = time.time()
    zeros = np.zeros(S, np.float32)
    for c in range(st.C):
        p = st.initial_chunk(c)
        w = O.decode16(p, st.orc_dtype)
        m, v = zeros.copy(), zeros.copy()
        g = st.source_chunk(c)
        O.adamw_f32seq(consts, g, w, m, v, p, st.orc_dtype, threads=16)
        got = st.staged(c)
        assert_same_bits(got["g16"], g, ("g16", c))
        for name, want in (("w", w), ("m", m), ("v", v), ("p16", p)):
            assert_same_bits(got[name], want, (name, "chunk", c, "first step, every element"))
        if c % 10 == 0 or c == st.C - 1:
            say(f"[fullsize] first step, every element: chunk {c + 1}/{st.C} ok ({time.time() - t0:.0f} s)")


def run_full(workload, dtype, steps, scaler_b=None, scaler_o=None, inf_step=None, outlier_every=0, sample=None,
             make_state=None, every_chunk=True):
    st = make_state() if make_state is not None else FullState(workload, dtype, scaler_b)
    try:
        hp_b, hp_o, hpd = hp_pair()
        C, S, N = st.C, st.S, st.N
        sample = sorted(set(sample(st) if callable(sample) else sample if sample is not None else [0, C // 2, C - 1]))
        inf_elem = synth.pick_element(synth.SEED_INF, inf_step, N) if inf_step else None
        if inf_elem is not None and inf_elem // S not in sample:
            sample.append(inf_elem // S)
        ost = O.new_state(scaler_o)
        shadow = {}                      # per sampled chunk: f64-oracle state, f32-sequence state, scale tracker
        for c in sample:
            h = st.chunk_host(c)
            shadow[c] = dict(f64={k: a.copy() for k, a in h.items()}, f32={k: a.copy() for k, a in h.items()},
                             trk=ScaleTracker(h["w"], h["m"], hpd))
        out = []
        for s in range(1, steps + 1):
            say(f"[fullsize] {workload} {dtype} step {s}/{steps}")
            sigma = ost.loss_scale
            synth.normal_16(synth.SEED_GRADS, s, 0, 0, N, 1e-3, dtype, "cuda", scale=sigma,
                            outlier_every=outlier_every, out=st.grad_src)
            if inf_step == s:
                st.grad_src.view(torch.int16)[inf_elem] = 0x7C00 if dtype == torch.float16 else 0x7F80
            st.run_step(hp_b)
            rep = B.pt_step_report_read(st.ctx)
            k = B.pt_update_consts_read(st.ctx)
            B.pt_step_end(st.ctx)
            torch.cuda.synchronize()
            st.check_pack()
            # norm, every element
            want_sq, want_inf = st.oracle_sqnorm(sigma)
            assert rep.found_inf == int(want_inf)
            after = B.pt_step_report_read(st.ctx)
            if want_inf:
                assert k.skip == 1 and inf_step == s
                for c in sample:
                    got = st.chunk_host(c)
                    for name in ("w", "m", "v", "p16"):
                        assert_same_bits(got[name], shadow[c]["f32"][name], (name, c, s))
                if scaler_o is not None:
                    ost.loss_scale = max(sigma * scaler_o.backoff, 1.0); ost.good_steps = 0
                assert after.step == ost.t and after.loss_scale == ost.loss_scale
                out.append(rep)
                continue
            want_norm = math.sqrt(want_sq)
            assert abs(rep.norm - want_norm) <= 1e-5 * want_norm
            # the oracle adds 2^26 terms per chunk one after the other in fp64: its own rounding
            # error is up to n * 2^-53 ~ 7e-9 relative (seen: 4e-11); the tree-shaped GPU sum is tighter
            assert abs(rep.sqnorm - want_sq) <= 1e-9 * want_sq
            clip = O.clip_coef(want_norm, hpd["max_norm"])
            gm = clip / sigma
            assert abs(rep.clip_coef - clip) <= 1e-9 * clip and abs(rep.grad_mult - gm) <= 6e-8 * gm
            ost.t += 1
            if scaler_o is not None:
                ost.good_steps += 1
            assert after.step == ost.t and after.loss_scale == ost.loss_scale
            # The fp32 sequence runs on the oracle's own constants.  Eight of the nine do not depend on the norm
            # and must equal the device's bit for bit; grad_mult does, and the oracle's one-after-the-other fp64
            # sum of 6.7e9 squares is itself only good to ~1e-10, so once in a thousand steps its fp32 rounding
            # may land on the neighbouring value: then (and only then) the device's grad_mult is taken.
            dev_c = np.array(list(k.c), dtype=np.float32)
            consts = O.consts_f32(hp_o, ost.t, gm)
            assert consts[:8].tobytes() == dev_c[:8].tobytes()
            assert abs(int(consts[8:].view(np.int32)[0]) - int(dev_c[8:].view(np.int32)[0])) <= 1
            if consts[8] != dev_c[8]:
                say(f"[fullsize] step {s}: grad_mult one ulp apart, taking the device's")
                consts[8] = dev_c[8]
            if s == 1 and every_chunk:
                check_every_chunk_after_the_first_step(st, consts)
            for c in sample:
                got = st.chunk_host(c)
                sh = shadow[c]
                # the chunk's gradients as the dense layout defines them, from the seeded source itself
                want_g = st.source_chunk(c)
                assert_same_bits(got["g16"], want_g, ("g16", c, s))
                got["g16"] = want_g
                sh["f32"]["g16"] = got["g16"]
                O.adamw_f32seq(consts, got["g16"], sh["f32"]["w"], sh["f32"]["m"], sh["f32"]["v"], sh["f32"]["p16"],
                               st.orc_dtype, threads=16)
                for name in ("w", "m", "v", "p16"):
                    assert_same_bits(got[name], sh["f32"][name], (name, c, s))
                O.adamw_f64(hp_o, ost.t, gm, got["g16"], sh["f64"]["w"], sh["f64"]["m"], sh["f64"]["v"], sh["f64"]["p16"],
                            st.orc_dtype, threads=16)
                sh["trk"].advance(ost.t, O.decode16(got["g16"], st.orc_dtype).astype(np.float64) * gm, sh["f64"]["v"])
                sh["trk"].check((got["w"], got["m"], got["v"]), (sh["f64"]["w"], sh["f64"]["m"], sh["f64"]["v"]), tol=1e-6)
                far = check_p16(O.decode16(got["p16"], st.orc_dtype), O.decode16(sh["f64"]["p16"], st.orc_dtype),
                                sh["f64"]["w"], sh["trk"].W, dtype == torch.float16)
                assert far <= far_cap(S)
            out.append(rep)
        st.check_padding()
        return out
    finally:
        st.close()


def test_llama7b_bf16_full_state_five_steps():
    """the headline configuration: 101 chunks resident, 5 steps"""
    reps = run_full("llama_7b", torch.bfloat16, steps=5)
    for r in reps:
        assert abs(r.norm - 82.09) < 0.05 and r.clip_coef < 0.0125          # 1e-3 * sqrt(6,738,415,616)


def test_gpt2xl_bf16_outliers_trigger_clipping_five_steps():
    reps = run_full("gpt2_xl", torch.bfloat16, steps=5, outlier_every=1000)
    for r in reps:
        assert abs(r.norm - 130.9) < 1.0                                     # 39.47 without the outliers


def test_llama7b_fp16_loss_scaling_with_planted_inf_six_steps():
    sb = B.pt_scaler_cfg(65536.0, 2.0, 0.5, 2000, 0)
    so = O.ScalerCfg(65536.0, 2.0, 0.5, 2000, 1)
    reps = run_full("llama_7b", torch.float16, steps=6, scaler_b=sb, scaler_o=so, inf_step=3, sample=[0])
    assert [r.found_inf for r in reps] == [0, 0, 1, 0, 0, 0]
    assert [r.loss_scale for r in reps] == [65536.0, 65536.0, 65536.0, 32768.0, 32768.0, 32768.0]


def test_llama13b_half_resident_half_streamed_from_pinned_host_memory():
    """The split configuration: 97 chunks (104 GB) resident; of the configuration's 97 host chunks as
    many as the box lets one process pin (the limit is the driver's, not the host's RAM: it is printed
    with the RAM size).  Norm over every element of all chunks; first step on every element of every
    chunk, resident and streamed; two steps on sampled chunks on both sides of the cut."""
    n_res = 97
    reps = run_full("llama_13b", torch.bfloat16, steps=2,
                    sample=lambda st: [0, n_res - 1, n_res, n_res + st.n_host // 2, st.C - 1],
                    make_state=lambda: SplitState("llama_13b", torch.bfloat16, n_res, 97))
    assert len(reps) == 2

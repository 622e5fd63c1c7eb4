"""Shared scaffolding of the GPU parity tests: a model state laid out in chunks on the
device (through the C-ABI binding) next to the same state as flat numpy arrays for
the oracle.  Holds no arithmetic of the method."""
from __future__ import annotations

import numpy as np
import torch

import oracle as O
from paper_2406_08334_amd import binding as B
from paper_2406_08334_amd import synth

HP = dict(lr=1e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, max_norm=1.0)


def hp_pair(**kw):
    d = dict(HP); d.update(kw)
    return B.hparams(**d), O.Hparams(**d), d


def to_u16(t: torch.Tensor) -> np.ndarray:
    """bits of a 16-bit tensor (any device) as numpy uint16"""
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


class ChunkedState:
    """Dense layout of `sizes` into chunks of S elements; arenas are [C, S] tensors so
    that arena.view(-1) IS the flat concatenation (plus padding) the oracle works on."""

    def __init__(self, sizes, S, dtype=torch.bfloat16, scaler=None, param_std=0.02, seed=0,
                 resident=None, init_params=True, grad_fp32=False):
        self.sizes = [int(s) for s in sizes]
        self.S = int(S)
        self.N = sum(self.sizes)
        self.dtype = dtype
        self.pt_dtype = B.PT_BF16 if dtype == torch.bfloat16 else B.PT_FP16
        self.orc_dtype = O.BF16 if dtype == torch.bfloat16 else O.FP16
        self.segs, self.C = B.pt_layout_dense(self.sizes, self.S)
        self.C = max(self.C, 1)
        self.seed = seed
        dev = "cuda"
        C, S = self.C, self.S
        self.ctx = B.pt_ctx_create(self.pt_dtype, S, C, scaler)
        self.grad_fp32 = grad_fp32
        if grad_fp32:                      # micro-batches are accumulated into fp32 gradient chunks
            B.pt_ctx_set_option(self.ctx, "grad_fp32", 1)
            self.g32 = torch.zeros(C, S, dtype=torch.float32, device=dev)
        # gradient tensors: one flat buffer, tensor t at the running offset (so odd sizes give
        # sources that are only 2-byte aligned)
        self.grad_src = torch.zeros(max(self.N, 1), dtype=dtype, device=dev)
        offs = np.cumsum([0] + self.sizes[:-1]).tolist() if self.sizes else []
        for s in self.segs:
            s.src = self.grad_src.data_ptr() + 2 * offs[s.tensor]
        self.plan = B.pt_pack_plan_create(self.ctx, self.segs)
        self.g16 = torch.zeros(C, S, dtype=dtype, device=dev)
        self.p16 = torch.zeros(C, S, dtype=dtype, device=dev)
        self.w = torch.zeros(C, S, dtype=torch.float32, device=dev)
        self.m = torch.zeros(C, S, dtype=torch.float32, device=dev)
        self.v = torch.zeros(C, S, dtype=torch.float32, device=dev)
        if init_params and self.N:
            synth.normal_16(synth.SEED_PARAMS + seed, 0, 0, 0, self.N, param_std, dtype, dev,
                            out=self.p16.view(-1)[:self.N])
            self.w.copy_(self.p16.float())
        torch.cuda.synchronize()

    # ---- per-chunk pointer lists
    def rows(self, arena, lo=0, hi=None):
        hi = self.C if hi is None else hi
        return [arena[c] for c in range(lo, hi)]

    def set_grads(self, step, std=1e-3, scale=1.0, outlier_every=0, micro=0):
        if self.N:
            synth.normal_16(synth.SEED_GRADS + self.seed, step, micro, 0, self.N, std, self.dtype, "cuda",
                            scale=scale, outlier_every=outlier_every, out=self.grad_src[:self.N])

    @property
    def grads(self):
        """the gradient chunks the norm and the update read"""
        return self.g32 if self.grad_fp32 else self.g16

    def accum(self, overwrite, take_norm):
        B.pt_chunk_accum_grads(self.ctx, self.plan, self.rows(self.g32), overwrite, take_norm)

    # ---- the calls
    def pack(self):
        B.pt_chunk_pack_grads(self.ctx, self.plan, self.rows(self.g16))

    def norm(self, recompute=False, finalize=True):
        B.pt_chunk_grad_sqnorm(self.ctx, self.rows(self.grads) if recompute else None, 0, self.C, finalize)

    def adamw(self, hp, lo=0, hi=None):
        hi = self.C if hi is None else hi
        B.pt_chunk_adamw_step(self.ctx, hp, lo, hi - lo, self.rows(self.grads, lo, hi), self.rows(self.w, lo, hi),
                              self.rows(self.m, lo, hi), self.rows(self.v, lo, hi), self.rows(self.p16, lo, hi))

    def end(self):
        B.pt_step_end(self.ctx)

    def step(self, hp):
        self.pack(); self.norm(); self.adamw(hp)
        rep = B.pt_step_report_read(self.ctx)
        self.end()
        return rep

    def report(self):
        return B.pt_step_report_read(self.ctx)

    def set_no_decay(self, tensors=(), runs=()):
        """Keeps whole tensors (by index) and/or raw (chunk, chunk_off, len) runs out of the weight
        decay; returns the same choice as a flat uint8 mask over [C * S] for the oracle."""
        segs = [B.pt_segment(0, 0, s.len, s.chunk_off, s.chunk, s.tensor) for s in self.segs if s.tensor in set(tensors)]
        segs += [B.pt_segment(0, 0, n, off, c, 0) for c, off, n in runs]
        B.pt_ctx_set_no_decay(self.ctx, segs)
        mask = np.zeros(self.C * self.S, dtype=np.uint8)
        for s in segs:
            mask[s.chunk * self.S + s.chunk_off: s.chunk * self.S + s.chunk_off + s.len] = 1
        return mask

    def oracle_packed(self, orc):
        """the source gradients packed by the ORACLE (dense layout), flat over [C * S]: what the oracle is
        fed, so that none of its inputs has passed through the HIP path"""
        src = to_u16(self.grad_src[:self.N]) if self.N else np.zeros(0, np.uint16)
        offs = np.cumsum([0] + self.sizes)
        return orc.pack_dense([src[offs[i]:offs[i + 1]] for i in range(len(self.sizes))], self.S, self.C).reshape(-1)

    # ---- host copies for the oracle
    def host_state(self):
        torch.cuda.synchronize()
        out = dict(g16=to_u16(self.g16).reshape(-1).copy(), p16=to_u16(self.p16).reshape(-1).copy(),
                   w=self.w.cpu().numpy().reshape(-1).copy(), m=self.m.cpu().numpy().reshape(-1).copy(),
                   v=self.v.cpu().numpy().reshape(-1).copy())
        if self.grad_fp32:
            out["g32"] = self.g32.cpu().numpy().reshape(-1).copy()
        return out

    def close(self):
        torch.cuda.synchronize()
        B.pt_pack_plan_destroy(self.plan)
        B.pt_ctx_destroy(self.ctx)
        self.plan = self.ctx = None


def same_bits(a: np.ndarray, b: np.ndarray) -> bool:
    a = np.ascontiguousarray(a); b = np.ascontiguousarray(b)
    return a.dtype == b.dtype and a.shape == b.shape and a.tobytes() == b.tobytes()


def assert_same_bits(got: np.ndarray, want: np.ndarray, label):
    """Bit-for-bit equality with a useful message (count and first mismatches)."""
    if same_bits(got, want):
        return
    assert got.shape == want.shape and got.dtype == want.dtype, (label, got.shape, want.shape)
    u = np.uint16 if got.dtype.itemsize == 2 else np.uint32
    gi, wi = got.reshape(-1).view(u), want.reshape(-1).view(u)
    idx = np.flatnonzero(gi != wi)
    k = idx[:6]
    raise AssertionError(f"{label}: {idx.size} of {gi.size} words differ; first at {k.tolist()} "
                         f"got {[hex(int(x)) for x in gi[k]]} want {[hex(int(x)) for x in wi[k]]}")

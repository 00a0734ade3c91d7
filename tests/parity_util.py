"""Shared plumbing of the GPU parity tests: builds the HIP-side group and the oracle-side inputs from the
same seeded tensors and compares them.  No arithmetic of the method lives here."""
from __future__ import annotations

import sys

import numpy as np
import torch

import oracle as orc
from paper_2404_06709_amd import binding as cq
from paper_2404_06709_amd import runtime as rt
from paper_2404_06709_amd import synth

TOL = {torch.float32: 1e-4, torch.bfloat16: 2e-2}   # max relative error per tensor, as the target states


def say(msg: str) -> None:
    print(msg, flush=True)
    sys.stdout.flush()


def rel_err(got, ref) -> float:
    """max_i |got_i - ref_i| / max_i |ref_i| (infinity-norm relative error of one tensor)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.abs(ref).max()
    return float(np.abs(got - ref).max() / (den if den > 0 else 1.0))


def odims(shape: synth.Shape, max_seq: int, dtype: torch.dtype) -> orc.Dims:
    return orc.Dims(shape.d_model, shape.n_heads, shape.head_dim, shape.d_ffn, max_seq, 10000.0, 1e-6,
                    orc.BF16 if dtype == torch.bfloat16 else orc.F32)


def gdims(shape: synth.Shape, max_seq: int, dtype: torch.dtype) -> cq.cqil_dims:
    return cq.make_dims(shape.d_model, shape.n_heads, shape.head_dim, shape.d_ffn, max_seq, dtype)


GUARD = 4096          # bytes of sentinel on each side of a guarded buffer
SENTINEL = 0xA7


class Guarded:
    """A device buffer of n bytes with sentinel-filled bands before and after it; check() asserts that the
    bands still hold the sentinel (a kernel that writes outside the buffer it was given fails here)."""

    def __init__(self, nbytes: int, device="cuda"):
        self.n = int(nbytes)
        pad = (-self.n) % 256
        self.raw = torch.full((GUARD + self.n + pad + GUARD,), SENTINEL, dtype=torch.uint8, device=device)
        self.body = self.raw[GUARD: GUARD + self.n]

    def view(self, dtype: torch.dtype, shape) -> torch.Tensor:
        return self.body.view(dtype).view(shape)

    def check(self, label: str) -> None:
        lo, hi = self.raw[:GUARD], self.raw[GUARD + self.n:]
        assert bool((lo == SENTINEL).all()) and bool((hi == SENTINEL).all()), f"{label}: wrote outside its buffer"


class Pair:
    """One group on both sides: HIP (rt.Group) and oracle (numpy weights + float64 caches)."""

    def __init__(self, shape: synth.Shape, P: int, dtype: torch.dtype, max_seq: int, b_max: int, seed: int,
                 w_std: float = 0.02, gain_jitter: float = 0.0, gen_device: str = "cpu"):
        self.shape, self.P, self.dtype, self.max_seq, self.b_max = shape, P, dtype, max_seq, b_max
        layers = synth.make_layers(P, shape, dtype, seed, w_std=w_std, gain_jitter=gain_jitter, device=gen_device)
        self.np_layers = [synth.layer_to_numpy(L) for L in layers]
        dev_layers = rt.to_device(layers)
        self.gd = gdims(shape, max_seq, dtype)
        self.od = odims(shape, max_seq, dtype)
        self.group = rt.Group(self.gd, dev_layers, b_max=b_max)
        torch.cuda.synchronize()
        del dev_layers, layers
        self.okc = orc.new_cache(P, b_max, self.od)
        self.ovc = orc.new_cache(P, b_max, self.od)
        self.lens = np.zeros(b_max, dtype=np.int32)

    def fill_cache(self, lens, seed: int, gen_device: str = "cpu") -> None:
        """N(0,1) values rounded to the storage type in slots [0, lens[b]) of every layer and head."""
        gen = synth.generator(seed, gen_device)
        g = self.group
        for b, S in enumerate(lens):
            S = int(S)
            if S == 0:
                continue
            shp = (self.P, self.shape.n_heads, S, self.shape.head_dim)
            kk = synth.normal(shp, 1.0, self.dtype, gen)
            vv = synth.normal(shp, 1.0, self.dtype, gen)
            g.k[:, b, :, :S] = kk.to(g.k.device)
            g.v[:, b, :, :S] = vv.to(g.v.device)
            self.okc[:, b, :, :S] = synth.widen(kk)
            self.ovc[:, b, :, :S] = synth.widen(vv)
        self.set_lens(lens)

    def set_lens(self, lens) -> None:
        self.lens[: len(lens)] = np.asarray(lens, dtype=np.int32)
        self.group.set_kv_len(list(lens) + [0] * (self.b_max - len(lens)))
        self.group.kv.max_kv_len = int(max(lens))

    def hidden(self, B: int, T: int, seed: int, std: float = 1.0) -> torch.Tensor:
        return synth.normal((B, T, self.shape.d_model), std, self.dtype, synth.generator(seed))

    def step(self, x: torch.Tensor, d: int, check: bool = True, label: str = ""):
        """Runs one group step on both sides from the same x (storage dtype, CPU tensor) and compares
        x_out, the attention outputs, the appended K/V slots and the untouched rest of the caches.
        Returns (gpu_out CPU tensor, oracle_out float64)."""
        B, T, _ = x.shape
        g = self.group
        lens = self.lens[:B].copy()
        if check:
            k_before, v_before = g.k.clone(), g.v.clone()
        g.kv.max_kv_len = int(lens.max())       # host-side bound for the sequences of this call
        # x_out and the workspace sit between sentinel bands: nothing may be written outside them
        es = x.element_size()
        gy = Guarded(x.numel() * es)
        gw = Guarded(cq.cqil_workspace_bytes(self.gd, self.P, B, T))
        y = g.forward(x.cuda(), d, advance=True, out=gy.view(x.dtype, x.shape), workspace=gw.body)
        torch.cuda.synchronize()
        gy.check(f"{label}: x_out")
        gw.check(f"{label}: workspace")
        ref, ref_attn, _ = orc.group_forward(self.od, self.np_layers, d, self.okc, self.ovc, lens, synth.widen(x),
                                             debug=True)
        tol = TOL[self.dtype]
        y_cpu = y.cpu()
        if check:
            e_out = rel_err(synth.widen(y_cpu), ref)
            attn = g.attn_out(B, T).cpu().numpy().reshape(self.P, B, T, -1)
            e_attn = rel_err(attn, ref_attn)
            # the feed-forward branch on its own scale: sum_i FFN_i = x_out - x - sum_i a_i on both sides.  The HIP
            # side's x_out carries one rounding to the storage type (half a unit in the last place of x_out),
            # which the bound adds to the tolerance in units of the branch's size.
            xw = synth.widen(x)
            ffn_ref = ref - xw - ref_attn.sum(axis=0)
            ffn_got = synth.widen(y_cpu) - xw - attn.astype(np.float64).sum(axis=0)
            half_ulp = 2.0 ** -9 if self.dtype == torch.bfloat16 else 2.0 ** -24
            ffn_scale = np.abs(ffn_ref).max()
            e_ffn = rel_err(ffn_got, ffn_ref)
            ffn_tol = tol + half_ulp * np.abs(ref).max() / (ffn_scale if ffn_scale > 0 else 1.0)
            kg, vg = g.k.cpu(), g.v.cpu()
            kb, vb = k_before.cpu(), v_before.cpu()
            del k_before, v_before
            e_k = e_v = 0.0
            for b in range(B):
                s0, s1 = int(lens[b]), int(lens[b]) + T
                e_k = max(e_k, rel_err(synth.widen(kg[:, b, :, s0:s1]), self.okc[:, b, :, s0:s1]))
                e_v = max(e_v, rel_err(synth.widen(vg[:, b, :, s0:s1]), self.ovc[:, b, :, s0:s1]))
                kb[:, b, :, s0:s1] = kg[:, b, :, s0:s1]
                vb[:, b, :, s0:s1] = vg[:, b, :, s0:s1]
            # everything outside the appended slots is preserved bit for bit
            assert torch.equal(kb.view(torch.uint8), kg.view(torch.uint8)), f"{label}: K cache disturbed"
            assert torch.equal(vb.view(torch.uint8), vg.view(torch.uint8)), f"{label}: V cache disturbed"
            say(f"  {label} B={B} T={T} d={d} lens={lens.tolist()}: x_out {e_out:.2e} attn {e_attn:.2e} "
                f"ffn {e_ffn:.2e} (bound {ffn_tol:.1e}) k {e_k:.2e} v {e_v:.2e} (tol {tol:.0e})")
            assert e_out <= tol, f"{label}: x_out rel err {e_out}"
            assert e_attn <= tol, f"{label}: attention output rel err {e_attn}"
            assert e_ffn <= ffn_tol, f"{label}: feed-forward branch rel err {e_ffn} (bound {ffn_tol})"
            assert e_k <= tol and e_v <= tol, f"{label}: appended K/V rel err {e_k} {e_v}"
            got_len = g.kv_len.cpu().numpy()[:B]
            assert (got_len == lens + T).all(), f"{label}: kv_len {got_len} vs {lens + T}"
            assert g.kv.max_kv_len == int(lens.max()) + T
        self.lens[:B] = lens + T
        return y_cpu, ref

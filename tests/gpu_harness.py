"""Runs the HIP path (through the C ABI binding) and the CPU oracle on the same seeded inputs and
compares them stage by stage.  Used by the -m gpu parity tests, the smoke check and nothing else."""
from __future__ import annotations

import numpy as np
import torch

from helpers import tol_ok
from oracle import evomoe_oracle as orc
from paper_2112_14397_amd import binding as B
from paper_2112_14397_amd import synth

RTOL = {"f32": 1e-5, "bf16": 2e-2}
BAND = 1e-6     # pairs with |g' - c| below this are excluded from the mask comparison (and counted)


def to_dev(a, dtype=None):
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(dtype) if dtype is not None else t


def np_of(t):
    return t.detach().float().cpu().numpy() if t.dtype in (torch.bfloat16,) else t.detach().cpu().numpy()


def mask_from_bits(bits_i64: np.ndarray, E: int) -> np.ndarray:
    u = bits_i64.astype(np.int64).view(np.uint64)
    return ((u[:, None] >> np.arange(E, dtype=np.uint64)[None, :]) & np.uint64(1)).astype(bool)


class GpuLayer:
    """Device copies of one LayerInputs + the buffers of the layer."""

    def __init__(self, inp: synth.LayerInputs, P_cap=None, backward=True):
        cfg = inp.cfg
        self.cfg = cfg
        dt = B.torch_dtype(cfg.dtype)
        self.shape = B.make_shape(cfg.T, cfg.d, cfg.E, cfg.F, cfg.dtype, cfg.act,
                                  P_cap if P_cap is not None else cfg.T * cfg.E)
        self.ctx = B.Context()
        self.x = to_dev(inp.x, dt)
        self.noise = to_dev(inp.noise)
        self.dy = to_dev(inp.dy, dt)
        self.params = B.LayerParams(Wg=to_dev(inp.Wg), bg=to_dev(inp.bg), W1=to_dev(inp.W1, dt),
                                    b1=to_dev(inp.b1), W2=to_dev(inp.W2, dt), b2=to_dev(inp.b2))
        self.buf = B.LayerBuffers(self.shape, backward=backward)

    def forward(self, tau, c):
        B.layer_forward(self.ctx, self.buf, self.params, self.x, self.noise, float(tau), float(c))
        return B.evomoe_num_pairs(self.ctx, self.buf.num_pairs)

    def backward(self, tau):
        B.layer_backward(self.ctx, self.buf, self.params, self.x, self.dy, float(tau))
        torch.cuda.synchronize()


def compare_forward(gl: GpuLayer, inp: synth.LayerInputs, tau, c, report=None, check_ffn=True):
    """Forward parity of every stage.  Returns (oracle forward, P, number of band pairs, number of
    band pairs the two sides decided differently)."""
    cfg = inp.cfg
    rt = RTOL[cfg.dtype]
    P = gl.forward(tau, c)
    b = gl.buf
    T, E = cfg.T, cfg.E

    ref_gate = orc.dts_gate(inp.x, inp.Wg, inp.bg, inp.noise, tau, c)
    gp = np_of(b.gprime)
    ok, worst = tol_ok(gp, ref_gate.gprime, 1e-5)
    assert ok, f"gprime worst err/bound {worst:.3g}"
    mask = mask_from_bits(np_of(b.mask_bits), E)
    band = np.abs(ref_gate.gprime - np.float64(np.float32(c))) < BAND
    diff = mask != ref_gate.mask
    # a fallback token's arg-max may be near-tied; treat rows that fell back on either side as band rows
    assert not (diff & ~band).any(), f"{int((diff & ~band).sum())} mask mismatches outside the band"
    n_band, n_flip = int(band.sum()), int(diff.sum())
    override = mask if n_flip else None
    fwd = orc.moe_layer_forward(inp.x, inp.Wg, inp.bg, inp.noise, tau, c, inp.W1, inp.b1, inp.W2,
                                inp.b2, cfg.act, mask_override=override) if check_ffn else None
    g = fwd.gate if check_ffn else orc.dts_gate(inp.x, inp.Wg, inp.bg, inp.noise, tau, c, override)
    dp = fwd.disp if check_ffn else orc.dispatch(g.mask, g.G)

    # integers: bit exact
    np.testing.assert_array_equal(np_of(b.counts), g.counts)
    np.testing.assert_array_equal(np_of(b.k), g.k)
    assert P == int(dp.expert_offsets[E]) == int(g.k.sum())
    np.testing.assert_array_equal(np_of(b.expert_offsets), dp.expert_offsets)
    np.testing.assert_array_equal(np_of(b.pair_token)[:P], dp.pair_token)
    np.testing.assert_array_equal(np_of(b.tok_off), dp.tok_off)
    np.testing.assert_array_equal(np_of(b.tok_rows)[:P], dp.tok_rows)
    gw = np_of(b.gate_w)
    np.testing.assert_array_equal(gw != 0, mask)
    np.testing.assert_array_equal(gw[mask], gp[mask])                      # kept weights are g', not renormalised
    np.testing.assert_array_equal(np_of(b.pair_gate)[:P], gp[dp.pair_token, dp.pair_expert])
    if report is not None:
        report.update(P=P, band=n_band, flipped=n_flip, fallback=g.n_fallback)
    if not check_ffn:
        return None, P, n_band, n_flip

    for name, got, ref in (("H", b.H, fwd.ffn.H), ("A", b.A, fwd.ffn.A), ("O", b.O, fwd.ffn.O)):
        ok, worst = tol_ok(np_of(got)[:P], ref, rt)
        assert ok, f"{name}: worst err/bound {worst:.3g} (rtol {rt})"
    ok, worst = tol_ok(np_of(b.y), fwd.y, rt)
    assert ok, f"y: worst err/bound {worst:.3g} (rtol {rt})"
    if cfg.act == "relu":
        # ReLU'(h) is a 0/1 decision on the sign of h.  Where the oracle's |h| is within float32
        # accumulation error of zero the two sides may decide differently; such elements (counted) take
        # the kernel's decision in the oracle's backward, exactly like near-threshold gate pairs.
        Hg = np_of(b.H)[:P].astype(np.float64)
        flips = (Hg > 0) != (fwd.ffn.H > 0)
        rms = float(np.sqrt(np.mean(fwd.ffn.H ** 2))) if P else 0.0
        assert (np.abs(fwd.ffn.H[flips]) <= 1e-5 * rms).all(), "ReLU sign differs away from zero"
        fwd.ffn.H[flips] = Hg[flips]
        if report is not None:
            report["relu_sign_flips"] = int(flips.sum())
    return fwd, P, n_band, n_flip


def compare_backward(gl: GpuLayer, inp: synth.LayerInputs, fwd: orc.LayerFwd, tau):
    cfg = inp.cfg
    rt = RTOL[cfg.dtype]
    gl.backward(tau)
    b = gl.buf
    P = int(fwd.disp.expert_offsets[cfg.E])
    ref = orc.moe_layer_backward(fwd, inp.dy, inp.x, inp.Wg, tau, inp.W1, inp.W2, cfg.act)
    checks = (("dO", np_of(b.dO)[:P], ref.dO), ("dG_pairs", np_of(b.dG_pairs)[:P], ref.dG_pairs),
              ("dXp", np_of(b.dXp)[:P], ref.ffn.dXp),
              ("dW1", np_of(b.dW1), ref.ffn.dW1), ("db1", np_of(b.db1), ref.ffn.db1),
              ("dW2", np_of(b.dW2), ref.ffn.dW2), ("db2", np_of(b.db2), ref.ffn.db2),
              ("dWg", np_of(b.dWg), ref.dWg), ("dbg", np_of(b.dbg), ref.dbg), ("dx", np_of(b.dx), ref.dx))
    worsts = {}
    for name, got, want in checks:
        ok, worst = tol_ok(got, want, rt)
        worsts[name] = worst
        assert ok, f"{name}: worst err/bound {worst:.3g} (rtol {rt})"
    return ref, worsts

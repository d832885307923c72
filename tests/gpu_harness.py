"""Runs the HIP path (through the C ABI binding) and the CPU oracle on the same seeded inputs and
compares them stage by stage.  Used by the -m gpu parity tests, the smoke check and nothing else."""
from __future__ import annotations

import numpy as np
import torch

from helpers import tol_ok, tol_stats
from oracle import evomoe_oracle as orc
from paper_2112_14397_amd import binding as B
import synth_inputs as synth

RTOL = {"f32": 1e-5, "bf16": 2e-2}
# Every output of a bf16 layer is held to the plain tolerance end to end, with one measured exception, for
# whole-layer comparisons of millions of elements only: dx.  Its gate share, W_g dz with dz ~ (g'/tau) dG and
# dG = <dy, O>, carries the bf16 rounding of the stored activations A (which the matrix cores consume as bf16,
# so it cannot be avoided) and of O, multiplied by 1/tau; rounding those two values alone in the float64 oracle
# puts the worst of config 2's 6.3 million dx elements at 1.2x the bound at tau = 0.3.  DX_TAIL bounds that tail:
# no element above DX_TAIL[0] x the bound and at most DX_TAIL[1] elements above 1x; per stage (the oracle's last
# stages fed with the dG and dXp the kernels produced) dx is held to 1x like everything else.
DX_TAIL = (1.35, 32)
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

    def __init__(self, inp: synth.LayerInputs, P_cap=None, backward=True, recompute=False):
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
        self.buf = B.LayerBuffers(self.shape, backward=backward, recompute=recompute)
        self.recompute = recompute

    def forward(self, tau, c, top1=False):
        B.layer_forward(self.ctx, self.buf, self.params, self.x, self.noise, float(tau), float(c), top1=top1)
        return B.evomoe_num_pairs(self.ctx, self.buf.num_pairs)

    def backward(self, tau, balance_alpha=None):
        B.layer_backward(self.ctx, self.buf, self.params, self.x, self.dy, float(tau),
                         balance_alpha=balance_alpha, recompute=self.recompute)
        torch.cuda.synchronize()


def compare_forward(gl: GpuLayer, inp: synth.LayerInputs, tau, c, report=None, check_ffn=True, top1=False):
    """Forward parity of every stage.  Returns (oracle forward, P, number of band pairs, number of
    band pairs the two sides decided differently).  top1: Algorithm 2's Top-1 branch instead of the
    threshold branch (c is ignored); the decision band is then a token whose two largest g' are within BAND."""
    cfg = inp.cfg
    rt = RTOL[cfg.dtype]
    P = gl.forward(tau, c, top1=top1)
    b = gl.buf
    T, E = cfg.T, cfg.E

    ref_gate = orc.top1_gate(inp.x, inp.Wg, inp.bg, inp.noise, tau) if top1 else \
        orc.dts_gate(inp.x, inp.Wg, inp.bg, inp.noise, tau, c)
    gp = np_of(b.gprime)
    ok, worst = tol_ok(gp, ref_gate.gprime, 1e-5)
    assert ok, f"gprime worst err/bound {worst:.3g}"
    mask = mask_from_bits(np_of(b.mask_bits), E)
    if top1:
        top2 = np.sort(ref_gate.gprime, axis=1)[:, -2:] if E > 1 else np.zeros((T, 2))
        near_tie = (top2[:, 1] - top2[:, 0]) < BAND if E > 1 else np.zeros(T, bool)
        band = np.repeat(near_tie[:, None], E, axis=1)
        assert (mask.sum(axis=1) == 1).all() and P == T, "Top-1: exactly one expert per token"
    else:
        band = np.abs(ref_gate.gprime - np.float64(np.float32(c))) < BAND
    diff = mask != ref_gate.mask
    # a fallback token's arg-max may be near-tied; treat rows that fell back on either side as band rows
    assert not (diff & ~band).any(), f"{int((diff & ~band).sum())} mask mismatches outside the band"
    n_band, n_flip = int(band.sum()), int(diff.sum())
    override = mask if (n_flip or top1) else None
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


def compare_backward(gl: GpuLayer, inp: synth.LayerInputs, fwd: orc.LayerFwd, tau, dx_tail=None, balance_alpha=None,
                     stats=None):
    """Every backward output against the oracle at the plain tolerance.  dx_tail = (factor, count), whole
    full-size layers only: dx may have up to `count` elements above the bound, none above factor x the bound.
    stats (a dict), if given, receives per output (worst, elements above 1x) for the per-row and the per-tensor
    form of the bound."""
    cfg = inp.cfg
    rt = RTOL[cfg.dtype]
    gl.backward(tau, balance_alpha=balance_alpha)
    b = gl.buf
    P = int(fwd.disp.expert_offsets[cfg.E])
    ref = orc.moe_layer_backward(fwd, inp.dy, inp.x, inp.Wg, tau, inp.W1, inp.W2, cfg.act)
    if balance_alpha is not None:
        # L = L_task + L_balance (Training Objective, second stage): the balance loss and its gradient
        loss_ref = orc.balance_loss(fwd.gate, balance_alpha)
        coef_ref = orc.balance_loss_grad(fwd.gate, balance_alpha)
        assert abs(float(np_of(b.bal_loss)[0]) - loss_ref) <= 1e-5 * abs(loss_ref), "balance loss"
        ok, worst = tol_ok(np_of(b.bal_coef)[None, :], coef_ref[None, :], 1e-5)
        assert ok, f"balance-loss gradient coefficients: worst err/bound {worst:.3g}"
        dp = fwd.disp
        ref.dz, ref.dWg, ref.dbg, dx_g = orc.dts_gate_bwd(ref.dG_pairs, dp.pair_token, dp.pair_expert,
                                                          fwd.gate.gprime, tau, inp.x, inp.Wg, dgprime_coef=coef_ref)
        ref.dx = ref.dx_experts + dx_g
    checks = (("dO", np_of(b.dO)[:P], ref.dO), ("dG_pairs", np_of(b.dG_pairs)[:P], ref.dG_pairs),
              ("dXp", np_of(b.dXp)[:P], ref.ffn.dXp),
              ("dW1", np_of(b.dW1), ref.ffn.dW1), ("db1", np_of(b.db1), ref.ffn.db1),
              ("dW2", np_of(b.dW2), ref.ffn.dW2), ("db2", np_of(b.db2), ref.ffn.db2),
              ("dWg", np_of(b.dWg), ref.dWg), ("dbg", np_of(b.dbg), ref.dbg), ("dx", np_of(b.dx), ref.dx))
    worsts = {}
    for name, got, want in checks:
        worst, above = tol_stats(got, want, rt)
        worsts[name] = worst
        if stats is not None:
            stats[name] = {"row": (round(worst, 3), above), "tensor": tuple(
                round(v, 3) if isinstance(v, float) else v for v in tol_stats(got, want, rt, per_tensor=True))}
        if name == "dx" and dx_tail is not None:
            assert worst <= dx_tail[0] and above <= dx_tail[1], \
                f"dx: worst err/bound {worst:.3g}, {above} elements above the bound (allowed {dx_tail})"
        else:
            assert above == 0, f"{name}: worst err/bound {worst:.3g}, {above} elements above it (rtol {rt})"
    return ref, worsts


def compare_backward_stages(gl: GpuLayer, inp: synth.LayerInputs, fwd: orc.LayerFwd, tau):
    """Every backward stage on its own, at the plain tolerance: the oracle's stage fed with what the kernels'
    stage consumed (the stored H, O, dO, dG, dXp, widened to float64) against what the kernels' stage
    produced.  This separates a stage's own error from what it inherits through bf16-stored intermediates."""
    cfg = inp.cfg
    rt = RTOL[cfg.dtype]
    b = gl.buf
    dp = fwd.disp
    P = int(dp.expert_offsets[cfg.E])
    f64 = lambda t: np_of(t)[:P].astype(np.float64)
    Hg, Og, dOg, dGg, dXpg = f64(b.H), f64(b.O), f64(b.dO), f64(b.dG_pairs), f64(b.dXp)
    worsts = {}

    def chk(name, got, want):
        ok, worst = tol_ok(got, want, rt)
        worsts[name] = worst
        assert ok, f"{name} (stage): worst err/bound {worst:.3g} (rtol {rt})"

    # combine backward from the stored O
    dO_s, dG_s = orc.combine_bwd(inp.dy, Og, dp.pair_gate, dp.pair_token)
    chk("dO", np_of(b.dO)[:P], dO_s)
    chk("dG_pairs", np_of(b.dG_pairs)[:P], dG_s)
    # expert FFN backward from the stored H: the dH chain takes dO = G dy as the kernels do (unrounded product),
    # the dW2 / db2 sums take the stored dO
    ffn_exact = orc.expert_ffn_bwd(dO_s, Hg, inp.x, dp.pair_token, dp.expert_offsets, inp.W1, inp.W2, cfg.act)
    chk("dXp", np_of(b.dXp)[:P], ffn_exact.dXp)
    chk("dW1", np_of(b.dW1), ffn_exact.dW1)
    chk("db1", np_of(b.db1), ffn_exact.db1)
    if cfg.dtype == "bf16":
        ffn_stored = orc.expert_ffn_bwd(dOg, Hg, inp.x, dp.pair_token, dp.expert_offsets, inp.W1, inp.W2, cfg.act)
    else:
        ffn_stored = ffn_exact
    chk("dW2", np_of(b.dW2), ffn_stored.dW2)
    chk("db2", np_of(b.db2), ffn_stored.db2)
    # dispatch and gate backward from the stored dXp and dG
    _, dWg, dbg, dx_g = orc.dts_gate_bwd(dGg, dp.pair_token, dp.pair_expert, fwd.gate.gprime, tau, inp.x, inp.Wg)
    dx_e = orc.dispatch_bwd(dXpg, dp.tok_off, dp.tok_rows, cfg.T)
    chk("dx", np_of(b.dx), dx_e + dx_g)
    chk("dWg", np_of(b.dWg), dWg)
    chk("dbg", np_of(b.dbg)[None, :], dbg[None, :])
    return worsts


# ---------------------------------------------------------------------------------------------------
# Full-size cases.  The oracle cannot run a whole full-size layer in seconds, so it is run on what it can
# compute one by one: (a) the gate and the dispatch of every token (cheap); (b) the whole layer, forward
# and backward, of a sample of tokens (every per-token and per-pair quantity of the layer depends on that
# token alone); (c) for chosen experts, all rows of the expert, which gives its complete weight and bias
# gradients; (d) the gate's parameter gradients, which sum over every token, from the dG the kernels
# produced (each sampled token's dG is itself checked in (b)), plus the zero-sum property of the softmax.
# ---------------------------------------------------------------------------------------------------

def _sub_layer(inp, cfg, tokens, tau, c, mask_rows, dy=True):
    """Oracle forward (+ backward) of the layer restricted to `tokens`, with the given selection mask."""
    fwd = orc.moe_layer_forward(inp.x[tokens], inp.Wg, inp.bg, inp.noise[tokens], tau, c, inp.W1, inp.b1,
                                inp.W2, inp.b2, cfg.act, mask_override=mask_rows)
    return fwd


def _relu_patch(cfg, fwd, H_gpu_rows, report, key):
    """ReLU'(h) is a 0/1 decision on the sign of h: where the oracle's |h| is within float32 accumulation
    error of zero, the oracle's backward takes the kernel's decision (counted), as for near-threshold pairs."""
    if cfg.act != "relu" or fwd.ffn.H.size == 0:
        return
    Hg = H_gpu_rows.astype(np.float64)
    flips = (Hg > 0) != (fwd.ffn.H > 0)
    rms = float(np.sqrt(np.mean(fwd.ffn.H ** 2)))
    assert (np.abs(fwd.ffn.H[flips]) <= 1e-5 * rms).all(), "ReLU sign differs away from zero"
    fwd.ffn.H[flips] = Hg[flips]
    report[key] = report.get(key, 0) + int(flips.sum())


def compare_full_size_sampled(gl: GpuLayer, inp: synth.LayerInputs, tau, c, n_tokens=192, experts=None,
                              seed=0, report=None, top1=False):
    cfg = inp.cfg
    rt = RTOL[cfg.dtype]
    report = {} if report is None else report
    T, E = cfg.T, cfg.E
    P = gl.forward(tau, c, top1=top1)
    gl.backward(tau)
    b = gl.buf

    # (a) gate and dispatch of every token
    ref_gate = orc.top1_gate(inp.x, inp.Wg, inp.bg, inp.noise, tau) if top1 else \
        orc.dts_gate(inp.x, inp.Wg, inp.bg, inp.noise, tau, c)
    gp = np_of(b.gprime)
    ok, worst = tol_ok(gp, ref_gate.gprime, 1e-5)
    assert ok, f"gprime worst err/bound {worst:.3g}"
    mask = mask_from_bits(np_of(b.mask_bits), E)
    if top1:
        top2 = np.sort(ref_gate.gprime, axis=1)[:, -2:]
        band = np.repeat(((top2[:, 1] - top2[:, 0]) < BAND)[:, None], E, axis=1)
        assert (mask.sum(axis=1) == 1).all() and P == T
    else:
        band = np.abs(ref_gate.gprime - np.float64(np.float32(c))) < BAND
    diff = mask != ref_gate.mask
    assert not (diff & ~band).any(), f"{int((diff & ~band).sum())} mask mismatches outside the band"
    g = orc.dts_gate(inp.x, inp.Wg, inp.bg, inp.noise, tau, c, mask if (diff.any() or top1) else None)
    dp = orc.dispatch(g.mask, g.G)
    np.testing.assert_array_equal(np_of(b.counts), g.counts)
    np.testing.assert_array_equal(np_of(b.k), g.k)
    assert P == int(dp.expert_offsets[E]) == int(g.k.sum())
    offs = np_of(b.expert_offsets)
    np.testing.assert_array_equal(offs, dp.expert_offsets)
    ptok = np_of(b.pair_token)[:P]
    np.testing.assert_array_equal(ptok, dp.pair_token)
    toff, trows = np_of(b.tok_off), np_of(b.tok_rows)[:P]
    np.testing.assert_array_equal(toff, dp.tok_off)
    np.testing.assert_array_equal(trows, dp.tok_rows)
    np.testing.assert_array_equal(np_of(b.pair_gate)[:P], gp[dp.pair_token, dp.pair_expert])
    report.update(P=P, band=int(band.sum()), flipped=int(diff.sum()), fallback=g.n_fallback)

    Hg, Ag, Og = np_of(b.H), np_of(b.A), np_of(b.O)
    dOg, dGg, dXpg = np_of(b.dO), np_of(b.dG_pairs), np_of(b.dXp)
    worsts = {}

    def chk(name, got, want):
        ok, worst = tol_ok(got, want, rt)
        worsts[name] = max(worsts.get(name, 0.0), worst)
        assert ok, f"{name}: worst err/bound {worst:.3g} (rtol {rt})"

    # (b) a sample of tokens through the whole layer: first, last, and a seeded draw; tokens that fell back
    # to their arg-max expert and the tokens with the most experts are always included when there are any
    rng = np.random.default_rng(seed)
    sample = set(rng.choice(T, size=min(n_tokens, T), replace=False).tolist()) | {0, T - 1}
    sample |= set(np.argsort(-g.k, kind="stable")[:4].tolist())
    no_score = np.nonzero(~(ref_gate.gprime > np.float64(np.float32(c))).any(axis=1))[0]
    sample |= set(no_score[:4].tolist())
    S = np.array(sorted(sample))
    fs = _sub_layer(inp, cfg, S, tau, c, mask[S])
    rows_gpu = np.concatenate([trows[toff[t]:toff[t + 1]] for t in S]) if len(S) else np.zeros(0, np.int64)
    rows_ref = fs.disp.tok_rows          # the sub-layer's rows in the same (token, ascending expert) order
    assert len(rows_gpu) == len(rows_ref)
    chk("H", Hg[rows_gpu], fs.ffn.H[rows_ref])
    chk("A", Ag[rows_gpu], fs.ffn.A[rows_ref])
    chk("O", Og[rows_gpu], fs.ffn.O[rows_ref])
    chk("y", np_of(b.y)[S], fs.y)
    _relu_patch(cfg, fs, Hg[rows_gpu][np.argsort(rows_ref)], report, "relu_sign_flips")
    bs = orc.moe_layer_backward(fs, inp.dy[S], inp.x[S], inp.Wg, tau, inp.W1, inp.W2, cfg.act)
    chk("dO", dOg[rows_gpu], bs.dO[rows_ref])
    chk("dG_pairs", dGg[rows_gpu], bs.dG_pairs[rows_ref])
    chk("dXp", dXpg[rows_gpu], bs.ffn.dXp[rows_ref])
    chk("dx", np_of(b.dx)[S], bs.dx)

    # (c) whole experts: every row of the expert, hence its complete parameter gradients
    if experts is None:
        sizes = np.diff(dp.expert_offsets)
        nonempty = np.nonzero(sizes)[0]
        experts = sorted({int(nonempty[np.argmax(sizes[nonempty])]), int(nonempty[np.argmin(sizes[nonempty])]),
                          int(nonempty[-1])})
    dW1g, db1g, dW2g, db2g = np_of(b.dW1), np_of(b.db1), np_of(b.dW2), np_of(b.db2)
    for e in experts:
        r0, r1 = int(offs[e]), int(offs[e + 1])
        toks = ptok[r0:r1]
        only_e = np.zeros((len(toks), E), bool)
        only_e[:, e] = True
        fe = _sub_layer(inp, cfg, toks, tau, c, only_e)
        assert fe.disp.expert_offsets[e + 1] - fe.disp.expert_offsets[e] == r1 - r0
        chk("H", Hg[r0:r1], fe.ffn.H)
        chk("A", Ag[r0:r1], fe.ffn.A)
        chk("O", Og[r0:r1], fe.ffn.O)
        _relu_patch(cfg, fe, Hg[r0:r1], report, "relu_sign_flips")
        be = orc.moe_layer_backward(fe, inp.dy[toks], inp.x[toks], inp.Wg, tau, inp.W1, inp.W2, cfg.act)
        chk("dXp", dXpg[r0:r1], be.ffn.dXp)
        chk("dW1", dW1g[e], be.ffn.dW1[e])
        chk("db1", db1g[e][None, :], be.ffn.db1[e][None, :])
        chk("dW2", dW2g[e], be.ffn.dW2[e])
        chk("db2", db2g[e][None, :], be.ffn.db2[e][None, :])
    # an expert with no rows has zero gradients
    for e in np.nonzero(np.diff(dp.expert_offsets) == 0)[0]:
        assert not dW1g[e].any() and not dW2g[e].any() and not db1g[e].any() and not db2g[e].any()

    # (d) the gate's parameter gradients from the kernels' own dG, and the softmax zero-sum property
    _, dWg_ref, dbg_ref, _ = orc.dts_gate_bwd(dGg[:P].astype(np.float64), dp.pair_token, dp.pair_expert,
                                               g.gprime, tau, inp.x, inp.Wg)
    chk("dWg", np_of(b.dWg), dWg_ref)
    chk("dbg", np_of(b.dbg)[None, :], dbg_ref[None, :])
    dbg = np_of(b.dbg).astype(np.float64)
    assert abs(dbg.sum()) <= 1e-4 * (np.abs(dbg).sum() + 1e-30), "softmax backward: sum_e dbg must vanish"
    report["experts"] = list(experts)
    report["sampled_tokens"] = int(len(S))
    return worsts

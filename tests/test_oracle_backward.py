"""Pins for the CPU oracle's backward pass (no GPU needed).

The paper derives no gradients, so the oracle's backward is pinned by (a)
central finite differences of the oracle's own, separately pinned, forward,
(b) float64 autograd of a differently-formulated layer (every expert applied
to every token with library ops, multiplied by the constant 0/1 selection),
and (c) identities that follow from the softmax.
"""
import numpy as np
import pytest
import torch

from oracle import evomoe_oracle as orc
import synth_inputs as synth


def _case(T=10, d=6, E=4, F=12, act="gelu", seed=11):
    cfg = synth.LayerConfig("t", T=T, d=d, E=E, F=F, act=act, dtype="f32", taus=(1.0,),
                            threshold=0.15, seed=seed, bias_std=0.1)
    inp = synth.make_layer_inputs(cfg)
    inp.Wg = (inp.Wg * 20).astype(np.float32)
    inp.W1 = (inp.W1 * 20).astype(np.float32)
    inp.W2 = (inp.W2 * 20).astype(np.float32)
    inp.bg = (0.05 * np.arange(E)).astype(np.float32)
    return cfg, inp


def _run(inp, tau, c, act, mask=None, **over):
    a = dict(x=inp.x, Wg=inp.Wg, bg=inp.bg, W1=inp.W1, b1=inp.b1, W2=inp.W2, b2=inp.b2)
    a.update(over)
    fwd = orc.moe_layer_forward(a["x"], a["Wg"], a["bg"], inp.noise, tau, c,
                                a["W1"], a["b1"], a["W2"], a["b2"], act, mask_override=mask)
    return fwd


def _torch_dense_layer(inp, tau, mask, act):
    """All experts on all tokens, then weight by (constant mask) * softmax."""
    t = lambda a: torch.tensor(np.asarray(a, np.float64), requires_grad=True)
    x, Wg, bg, W1, b1, W2, b2 = map(t, (inp.x, inp.Wg, inp.bg, inp.W1, inp.b1, inp.W2, inp.b2))
    z = x @ Wg + bg + torch.tensor(inp.noise.astype(np.float64))
    gp = torch.softmax(z / tau, dim=1)
    G = gp * torch.tensor(mask.astype(np.float64))
    h = torch.einsum("sd,efd->sef", x, W1) + b1[None]
    a = torch.nn.functional.gelu(h) if act == "gelu" else torch.relu(h)
    o = torch.einsum("sef,edf->sed", a, W2) + b2[None]
    y = (G[:, :, None] * o).sum(1)
    return y, dict(x=x, Wg=Wg, bg=bg, W1=W1, b1=b1, W2=W2, b2=b2)


@pytest.mark.parametrize("act,tau,c", [("gelu", 1.0, 0.15), ("relu", 0.5, 0.1), ("gelu", 2.0, 0.0)])
def test_backward_matches_autograd_of_dense_formulation(act, tau, c):
    cfg, inp = _case(act=act)
    fwd = _run(inp, tau, c, act)
    assert np.abs(fwd.gate.gprime - c).min() > 1e-4          # selection locally constant
    bwd = orc.moe_layer_backward(fwd, inp.dy, inp.x, inp.Wg, tau, inp.W1, inp.W2, act)
    y, leaves = _torch_dense_layer(inp, tau, fwd.gate.mask, act)
    np.testing.assert_allclose(fwd.y, y.detach().numpy(), rtol=1e-11, atol=1e-13)
    y.backward(torch.tensor(inp.dy.astype(np.float64)))
    g = {k: v.grad.numpy() for k, v in leaves.items()}
    kw = dict(rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(bwd.dx, g["x"], **kw)
    np.testing.assert_allclose(bwd.dWg, g["Wg"], **kw)
    np.testing.assert_allclose(bwd.dbg, g["bg"], **kw)
    np.testing.assert_allclose(bwd.ffn.dW1, g["W1"], **kw)
    np.testing.assert_allclose(bwd.ffn.db1, g["b1"], **kw)
    np.testing.assert_allclose(bwd.ffn.dW2, g["W2"], **kw)
    np.testing.assert_allclose(bwd.ffn.db2, g["b2"], **kw)
    if c > 0:
        assert (~fwd.gate.mask).any()
        # experts that received no token get exactly zero weight gradient; unselected
        # columns of W_g still receive gradient through the softmax normaliser
        assert np.abs(bwd.dWg).min() > 0


def test_backward_matches_central_finite_differences():
    act, tau, c = "gelu", 0.8, 0.15
    cfg, inp = _case(T=6, d=5, E=3, F=7, act=act, seed=5)
    fwd = _run(inp, tau, c, act)
    mask = fwd.gate.mask
    assert np.abs(fwd.gate.gprime - c).min() > 1e-3
    bwd = orc.moe_layer_backward(fwd, inp.dy, inp.x, inp.Wg, tau, inp.W1, inp.W2, act)
    dy = inp.dy.astype(np.float64)
    L = lambda **o: float((_run(inp, tau, c, act, mask=mask, **o).y * dy).sum())
    grads = dict(x=bwd.dx, Wg=bwd.dWg, bg=bwd.dbg, W1=bwd.ffn.dW1, b1=bwd.ffn.db1,
                 W2=bwd.ffn.dW2, b2=bwd.ffn.db2)
    rng = np.random.default_rng(0)
    eps = 1e-6
    for name, g in grads.items():
        base = np.asarray(getattr(inp, name), np.float64)
        for _ in range(6):
            idx = tuple(rng.integers(0, n) for n in base.shape)
            p = base.copy(); p[idx] += eps
            m = base.copy(); m[idx] -= eps
            fd = (L(**{name: p}) - L(**{name: m})) / (2 * eps)
            assert abs(fd - g[idx]) <= 1e-6 * (abs(g[idx]) + np.abs(g).max()), (name, idx, fd, g[idx])


def test_softmax_backward_identities():
    act, tau, c = "relu", 0.7, 0.12
    cfg, inp = _case(T=14, act=act)
    fwd = _run(inp, tau, c, act)
    bwd = orc.moe_layer_backward(fwd, inp.dy, inp.x, inp.Wg, tau, inp.W1, inp.W2, act)
    np.testing.assert_allclose(bwd.dz.sum(axis=1), 0.0, atol=1e-14)     # shift invariance of softmax
    np.testing.assert_allclose(bwd.dbg.sum(), 0.0, atol=1e-13)
    # dz scales as 1/tau for fixed g' and dG
    dp = fwd.disp
    dz2, *_ = orc.dts_gate_bwd(bwd.dG_pairs, dp.pair_token, dp.pair_expert, fwd.gate.gprime, 2 * tau, inp.x, inp.Wg)
    np.testing.assert_allclose(dz2, bwd.dz / 2, rtol=1e-13)
    # pieces add up: dx = expert path + gate path
    np.testing.assert_allclose(bwd.dx - bwd.dx_experts, bwd.dz @ inp.Wg.astype(np.float64).T, rtol=1e-12, atol=1e-15)


def test_combine_bwd_against_scalar_loops():
    cfg, inp = _case(T=7, d=4, E=3, F=5, act="relu")
    fwd = _run(inp, 1.0, 0.2, "relu")
    dp = fwd.disp
    dO, dG = orc.combine_bwd(inp.dy, fwd.ffn.O, dp.pair_gate, dp.pair_token)
    for r in range(len(dp.pair_token)):
        s = dp.pair_token[r]
        for j in range(cfg.d):
            assert abs(dO[r, j] - dp.pair_gate[r] * float(inp.dy[s, j])) < 1e-15
        assert abs(dG[r] - sum(float(inp.dy[s, j]) * fwd.ffn.O[r, j] for j in range(cfg.d))) < 1e-13


def test_unrouted_expert_gets_zero_weight_gradient():
    cfg, inp = _case(T=8, E=4, act="gelu")
    mask = np.zeros((cfg.T, cfg.E), bool)
    mask[:, 0] = True
    mask[::2, 2] = True
    fwd = _run(inp, 1.0, 0.1, "gelu", mask=mask)
    bwd = orc.moe_layer_backward(fwd, inp.dy, inp.x, inp.Wg, 1.0, inp.W1, inp.W2, "gelu")
    for i in (1, 3):
        assert not bwd.ffn.dW1[i].any() and not bwd.ffn.dW2[i].any()
        assert not bwd.ffn.db1[i].any() and not bwd.ffn.db2[i].any()
    assert bwd.ffn.dW1[0].any() and bwd.ffn.dW2[2].any()


# ---------------------------------------------------------------------------------------------
# Balance loss (Eq. balance_loss), its gradient, and the training-phase schedule
# ---------------------------------------------------------------------------------------------

def test_balance_loss_closed_forms():
    """Uniform routing: every token selects every expert and g' = 1/N -> L = alpha*N*sum_i (T/T^2)(T/N) = alpha*N.
    One-hot routing to a single expert with g' = one-hot -> count = (T,0,..), sum g' = (T,0,..) -> L = alpha*N."""
    T, E, alpha = 12, 4, 0.1
    gp = np.full((T, E), 1.0 / E)
    g = orc.GateOut(gp, gp.copy(), np.ones((T, E), bool), np.full(E, T), np.full(T, E), 0)
    assert orc.balance_loss(g, alpha) == pytest.approx(alpha * E)
    oh = np.zeros((T, E)); oh[:, 2] = 1.0
    g = orc.GateOut(oh, oh.copy(), oh.astype(bool), np.array([0, 0, T, 0]), np.ones(T, int), 0)
    assert orc.balance_loss(g, alpha) == pytest.approx(alpha * E)
    # perfectly balanced top-1 routing with uniform probabilities is the minimum alpha (Switch-style loss)
    m = np.zeros((T, E), bool); m[np.arange(T), np.arange(T) % E] = True
    g = orc.GateOut(gp, np.where(m, gp, 0), m, np.full(E, T // E), np.ones(T, int), 0)
    assert orc.balance_loss(g, alpha) == pytest.approx(alpha)
    np.testing.assert_allclose(orc.balance_loss_grad(g, alpha), alpha * E * (T // E) / T ** 2)


def test_balance_loss_gradient_matches_finite_differences_and_autograd():
    cfg, inp = _case(T=9, d=5, E=4)
    tau, c, alpha = 0.8, 0.15, 0.1
    gate = orc.dts_gate(inp.x, inp.Wg, inp.bg, inp.noise, tau, c)
    dp = orc.dispatch(gate.mask, gate.G)
    coef = orc.balance_loss_grad(gate, alpha)
    zero = np.zeros(len(dp.pair_token))
    dz, dWg, dbg, dx_g = orc.dts_gate_bwd(zero, dp.pair_token, dp.pair_expert, gate.gprime, tau, inp.x, inp.Wg,
                                          dgprime_coef=coef)

    def loss(Wg=inp.Wg, bg=inp.bg, x=inp.x):
        g = orc.dts_gate(x, Wg, bg, inp.noise, tau, c, mask_override=gate.mask)     # counts held constant
        return orc.balance_loss(g, alpha)

    h = 1e-6
    for (i, j) in ((0, 0), (3, 2), (4, 3)):
        Wp, Wm = inp.Wg.astype(np.float64).copy(), inp.Wg.astype(np.float64).copy()
        Wp[i, j] += h; Wm[i, j] -= h
        assert (loss(Wg=Wp) - loss(Wg=Wm)) / (2 * h) == pytest.approx(dWg[i, j], rel=1e-5, abs=1e-10)
    for j in range(cfg.E):
        bp, bm = inp.bg.astype(np.float64).copy(), inp.bg.astype(np.float64).copy()
        bp[j] += h; bm[j] -= h
        assert (loss(bg=bp) - loss(bg=bm)) / (2 * h) == pytest.approx(dbg[j], rel=1e-5, abs=1e-10)
    xp, xm = inp.x.astype(np.float64).copy(), inp.x.astype(np.float64).copy()
    xp[2, 1] += h; xm[2, 1] -= h
    assert (loss(x=xp) - loss(x=xm)) / (2 * h) == pytest.approx(dx_g[2, 1], rel=1e-5, abs=1e-10)

    # autograd of the same loss written with torch ops
    t = lambda a: torch.tensor(np.asarray(a, np.float64), requires_grad=True)
    x, Wg, bg = t(inp.x), t(inp.Wg), t(inp.bg)
    gp = torch.softmax((x @ Wg + bg + torch.tensor(inp.noise.astype(np.float64))) / tau, dim=1)
    counts = torch.tensor(gate.counts.astype(np.float64))
    L = alpha * cfg.E * (counts / cfg.T ** 2 * gp.sum(dim=0)).sum()
    L.backward()
    assert float(L.detach()) == pytest.approx(orc.balance_loss(gate, alpha))
    np.testing.assert_allclose(dWg, Wg.grad.numpy(), rtol=1e-10, atol=1e-14)
    np.testing.assert_allclose(dbg, bg.grad.numpy(), rtol=1e-10, atol=1e-14)
    np.testing.assert_allclose(dx_g, x.grad.numpy(), rtol=1e-10, atol=1e-14)


def test_dense_coefficient_adds_to_pair_gradients():
    """Linearity: gate backward of (pair gradients + dense coefficients) = sum of the two backward passes."""
    cfg, inp = _case()
    tau, c = 1.0, 0.15
    gate = orc.dts_gate(inp.x, inp.Wg, inp.bg, inp.noise, tau, c)
    dp = orc.dispatch(gate.mask, gate.G)
    rng = np.random.default_rng(5)
    dGp, coef = rng.standard_normal(len(dp.pair_token)), rng.standard_normal(cfg.E)
    a = orc.dts_gate_bwd(dGp, dp.pair_token, dp.pair_expert, gate.gprime, tau, inp.x, inp.Wg)
    b = orc.dts_gate_bwd(0 * dGp, dp.pair_token, dp.pair_expert, gate.gprime, tau, inp.x, inp.Wg, dgprime_coef=coef)
    ab = orc.dts_gate_bwd(dGp, dp.pair_token, dp.pair_expert, gate.gprime, tau, inp.x, inp.Wg, dgprime_coef=coef)
    for u, v, w in zip(a, b, ab):
        np.testing.assert_allclose(u + v, w, rtol=1e-12, atol=1e-14)


def test_schedule_follows_the_papers_step_counts():
    """Experimental Setup: first 5k steps expert-diversify, following 5k steps anneal 2.0 -> 0.3; Top-1 after."""
    T_S, T_D = 5000, 5000
    assert orc.schedule(0, T_S, T_D).stage == 1 and orc.schedule(4999, T_S, T_D).stage == 1
    first, last = orc.schedule(5000, T_S, T_D), orc.schedule(9999, T_S, T_D)
    assert (first.stage, first.top1, first.tau) == (2, False, 2.0)
    assert (last.stage, last.top1) == (2, False) and last.tau == pytest.approx(0.3)
    after = orc.schedule(10000, T_S, T_D)
    assert (after.stage, after.top1) == (2, True) and after.tau == pytest.approx(0.3)
    taus = [orc.schedule(i, T_S, T_D).tau for i in range(5000, 10000)]
    assert all(a > b for a, b in zip(taus, taus[1:]))                       # strictly annealing
    assert np.allclose(np.diff(taus), np.diff(taus)[0])                     # evenly: a linear ramp
    # six evenly spaced temperatures between the paper's end points 2.0 and 0.3 (step 0.34), written out
    assert [round(orc.schedule(i, 0, 6).tau, 6) for i in range(6)] == [2.0, 1.66, 1.32, 0.98, 0.64, 0.3]
    assert orc.schedule(2500 + 5000 - 1, T_S, T_D).tau == pytest.approx(2.0 - 1.7 * 2499 / 4999)   # mid-ramp
    assert orc.schedule(7, 0, 1).top1 and orc.schedule(0, 0, 1).tau == 2.0

"""Pins for the CPU oracle's forward pass (no GPU needed).

Each test checks the oracle against something other than itself: numbers the
paper prints, closed forms, limits the paper states, textbook values, or a
literal scalar brute force of Algorithm 1 / Algorithm 2.
"""
import math
import os

import numpy as np
import pytest

from oracle import evomoe_oracle as orc
import synth_inputs as synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _tiny(T=24, d=8, E=4, F=16, act="gelu", seed=7, bias=0.05):
    cfg = synth.LayerConfig("t", T=T, d=d, E=E, F=F, act=act, dtype="f32", taus=(1.0,),
                            threshold=0.1, seed=seed, bias_std=bias)
    inp = synth.make_layer_inputs(cfg)
    # bigger gate weights so that routing is not dominated by noise alone
    inp.Wg = (inp.Wg * 25).astype(np.float32)
    inp.bg = (0.1 * np.arange(E)).astype(np.float32)
    return cfg, inp


# ---- paper's worked example ------------------------------------------------

def _read_golden():
    vals = {}
    for line in open(os.path.join(GOLDEN, "paper_gate_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        vals[k] = [float(t) for t in v]
    return vals


def test_paper_worked_gate_example():
    g = _read_golden()
    x = np.array([g["x_s"]])
    logits = np.array(g["logits"])
    dec = int(g["decimals"][0])
    # Build a W_g (D x N, N = 2 kept experts) whose product with the paper's x_s is the paper's
    # two kept similarities; minimum-norm solution of x W = logits.
    W = np.outer(x[0], logits[:2]) / float(x[0] @ x[0])
    np.testing.assert_allclose(x @ W, logits[None, :2], atol=1e-12)
    out = orc.dts_gate(x, W, None, None, tau=1.0, threshold=0.0)
    assert np.all(np.round(out.gprime[0], dec) == np.array(g["gate"][:2]))
    # ... and the paper's combination y = 0.35 e0(x) + 0.65 e1(x), with e2 dropped
    rng = np.random.default_rng(0)
    W1 = rng.standard_normal((2, 5, 3)); W2 = rng.standard_normal((2, 3, 5))
    b1 = rng.standard_normal((2, 5)); b2 = rng.standard_normal((2, 3))
    fwd = orc.moe_layer_forward(x, W, None, None, 1.0, 0.0, W1, b1, W2, b2, "relu")
    e = [W2[i] @ np.maximum(W1[i] @ x[0] + b1[i], 0) + b2[i] for i in range(2)]
    w = out.gprime[0]
    np.testing.assert_allclose(fwd.y[0], w[0] * e[0] + w[1] * e[1], rtol=1e-13)
    assert abs(w[0] - 0.35) < 5e-3 and abs(w[1] - 0.65) < 5e-3


def test_paper_example_three_experts_threshold_drops_nothing_but_weights_match_softmax():
    # The same three similarities through the DTS gate (softmax BEFORE selection): library softmax.
    g = _read_golden()
    z = np.array([g["logits"]])
    from scipy.special import softmax
    for tau in (2.0, 1.0, 0.3):
        np.testing.assert_allclose(orc.temperature_softmax(z, tau), softmax(z / tau, axis=1), rtol=1e-14)


# ---- closed forms and limits -------------------------------------------------

def test_two_expert_sigmoid_closed_form():
    rng = np.random.default_rng(1)
    z = rng.standard_normal((50, 2)) * 3
    for tau in (0.3, 1.0, 2.0):
        gp = orc.temperature_softmax(z, tau)
        s = 1.0 / (1.0 + np.exp(-(z[:, 0] - z[:, 1]) / tau))
        np.testing.assert_allclose(gp[:, 0], s, rtol=1e-13)
        np.testing.assert_allclose(gp[:, 1], 1 - s, rtol=1e-12, atol=1e-15)


def test_softmax_rows_sum_to_one_and_shift_invariant():
    rng = np.random.default_rng(2)
    z = rng.standard_normal((40, 7)) * 5
    gp = orc.temperature_softmax(z, 0.7)
    np.testing.assert_allclose(gp.sum(1), 1.0, rtol=1e-14)
    np.testing.assert_allclose(orc.temperature_softmax(z + 123.456, 0.7), gp, rtol=1e-11)


def test_logits_use_Wg_as_D_by_N_and_add_bias_and_noise():
    # scalar loops: z_si = sum_k x_sk Wg_ki + bg_i + zeta_si
    cfg, inp = _tiny()
    z = orc.gate_logits(inp.x, inp.Wg, inp.bg, inp.noise)
    for s in (0, 5, 23):
        for i in range(cfg.E):
            ref = sum(float(inp.x[s, k]) * float(inp.Wg[k, i]) for k in range(cfg.d))
            ref += float(inp.bg[i]) + float(inp.noise[s, i])
            assert abs(z[s, i] - ref) < 1e-12


def test_noise_is_added_before_division_by_tau():
    z = np.array([[0.3, -0.2, 0.1]])
    noise = np.array([[1.0, 0.0, -1.0]])
    x = np.eye(3)[:1] * 0 + np.array([[1.0, 0, 0]])
    Wg = np.zeros((3, 3)); Wg[0] = z[0]
    tau = 0.5
    gp = orc.dts_gate(x, Wg, None, noise, tau, 0.0).gprime
    a = (z + noise) / tau
    ref = np.exp(a) / np.exp(a).sum()
    np.testing.assert_allclose(gp, ref, rtol=1e-13)


def test_dense_limit_routes_every_token_to_every_expert():
    cfg, inp = _tiny(T=32, E=4)
    out = orc.dts_gate(inp.x, inp.Wg, inp.bg, inp.noise, tau=1e7, threshold=0.0)
    assert out.mask.all()
    assert (out.counts == cfg.T).all() and (out.k == cfg.E).all()
    np.testing.assert_allclose(out.gprime, 1.0 / cfg.E, rtol=1e-5)
    np.testing.assert_allclose(out.G.sum(1), 1.0, rtol=1e-13)   # nothing dropped => weights sum to 1


def test_low_temperature_collapses_to_top1():
    cfg, inp = _tiny(T=64, E=4)
    z = orc.gate_logits(inp.x, inp.Wg, inp.bg, inp.noise)
    out = orc.dts_gate(inp.x, inp.Wg, inp.bg, inp.noise, tau=1e-3, threshold=0.1)
    assert (out.k == 1).all()
    assert (out.mask.argmax(1) == z.argmax(1)).all()
    np.testing.assert_allclose(out.G.max(1), 1.0, rtol=1e-9)
    t1 = orc.top1_gate(inp.x, inp.Wg, inp.bg, inp.noise, tau=1.0)
    assert (t1.mask.argmax(1) == z.argmax(1)).all() and (t1.k == 1).all()
    gp = orc.temperature_softmax(z, 1.0)
    np.testing.assert_array_equal(t1.G.max(1), gp.max(1))       # un-renormalised score


def test_threshold_is_strict_kept_scores_are_not_renormalised():
    # E = 4 equal logits -> every score is exactly 0.25
    x = np.ones((3, 2)); Wg = np.zeros((2, 4))
    out = orc.dts_gate(x, Wg, None, None, 1.0, 0.25)   # 0.25 > 0.25 is false -> fallback top-1
    assert out.n_fallback == 3 and (out.k == 1).all() and (out.mask[:, 0]).all()
    np.testing.assert_array_equal(out.G[:, 0], 0.25)
    out = orc.dts_gate(x, Wg, None, None, 1.0, np.nextafter(np.float32(0.25), np.float32(0)))
    assert out.n_fallback == 0 and out.mask.all()
    # kept weights equal g' exactly and sum to the kept mass, not to 1
    cfg, inp = _tiny(T=40)
    out = orc.dts_gate(inp.x, inp.Wg, inp.bg, inp.noise, 1.0, 0.2)
    assert ((out.G > 0) == out.mask).all()
    np.testing.assert_array_equal(out.G[out.mask], out.gprime[out.mask])
    assert (out.gprime[~out.mask] <= 0.2 + 1e-9).all() and (out.gprime[out.mask] > 0.2 - 1e-9).all()
    dropped = np.where(out.mask, 0, out.gprime).sum(1)
    np.testing.assert_allclose(out.G.sum(1), 1 - dropped, rtol=1e-12)
    assert (out.G.sum(1) < 1).any()
    assert ((out.k >= 1) & (out.k <= cfg.E)).all()


def test_pairs_shrink_monotonically_as_temperature_drops():
    for name in ("tiny",):
        cfg = synth.CONFIGS[name]
        inp = synth.make_layer_inputs(cfg)
        P = [int(orc.dts_gate(inp.x, inp.Wg, inp.bg, inp.noise, t, cfg.threshold).k.sum())
             for t in (4.0, 2.0, 1.0, 0.5, 0.3, 0.1)]
        assert all(a >= b for a, b in zip(P, P[1:])), P
        assert P[-1] >= cfg.T


# ---- dispatch -----------------------------------------------------------------

def test_dispatch_against_double_loop_and_invariants():
    cfg, inp = _tiny(T=37, E=5)
    g = orc.dts_gate(inp.x, inp.Wg, inp.bg, inp.noise, 1.0, 0.15)
    dp = orc.dispatch(g.mask, g.G)
    T, E = cfg.T, cfg.E
    # brute force: walk experts, then tokens
    rows = [(s, i) for i in range(E) for s in range(T) if g.mask[s, i]]
    P = len(rows)
    assert dp.expert_offsets[E] == P == g.counts.sum() == g.k.sum()
    assert [tuple(p) for p in zip(dp.pair_token, dp.pair_expert)] == rows
    for i in range(E):
        assert dp.expert_offsets[i] == sum(1 for (_, e) in rows if e < i)
        seg = dp.pair_token[dp.expert_offsets[i]:dp.expert_offsets[i + 1]]
        assert (np.diff(seg) > 0).all()
    for r, (s, i) in enumerate(rows):
        assert dp.pair_gate[r] == g.G[s, i] == g.gprime[s, i]
    # token CSR is the inverse map, experts ascending per token
    for s in range(T):
        mine = dp.tok_rows[dp.tok_off[s]:dp.tok_off[s + 1]]
        assert [rows[r] for r in mine] == [(s, i) for i in range(E) if g.mask[s, i]]
    assert dp.tok_off[T] == P
    assert sorted(dp.tok_rows.tolist()) == list(range(P))


# ---- activation: textbook values ----------------------------------------------

def test_activation_textbook_values():
    Phi1 = 0.8413447460685429     # standard normal CDF at 1
    assert abs(orc.activation(np.array([1.0]), "gelu")[0] - Phi1) < 1e-15
    assert orc.activation(np.array([0.0]), "gelu")[0] == 0.0
    h = np.linspace(-4, 4, 33)
    np.testing.assert_allclose(orc.activation(h, "gelu") - orc.activation(-h, "gelu"), h, atol=1e-15)
    ref = np.array([0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in h])
    np.testing.assert_allclose(orc.activation(h, "gelu"), ref, rtol=1e-14, atol=1e-17)
    assert abs(orc.activation_grad(np.array([0.0]), "gelu")[0] - 0.5) < 1e-16
    # gelu'(1) = Phi(1) + phi(1)
    assert abs(orc.activation_grad(np.array([1.0]), "gelu")[0] - (Phi1 + 0.24197072451914337)) < 1e-15
    np.testing.assert_array_equal(orc.activation(np.array([-1.0, 0.0, 2.0]), "relu"), [0.0, 0.0, 2.0])
    np.testing.assert_array_equal(orc.activation_grad(np.array([-1.0, 0.0, 2.0]), "relu"), [0.0, 0.0, 1.0])
    # derivative vs central difference
    eps = 1e-6
    fd = (orc.activation(h + eps, "gelu") - orc.activation(h - eps, "gelu")) / (2 * eps)
    np.testing.assert_allclose(orc.activation_grad(h, "gelu"), fd, atol=1e-9)


# ---- whole layer: literal Algorithm 1 ------------------------------------------

def _scalar_layer(inp, tau, c, act):
    """Algorithm 1's inner loops with Algorithm 2 inlined, in Python scalars."""
    x, Wg, bg, nz = (np.asarray(a, np.float64) if a is not None else None
                     for a in (inp.x, inp.Wg, inp.bg, inp.noise))
    T, d = x.shape
    E = Wg.shape[1]
    F = inp.W1.shape[1]
    ys, ids = [], []
    for s in range(T):
        z = []
        for i in range(E):
            v = 0.0
            for k in range(d):
                v += x[s, k] * Wg[k, i]
            z.append((v + (bg[i] if bg is not None else 0.0) + nz[s, i]) / tau)
        m = max(z)
        ex = [math.exp(v - m) for v in z]
        tot = sum(ex)
        g = [v / tot for v in ex]
        sel = [i for i in range(E) if g[i] > float(np.float32(c))]
        if not sel:
            sel = [max(range(E), key=lambda i: (g[i], -i))]
        y = [0.0] * d
        for i in sel:
            h = [sum(float(inp.W1[i, f, k]) * x[s, k] for k in range(d)) + float(inp.b1[i, f]) for f in range(F)]
            if act == "relu":
                a = [max(v, 0.0) for v in h]
            else:
                a = [0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in h]
            o = [sum(float(inp.W2[i, j, f]) * a[f] for f in range(F)) + float(inp.b2[i, j]) for j in range(d)]
            for j in range(d):
                y[j] += g[i] * o[j]
        ys.append(y); ids.append(sel)
    return np.array(ys), ids


@pytest.mark.parametrize("act,tau,c", [("gelu", 1.0, 0.2), ("relu", 0.4, 0.1), ("gelu", 8.0, 0.3)])
def test_layer_matches_literal_scalar_loops(act, tau, c):
    cfg, inp = _tiny(T=12, d=6, E=4, F=10, act=act)
    y_ref, ids = _scalar_layer(inp, tau, c, act)
    fwd = orc.moe_layer_forward(inp.x, inp.Wg, inp.bg, inp.noise, tau, c, inp.W1, inp.b1, inp.W2, inp.b2, act)
    assert [np.nonzero(r)[0].tolist() for r in fwd.gate.mask] == ids
    np.testing.assert_allclose(fwd.y, y_ref, rtol=1e-12, atol=1e-14)
    if c == 0.3:
        assert fwd.gate.n_fallback > 0       # this case exercises the len(id_s) >= 1 rule


def test_dense_limit_layer_is_mean_of_plain_ffns():
    cfg, inp = _tiny(T=20, d=8, E=3, F=12, act="gelu")
    fwd = orc.moe_layer_forward(inp.x, inp.Wg, inp.bg, inp.noise, 1e9, 0.0,
                                inp.W1, inp.b1, inp.W2, inp.b2, "gelu")
    from scipy.stats import norm
    x = inp.x.astype(np.float64)
    acc = 0
    for i in range(cfg.E):   # library GEMMs over ALL tokens, no routing at all
        h = x @ inp.W1[i].astype(np.float64).T + inp.b1[i]
        acc = acc + (h * norm.cdf(h)) @ inp.W2[i].astype(np.float64).T + inp.b2[i]
    np.testing.assert_allclose(fwd.y, acc / cfg.E, rtol=1e-7, atol=1e-10)


def test_single_expert_layer_is_plain_ffn_scaled_by_one():
    cfg, inp = _tiny(T=9, d=5, E=1, F=7, act="relu")
    fwd = orc.moe_layer_forward(inp.x, inp.Wg, inp.bg, inp.noise, 1.0, 0.5,
                                inp.W1, inp.b1, inp.W2, inp.b2, "relu")
    x = inp.x.astype(np.float64)
    ref = np.maximum(x @ inp.W1[0].T.astype(np.float64) + inp.b1[0], 0) @ inp.W2[0].T.astype(np.float64) + inp.b2[0]
    np.testing.assert_allclose(fwd.y, ref, rtol=1e-13)
    assert (fwd.gate.G == 1.0).all()


def test_combine_is_linear_in_gate_weights():
    cfg, inp = _tiny(T=16)
    fwd = orc.moe_layer_forward(inp.x, inp.Wg, inp.bg, inp.noise, 1.0, 0.1,
                                inp.W1, inp.b1, inp.W2, inp.b2, "gelu")
    dp = fwd.disp
    y2 = orc.combine(fwd.ffn.O, 2.5 * dp.pair_gate, dp.tok_off, dp.tok_rows, cfg.T)
    np.testing.assert_allclose(y2, 2.5 * fwd.y, rtol=1e-13)


def test_balance_loss_uniform_routing_value():
    # all tokens to all experts with uniform scores: alpha*N*sum_i (T/T^2)*(T/N) = alpha*N
    x = np.ones((10, 2)); Wg = np.zeros((2, 4))
    g = orc.dts_gate(x, Wg, None, None, 1.0, 0.0)
    assert abs(orc.balance_loss(g, alpha=0.1) - 0.1 * 4) < 1e-15


def test_bf16_storage_rounding_helpers():
    import torch
    a = np.random.default_rng(3).standard_normal(4096).astype(np.float32) * 3
    a[:4] = [1.0, 1.00390625, 1.01171875, -0.0]         # ties: round to even
    bits = synth.f32_to_bf16_bits(a)
    ref = torch.from_numpy(a).to(torch.bfloat16)
    np.testing.assert_array_equal(bits.view(np.int16), ref.view(torch.int16).numpy())
    np.testing.assert_array_equal(synth.bf16_bits_to_f32(bits), ref.float().numpy())

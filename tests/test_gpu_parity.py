"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs.

Integers (mask, counts, offsets, indices) must be bit exact, except mask bits of pairs whose oracle score
is within 1e-6 of the threshold (counted and reported); floats must satisfy
|gpu - ref| <= rtol * (|ref| + rms(ref row)) with rtol 1e-5 (float32 layer) or 2e-2 (bf16 layer).
"""
import dataclasses

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import synth_inputs as synth  # noqa: E402


def _harness():
    import gpu_harness
    return gpu_harness


def _mk(name, T, d, E, F, act, dtype, c, seed, bias=0.02, gate_scale=1.0, bg0=0.0):
    cfg = synth.LayerConfig(name, T=T, d=d, E=E, F=F, act=act, dtype=dtype, taus=(1.0,), threshold=c,
                            seed=seed, bias_std=bias, gate_bias_e0=bg0)
    inp = synth.make_layer_inputs(cfg)
    if gate_scale != 1.0:
        inp.Wg = (inp.Wg * gate_scale).astype(np.float32)
    return cfg, inp


# ---- config 1 exactly as specified: tiny fp32 forward, three temperatures --------------------------

@pytest.mark.parametrize("tau", synth.CONFIGS["tiny"].taus)
def test_config1_tiny_fp32_forward(tau):
    h = _harness()
    cfg = synth.CONFIGS["tiny"]
    inp = synth.make_layer_inputs(cfg)
    gl = h.GpuLayer(inp, backward=True)
    rep = {}
    fwd, P, band, flip = h.compare_forward(gl, inp, tau, cfg.threshold, rep)
    print(f"tiny tau={tau}: P={P} band={band} flipped={flip}")
    h.compare_backward(gl, inp, fwd, tau)      # not required by the config; isolates logic from bf16 rounding


# ---- ragged shapes spanning several tiles with tails, both storage types -----------------------------

RAGGED = [
    # name            T    d    E   F    act     dtype  c     seed
    ("f32-ragged",    333, 72,  5,  136, "gelu", "f32", 0.12, 101),
    ("f32-relu",      517, 64,  16, 200, "relu", "f32", 0.04, 102),
    ("bf16-ragged",   777, 136, 7,  264, "gelu", "bf16", 0.10, 103),
    ("bf16-e33",      1030, 128, 33, 320, "relu", "bf16", 0.02, 104),
    ("bf16-e64",      2100, 256, 64, 512, "gelu", "bf16", 0.012, 105),
    ("f32-e64",       600, 64,  64, 128, "gelu", "f32", 0.012, 106),
    ("bf16-e1",       130, 64,  1,  128, "gelu", "bf16", 0.5, 107),
    ("bf16-e24",      900, 192, 24, 256, "gelu", "bf16", 0.03, 108),
]


@pytest.mark.parametrize("case", RAGGED, ids=[c[0] for c in RAGGED])
@pytest.mark.parametrize("tau", [2.0, 0.4])
def test_ragged_forward_backward(case, tau):
    h = _harness()
    name, T, d, E, F, act, dtype, c, seed = case
    # W_g is scaled up so that routing depends on the tokens, not only on the noise.  The bf16 cases
    # stay closer to the configs' N(0, 0.02) gate: the gate's share of dx carries the bf16 rounding of O
    # multiplied by |W_g| / tau, so a much larger gate at low tau would exceed what bf16 storage can give.
    cfg, inp = _mk(name, T, d, E, F, act, dtype, c, seed, gate_scale=8.0 if dtype == "f32" else 2.0)
    gl = h.GpuLayer(inp)
    rep = {}
    fwd, P, band, flip = h.compare_forward(gl, inp, tau, c, rep)
    ref, worsts = h.compare_backward(gl, inp, fwd, tau)
    print(f"{name} tau={tau}: {rep} worst={ {k: round(v, 3) for k, v in worsts.items()} }")


# ---- the limits the paper states -------------------------------------------------------------------

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_dense_limit_all_experts(dtype):
    h = _harness()
    cfg, inp = _mk("dense", 260, 64, 8, 128, "gelu", dtype, 0.0, 201)
    gl = h.GpuLayer(inp)
    fwd, P, band, flip = h.compare_forward(gl, inp, 1e6, 0.0)
    assert P == cfg.T * cfg.E
    assert (h.np_of(gl.buf.counts) == cfg.T).all()
    h.compare_backward(gl, inp, fwd, 1e6)


def test_low_temperature_is_top1():
    h = _harness()
    cfg, inp = _mk("top1", 500, 64, 8, 128, "relu", "bf16", 0.1, 202, gate_scale=10.0)
    gl = h.GpuLayer(inp)
    fwd, P, band, flip = h.compare_forward(gl, inp, 1e-4, 0.1)
    assert P == cfg.T and (h.np_of(gl.buf.k) == 1).all()
    h.compare_backward(gl, inp, fwd, 1e-4)


def test_fallback_keeps_argmax_expert():
    h = _harness()
    # c above 1/E at a high temperature: no score passes, every token falls back to its arg-max
    cfg, inp = _mk("fallback", 300, 64, 8, 128, "gelu", "f32", 0.2, 203, gate_scale=10.0)
    gl = h.GpuLayer(inp)
    rep = {}
    fwd, P, band, flip = h.compare_forward(gl, inp, 50.0, 0.2, rep)
    assert rep["fallback"] == cfg.T and P == cfg.T


def test_expert_with_no_tokens_and_skewed_load():
    h = _harness()
    cfg, inp = _mk("empty", 400, 64, 6, 128, "gelu", "bf16", 0.1, 204, gate_scale=5.0)
    inp.bg = np.array([3.0, 0, -60.0, 0, 0, -60.0], np.float32)       # experts 2 and 5 never selected
    gl = h.GpuLayer(inp)
    fwd, P, band, flip = h.compare_forward(gl, inp, 0.7, 0.1)
    cnt = h.np_of(gl.buf.counts)
    assert cnt[2] == 0 and cnt[5] == 0 and cnt[0] > cnt[1]
    ref, _ = h.compare_backward(gl, inp, fwd, 0.7)
    assert not h.np_of(gl.buf.dW1)[2].any() and not h.np_of(gl.buf.dW2)[5].any()


def test_full_width_layer_with_empty_experts_takes_the_grouped_tile_order():
    """d = 768, F = 3072 as in configs 2 and 3, few tokens: the launches fill the whole persistent grid, GEMM1 and dH
    walk their tiles expert by expert in column groups with one share of the sequence per XCD, and two experts
    have no rows at all (their tile ranges are empty and must be stepped over)."""
    h = _harness()
    cfg, inp = _mk("wide", 1536, 768, 16, 3072, "gelu", "bf16", 0.05, 207, gate_scale=3.0)
    bg = np.zeros(16, np.float32)
    bg[[2, 11]] = -60.0                                             # never selected
    bg[7] = 2.0                                                     # selected by almost every token
    inp.bg = bg
    gl = h.GpuLayer(inp)
    fwd, P, band, flip = h.compare_forward(gl, inp, 1.0, 0.05)
    cnt = h.np_of(gl.buf.counts)
    assert cnt[2] == 0 and cnt[11] == 0 and cnt[7] > 2 * np.median(cnt)
    assert P > 3000                                                 # several row tiles per expert
    h.compare_backward(gl, inp, fwd, 1.0, dx_tail=h.DX_TAIL)
    assert not h.np_of(gl.buf.dW1)[2].any() and not h.np_of(gl.buf.dW2)[11].any()


def test_no_noise_no_bias_pointers():
    h = _harness()
    cfg, inp = _mk("nonoise", 200, 64, 4, 128, "relu", "f32", 0.1, 205, bias=0.0, gate_scale=20.0)
    inp.noise = np.zeros_like(inp.noise)
    gl = h.GpuLayer(inp)
    gl.noise = None
    gl.params.b1 = None
    gl.params.b2 = None
    fwd, *_ = h.compare_forward(gl, inp, 1.0, 0.1)
    h.compare_backward(gl, inp, fwd, 1.0)


# ---- determinism, accumulate flag, x_perm, capacity ---------------------------------------------------

def test_bitwise_reproducible_and_accumulate():
    h = _harness()
    cfg, inp = _mk("repro", 700, 128, 8, 256, "gelu", "bf16", 0.05, 301, gate_scale=6.0)
    gl = h.GpuLayer(inp)
    gl.forward(1.0, 0.05); gl.backward(1.0)
    names = ("gprime", "mask_bits", "counts", "pair_token", "tok_rows", "H", "A", "O", "y",
             "dO", "dG_pairs", "dXp", "dx", "dW1", "dW2", "db1", "db2", "dWg", "dbg")
    first = {n: getattr(gl.buf, n).clone() for n in names}
    gl.forward(1.0, 0.05); gl.backward(1.0)
    for n in names:
        assert torch.equal(first[n].view(torch.uint8), getattr(gl.buf, n).view(torch.uint8)), n
    # accumulate: running backward again with accumulate=1 doubles the weight gradients
    from paper_2112_14397_amd import binding as B
    b = gl.buf
    B.evomoe_expert_ffn_bwd(gl.ctx, gl.shape, b.dO, b.H, b.A, gl.x, b.pair_token, b.expert_offsets,
                            gl.params.W1, gl.params.W2, gl.dy, b.pair_gate, b.dW1, b.db1, b.dW2, b.db2, b.dXp, True,
                            b.workspace)
    torch.cuda.synchronize()
    # against the oracle: twice its gradients, at the layer's tolerance (the running sums are read back and
    # stored in the layer's type, so a second rounding of the same size comes on top of the first)
    fwd = h.orc.moe_layer_forward(inp.x, inp.Wg, inp.bg, inp.noise, 1.0, 0.05, inp.W1, inp.b1, inp.W2, inp.b2,
                                  cfg.act, mask_override=h.mask_from_bits(h.np_of(b.mask_bits), cfg.E))
    ref = h.orc.moe_layer_backward(fwd, inp.dy, inp.x, inp.Wg, 1.0, inp.W1, inp.W2, cfg.act)
    for n, want in (("dW1", ref.ffn.dW1), ("dW2", ref.ffn.dW2), ("db1", ref.ffn.db1), ("db2", ref.ffn.db2)):
        ok, worst = h.tol_ok(h.np_of(getattr(b, n)), 2 * want, h.RTOL["bf16"])
        assert ok, (n, worst)


def test_xperm_gather_and_pregathered_input():
    h = _harness()
    from paper_2112_14397_amd import binding as B
    cfg, inp = _mk("xperm", 300, 64, 4, 128, "gelu", "bf16", 0.1, 302, gate_scale=6.0)
    gl = h.GpuLayer(inp)
    P = gl.forward(1.0, 0.1)
    b = gl.buf
    xp = torch.zeros(gl.shape.P_cap, cfg.d, dtype=torch.bfloat16, device="cuda")
    B.evomoe_dispatch(gl.ctx, gl.shape, b.mask_bits, b.gprime, b.expert_offsets, b.pair_token, b.pair_gate,
                      b.tok_off, b.tok_rows, b.num_pairs, gl.x, xp)
    torch.cuda.synchronize()
    assert torch.equal(xp[:P], gl.x[b.pair_token[:P].long()])
    O1 = b.O.clone()
    B.evomoe_expert_ffn(gl.ctx, gl.shape, xp, None, b.expert_offsets, gl.params.W1, gl.params.b1,
                        gl.params.W2, gl.params.b2, b.H, b.A, b.O)
    torch.cuda.synchronize()
    assert torch.equal(O1[:P], b.O[:P])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_capacity_overflow_is_reported_and_stays_in_bounds(dtype):
    h = _harness()
    from paper_2112_14397_amd import binding as B
    cfg, inp = _mk("cap", 256, 64, 8, 128, "gelu", dtype, 0.0, 303)
    gl = h.GpuLayer(inp, P_cap=300)
    with pytest.raises(B.EvoMoEError) as ei:
        gl.forward(1e6, 0.0)          # dense: P = 2048 > 300
    assert ei.value.status == B.EVOMOE_ECAPACITY
    gl.backward(1e6)                  # clamps to P_cap; must not fault
    # the context is usable again afterwards
    P = gl.forward(0.01, 0.5)
    assert P == cfg.T


def test_argument_errors():
    h = _harness()
    from paper_2112_14397_amd import binding as B
    cfg, inp = _mk("args", 64, 64, 4, 64, "gelu", "f32", 0.1, 304)
    gl = h.GpuLayer(inp)
    b = gl.buf
    bad = B.make_shape(64, 64, 65, 64, "f32", "gelu", 256)
    with pytest.raises(B.EvoMoEError) as ei:
        B.evomoe_dts_gate(gl.ctx, bad, gl.x, gl.params.Wg, None, None, 1.0, 0.1, b.gprime, None, b.mask_bits, b.counts, None)
    assert ei.value.status == B.EVOMOE_EUNSUPPORTED
    with pytest.raises(B.EvoMoEError) as ei:
        B.evomoe_dts_gate(gl.ctx, gl.shape, gl.x, gl.params.Wg, None, None, 0.0, 0.1, b.gprime, None, b.mask_bits, b.counts, None)
    assert ei.value.status == B.EVOMOE_EINVAL
    with pytest.raises(B.EvoMoEError) as ei:
        B.evomoe_dts_gate(gl.ctx, gl.shape, None, gl.params.Wg, None, None, 1.0, 0.1, b.gprime, None, b.mask_bits, b.counts, None)
    assert ei.value.status == B.EVOMOE_EINVAL
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.EvoMoEError) as ei:
        B.evomoe_expert_ffn_bwd(gl.ctx, gl.shape, b.dO, b.H, b.A, gl.x, b.pair_token, b.expert_offsets,
                                gl.params.W1, gl.params.W2, None, None, b.dW1, b.db1, b.dW2, b.db2, b.dXp, False, small)
    assert ei.value.status == B.EVOMOE_EWORKSPACE


def test_step_can_be_captured_in_a_hip_graph_and_replayed():
    """The steady-state calls allocate nothing, clear nothing with memsets and never synchronise, so a caller may
    capture forward + backward in a HIP graph.  Replays (with eager work and synchronisations between them, at a
    different temperature) must reproduce the eager result bit for bit."""
    cfg = synth.LayerConfig("graph", T=600, d=128, E=8, F=256, act="gelu", dtype="bf16", taus=(1.0,),
                            threshold=0.08, seed=91, bias_std=0.05)
    inp = synth.make_layer_inputs(cfg)
    H = _harness()
    from paper_2112_14397_amd import binding as B
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        gl = H.GpuLayer(inp)                      # context bound to the side stream
        b = gl.buf

        def step(tau):
            B.layer_forward(gl.ctx, b, gl.params, gl.x, gl.noise, tau, cfg.threshold)
            B.layer_backward(gl.ctx, b, gl.params, gl.x, gl.dy, tau)

        step(0.9); step(0.5)                      # first calls size the context's scratch
        side.synchronize()
        P = B.evomoe_num_pairs(gl.ctx, b.num_pairs)
        want = {k: getattr(b, k).clone() for k in ("y", "dx", "dW1", "dW2", "dWg", "db1", "mask_bits", "tok_off")}
        want_rows = b.tok_rows[:P].clone()        # entries beyond P are whatever an earlier, denser step left
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            step(0.5)
        for _ in range(3):
            step(1.7)                             # eager work at another temperature in between
            side.synchronize()
            assert not torch.equal(b.mask_bits, want["mask_bits"])
            g.replay()
            side.synchronize()
            for k, v in want.items():
                assert torch.equal(getattr(b, k), v), f"{k} differs after a graph replay"
            assert torch.equal(b.tok_rows[:P], want_rows)


# ---- dispatch on its own: arbitrary masks (not a gate's), many 256-token blocks --------------------

@pytest.mark.parametrize("T,E,density", [(70001, 5, 0.4), (33000, 64, 0.08), (300, 64, 1.0), (1000, 33, 0.0)])
def test_dispatch_alone_on_random_masks(T, E, density):
    import torch
    from oracle import evomoe_oracle as orc
    from paper_2112_14397_amd import binding as B
    rng = np.random.default_rng(1234 + T + E)
    mask = rng.random((T, E)) < density
    if density == 0.0:
        mask[7, 3] = True                     # a single pair: every other block and expert is empty
    scores = rng.random((T, E), dtype=np.float32)
    bits = np.zeros(T, np.uint64)
    for e in range(E):
        bits |= mask[:, e].astype(np.uint64) << np.uint64(e)
    ref = orc.dispatch(mask, scores)
    P = int(ref.expert_offsets[E])
    P_cap = max(P, 1) + 17
    ctx = B.Context()
    shape = B.make_shape(T, 64, E, 64, "f32", "relu", P_cap)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    d_bits, d_scores = dev(bits.view(np.int64)), dev(scores)
    i32 = lambda n: torch.full((n,), -7, dtype=torch.int32, device="cuda")
    offs, ptok, toff, trows = i32(E + 1), i32(P_cap), i32(T + 1), i32(P_cap)
    pgate = torch.full((P_cap,), -7.0, dtype=torch.float32, device="cuda")
    npairs = torch.zeros(1, dtype=torch.int64, device="cuda")
    for _ in range(2):                        # twice: the context's scratch is reused
        B.evomoe_dispatch(ctx, shape, d_bits, d_scores, offs, ptok, pgate, toff, trows, npairs)
    assert B.evomoe_num_pairs(ctx, npairs) == P
    assert np.array_equal(offs.cpu().numpy(), ref.expert_offsets)
    assert np.array_equal(toff.cpu().numpy(), ref.tok_off)
    assert np.array_equal(ptok.cpu().numpy()[:P], ref.pair_token)
    assert np.array_equal(trows.cpu().numpy()[:P], ref.tok_rows)
    assert np.array_equal(pgate.cpu().numpy()[:P], ref.pair_gate.astype(np.float32))
    assert (ptok.cpu().numpy()[P:] == -7).all() and (trows.cpu().numpy()[P:] == -7).all()


def test_gelu_far_outside_the_fitted_range():
    """W1 scaled by 16 (exact in bf16) spreads the pre-activations to |h| of about 10: the bf16 kernels' polynomial
    GeLU has to take the exact limits beyond its fitted range (gelu = h, gelu' = 1 for large h; both 0 for very
    negative h).  Every feature still sees moderate h for some tokens, so every row of the gradients has a scale."""
    h = _harness()
    cfg, inp = _mk("gelu-tails", 300, 64, 4, 128, "gelu", "bf16", 0.1, 305, gate_scale=2.0)
    inp.W1 = (inp.W1 * np.float32(16.0)).astype(np.float32)
    gl = h.GpuLayer(inp)
    fwd, P, *_ = h.compare_forward(gl, inp, 1.0, 0.1)
    assert np.abs(fwd.ffn.H).max() > 8.0 and (np.abs(fwd.ffn.H) > 4.2).mean() > 0.05
    h.compare_backward(gl, inp, fwd, 1.0)
    h.compare_backward_stages(gl, inp, fwd, 1.0)


# ---- the gate at a token count beyond the configs' ------------------------------------------------------

@pytest.mark.parametrize("E,c", [(16, 0.05), (24, 0.03), (7, 0.12)])
def test_gate_alone_many_tokens(E, c):
    from oracle import evomoe_oracle as orc
    from paper_2112_14397_amd import binding as B
    T, d, tau = 70003, 136, 0.8
    rng = np.random.default_rng(4321 + E)
    x = torch.from_numpy(rng.standard_normal((T, d)).astype(np.float32)).to(torch.bfloat16)
    Wg = (rng.standard_normal((d, E)) * 0.3).astype(np.float32)
    bg = (rng.standard_normal(E) * 0.1).astype(np.float32)
    u = rng.random((T, E)).clip(1e-6, 1 - 1e-6)
    noise = (-np.log(-np.log(u))).astype(np.float32)
    ref = orc.dts_gate(x.float().numpy().astype(np.float64), Wg, bg, noise, tau, c)
    ctx = B.Context()
    shape = B.make_shape(T, d, E, 64, "bf16", "gelu", T * E)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    gp = torch.empty(T, E, dtype=torch.float32, device="cuda")
    gw = torch.empty(T, E, dtype=torch.float32, device="cuda")
    mb = torch.zeros(T, dtype=torch.int64, device="cuda")
    cn = torch.zeros(E, dtype=torch.int32, device="cuda")
    kt = torch.zeros(T, dtype=torch.int32, device="cuda")
    bh = torch.full(((T + 255) // 256, E), -5, dtype=torch.int32, device="cuda")
    B.evomoe_dts_gate(ctx, shape, x.cuda(), dev(Wg), dev(bg), dev(noise), tau, c, gp, gw, mb, cn, kt, bh)
    g = gp.cpu().numpy()
    from helpers import tol_ok
    ok, worst = tol_ok(g, ref.gprime, 1e-5)
    assert ok, f"gprime worst err/bound {worst:.3g}"
    bits = mb.cpu().numpy().view(np.uint64)
    mask = ((bits[:, None] >> np.arange(E, dtype=np.uint64)[None, :]) & np.uint64(1)).astype(bool)
    band = np.abs(ref.gprime - np.float64(np.float32(c))) < 1e-6
    diff = mask != ref.mask
    # only pairs inside the band may differ (a token none of whose scores passes keeps its arg-max: no such token
    # exists at these thresholds, which the oracle's count confirms)
    assert ref.n_fallback == 0
    assert not (diff & ~band).any(), f"{int((diff & ~band).sum())} mask bits differ outside the band"
    print(f"gate alone E={E}: {int(band.sum())} pairs inside the band, {int(diff.sum())} of them decided differently")
    hist = np.add.reduceat(mask.astype(np.int64), np.arange(0, T, 256), axis=0)
    assert np.array_equal(bh.cpu().numpy(), hist), "per-256-token histograms"
    assert np.array_equal(kt.cpu().numpy(), mask.sum(axis=1))
    assert np.array_equal(cn.cpu().numpy(), mask.sum(axis=0))
    w = gw.cpu().numpy()
    assert np.array_equal(w != 0, mask) and np.array_equal(w[mask], g[mask])

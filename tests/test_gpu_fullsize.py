"""Full-size parity (configs 2-5) in the launch configuration the benchmark times: per-pair buffers sized
from the pair count (not T*E), one context, forward then backward.  Whole-layer comparison where the oracle
can afford it (late, sparse temperatures), otherwise the oracle on sampled tokens and on whole experts."""
import numpy as np
import pytest
import torch

from paper_2112_14397_amd import binding as B
import synth_inputs as synth
import gpu_harness as H

pytestmark = pytest.mark.gpu

_inputs = {}


def inputs(name):
    if name not in _inputs:
        _inputs.clear()                      # one full-size input set at a time (host memory)
        _inputs[name] = synth.make_layer_inputs(synth.CONFIGS[name])
    return _inputs[name]


def bench_like_layer(inp, tau):
    """P_cap as the benchmark sizes it: pair count of a probe pass + 2 % + 256."""
    cfg = inp.cfg
    probe = H.GpuLayer(inp, P_cap=cfg.T * cfg.E, backward=False)
    shape8 = B.make_shape(cfg.T, cfg.d, cfg.E, 8, cfg.dtype, cfg.act, cfg.T * cfg.E)
    b = probe.buf
    B.evomoe_dts_gate(probe.ctx, shape8, probe.x, probe.params.Wg, probe.params.bg, probe.noise, float(tau),
                      float(cfg.threshold), b.gprime, None, b.mask_bits, b.counts, b.k)
    P = int(b.k.sum().item())
    del probe, b
    torch.cuda.empty_cache()
    return H.GpuLayer(inp, P_cap=int(P * 1.02) + 256, backward=True), P


# every temperature of every config: the gate and the dispatch of all tokens, bit for bit
EVERY_TAU = [(n, i) for n in ("gpt", "roberta", "mt", "large") for i in range(len(synth.CONFIGS[n].taus))]


@pytest.mark.parametrize("name,ti", EVERY_TAU, ids=[f"{n}-tau{i}" for n, i in EVERY_TAU])
def test_full_size_gate_and_dispatch_at_every_temperature(name, ti):
    inp = inputs(name)
    cfg = inp.cfg
    tau = cfg.taus[ti]
    key = (name, "gate-only")
    if key not in _layers:
        _layers.clear()
        torch.cuda.empty_cache()
        # only the gate and the dispatch are compared: the narrowest expert width the bf16 FFN accepts keeps the
        # per-pair buffers small at P_cap = T * E
        small = synth.small_variant(cfg, T=cfg.T, F=64)
        slim = type(inp)(cfg=small, x=inp.x, Wg=inp.Wg, bg=inp.bg, noise=inp.noise, W1=inp.W1[:, :64],
                         b1=inp.b1[:, :64], W2=inp.W2[:, :, :64], b2=inp.b2, dy=inp.dy)
        _layers[key] = (H.GpuLayer(slim, backward=False), slim)
    gl, slim = _layers[key]
    rep = {}
    H.compare_forward(gl, slim, tau, cfg.threshold, report=rep, check_ffn=False)
    print(f"\n{name} tau={tau:.3f}: {rep}")


_layers = {}

SAMPLED = [("gpt", 0), ("gpt", 3), ("roberta", 0), ("roberta", -1), ("mt", 0), ("large", 0), ("large", 3),
           ("large", -1)]


@pytest.mark.parametrize("name,ti", SAMPLED, ids=[f"{n}-tau{i}" for n, i in SAMPLED])
def test_full_size_sampled(name, ti):
    _layers.clear()
    inp = inputs(name)
    cfg = inp.cfg
    tau = cfg.taus[ti]
    gl, P = bench_like_layer(inp, tau)
    rep = {}
    worst = H.compare_full_size_sampled(gl, inp, tau, cfg.threshold, report=rep)
    assert rep["P"] == P
    print(f"\n{name} tau={tau:.3f}: {rep}  worst err/bound " + " ".join(f"{k}={v:.2f}" for k, v in worst.items()))


WHOLE = [("gpt", -1), ("gpt", 3), ("roberta", -1), ("mt", 0)]


@pytest.mark.parametrize("name,ti", WHOLE, ids=[f"{n}-tau{i}" for n, i in WHOLE])
def test_full_size_whole_layer(name, ti):
    """Late in the sweep the layer is sparse enough for the oracle to run all of it: every output of every
    stage, forward and backward, element by element."""
    _layers.clear()
    inp = inputs(name)
    cfg = inp.cfg
    tau = cfg.taus[ti]
    gl, P = bench_like_layer(inp, tau)
    rep, stats = {}, {}
    fwd, P2, _, _ = H.compare_forward(gl, inp, tau, cfg.threshold, report=rep)
    assert P2 == P
    # every output at the plain tolerance end to end, except the measured tail of dx (gpu_harness.DX_TAIL);
    # and every stage at the plain tolerance on the inputs the kernels' stage actually had
    _, worst = H.compare_backward(gl, inp, fwd, tau, dx_tail=H.DX_TAIL if cfg.dtype == "bf16" else None, stats=stats)
    stage = H.compare_backward_stages(gl, inp, fwd, tau)
    print(f"\n{name} tau={tau:.3f}: {rep}  worst err/bound " + " ".join(f"{k}={v:.2f}" for k, v in worst.items())
          + "  stages: " + " ".join(f"{k}={v:.2f}" for k, v in stage.items())
          + "\n  (worst, elements above the bound) per-row rms / per-tensor rms: "
          + " ".join(f"{k}={v['row']}/{v['tensor']}" for k, v in stats.items()))

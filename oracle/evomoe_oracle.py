"""CPU oracle for the DTS-Gate MoE layer (EvoMoE, arXiv 2112.14397).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the HIP
library is checked against.  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import it; the product path never does, and this file
imports nothing from the product package.

Everything is float64 numpy.  Inputs arrive as the exact values the GPU
receives (bf16 tensors widened to float); nothing is rounded in here.  A
library matmul is used where the paper writes a matrix-vector product for a
batch of tokens; there is no tiling, fusion or reordering.

Readings of the paper this oracle takes where the text is silent or garbled:
  * the softmax of the temperature gate normalises over the N experts of one
    token (the printed denominator's index is a typo);
  * the threshold test is strict, g'(x_s)_i > c, on the softmax output, and
    kept scores are NOT renormalised (Stage 2, "Content-based Sparsity");
  * DTS-Gate's comment N >= len(id_s) >= 1 is enforced: a token with no score
    above c keeps its arg-max expert (lowest index on ties) at its score g';
  * rows are ordered expert-major, token-ascending; the weighted sum over a
    token's experts runs in ascending expert id (Algorithm 1's inner loop);
  * GeLU is the exact x*Phi(x); ReLU'(0) = 0;
  * backward is plain calculus with the 0/1 selection treated as a constant;
    the paper derives none.

Pins (tests/test_oracle_*.py, all run without a GPU): the paper's worked gate
example, the E=2 sigmoid closed form, the dense (tau->inf, c=0) and top-1
(tau->0) limits, textbook values of Phi, a literal per-token brute force of
Algorithm 1, torch-CPU float64 autograd of an all-experts formulation, and
central finite differences; the balance loss and its gradient by a closed form,
finite differences and autograd; the schedule by the paper's quoted step counts;
the diversify masks by the published SplitMix64 test vectors, the two limits of
the mask ratio and binomial bounds on the masked fraction.
No function here is "parity unpinned".
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np
from scipy.special import erf as _erf

F64 = np.float64


# ---------------------------------------------------------------------------
# Gate  (Stage 2: Eq. "gumbel_softmax", Eq. "adaptive_sparsity", Algorithm 2)
# ---------------------------------------------------------------------------

def gate_logits(x, Wg, bg=None, noise=None):
    """z_s = x_s . W_g (+ b_g) + zeta_s   -- the argument of Eq. gumbel_softmax
    before the division by tau.  W_g is D x N (Sparse Gate Network paragraph)."""
    z = np.asarray(x, F64) @ np.asarray(Wg, F64)
    if bg is not None:
        z = z + np.asarray(bg, F64)[None, :]
    if noise is not None:
        z = z + np.asarray(noise, F64)
    return z


def temperature_softmax(z, tau):
    """g'(x_s)_i = exp(z_si / tau) / sum_j exp(z_sj / tau), j over the N experts
    (Eq. gumbel_softmax).  The row maximum is subtracted first; that leaves the
    value unchanged and keeps exp() in range."""
    a = np.asarray(z, F64) / F64(tau)
    a = a - a.max(axis=1, keepdims=True)
    e = np.exp(a)
    return e / e.sum(axis=1, keepdims=True)


@dataclass
class GateOut:
    gprime: np.ndarray   # [T,E] g'
    G: np.ndarray        # [T,E] g' where selected, else 0 (not renormalised)
    mask: np.ndarray     # [T,E] bool
    counts: np.ndarray   # [E] int64, tokens routed to each expert
    k: np.ndarray        # [T] int64, experts selected per token
    n_fallback: int      # tokens that had no score above c


def dts_gate(x, Wg, bg, noise, tau, threshold, mask_override=None) -> GateOut:
    """Dense-to-Sparse gate, threshold branch of Algorithm 2.

    mask_override (bool [T,E]) replaces the selection; it exists so that, when
    the two sides legitimately differ on a pair whose score is within rounding
    of c, everything downstream can still be compared on one selection.
    """
    gp = temperature_softmax(gate_logits(x, Wg, bg, noise), tau)
    c = F64(np.float32(threshold))          # the caller passes c as a float32
    mask = gp > c                            # strict (Eq. adaptive_sparsity)
    empty = ~mask.any(axis=1)
    n_fallback = int(empty.sum())
    if n_fallback:                           # Algorithm 2: len(id_s) >= 1
        rows = np.nonzero(empty)[0]
        mask[rows, gp[rows].argmax(axis=1)] = True   # argmax: lowest index on ties
    if mask_override is not None:
        mask = np.asarray(mask_override, bool).copy()
    G = np.where(mask, gp, 0.0)
    return GateOut(gp, G, mask, mask.sum(axis=0).astype(np.int64),
                   mask.sum(axis=1).astype(np.int64), n_fallback)


def top1_gate(x, Wg, bg, noise, tau) -> GateOut:
    """Top-1 branch of Algorithm 2 (after T_D iterations): the arg-max expert,
    weighted by its un-renormalised score g'."""
    gp = temperature_softmax(gate_logits(x, Wg, bg, noise), tau)
    mask = np.zeros_like(gp, bool)
    mask[np.arange(gp.shape[0]), gp.argmax(axis=1)] = True
    G = np.where(mask, gp, 0.0)
    return GateOut(gp, G, mask, mask.sum(axis=0).astype(np.int64),
                   mask.sum(axis=1).astype(np.int64), 0)


# ---------------------------------------------------------------------------
# Dispatch  (Stage 1 text: "Tokens will be dispatched to corresponding experts")
# ---------------------------------------------------------------------------

@dataclass
class DispatchOut:
    expert_offsets: np.ndarray  # [E+1] first row of each expert; [E] = P
    pair_token: np.ndarray      # [P] token of each row
    pair_expert: np.ndarray     # [P] expert of each row
    pair_gate: np.ndarray       # [P] G of each row
    tok_off: np.ndarray         # [T+1] CSR offsets; token s owns tok_rows[tok_off[s]:tok_off[s+1]]
    tok_rows: np.ndarray        # [P] rows of token s, ascending expert id


def dispatch(mask, G) -> DispatchOut:
    """Variable-k permutation: one row per selected (token, expert) pair, rows
    grouped by expert (ascending), tokens ascending inside an expert."""
    mask = np.asarray(mask, bool)
    T, E = mask.shape
    counts = mask.sum(axis=0)
    offsets = np.zeros(E + 1, np.int64)
    offsets[1:] = np.cumsum(counts)
    P = int(offsets[E])
    pair_token = np.empty(P, np.int64)
    pair_expert = np.empty(P, np.int64)
    row_of = -np.ones((T, E), np.int64)
    for i in range(E):
        toks = np.nonzero(mask[:, i])[0]                 # ascending token id
        r0 = offsets[i]
        pair_token[r0:r0 + len(toks)] = toks
        pair_expert[r0:r0 + len(toks)] = i
        row_of[toks, i] = r0 + np.arange(len(toks))
    pair_gate = np.asarray(G, F64)[pair_token, pair_expert]
    k = mask.sum(axis=1)
    tok_off = np.zeros(T + 1, np.int64)
    tok_off[1:] = np.cumsum(k)
    tok_rows = row_of[mask]                              # row-major walk: token, then expert ascending
    return DispatchOut(offsets, pair_token, pair_expert, pair_gate, tok_off, tok_rows.astype(np.int64))


# ---------------------------------------------------------------------------
# Expert FFN  (Eq. "ffn";  GeLU per the Hyper-Parameter Detail paragraph)
# ---------------------------------------------------------------------------

def activation(h, act):
    h = np.asarray(h, F64)
    if act == "relu":
        return np.maximum(h, 0.0)
    if act == "gelu":
        return h * 0.5 * (1.0 + _erf(h / np.sqrt(2.0)))      # x * Phi(x)
    raise ValueError(act)


def activation_grad(h, act):
    h = np.asarray(h, F64)
    if act == "relu":
        return (h > 0.0).astype(F64)
    if act == "gelu":
        Phi = 0.5 * (1.0 + _erf(h / np.sqrt(2.0)))
        phi = np.exp(-0.5 * h * h) / np.sqrt(2.0 * np.pi)
        return Phi + h * phi
    raise ValueError(act)


@dataclass
class FFNOut:
    H: np.ndarray   # [P,F] W1 x + b1 (pre-activation)
    A: np.ndarray   # [P,F] act(H)
    O: np.ndarray   # [P,d] W2 A + b2 = e_i(x_s) for the row's (s,i)


def expert_ffn(x, pair_token, expert_offsets, W1, b1, W2, b2, act) -> FFNOut:
    """e_i(x_s) = W2_i . act(W1_i . x_s + b1_i) + b2_i for every selected pair,
    W1_i in R^{F x D}, W2_i in R^{D x F} (Eq. ffn)."""
    x = np.asarray(x, F64)
    E = len(expert_offsets) - 1
    P = int(expert_offsets[E])
    F_, d = W1.shape[1], W1.shape[2]
    H = np.empty((P, F_), F64)
    A = np.empty((P, F_), F64)
    O = np.empty((P, d), F64)
    for i in range(E):
        r0, r1 = int(expert_offsets[i]), int(expert_offsets[i + 1])
        if r1 == r0:
            continue
        Xi = x[pair_token[r0:r1]]
        H[r0:r1] = Xi @ np.asarray(W1[i], F64).T + np.asarray(b1[i], F64)[None, :]
        A[r0:r1] = activation(H[r0:r1], act)
        O[r0:r1] = A[r0:r1] @ np.asarray(W2[i], F64).T + np.asarray(b2[i], F64)[None, :]
    return FFNOut(H, A, O)


# ---------------------------------------------------------------------------
# Combine  (Eq. "moe_weighted_sum_problem";  Algorithm 1 inner loops)
# ---------------------------------------------------------------------------

def combine(O, pair_gate, tok_off, tok_rows, T):
    """y_s = sum over id in id_s (ascending) of G_{s,id} * e_id(x_s)."""
    d = O.shape[1]
    y = np.zeros((T, d), F64)
    kmax = int((tok_off[1:] - tok_off[:-1]).max()) if T else 0
    for j in range(kmax):                      # j-th selected expert of every token that has one
        has = (tok_off[:-1] + j) < tok_off[1:]
        rows = tok_rows[tok_off[:-1][has] + j]
        y[has] += pair_gate[rows][:, None] * O[rows]
    return y


# ---------------------------------------------------------------------------
# Whole layer forward
# ---------------------------------------------------------------------------

@dataclass
class LayerFwd:
    gate: GateOut
    disp: DispatchOut
    ffn: FFNOut
    y: np.ndarray


def moe_layer_forward(x, Wg, bg, noise, tau, threshold, W1, b1, W2, b2, act,
                      mask_override=None, top1=False) -> LayerFwd:
    g = top1_gate(x, Wg, bg, noise, tau) if top1 else \
        dts_gate(x, Wg, bg, noise, tau, threshold, mask_override)
    dp = dispatch(g.mask, g.G)
    f = expert_ffn(x, dp.pair_token, dp.expert_offsets, W1, b1, W2, b2, act)
    y = combine(f.O, dp.pair_gate, dp.tok_off, dp.tok_rows, np.asarray(x).shape[0])
    return LayerFwd(g, dp, f, y)


# ---------------------------------------------------------------------------
# Backward (derived from the forward equations; selection is a constant)
# ---------------------------------------------------------------------------

def combine_bwd(dy, O, pair_gate, pair_token):
    """From y_s = sum G_r O_r:  dO_r = G_r dy_{s(r)},  dG_r = <dy_{s(r)}, O_r>."""
    dy = np.asarray(dy, F64)
    dys = dy[pair_token]
    dO = pair_gate[:, None] * dys
    dG = np.einsum("rd,rd->r", dys, O)
    return dO, dG


@dataclass
class FFNGrads:
    dW1: np.ndarray
    db1: np.ndarray
    dW2: np.ndarray
    db2: np.ndarray
    dXp: np.ndarray   # [P,d] gradient w.r.t. the expert's input row
    dH: np.ndarray    # [P,F]


def expert_ffn_bwd(dO, H, x, pair_token, expert_offsets, W1, W2, act) -> FFNGrads:
    """Backward of O = W2 act(W1 x + b1) + b2 per expert over its rows."""
    x = np.asarray(x, F64)
    E = len(expert_offsets) - 1
    P = int(expert_offsets[E])
    F_, d = W1.shape[1], W1.shape[2]
    dW1 = np.zeros((E, F_, d), F64)
    db1 = np.zeros((E, F_), F64)
    dW2 = np.zeros((E, d, F_), F64)
    db2 = np.zeros((E, d), F64)
    dXp = np.zeros((P, d), F64)
    dH = np.zeros((P, F_), F64)
    for i in range(E):
        r0, r1 = int(expert_offsets[i]), int(expert_offsets[i + 1])
        if r1 == r0:
            continue
        Xi = x[pair_token[r0:r1]]
        Ai = activation(H[r0:r1], act)
        dOi = dO[r0:r1]
        db2[i] = dOi.sum(axis=0)
        dW2[i] = dOi.T @ Ai
        dA = dOi @ np.asarray(W2[i], F64)
        dHi = dA * activation_grad(H[r0:r1], act)
        dH[r0:r1] = dHi
        db1[i] = dHi.sum(axis=0)
        dW1[i] = dHi.T @ Xi
        dXp[r0:r1] = dHi @ np.asarray(W1[i], F64)
    return FFNGrads(dW1, db1, dW2, db2, dXp, dH)


def dispatch_bwd(dXp, tok_off, tok_rows, T):
    """dx_s = sum of dXp over the rows of token s (ascending expert id)."""
    d = dXp.shape[1]
    dx = np.zeros((T, d), F64)
    kmax = int((tok_off[1:] - tok_off[:-1]).max()) if T else 0
    for j in range(kmax):
        has = (tok_off[:-1] + j) < tok_off[1:]
        rows = tok_rows[tok_off[:-1][has] + j]
        dx[has] += dXp[rows]
    return dx


def dts_gate_bwd(dG_pairs, pair_token, pair_expert, gprime, tau, x, Wg, dgprime_coef=None):
    """Backward of G = mask * softmax(z / tau), z = x W_g + b_g + zeta.

    dG_si is dG_pairs at selected pairs and 0 elsewhere.  Softmax backward:
    dz_sj = (g'_sj / tau) * (dG_sj - sum_i dG_si g'_si).  Unselected columns
    still receive gradient through the normaliser.
    dgprime_coef [E], optional: a gradient with respect to g'_si that is the
    same for every token (the balance loss's, see balance_loss_grad); it is
    added to dG_si for every (s, i), selected or not.
    Returns dz, dWg, dbg and the gate's contribution to dx.
    """
    T, E = gprime.shape
    dG = np.zeros((T, E), F64)
    dG[pair_token, pair_expert] = dG_pairs
    if dgprime_coef is not None:
        dG = dG + np.asarray(dgprime_coef, F64)[None, :]
    inner = (dG * gprime).sum(axis=1, keepdims=True)
    dz = gprime * (dG - inner) / F64(tau)
    dWg = np.asarray(x, F64).T @ dz
    dbg = dz.sum(axis=0)
    dx_gate = dz @ np.asarray(Wg, F64).T
    return dz, dWg, dbg, dx_gate


@dataclass
class LayerBwd:
    dO: np.ndarray
    dG_pairs: np.ndarray
    ffn: FFNGrads
    dz: np.ndarray
    dWg: np.ndarray
    dbg: np.ndarray
    dx_experts: np.ndarray   # dispatch_bwd output alone
    dx: np.ndarray           # full gradient w.r.t. x


def moe_layer_backward(fwd: LayerFwd, dy, x, Wg, tau, W1, W2, act) -> LayerBwd:
    dp = fwd.disp
    T = np.asarray(x).shape[0]
    dO, dGp = combine_bwd(dy, fwd.ffn.O, dp.pair_gate, dp.pair_token)
    fg = expert_ffn_bwd(dO, fwd.ffn.H, x, dp.pair_token, dp.expert_offsets, W1, W2, act)
    dx_e = dispatch_bwd(fg.dXp, dp.tok_off, dp.tok_rows, T)
    dz, dWg, dbg, dx_g = dts_gate_bwd(dGp, dp.pair_token, dp.pair_expert, fwd.gate.gprime, tau, x, Wg)
    return LayerBwd(dO, dGp, fg, dz, dWg, dbg, dx_e, dx_e + dx_g)


# ---------------------------------------------------------------------------
# Balance loss (Eq. "balance_loss") -- used by the roberta-config skew script
# and kept as the definition for the "next" row that adds it to the path.
# ---------------------------------------------------------------------------

def balance_loss(gate: GateOut, alpha=0.1):
    """alpha * N * sum_i (count_i / |B|^2) * sum_s g'_si."""
    T, E = gate.gprime.shape
    return F64(alpha) * E * float((gate.counts / F64(T) ** 2 * gate.gprime.sum(axis=0)).sum())


def balance_loss_grad(gate: GateOut, alpha=0.1):
    """d L_balance / d g'_si = alpha * N * count_i / |B|^2 for every token s.

    The count is an indicator sum (Eq. "balance_loss"): piecewise constant in
    the gate's parameters, so it is a constant of the differentiation, as in
    the Switch-style loss the paper refers to.  Returns the [E] coefficient
    vector that dts_gate_bwd takes as dgprime_coef."""
    T, E = gate.gprime.shape
    return F64(alpha) * E * gate.counts.astype(F64) / F64(T) ** 2


# ---------------------------------------------------------------------------
# Training phases (Algorithm 1's loop bounds; Algorithm 2's T_D switch; the
# Sparsity Scheduler paragraph; "we decay temperature from max_value to
# min_value in the first ... iterations and switch to Top1 then")
# ---------------------------------------------------------------------------

@dataclass
class Phase:
    stage: int      # 1 = expert-diversify (one shared expert, no gate), 2 = gate-sparsify
    top1: bool      # stage 2 only: Algorithm 2's else-branch
    tau: float      # stage 2 only


def schedule(iteration, T_S, T_D, tau_hi=2.0, tau_lo=0.3) -> Phase:
    """Phase of training iteration `iteration` (0-based).

    Iterations [0, T_S) train the shared expert.  The next T_D iterations run
    the threshold gate while tau goes from tau_hi to tau_lo, both end points
    reached (a linear ramp: the paper gives the end points and the duration
    only).  From T_S + T_D on the gate is Top-1 at tau_lo.  T_D counts from the
    start of stage 2 (Algorithm 2 compares it with the current iteration; the
    experiments quote it as the number of steps after the first stage)."""
    if iteration < T_S:
        return Phase(1, False, float("nan"))
    j = iteration - T_S
    if j < T_D:
        tau = tau_hi if T_D == 1 else tau_hi - (tau_hi - tau_lo) * (j / F64(T_D - 1))
        return Phase(2, False, float(tau))
    return Phase(2, True, float(tau_lo))


# ---------------------------------------------------------------------------
# Expert-diversify (Stage 1; Algorithm 1's loop  e_i <- diversify(e, i))
# ---------------------------------------------------------------------------
# The paper spawns the N experts from the one shared expert by a random mask
# that sets part of its weights to 0, a different mask per expert; it gives
# neither the masked fraction nor the random source.  Readings taken here: the
# fraction is an argument; every weight of W1 and W2 is masked independently
# with that probability; biases are copied unmasked; the random numbers come
# from a counter-based generator, so that both sides can draw the same ones:
# weight number j of tensor t (0 = W1, 1 = W2) of expert i uses output number
# (t << 62 | i << 48 | j) of the SplitMix64 sequence (Steele, Lea & Flood 2014;
# Vigna's public-domain constants) seeded with `seed`, and is masked when the
# top 24 bits of that output are below floor(ratio * 2^24).

_U64 = np.uint64


def splitmix64_output(seed, n):
    """Output number n (0-based, scalar or uint64 array) of the SplitMix64 sequence seeded with `seed`."""
    with np.errstate(over="ignore"):
        z = _U64(seed) + (np.asarray(n, _U64) + _U64(1)) * _U64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> _U64(30))) * _U64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> _U64(27))) * _U64(0x94D049BB133111EB)
        return z ^ (z >> _U64(31))


def diversify_keep_mask(seed, mask_ratio, tensor, expert, n_weights):
    """bool [n_weights]: True where expert `expert` keeps weight j of tensor `tensor` (0 = W1, 1 = W2)."""
    limit = int(np.floor(np.float64(np.float32(mask_ratio)) * 2.0 ** 24))      # the caller passes a float32
    ctr = (_U64(tensor) << _U64(62)) | (_U64(expert) << _U64(48)) | np.arange(n_weights, dtype=_U64)
    return (splitmix64_output(seed, ctr) >> _U64(40)).astype(np.int64) >= limit


def diversify(W1_shared, b1_shared, W2_shared, b2_shared, E, seed, mask_ratio):
    """e_i <- diversify(e, i) for i = 0..E-1: copies of the shared expert (W1 [F,d], b1 [F], W2 [d,F], b2 [d])
    with a different random part of the weights set to 0 in each.  Returns W1 [E,F,d], b1 [E,F], W2 [E,d,F],
    b2 [E,d] in the dtype of the inputs."""
    W1_shared = np.asarray(W1_shared)
    W2_shared = np.asarray(W2_shared)
    W1 = np.empty((E,) + W1_shared.shape, W1_shared.dtype)
    W2 = np.empty((E,) + W2_shared.shape, W2_shared.dtype)
    for i in range(E):
        keep1 = diversify_keep_mask(seed, mask_ratio, 0, i, W1_shared.size).reshape(W1_shared.shape)
        keep2 = diversify_keep_mask(seed, mask_ratio, 1, i, W2_shared.size).reshape(W2_shared.shape)
        W1[i] = np.where(keep1, W1_shared, 0)
        W2[i] = np.where(keep2, W2_shared, 0)
    b1 = np.repeat(np.asarray(b1_shared)[None, :], E, axis=0)
    b2 = np.repeat(np.asarray(b2_shared)[None, :], E, axis=0)
    return W1, b1, W2, b2

"""Thin ctypes binding of libevomoe.so (the C ABI declared in include/evomoe.h).

Argument marshalling only: every step of the layer runs in the HIP kernels.
torch is used for device memory and the stream, nothing else.  There is no CPU
fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libevomoe.so")   # tests and tools may point this elsewhere before lib()

EVOMOE_F32, EVOMOE_BF16 = 0, 1
EVOMOE_RELU, EVOMOE_GELU_ERF = 0, 1
EVOMOE_OK, EVOMOE_EINVAL, EVOMOE_EUNSUPPORTED, EVOMOE_ECAPACITY, EVOMOE_EWORKSPACE, EVOMOE_EHIP = 0, -1, -2, -3, -4, -5
EVOMOE_ESTATIC = -6

ENTRY_POINTS = (
    "evomoe_create", "evomoe_destroy", "evomoe_status_string", "evomoe_workspace_bytes",
    "evomoe_dts_gate", "evomoe_dispatch", "evomoe_expert_ffn", "evomoe_combine",
    "evomoe_combine_bwd", "evomoe_expert_ffn_bwd", "evomoe_dispatch_bwd", "evomoe_dts_gate_bwd",
    "evomoe_num_pairs", "evomoe_profile_select", "evomoe_profile_read",
    "evomoe_dts_gate_top1", "evomoe_balance_loss", "evomoe_dts_gate_bwd_balance",
    "evomoe_workspace_bytes_recompute", "evomoe_expert_ffn_bwd_recompute", "evomoe_schedule",
    "evomoe_hint_pairs", "evomoe_diversify", "evomoe_dispatch_static",
)

KERNEL_IDS = ("gate", "dispatch_hist", "dispatch_scatter", "ffn_gemm1", "ffn_gemm2", "combine", "combine_bwd",
              "ffn_bwd_dh", "ffn_bwd_dx", "ffn_bwd_dw2", "ffn_bwd_dw1", "ffn_bwd_db", "dispatch_bwd",
              "gate_bwd_dz", "gate_bwd_main", "gate_bwd_reduce", "balance_loss", "diversify")
EVOMOE_K_ALL, EVOMOE_K_NONE = -2, -1


class EvoMoEError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().evomoe_status_string(status).decode()
        super().__init__(f"{where}: {msg} ({status})")


class Phase(ctypes.Structure):
    _fields_ = [("stage", ctypes.c_int32), ("top1", ctypes.c_int32), ("tau", ctypes.c_float)]


class Shape(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("d", ctypes.c_int32), ("E", ctypes.c_int32), ("F", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("act", ctypes.c_int32), ("P_cap", ctypes.c_int64)]


_lib = None


def lib() -> ctypes.CDLL:
    """Load libevomoe.so; raises if it is missing (build it with `python -m paper_2112_14397_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} not found: the HIP library is not built "
                               "(run `python -m paper_2112_14397_amd.build`); there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        vp, f32, i32, sz = ctypes.c_void_p, ctypes.c_float, ctypes.c_int, ctypes.c_size_t
        sp = ctypes.POINTER(Shape)
        L.evomoe_create.argtypes = [ctypes.POINTER(vp), vp]
        L.evomoe_destroy.argtypes = [vp]
        L.evomoe_status_string.argtypes = [i32]
        L.evomoe_status_string.restype = ctypes.c_char_p
        L.evomoe_workspace_bytes.argtypes = [sp]
        L.evomoe_workspace_bytes.restype = sz
        L.evomoe_dts_gate.argtypes = [vp, sp, vp, vp, vp, vp, f32, f32, vp, vp, vp, vp, vp, vp]
        L.evomoe_dispatch.argtypes = [vp, sp] + [vp] * 11
        L.evomoe_dispatch_static.argtypes = [vp, sp] + [vp] * 10
        L.evomoe_expert_ffn.argtypes = [vp, sp] + [vp] * 10
        L.evomoe_combine.argtypes = [vp, sp] + [vp] * 5
        L.evomoe_combine_bwd.argtypes = [vp, sp] + [vp] * 7
        L.evomoe_expert_ffn_bwd.argtypes = [vp, sp] + [vp] * 15 + [i32, vp, sz]
        L.evomoe_dispatch_bwd.argtypes = [vp, sp] + [vp] * 4
        L.evomoe_dts_gate_bwd.argtypes = [vp, sp, vp, vp, vp, vp, vp, f32, vp, vp, vp, vp, vp, vp, sz]
        L.evomoe_num_pairs.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_int64)]
        L.evomoe_dts_gate_top1.argtypes = [vp, sp, vp, vp, vp, vp, f32, vp, vp, vp, vp, vp, vp]
        L.evomoe_balance_loss.argtypes = [vp, sp, vp, vp, f32, vp, vp]
        L.evomoe_dts_gate_bwd_balance.argtypes = [vp, sp, vp, vp, vp, vp, vp, f32, vp, vp, vp, f32, vp, vp, vp, vp, sz]
        L.evomoe_workspace_bytes_recompute.argtypes = [sp]
        L.evomoe_workspace_bytes_recompute.restype = sz
        L.evomoe_expert_ffn_bwd_recompute.argtypes = [vp, sp] + [vp] * 14 + [i32, vp, sz]
        L.evomoe_hint_pairs.argtypes = [vp, ctypes.c_int64]
        L.evomoe_diversify.argtypes = [vp, sp, vp, vp, vp, vp, ctypes.c_uint64, f32, vp, vp, vp, vp]
        L.evomoe_schedule.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, f32, f32, ctypes.POINTER(Phase)]
        L.evomoe_profile_select.argtypes = [vp, i32]
        L.evomoe_profile_read.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
        for n in ENTRY_POINTS:
            if n not in ("evomoe_status_string", "evomoe_workspace_bytes", "evomoe_workspace_bytes_recompute"):
                getattr(L, n).restype = i32
        _lib = L
    return _lib


def _p(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device, contiguous tensors only"
    return ctypes.c_void_p(t.data_ptr())


def _chk(st: int, where: str):
    if st != EVOMOE_OK:
        raise EvoMoEError(st, where)


def make_shape(T, d, E, F, dtype: str, act: str, P_cap: int) -> Shape:
    return Shape(T, d, E, F, {"f32": EVOMOE_F32, "bf16": EVOMOE_BF16}[dtype],
                 {"relu": EVOMOE_RELU, "gelu": EVOMOE_GELU_ERF}[act], P_cap)


def torch_dtype(dtype: str):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]


class Context:
    """evomoe_ctx bound to torch's current stream on the current device."""

    def __init__(self, stream: Optional[torch.cuda.Stream] = None):
        self._h = ctypes.c_void_p()
        s = stream if stream is not None else torch.cuda.current_stream()
        _chk(lib().evomoe_create(ctypes.byref(self._h), ctypes.c_void_p(s.cuda_stream)), "evomoe_create")
        self.stream = s

    def close(self):
        if self._h:
            lib().evomoe_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ---- one function per C entry point, same names and argument order ----------------------------

def evomoe_workspace_bytes(shape: Shape) -> int:
    return int(lib().evomoe_workspace_bytes(ctypes.byref(shape)))


def evomoe_dts_gate(ctx, shape, x, Wg, bg, noise, tau, threshold, gprime, gate_w, mask_bits, counts, k_per_token,
                    block_hist=None):
    _chk(lib().evomoe_dts_gate(ctx._h, ctypes.byref(shape), _p(x), _p(Wg), _p(bg), _p(noise), tau, threshold,
                               _p(gprime), _p(gate_w), _p(mask_bits), _p(counts), _p(k_per_token), _p(block_hist)),
         "evomoe_dts_gate")


def evomoe_dispatch(ctx, shape, mask_bits, scores, expert_offsets, pair_token, pair_gate, tok_off, tok_rows,
                    num_pairs, x=None, x_perm=None, block_hist=None):
    _chk(lib().evomoe_dispatch(ctx._h, ctypes.byref(shape), _p(mask_bits), _p(scores), _p(expert_offsets),
                               _p(pair_token), _p(pair_gate), _p(tok_off), _p(tok_rows), _p(num_pairs),
                               _p(x), _p(x_perm), _p(block_hist)), "evomoe_dispatch")


def evomoe_dispatch_static(ctx, shape, mask_bits, scores, expert_offsets, pair_token, pair_gate, tok_off, tok_rows,
                           num_pairs, x=None, x_perm=None):
    _chk(lib().evomoe_dispatch_static(ctx._h, ctypes.byref(shape), _p(mask_bits), _p(scores), _p(expert_offsets),
                                      _p(pair_token), _p(pair_gate), _p(tok_off), _p(tok_rows), _p(num_pairs),
                                      _p(x), _p(x_perm)), "evomoe_dispatch_static")


def evomoe_expert_ffn(ctx, shape, x, pair_token, expert_offsets, W1, b1, W2, b2, H, A, O):
    _chk(lib().evomoe_expert_ffn(ctx._h, ctypes.byref(shape), _p(x), _p(pair_token), _p(expert_offsets),
                                 _p(W1), _p(b1), _p(W2), _p(b2), _p(H), _p(A), _p(O)), "evomoe_expert_ffn")


def evomoe_combine(ctx, shape, O, pair_gate, tok_off, tok_rows, y):
    _chk(lib().evomoe_combine(ctx._h, ctypes.byref(shape), _p(O), _p(pair_gate), _p(tok_off), _p(tok_rows), _p(y)),
         "evomoe_combine")


def evomoe_combine_bwd(ctx, shape, dy, O, pair_gate, pair_token, expert_offsets, dO, dG_pairs):
    _chk(lib().evomoe_combine_bwd(ctx._h, ctypes.byref(shape), _p(dy), _p(O), _p(pair_gate), _p(pair_token),
                                  _p(expert_offsets), _p(dO), _p(dG_pairs)), "evomoe_combine_bwd")


def evomoe_expert_ffn_bwd(ctx, shape, dO, H, A, x, pair_token, expert_offsets, W1, W2, dy, pair_gate, dW1, db1, dW2,
                          db2, dXp, accumulate, workspace):
    _chk(lib().evomoe_expert_ffn_bwd(ctx._h, ctypes.byref(shape), _p(dO), _p(H), _p(A), _p(x), _p(pair_token),
                                     _p(expert_offsets), _p(W1), _p(W2), _p(dy), _p(pair_gate), _p(dW1), _p(db1),
                                     _p(dW2), _p(db2),
                                     _p(dXp), int(accumulate), _p(workspace),
                                     workspace.numel() * workspace.element_size()), "evomoe_expert_ffn_bwd")


def evomoe_dispatch_bwd(ctx, shape, dXp, tok_off, tok_rows, dx):
    _chk(lib().evomoe_dispatch_bwd(ctx._h, ctypes.byref(shape), _p(dXp), _p(tok_off), _p(tok_rows), _p(dx)),
         "evomoe_dispatch_bwd")


def evomoe_dts_gate_bwd(ctx, shape, dG_pairs, tok_off, tok_rows, gprime, mask_bits, tau, x, Wg, dWg, dbg, dx,
                        workspace):
    _chk(lib().evomoe_dts_gate_bwd(ctx._h, ctypes.byref(shape), _p(dG_pairs), _p(tok_off), _p(tok_rows),
                                   _p(gprime), _p(mask_bits), tau, _p(x), _p(Wg), _p(dWg), _p(dbg), _p(dx),
                                   _p(workspace), workspace.numel() * workspace.element_size()),
         "evomoe_dts_gate_bwd")


def evomoe_dts_gate_top1(ctx, shape, x, Wg, bg, noise, tau, gprime, gate_w, mask_bits, counts, k_per_token,
                         block_hist=None):
    _chk(lib().evomoe_dts_gate_top1(ctx._h, ctypes.byref(shape), _p(x), _p(Wg), _p(bg), _p(noise), tau,
                                    _p(gprime), _p(gate_w), _p(mask_bits), _p(counts), _p(k_per_token),
                                    _p(block_hist)), "evomoe_dts_gate_top1")


def evomoe_balance_loss(ctx, shape, gprime, counts, alpha, loss, dgprime_coef):
    _chk(lib().evomoe_balance_loss(ctx._h, ctypes.byref(shape), _p(gprime), _p(counts), alpha, _p(loss),
                                   _p(dgprime_coef)), "evomoe_balance_loss")


def evomoe_dts_gate_bwd_balance(ctx, shape, dG_pairs, tok_off, tok_rows, gprime, mask_bits, tau, x, Wg,
                                dgprime_coef, loss_scale, dWg, dbg, dx, workspace):
    _chk(lib().evomoe_dts_gate_bwd_balance(ctx._h, ctypes.byref(shape), _p(dG_pairs), _p(tok_off), _p(tok_rows),
                                           _p(gprime), _p(mask_bits), tau, _p(x), _p(Wg), _p(dgprime_coef),
                                           loss_scale, _p(dWg), _p(dbg), _p(dx), _p(workspace),
                                           workspace.numel() * workspace.element_size()),
         "evomoe_dts_gate_bwd_balance")


def evomoe_workspace_bytes_recompute(shape: Shape) -> int:
    return int(lib().evomoe_workspace_bytes_recompute(ctypes.byref(shape)))


def evomoe_expert_ffn_bwd_recompute(ctx, shape, dO, x, pair_token, expert_offsets, W1, b1, W2, dy, pair_gate, dW1,
                                    db1, dW2, db2, dXp, accumulate, workspace):
    _chk(lib().evomoe_expert_ffn_bwd_recompute(ctx._h, ctypes.byref(shape), _p(dO), _p(x), _p(pair_token),
                                               _p(expert_offsets), _p(W1), _p(b1), _p(W2), _p(dy), _p(pair_gate),
                                               _p(dW1), _p(db1),
                                               _p(dW2), _p(db2), _p(dXp), int(accumulate), _p(workspace),
                                               workspace.numel() * workspace.element_size()),
         "evomoe_expert_ffn_bwd_recompute")


def evomoe_schedule(iteration, T_S, T_D, tau_hi=2.0, tau_lo=0.3) -> Phase:
    ph = Phase()
    _chk(lib().evomoe_schedule(iteration, T_S, T_D, tau_hi, tau_lo, ctypes.byref(ph)), "evomoe_schedule")
    return ph


def evomoe_diversify(ctx, shape, W1_shared, b1_shared, W2_shared, b2_shared, seed, mask_ratio, W1, b1, W2, b2):
    _chk(lib().evomoe_diversify(ctx._h, ctypes.byref(shape), _p(W1_shared), _p(b1_shared), _p(W2_shared),
                                _p(b2_shared), int(seed), float(mask_ratio), _p(W1), _p(b1), _p(W2), _p(b2)),
         "evomoe_diversify")


def evomoe_hint_pairs(ctx, expected_pairs: int) -> None:
    _chk(lib().evomoe_hint_pairs(ctx._h, int(expected_pairs)), "evomoe_hint_pairs")


def evomoe_num_pairs(ctx, num_pairs) -> int:
    out = ctypes.c_int64(0)
    _chk(lib().evomoe_num_pairs(ctx._h, _p(num_pairs), ctypes.byref(out)), "evomoe_num_pairs")
    return int(out.value)


def evomoe_profile_select(ctx, kernel) -> None:
    """kernel: a name from KERNEL_IDS, "all" or None (off)."""
    kid = EVOMOE_K_NONE if kernel is None else EVOMOE_K_ALL if kernel == "all" else KERNEL_IDS.index(kernel)
    _chk(lib().evomoe_profile_select(ctx._h, kid), "evomoe_profile_select")


def evomoe_profile_read(ctx) -> dict:
    """{kernel name: (total milliseconds, launches)} for the kernels bracketed since the last read."""
    n = len(KERNEL_IDS)
    ms = (ctypes.c_double * n)()
    cnt = (ctypes.c_int64 * n)()
    _chk(lib().evomoe_profile_read(ctx._h, ms, cnt), "evomoe_profile_read")
    return {KERNEL_IDS[i]: (float(ms[i]), int(cnt[i])) for i in range(n) if cnt[i]}


# ---- buffers for one layer + the call sequence (allocation and ordering only) -------------------

@dataclass
class LayerParams:
    Wg: torch.Tensor
    bg: Optional[torch.Tensor]
    W1: torch.Tensor
    b1: Optional[torch.Tensor]
    W2: torch.Tensor
    b2: Optional[torch.Tensor]


class LayerBuffers:
    """Every output / saved tensor of one forward+backward pass, allocated once."""

    def __init__(self, shape: Shape, device="cuda", backward=True, recompute=False):
        T, d, E, F, P = shape.T, shape.d, shape.E, shape.F, shape.P_cap
        dt = torch.bfloat16 if shape.dtype == EVOMOE_BF16 else torch.float32
        z = lambda *s, dtype=dt: torch.zeros(*s, dtype=dtype, device=device)
        f32, i32, i64 = torch.float32, torch.int32, torch.int64
        self.shape = shape
        self.gprime = z(T, E, dtype=f32); self.gate_w = z(T, E, dtype=f32)
        self.mask_bits = z(T, dtype=i64); self.counts = z(E, dtype=i32); self.k = z(T, dtype=i32)
        self.expert_offsets = z(E + 1, dtype=i32); self.pair_token = z(P, dtype=i32)
        self.pair_gate = z(P, dtype=f32); self.tok_off = z(T + 1, dtype=i32); self.tok_rows = z(P, dtype=i32)
        self.num_pairs = z(1, dtype=i64); self.block_hist = z((T + 255) // 256, E, dtype=i32)
        self.H = z(P, F); self.A = z(P, F); self.O = z(P, d); self.y = z(T, d)
        if backward:
            self.dO = z(P, d); self.dG_pairs = z(P, dtype=f32); self.dXp = z(P, d); self.dx = z(T, d)
            self.dW1 = z(E, F, d); self.dW2 = z(E, d, F); self.db1 = z(E, F, dtype=f32); self.db2 = z(E, d, dtype=f32)
            self.dWg = z(d, E, dtype=f32); self.dbg = z(E, dtype=f32)
            nbytes = evomoe_workspace_bytes_recompute(shape) if recompute else evomoe_workspace_bytes(shape)
            self.workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
            self.bal_loss = z(1, dtype=f32); self.bal_coef = z(E, dtype=f32)


def layer_forward(ctx, b: LayerBuffers, p: LayerParams, x, noise, tau, threshold, write_gate_w=True, top1=False):
    s = b.shape
    if top1:
        evomoe_dts_gate_top1(ctx, s, x, p.Wg, p.bg, noise, tau, b.gprime, b.gate_w if write_gate_w else None,
                             b.mask_bits, b.counts, b.k, b.block_hist)
    else:
        evomoe_dts_gate(ctx, s, x, p.Wg, p.bg, noise, tau, threshold, b.gprime, b.gate_w if write_gate_w else None,
                        b.mask_bits, b.counts, b.k, b.block_hist)
    evomoe_dispatch(ctx, s, b.mask_bits, b.gprime, b.expert_offsets, b.pair_token, b.pair_gate, b.tok_off,
                    b.tok_rows, b.num_pairs, block_hist=b.block_hist)
    evomoe_expert_ffn(ctx, s, x, b.pair_token, b.expert_offsets, p.W1, p.b1, p.W2, p.b2, b.H, b.A, b.O)
    evomoe_combine(ctx, s, b.O, b.pair_gate, b.tok_off, b.tok_rows, b.y)


def layer_backward(ctx, b: LayerBuffers, p: LayerParams, x, dy, tau, accumulate=False, balance_alpha=None,
                   recompute=False):
    """balance_alpha: also evaluate the balance loss and add its gradient in the gate backward (needs
    b.bal_loss [1] f32 and b.bal_coef [E] f32).  recompute: the FFN backward recomputes H and A (needs
    b.workspace of evomoe_workspace_bytes_recompute bytes); b.H and b.A are then not read."""
    s = b.shape
    evomoe_combine_bwd(ctx, s, dy, b.O, b.pair_gate, b.pair_token, b.expert_offsets, b.dO, b.dG_pairs)
    if recompute:
        evomoe_expert_ffn_bwd_recompute(ctx, s, b.dO, x, b.pair_token, b.expert_offsets, p.W1, p.b1, p.W2,
                                        dy, b.pair_gate, b.dW1, b.db1, b.dW2, b.db2, b.dXp, accumulate, b.workspace)
    else:
        evomoe_expert_ffn_bwd(ctx, s, b.dO, b.H, b.A, x, b.pair_token, b.expert_offsets, p.W1, p.W2,
                              dy, b.pair_gate, b.dW1, b.db1, b.dW2, b.db2, b.dXp, accumulate, b.workspace)
    evomoe_dispatch_bwd(ctx, s, b.dXp, b.tok_off, b.tok_rows, b.dx)
    if balance_alpha is not None:
        evomoe_balance_loss(ctx, s, b.gprime, b.counts, float(balance_alpha), b.bal_loss, b.bal_coef)
        evomoe_dts_gate_bwd_balance(ctx, s, b.dG_pairs, b.tok_off, b.tok_rows, b.gprime, b.mask_bits, tau, x, p.Wg,
                                    b.bal_coef, 1.0, b.dWg, b.dbg, b.dx, b.workspace)
    else:
        evomoe_dts_gate_bwd(ctx, s, b.dG_pairs, b.tok_off, b.tok_rows, b.gprime, b.mask_bits, tau, x, p.Wg,
                            b.dWg, b.dbg, b.dx, b.workspace)

"""evomoe_dispatch_static (the dispatch entry point that allocates nothing: its histogram table is a static
device array of the library) against evomoe_dispatch, through the C ABI: bit-identical outputs, twice in a row, the
second call on a smaller input (the shared table keeps the first call's contents)."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2112_14397_amd import binding as B

pytestmark = pytest.mark.gpu


def _masks(T, E, density, seed):
    rng = np.random.default_rng(seed)
    mask = rng.random((T, E)) < density
    mask[np.arange(T), rng.integers(0, E, T)] = True          # every token selects at least one expert
    bits = np.zeros(T, np.uint64)
    for e in range(E):
        bits |= mask[:, e].astype(np.uint64) << np.uint64(e)
    scores = rng.random((T, E), dtype=np.float32)
    return bits, scores, int(mask.sum())


def _run(entry, ctx, T, E, bits, scores, P_cap, x=None):
    """Calls the raw C symbol `entry` and returns every output as numpy arrays."""
    L = B.lib()
    shape = B.make_shape(T, 64, E, 64, "f32", "relu", P_cap)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    d_bits, d_scores = dev(bits.view(np.int64)), dev(scores)
    i32 = lambda n: torch.full((n,), -7, dtype=torch.int32, device="cuda")
    offs, ptok, toff, trows = i32(E + 1), i32(P_cap), i32(T + 1), i32(P_cap)
    pgate = torch.full((P_cap,), -7.0, dtype=torch.float32, device="cuda")
    npairs = torch.zeros(1, dtype=torch.int64, device="cuda")
    xp = torch.full((P_cap, 64), -7.0, dtype=torch.float32, device="cuda") if x is not None else None
    p = lambda t: None if t is None else ctypes.c_void_p(t.data_ptr())
    args = [ctx._h, ctypes.byref(shape), p(d_bits), p(d_scores), p(offs), p(ptok), p(pgate), p(toff), p(trows),
            p(npairs), p(x), p(xp)]
    if entry == "evomoe_dispatch":
        args.append(None)                                      # no block_hist: the call counts the table itself
    st = getattr(L, entry)(*args)
    assert st == B.EVOMOE_OK, (entry, st)
    torch.cuda.synchronize()
    out = [t.cpu().numpy() for t in (offs, ptok, pgate, toff, trows, npairs)]
    if xp is not None:
        out.append(xp.cpu().numpy())
    return out


def test_static_dispatch_matches_dispatch_twice_second_call_smaller():
    ctx = B.Context()
    for T, E, density, seed, with_x in ((40000, 37, 0.15, 11, True), (3000, 5, 0.5, 12, False)):
        bits, scores, P = _masks(T, E, density, seed)
        x = torch.from_numpy(np.random.default_rng(seed).standard_normal((T, 64)).astype(np.float32)).cuda() \
            if with_x else None
        want = _run("evomoe_dispatch", ctx, T, E, bits, scores, P + 9, x)
        got = _run("evomoe_dispatch_static", ctx, T, E, bits, scores, P + 9, x)
        assert int(got[5][0]) == P
        for a, b in zip(got, want):
            assert np.array_equal(a, b)


def test_static_dispatch_rejects_what_its_table_cannot_hold():
    ctx = B.Context()
    T, E = 256 * 1100, 64                                      # 1100 blocks x 64 experts > 65536 entries
    shape = B.make_shape(T, 64, E, 64, "f32", "relu", 1024)
    one = torch.zeros(16, dtype=torch.int64, device="cuda")
    p = ctypes.c_void_p(one.data_ptr())
    st = B.lib().evomoe_dispatch_static(ctx._h, ctypes.byref(shape), p, p, p, p, p, p, p, p, None, None)
    assert st == B.EVOMOE_ESTATIC and b"static" in B.lib().evomoe_status_string(st)

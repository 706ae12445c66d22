"""tensair_dasgd_apply_static (the entry point that allocates nothing: its index scratch is a fixed device
array inside the library) against tensair_dasgd_apply on the same inputs, through the C ABI.  Both run
the same kernels in the same order, so the tables must agree bit for bit; the existing entry point is
itself held to the oracle by test_gpu_parity.py.  Two calls in a row, the second with a smaller input
(the scratch keeps the first call's contents)."""
import numpy as np
import pytest
import torch

import oracle
from helpers import BF16_ULP, TOL_DELTA, TOL_TABLE, bf16_ulp_err, rel_l2
from paper_2211_10280_amd import binding as B

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


def _tables(V, D, stride, dtype, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(2):
        w = np.zeros((V, stride), np.float32)
        w[:, :D] = rng.standard_normal((V, D)).astype(np.float32) * 0.3
        t = torch.from_numpy(w).cuda()
        out.append(t.to(torch.bfloat16) if dtype == "bf16" else t)
    return out


def _host(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.cpu().numpy()


def _sources(rng, V, D, K):
    """own + K peers with a mix of sizes: empty, one row, sparse, dense, first and last row of the vocabulary"""
    bufs, host = [], []
    for k in range(K + 1):
        ui = [max(V // 3, 1), 0, 1, V // 7, V][k % 5]
        uo = [max(V // 4, 1), V, V // 2, 1, 0][k % 5]
        ids_in = np.sort(rng.choice(V, size=ui, replace=False)).astype(np.int32)
        ids_out = np.sort(rng.choice(V, size=uo, replace=False)).astype(np.int32)
        rows_in = (rng.standard_normal((ui, D)) * 0.1).astype(np.float32)
        rows_out = (rng.standard_normal((uo, D)) * 0.1).astype(np.float32)
        gb = B.GradBuffers(ui + 2, uo + 3, D)
        gb.load(ids_in, rows_in, ids_out, rows_out)
        bufs.append(gb)
        host.append(((ids_in, rows_in), (ids_out, rows_out)))
    return bufs, host


CALLS = [
    # V,         D,   stride, K,  dtype    first the larger input, then smaller ones on the same scratch
    (1_500_000, 32, 32, 15, "bf16"),      # close to the limits (2^21 rows, 15 peers)
    (70_001, 128, 128, 7, "f32"),
    (4_099, 300, 304, 3, "f32"),
    (63, 8, 8, 0, "bf16"),
]


def test_static_apply_equals_the_workspace_apply_on_consecutive_calls():
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    for V, D, stride, K, dtype in CALLS:
        _say("static apply", V, D, stride, K, dtype)
        rng = np.random.default_rng(V + K)
        ref_in, ref_out = _tables(V, D, stride, dtype, seed=K + 2)
        got_in, got_out = ref_in.clone(), ref_out.clone()
        orig_in, orig_out = _host(ref_in), _host(ref_out)
        bufs, host = _sources(rng, V, D, K)
        bd = B.F32 if dtype == "f32" else B.BF16
        m = B.Model(V, D, bd, 2, 3, 64, K, 1, np.ones(V, np.uint64), row_stride=stride, tables=(ref_in, ref_out))
        m.dasgd_apply(bufs[0], bufs[1:], 0.025)
        m.status()
        B.tensair_dasgd_apply_static(got_in, got_out, D, bufs[0], bufs[1:], 0.025, status=status)
        torch.cuda.synchronize()
        assert int(status.item()) == 0
        a_in, a_out, b_in, b_out = _host(got_in), _host(got_out), _host(ref_in), _host(ref_out)
        assert np.array_equal(a_in, b_in) and np.array_equal(a_out, b_out)
        assert (a_in != orig_in).any() and (a_out != orig_out).any()        # the update did something
        m.close()
        if V <= 100_000:      # and directly against the oracle, at the usual bars
            od = oracle.F32 if dtype == "f32" else oracle.BF16
            for got, orig, side in ((a_in, orig_in, 0), (a_out, orig_out, 1)):
                want = orig.copy()
                oracle.dasgd_apply_table(want, D, od, [h[side] for h in host], 0.025)
                if dtype == "bf16":
                    assert bf16_ulp_err(got, want, peak_bits=orig & 0x7FFF) <= BF16_ULP
                else:
                    assert rel_l2(got, want) <= TOL_TABLE
                    assert rel_l2(got.astype(np.float64) - orig, want.astype(np.float64) - orig) <= TOL_DELTA


def test_static_apply_without_own_gradient_and_with_bad_ids():
    V, D = 2_000, 16
    rng = np.random.default_rng(7)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    ref_in, ref_out = _tables(V, D, D, "f32", seed=1)
    got_in, got_out = ref_in.clone(), ref_out.clone()
    bufs, _ = _sources(rng, V, D, 2)
    m = B.Model(V, D, B.F32, 2, 3, 64, 2, 1, np.ones(V, np.uint64), tables=(ref_in, ref_out))
    m.dasgd_apply(None, bufs[1:], 0.1)                       # peers only
    m.status()
    B.tensair_dasgd_apply_static(got_in, got_out, D, None, bufs[1:], 0.1, status=status)
    torch.cuda.synchronize()
    assert torch.equal(got_in, ref_in) and torch.equal(got_out, ref_out) and int(status.item()) == 0
    # ids out of range and out of order: skipped safely, reported in the caller's status word
    bad = B.GradBuffers(8, 8, D)
    bad.load(np.array([5, 3, 9000], np.int32), np.ones((3, D), np.float32), np.array([1], np.int32),
             np.ones((1, D), np.float32))
    B.tensair_dasgd_apply_static(got_in, got_out, D, None, [bad], 0.1, status=status)
    torch.cuda.synchronize()
    assert int(status.item()) & 3 == 3
    # sizes beyond the fixed scratch are refused before anything is enqueued
    with pytest.raises(B.TensairError) as e:
        B.tensair_dasgd_apply_static(got_in, got_out, D, None, [bad] * (B.STATIC_MAX_PEERS + 1), 0.1)
    assert e.value.code == B.ECAPACITY
    m.close()

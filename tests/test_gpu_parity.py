"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element.

Integer results (negatives, unique row ids, segment offsets, row counts, initial tables) must be
bit-exact; fp32 gradient rows and tables within the tolerances of tests/helpers.py (tables 1e-4, their change
since the start 1e-3, rows 1e-4).  bf16 tables: a single application from identical inputs -- the apply tests and
every step of the teacher-forced runs -- within 2 ulp (of the element's own value at the configurations' step
size; of the larger of the old and the new value where a raised step size makes them cancel); free-running
chains of N steps within the chain bars of tests/helpers.py, with the strict distance printed beside them.
Inputs are seeded and synthetic (Zipf token streams); multi-step runs start from the fresh model of the
configuration and from adopted pre-trained tables."""
import functools

import numpy as np
import pytest
import torch

import oracle
from helpers import (BF16_CHAIN_FRAC, BF16_CHAIN_MAX, BF16_MSG_CHAIN_FRAC, BF16_MSG_CHAIN_MAX, BF16_ULP, FORCED_BEYOND, TOL_DELTA, TOL_LOSS, TOL_ROWS, TOL_TABLE, bf16_to_f32, bf16_ulp_err,
                     bf16_ulp_err_t, delta_rel_l2_t, rel_l2, rel_l2_t, rows_rel, to_dev, ulp_err_at_t, ulp_stats_t)
from oracle.driver import OracleWorker
from paper_2211_10280_amd import binding as B
import workload as W
from paper_2211_10280_amd.trainer import DasgdWorker

pytestmark = pytest.mark.gpu

DT = {"f32": (B.F32, oracle.F32, torch.float32, np.float32),
      "bf16": (B.BF16, oracle.BF16, torch.bfloat16, np.uint16)}


def _say(*a):
    print(*a, flush=True)


def _tables_to_dev(w_np, dtype):
    if dtype == "bf16":
        return torch.from_numpy(w_np.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(w_np).cuda()


def _tables_to_host(t, dtype):
    if dtype == "bf16":
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def _random_tables(V, D, stride, dtype, seed, scale=0.3):
    """'Pre-trained' tables as test data (both sides receive the same bits)."""
    if V * D > 50_000_000:       # large tables: drawn on the GPU (seeded), then handed to both sides
        gen = torch.Generator(device="cuda").manual_seed(seed)
        out = []
        for _ in range(2):
            t = torch.zeros((V, stride), device="cuda")
            t[:, :D] = torch.randn((V, D), device="cuda", generator=gen) * scale
            out.append(_tables_to_host(t.to(torch.bfloat16) if dtype == "bf16" else t, dtype))
        return out[0], out[1]
    rng = np.random.default_rng(seed)
    a = np.zeros((V, stride), np.float32)
    b = np.zeros((V, stride), np.float32)
    a[:, :D] = rng.standard_normal((V, D)).astype(np.float32) * scale
    b[:, :D] = rng.standard_normal((V, D)).astype(np.float32) * scale
    if dtype == "bf16":
        conv = lambda x: torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()
        return conv(a), conv(b)
    return a, b


# ------------------------------------------------------------------ init
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("V,D,stride", [(1000, 32, 32), (777, 300, 304), (64, 4, 8)])
def test_init_tables_bit_exact(dtype, V, D, stride):
    _say("init", dtype, V, D, stride)
    bd, od, _, _ = DT[dtype]
    counts = np.ones(V, np.uint64)
    m = B.Model(V, D, bd, 2, 5, 64, 0, 0x1234567890ABCDEF, counts, row_stride=stride)
    want_in, want_out = oracle.init_tables(V, D, stride, od, 0x1234567890ABCDEF)
    got_in, got_out = _tables_to_host(m.w_in, dtype), _tables_to_host(m.w_out, dtype)
    assert np.array_equal(got_in.view(np.uint8), want_in.view(np.uint8))
    assert np.array_equal(got_out.view(np.uint8), want_out.view(np.uint8))
    m.close()


# ------------------------------------------------------------------ alias table
@pytest.mark.parametrize("V,s", [(1000, 1.0), (50_000, 1.0), (300_000, 1.1)])
def test_alias_table_equals_oracle(V, s):
    _say("alias", V, s)
    tok = W.zipf_stream(V, s, 400_000, 11)
    counts = W.unigram_counts(tok, V)
    m = B.Model(V, 32, B.F32, 2, 5, 64, 0, 1, counts)
    thr, alias = m.alias()
    othr, oalias = oracle.alias_build(counts)
    assert np.array_equal(thr, othr) and np.array_equal(alias, oalias)
    m.close()


# ------------------------------------------------------------------ gradient calculation
GRAD_CASES = [
    # V,    D,   stride, T,     zipf, w, N,  B,    begin, dtype
    (1000, 32, 32, 10_000, 1.0, 2, 5, 64, 0, "f32"),            # stream start: clipped windows
    (1000, 32, 32, 10_000, 1.0, 2, 5, 16, 9_984, "f32"),        # last, partial batch at the stream end
    (5000, 300, 300, 40_000, 1.1, 5, 10, 512, 1024, "f32"),     # D=300: ragged second chunk pass
    (5000, 300, 320, 40_000, 1.1, 5, 10, 300, 777, "f32"),      # padded row stride
    (5000, 128, 128, 40_000, 1.0, 5, 5, 1024, 2048, "bf16"),
    (2000, 512, 512, 30_000, 1.05, 5, 10, 256, 4096, "bf16"),
    (200, 256, 256, 20_000, 1.5, 8, 15, 1024, 512, "f32"),      # hot rows: segments span many tiles
    (200, 64, 64, 40_000, 1.5, 8, 15, 2304, 512, "f32"),        # 18k tiles: hot rows chained through block partials
    (3, 64, 64, 5_000, 0.5, 3, 4, 700, 100, "f32"),             # three rows take everything
    (100_000, 1024, 1024, 30_000, 1.0, 2, 3, 64, 5, "f32"),     # widest row (4 chunk passes), 17 key bits
    (300, 4, 4, 2_000, 1.0, 1, 0, 128, 0, "f32"),               # narrowest row, no negatives
    (900, 520, 520, 6_000, 1.0, 2, 3, 96, 40, "bf16"),          # two full register sets + a tail of 8 elements
    (900, 772, 776, 6_000, 1.0, 2, 3, 96, 40, "f32"),           # three + a tail of 4, padded stride
    (900, 320, 320, 6_000, 1.0, 2, 3, 96, 40, "f32"),           # one + a full tail of 64
    (5_000_000, 8, 8, 50_000, 0.8, 4, 6, 2048, 3000, "f32"),    # 23 key bits: three radix passes
    # a steep word distribution over few words and 2^18 occurrences and more: long rows on both sides, with
    # rows held as one register set + tail at a padded stride, in bf16, and as two register sets + tail
    (150, 300, 320, 30_000, 1.5, 8, 15, 1024, 512, "f32"),
    (150, 512, 512, 30_000, 1.4, 8, 15, 1100, 300, "bf16"),
    (5000, 520, 520, 30_000, 1.5, 8, 15, 1024, 100, "f32"),
]


@pytest.mark.parametrize("case", GRAD_CASES, ids=lambda c: f"V{c[0]}_D{c[1]}_B{c[7]}_{c[9]}")
def test_sgns_grad_parity(case):
    _grad_parity(case)


@pytest.mark.parametrize("case", [
    (30, 32, 32, 5_000, 1.2, 3, 6, 200, 50, "f32"),             # a third of the draws collide
    (3, 64, 64, 5_000, 0.5, 3, 4, 700, 100, "f32"),             # three words: most second draws collide again
    (5000, 300, 300, 40_000, 1.1, 5, 10, 512, 1024, "f32"),
    (2000, 512, 512, 30_000, 1.05, 5, 10, 256, 4096, "bf16"),
], ids=lambda c: f"V{c[0]}_D{c[1]}_B{c[7]}_{c[9]}")
def test_sgns_grad_parity_with_resampled_negatives(case):
    """The variant in which a negative equal to the pair's center or context word is drawn once more."""
    _grad_parity(case, resample=True)


def _random_grad_cases(n, seed):
    """Seeded shapes: narrow to wide rows, windows 1..6, 0..12 negatives, batches from one center up, streams
    from flat to steep, vocabularies from two words up, batches at the start, inside and at the end of the
    stream."""
    rng = np.random.default_rng(seed)
    dims = [4, 8, 16, 36, 64, 100, 128, 132, 256, 260, 300, 384, 516, 1024]
    out = []
    for i in range(n):
        D = dims[(i * 5 + int(rng.integers(0, 2))) % len(dims)]
        V = int(rng.choice([2, 7, 100, 1500, 30_000, 70_000]))
        T = int(rng.integers(50, 6000))
        w, N = int(rng.integers(1, 7)), int(rng.integers(0, 13))
        Bc = int(rng.integers(1, max(2, min(T, 60_000 // (D // 4 + 8)))))
        Bc = min(Bc, T)
        begin = int(rng.choice([0, T - Bc, int(rng.integers(0, T - Bc + 1))]))
        out.append((V, D, D + 4 * int(rng.integers(0, 3)), T, float(rng.choice([0.6, 1.0, 1.4])), w, N, Bc, begin,
                    "bf16" if rng.integers(0, 2) else "f32"))
    return out


@pytest.mark.parametrize("case", _random_grad_cases(24, 2211_10280), ids=lambda c: "-".join(str(x) for x in c))
def test_sgns_grad_parity_random_shapes(case):
    _grad_parity(case)


def _grad_parity(case, resample=False):
    V, D, stride, T, zs, w, N, Bc, begin, dtype = case
    _say("grad case", case, "resampled negatives" if resample else "")
    bd, od, tdt, _ = DT[dtype]
    tok = W.zipf_stream(V, zs, T, 5)
    counts = W.unigram_counts(tok, V)
    Wi, Wo = _random_tables(V, D, stride, dtype, seed=V + D)
    d_in, d_out = _tables_to_dev(Wi, dtype), _tables_to_dev(Wo, dtype)
    m = B.Model(V, D, bd, w, N, Bc, 0, 0xC0FFEE, counts, worker_id=3, row_stride=stride, tables=(d_in, d_out),
                flags=B.RESAMPLE_NEGATIVES if resample else 0)
    thr, alias = oracle.alias_build(counts)
    og = oracle.sgns_grad(tok, w, N, begin, Bc, D, od, Wi, Wo, thr, alias, 0xC0FFEE, 3, 2, resample=resample)
    P = og.P
    if resample and V <= 30:      # the variant does something here
        pos, q = oracle.pairs(T, w, begin, Bc)
        assert (og.negatives != oracle.sample_negatives(V, thr, alias, 0xC0FFEE, 3, 2, pos, q, N)).any()
    assert m.pair_count(T, begin, Bc) == P

    dtok = torch.from_numpy(tok).cuda()
    g = m.grad_buffers(Bc)
    loss = torch.zeros(1, device="cuda")
    neg = torch.full((max(P * N, 1),), -1, dtype=torch.int32, device="cuda")
    seg_in = torch.full((g.cap_in + 1,), -1, dtype=torch.int32, device="cuda")
    seg_out = torch.full((g.cap_out + 1,), -1, dtype=torch.int32, device="cuda")
    m.sgns_grad(dtok, begin, Bc, 2, g, mean_loss=loss, negatives_dbg=neg, seg_offsets_in=seg_in,
                seg_offsets_out=seg_out)
    m.status()
    ui, uo = g.sizes()
    (ids_in, rows_in), (ids_out, rows_out) = g.to_host()
    # integers: bit-exact
    assert np.array_equal(neg.cpu().numpy()[: P * N].reshape(P, N), og.negatives)
    assert ui == og.gin.ids.size and uo == og.gout.ids.size
    assert np.array_equal(ids_in, og.gin.ids) and np.array_equal(ids_out, og.gout.ids)
    assert np.array_equal(seg_in.cpu().numpy()[: ui + 1], og.gin.seg.astype(np.int32))
    assert np.array_equal(seg_out.cpu().numpy()[: uo + 1], og.gout.seg.astype(np.int32))
    # floating point
    e_in, e_out = rows_rel(rows_in, og.gin.rows), rows_rel(rows_out, og.gout.rows)
    e_loss = abs(float(loss.item()) - og.loss) / og.loss
    _say(f"   P={P} U_in={ui} U_out={uo} rows_rel in={e_in:.2e} out={e_out:.2e} loss_rel={e_loss:.2e}")
    assert e_in <= TOL_ROWS and e_out <= TOL_ROWS and e_loss <= TOL_LOSS
    # the tables are read-only for the gradient calculation
    assert np.array_equal(_tables_to_host(d_in, dtype), Wi) and np.array_equal(_tables_to_host(d_out, dtype), Wo)
    m.close()


def test_sgns_grad_fresh_model_closed_form():
    """W_out = 0: loss is (N+1) ln 2 whatever the batch, every Gin row is exactly zero."""
    cfg = W.CONFIGS[1]
    tok, counts = W.make_stream(cfg)
    m = B.Model(cfg.vocab, cfg.dim, B.F32, cfg.window, cfg.negatives, cfg.batch, 0, cfg.seed, counts)
    g = m.grad_buffers()
    loss = torch.zeros(1, device="cuda")
    m.sgns_grad(torch.from_numpy(tok).cuda(), 640, 64, 0, g, mean_loss=loss)
    (ids_in, rows_in), _ = g.to_host()
    assert abs(loss.item() - 6 * np.log(2.0)) < 1e-5
    assert ids_in.size > 0 and not rows_in.any()
    m.close()


def test_empty_batches():
    V, D = 50, 8
    counts = np.ones(V, np.uint64)
    m = B.Model(V, D, B.F32, 2, 3, 16, 0, 1, counts)
    g = m.grad_buffers()
    g.n_rows.fill_(99)
    loss = torch.ones(1, device="cuda")
    tok1 = torch.zeros(1, dtype=torch.int32, device="cuda")
    m.sgns_grad(tok1, 0, 1, 0, g, mean_loss=loss)                 # one token: a center without context
    assert g.sizes() == (0, 0) and loss.item() == 0.0
    g.n_rows.fill_(99)
    tok = torch.arange(40, dtype=torch.int32, device="cuda")
    m.sgns_grad(tok, 7, 0, 0, g)                                  # zero centers
    assert g.sizes() == (0, 0)
    before = m.w_in.clone()
    m.dasgd_apply(g, [], 0.5)                                     # applying an empty gradient changes nothing
    m.status()
    assert torch.equal(before, m.w_in)
    # a step on a mini-batch without pairs: empty own gradient, empty message, tables untouched
    msg = m.packed_buffers()
    msg.n_rows.fill_(99)
    g.n_rows.fill_(99)
    m.step_packed(tok1, 0, 1, 0, [], 0.5, g, msg)
    m.step(tok1, 0, 1, 0, [], 0.5, g)
    m.status()
    assert g.sizes() == (0, 0) and msg.sizes() == (0, 0) and torch.equal(before, m.w_in)
    m.close()


# ------------------------------------------------------------------ gradient application
def _rand_sparse(rng, V, D, U):
    ids = np.sort(rng.choice(V, size=U, replace=False)).astype(np.int32)
    return ids, (rng.standard_normal((U, D)) * 0.1).astype(np.float32)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("V,D,stride,K,own", [(1000, 32, 32, 0, True), (4099, 300, 300, 3, True),
                                              (4099, 300, 320, 7, True), (70_001, 128, 128, 15, True),
                                              (513, 512, 512, 31, True), (2000, 64, 64, 4, False),
                                              (63, 8, 8, 2, True),
                                              # tables beyond 1 GiB: the variant that goes around the caches, rows
                                              # that do not end on cache-line borders, and rows padded to them
                                              (1_000_003, 300, 300, 2, True), (1_000_003, 300, 320, 2, True)])
def test_dasgd_apply_parity(dtype, V, D, stride, K, own):
    _apply_parity(dtype, V, D, stride, K, own)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("V,D,stride,K", [(70_001, 300, 320, 3), (20_011, 512, 512, 15), (4099, 132, 132, 0),
                                          (300_007, 1024, 1024, 1),
                                          # rows of at most 32 chunks: groups of 32 and of 16 lanes
                                          (70_001, 128, 128, 7), (50_000, 100, 104, 15), (20_011, 64, 64, 3),
                                          (30_000, 36, 36, 1)])
def test_dasgd_apply_parity_few_rows_of_a_large_vocabulary(dtype, V, D, stride, K):
    """Gradients that touch a few per cent of the vocabulary: the update then runs in its shape for sparse
    unions (more vocabulary rows per wave)."""
    _apply_parity(dtype, V, D, stride, K, True, thin=40)


def _random_apply_shapes(n, seed):
    """Seeded shapes off the beaten track: every lane grouping of the table update (D <= 32, <= 64, <= 128, one to
    four chunk passes of a whole wave), dimensions just below and above the borders between them, padded and
    dense rows, vocabularies that end inside a 64-row word, 0 to 15 peers."""
    rng = np.random.default_rng(seed)
    dims = [4, 8, 28, 32, 36, 60, 64, 68, 100, 124, 128, 132, 200, 252, 256, 260, 300, 508, 516, 768, 772, 1020, 1024]
    out = []
    for i in range(n):
        D = dims[(i * 7 + int(rng.integers(0, 3))) % len(dims)]
        V = int(rng.choice([1, 2, 63, 64, 65, 127, 500, 1000, 4097, 6001]))
        stride = D + 4 * int(rng.integers(0, 3))
        K = int(rng.integers(0, 16))
        out.append(("bf16" if rng.integers(0, 2) else "f32", V, D, stride, K, bool(rng.integers(0, 4))))
    return out


@pytest.mark.parametrize("dtype,V,D,stride,K,own", _random_apply_shapes(28, 20221118),
                         ids=lambda v: str(v))
def test_dasgd_apply_parity_random_shapes(dtype, V, D, stride, K, own):
    _apply_parity(dtype, V, D, stride, K, own)


def _apply_parity(dtype, V, D, stride, K, own, thin=1):
    _say("apply", dtype, V, D, stride, K, own, f"sizes / {thin}")
    bd, od, _, _ = DT[dtype]
    rng = np.random.default_rng(V * 31 + K)
    Wi, Wo = _random_tables(V, D, stride, dtype, seed=K + 1)
    d_in, d_out = _tables_to_dev(Wi, dtype), _tables_to_dev(Wo, dtype)
    m = B.Model(V, D, bd, 2, 3, 64, K, 1, np.ones(V, np.uint64), row_stride=stride, tables=(d_in, d_out))
    srcs_in, srcs_out, bufs = [], [], []
    for k in range(K + 1):
        # mix of sizes: empty, single row, dense, first/last row of the vocabulary
        Ui = [0, 1, V // 7, V // 2, V][k % 5] if k else max(V // 3, 1)
        Uo = [V, V // 2, 1, 0, V // 5][k % 5] if k else max(V // 4, 1)
        if thin > 1:
            Ui, Uo = (Ui + thin - 1) // thin, (Uo + thin - 1) // thin
        si, so = _rand_sparse(rng, V, D, Ui), _rand_sparse(rng, V, D, Uo)
        gb = B.GradBuffers(max(Ui, 1) + 3, max(Uo, 1) + 5, D)
        gb.load(si[0], si[1], so[0], so[1])
        bufs.append(gb)
        srcs_in.append(si)
        srcs_out.append(so)
    lr = 0.025
    if own:
        m.dasgd_apply(bufs[0], bufs[1:], lr)
    else:
        m.dasgd_apply(None, bufs[1:], lr)
        srcs_in, srcs_out = srcs_in[1:], srcs_out[1:]
    m.status()
    Oi, Oo = Wi.copy(), Wo.copy()
    oracle.dasgd_apply_table(Oi, D, od, srcs_in, lr)
    oracle.dasgd_apply_table(Oo, D, od, srcs_out, lr)
    for got_t, want, orig, srcs in ((d_in, Oi, Wi, srcs_in), (d_out, Oo, Wo, srcs_out)):
        got = _tables_to_host(got_t, dtype)
        touched = np.zeros(V, bool)
        for ids, _ in srcs:
            touched[ids] = True
        # rows outside the union and all padding: bit-identical to the input
        assert np.array_equal(got[~touched], orig[~touched])
        assert np.array_equal(got[:, D:], orig[:, D:])
        if dtype == "bf16":
            # in ulps of the larger of the old and the new value: where W and alpha * sum cancel (one element
            # in 10^8 or so is left with 10^-7 of its old magnitude) the fp32 sum's rounding, harmless against
            # the operands, is many ulps of the remainder
            d = bf16_ulp_err(got, want, peak_bits=orig & 0x7FFF)
            _say(f"   bf16 max ulp error {d}")
            assert d <= BF16_ULP
        else:
            e = rel_l2(got, want)
            ed = rel_l2(got.astype(np.float64) - orig, want.astype(np.float64) - orig)
            _say(f"   table rel {e:.2e} delta rel {ed:.2e}")
            assert e <= TOL_TABLE and ed <= TOL_DELTA
            assert np.abs(got - want).max() <= 4 * np.finfo(np.float32).eps * max(1.0, np.abs(want).max())
    m.close()


@pytest.mark.parametrize("V,D,stride,K", [(1000, 32, 32, 0), (4099, 300, 304, 7), (70, 1024, 1024, 2),
                                          (1_100_003, 300, 300, 3)])
def test_dasgd_apply_with_stochastic_rounding(V, D, stride, K):
    """The variant of the table update that rounds bf16 tables stochastically, two updates in a row (serial
    numbers 0 and 1).  Both sides take the decision from the fp32 value of W - alpha * sum and the same random
    bits; the GPU's fp32 sum and the oracle's double sum differ in the last bits of that value, so an element
    whose discarded bits plus random bits land within that distance of a carry (a few in 2^16) comes out one
    ulp apart: at most 1e-3 of the touched elements may differ, and by one ulp only (measured: 2e-7 of them)."""
    _say("apply with stochastic rounding", V, D, stride, K)
    rng = np.random.default_rng(V + K)
    seed = 0x5EED5EED5EED
    Wi, Wo = _random_tables(V, D, stride, "bf16", seed=K + 9)
    d_in, d_out = _tables_to_dev(Wi, "bf16"), _tables_to_dev(Wo, "bf16")
    m = B.Model(V, D, B.BF16, 2, 3, 64, K, seed, np.ones(V, np.uint64), row_stride=stride, tables=(d_in, d_out),
                flags=B.STOCHASTIC_ROUNDING)
    Oi, Oo = Wi.copy(), Wo.copy()
    for serial in range(2):
        srcs_in, srcs_out, bufs = [], [], []
        for k in range(K + 1):
            Ui = [V // 3, 1, V // 7, V // 2][k % 4]
            Uo = [V // 4, V // 2, 1, V // 5][k % 4]
            si, so = _rand_sparse(rng, V, D, Ui), _rand_sparse(rng, V, D, Uo)
            gb = B.GradBuffers(Ui + 3, Uo + 5, D)
            gb.load(si[0], si[1], so[0], so[1])
            bufs.append(gb)
            srcs_in.append(si)
            srcs_out.append(so)
        before = (Oi.copy(), Oo.copy())
        m.dasgd_apply(bufs[0], bufs[1:], 0.025)
        m.status()
        oracle.dasgd_apply_table(Oi, D, oracle.BF16, srcs_in, 0.025, stochastic=(seed, serial, 0))
        oracle.dasgd_apply_table(Oo, D, oracle.BF16, srcs_out, 0.025, stochastic=(seed, serial, 1))
        for got_t, want, orig, srcs in ((d_in, Oi, before[0], srcs_in), (d_out, Oo, before[1], srcs_out)):
            got = _tables_to_host(got_t, "bf16")
            touched = np.zeros(V, bool)
            for ids, _ in srcs:
                touched[ids] = True
            assert np.array_equal(got[~touched], orig[~touched]) and np.array_equal(got[:, D:], orig[:, D:])
            differ = got[touched][:, :D] != want[touched][:, :D]
            # in ulps of the larger of the old and the new value (see test_dasgd_apply_parity: cancellation)
            dist = bf16_ulp_err(got[touched], want[touched], peak_bits=orig[touched] & 0x7FFF)
            _say(f"   serial {serial}: {int(differ.sum())} of {differ.size} touched elements differ, largest distance {dist:.2f} ulp")
            assert differ.mean() <= 1e-3 and dist <= 1
            assert (got[touched] != orig[touched]).any()
        # carry on from the oracle's tables so that the second update starts from identical inputs
        d_in.copy_(_tables_to_dev(Oi, "bf16"))
        d_out.copy_(_tables_to_dev(Oo, "bf16"))
    m.close()
    # an fp32 model ignores the flag
    Fi, Fo = _random_tables(500, 16, 16, "f32", seed=3)
    res = []
    for flags in (0, B.STOCHASTIC_ROUNDING):
        a_in, a_out = _tables_to_dev(Fi, "f32"), _tables_to_dev(Fo, "f32")
        mm = B.Model(500, 16, B.F32, 2, 3, 64, 0, seed, np.ones(500, np.uint64), tables=(a_in, a_out), flags=flags)
        gb = B.GradBuffers(100, 100, 16)
        r2 = np.random.default_rng(1)
        si, so = _rand_sparse(r2, 500, 16, 100), _rand_sparse(r2, 500, 16, 100)
        gb.load(si[0], si[1], so[0], so[1])
        mm.dasgd_apply(gb, [], 0.1)
        mm.status()
        res.append((a_in.cpu().numpy(), a_out.cpu().numpy()))
        mm.close()
    assert np.array_equal(res[0][0], res[1][0]) and np.array_equal(res[0][1], res[1][1])


def test_apply_is_eq1_and_merged_equals_sequential():
    """K = 0 reproduces theta - alpha*g exactly (one fused multiply-add per element); merging K+1
    gradients equals applying them one message at a time up to fp32 rounding (Algorithm 1)."""
    V, D = 3000, 64
    rng = np.random.default_rng(5)
    Wi, Wo = _random_tables(V, D, D, "f32", seed=3)
    srcs = [(_rand_sparse(rng, V, D, 900), _rand_sparse(rng, V, D, 1200)) for _ in range(4)]
    bufs = []
    for si, so in srcs:
        gb = B.GradBuffers(900, 1200, D)
        gb.load(si[0], si[1], so[0], so[1])
        bufs.append(gb)
    lr = np.float32(0.025)
    a_in, a_out = _tables_to_dev(Wi, "f32"), _tables_to_dev(Wo, "f32")
    m = B.Model(V, D, B.F32, 2, 3, 64, 3, 1, np.ones(V, np.uint64), tables=(a_in, a_out))
    m.dasgd_apply(bufs[0], [], float(lr))
    want = Wi.copy()
    ids, rows = srcs[0][0]
    want[ids] = (Wi[ids].astype(np.float64) - np.float64(lr) * rows.astype(np.float64)).astype(np.float32)
    assert np.array_equal(a_in.cpu().numpy(), want)          # Eq. 1, exactly rounded
    for gb in bufs[1:]:
        m.dasgd_apply(gb, [], float(lr))                      # one apply_gradient per message
    b_in, b_out = _tables_to_dev(Wi, "f32"), _tables_to_dev(Wo, "f32")
    m.rebind(b_in, b_out, 0)
    m.dasgd_apply(bufs[0], bufs[1:], float(lr))               # merged
    m.status()
    assert rel_l2(b_in.cpu().numpy(), a_in.cpu().numpy()) < 1e-6
    assert rel_l2(b_out.cpu().numpy(), a_out.cpu().numpy()) < 1e-6
    m.close()


# ------------------------------------------------------------------ multi-step runs (train)
@functools.lru_cache(maxsize=2)
def _stream_cached(vocab, zipf_s, tokens, seed):
    tok = W.zipf_stream(vocab, zipf_s, tokens, seed)
    return tok, W.unigram_counts(tok, vocab)


def _stream(cfg):
    """W.make_stream(cfg), kept between the tests that use the same stream (100 M tokens take a while)."""
    return _stream_cached(cfg.vocab, cfg.zipf_s, cfg.tokens, cfg.stream_seed)


@functools.lru_cache(maxsize=1)
def _oracle_init_tables(V, D, dtype, seed):
    """The oracle's fresh model of a large configuration, made once for the tests that start from it (the
    oracle fills two tables of 10^9 elements in a quarter of a minute)."""
    return oracle.init_tables(V, D, D, oracle.F32 if dtype == "f32" else oracle.BF16, seed)


def _run_both(cfg, steps, threads=16, prefetch=True, bf16_messages=False, loose_bf16_chain=False,
              pretrained=None, forced=False, min_moved=None):
    """The same worker steps on the GPU (DasgdWorker) and in the oracle (OracleWorker), compared step by step
    (own gradient, loss, peers' row ids) and at the end (tables).

    pretrained: None = the fresh model of the configuration (W_out = 0: every logit is 0 at first and the
        W_in side of the gradient vanishes); a number = both sides adopt the same random tables of that scale
        (the paper's other start mode, a pre-trained model), so that the sigmoids leave 1/2 and both tables move.
    forced: teacher forcing -- before every step the GPU's tables are overwritten with the oracle's, so that
        every step starts from identical inputs and is held, alone, to the single-application bars
        (bf16: <= 2 ulp of the element's own value, outright; f32: <= 2 ulp of fp32).
    min_moved: smallest fraction of the touched elements (rows listed in any applied gradient x dim) that must
        have changed, per table -- a run in which nothing moves proves nothing."""
    tok, counts = _stream(cfg)
    tables = dev = None
    D = cfg.dim
    if pretrained is not None:
        # the oracle keeps dense rows; the GPU side gets the same values at the row pitch the trainer chooses
        # (every row on a 128-byte line: 320 elements for dim 300), padding columns zero
        tables = _random_tables(cfg.vocab, D, D, cfg.dtype, seed=100 + cfg.idx, scale=pretrained)
        stride = B.tensair_aligned_row_stride(D, DT[cfg.dtype][0])
        dev = []
        for w in tables:
            t = torch.zeros((cfg.vocab, stride), dtype=DT[cfg.dtype][2], device="cuda")
            t[:, :D] = to_dev(w)
            dev.append(t)
        dev = tuple(dev)
    gw = DasgdWorker(cfg, tok, counts, prefetch=prefetch, bf16_messages=bf16_messages, tables=dev)
    if tables is None and cfg.vocab * cfg.dim >= 1 << 28:
        tables = _oracle_init_tables(cfg.vocab, cfg.dim, cfg.dtype, cfg.seed)   # OracleWorker copies them
    ow = OracleWorker(cfg, tok, counts, threads=threads, bf16_messages=bf16_messages, tables=tables)
    w0 = (to_dev(ow.W_in), to_dev(ow.W_out))
    live = lambda: (gw.model.w_in[:, :D], gw.model.w_out[:, :D])        # the tables without their padding
    assert torch.equal(live()[0], w0[0]) and torch.equal(live()[1], w0[1])     # same initial model, bit for bit
    bf16 = cfg.dtype == "bf16"
    worst_rows = 0.0
    peak = [ow.W_in & 0x7FFF, ow.W_out & 0x7FFF] if bf16 and not forced else None
    touched = [np.zeros(cfg.vocab, bool), np.zeros(cfg.vocab, bool)]
    names = ("W_in", "W_out")
    for t in range(steps):
        if forced:
            before = (to_dev(ow.W_in), to_dev(ow.W_out))
            live()[0].copy_(before[0])
            live()[1].copy_(before[1])
        gw.step(want_loss=True)
        grads = ow.step()
        if peak is not None:
            np.maximum(peak[0], ow.W_in & 0x7FFF, out=peak[0])
            np.maximum(peak[1], ow.W_out & 0x7FFF, out=peak[1])
        for g in grads:
            touched[0][g.gin.ids] = True
            touched[1][g.gout.ids] = True
        og = grads[0]
        # per call: the own gradient
        (ids_in, rows_in), (ids_out, rows_out) = gw.own.to_host()
        assert np.array_equal(ids_in, og.gin.ids) and np.array_equal(ids_out, og.gout.ids), f"step {t}"
        e = max(rows_rel(rows_in, og.gin.rows), rows_rel(rows_out, og.gout.rows))
        worst_rows = max(worst_rows, e)
        assert abs(gw.mean_loss.item() - og.loss) <= TOL_LOSS * og.loss, f"step {t}"
        # peers: row ids bit-exact as well (they were computed on the GPU from the GPU's own snapshots)
        peer_side = gw.peer_bufs if cfg.grad_buffer == 1 else [p[0] for p in gw.peer_acc]
        for k, pg in enumerate(grads[1:]):
            pi, po = peer_side[k].ids_to_host()
            assert np.array_equal(pi, pg.gin.ids) and np.array_equal(po, pg.gout.ids), f"step {t} peer {k + 1}"
        if cfg.grad_buffer > 1 and (t + 1) % cfg.grad_buffer == 0:
            # the buffer this worker broadcasts: the sum of its last grad_buffer gradients
            (bi, br), (bo, bq) = gw.sent.to_host()
            assert np.array_equal(bi, ow.sent.gin.ids) and np.array_equal(bo, ow.sent.gout.ids), f"step {t}"
            worst_rows = max(worst_rows, rows_rel(br, ow.sent.gin.rows), rows_rel(bq, ow.sent.gout.rows))
        if forced:
            # this step alone, from identical inputs, against the bars of a single application
            for ti, (name, got_t, want) in enumerate(zip(names, live(), (ow.W_in, ow.W_out))):
                want_t = to_dev(want)
                st = ulp_stats_t(got_t, want_t, before[ti])
                at_max, _ = ulp_err_at_t(got_t, want_t, before[ti])
                _say(f"   step {t} {name}: {st['moved']} elements moved; distance in ulps of the value itself: max {st['max']}, "
                     f"{st['differ']:.2e} differ, {st['beyond2']:.2e} beyond 2; in ulps of the larger of old and new value: "
                     f"max {at_max:.2f}")
                if bf16:
                    # <= 2 ulp of the larger of the old and the new value, always; <= 2 ulp of the value itself,
                    # outright, at the configuration's own step size.  With a step size raised until a large part of
                    # the elements move, updates as large as the values occur by the million, and an element left
                    # with 2^-12 of its old magnitude by such a cancellation sees the rounding of the fp32 sum
                    # (2^-24 of the operands) as a whole ulp of its own: a few in 10^7 elements, bounded here
                    assert at_max <= BF16_ULP, f"step {t} {name}"
                    if cfg.lr == W.CONFIGS[cfg.idx].lr:
                        assert st["max"] <= BF16_ULP, f"step {t} {name}"
                    else:
                        assert st["beyond2"] <= FORCED_BEYOND, f"step {t} {name}"
                else:
                    e, ed = rel_l2_t(got_t, want_t), delta_rel_l2_t(got_t, want_t, before[ti])
                    _say(f"   step {t} {name}: table rel {e:.2e}, delta rel {ed:.2e}")
                    assert e <= TOL_TABLE and ed <= TOL_DELTA, f"step {t} {name}"
    gw.model.status()
    if bf16_messages and cfg.grad_buffer == 1:
        # the message this worker broadcast last: its own gradient rounded once -- the oracle's own gradient to
        # within the gradient's bar plus half a bfloat16 ulp (2^-9 of an element)
        (mi, mb_in), (mo, mb_out) = gw.own_msg.to_host()
        og = ow.last_own
        assert np.array_equal(mi, og.gin.ids) and np.array_equal(mo, og.gout.ids)
        e = max(rows_rel(oracle.grad_unpack_rows(mb_in), og.gin.rows), rows_rel(oracle.grad_unpack_rows(mb_out), og.gout.rows))
        _say(f"   own message against the oracle's own gradient: {e:.2e}")
        assert e <= 2.0 ** -8
    _say(f"   {cfg.name}: {steps} steps{' (teacher-forced)' if forced else ''}"
         f"{' from pre-trained tables' if pretrained is not None else ''}, worst own-gradient row error {worst_rows:.2e}")
    # bf16: once the two sides' tables differ by a rounding (<= 2 ulp is allowed), the gradients
    # computed from them differ by up to one bf16 ulp (2^-8) of their inputs
    assert worst_rows <= (TOL_ROWS if cfg.dtype == "f32" or forced else 2.0 ** -8)
    for full in (gw.model.w_in, gw.model.w_out):                       # the padding columns stay zero
        assert full.shape[1] == D or not full[:, D:].any().item()
    for ti, (got_t, want, name) in enumerate(((live()[0], ow.W_in, "W_in"), (live()[1], ow.W_out, "W_out"))):
        want_t = to_dev(want)
        st = ulp_stats_t(got_t, want_t, w0[ti])
        n_touched = int(touched[ti].sum()) * cfg.dim
        moved_frac = st["moved"] / max(n_touched, 1)
        _say(f"   {name}: {st['moved']} elements moved = {moved_frac:.3f} of the {n_touched} touched; strict distance to the "
             f"oracle: max {st['max']} ulp, {st['differ']:.2e} differ, {st['beyond2']:.2e} beyond 2 ulp")
        assert st["moved"] > 0
        if min_moved is not None:
            assert moved_frac >= min_moved, name
        if forced:
            continue                      # every step was held to the bar on its own
        if bf16:
            d, beyond, same = bf16_ulp_err_t(got_t, want_t, to_dev(peak[ti]))
            _say(f"   {name}: bf16 ulp error at the element's largest magnitude of the run: max {d:.2f}, "
                 f"fraction beyond {BF16_ULP} ulp {beyond:.2e}, bit-identical {same:.6f}")
            frac, most = ((BF16_MSG_CHAIN_FRAC, BF16_MSG_CHAIN_MAX) if (bf16_messages and cfg.peers) or loose_bf16_chain
                          else (BF16_CHAIN_FRAC, BF16_CHAIN_MAX))
            assert beyond <= frac and d <= most
        else:
            e = rel_l2_t(got_t, want_t)
            ed = delta_rel_l2_t(got_t, want_t, w0[ti])
            _say(f"   {name}: table rel {e:.2e}, delta rel {ed:.2e}")
            assert e <= TOL_TABLE and ed <= TOL_DELTA, name
    gw.model.close()
    return gw, ow


def test_train_config1_full_pass():
    """Tiny SGNS, all 157 mini-batches of one pass (the last has 16 centers), single worker."""
    _run_both(W.CONFIGS[1], 157, threads=1)


@pytest.mark.parametrize("name,kw,steps", [
    ("cfg2_small", dict(vocab=5_000, tokens=200_000, batch=256), 12),
    ("cfg3_small", dict(vocab=20_000, tokens=300_000, batch=256), 8),
    ("cfg4_small", dict(vocab=500, tokens=200_000, batch=1024), 4),
    ("cfg5_small", dict(vocab=20_000, tokens=300_000, batch=256), 5),
])
@pytest.mark.parametrize("prefetch", [True, False], ids=["prefetch", "inline"])
def test_train_scaled_configs(name, kw, steps, prefetch):
    """The shapes of configurations 2-5 (dim, window, negatives, peers, staleness, dtype) at a vocabulary
    and batch the oracle finishes in seconds; several radix/segment tiles and ragged tails.  Once with the
    next mini-batch prefetched after every step, once with every step self-contained."""
    base = W.CONFIGS[int(name[3])]
    _say("train", name, "prefetch" if prefetch else "inline")
    _run_both(base.scaled(name=name, **kw), steps, prefetch=prefetch)


@pytest.mark.parametrize("name,kw,steps,min_moved", [
    ("cfg2_small", dict(vocab=5_000, tokens=200_000, batch=256), 12, 0.9),
    ("cfg3_small", dict(vocab=20_000, tokens=300_000, batch=256), 8, 0.9),
    ("cfg4_small", dict(vocab=500, tokens=200_000, batch=1024), 4, 0.9),
    ("cfg5_small", dict(vocab=20_000, tokens=300_000, batch=256), 5, 0.005),
    # bf16 tables at the configuration's step size drop most updates (they are below half an ulp of the element):
    # the same chain with the step size raised until a tenth, and then most, of the touched elements move
    ("cfg5_small_lr0.25", dict(vocab=20_000, tokens=300_000, batch=256, lr=0.25), 5, 0.05),
    ("cfg5_small_lr2.5", dict(vocab=20_000, tokens=300_000, batch=256, lr=2.5), 5, 0.5),
])
def test_train_scaled_configs_from_pretrained_tables(name, kw, steps, min_moved):
    """The same shapes started from a pre-trained model (the paper's other start mode): the sigmoids are away
    from 1/2, both sides of the gradient are non-trivial and both tables move at every step."""
    base = W.CONFIGS[int(name[3])]
    _say("train from pre-trained tables", name)
    _run_both(base.scaled(name=name, **kw), steps, pretrained=0.25, min_moved=min_moved)


@pytest.mark.parametrize("name,kw,steps,min_moved", [
    ("cfg5_small", dict(vocab=20_000, tokens=300_000, batch=256), 6, 0.005),
    ("cfg5_small_lr2.5", dict(vocab=20_000, tokens=300_000, batch=256, lr=2.5), 6, 0.5),
    ("cfg5_small_lr25", dict(vocab=20_000, tokens=300_000, batch=256, lr=25.0), 6, 0.9),
    ("cfg3_small", dict(vocab=20_000, tokens=300_000, batch=256), 4, 0.9),
])
def test_train_scaled_configs_teacher_forced(name, kw, steps, min_moved):
    """Every step from the oracle's tables, each held alone to the bar of a single application."""
    base = W.CONFIGS[int(name[3])]
    _say("train teacher-forced", name)
    _run_both(base.scaled(name=name, **kw), steps, pretrained=0.25, forced=True, min_moved=min_moved)


@pytest.mark.parametrize("idx,n,steps", [(2, 2, 9), (3, 3, 7), (5, 2, 5)])
def test_train_with_gradient_buffer(idx, n, steps):
    """maxGradBuffer = n of Algorithm 1: every instance sums n gradients per broadcast, so the peers' sums
    arrive at every n-th step; tables, own gradients and the broadcast buffers against the oracle."""
    cfg = W.CONFIGS[idx].scaled(name=f"cfg{idx}_buf{n}", vocab=20_000, tokens=300_000, batch=256, grad_buffer=n)
    _say("train with gradient buffer", cfg.name)
    _run_both(cfg, steps)


@pytest.mark.parametrize("idx,steps", [(2, 50), (3, 20), (4, 20), (5, 5)])
def test_train_full_size_configs(idx, steps):
    """Configurations 2-5 at their full sizes, in the launch configuration the benchmark times, from the fresh
    model of the configurations."""
    _say("train full size", idx)
    _run_both(W.CONFIGS[idx], steps)


@pytest.mark.parametrize("idx,steps", [(2, 10), (3, 4), (4, 3)])
def test_train_full_size_configs_from_pretrained_tables(idx, steps):
    """The fp32 configurations at full size from a pre-trained model: nearly every touched element of both tables
    moves at every step."""
    _say("train full size from pre-trained tables", idx)
    _run_both(W.CONFIGS[idx], steps, pretrained=0.25, min_moved=0.9)


@pytest.mark.parametrize("lr,steps,min_moved", [(0.025, 3, None), (80.0, 2, 0.25)])
def test_train_config5_full_size_teacher_forced(lr, steps, min_moved):
    """Configuration 5 at full size from a pre-trained model, every step from the oracle's tables and held alone
    to 2 bf16 ulp: of the value itself at the configuration's step size; with the step size raised until most
    touched elements move (the same update per occurrence as 2.5 at the scaled size), of the larger of the old and
    the new value."""
    _say("train config 5 teacher-forced, lr", lr)
    _run_both(W.CONFIGS[5].scaled(lr=lr), steps, pretrained=0.25, forced=True, min_moved=min_moved)


@pytest.mark.parametrize("prefetch", [True, False], ids=["prefetch", "inline"])
def test_train_with_resampled_negatives(prefetch):
    """Training with the resampling variant on a vocabulary small enough for collisions in every mini-batch."""
    cfg = W.CONFIGS[2].scaled(name="cfg2_resample", vocab=400, tokens=100_000, batch=256, resample=True)
    _say("train with resampled negatives", cfg.name)
    _run_both(cfg, 8, prefetch=prefetch)


def test_train_with_stochastic_rounding():
    """Configuration 5's shape with the table update rounding the bf16 tables stochastically.  The two sides
    decide from fp32 values that differ by their own rounding noise, so about 1e-4 of the updated elements per
    step come out one ulp apart; the chain bars are those of the other variant whose decisions are taken from
    slightly different inputs (bf16 messages)."""
    cfg = W.CONFIGS[5].scaled(name="cfg5_stochastic", vocab=20_000, tokens=300_000, batch=256, stochastic_rounding=True)
    _say("train with stochastic rounding", cfg.name)
    _run_both(cfg, 5, loose_bf16_chain=True)


@pytest.mark.parametrize("idx,n,steps", [(2, 1, 9), (3, 1, 7), (3, 2, 6), (5, 1, 5)])
def test_train_with_bf16_messages(idx, n, steps):
    """The peers' gradients travel as bfloat16 messages (rounded once by the sender, after any summing in
    its buffer): tables and own gradients against the oracle driven the same way."""
    cfg = W.CONFIGS[idx].scaled(name=f"cfg{idx}_bf16msg_buf{n}", vocab=20_000, tokens=300_000, batch=256, grad_buffer=n)
    _say("train with bf16 messages", cfg.name)
    _run_both(cfg, steps, bf16_messages=True)


# ------------------------------------------------------------------ gradient buffer (gradients += gradient)
def _load_grad(m, rng, V, D, ui, uo, cap_pad=3):
    gi, go = _rand_sparse(rng, V, D, ui), _rand_sparse(rng, V, D, uo)
    buf = B.GradBuffers(ui + cap_pad, uo + cap_pad, D)
    buf.load(gi[0], gi[1], go[0], go[1])
    return buf, gi, go


@pytest.mark.parametrize("V,D,ua,ub", [(1000, 32, (40, 300), (25, 500)),      # overlapping
                                        (4099, 300, (0, 0), (17, 2100)),       # empty buffer + gradient (first +=)
                                        (4099, 300, (300, 4099), (299, 4099)), # every row of W_out in both
                                        (70, 1024, (1, 33), (69, 2)),          # widest row, V not a multiple of 64
                                        (200_000, 8, (5000, 120_000), (7000, 90_000))])   # several scan blocks
def test_grad_add_parity(V, D, ua, ub):
    _say("grad_add", V, D, ua, ub)
    rng = np.random.default_rng(V + D)
    m = B.Model(V, D, B.F32, 2, 3, 16, 0, 1, np.ones(V, np.uint64))
    a, a_in, a_out = _load_grad(m, rng, V, D, *ua)
    b, b_in, b_out = _load_grad(m, rng, V, D, *ub)
    out = B.GradBuffers(min(V, ua[0] + ub[0]) + 1, min(V, ua[1] + ub[1]) + 1, D)
    out.in_rows.fill_(float("nan"))
    out.out_rows.fill_(float("nan"))
    m.grad_add(a, b, out)
    m.status()
    (ids_in, rows_in), (ids_out, rows_out) = out.to_host()
    w_in = oracle.grad_add_rows(a_in, b_in, D)
    w_out = oracle.grad_add_rows(a_out, b_out, D)
    assert np.array_equal(ids_in, w_in[0]) and np.array_equal(ids_out, w_out[0])
    # one float addition per element, correctly rounded on both sides: bit-exact
    assert np.array_equal(rows_in, w_in[1]) and np.array_equal(rows_out, w_out[1])
    # the inputs are read-only
    assert np.array_equal(a.out_rows[: ua[1]].cpu().numpy(), a_out[1]) and a.sizes() == ua
    m.close()


def test_grad_add_of_real_gradients_and_errors():
    cfg = W.CONFIGS[3].scaled(name="cfg3_add", vocab=20_000, tokens=300_000, batch=256)
    tok, counts = W.make_stream(cfg)
    m = B.Model(cfg.vocab, cfg.dim, B.F32, cfg.window, cfg.negatives, cfg.batch, 1, cfg.seed, counts)
    dtok = torch.from_numpy(tok).cuda()
    g1, g2 = m.grad_buffers(), m.grad_buffers()
    # a table with non-zero W_out so that both sides of the gradient are non-trivial
    m.w_out.copy_(torch.from_numpy(_random_tables(cfg.vocab, cfg.dim, cfg.dim, "f32", 3)[1]).cuda())
    m.sgns_grad(dtok, 0, 256, 0, g1)
    m.sgns_grad(dtok, 256, 256, 0, g2)
    acc = B.GradBuffers(min(cfg.vocab, 2 * g1.cap_in), min(cfg.vocab, 2 * g1.cap_out), cfg.dim)
    m.grad_add(g1, g2, acc)
    m.status()
    (i1, r1), (o1, q1) = g1.to_host()
    (i2, r2), (o2, q2) = g2.to_host()
    (ia, ra), (oa, qa) = acc.to_host()
    wi, wo = oracle.grad_add_rows((i1, r1), (i2, r2), cfg.dim), oracle.grad_add_rows((o1, q1), (o2, q2), cfg.dim)
    assert np.array_equal(ia, wi[0]) and np.array_equal(oa, wo[0])
    assert np.array_equal(ra, wi[1]) and np.array_equal(qa, wo[1])
    assert ia.size < i1.size + i2.size and oa.size < o1.size + o2.size          # rows in common were merged
    # applying the sum = applying the parts in one merged update (Eq. 1 is linear), to float rounding
    w0_in, w0_out = m.w_in.clone(), m.w_out.clone()
    m.dasgd_apply(acc, [], 0.025)
    s_in, s_out = m.w_in.clone(), m.w_out.clone()
    m.w_in.copy_(w0_in)
    m.w_out.copy_(w0_out)
    m.dasgd_apply(g1, [g2], 0.025)
    assert (s_out - m.w_out).abs().max().item() <= 2e-7 * w0_out.abs().max().item()
    assert (s_in - m.w_in).abs().max().item() <= 2e-7 * w0_in.abs().max().item()
    # errors: shared buffers are refused; an output that is too small is cut off and reported
    with pytest.raises(B.TensairError) as e:
        m.grad_add(g1, g2, g1)
    assert e.value.code == B.EINVAL
    small = B.GradBuffers(4, 4, cfg.dim)
    m.grad_add(g1, g2, small)
    with pytest.raises(B.TensairError) as e:
        m.status()
    assert e.value.code == B.EDATA and small.sizes() == (4, 4)
    assert np.array_equal(small.out_ids.cpu().numpy(), wo[0][:4])
    m.status()
    m.close()


# ------------------------------------------------------------------ gradient messages in bfloat16
def _awkward_rows(rng, U, D):
    """Gradient-like rows salted with what rounding has to get right: ties on both sides of a power of two,
    the largest finite values, infinities, NaN, subnormals, signed zeros."""
    r = (rng.standard_normal((U, D)) * rng.choice([1e-30, 1e-6, 1e-2, 1.0, 1e20], (U, D))).astype(np.float32)
    special = np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 - 2.0 ** -9, -1 - 2.0 ** -8, 3.3895e38, 3.396e38, 3.4e38,
                        np.inf, -np.inf, np.nan, 0.0, -0.0, 1e-40, -1e-45, 2.0 ** -133], dtype=np.float32)
    flat = r.reshape(-1)
    at = rng.choice(flat.size, size=min(flat.size, 4 * special.size), replace=False)
    flat[at] = np.resize(special, at.size)
    return r


@pytest.mark.parametrize("V,D,ui,uo", [(1000, 32, 40, 300), (4099, 300, 0, 2100), (70, 1024, 1, 70),
                                       (50_000, 4, 0, 0), (300_000, 128, 4096, 250_000)])
def test_grad_pack_parity(V, D, ui, uo):
    """Bit-exact: counts, ids and every rounded element of the message."""
    _say("grad_pack", V, D, ui, uo)
    rng = np.random.default_rng(V + D + ui)
    m = B.Model(V, D, B.F32, 2, 3, 64, 0, 1, np.ones(V, np.uint64))
    gi = (np.sort(rng.choice(V, ui, replace=False)).astype(np.int32), _awkward_rows(rng, ui, D))
    go = (np.sort(rng.choice(V, uo, replace=False)).astype(np.int32), _awkward_rows(rng, uo, D))
    g = B.GradBuffers(ui + 2, uo + 3, D)
    g.load(gi[0], gi[1], go[0], go[1])
    msg = B.PackedBuffers(ui + 1, uo, D)
    msg.in_rows.fill_(0x1234)                                   # rows beyond n_rows are not written
    m.grad_pack(g, msg)
    m.status()
    assert msg.sizes() == (ui, uo)
    (ii, bi), (io, bo) = msg.to_host()
    assert np.array_equal(ii, gi[0]) and np.array_equal(io, go[0])
    assert np.array_equal(bi, oracle.grad_pack_rows(gi[1])) and np.array_equal(bo, oracle.grad_pack_rows(go[1]))
    assert (msg.in_rows[ui:].cpu().numpy() == 0x1234).all()
    m.close()


@pytest.mark.parametrize("K", [0, 3])
def test_step_packed_writes_the_own_gradient_as_a_message(K):
    """tensair_step_packed with own_msg_out: the message equals tensair_grad_pack of own_out bit for bit (and
    that one equals the oracle's rounding, test_grad_pack_parity), with and without peers; a message buffer
    that is too small is refused on the host."""
    cfg = W.CONFIGS[3].scaled(name="cfg3_msg", vocab=20_000, tokens=200_000, batch=300, peers=K)
    tok, counts = W.make_stream(cfg)
    dtok = torch.from_numpy(tok).cuda()
    m = B.Model(cfg.vocab, cfg.dim, B.F32, cfg.window, cfg.negatives, cfg.batch, K, cfg.seed, counts)
    m.w_out.copy_(m.w_in)
    peers = []
    for k in range(K):
        g = m.grad_buffers()
        m.sgns_grad(dtok, 1000 * (k + 1), cfg.batch, 0, g)
        msg = m.packed_buffers()
        m.grad_pack(g, msg)
        peers.append(msg)
    own, own_msg, ref = m.grad_buffers(), m.packed_buffers(), m.packed_buffers()
    own_msg.in_rows.fill_(0x1234)
    own_msg.out_rows.fill_(0x1234)
    m.step_packed(dtok, 5000, cfg.batch, 0, peers, cfg.lr, own, own_msg)
    m.grad_pack(own, ref)
    m.status()
    ui, uo = own.sizes()
    assert ui > 0 and uo > 0 and own_msg.sizes() == (ui, uo)
    (ai, ab), (ao, aq) = own_msg.to_host()
    (bi, bb), (bo, bq) = ref.to_host()
    assert np.array_equal(ai, bi) and np.array_equal(ao, bo) and np.array_equal(ab, bb) and np.array_equal(aq, bq)
    assert (own_msg.out_rows[uo:].cpu().numpy() == 0x1234).all()        # nothing beyond the rows that exist
    small = B.PackedBuffers(own.cap_in, own.cap_out - 1, cfg.dim)
    with pytest.raises(B.TensairError) as e:
        m.step_packed(dtok, 5000, cfg.batch, 0, peers, cfg.lr, own, small)
    assert e.value.code == B.ECAPACITY
    m.status()
    m.close()


def test_grad_pack_errors():
    V, D = 500, 16
    rng = np.random.default_rng(3)
    m = B.Model(V, D, B.F32, 2, 3, 64, 2, 1, np.ones(V, np.uint64))
    g, gi, go = _load_grad(m, rng, V, D, 30, 200)
    small = B.PackedBuffers(30, 150, D)                          # too few rows on the W_out side
    m.grad_pack(g, small)
    with pytest.raises(B.TensairError) as e:
        m.status()
    assert e.value.code == B.EDATA
    assert small.sizes() == (30, 150)
    (_, _), (io, bo) = small.to_host()
    assert np.array_equal(io, go[0][:150]) and np.array_equal(bo, oracle.grad_pack_rows(go[1][:150]))
    # a message whose source claims more rows than it holds is cut off at the capacity
    g.n_rows.copy_(torch.tensor([30, 10_000], dtype=torch.int32))
    big = B.PackedBuffers(64, 4000, D)
    m.grad_pack(g, big)
    with pytest.raises(B.TensairError):
        m.status()
    assert big.sizes() == (30, g.cap_out)
    # host-side refusals
    alias = B.PackedBuffers(30, 200, D)
    alias.c.out.row_ids = g.c.out.row_ids
    with pytest.raises(B.TensairError) as e:
        m.grad_pack(g, alias)
    assert e.value.code == B.EINVAL
    assert B.lib().tensair_grad_pack(m.h, None, None, None) == B.EINVAL
    assert B.lib().tensair_dasgd_apply_packed(m.h, None, None, 1, 0.1, None) == B.EINVAL
    with pytest.raises(B.TensairError) as e:                    # more peers than the model was made for
        m.dasgd_apply_packed(None, [small, small, small], 0.1)
    assert e.value.code == B.ECAPACITY
    m.status()
    m.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("V,D,stride,K,own,thin", [(1000, 32, 32, 1, True, 1), (4099, 300, 304, 7, True, 1),
                                              (513, 512, 512, 31, True, 1), (2000, 64, 64, 4, False, 1),
                                              (70, 1024, 1024, 2, True, 1), (1_000_003, 300, 300, 3, True, 1),
                                              # a few per cent of the rows touched: the shape for sparse unions
                                              (70_001, 300, 320, 7, True, 40), (20_011, 64, 64, 3, True, 40)])
def test_dasgd_apply_packed_parity(dtype, V, D, stride, K, own, thin):
    """Eq. 1 with the peers' gradients given as bfloat16 messages (the same bits on both sides), the own
    gradient in fp32."""
    _say("apply packed", dtype, V, D, stride, K, own, f"sizes / {thin}")
    bd, od, _, _ = DT[dtype]
    rng = np.random.default_rng(V * 17 + K)
    Wi, Wo = _random_tables(V, D, stride, dtype, seed=K + 5)
    d_in, d_out = _tables_to_dev(Wi, dtype), _tables_to_dev(Wo, dtype)
    m = B.Model(V, D, bd, 2, 3, 64, K, 1, np.ones(V, np.uint64), row_stride=stride, tables=(d_in, d_out))
    Ui, Uo = max(V // 3 // thin, 1), max(V // 4 // thin, 1)
    si, so = _rand_sparse(rng, V, D, Ui), _rand_sparse(rng, V, D, Uo)
    own_buf = B.GradBuffers(Ui + 3, Uo + 5, D)
    own_buf.load(si[0], si[1], so[0], so[1])
    srcs_in, srcs_out, msgs = [si], [so], []
    for k in range(1, K + 1):
        Ui = ([0, 1, V // 7, V // 2, V][k % 5] + thin - 1) // thin
        Uo = ([V, V // 2, 1, 0, V // 5][k % 5] + thin - 1) // thin
        pi, po = _rand_sparse(rng, V, D, Ui), _rand_sparse(rng, V, D, Uo)
        bi, bo = oracle.grad_pack_rows(pi[1]), oracle.grad_pack_rows(po[1])
        msg = B.PackedBuffers(max(Ui, 1) + 3, max(Uo, 1) + 5, D)
        msg.load(pi[0], bi, po[0], bo)
        msgs.append(msg)
        srcs_in.append((pi[0], oracle.grad_unpack_rows(bi)))
        srcs_out.append((po[0], oracle.grad_unpack_rows(bo)))
    lr = 0.025
    if own:
        m.dasgd_apply_packed(own_buf, msgs, lr)
    else:
        m.dasgd_apply_packed(None, msgs, lr)
        srcs_in, srcs_out = srcs_in[1:], srcs_out[1:]
    m.status()
    Oi, Oo = Wi.copy(), Wo.copy()
    oracle.dasgd_apply_table(Oi, D, od, srcs_in, lr)
    oracle.dasgd_apply_table(Oo, D, od, srcs_out, lr)
    for got_t, want, orig, srcs in ((d_in, Oi, Wi, srcs_in), (d_out, Oo, Wo, srcs_out)):
        got = _tables_to_host(got_t, dtype)
        touched = np.zeros(V, bool)
        for ids, _ in srcs:
            touched[ids] = True
        assert np.array_equal(got[~touched], orig[~touched])
        assert np.array_equal(got[:, D:], orig[:, D:])
        if dtype == "bf16":
            # in ulps of the larger of the old and the new value: where W and alpha * sum cancel (one element
            # in 10^8 or so is left with 10^-7 of its old magnitude) the fp32 sum's rounding, harmless against
            # the operands, is many ulps of the remainder
            d = bf16_ulp_err(got, want, peak_bits=orig & 0x7FFF)
            _say(f"   bf16 max ulp error {d}")
            assert d <= BF16_ULP
        else:
            e = rel_l2(got[:, :D], want[:, :D])
            ed = rel_l2(got[:, :D].astype(np.float64) - orig[:, :D], want[:, :D].astype(np.float64) - orig[:, :D])
            _say(f"   table rel {e:.2e}, delta rel {ed:.2e}")
            assert e <= TOL_TABLE and ed <= TOL_DELTA
    m.close()


# ------------------------------------------------------------------ dense apply, lookup, cosine difference
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n,K", [(1, 1), (7, 3), (4096, 0), (1_000_003, 8), (300 * 4099, 32),
                                 (2 ** 25 + 3, 8)])      # above 1 GiB in all: the variant that goes around the caches
def test_dense_apply_parity(dtype, n, K):
    """Eq. 1 on a dense model with K gradient blocks: fp32 within 1e-6 of the oracle's double sum (far inside
    the 1e-4 bar), bf16 within 2 ulp; K = 0 leaves theta alone."""
    _say("dense_apply", dtype, n, K)
    rng = np.random.default_rng(n + K)
    bd, od, tdt, _ = DT[dtype]
    th = rng.standard_normal(n).astype(np.float32)
    theta = th if dtype == "f32" else oracle._bf16_round(th.astype(np.float64))
    grads = [(rng.standard_normal(n) * 0.5).astype(np.float32) for _ in range(K)]
    d_theta = _tables_to_dev(theta.reshape(1, -1), dtype).reshape(-1)
    d_grads = [torch.from_numpy(g).cuda() for g in grads]
    B.tensair_dense_apply(d_theta, d_grads, 0.025)
    torch.cuda.synchronize()
    got = _tables_to_host(d_theta.reshape(1, -1), dtype).reshape(-1)
    want = oracle.dense_apply(theta.copy(), od, grads, 0.025)
    if K == 0:
        assert np.array_equal(got, theta)
    elif dtype == "f32":
        assert np.abs(got.astype(np.float64) - want).max() <= 1e-6 * max(1.0, np.abs(want).max())
        assert rel_l2(got, want) <= TOL_TABLE * 1e-2
    else:
        assert bf16_ulp_err(got, want, None) <= BF16_ULP
    for g, dg in zip(grads, d_grads):
        assert np.array_equal(dg.cpu().numpy(), g)


def test_dense_apply_errors():
    th = torch.zeros(64, device="cuda")
    g = torch.zeros(64, device="cuda")
    with pytest.raises(B.TensairError) as e:
        B.tensair_dense_apply(th, [g] * 33, 0.1)            # more blocks than the boundary takes
    assert e.value.code == B.ECAPACITY
    with pytest.raises(B.TensairError) as e:
        B.tensair_dense_apply(th[1:], [g[1:]], 0.1)         # not 16-byte aligned
    assert e.value.code == B.EINVAL


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("V,D,stride", [(1000, 32, 32), (4099, 300, 304), (70, 1024, 1024)])
def test_lookup_and_cosine_difference_parity(dtype, V, D, stride):
    _say("lookup/cosine", dtype, V, D, stride)
    bd, od, tdt, _ = DT[dtype]
    A, Bt = _random_tables(V, D, stride, dtype, seed=V), _random_tables(V, D, stride, dtype, seed=V + 1)[0]
    A_in, A_out = A
    # a few special rows: equal, opposite, zero in both, zero in one
    Bt[0] = A_in[0]
    Bt[1, :D] = (A_in[1, :D] ^ np.uint16(0x8000)) if dtype == "bf16" else -A_in[1, :D]
    A_in[2], Bt[2] = 0, 0
    Bt[3] = 0
    m = B.Model(V, D, bd, 2, 3, 16, 0, 1, np.ones(V, np.uint64), row_stride=stride,
                tables=(_tables_to_dev(A_in, dtype), _tables_to_dev(A_out, dtype)))
    rng = np.random.default_rng(V)
    ids = rng.integers(0, V, size=777).astype(np.int32)
    d_ids = torch.from_numpy(ids).cuda()
    for table, W_np in ((0, A_in), (1, A_out)):
        out = torch.full((ids.size, D), float("nan"), device="cuda")
        m.lookup(table, d_ids, out)
        m.status()
        assert np.array_equal(out.cpu().numpy(), oracle.lookup(W_np, od, D, ids))        # a copy: bit-exact
    # an id out of range: zeros and an error, no fault
    bad = torch.tensor([5, V, -1], dtype=torch.int32, device="cuda")
    out = torch.full((3, D), float("nan"), device="cuda")
    m.lookup(0, bad, out)
    with pytest.raises(B.TensairError) as e:
        m.status()
    assert e.value.code == B.EDATA and not out[1:].any().item()
    assert np.array_equal(out[0].cpu().numpy(), oracle.lookup(A_in, od, D, [5])[0])
    # cosine difference of the two tables
    diff = torch.full((V,), float("nan"), device="cuda")
    B.tensair_cosine_difference(m.w_in, _tables_to_dev(Bt, dtype), D, diff)
    torch.cuda.synchronize()
    want = oracle.cosine_difference(A_in, Bt, od, D)
    got = diff.cpu().numpy().astype(np.float64)
    _say(f"   cosine difference: max abs error {np.abs(got - want).max():.2e}, mean difference {want.mean():.4f}")
    assert np.abs(got - want).max() <= 2e-6
    assert got[0] <= 2e-6 and abs(got[1] - 2.0) <= 2e-6 and got[2] == 0.0 and got[3] == 1.0
    m.close()


# ------------------------------------------------------------------ prefetch of the coming mini-batch
def _grad_snapshot(g, loss=None, seg_in=None, seg_out=None):
    ui, uo = g.sizes()
    out = [ui, uo, g.in_ids[:ui].cpu().numpy().copy(), g.out_ids[:uo].cpu().numpy().copy(),
           g.in_rows[:ui].cpu().numpy().copy(), g.out_rows[:uo].cpu().numpy().copy()]
    if loss is not None:
        out.append(loss.cpu().numpy().copy())
    if seg_in is not None:
        out += [seg_in[: ui + 1].cpu().numpy().copy(), seg_out[: uo + 1].cpu().numpy().copy()]
    return out


def _same(a, b):
    return len(a) == len(b) and all(np.array_equal(x, y) for x, y in zip(a, b))


def test_prefetch_gives_the_same_bits():
    """tensair_prefetch only moves work in time: a gradient call that consumes it returns exactly what
    a call without it returns; a prefetch for another mini-batch is dropped."""
    V, D, T, w, N, Bc = 5000, 300, 40_000, 5, 10, 512
    tok = W.zipf_stream(V, 1.1, T, 5)
    counts = W.unigram_counts(tok, V)
    Wi, Wo = _random_tables(V, D, D, "f32", seed=11)
    m = B.Model(V, D, B.F32, w, N, Bc, 0, 77, counts, worker_id=2, tables=(_tables_to_dev(Wi, "f32"),
                                                                          _tables_to_dev(Wo, "f32")))
    dtok = torch.from_numpy(tok).cuda()
    g = m.grad_buffers()
    loss = torch.zeros(1, device="cuda")
    seg_in = torch.zeros(g.cap_in + 1, dtype=torch.int32, device="cuda")
    seg_out = torch.zeros(g.cap_out + 1, dtype=torch.int32, device="cuda")
    kw = dict(mean_loss=loss, seg_offsets_in=seg_in, seg_offsets_out=seg_out)

    def plain(begin, n, epoch):
        m.sgns_grad(dtok, begin, n, epoch, g, **kw)
        return _grad_snapshot(g, loss, seg_in, seg_out)

    ref_a, ref_b, ref_c = plain(1024, 512, 1), plain(1536, 300, 1), plain(0, 100, 0)
    for buf in (g.in_ids, g.out_ids, g.in_rows, g.out_rows, g.n_rows, seg_in, seg_out):
        buf.zero_()
    # consumed
    m.prefetch(dtok, 1024, 512, 1)
    assert _same(plain(1024, 512, 1), ref_a)
    # prefetched while the previous call is still in the queue, consumed by the next one, twice in a row
    m.prefetch(dtok, 1536, 300, 1)
    got_b = plain(1536, 300, 1)
    m.prefetch(dtok, 0, 100, 0)
    got_c = plain(0, 100, 0)
    assert _same(got_b, ref_b) and _same(got_c, ref_c)
    # not matching (other range, other epoch): dropped
    m.prefetch(dtok, 1536, 300, 1)
    assert _same(plain(1024, 512, 1), ref_a)
    m.prefetch(dtok, 1024, 512, 2)
    assert _same(plain(1024, 512, 1), ref_a)
    # two announcements consumed in order (the second is prepared during the first one's call); a third
    # replaces the second
    m.prefetch(dtok, 0, 100, 0)
    m.prefetch(dtok, 1024, 512, 2)
    m.prefetch(dtok, 1536, 300, 1)
    got_c = plain(0, 100, 0)
    got_b = plain(1536, 300, 1)
    assert _same(got_c, ref_c) and _same(got_b, ref_b)
    # a call for the second announcement while the first is waiting: both dropped
    m.prefetch(dtok, 0, 100, 0)
    m.prefetch(dtok, 1536, 300, 1)
    assert _same(plain(1536, 300, 1), ref_b)
    assert _same(plain(0, 100, 0), ref_c)
    # nothing to prepare (a batch without pairs), then a normal call
    one = torch.zeros(1, dtype=torch.int32, device="cuda")
    m.prefetch(one, 0, 1, 0)
    assert _same(plain(0, 100, 0), ref_c)
    # a call that wants the negatives takes the inline path even when its batch was prefetched
    P = m.pair_count(T, 1024, 512)
    neg = torch.full((P * N,), -1, dtype=torch.int32, device="cuda")
    m.prefetch(dtok, 1024, 512, 1)
    m.sgns_grad(dtok, 1024, 512, 1, g, negatives_dbg=neg, **kw)
    assert _same(_grad_snapshot(g, loss, seg_in, seg_out), ref_a) and int(neg.min()) >= 0
    # the worker id enters the negatives: a prefetch made under another id is not used
    m.prefetch(dtok, 1024, 512, 1)
    m.rebind(m.w_in, m.w_out, 3)
    other = plain(1024, 512, 1)
    m.rebind(m.w_in, m.w_out, 2)
    assert not _same(other, ref_a) and _same(plain(1024, 512, 1), ref_a)
    # argument errors as for the gradient call
    with pytest.raises(B.TensairError) as e:
        m.prefetch(dtok, T - 10, 20, 0)
    assert e.value.code == B.EINVAL
    with pytest.raises(B.TensairError) as e:
        m.prefetch(dtok, 0, Bc + 1, 0)
    assert e.value.code == B.ECAPACITY
    m.status()
    m.close()


@pytest.mark.parametrize("name,idx,kw", [
    ("cfg3_pf", 3, dict(vocab=20_000, tokens=300_000, batch=256)),
    ("cfg5_pf", 5, dict(vocab=20_000, tokens=300_000, batch=256)),
    # mini-batches above 2^20 occurrences are not prepared beside a step; with a long table update to follow
    # (wide rows, 15 peers) the one after the current is still prepared under that update ...
    ("cfg5_big_long_update", 5, dict(vocab=300_000, tokens=1_000_000, batch=12_000)),
    # ... and with a short one (narrow rows, 1 peer) every announcement is left to the consuming call
    ("cfg2_big_short_update", 2, dict(vocab=50_000, dim=32, tokens=1_000_000, batch=20_000, peers=1)),
])
def test_training_with_and_without_prefetch_is_bit_identical(name, idx, kw):
    """Several DASGD steps (peers, staleness) with the next mini-batch prefetched after every step against
    the same steps without: own gradients, losses and final tables agree bit for bit."""
    cfg = W.CONFIGS[idx].scaled(name=name, **kw)
    tok, counts = W.make_stream(cfg)
    a = DasgdWorker(cfg, tok, counts, prefetch=True)
    b = DasgdWorker(cfg, tok, counts, prefetch=False)
    for t in range(6):
        a.step(want_loss=True)
        b.step(want_loss=True)
        assert _same(_grad_snapshot(a.own, a.mean_loss), _grad_snapshot(b.own, b.mean_loss)), f"step {t}"
    a.model.status()
    b.model.status()
    for x, y in zip(a.tables_to_host(), b.tables_to_host()):
        assert np.array_equal(x, y)
    a.model.close()
    b.model.close()


def _same_on_device(a, b):
    """Own gradient and loss of two workers, compared where they are."""
    (ai, ao), (bi, bo) = a.own.sizes(), b.own.sizes()
    return ((ai, ao) == (bi, bo) and torch.equal(a.own.in_ids[:ai], b.own.in_ids[:bi])
            and torch.equal(a.own.out_ids[:ao], b.own.out_ids[:bo])
            and torch.equal(a.own.in_rows[:ai], b.own.in_rows[:bi])
            and torch.equal(a.own.out_rows[:ao], b.own.out_rows[:bo]) and torch.equal(a.mean_loss, b.mean_loss))


@pytest.mark.parametrize("idx,steps", [(1, 500), (2, 1000), (3, 200), (4, 60), (5, 16)])
def test_long_runs_with_and_without_prefetch_are_bit_identical(idx, steps):
    """The full-size configurations for many steps, two workers side by side on one stream: one announces every
    coming mini-batch (preparation on the library's second stream: under the table update, beside the forward
    pass, or left to the consuming call, as the configuration has it; index jobs riding in other launches, two
    sets of masks and workspaces taking turns), the other does not.  Anything that ran before what it depends
    on had finished would show as a difference in some step's gradient or in the final tables."""
    cfg = W.CONFIGS[idx]
    tok, counts = _stream(cfg)
    a = DasgdWorker(cfg, tok, counts, prefetch=True)
    b = DasgdWorker(cfg, tok, counts, prefetch=False)
    for t in range(steps):
        a.step(want_loss=True)
        b.step(want_loss=True)
        if t % 5 == 4 or t == steps - 1:
            assert _same_on_device(a, b), f"step {t}"
    a.model.status()
    b.model.status()
    assert torch.equal(a.model.w_in, b.model.w_in) and torch.equal(a.model.w_out, b.model.w_out)
    a.model.close()
    b.model.close()


@pytest.mark.parametrize("idx,steps,kw,bf16_messages", [
    (3, 60, {}, True), (5, 12, {}, True), (3, 61, dict(grad_buffer=3), False), (3, 40, dict(grad_buffer=2), True),
    (5, 12, dict(stochastic_rounding=True), False), (4, 30, dict(resample=True), False),
], ids=["cfg3_msg", "cfg5_msg", "cfg3_buffer3", "cfg3_buffer2_msg", "cfg5_stochastic", "cfg4_resample"])
def test_long_runs_of_the_variants_with_and_without_prefetch_are_bit_identical(idx, steps, kw, bf16_messages):
    """The same for the variants: gradients as bfloat16 messages, maxGradBuffer above one (with and without
    messages), stochastic rounding of bf16 tables, redrawn negatives."""
    cfg = W.CONFIGS[idx].scaled(**kw) if kw else W.CONFIGS[idx]
    tok, counts = _stream(cfg)
    a = DasgdWorker(cfg, tok, counts, prefetch=True, bf16_messages=bf16_messages)
    b = DasgdWorker(cfg, tok, counts, prefetch=False, bf16_messages=bf16_messages)
    for t in range(steps):
        a.step(want_loss=True)
        b.step(want_loss=True)
        if t % 5 == 4 or t == steps - 1:
            assert _same_on_device(a, b), f"step {t}"
    a.model.status()
    b.model.status()
    assert torch.equal(a.model.w_in, b.model.w_in) and torch.equal(a.model.w_out, b.model.w_out)
    a.model.close()
    b.model.close()


# ------------------------------------------------------------------ measurement aids
def test_streaming_probes_move_what_they_say():
    """The probes behind the bandwidth ceilings of the benchmark line: both copies reproduce their source, the
    three-reads-per-write probe writes the sum of its three source blocks, the read-only probe writes nothing
    beyond one chunk per workgroup."""
    n = 1 << 20                                             # floats per block (4 MiB), not a multiple of the grid
    n -= 12
    src = torch.randn(3 * n, device="cuda")
    for mode in (0, 1):
        dst = torch.zeros(n + 8, device="cuda")
        B.tensair_stream_probe(dst, src, 4 * n, mode)
        torch.cuda.synchronize()
        assert torch.equal(dst[:n], src[:n]) and not dst[n:].any().item()
    dst = torch.zeros(n + 8, device="cuda")
    B.tensair_stream_probe(dst, src, 4 * n, 3)
    torch.cuda.synchronize()
    assert torch.equal(dst[:n], (src[:n] + src[n:2 * n]) + src[2 * n:]) and not dst[n:].any().item()
    dst = torch.full((1 << 16,), 7.0, device="cuda")        # 256 KiB: the most the read-only probe may touch
    guard = dst.clone()
    B.tensair_stream_probe(dst, src, 4 * n, 2)
    torch.cuda.synchronize()
    blocks = min((n // 4 + 255) // 256, 256 * 64)
    assert torch.equal(dst[4 * blocks:], guard[4 * blocks:])
    with pytest.raises(B.TensairError):
        B.tensair_stream_probe(dst, src, 4 * n, 9)


# ------------------------------------------------------------------ error paths
def test_errors_are_reported_not_faults():
    V, D = 500, 16
    m = B.Model(V, D, B.F32, 2, 3, 32, 2, 1, np.ones(V, np.uint64))
    tok = torch.zeros(100, dtype=torch.int32, device="cuda")
    g = m.grad_buffers()
    with pytest.raises(B.TensairError) as e:
        m.sgns_grad(tok, 90, 20, 0, g)                       # runs past the stream
    assert e.value.code == B.EINVAL
    with pytest.raises(B.TensairError) as e:
        m.sgns_grad(tok, 0, 33, 0, g)                        # above max_centers
    assert e.value.code == B.ECAPACITY
    small = B.GradBuffers(4, 4, D)
    with pytest.raises(B.TensairError) as e:
        m.sgns_grad(tok, 0, 32, 0, small)                    # gradient buffers too small
    assert e.value.code == B.ECAPACITY
    with pytest.raises(B.TensairError) as e:
        m.dasgd_apply(g, [g, g, g], 0.1)                     # above max_peers
    assert e.value.code == B.ECAPACITY
    # a peer gradient with unsorted / out-of-range ids: skipped safely, reported by status
    bad = B.GradBuffers(8, 8, D)
    bad.load(np.array([5, 3, 900], np.int32), np.ones((3, D), np.float32), np.array([1], np.int32),
             np.ones((1, D), np.float32))
    m.dasgd_apply(None, [bad], 0.1)
    with pytest.raises(B.TensairError) as e:
        m.status()
    assert e.value.code == B.EDATA
    m.status()                                               # the status word was cleared
    m.close()

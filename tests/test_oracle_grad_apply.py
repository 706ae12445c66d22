"""Pins for the oracle's gradient calculation and gradient application (CPU only).

Each test checks the oracle against something other than itself: a closed form, a
hand-worked example, finite differences, a tensor library's autograd, a dense
brute-force accumulation, or an algebraic identity of Eq. 1."""
import math

import numpy as np
import pytest
import torch

import oracle


def _tiny(V=11, D=4, T=30, seed=0, dtype=oracle.F64, w_out_zero=False):
    rng = np.random.default_rng(seed)
    tok = rng.integers(0, V, size=T).astype(np.int32)
    counts = np.bincount(tok, minlength=V).astype(np.uint64)
    thr, alias = oracle.alias_build(counts)
    npdt = {oracle.F64: np.float64, oracle.F32: np.float32}[dtype]
    W_in = (rng.standard_normal((V, D)) * 0.5).astype(npdt)
    W_out = np.zeros((V, D), npdt) if w_out_zero else (rng.standard_normal((V, D)) * 0.5).astype(npdt)
    return tok, thr, alias, W_in, W_out


def _dense(sr, V):
    out = np.zeros((V, sr.rows64.shape[1]))
    out[sr.ids] = sr.rows64
    return out


# ------------------------------------------------------------------ closed forms
@pytest.mark.parametrize("N", [1, 5, 10, 15])
def test_loss_and_gradients_closed_form_when_w_out_is_zero(N):
    """All logits are 0: loss = (N+1) ln 2, Gin = 0, Gout[j] = (1/P) sum_occ (1/2 - label) v_c."""
    V, D, T, w = 13, 6, 40, 3
    tok, thr, alias, W_in, W_out = _tiny(V, D, T, seed=N, w_out_zero=True)
    g = oracle.sgns_grad(tok, w, N, 4, 9, D, oracle.F64, W_in, W_out, thr, alias, 11, 0, 0, want64=True)
    assert g.loss == pytest.approx((N + 1) * math.log(2.0), rel=1e-14)
    assert not g.gin.rows64.any()
    assert g.gin.ids.tolist() == sorted(set(tok[4:13].tolist()))       # listed although zero
    pos, q = oracle.pairs(T, w, 4, 9)
    want = np.zeros((V, D))
    for i, (p, qq) in enumerate(zip(pos, q)):
        o = qq - w if qq < w else qq - w + 1
        want[tok[p + o]] += (0.5 - 1.0) * W_in[tok[p]] / g.P
        for k in range(N):
            want[g.negatives[i, k]] += 0.5 * W_in[tok[p]] / g.P
    assert np.allclose(_dense(g.gout, V), want, rtol=1e-13, atol=1e-16)


def test_hand_worked_pair_d2():
    """v = (ln 3, 0), u_pos = (1, 7), u_neg = (0, 0), one pair, one negative:
    s_pos = ln 3, sigma = 3/4, g_pos = -1/4, g_neg = +1/2, loss = ln(4/3) + ln 2."""
    tok = np.array([0, 1], dtype=np.int32)           # center at position 0, context = token 1
    W_in = np.zeros((3, 2)); W_in[0] = (math.log(3.0), 0.0)
    W_out = np.zeros((3, 2)); W_out[1] = (1.0, 7.0)
    thr = np.full(3, 0xFFFFFFFF, np.uint32); alias = np.arange(3, dtype=np.int32)
    g = oracle.sgns_grad(tok, 1, 1, 0, 1, 2, oracle.F64, W_in, W_out, thr, alias, 0, 0, 0,
                         neg_override=np.array([[2]], np.int32), want64=True)
    assert g.P == 1
    assert g.loss == pytest.approx(math.log(4.0 / 3.0) + math.log(2.0), rel=1e-14)
    assert g.gin.ids.tolist() == [0]
    assert np.allclose(g.gin.rows64[0], [-0.25 * 1.0, -0.25 * 7.0], rtol=1e-14)
    assert g.gout.ids.tolist() == [1, 2]
    assert np.allclose(g.gout.rows64[0], [-0.25 * math.log(3.0), 0.0], rtol=1e-14)
    assert np.allclose(g.gout.rows64[1], [0.5 * math.log(3.0), 0.0], rtol=1e-14)
    assert g.gin.seg.tolist() == [0, 1] and g.gout.seg.tolist() == [0, 1, 2]


# ------------------------------------------------------------------ finite differences
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_gradient_by_central_finite_differences(seed):
    V, D, T, w, N = 11, 4, 30, 2, 3
    tok, thr, alias, W_in, W_out = _tiny(V, D, T, seed)
    begin, n = 5, 3
    base = oracle.sgns_grad(tok, w, N, begin, n, D, oracle.F64, W_in, W_out, thr, alias, 5, 0, 0, want64=True)
    neg = base.negatives.copy()
    # make sure the degenerate coincidences are exercised: a negative equal to its center and to its context
    pos, q = oracle.pairs(T, w, begin, n)
    o0 = q[0] - w if q[0] < w else q[0] - w + 1
    neg[0, 0] = tok[pos[0]]
    neg[0, 1] = tok[pos[0] + o0]
    base = oracle.sgns_grad(tok, w, N, begin, n, D, oracle.F64, W_in, W_out, thr, alias, 5, 0, 0,
                            neg_override=neg, want64=True)
    Gin, Gout = _dense(base.gin, V), _dense(base.gout, V)

    def loss(A, B):
        return oracle.sgns_grad(tok, w, N, begin, n, D, oracle.F64, A, B, thr, alias, 5, 0, 0,
                                neg_override=neg).loss

    h = 1e-5
    for (W, G, which) in ((W_in, Gin, 0), (W_out, Gout, 1)):
        fd = np.zeros_like(G)
        for r in range(V):
            for d in range(D):
                Wp, Wm = W.copy(), W.copy()
                Wp[r, d] += h
                Wm[r, d] -= h
                fd[r, d] = ((loss(Wp, W_out) - loss(Wm, W_out)) if which == 0
                            else (loss(W_in, Wp) - loss(W_in, Wm))) / (2 * h)
        assert np.allclose(fd, G, rtol=1e-7, atol=1e-9), which
        # rows the sparse form does not list have zero derivative
        listed = set((base.gin if which == 0 else base.gout).ids.tolist())
        for r in range(V):
            if r not in listed:
                assert not fd[r].any()


# ------------------------------------------------------------------ library autograd
def test_gradient_matches_autograd_of_the_sgns_loss():
    V, D, T, w, N = 40, 8, 120, 3, 5
    tok, thr, alias, W_in, W_out = _tiny(V, D, T, seed=7)
    begin, n = 10, 32
    g = oracle.sgns_grad(tok, w, N, begin, n, D, oracle.F64, W_in, W_out, thr, alias, 21, 2, 1, want64=True)
    pos, q = oracle.pairs(T, w, begin, n)
    off = np.where(q < w, q - w, q - w + 1)
    c = torch.from_numpy(tok[pos].astype(np.int64))
    x = torch.from_numpy(tok[pos + off].astype(np.int64))
    ng = torch.from_numpy(g.negatives.astype(np.int64))
    A = torch.tensor(W_in, requires_grad=True)
    B = torch.tensor(W_out, requires_grad=True)
    v = A[c]
    s_pos = (v * B[x]).sum(-1)
    s_neg = torch.einsum("pd,pnd->pn", v, B[ng])
    L = (torch.nn.functional.softplus(-s_pos) + torch.nn.functional.softplus(s_neg).sum(-1)).mean()
    L.backward()
    assert g.loss == pytest.approx(float(L.detach()), rel=1e-12)
    assert np.allclose(_dense(g.gin, V), A.grad.numpy(), rtol=1e-10, atol=1e-14)
    assert np.allclose(_dense(g.gout, V), B.grad.numpy(), rtol=1e-10, atol=1e-14)


# ------------------------------------------------------------------ duplicates / sparse form
@pytest.mark.parametrize("hot", [False, True])
def test_sparse_form_against_dense_brute_force(hot):
    V, D, T, w, N = 9, 3, 50, 4, 6
    tok, thr, alias, W_in, W_out = _tiny(V, D, T, seed=3)
    if hot:
        tok[:] = 4                                   # every center and context is the same row
        thr, alias = oracle.alias_build(np.bincount(tok, minlength=V).astype(np.uint64))
    g = oracle.sgns_grad(tok, w, N, 0, T, D, oracle.F64, W_in, W_out, thr, alias, 8, 0, 0, want64=True)
    pos, q = oracle.pairs(T, w, 0, T)
    Gin, Gout = np.zeros((V, D)), np.zeros((V, D))
    occ_in, occ_out = np.zeros(V, np.int64), np.zeros(V, np.int64)
    for i, (p, qq) in enumerate(zip(pos, q)):
        o = qq - w if qq < w else qq - w + 1
        c = tok[p]
        occ_in[c] += 1
        for k, j in enumerate([tok[p + o]] + g.negatives[i].tolist()):
            s = float(W_in[c] @ W_out[j])
            gg = (1.0 / (1.0 + math.exp(-s)) - (1.0 if k == 0 else 0.0)) / len(pos)
            Gin[c] += gg * W_out[j]
            Gout[j] += gg * W_in[c]
            occ_out[j] += 1
    for sr, G, occ in ((g.gin, Gin, occ_in), (g.gout, Gout, occ_out)):
        assert sr.ids.tolist() == np.nonzero(occ)[0].tolist()            # ascending unique = nonzero bins
        assert sr.seg.tolist() == np.concatenate([[0], np.cumsum(occ[occ > 0])]).tolist()
        assert np.allclose(_dense(sr, V), G, rtol=1e-12, atol=1e-15)
    assert g.gout.seg[-1] == len(pos) * (N + 1) and g.gin.seg[-1] == len(pos)
    if hot:
        assert g.gin.ids.tolist() == [4]
    # float export is the rounded double accumulator
    assert np.array_equal(g.gout.rows, g.gout.rows64.astype(np.float32))


def test_empty_batch():
    tok, thr, alias, W_in, W_out = _tiny()
    g = oracle.sgns_grad(tok, 2, 3, 5, 0, 4, oracle.F64, W_in, W_out, thr, alias, 1, 0, 0)
    assert g.P == 0 and g.gin.ids.size == 0 and g.gout.ids.size == 0 and g.loss == 0.0
    # a single-token stream has a center but no context
    g = oracle.sgns_grad(np.array([3], np.int32), 2, 3, 0, 1, 4, oracle.F64, W_in, W_out, thr, alias, 1, 0, 0)
    assert g.P == 0


# ------------------------------------------------------------------ apply (Eq. 1)
def _rand_sparse(rng, V, D, U):
    ids = np.sort(rng.choice(V, size=U, replace=False)).astype(np.int32)
    return ids, rng.standard_normal((U, D)).astype(np.float32)


def test_apply_is_eq1_for_a_single_gradient():
    rng = np.random.default_rng(0)
    V, D = 50, 6
    W = rng.standard_normal((V, D)).astype(np.float32)
    W0 = W.copy()
    ids, rows = _rand_sparse(rng, V, D, 17)
    lr = 0.025
    oracle.dasgd_apply_table(W, D, oracle.F32, [(ids, rows)], lr)
    want = W0.copy()
    want[ids] = (W0[ids].astype(np.float64) - float(np.float32(lr)) * rows.astype(np.float64)).astype(np.float32)
    assert np.array_equal(W, want)
    untouched = np.setdiff1d(np.arange(V), ids)
    assert np.array_equal(W[untouched].view(np.uint32), W0[untouched].view(np.uint32))


def test_apply_respects_row_stride_padding():
    rng = np.random.default_rng(1)
    V, D, S = 20, 5, 8
    W = rng.standard_normal((V, S)).astype(np.float32)
    W0 = W.copy()
    ids, rows = _rand_sparse(rng, V, D, 9)
    oracle.dasgd_apply_table(W, D, oracle.F32, [(ids, rows)], 0.5)
    assert np.array_equal(W[:, D:], W0[:, D:])
    assert not np.array_equal(W[ids, :D], W0[ids, :D])


def test_merged_apply_equals_sequential_applies_and_ignores_peer_order():
    rng = np.random.default_rng(2)
    V, D, K = 80, 7, 5
    W0 = rng.standard_normal((V, D))
    srcs = [_rand_sparse(rng, V, D, int(rng.integers(1, 40))) for _ in range(K + 1)]
    merged = W0.copy()
    oracle.dasgd_apply_table(merged, D, oracle.F64, srcs, 0.025)
    seq = W0.copy()
    for s in srcs:                                       # Algorithm 1: one apply_gradient per message
        oracle.dasgd_apply_table(seq, D, oracle.F64, [s], 0.025)
    assert np.allclose(merged, seq, rtol=1e-14, atol=1e-15)
    perm = W0.copy()
    oracle.dasgd_apply_table(perm, D, oracle.F64, [srcs[0]] + srcs[:0:-1], 0.025)
    assert np.allclose(merged, perm, rtol=1e-15, atol=1e-16)
    # summed, not averaged: two copies of one gradient move the row twice as far
    a, b = W0.copy(), W0.copy()
    oracle.dasgd_apply_table(a, D, oracle.F64, [srcs[0]], 0.025)
    oracle.dasgd_apply_table(b, D, oracle.F64, [srcs[0], srcs[0]], 0.025)
    i = srcs[0][0]
    assert np.allclose(b[i] - W0[i], 2 * (a[i] - W0[i]), rtol=1e-12)


@pytest.mark.parametrize("dtype", [oracle.F32, oracle.BF16])
def test_apply_then_unapply_restores_within_rounding(dtype):
    rng = np.random.default_rng(4)
    V, D = 60, 8
    Wf = (rng.standard_normal((V, D)) * 0.1).astype(np.float32)
    if dtype == oracle.BF16:
        W = torch.from_numpy(Wf).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()
    else:
        W = Wf.copy()
    W0 = W.copy()
    ids, rows = _rand_sparse(rng, V, D, 25)
    oracle.dasgd_apply_table(W, D, dtype, [(ids, rows)], 0.025)
    assert not np.array_equal(W, W0)
    W1 = W.copy()
    oracle.dasgd_apply_table(W, D, dtype, [(ids, -rows)], 0.025)

    def val(a):
        return (a.astype(np.float64) if dtype == oracle.F32 else oracle.bf16_to_f32(a).astype(np.float64))

    def ulp(a):
        bits = 23 if dtype == oracle.F32 else 7
        return 2.0 ** (np.floor(np.log2(np.maximum(np.abs(val(a)), 1e-30))) - bits)

    # two roundings, each at most half a unit in the last place of the value it produced:
    # floating-point subtraction is not invertible, so "restores" can only mean this bound
    assert np.all(np.abs(val(W) - val(W0)) <= 0.5 * (ulp(W1) + ulp(W)) * (1 + 1e-12))
    # exact when every intermediate is representable: table on a 2^-4 grid, update 2^-3
    Wg = (rng.integers(-32, 33, size=(V, D)) / 16.0).astype(np.float32)
    W = (torch.from_numpy(Wg).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()
         if dtype == oracle.BF16 else Wg.copy())
    W0 = W.copy()
    rows2 = np.full_like(rows, 0.5)
    oracle.dasgd_apply_table(W, D, dtype, [(ids, rows2)], 0.25)
    assert np.array_equal(val(W)[ids], val(W0)[ids] - 0.125)
    oracle.dasgd_apply_table(W, D, dtype, [(ids, -rows2)], 0.25)
    assert np.array_equal(W, W0)


def test_bf16_apply_rounds_once_from_the_exact_sum():
    """Three gradients whose individual updates are each below half a bf16 ulp move the row
    when summed first (fp32-accumulated, rounded once) -- K+1 separate roundings would not."""
    W = np.array([[0x3F80]], dtype=np.uint16)                    # 1.0; ulp above = 2^-7
    g = np.array([[-(2.0 ** -9) * 1.1]], dtype=np.float32)       # update +0.275 ulp each at lr = 1
    ids = np.array([0], np.int32)
    one = W.copy()
    oracle.dasgd_apply_table(one, 1, oracle.BF16, [(ids, g)], 1.0)
    assert one[0, 0] == 0x3F80
    three = W.copy()
    oracle.dasgd_apply_table(three, 1, oracle.BF16, [(ids, g)] * 3, 1.0)
    assert three[0, 0] == 0x3F81


def test_single_worker_step_is_minibatch_sgd():
    """With one rank the update is plain synchronous SGD (Section 4.1): one oracle step equals
    theta - alpha * autograd gradient of the batch-mean loss."""
    V, D, T, w, N = 30, 5, 80, 2, 4
    tok, thr, alias, W_in, W_out = _tiny(V, D, T, seed=9)
    g = oracle.sgns_grad(tok, w, N, 0, 16, D, oracle.F64, W_in, W_out, thr, alias, 3, 0, 0)
    A, B = W_in.copy(), W_out.copy()
    oracle.dasgd_apply(A, B, D, oracle.F64, [g], 0.025)
    pos, q = oracle.pairs(T, w, 0, 16)
    off = np.where(q < w, q - w, q - w + 1)
    tA = torch.tensor(W_in, requires_grad=True)
    tB = torch.tensor(W_out, requires_grad=True)
    v = tA[torch.from_numpy(tok[pos].astype(np.int64))]
    sp = (v * tB[torch.from_numpy(tok[pos + off].astype(np.int64))]).sum(-1)
    sn = torch.einsum("pd,pnd->pn", v, tB[torch.from_numpy(g.negatives.astype(np.int64))])
    (torch.nn.functional.softplus(-sp) + torch.nn.functional.softplus(sn).sum(-1)).mean().backward()
    lr = float(np.float32(0.025))
    # the sparse gradient crosses the interface as float32, hence the 1e-7 relative slack
    assert np.allclose(A, W_in - lr * tA.grad.numpy(), rtol=0, atol=2e-8)
    assert np.allclose(B, W_out - lr * tB.grad.numpy(), rtol=0, atol=2e-8)


# ------------------------------------------------------------------ gradient buffer (Algorithm 1: gradients += gradient)
def _rand_rows(rng, V, D, U, zero_rows=0):
    ids = np.sort(rng.choice(V, size=U, replace=False)).astype(np.int32)
    rows = rng.standard_normal((U, D)).astype(np.float32)
    rows[:zero_rows] = 0.0
    return ids, rows


def test_grad_add_is_the_dense_sum_on_the_union():
    """Brute force: scatter both lists into a dense [V, D] table with a 'listed' flag per row."""
    rng = np.random.default_rng(5)
    V, D = 37, 3
    for ua, ub in ((0, 0), (0, 5), (7, 0), (9, 11), (37, 37), (1, 1)):
        a = _rand_rows(rng, V, D, ua, zero_rows=min(2, ua))
        b = _rand_rows(rng, V, D, ub)
        dense = [[0.0] * D for _ in range(V)]
        listed = [False] * V
        for ids, rows in (a, b):
            for i, r in enumerate(ids):
                listed[r] = True
                for d in range(D):
                    dense[r][d] += float(rows[i, d])
        ids, rows = oracle.grad_add_rows(a, b, D)
        want_ids = [r for r in range(V) if listed[r]]
        assert ids.dtype == np.int32 and rows.dtype == np.float32
        assert ids.tolist() == want_ids                      # a row listed with a zero gradient stays listed
        for i, r in enumerate(want_ids):
            assert rows[i].tolist() == [float(np.float32(x)) for x in dense[r]]


def test_grad_add_identities():
    rng = np.random.default_rng(6)
    V, D = 500, 8
    a, b = _rand_rows(rng, V, D, 120), _rand_rows(rng, V, D, 200)
    empty = (np.zeros(0, np.int32), np.zeros((0, D), np.float32))
    ids, rows = oracle.grad_add_rows(a, empty, D)
    assert np.array_equal(ids, a[0]) and np.array_equal(rows, a[1])           # a + nothing = a
    ab, ba = oracle.grad_add_rows(a, b, D), oracle.grad_add_rows(b, a, D)
    assert np.array_equal(ab[0], ba[0]) and np.array_equal(ab[1], ba[1])      # commutative, bit for bit
    assert np.array_equal(ab[0], np.union1d(a[0], b[0]))
    both = np.intersect1d(a[0], b[0])
    assert both.size > 0
    r = both[0]
    want = a[1][np.searchsorted(a[0], r)] + b[1][np.searchsorted(b[0], r)]    # float32 add is correctly rounded
    assert np.array_equal(ab[1][np.searchsorted(ab[0], r)], want)
    aa = oracle.grad_add_rows(a, a, D)
    assert np.array_equal(aa[1], 2 * a[1])                                    # doubling is exact


def test_applying_a_summed_gradient_is_applying_its_parts():
    """Eq. 1 is linear in the gradient: one application of a + b moves the table like the merged
    application of a and b (up to the float rounding of the sum; exactly on a dyadic grid)."""
    rng = np.random.default_rng(7)
    V, D = 300, 4
    W0 = rng.standard_normal((V, D)).astype(np.float32)
    a, b = _rand_rows(rng, V, D, 90), _rand_rows(rng, V, D, 140)
    s = oracle.grad_add_rows(a, b, D)
    W1, W2 = W0.copy(), W0.copy()
    oracle.dasgd_apply_table(W1, D, oracle.F32, [s], 0.025)
    oracle.dasgd_apply_table(W2, D, oracle.F32, [a, b], 0.025)
    assert np.abs(W1 - W2).max() <= 2e-7 * np.abs(W0).max() and not np.array_equal(W1, W0)
    untouched = np.setdiff1d(np.arange(V), s[0])
    assert np.array_equal(W1[untouched], W0[untouched])
    # dyadic grid: every product and sum is exact, so the two ways agree bit for bit
    Wd = (rng.integers(-64, 64, (V, D)) / 8.0).astype(np.float32)
    ad = (a[0], (rng.integers(-16, 16, a[1].shape) / 4.0).astype(np.float32))
    bd = (b[0], (rng.integers(-16, 16, b[1].shape) / 4.0).astype(np.float32))
    W1, W2 = Wd.copy(), Wd.copy()
    oracle.dasgd_apply_table(W1, D, oracle.F32, [oracle.grad_add_rows(ad, bd, D)], 0.5)
    oracle.dasgd_apply_table(W2, D, oracle.F32, [ad, bd], 0.5)
    assert np.array_equal(W1, W2)


# ------------------------------------------------------------------ dense apply, lookup, cosine difference
def test_vectorised_bf16_rounding_is_the_scalar_one():
    rng = np.random.default_rng(8)
    x = np.concatenate([rng.standard_normal(30_000) * rng.choice([1e-30, 1e-3, 1.0, 1e5, 1e30], 30_000),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, -1.00390625, 0.99609375 + 2.0 ** -10, 3.0e38]])
    got = oracle._bf16_round(x)
    want = np.array([oracle.double_to_bf16(float(v)) for v in x], dtype=np.uint16)
    assert np.array_equal(got, want)


def test_dense_apply_is_eq1_and_the_sparse_apply_with_every_row_listed():
    rng = np.random.default_rng(9)
    V, D = 50, 6
    theta0 = rng.standard_normal(V * D).astype(np.float32)
    g = [rng.standard_normal(V * D).astype(np.float32) for _ in range(4)]
    # K = 0: Eq. 1 in double, rounded once
    t = oracle.dense_apply(theta0.copy(), oracle.F32, g[:1], 0.1)
    want = (theta0.astype(np.float64) - float(np.float32(0.1)) * g[0].astype(np.float64)).astype(np.float32)
    assert np.array_equal(t, want)
    # a dense gradient is a sparse one that lists every row: same result as the sparse routine, bit for bit
    t = oracle.dense_apply(theta0.copy(), oracle.F32, g, 0.025)
    W = theta0.copy().reshape(V, D)
    ids = np.arange(V, dtype=np.int32)
    oracle.dasgd_apply_table(W, D, oracle.F32, [(ids, x.reshape(V, D)) for x in g], 0.025)
    assert np.array_equal(t, W.reshape(-1))
    # bf16: one rounding from the exact sum
    tb = oracle._bf16_round(theta0.astype(np.float64))
    t2 = oracle.dense_apply(tb.copy(), oracle.BF16, g, 0.025)
    Wb = tb.copy().reshape(V, D)
    oracle.dasgd_apply_table(Wb, D, oracle.BF16, [(ids, x.reshape(V, D)) for x in g], 0.025)
    assert np.array_equal(t2, Wb.reshape(-1))
    # no gradients: nothing moves
    assert np.array_equal(oracle.dense_apply(theta0.copy(), oracle.F32, [], 0.5), theta0)


def test_lookup_and_cosine_difference_closed_forms():
    W = np.array([[3, 4, 9], [4, 3, 9], [0, 0, 9], [-3, -4, 9], [6, 8, 9], [4, -3, 9]], dtype=np.float32)   # last column = padding
    rows = oracle.lookup(W, oracle.F32, 2, [4, 0, 0])
    assert rows.dtype == np.float32 and rows.tolist() == [[6, 8], [3, 4], [3, 4]]
    A = W[[0, 0, 0, 0, 0, 2, 2]]
    Bt = W[[0, 1, 3, 4, 5, 2, 0]]
    d = oracle.cosine_difference(A, Bt, oracle.F32, 2)
    # same vector 0; (3,4).(4,3) = 24/25; opposite 2; scaled copy 0; orthogonal 1; zero vs zero 0; zero vs non-zero 1
    assert np.allclose(d, [0.0, 0.04, 2.0, 0.0, 1.0, 0.0, 1.0], atol=1e-15)
    rng = np.random.default_rng(10)
    X, Y = rng.standard_normal((40, 7)).astype(np.float32), rng.standard_normal((40, 7)).astype(np.float32)
    d = oracle.cosine_difference(X, Y, oracle.F32, 7)
    assert np.allclose(d, oracle.cosine_difference(Y, X, oracle.F32, 7), atol=1e-15)            # symmetric
    assert np.allclose(d, oracle.cosine_difference(3 * X, 0.5 * Y, oracle.F32, 7), atol=1e-12)  # scale-free
    assert ((d >= 0) & (d <= 2)).all()
    t = torch.nn.functional.cosine_similarity(torch.from_numpy(X).double(), torch.from_numpy(Y).double(), dim=1)
    assert np.allclose(d, 1.0 - t.numpy(), atol=1e-12)
    # bf16 tables are widened exactly
    Xb = oracle._bf16_round(X.astype(np.float64))
    assert np.array_equal(oracle.lookup(Xb, oracle.BF16, 7, [5]), oracle.bf16_to_f32(Xb[[5]]))


# ------------------------------------------------------------------ gradient messages in bfloat16
def test_bf16_message_rounding_worked_values_and_a_library_conversion():
    """Hand-worked roundings (ties to even on both sides of 1, the midpoint beyond the largest finite
    value, signs, subnormals), then a tensor library's float32 -> bfloat16 conversion on a million
    values of gradient-like magnitude."""
    f = np.float32
    x = np.array([1.0, 1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -20, -1 - 2.0 ** -8,
                  1 - 2.0 ** -9, 1 - 3 * 2.0 ** -9,
                  0.0, -0.0, np.inf, -np.inf, 3.3895313892515355e38, 3.396e38, 3.397e38, 2.0 ** -133], dtype=f)
    want = [0x3F80, 0x3F80, 0x3F82, 0x3F81, 0xBF80,
            0x3F80, 0x3F7E,       # below 1 the spacing is 2^-8: 1 - 2^-9 ties up to 1 (even), 1 - 3*2^-9 ties down to 0x3F7E
            0x0000, 0x8000, 0x7F80, 0xFF80, 0x7F7F, 0x7F7F, 0x7F80, 0x0001]
    assert oracle.grad_pack_rows(x).tolist() == want
    assert oracle.grad_pack_rows(np.array([np.nan], f)).tolist() == [0x7FC0]
    rng = np.random.default_rng(11)
    r = (rng.standard_normal(1_000_000) * rng.choice([1e-8, 1e-4, 1e-2, 1.0], 1_000_000)).astype(f)
    lib = torch.from_numpy(r).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = oracle.grad_pack_rows(r)
    assert np.array_equal(got, lib)
    # what the receiver sees: within half a unit in the last place (at most 2^-8 relative), sign-symmetric, idempotent
    back = oracle.grad_unpack_rows(got)
    assert (np.abs(back.astype(np.float64) - r) <= 2.0 ** -8 * np.abs(r)).all()
    assert np.array_equal(oracle.grad_pack_rows(-r), got ^ np.uint16(0x8000))
    assert np.array_equal(oracle.grad_pack_rows(back), got)


def test_bf16_messages_move_the_update_by_at_most_their_rounding():
    """Eq. 1 with peers' gradients that travelled as bfloat16: the own gradient is untouched, listed rows
    stay listed, and the table differs from the one updated with the float gradients by at most
    alpha * sum_k 2^-8 |g_k| per element (plus the final float rounding)."""
    rng = np.random.default_rng(12)
    V, D, lr = 40, 8, 0.5
    W0 = rng.standard_normal((V, D)).astype(np.float32)
    srcs = []
    for k in range(4):
        ids = np.sort(rng.choice(V, size=[17, 1, 40, 9][k], replace=False)).astype(np.int32)
        srcs.append((ids, rng.standard_normal((ids.size, D)).astype(np.float32)))
    through = [srcs[0]] + [(i, oracle.grad_unpack_rows(oracle.grad_pack_rows(r))) for i, r in srcs[1:]]
    A, Bt = W0.copy(), W0.copy()
    oracle.dasgd_apply_table(A, D, oracle.F32, srcs, lr)
    oracle.dasgd_apply_table(Bt, D, oracle.F32, through, lr)
    bound = np.zeros((V, D))
    for ids, rows in srcs[1:]:
        bound[ids] += 2.0 ** -8 * np.abs(rows)
    assert (np.abs(A.astype(np.float64) - Bt) <= lr * bound + 2.0 ** -22 * np.abs(A)).all()
    own_only = np.setdiff1d(srcs[0][0], np.concatenate([s[0] for s in srcs[1:]]))
    assert np.array_equal(A[own_only], Bt[own_only])
    assert (A != Bt).any()
    # the Grad-level helper rounds both tables' rows once and keeps everything else
    g = oracle.Grad(3, 0.5, np.zeros((3, 2), np.int32), oracle.SparseRows(srcs[1][0], srcs[1][1], np.zeros(2, np.int64)),
                    oracle.SparseRows(srcs[2][0], srcs[2][1], np.zeros(41, np.int64)))
    h = oracle.grad_through_bf16(g)
    assert h.P == 3 and np.array_equal(h.gin.ids, g.gin.ids) and np.array_equal(h.gout.rows, through[2][1])


# ------------------------------------------------------------------ stochastic rounding of bf16 tables
def test_stochastic_rounding_by_hand_neighbours_and_expectation():
    """The variant of Eq. 1's store for bfloat16 tables: one decision recomputed from the Philox block; every
    result is one of the two bfloat16 neighbours of the exact value; an exactly representable result never
    moves; the mean over many draws is the exact value (where round-to-nearest loses the whole update);
    same serial reproduces, another serial decides anew; float tables ignore it."""
    V, D, lr, seed = 64, 8, 0.025, 0xFEEDFACE12345678
    rng = np.random.default_rng(21)
    W0 = oracle.grad_pack_rows((rng.standard_normal((V, D)) * 0.5).astype(np.float32))     # a bfloat16 table
    ids = np.sort(rng.choice(V, 40, replace=False)).astype(np.int32)
    g = (rng.standard_normal((40, D)) * 0.3).astype(np.float32)
    exact = oracle.bf16_to_f32(W0).astype(np.float64)
    exact[ids] -= float(np.float32(lr)) * g.astype(np.float64)
    X = W0.copy()
    oracle.dasgd_apply_table(X, D, oracle.BF16, [(ids, g)], lr, stochastic=(seed, 5, 1))
    # by hand: element (row, col) of table 1 at serial 5
    row, col = int(ids[7]), 3
    i = row * D + col
    r = oracle.philox4x32_10([(i >> 2) & 0xFFFFFFFF, (i >> 2) >> 32, 5, 0x53524E44 + 1], [seed & 0xFFFFFFFF, seed >> 32])
    u = int(np.float32(exact[row, col]).view(np.uint32))
    assert int(X[row, col]) == ((u + (int(r[i & 3]) & 0xFFFF)) >> 16) & 0xFFFF
    # neighbours: truncation towards zero of the single-precision value, or one step away from zero
    f32 = exact.astype(np.float32)
    down = (f32.view(np.uint32) >> 16).astype(np.uint16)
    assert (((X == down) | (X == down + 1))).all()
    untouched = np.setdiff1d(np.arange(V), ids)
    assert np.array_equal(X[untouched], W0[untouched])
    # representable results stay: gradient 0, and a gradient that moves the value by exactly one bfloat16 step
    Z = W0.copy()
    oracle.dasgd_apply_table(Z, D, oracle.BF16, [(ids, np.zeros_like(g))], lr, stochastic=(seed, 6, 0))
    assert np.array_equal(Z, W0)
    # expectation: 1.0 - alpha * 0.01 is a quarter of the way down to the next bfloat16 below 1 (spacing 2^-8)
    ones = np.full((V, D), 0x3F80, np.uint16)
    allids = np.arange(V, dtype=np.int32)
    small = np.full((V, D), 0.01, np.float32)
    total, n = 0.0, 300
    for serial in range(n):
        Y = ones.copy()
        oracle.dasgd_apply_table(Y, D, oracle.BF16, [(allids, small)], lr, stochastic=(seed, serial, 0))
        assert set(np.unique(Y)) <= {0x3F80, 0x3F7F}
        total += float(oracle.bf16_to_f32(Y).astype(np.float64).mean())
    want = 1.0 - float(np.float32(lr)) * float(np.float32(0.01))
    step = 2.0 ** -8                                     # distance between the two candidates
    p = (1.0 - want) / step                              # probability of the lower one
    sd = step * np.sqrt(p * (1 - p) / (n * V * D))
    assert abs(total / n - want) < 6 * sd
    Y = ones.copy()
    oracle.dasgd_apply_table(Y, D, oracle.BF16, [(allids, small)], lr)
    assert (Y == 0x3F80).all()                           # nearest-even: the update is lost
    # reproducible per serial, different across serials and tables
    A, Bt, Ct, Dt = ones.copy(), ones.copy(), ones.copy(), ones.copy()
    oracle.dasgd_apply_table(A, D, oracle.BF16, [(allids, small)], lr, stochastic=(seed, 9, 0))
    oracle.dasgd_apply_table(Bt, D, oracle.BF16, [(allids, small)], lr, stochastic=(seed, 9, 0))
    oracle.dasgd_apply_table(Ct, D, oracle.BF16, [(allids, small)], lr, stochastic=(seed, 10, 0))
    oracle.dasgd_apply_table(Dt, D, oracle.BF16, [(allids, small)], lr, stochastic=(seed, 9, 1))
    assert np.array_equal(A, Bt) and not np.array_equal(A, Ct) and not np.array_equal(A, Dt)
    # float tables: the flag changes nothing
    F1 = oracle.bf16_to_f32(W0).copy()
    F2 = F1.copy()
    oracle.dasgd_apply_table(F1, D, oracle.F32, [(ids, g)], lr)
    oracle.dasgd_apply_table(F2, D, oracle.F32, [(ids, g)], lr, stochastic=(seed, 5, 1))
    assert np.array_equal(F1, F2)

"""Pins for the oracle's integer primitives: Philox, alias table, pair enumeration,
negative draws, initialisation, bf16 rounding, staleness.  CPU only."""
import math
import os

import numpy as np
import pytest
import torch

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ Philox
def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLD, "philox4x32_10_kat.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        out = oracle.philox4x32_10(v[0:4], v[4:6])
        assert [int(x) for x in out] == v[6:10]


def test_philox_is_a_bijection_on_a_small_slice_and_key_sensitive():
    # distinct counters never collide (the round function is a permutation of the counter)
    outs = {tuple(int(x) for x in oracle.philox4x32_10([i, 0, 0, 0], [7, 9])) for i in range(2000)}
    assert len(outs) == 2000
    a = oracle.philox4x32_10([1, 2, 3, 4], [5, 6])
    b = oracle.philox4x32_10([1, 2, 3, 4], [5, 7])
    assert not np.array_equal(a, b)


# ------------------------------------------------------------------ alias table
def _alias_mass(thr, alias):
    """Probability mass each id receives from the table, in units of 1/(V*2^32)."""
    V = thr.shape[0]
    mass = np.zeros(V, dtype=object)
    for i in range(V):
        t = int(thr[i])
        acc = (1 << 32) if t == 0xFFFFFFFF and int(alias[i]) == i else t
        mass[i] += acc
        mass[int(alias[i])] += (1 << 32) - acc
    return mass


@pytest.mark.parametrize("seed,V", [(0, 17), (1, 100), (2, 1000)])
def test_alias_mass_matches_unigram_pow_075(seed, V):
    rng = np.random.default_rng(seed)
    counts = rng.zipf(1.3, size=V).astype(np.uint64)
    counts[rng.integers(0, V, size=V // 10)] = 0          # some ids never occur
    counts[0] = max(int(counts[0]), 1)
    thr, alias = oracle.alias_build(counts)
    mass = _alias_mass(thr, alias)
    w = counts.astype(np.float64) ** 0.75
    want = w / w.sum()
    got = np.array([float(m) for m in mass]) / (V * 2.0 ** 32)
    # flooring each threshold loses < 2^-32 per bucket; an id collects from at most V buckets
    assert np.all(np.abs(got - want) <= V * 2.0 ** -32 + 1e-15)
    assert sum(int(m) for m in mass) == V << 32
    # ids with zero count get essentially no mass (at most the floor residue of their own bucket)
    assert np.all(got[counts == 0] <= 2.0 ** -32)
    assert np.all((alias >= 0) & (alias < V))


def test_alias_special_cases():
    thr, alias = oracle.alias_build(np.array([5], dtype=np.uint64))
    assert int(thr[0]) == 0xFFFFFFFF and int(alias[0]) == 0
    thr, alias = oracle.alias_build(np.full(64, 3, dtype=np.uint64))
    assert np.all(thr == 0xFFFFFFFF) and np.array_equal(alias, np.arange(64))
    with pytest.raises(ValueError):
        oracle.alias_build(np.zeros(4, dtype=np.uint64))
    # two ids, weights 1 and 16^0.75 = 8 -> p = (1/9, 8/9): bucket 0 keeps 2/9, rest goes to id 1
    thr, alias = oracle.alias_build(np.array([1, 16], dtype=np.uint64))
    assert int(alias[0]) == 1 and int(thr[0]) == math.floor(2.0 / 9.0 * 2 ** 32)
    assert int(thr[1]) == 0xFFFFFFFF


def test_negative_draws_follow_the_noise_distribution():
    V = 50
    counts = (1000.0 / np.arange(1, V + 1)).astype(np.uint64) + 1
    thr, alias = oracle.alias_build(counts)
    n = 400_000
    pos = np.arange(n, dtype=np.int64)
    q = np.zeros(n, dtype=np.int32)
    neg = oracle.sample_negatives(V, thr, alias, 1234, 0, 0, pos, q, 1)[:, 0]
    w = counts.astype(np.float64) ** 0.75
    expect = w / w.sum() * n
    obs = np.bincount(neg, minlength=V).astype(np.float64)
    chi2 = ((obs - expect) ** 2 / expect).sum()
    # 49 degrees of freedom: mean 49, sd ~9.9; 110 is > 6 sd
    assert chi2 < 110.0


def test_negative_draw_definition_by_hand():
    """One draw recomputed step by step from the counter layout."""
    V = 1000
    counts = np.arange(1, V + 1, dtype=np.uint64)
    thr, alias = oracle.alias_build(counts)
    seed, worker, epoch, pos, q, slot = (0xABCDEF0123456789, 3, 2, (5 << 32) + 77, 4, 6)
    r = oracle.philox4x32_10([pos & 0xFFFFFFFF, pos >> 32, q * 65536 + slot, worker + 65536 * epoch],
                             [seed & 0xFFFFFFFF, seed >> 32])
    b = (int(r[0]) * V) >> 32
    want = b if int(r[1]) < int(thr[b]) else int(alias[b])
    got = oracle.sample_negatives(V, thr, alias, seed, worker, epoch, np.array([pos]), np.array([q]), 8)
    assert int(got[0, slot]) == want


def test_negatives_do_not_depend_on_batching():
    V, T, w, N = 200, 500, 3, 4
    counts = np.ones(V, dtype=np.uint64)
    thr, alias = oracle.alias_build(counts)

    def run(B):
        out = []
        for begin in range(0, T, B):
            pos, q = oracle.pairs(T, w, begin, min(B, T - begin))
            out.append(oracle.sample_negatives(V, thr, alias, 99, 1, 0, pos, q, N))
        return np.concatenate(out)

    assert np.array_equal(run(64), run(7))


def test_resampled_negatives_by_hand_and_by_their_statistics():
    """The variant that draws a colliding negative once more: every entry recomputed step by step from the
    Philox block (first draw from words 0/1; if it equals the pair's center or context word, the draw from
    words 2/3), on a vocabulary small enough for collisions to be common; without a collision it is the base
    draw; collisions become rarer by about the collision probability itself."""
    V, T, w, N = 6, 300, 2, 5
    rng = np.random.default_rng(5)
    tok = rng.integers(0, V, size=T).astype(np.int32)
    counts = np.bincount(tok, minlength=V).astype(np.uint64)
    thr, alias = oracle.alias_build(counts)
    seed, worker, epoch = 0x1122334455667788, 2, 1
    pos, q = oracle.pairs(T, w, 0, T)
    base = oracle.sample_negatives(V, thr, alias, seed, worker, epoch, pos, q, N)
    got = oracle.sample_negatives(V, thr, alias, seed, worker, epoch, pos, q, N, resample_tok=tok, w=w)

    def pick(r_bucket, r_accept):
        b = (int(r_bucket) * V) >> 32
        return b if int(r_accept) < int(thr[b]) else int(alias[b])

    hits_before = hits_after = 0
    for i in range(0, pos.size, 7):             # a seventh of the pairs, every slot
        p, qq = int(pos[i]), int(q[i])
        o = qq - w if qq < w else qq - w + 1
        center, context = int(tok[p]), int(tok[p + o])
        for k in range(N):
            r = oracle.philox4x32_10([p & 0xFFFFFFFF, p >> 32, qq * 65536 + k, worker + 65536 * epoch],
                                     [seed & 0xFFFFFFFF, seed >> 32])
            first = pick(r[0], r[1])
            want = pick(r[2], r[3]) if first in (center, context) else first
            assert int(got[i, k]) == want and int(base[i, k]) == first
    o_all = np.where(q < w, q - w, q - w + 1)
    cen, ctx = tok[pos][:, None], tok[pos + o_all][:, None]
    hits_before = int(((base == cen) | (base == ctx)).sum())
    hits_after = int(((got == cen) | (got == ctx)).sum())
    same = (base != cen) & (base != ctx)
    assert np.array_equal(got[same], base[same])          # no collision: the base draw
    assert hits_before > 0.2 * base.size                  # collisions are common here ...
    assert hits_after < 0.6 * hits_before                 # ... and the second draw removes most of them
    # the gradient routine with the variant switched on uses exactly these negatives
    D = 4
    W_in = (rng.standard_normal((V, D)) * 0.3).astype(np.float32)
    W_out = (rng.standard_normal((V, D)) * 0.3).astype(np.float32)
    g = oracle.sgns_grad(tok, w, N, 10, 40, D, oracle.F32, W_in, W_out, thr, alias, seed, worker, epoch, resample=True)
    p2, q2 = oracle.pairs(T, w, 10, 40)
    assert np.array_equal(g.negatives, oracle.sample_negatives(V, thr, alias, seed, worker, epoch, p2, q2, N,
                                                               resample_tok=tok, w=w))


# ------------------------------------------------------------------ pairs
@pytest.mark.parametrize("T,w", [(1, 2), (2, 3), (5, 2), (20, 3), (20, 8), (7, 10)])
def test_pairs_brute_force_and_closed_form(T, w):
    pos, q = oracle.pairs(T, w, 0, T)
    want = []
    for p in range(T):
        for o in list(range(-w, 0)) + list(range(1, w + 1)):
            if 0 <= p + o < T:
                want.append((p, o))
    got = [(int(p), int(qq) - w if qq < w else int(qq) - w + 1) for p, qq in zip(pos, q)]
    assert got == want
    # every ordered pair of distinct positions at distance <= w, counted once
    assert len(got) == sum(min(w, T - 1 - i) + min(w, i) for i in range(T))
    if T > w:
        assert len(got) == 2 * w * T - w * (w + 1)


def test_pairs_of_config1_pass():
    T, w, B = 10_000, 2, 64
    total = sum(len(oracle.pairs(T, w, b, min(B, T - b))[0]) for b in range(0, T, B))
    assert total == 4 * T - w * (w + 1) == 39_994


# ------------------------------------------------------------------ init
def test_init_tables_distribution_and_definition():
    V, D = 300, 20
    w_in, w_out = oracle.init_tables(V, D, D + 4, oracle.F32, 2001)
    assert not w_out.any()
    assert not w_in[:, D:].any()
    x = w_in[:, :D].astype(np.float64)
    assert x.min() >= -0.5 / D and x.max() < 0.5 / D
    n = x.size
    assert abs(x.mean()) < 4 * (1.0 / D) / math.sqrt(12 * n)
    assert abs(x.var() - (1.0 / D) ** 2 / 12) < 0.1 * (1.0 / D) ** 2 / 12
    # element (row 7, col 5): index i = 7*D+5, word i%4 of the block i//4
    i = 7 * D + 5
    r = oracle.philox4x32_10([i // 4, 0, 0, 0x494E4954], [2001, 0])
    u = np.float32(int(r[i % 4]) >> 8) * np.float32(2.0 ** -24)
    want = (u - np.float32(0.5)) * (np.float32(1.0) / np.float32(D))
    assert w_in[7, 5] == np.float32(want)


def test_init_bf16_is_rounded_f32_init():
    V, D = 64, 16
    a, _ = oracle.init_tables(V, D, D, oracle.F32, 5)
    b, _ = oracle.init_tables(V, D, D, oracle.BF16, 5)
    want = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(b, want)


# ------------------------------------------------------------------ bf16 rounding
def test_double_to_bf16_matches_library_rounding_on_floats_and_ties():
    rng = np.random.default_rng(3)
    xs = np.concatenate([
        rng.standard_normal(2000).astype(np.float32),
        (rng.standard_normal(500) * 1e-3).astype(np.float32),
        np.array([0.0, -0.0, 1.0, -1.0, 1.00390625, 1.01171875, 3.3895313892515355e38, 1e-40, 9.1835e-41,
                  np.float32(2.0 ** -133), np.float32(2.0 ** -134), 65280.0, 65408.0], dtype=np.float32),
    ])
    want = torch.from_numpy(xs).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle.double_to_bf16(float(x)) for x in xs], dtype=np.uint16)
    assert np.array_equal(got, want)
    # a double that sits just above a float tie must round up even though its float image is the tie
    tie = 1.0 + 2.0 ** -8            # exactly half-way between bf16 1.0 and 1.0078125 -> even = 1.0
    assert oracle.double_to_bf16(tie) == 0x3F80
    assert oracle.double_to_bf16(tie + 2.0 ** -40) == 0x3F81


# ------------------------------------------------------------------ staleness
def test_staleness_worked_example_of_the_paper():
    for line in open(os.path.join(GOLD, "staleness_example.txt")):
        if not line.strip() or line[0] == "#":
            continue
        name, gi, gj, want = [f.strip() for f in line.split(";")]
        assert oracle.staleness(gi.split(), gj.split()) == int(want), name
    # symmetric difference, not a one-sided difference
    assert oracle.staleness({"a", "b"}, {"b", "c", "d"}) == 3


# ------------------------------------------------------------------ sanitizers
def test_oracle_runs_clean_under_address_and_ub_sanitizers():
    """The oracle's C source, driven over small inputs that reach its edges, under gcc's address and
    undefined-behaviour sanitizers (a program of its own: an out-of-bounds access, a leak or an overflow
    ends it with a report and a non-zero status)."""
    import subprocess
    exe = oracle.build_sanitize_check()
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "sanitize_check: ok" in r.stdout and "ERROR" not in r.stderr

"""Pins of the oracle's worker sequencing (oracle/driver.py) and of the shared input schedule (workload.py).
CPU only.

What fixes the expected values here is the paper, not the driver: Section 3.1 and Algorithm 1 (train) say
that a Model instance computes its own gradient on the model as it stands, applies it, and only then
applies the gradients that arrived; Section 3.1 defines on which (older) model a received gradient was
computed; Section 4.1 says that a single instance is synchronous mini-batch SGD; Algorithm 1 says that the
summed buffer is sent when gradients_count reaches maxGradBuffer and starts again.  Every test below writes
the steps out one by one -- explicit snapshot copies, explicit batch ranges, explicit staleness table --
with the already pinned ``oracle.sgns_grad`` / ``oracle.dasgd_apply`` / ``oracle.grad_add`` (or Eq. 1 retyped
in numpy) and compares the driver with that sequence bit for bit.
"""
import os

import numpy as np
import pytest

import oracle
import workload as W
from oracle.driver import GSets, OracleWorker

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _tiny(**kw):
    base = dict(idx=9, name="tiny", vocab=40, dim=8, dtype="f32", tokens=400, zipf_s=1.0, window=2, negatives=3,
                batch=6, peers=2, max_stale=2, lr=0.5, parity_steps=4)
    base.update(kw)
    return W.Config(**base)


def _setup(cfg, seed=1):
    """Stream, counts and 'pre-trained' tables large enough that every step moves the model visibly (so that a
    gradient taken on the wrong snapshot has other bits)."""
    tok, counts = W.make_stream(cfg)
    rng = np.random.default_rng(seed)
    Wi = (rng.standard_normal((cfg.vocab, cfg.dim)) * 0.5).astype(np.float32)
    Wo = (rng.standard_normal((cfg.vocab, cfg.dim)) * 0.5).astype(np.float32)
    if cfg.dtype == "bf16":
        Wi, Wo = oracle._bf16_round(Wi.astype(np.float64)), oracle._bf16_round(Wo.astype(np.float64))
    return tok, counts, Wi, Wo


def _batch(cfg, j):
    """Global mini-batch j of the tumbling window, retyped: consecutive runs of `batch` centers, the last of a
    pass partial, then the stream again with the epoch one higher."""
    per_pass = (cfg.tokens + cfg.batch - 1) // cfg.batch
    epoch, b = j // per_pass, j % per_pass
    begin = b * cfg.batch
    return begin, min(cfg.batch, cfg.tokens - begin), epoch


def _grad(cfg, tok, thr, alias, theta, j, worker):
    begin, n, epoch = _batch(cfg, j)
    dt = oracle.F32 if cfg.dtype == "f32" else oracle.BF16
    return oracle.sgns_grad(tok, cfg.window, cfg.negatives, begin, n, cfg.dim, dt, theta[0], theta[1], thr, alias,
                            cfg.seed, worker, epoch)


def _same_grad(a, b):
    return (np.array_equal(a.gin.ids, b.gin.ids) and np.array_equal(a.gout.ids, b.gout.ids) and
            np.array_equal(a.gin.rows, b.gin.rows) and np.array_equal(a.gout.rows, b.gout.rows))


# ------------------------------------------------------------------ the shared schedule (workload.py)
def test_batches_are_dealt_round_robin_over_a_tumbling_window():
    cfg = W.CONFIGS[1]                                   # 10 000 tokens, 64 centers: 157 batches, the last has 16
    assert cfg.n_batches == 157
    assert W.batch_slice(cfg, 0) == (0, 64, 0)
    assert W.batch_slice(cfg, 156) == (9984, 16, 0)
    assert W.batch_slice(cfg, 157) == (0, 64, 1)         # the stream again, next epoch
    cfg = _tiny(peers=2)
    for t in range(70):                                  # more than one pass of 67 batches
        for k in range(3):
            # step (4) of the dataflow: every mini-batch goes to one instance; instance k gets batch t(K+1)+k
            assert W.worker_batch(cfg, t, k) == _batch(cfg, t * 3 + k)
    seen = [W.worker_batch(cfg, t, k) for t in range(4) for k in range(3)]
    assert len(set(seen)) == len(seen)                   # disjoint data per instance
    for begin, n, _ in seen:
        assert W.pairs_in_batch(cfg, begin, n) == oracle.pairs(cfg.tokens, cfg.window, begin, n)[0].size


def test_staleness_draws_are_seeded_uniform_and_in_range():
    cfg = _tiny(peers=3, max_stale=4)
    d = W.stale_draws(cfg, 4096)
    assert d.shape == (4096, 3) and d.min() == 0 and d.max() == 4
    assert np.array_equal(d, W.stale_draws(cfg, 4096))                       # a function of the seed
    assert not np.array_equal(d, W.stale_draws(cfg.scaled(idx=8), 4096))     # and of nothing else
    freq = np.bincount(d.ravel(), minlength=5) / d.size
    assert np.abs(freq - 0.2).max() < 0.02
    assert W.stale_draws(_tiny(peers=2, max_stale=0), 10).max() == 0
    assert W.stale_draws(_tiny(peers=0), 10).shape == (10, 0)


# ------------------------------------------------------------------ Section 3.1 / Algorithm 1: one step after another
STALE = np.array([[0, 0], [1, 0], [2, 1], [0, 2], [1, 1]])     # how old the model each peer computed on is, per step


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_worker_steps_equal_the_sequence_written_out_by_hand(dtype):
    cfg = _tiny(dtype=dtype)
    tok, counts, Wi, Wo = _setup(cfg)
    thr, alias = oracle.alias_build(counts)
    dt = oracle.F32 if dtype == "f32" else oracle.BF16
    ow = OracleWorker(cfg, tok, counts, tables=(Wi, Wo))
    ow.stale = STALE.copy()
    thetas = [(Wi.copy(), Wo.copy())]                    # theta_0, theta_1, ...: the model before each step
    used = set()
    for t in range(len(STALE)):
        cur = thetas[t]
        # own gradient on theta_t (nothing of step t has been applied yet) ...
        own = _grad(cfg, tok, thr, alias, cur, 3 * t + 0, 0)
        # ... peer k's on the model this worker had max(0, t - s) steps ago, on the peer's own mini-batch and draws
        peers = []
        for k in (1, 2):
            src = max(0, t - int(STALE[t, k - 1]))
            used.add(t - src)
            peers.append(_grad(cfg, tok, thr, alias, thetas[src], 3 * t + k, k))
        # apply_gradient of the own gradient and of the two messages, same alpha
        nxt = (cur[0].copy(), cur[1].copy())
        oracle.dasgd_apply(nxt[0], nxt[1], cfg.dim, dt, [own] + peers, cfg.lr)
        thetas.append(nxt)

        got = ow.step()
        assert len(got) == 3 and all(_same_grad(g, w) for g, w in zip(got, [own] + peers)), f"step {t}"
        assert np.array_equal(ow.W_in, nxt[0]) and np.array_equal(ow.W_out, nxt[1]), f"step {t}"
        # Section 3.1: the own gradient has staleness 0; peer k's gradient meets a model that has applied the
        # (t - src) * 3 gradients of the steps in between, this step's own gradient and the peers before it
        assert ow.last_staleness == [(t - max(0, t - int(STALE[t, k - 1]))) * 3 + k for k in (1, 2)]
    assert used == {0, 1, 2}                             # every age occurred
    # the run is sensitive to what it pins: a peer gradient taken on the current model instead of the stale
    # one, or the own gradient taken after the peers were applied, has other bits
    t = 2
    assert not _same_grad(_grad(cfg, tok, thr, alias, thetas[t], 3 * t + 1, 1),
                          _grad(cfg, tok, thr, alias, thetas[t - 2], 3 * t + 1, 1))
    assert not _same_grad(_grad(cfg, tok, thr, alias, thetas[t], 3 * t, 0),
                          _grad(cfg, tok, thr, alias, thetas[t + 1], 3 * t, 0))


def test_a_single_instance_is_plain_minibatch_sgd():
    """Section 4.1: with one rank the updates are those of synchronous SGD -- theta <- theta - alpha * grad on the
    mini-batches in stream order (Eq. 1 retyped in numpy, no call of the oracle's apply)."""
    cfg = _tiny(peers=0, max_stale=0)
    tok, counts, Wi, Wo = _setup(cfg, seed=2)
    thr, alias = oracle.alias_build(counts)
    ow = OracleWorker(cfg, tok, counts, tables=(Wi, Wo))
    a, b = Wi.copy(), Wo.copy()
    alpha = np.float64(np.float32(cfg.lr))
    for t in range(5):
        g = _grad(cfg, tok, thr, alias, (a, b), t, 0)
        a[g.gin.ids] = (a[g.gin.ids].astype(np.float64) - alpha * g.gin.rows.astype(np.float64)).astype(np.float32)
        b[g.gout.ids] = (b[g.gout.ids].astype(np.float64) - alpha * g.gout.rows.astype(np.float64)).astype(np.float32)
        got = ow.step()
        assert len(got) == 1 and ow.last_staleness == []
        assert np.array_equal(ow.W_in, a) and np.array_equal(ow.W_out, b), f"step {t}"
    assert not np.array_equal(a, Wi) and not np.array_equal(b, Wo)


@pytest.mark.parametrize("n", [2, 3])
def test_gradient_buffers_are_sent_every_nth_step_and_start_again(n):
    """Algorithm 1, train(): gradients += gradient; when gradients_count reaches maxGradBuffer the buffer is sent
    and a new one begins.  One peer, whose buffer therefore arrives at steps n-1, 2n-1, ... holding its last n
    gradients (each computed when its step took place, on the model its staleness names)."""
    cfg = _tiny(peers=1, max_stale=1, grad_buffer=n)
    tok, counts, Wi, Wo = _setup(cfg, seed=3)
    thr, alias = oracle.alias_build(counts)
    ow = OracleWorker(cfg, tok, counts, tables=(Wi, Wo))
    stale = np.array([[0], [1], [1], [0], [1], [1], [0]])
    ow.stale = stale.copy()
    thetas = [(Wi.copy(), Wo.copy())]
    own_buf = peer_buf = None
    for t in range(2 * n + 1):
        cur = thetas[t]
        own = _grad(cfg, tok, thr, alias, cur, 2 * t, 0)
        peer = _grad(cfg, tok, thr, alias, thetas[max(0, t - int(stale[t, 0]))], 2 * t + 1, 1)
        own_buf = own if own_buf is None else oracle.grad_add(own_buf, own, cfg.dim)
        peer_buf = peer if peer_buf is None else oracle.grad_add(peer_buf, peer, cfg.dim)
        sends = (t + 1) % n == 0                        # gradients_count has reached maxGradBuffer
        nxt = (cur[0].copy(), cur[1].copy())
        oracle.dasgd_apply(nxt[0], nxt[1], cfg.dim, oracle.F32, [own] + ([peer_buf] if sends else []), cfg.lr)
        thetas.append(nxt)
        got = ow.step()
        assert len(got) == (2 if sends else 1), f"step {t}"
        assert _same_grad(got[0], own)
        assert np.array_equal(ow.W_in, nxt[0]) and np.array_equal(ow.W_out, nxt[1]), f"step {t}"
        if sends:
            assert _same_grad(got[1], peer_buf) and _same_grad(ow.sent, own_buf)
            assert len(ow.last_staleness) == n          # the n gradients inside the peer's buffer
            own_buf = peer_buf = None                   # a new buffer begins
        else:
            assert ow.last_staleness == []
    # at the last step (one past a send) the buffers hold that step's gradient alone
    assert _same_grad(ow.own_buffer, own) and _same_grad(ow.peer_buffers[0], peer)


def test_bf16_messages_round_what_the_peers_send_once_after_summing():
    cfg = _tiny(peers=1, max_stale=0, grad_buffer=2)
    tok, counts, Wi, Wo = _setup(cfg, seed=4)
    thr, alias = oracle.alias_build(counts)
    ow = OracleWorker(cfg, tok, counts, tables=(Wi, Wo), bf16_messages=True)
    cur = (Wi.copy(), Wo.copy())
    peer_buf = None
    for t in range(2):
        own = _grad(cfg, tok, thr, alias, cur, 2 * t, 0)
        peer = _grad(cfg, tok, thr, alias, cur, 2 * t + 1, 1)
        peer_buf = peer if peer_buf is None else oracle.grad_add(peer_buf, peer, cfg.dim)
        msgs = [oracle.grad_through_bf16(peer_buf)] if t == 1 else []
        oracle.dasgd_apply(cur[0], cur[1], cfg.dim, oracle.F32, [own] + msgs, cfg.lr)
        got = ow.step()
        assert _same_grad(got[0], own)                  # the own gradient stays float
        assert np.array_equal(ow.W_in, cur[0]) and np.array_equal(ow.W_out, cur[1])
    assert not _same_grad(got[1], peer_buf) and _same_grad(got[1], oracle.grad_through_bf16(peer_buf))


# ------------------------------------------------------------------ Section 3.1: the G sets
def test_gsets_reproduce_the_worked_example_of_the_paper():
    """Five mini-batches dealt to three models, maxGradBuffer = 1 (text around the staleness figure): Model 2
    computes and applies blue, then yellow; Model 3 computed green and Model 1 computed red before either had
    applied anything; Model 2 applies green after yellow, and red after green."""
    want = {}
    for line in open(os.path.join(GOLD, "staleness_example.txt")):
        if line.strip() and not line.startswith("#"):
            name, _, _, s = [x.strip() for x in line.split(";")]
            want[name] = int(s)
    g = GSets()
    g.computed(2, "blue")
    g.computed(3, "green")
    g.computed(1, "red")
    assert g.applied(2, "blue") == want["own_blue"] == 0
    assert g.applied(3, "green") == 0 and g.applied(1, "red") == 0      # applied by the models that computed them
    g.computed(2, "yellow")
    assert g.applied(2, "yellow") == 0
    assert g.applied(2, "green") == want["green_3_to_2"] == 2
    assert g.applied(2, "red") == want["red_1_to_2"] == 3
    assert g.G[2] == {"blue", "yellow", "green", "red"}

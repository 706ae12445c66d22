"""Oracle-side simulation of one DASGD worker among K+1 Model instances.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).  Follows Algorithm 1 and the
ordering of Section 3.1 of TensAIR (arXiv 2211.10280): at step t the worker
computes its own gradient on theta_t, then applies it together with the K
gradients that arrived; peer k's gradient was computed on the peer's own
mini-batch against theta_{max(0, t - s)}, s being how many of this worker's steps
old the model was that the peer computed on.  With maxGradBuffer = n > 1 every
instance sums its gradients ("gradients += gradient") and broadcasts the sum after
every n-th of its steps: the K peer buffers then arrive together at this worker's
steps n-1, 2n-1, ..., each holding that peer's gradients of the last n steps (every
one computed when its step took place, on the snapshot its s names), and no peer
gradient is applied at the steps in between.

Pinned on the CPU by ``tests/test_oracle_driver.py``: a run of this class against the
same steps written out one by one from ``oracle.sgns_grad`` / ``oracle.dasgd_apply``
and explicit snapshot copies, bit for bit; a single instance against Eq. 1 retyped in
numpy; the buffer schedule for n = 2 and 3; ``GSets`` against the worked example of
Section 3.1.
"""
from __future__ import annotations

import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

import oracle
import workload as W


class GSets:
    """Bookkeeping of Section 3.1: G_i is the set of gradients Model i has applied; the
    staleness of a gradient, when Model j applies it, is |G_i u G_j| - |G_i n G_j| with G_i
    taken when Model i computed it and G_j when Model j applies it."""

    def __init__(self):
        self.G = {}            # model -> names of the gradients it has applied
        self.at_compute = {}   # gradient name -> G of the computing model at that moment

    def computed(self, model, name, G=None):
        """Model ``model`` computes gradient ``name`` now (or on a model that had applied ``G``)."""
        self.at_compute[name] = frozenset(self.G.get(model, ()) if G is None else G)

    def applied(self, model, name) -> int:
        """Model ``model`` applies gradient ``name`` now; returns the gradient's staleness."""
        mine = self.G.setdefault(model, set())
        s = oracle.staleness(self.at_compute[name], mine)
        mine.add(name)
        return s


class OracleWorker:
    def __init__(self, cfg: W.Config, tokens: np.ndarray, counts: np.ndarray, threads: int = 1,
                 bf16_messages: bool = False, tables=None):
        """tables: (W_in, W_out) of a pre-trained model to start from (copied); None: a fresh one."""
        self.cfg = cfg
        self.tok = np.ascontiguousarray(tokens, dtype=np.int32)
        self.dtype = oracle.F32 if cfg.dtype == "f32" else oracle.BF16
        self.thr, self.alias = oracle.alias_build(counts)
        if tables is None:
            self.W_in, self.W_out = oracle.init_tables(cfg.vocab, cfg.dim, cfg.dim, self.dtype, cfg.seed)
        else:
            self.W_in, self.W_out = (np.array(t, copy=True, order="C") for t in tables)
        self.history = {}            # step -> (W_in, W_out) copies of theta_step
        self.step_no = 0
        self.stale = None
        self.threads = threads
        self.bf16_messages = bf16_messages   # peers' gradients arrive rounded to bfloat16 (variant)
        self.last_own = None
        self.last_peers = []
        # Section 3.1: this worker is Model 0, peer k is Model k; gradients are named (step, model)
        self.gsets = GSets()
        self.applied_at = {}         # gradient name -> step at which this worker applied it
        self.last_staleness = []     # of the peer gradients applied at the latest step, in order of application
        self.waiting = [[] for _ in range(cfg.peers)]   # names of the gradients in each peer's unsent buffer
        # maxGradBuffer: the sums not yet broadcast (None = empty), this worker's and the peers'
        self.own_buffer = None
        self.peer_buffers = [None] * cfg.peers
        self.sent = None             # the buffer this worker broadcast most recently

    def _grad(self, W_in, W_out, begin, n, epoch, worker):
        c = self.cfg
        return oracle.sgns_grad(self.tok, c.window, c.negatives, begin, n, c.dim, self.dtype, W_in, W_out,
                                self.thr, self.alias, c.seed, worker, epoch, resample=c.resample)

    def step(self, n_steps_hint=4096):
        c = self.cfg
        t = self.step_no
        if self.stale is None or self.stale.shape[0] <= t:
            self.stale = W.stale_draws(c, max(n_steps_hint, t + 1))
        if c.peers and c.max_stale:
            self.history[t] = (self.W_in.copy(), self.W_out.copy())
            for old in [s for s in self.history if s < t - c.max_stale]:
                del self.history[old]
        # calculate_gradient: the own one on theta_t, before anything of this step is applied
        jobs = [(self.W_in, self.W_out) + W.worker_batch(c, t, 0) + (0,)]
        self.gsets.computed(0, (t, 0))
        for k in range(1, c.peers + 1):
            s = int(self.stale[t, k - 1]) if c.max_stale else 0
            src = max(0, t - s)
            A, Bt = self.history[src] if c.max_stale else (self.W_in, self.W_out)
            jobs.append((A, Bt) + W.worker_batch(c, t, k) + (k,))
            # the peer is a replica that had applied what this worker had applied when it was theta_src
            self.gsets.computed(k, (t, k), G={g for g, at in self.applied_at.items() if at < src})
            self.waiting[k - 1].append((t, k))
        if self.threads > 1 and len(jobs) > 1:
            with ThreadPoolExecutor(self.threads) as ex:
                grads = list(ex.map(lambda j: self._grad(*j), jobs))
            self.t_own = float("nan")
        else:
            t0 = time.perf_counter()
            grads = [self._grad(*jobs[0])]
            self.t_own = time.perf_counter() - t0            # the worker's own calculate_gradient
            grads += [self._grad(*j) for j in jobs[1:]]      # what the other instances would have sent
        n = c.grad_buffer
        arrive = True
        if n > 1:
            # gradients += gradient, for this worker and for every peer; what arrives at this step
            add = lambda buf, g: g if buf is None else oracle.grad_add(buf, g, c.dim)
            self.own_buffer = add(self.own_buffer, grads[0])
            self.peer_buffers = [add(b, g) for b, g in zip(self.peer_buffers, grads[1:])]
            arrive = (t + 1) % n == 0
            grads = [grads[0]] + (self.peer_buffers if arrive else [])
            if arrive:
                self.sent = self.own_buffer
                self.own_buffer = None
                self.peer_buffers = [None] * c.peers
        if self.bf16_messages:       # what is sent is rounded once, after any summing in the sender's buffer
            grads = [grads[0]] + [oracle.grad_through_bf16(g) for g in grads[1:]]
        t0 = time.perf_counter()
        # apply_gradient: the own gradient first, then the messages that arrived, with the same alpha (merged
        # into one update per row); stochastic rounding (variant): the serial number of this worker's table
        # update is its step number
        oracle.dasgd_apply(self.W_in, self.W_out, c.dim, self.dtype, grads, c.lr,
                           stochastic=(c.seed, t) if c.stochastic_rounding else None)
        self.t_apply = time.perf_counter() - t0
        own_staleness = self._applied((t, 0), t)
        assert own_staleness == 0    # computed and applied by the same model with nothing in between
        self.last_staleness = []
        if arrive:
            for k in range(c.peers):
                self.last_staleness += [self._applied(name, t) for name in self.waiting[k]]
                self.waiting[k] = []
        self.last_own, self.last_peers = grads[0], grads[1:]
        self.step_no += 1
        return grads

    def _applied(self, name, t):
        self.applied_at[name] = t
        return self.gsets.applied(0, name)

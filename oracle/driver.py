"""Oracle-side simulation of one DASGD worker among K+1 Model instances.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).  Follows Algorithm 1 and the
ordering of Section 3.1 of TensAIR (arXiv 2211.10280): at step t the worker
computes its own gradient on theta_t, then applies it together with the K
gradients that arrived; peer k's gradient was computed on the peer's own
mini-batch against theta_{max(0, t - s)}, s being that gradient's staleness
counted in this worker's steps.  With maxGradBuffer = n > 1 every instance sums
its gradients ("gradients += gradient") and broadcasts the sum after every n-th of
its steps: the K peer buffers then arrive together at this worker's steps n-1,
2n-1, ..., each holding that peer's gradients of the last n steps (every one
computed when its step took place, on the snapshot its staleness names), and no
peer gradient is applied at the steps in between.
"""
from __future__ import annotations

import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

import oracle
from paper_2211_10280_amd import workload as W


class OracleWorker:
    def __init__(self, cfg: W.Config, tokens: np.ndarray, counts: np.ndarray, threads: int = 1,
                 bf16_messages: bool = False):
        self.cfg = cfg
        self.tok = np.ascontiguousarray(tokens, dtype=np.int32)
        self.dtype = oracle.F32 if cfg.dtype == "f32" else oracle.BF16
        self.thr, self.alias = oracle.alias_build(counts)
        self.W_in, self.W_out = oracle.init_tables(cfg.vocab, cfg.dim, cfg.dim, self.dtype, cfg.seed)
        self.history = {}            # step -> (W_in, W_out) copies of theta_step
        self.step_no = 0
        self.stale = None
        self.threads = threads
        self.bf16_messages = bf16_messages   # peers' gradients arrive rounded to bfloat16 (variant)
        self.last_own = None
        self.last_peers = []
        # G sets of Section 3.1: gradients this worker has applied, as (step, worker) names
        self.applied = set()
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
        jobs = [(self.W_in, self.W_out) + W.worker_batch(c, t, 0) + (0,)]
        self.last_staleness = []
        for k in range(1, c.peers + 1):
            s = int(self.stale[t, k - 1]) if c.max_stale else 0
            src = max(0, t - s)
            A, Bt = self.history[src] if c.max_stale else (self.W_in, self.W_out)
            jobs.append((A, Bt) + W.worker_batch(c, t, k) + (k,))
            # staleness of Section 3.1 between the snapshot the peer used and this worker now
            G_peer = {g for g in self.applied if g[0] < src}
            self.last_staleness.append(oracle.staleness(G_peer, self.applied))
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
        # stochastic rounding (variant): the serial number of this worker's table update is its step number
        oracle.dasgd_apply(self.W_in, self.W_out, c.dim, self.dtype, grads, c.lr,
                           stochastic=(c.seed, t) if c.stochastic_rounding else None)
        self.t_apply = time.perf_counter() - t0
        self.applied |= {(t, k) for k in range(c.peers + 1)}
        self.last_own, self.last_peers = grads[0], grads[1:]
        self.step_no += 1
        return grads

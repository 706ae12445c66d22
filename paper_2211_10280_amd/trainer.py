"""One DASGD worker among K+1 Model instances, on one GPU.

Drives ``tensair_step`` over a synthetic workload the way the paper's dataflow
would (TensAIR, arXiv 2211.10280, Algorithm 1 and Section 3.1): this worker
receives every (K+1)-th mini-batch; before each of its steps the K gradients of
the other instances "arrive".  With one GPU there are no other instances, so
their gradients are produced here with ``tensair_sgns_grad`` on the peers' own
mini-batches against a snapshot of this worker's model that is 0..max_stale
steps old (the staleness of Section 3.1, counted in this worker's steps).
With maxGradBuffer = n > 1 (Algorithm 1) every instance sums its gradients with
``tensair_grad_add`` and sends the sum after every n-th step, so the K peer
buffers arrive together at steps n-1, 2n-1, ... and none in between.
With ``bf16_messages`` the peers' gradients travel as bfloat16 messages
(``tensair_grad_pack`` on the sender's side, ``tensair_step_packed`` here).
Everything numerical happens inside the library; this file only sequences calls
and keeps buffers.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B
import workload as W


class DasgdWorker:
    def __init__(self, cfg: W.Config, tokens: np.ndarray, counts: np.ndarray, device="cuda", prefetch=True,
                 row_stride=None, bf16_messages=False, tables=None):
        """tables: (w_in, w_out) device tensors of a pre-trained model to train on in place; None: a fresh one.
        row_stride: elements between table rows; None: the pitch that starts every row on a 128-byte line
        (of the given tables, if any)."""
        self.cfg = cfg
        self.bf16_messages = bf16_messages
        self.prefetch = prefetch     # announce coming mini-batches with tensair_prefetch
        self.announced = -1          # last step whose mini-batch has been announced
        self.device = device
        dt = B.F32 if cfg.dtype == "f32" else B.BF16
        if tables is not None:
            row_stride = tables[0].shape[1]
        elif row_stride is None:
            row_stride = B.tensair_aligned_row_stride(cfg.dim, dt)
        flags = (B.RESAMPLE_NEGATIVES if cfg.resample else 0) | (B.STOCHASTIC_ROUNDING if cfg.stochastic_rounding else 0)
        self.tokens = torch.from_numpy(np.ascontiguousarray(tokens, dtype=np.int32)).to(device)
        self.model = B.Model(cfg.vocab, cfg.dim, dt, cfg.window, cfg.negatives, cfg.batch,
                             max(cfg.peers, 0), cfg.seed, counts, worker_id=0, row_stride=row_stride,
                             device=device, flags=flags, tables=tables)
        # a second handle computes the peers' gradients on snapshots (its tables are rebound per call)
        self.peer_model = None
        if cfg.peers > 0:
            self.peer_model = B.Model(cfg.vocab, cfg.dim, dt, cfg.window, cfg.negatives, cfg.batch, 0,
                                      cfg.seed, counts, worker_id=1, row_stride=row_stride, flags=flags,
                                      tables=(self.model.w_in, self.model.w_out), device=device)
        self.own = self.model.grad_buffers()
        self.peer_bufs = [self.model.grad_buffers() for _ in range(cfg.peers)]
        self.snapshots = {}          # step -> (w_in, w_out) clones of theta_step
        self.mean_loss = torch.zeros(1, dtype=torch.float32, device=device)
        self.step_no = 0
        self.stale = None
        # maxGradBuffer > 1: sums not yet sent, two buffers each (tensair_grad_add writes a third operand)
        self.sent = None
        if cfg.grad_buffer > 1:
            n = cfg.grad_buffer
            big = lambda: B.GradBuffers(min(cfg.vocab, n * self.own.cap_in), min(cfg.vocab, n * self.own.cap_out),
                                        cfg.dim, device)
            self.own_acc = [big(), big()]
            self.peer_acc = [[big(), big()] for _ in range(cfg.peers)]
        if bf16_messages:
            n = max(cfg.grad_buffer, 1)
            msg = lambda: B.PackedBuffers(min(cfg.vocab, n * self.own.cap_in), min(cfg.vocab, n * self.own.cap_out),
                                          cfg.dim, device)
            self.peer_msgs = [msg() for _ in range(cfg.peers)]
            self.own_msg = msg()         # what this worker broadcasts

    # -- peers -------------------------------------------------------------
    def _snapshot(self, t):
        if self.cfg.peers == 0:
            return
        if self.cfg.max_stale == 0:
            self.snapshots = {t: (self.model.w_in, self.model.w_out)}   # only theta_t itself is used
            return
        self.snapshots[t] = (self.model.w_in.clone(), self.model.w_out.clone())
        for old in [s for s in self.snapshots if s < t - self.cfg.max_stale]:
            del self.snapshots[old]

    def make_peer_grads(self, t, n_steps_hint=4096):
        """Gradients of peers 1..K for step t, each on theta_{max(0, t - staleness)}."""
        cfg = self.cfg
        if self.stale is None or self.stale.shape[0] <= t:
            self.stale = W.stale_draws(cfg, max(n_steps_hint, t + 1))
        self._snapshot(t)
        for k in range(1, cfg.peers + 1):
            s = int(self.stale[t, k - 1])
            w_in, w_out = self.snapshots[max(0, t - s)]
            begin, n, epoch = W.worker_batch(cfg, t, k)
            self.peer_model.rebind(w_in, w_out, k)
            self.peer_model.sgns_grad(self.tokens, begin, n, epoch, self.peer_bufs[k - 1])
        out = self._buffer_peers(t) if cfg.grad_buffer > 1 else self.peer_bufs
        if self.bf16_messages:     # what a peer sends is rounded once, after any summing in its buffer
            for g, msg in zip(out, self.peer_msgs):
                self.model.grad_pack(g, msg)
            out = self.peer_msgs[:len(out)]
        return out

    def _accumulate(self, pair, g, first):
        """pair[0] <- pair[0] + g (gradients += gradient); an empty sum at the start of a window."""
        if first:
            pair[0].n_rows.zero_()
        self.model.grad_add(pair[0], g, pair[1])
        pair[0], pair[1] = pair[1], pair[0]

    def _buffer_peers(self, t):
        n = self.cfg.grad_buffer
        for k in range(self.cfg.peers):
            self._accumulate(self.peer_acc[k], self.peer_bufs[k], t % n == 0)
        return [p[0] for p in self.peer_acc] if (t + 1) % n == 0 else []

    # -- one step -----------------------------------------------------------
    def step(self, peers=None, want_loss=False):
        """tensair_step for this worker's mini-batch of the current step."""
        cfg = self.cfg
        t = self.step_no
        if peers is None:
            peers = self.make_peer_grads(t) if cfg.peers else []
        begin, n, epoch = W.worker_batch(cfg, t, 0)
        # the worker's coming mini-batches are already waiting in its input queue: once this step's
        # mini-batch has been announced, the next one is announced before the step, so that the library
        # prepares it during the step
        if self.prefetch and self.announced == t:
            self._announce(t + 1)
        loss = self.mean_loss if want_loss else None
        if self.bf16_messages:
            # without a buffer the own gradient is what this worker sends: it leaves the step as a message too
            msg = self.own_msg if cfg.grad_buffer == 1 else None
            self.model.step_packed(self.tokens, begin, n, epoch, peers, cfg.lr, self.own, msg, loss)
        else:
            self.model.step(self.tokens, begin, n, epoch, peers, cfg.lr, self.own, loss)
        if cfg.grad_buffer > 1:
            self._accumulate(self.own_acc, self.own, t % cfg.grad_buffer == 0)
            if (t + 1) % cfg.grad_buffer == 0:
                self.sent = self.own_acc[0]      # what this worker would broadcast now
                if self.bf16_messages:
                    self.model.grad_pack(self.sent, self.own_msg)
        self.step_no += 1
        if self.prefetch and self.announced < t + 1:
            self._announce(t + 1)
        return begin, n, epoch

    def _announce(self, t):
        begin, n, epoch = W.worker_batch(self.cfg, t, 0)
        self.model.prefetch(self.tokens, begin, n, epoch)
        self.announced = t

    def restart(self):
        """Back to step 0 (the tables are the caller's business); pending announcements no longer
        match and are dropped by the library at the next step."""
        self.step_no = 0
        self.announced = -1

    def tables_to_host(self):
        """The two tables without their padding columns, as numpy arrays (bf16 as uint16 bits)."""
        D = self.cfg.dim
        w_in, w_out = self.model.w_in[:, :D].contiguous(), self.model.w_out[:, :D].contiguous()
        if self.cfg.dtype == "bf16":
            return (w_in.view(torch.int16).cpu().numpy().view(np.uint16),
                    w_out.view(torch.int16).cpu().numpy().view(np.uint16))
        return w_in.cpu().numpy(), w_out.cpu().numpy()

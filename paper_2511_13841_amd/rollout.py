"""A batch of sequences on the GPU plus the seeded synthetic drafter that feeds it.

Used by bench.py and by the measurement tools of this package (latency model fit, rollout makespan).
Everything that computes runs behind the C ABI; this class only prepares inputs and keeps the
host-side bookkeeping of a rollout (current lengths, what has been emitted, what the drafter proposes).
"""
import sys
import time

import numpy as np

import das_inputs as di


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Rollout:
    """A batch of sequences on the GPU plus the synthetic drafter that feeds it."""

    def __init__(self, wl, batch=None, n_layers=None, context="synth", seed=None, max_steps=32, kmax=None):
        from . import binding as das
        self.wl = wl
        shape = di.MODELS[wl.model]
        if n_layers is not None:
            shape = shape.replace(n_layers=n_layers)
        self.shape = shape
        self.B = wl.batch if batch is None else batch
        self.seed = wl.seed if seed is None else seed
        self.ctx0 = di.context_lengths(wl, batch=self.B, seed=self.seed)
        self.kmax = di.max_budget(wl) if kmax is None else kmax
        grow = max_steps * (self.kmax + 1) + self.kmax + 2
        self.horizon = grow
        pages = int(sum(-(-(int(c) + grow) // 16) for c in self.ctx0)) + 64
        max_ctx = -(-(int(self.ctx0.max()) + grow + 16) // 16) * 16
        # (a prefill pass takes up to max_rows prompt tokens and streams the weights once: room for 2048 of them)
        max_rows = max(self.B * (self.kmax + 1), 2048 if context == "prefill" else 256)
        # random-init weights N(0, 0.02^2) from seed 0, drawn on the device by the library (the same values as
        # das_inputs.weights_bf16(shape, 0), which is generated on the host only if somebody asks for `blob`)
        self._blob = None
        t0 = time.time()
        self.dm = das.DasModel(das.config_for(shape, max_seqs=self.B, max_ctx=max_ctx, max_rows=max_rows,
                                              max_draft=self.kmax, num_pages=pages), None, seed=0)
        log(f"[rollout] model initialised and packed on the device in {time.time() - t0:.1f}s; KV pool {pages} pages "
            f"({pages * 16 * shape.kv_bytes_per_token / 1e9:.1f} GB)")
        self.ids = list(range(self.B))
        rng = np.random.default_rng(self.seed + 17)
        t0 = time.time()
        if context == "prefill":
            prompts = di.prompts(self.ctx0, shape.vocab, self.seed)
            self.pending0 = self.dm.prefill(self.ids, prompts)
        else:
            self.pending0 = rng.integers(0, shape.vocab, size=self.B, dtype=np.int32)
            for i in self.ids:
                self.dm.seq_create(i, int(self.ctx0[i]), int(self.pending0[i]))
                self.dm.kv_synth(i, self.seed, i)
        self.context_s = time.time() - t0
        log(f"[rollout] contexts ({context}): {int(self.ctx0.sum())} tokens in {self.context_s:.1f}s")
        self.ctx = self.ctx0.copy()
        self.pending = self.pending0.copy()
        self.future = None
        self.faithful = False
        self.rollback = False            # time the verify pass alone: every step is rolled back instead of committed

    @property
    def blob(self):
        """The canonical weight blob of the same model on the host (for a CPU baseline)."""
        if self._blob is None:
            t0 = time.time()
            self._blob = di.weights_bf16(self.shape, seed=0)
            log(f"[rollout] host copy of the weights ({self._blob.size * 2 / 1e9:.2f} GB) generated in {time.time() - t0:.1f}s")
        return self._blob

    def close(self):
        self.dm.free()
        self._blob = None

    def generate_trajectories(self):
        """Plain decoding (k=0 verify steps) for `horizon` tokens, then rewind.  future[i][0] is the pending token."""
        t0 = time.time()
        fut = np.empty((self.B, self.horizon + 1), np.int32)
        fut[:, 0] = self.pending0
        empty = [[] for _ in self.ids]
        for t in range(self.horizon):
            acc, nxt = self.dm.verify_step(self.ids, self.ctx0 + t, empty)
            self.dm.kv_commit(self.ids, acc, nxt)
            fut[:, t + 1] = nxt
        self.dm.seq_rewind(self.ids, self.ctx0, self.pending0)
        self.future = fut
        # the drafter's proposals: the true continuation with every position independently kept with
        # probability p (a contiguous copy out of this buffer is what a suffix match would return)
        rng = np.random.default_rng(self.seed + 29)
        bad = rng.random(fut.shape) >= self.wl.accept_p
        self.proposal = np.where(bad, rng.integers(0, self.shape.vocab, size=fut.shape, dtype=np.int32), fut)
        self.emitted = np.ones(self.B, np.int64)       # trajectory tokens decided so far (the pending one)
        log(f"[rollout] {self.horizon} plain decode steps for the drafter in {time.time() - t0:.1f}s "
            f"({(time.time() - t0) / self.horizon * 1e3:.2f} ms/step)")

    def random_proposals(self):
        rng = np.random.default_rng(self.seed + 31)
        self.proposal = rng.integers(0, self.shape.vocab, size=(self.B, self.horizon + 1), dtype=np.int32)
        self.emitted = np.ones(self.B, np.int64)

    def sampling_inputs(self, ks):
        """Seeded uniforms of a stochastic step, one pair per row, keyed by (sequence, absolute position).
        Controlled mode: a draft position is force-accepted (u_accept = 0) with the drafter's probability p,
        otherwise judged honestly (p_target of a random token under random-init weights is ~1e-5)."""
        keys = np.repeat(np.arange(self.B), ks + 1)
        pos = np.concatenate([np.arange(c, c + k + 1) for c, k in zip(self.ctx, ks)])
        ua = di.uniforms(self.seed, keys, pos, 0)
        us = di.uniforms(self.seed, keys, pos, 1)
        if not self.faithful:
            force = di.uniforms(self.seed, keys, pos, 2) < self.wl.accept_p
            ua = np.where(force, 0.0, ua).astype(np.float32)
        return (self.wl.temperature, ua, us)

    def step(self, sampling=None):
        ks = di.draft_budgets(self.wl, self.ctx)
        drafts = [self.proposal[i, self.emitted[i]:self.emitted[i] + ks[i]] for i in range(self.B)]
        if sampling is None and self.wl.mode == "stochastic":
            sampling = self.sampling_inputs(ks)
        acc, nxt = self.dm.verify_step(self.ids, self.ctx, drafts, sampling)
        if self.rollback:
            self.dm.kv_rollback(self.ids)
            return ks, acc, nxt
        self.dm.kv_commit(self.ids, acc, nxt)
        self.ctx = self.ctx + 1 + acc
        self.emitted += 1 + acc
        self.pending = nxt
        return ks, acc, nxt

    def step_shape(self):
        ks = di.draft_budgets(self.wl, self.ctx)
        return int((ks + 1).sum()), int((self.ctx.astype(np.int64) + 1 + ks).sum())

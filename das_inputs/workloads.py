"""Model shapes and the five synthetic workloads (lengths, budgets, drafts).

Every recipe is seeded.  The shapes stand in for the rollouts of the paper's
math and code RL runs (Sec. 5), which are not available offline; only the
long-tailed shape of the length distribution (Sec. 3, Fig. 1) is kept.
"""
from dataclasses import dataclass
import numpy as np


@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_theta: float = 1.0e6
    rms_eps: float = 1.0e-6

    def replace(self, **kw):
        d = dict(self.__dict__)
        d.update(kw)
        return ModelShape(**d)

    @property
    def kv_bytes_per_token(self):
        return self.n_layers * 2 * self.n_kv_heads * self.head_dim * 2

    @property
    def layer_params(self):
        d, qd, kd = self.d_model, self.n_q_heads * self.head_dim, self.n_kv_heads * self.head_dim
        return d * (qd + 2 * kd) + qd * d + 3 * d * self.d_ffn

    @property
    def streamed_params(self):
        """matrix parameters read once per forward (layers + LM head)"""
        return self.n_layers * self.layer_params + self.vocab * self.d_model


MODELS = {
    "tiny": ModelShape("tiny", 2, 256, 4, 2, 64, 688, 2048, rope_theta=1.0e4),
    "1.5b": ModelShape("1.5b", 28, 1536, 12, 2, 128, 8960, 151936),
    "7b": ModelShape("7b", 28, 3584, 28, 4, 128, 18944, 151936),
}


@dataclass(frozen=True)
class Workload:
    name: str
    config_id: int
    model: str
    batch: int
    accept_p: float
    mode: str            # "greedy" | "stochastic"
    lengths: str         # recipe name
    budgets: str         # recipe name
    temperature: float = 1.0

    @property
    def seed(self):
        return 1000 + self.config_id


WORKLOADS = {
    "c1": Workload("c1", 1, "tiny", 4, 0.7, "greedy", "uniform16_64", "k4"),
    "c2": Workload("c2", 2, "1.5b", 64, 0.6, "greedy", "lognormal2048", "k4"),
    "c3": Workload("c3", 3, "7b", 128, 0.7, "greedy", "mix_1k4k_16k32k", "quartile"),
    "c4": Workload("c4", 4, "7b", 16, 0.8, "greedy", "uniform32k_64k", "k16"),
    "c5": Workload("c5", 5, "7b", 256, 0.7, "stochastic", "pareto512", "loglen"),
}


def workload(name):
    return WORKLOADS[name]


def context_lengths(wl, batch=None, seed=None):
    """Committed context length of every sequence of the batch (int32[B])."""
    B = wl.batch if batch is None else batch
    rng = np.random.default_rng(wl.seed if seed is None else seed)
    r = wl.lengths
    if r == "uniform16_64":
        n = rng.integers(16, 65, size=B)
    elif r == "lognormal2048":
        n = np.clip(np.rint(np.exp(np.log(2048.0) + rng.standard_normal(B))), 256, 16384)
    elif r == "mix_1k4k_16k32k":
        n_tail = int(round(0.1 * B))
        short = rng.integers(1024, 4097, size=B - n_tail)
        tail = rng.integers(16384, 32769, size=n_tail)
        n = np.concatenate([short, tail])
        rng.shuffle(n)
    elif r == "uniform32k_64k":
        n = rng.integers(32768, 65537, size=B)
    elif r == "pareto512":
        u = rng.random(B)
        n = np.minimum(np.floor(512.0 * (1.0 - u) ** (-1.0 / 1.5)), 32768)
    else:
        raise ValueError(r)
    return n.astype(np.int32)


def draft_budgets(wl, ctx_lens):
    """Per-sequence draft budget k_i from the current lengths (int32[B])."""
    c = np.asarray(ctx_lens, dtype=np.int64)
    r = wl.budgets
    if r[0] == "k" and r[1:].isdigit():            # uniform chains: "k4", "k16", ...
        return np.full(c.shape, int(r[1:]), np.int32)
    if r == "quartile":
        # rank by current length within the batch; shortest quartile -> 2 ... longest -> 16
        order = np.argsort(c, kind="stable")
        rank = np.empty_like(order)
        rank[order] = np.arange(c.size)
        q = (rank * 4) // c.size
        return np.array([2, 4, 8, 16], np.int32)[q]
    if r == "loglen":
        k = np.floor(32.0 * np.log2(np.maximum(c, 1) / 512.0) / 6.0)
        return np.clip(k, 0, 32).astype(np.int32)
    raise ValueError(r)


def max_budget(wl):
    """Largest k_i the workload's budget recipe can return."""
    r = wl.budgets
    if r[0] == "k" and r[1:].isdigit():
        return int(r[1:])
    return {"quartile": 16, "loglen": 32}[r]


def prompts(lengths, vocab, seed):
    """Uniform random prompt tokens; returns a list of int32 arrays."""
    rng = np.random.default_rng(seed)
    return [rng.integers(0, vocab, size=int(n), dtype=np.int32) for n in lengths]


def make_drafts(future, k, p, vocab, rng):
    """Chain draft of length k: the true continuation `future[:k]` with every
    position independently replaced by a uniform random token with prob 1-p."""
    k = int(k)
    d = np.array(future[:k], dtype=np.int32)
    assert d.size == k, "trajectory too short for the requested draft"
    bad = rng.random(k) >= p
    d[bad] = rng.integers(0, vocab, size=int(bad.sum()), dtype=np.int32)
    return d


def corrupt_history(traj, p, vocab, rng):
    """Repeated-span history: the trajectory with every token kept with prob p;
    a draft is then a contiguous copy out of it, as a suffix match would give."""
    h = np.array(traj, dtype=np.int32)
    bad = rng.random(h.size) >= p
    h[bad] = rng.integers(0, vocab, size=int(bad.sum()), dtype=np.int32)
    return h


def expected_accept_len(p, k, vocab):
    """E[accepted drafts] for independent per-position correctness p' = p+(1-p)/V."""
    pp = p + (1.0 - p) / vocab
    if k == 0:
        return 0.0
    return pp * (1.0 - pp ** k) / (1.0 - pp)

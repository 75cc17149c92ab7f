"""CPU oracle, decoding logic -- TEST INFRASTRUCTURE ONLY.

The model forward lives in das_oracle.c (fp32 values, fp64 reductions).  This
file writes out, on top of it, what the verification step of DAS must return:

* plain autoregressive decoding, one token per forward -- the definition the
  method must reproduce (abstract, Sec. 5.1, Sec. 6: speculation does not
  change the model's outputs);
* the speculative round (Sec. 3, Fig. 3 right, Sec. 4.1.2): the target scores
  the pending token and the k draft tokens in one pass; the longest draft
  prefix that plain decoding would also have produced is accepted and the
  target's own token after it is emitted;
* for sampled rollouts, the rejection rule of speculative sampling that the
  paper cites (Sec. 2, Leviathan et al.), specialised to a deterministic
  (point-mass) drafter: accept draft x with probability p_target(x); on the
  first rejection resample from the target distribution with x removed and
  renormalised; if every draft is accepted sample the bonus token from p.

Readings taken where the paper is silent are listed in the repository's design
notes (ties -> lowest index; inverse CDF in ascending vocabulary order).
"""
import ctypes as C
import os
import subprocess
import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libdas_oracle.so")
_lib = None


class _Cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] + \
               [("rope_theta", C.c_float), ("rms_eps", C.c_float)]


def build(force=True):
    src = os.path.join(_HERE, "das_oracle.c")
    if not force and os.path.exists(_SO) and os.path.getmtime(_SO) >= os.path.getmtime(src):
        return _SO
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-mavx2", "-mfma", "-shared", "-fPIC", "-o", _SO, src, "-lm"])
    return _SO


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            build()
        lib = C.CDLL(_SO)
        lib.orc_model_create.restype = C.c_void_p
        lib.orc_model_create.argtypes = [C.POINTER(_Cfg), C.c_void_p]
        lib.orc_model_destroy.argtypes = [C.c_void_p]
        lib.orc_seq_create.restype = C.c_void_p
        lib.orc_seq_create.argtypes = [C.c_void_p, C.c_int32]
        lib.orc_seq_destroy.argtypes = [C.c_void_p]
        lib.orc_seq_kv.restype = C.c_void_p
        lib.orc_seq_kv.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32]
        lib.orc_forward.restype = C.c_int
        lib.orc_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p]
        lib.orc_num_threads.restype = C.c_int32
        lib.orc_op_rmsnorm.argtypes = [C.c_void_p, C.c_void_p, C.c_float, C.c_int32, C.c_void_p]
        lib.orc_op_rope.argtypes = [C.c_void_p, C.c_int32, C.c_int64, C.c_double]
        lib.orc_op_linear.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_int32]
        _lib = lib
    return _lib


def num_threads():
    return int(_load().orc_num_threads())


# --------------------------------------------------------------------------- acceptance rules

def greedy_accept(g, drafts):
    """g[j] = target's greedy token after row j (rows 0..k); drafts d_1..d_k.
    Returns (a, next): the longest prefix with d_j == g[j-1] and the target's
    token after it."""
    a = 0
    k = len(drafts)
    while a < k and int(drafts[a]) == int(g[a]):
        a += 1
    return a, int(g[a])


def softmax_weights(logits_row, tau):
    """Unnormalised target weights w_v = exp(l_v/tau - max) in fp64, and Z."""
    x = np.asarray(logits_row, dtype=np.float64) / float(tau)
    w = np.exp(x - x.max())
    return w, float(w.sum())


def inverse_cdf(w, u):
    """Smallest index v with sum_{y<=v} w_y > u * sum(w); clamped to the last
    index of non-zero weight."""
    cs = np.cumsum(w)
    v = int(np.searchsorted(cs, float(u) * cs[-1], side="right"))
    last = int(np.nonzero(w)[0][-1])
    return min(v, last)


def stochastic_accept(logits, drafts, tau, u_accept, u_sample):
    """Rejection-sampling verification of a deterministic chain draft.
    logits[j] (rows 0..k), drafts d_1..d_k, one uniform per row for the accept
    test (row j tests d_{j+1}) and one for sampling.  Returns (a, next)."""
    k = len(drafts)
    for j in range(k):
        w, Z = softmax_weights(logits[j], tau)
        d = int(drafts[j])
        if float(u_accept[j]) * Z < w[d]:
            continue                      # accepted with probability p(d)
        w = w.copy()
        w[d] = 0.0                        # residual max(0, p - delta_d), renormalised by inverse_cdf
        return j, inverse_cdf(w, u_sample[j])
    w, _ = softmax_weights(logits[k], tau)
    return k, inverse_cdf(w, u_sample[k])


# --------------------------------------------------------------------------- model + sequences

class OracleSeq:
    """One sequence: dense KV of `cap` positions, `len` committed, one pending token."""

    def __init__(self, model, cap):
        self.model = model
        self.cap = int(cap)
        self.h = _load().orc_seq_create(model.h, self.cap)
        if not self.h:
            raise MemoryError("oracle KV allocation failed")
        self.len = 0
        self.pending = -1
        self.tokens = []          # every token whose KV is committed

    def kv(self, layer, which):
        s = self.model.shape
        ptr = _load().orc_seq_kv(self.model.h, self.h, layer, which)
        n = self.cap * s.n_kv_heads * s.head_dim
        return np.ctypeslib.as_array(C.cast(ptr, C.POINTER(C.c_float)), shape=(n,)).reshape(
            self.cap, s.n_kv_heads, s.head_dim)

    def close(self):
        if self.h:
            _load().orc_seq_destroy(self.h)
            self.h = None

    def __del__(self):
        self.close()


class OracleModel:
    def __init__(self, shape, weights_f32):
        self.shape = shape
        self.w = np.ascontiguousarray(weights_f32, dtype=np.float32)   # kept alive: borrowed by C
        cfg = _Cfg(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                   shape.d_ffn, shape.vocab, shape.rope_theta, shape.rms_eps)
        self.h = _load().orc_model_create(C.byref(cfg), self.w.ctypes.data)

    def close(self):
        if self.h:
            _load().orc_model_destroy(self.h)
            self.h = None

    def __del__(self):
        self.close()

    def new_seq(self, cap):
        return OracleSeq(self, cap)

    def forward(self, seq, start_pos, tokens, first_logit_row=0):
        """Rows start_pos.. of `seq` (KV written, nothing committed); logits of rows >= first_logit_row."""
        tok = np.ascontiguousarray(tokens, dtype=np.int32)
        n = tok.size
        out = np.empty((n - first_logit_row, self.shape.vocab), dtype=np.float32)
        rc = _load().orc_forward(self.h, seq.h, int(start_pos), n, tok.ctypes.data, int(first_logit_row),
                                 out.ctypes.data)
        if rc != 0:
            raise ValueError("orc_forward: bad argument")
        return out

    # -- plain definition -------------------------------------------------
    def prefill(self, seq, prompt):
        """KV for the whole prompt; returns the last position's logits.  The caller
        decides the first pending token from them (argmax or a sample)."""
        logits = self.forward(seq, 0, prompt, first_logit_row=len(prompt) - 1)[0]
        seq.len = len(prompt)
        seq.tokens = [int(t) for t in prompt]
        return logits

    def ar_greedy(self, seq, n_tokens):
        """Plain decoding: n_tokens forwards of one token each, from (len, pending).
        Returns the tokens emitted after the pending one."""
        out = []
        for _ in range(n_tokens):
            logits = self.forward(seq, seq.len, [seq.pending])[0]
            self.commit(seq, 0, int(np.argmax(logits)), [])
            out.append(seq.pending)
        return out

    # -- the speculative round ---------------------------------------------
    def verify_logits(self, seq, drafts):
        """One pass over [pending, d_1..d_k] at positions len..len+k."""
        toks = [seq.pending] + [int(t) for t in drafts]
        return self.forward(seq, seq.len, toks)

    def verify_greedy(self, seq, drafts):
        logits = self.verify_logits(seq, drafts)
        g = np.argmax(logits, axis=1)            # first maximum = lowest index on ties
        a, nxt = greedy_accept(g, drafts)
        return a, nxt, logits

    def verify_stochastic(self, seq, drafts, tau, u_accept, u_sample):
        logits = self.verify_logits(seq, drafts)
        a, nxt = stochastic_accept(logits, drafts, tau, u_accept, u_sample)
        return a, nxt, logits

    def commit(self, seq, a, next_token, drafts):
        """Accepted tokens advance generation: KV of the pending token and of the
        first `a` drafts is kept, the rest of the block is discarded."""
        seq.tokens += [seq.pending] + [int(t) for t in drafts[:a]]
        seq.len += 1 + a
        seq.pending = int(next_token)

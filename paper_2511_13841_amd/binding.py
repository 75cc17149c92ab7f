"""ctypes binding of include/das.h.  Same names, argument marshalling only."""
import ctypes as C
import os
import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libdas.so")

DAS_OK, DAS_ERR_INVALID, DAS_ERR_STATE, DAS_ERR_NOMEM, DAS_ERR_DEVICE = 0, -1, -2, -3, -4


class DasError(RuntimeError):
    def __init__(self, code, what):
        self.code = code
        msg = f"{what}: {lib().das_strerror(code).decode()} ({code})"
        if code == DAS_ERR_DEVICE:
            msg += " -- " + lib().das_last_device_error().decode()
        super().__init__(msg)


class das_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] + \
               [("rope_theta", C.c_float), ("rms_eps", C.c_float)] + \
               [(n, C.c_int32) for n in ("page_size", "max_seqs", "max_ctx", "max_rows", "max_draft")] + \
               [("num_pages", C.c_int64)]


class das_sampling(C.Structure):
    _fields_ = [("temperature", C.c_float), ("u_accept", C.c_void_p), ("u_sample", C.c_void_p)]


_lib = None


def lib():
    """The loaded libdas.so.  There is no fallback: a missing library is an error."""
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            raise ImportError(f"{_SO} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                              "(hipcc --offload-arch=gfx950); there is no CPU fallback")
        try:                # PyTorch ships its own HIP runtime: let it load first, so that this library binds to the same one
            import torch    # noqa: F401  (loading the library first and torch afterwards leaves the process with two runtimes and no device)
        except Exception:
            pass
        L = C.CDLL(_SO)
        P, I, VP = C.c_void_p, C.c_int32, C.c_void_p
        sig = {
            "das_model_load": [C.POINTER(das_config), C.c_uint64, VP, VP, C.POINTER(P)],
            "das_model_free": [P],
            "das_prefill": [P, I, VP, VP, VP, C.POINTER(das_sampling), VP],
            "das_verify_step": [P, I, VP, VP, VP, VP, C.POINTER(das_sampling), VP, VP],
            "das_kv_commit": [P, I, VP, VP, VP],
            "das_kv_rollback": [P, I, VP],
            "das_seq_free": [P, I, VP],
            "das_seq_rewind": [P, I, VP, VP, VP],
            "das_seq_create": [P, I, I, I],
            "das_kv_import": [P, I, I, I, I, VP, VP],
            "das_kv_export": [P, I, I, I, I, VP, VP],
            "das_kv_synth": [P, I, C.c_uint64, C.c_uint64],
            "das_debug_num_rows": [P, C.POINTER(I)],
            "das_debug_keep_logits": [P, I],
            "das_debug_logits": [P, I, I, VP],
            "das_debug_row_argmax": [P, VP],
            "das_debug_seq": [P, I, C.POINTER(I), C.POINTER(I), C.POINTER(I), VP, C.POINTER(I)],
            "das_debug_free_pages": [P, C.POINTER(C.c_int64)],
            "das_debug_kv_saturated": [P, C.POINTER(C.c_int64)],
            "das_debug_gemm_time": [I, I, I, I, I, I, I, C.POINTER(C.c_double)],
            "das_debug_gemm": [I, I, I, VP, VP, VP],
            "das_debug_gemm_epilogues": [I, I, VP, I, VP, VP, VP, I, VP, VP],
            "das_gemm_noalloc": [I, I, I, VP, VP, VP, VP],
            "das_debug_copy": [C.c_int64, I],
            "das_debug_copy_ring": [I, I, I, I, I, I, C.POINTER(C.c_double), C.POINTER(C.c_double)],
            "das_debug_mfma_loop": [I, I, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_double)],
            "das_profile_enable": [P, I],
            "das_profile_reset": [P],
            "das_profile_read": [P, I, C.POINTER(C.c_double), C.POINTER(C.c_int64)],
        }
        for name, args in sig.items():
            f = getattr(L, name)
            f.argtypes = args
            f.restype = C.c_int
        L.das_profile_name.argtypes = [I]
        L.das_profile_name.restype = C.c_char_p
        L.das_strerror.argtypes = [C.c_int]
        L.das_strerror.restype = C.c_char_p
        L.das_last_device_error.argtypes = []
        L.das_last_device_error.restype = C.c_char_p
        _lib = L
    return _lib


def _chk(code, what):
    if code != DAS_OK:
        raise DasError(code, what)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def config_for(shape, max_seqs, max_ctx, max_rows, max_draft, num_pages):
    """das_config from a model shape (any object with the seven dimension fields, rope_theta, rms_eps)."""
    return das_config(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn,
                      shape.vocab, shape.rope_theta, shape.rms_eps, 16, max_seqs, max_ctx, max_rows, max_draft,
                      num_pages)


def kernel_classes():
    """Names of the kernel classes das_profile_read reports, in index order."""
    out, i = [], 0
    while True:
        n = lib().das_profile_name(i)
        if n is None:
            return out
        out.append(n.decode())
        i += 1


def debug_gemm(a_bf16, w_bf16):
    a = np.ascontiguousarray(a_bf16, dtype=np.uint16)
    w = np.ascontiguousarray(w_bf16, dtype=np.uint16)
    M, K = a.shape
    N = w.shape[0]
    c = np.empty((M, N), np.float32)
    _chk(lib().das_debug_gemm(M, N, K, a.ctypes.data, w.ctypes.data, c.ctypes.data), "das_debug_gemm")
    return c


def gemm_noalloc(M, N, K, a_dev, w_dev, c_dev, stream=None):
    """das_gemm_noalloc on raw device addresses (ints): enqueues on `stream`, does not synchronise, allocates nothing."""
    _chk(lib().das_gemm_noalloc(int(M), int(N), int(K), C.c_void_p(int(a_dev)), C.c_void_p(int(w_dev)), C.c_void_p(int(c_dev)),
                                C.c_void_p(int(stream or 0))), "das_gemm_noalloc")


def debug_gemm_silu(a_bf16, wg_bf16, wu_bf16):
    """silu(a wg^T) * (a wu^T) through the gate/up GEMM; the kernel's bf16 result as fp32 [M][F]."""
    a = np.ascontiguousarray(a_bf16, dtype=np.uint16)
    wg = np.ascontiguousarray(wg_bf16, dtype=np.uint16)
    wu = np.ascontiguousarray(wu_bf16, dtype=np.uint16)
    M, K = a.shape
    F = wg.shape[0]
    out = np.empty((M, F), np.float32)
    _chk(lib().das_debug_gemm_epilogues(M, K, a.ctypes.data, F, wg.ctypes.data, wu.ctypes.data, out.ctypes.data, 0, None, None),
         "das_debug_gemm_epilogues")
    return out


def debug_gemm_rowmax(a_bf16, w_bf16):
    """Lowest column of every row's maximum of a w^T through the LM-head GEMM that writes no logits."""
    a = np.ascontiguousarray(a_bf16, dtype=np.uint16)
    w = np.ascontiguousarray(w_bf16, dtype=np.uint16)
    M, K = a.shape
    col = np.empty(M, np.int32)
    _chk(lib().das_debug_gemm_epilogues(M, K, a.ctypes.data, 0, None, None, None, w.shape[0], w.ctypes.data, col.ctypes.data),
         "das_debug_gemm_epilogues")
    return col


def debug_gemm_time(epi, M, N, K, iters=20, weight_sets=4, copies_only=False):
    """Mean device time (us) of one projection GEMM launch of this shape; epi: 1 residual, 2 gate/up, 3 fp32 out, 4 row max.
    copies_only: the same launches with the arithmetic switched off (tile copies and barriers only)."""
    us = C.c_double()
    _chk(lib().das_debug_gemm_time(int(epi), int(M), int(N), int(K), int(iters), int(weight_sets), int(bool(copies_only)), C.byref(us)),
         "das_debug_gemm_time")
    return us.value


def debug_copy_ring(workgroups, stages, copies, shared_copies, tiles=256, non_temporal=False):
    """The kernels' HBM/L2 -> LDS copy ring by itself: (us per launch, bytes copied into LDS by one launch)."""
    us, nb = C.c_double(), C.c_double()
    _chk(lib().das_debug_copy_ring(int(workgroups), int(stages), int(copies), int(shared_copies), int(tiles), int(bool(non_temporal)),
                                   C.byref(us), C.byref(nb)), "das_debug_copy_ring")
    return us.value, nb.value


def debug_mfma_loop(mode, iters=4000):
    """The matrix pipe by itself (mode 0 register operands, 1 operands from LDS, 2 with the GEMM's copy traffic):
    (ns per MFMA and SIMD, shader clock in GHz, PFLOP/s of the launch)."""
    ns, ghz, pf = C.c_double(), C.c_double(), C.c_double()
    _chk(lib().das_debug_mfma_loop(int(mode), int(iters), C.byref(ns), C.byref(ghz), C.byref(pf)), "das_debug_mfma_loop")
    return ns.value, ghz.value, pf.value


def debug_copy(nbytes, repeats=1):
    _chk(lib().das_debug_copy(int(nbytes), int(repeats)), "das_debug_copy")


class DasModel:
    """Owner of one das_model handle.  Methods carry the C names without the das_ prefix."""

    def __init__(self, cfg, weights_bf16=None, stream=None, keep_logits=False, seed=0):
        """weights_bf16: the canonical blob, or None to let the library draw N(0, 0.02^2) weights from `seed` on the device."""
        self.cfg = cfg
        w = np.ascontiguousarray(weights_bf16, dtype=np.uint16) if weights_bf16 is not None else None
        h = C.c_void_p()
        if stream is None:
            try:                                   # PyTorch only lends its current HIP stream
                import torch
                if torch.cuda.is_available():
                    stream = torch.cuda.current_stream().cuda_stream
            except Exception:
                stream = None
        _chk(lib().das_model_load(C.byref(cfg), int(seed), w.ctypes.data if w is not None else None, C.c_void_p(stream or 0), C.byref(h)),
             "das_model_load")
        self.h = h
        if keep_logits:
            self.keep_logits(True)

    def free(self):
        if getattr(self, "h", None):
            lib().das_model_free(self.h)
            self.h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass

    @staticmethod
    def _samp(sampling):
        if sampling is None:
            return None, ()
        temp, ua, us = sampling
        us = np.ascontiguousarray(us, dtype=np.float32)
        ua = np.ascontiguousarray(ua, dtype=np.float32) if ua is not None else None
        s = das_sampling(float(temp), ua.ctypes.data if ua is not None else None, us.ctypes.data)
        return C.byref(s), (s, ua, us)

    def prefill(self, seq_ids, prompts, sampling=None):
        ids = _i32(seq_ids)
        lens = _i32([len(p) for p in prompts])
        toks = _i32(np.concatenate([np.asarray(p, dtype=np.int32) for p in prompts])) if len(prompts) else _i32([])
        nxt = np.empty(len(ids), np.int32)
        sp, keep = self._samp(sampling)
        _chk(lib().das_prefill(self.h, len(ids), ids.ctypes.data, toks.ctypes.data, lens.ctypes.data, sp, nxt.ctypes.data),
             "das_prefill")
        return nxt

    def verify_step(self, seq_ids, ctx_lens, drafts, sampling=None):
        """drafts: list of per-sequence token arrays.  Returns (accept_len, next_token)."""
        ids, ctx = _i32(seq_ids), _i32(ctx_lens)
        dl = _i32([len(d) for d in drafts])
        flat = [np.asarray(d, dtype=np.int32) for d in drafts if len(d)]
        dt = _i32(np.concatenate(flat)) if flat else _i32([0])
        acc, nxt = np.empty(len(ids), np.int32), np.empty(len(ids), np.int32)
        sp, keep = self._samp(sampling)
        _chk(lib().das_verify_step(self.h, len(ids), ids.ctypes.data, ctx.ctypes.data, dt.ctypes.data, dl.ctypes.data, sp,
                                   acc.ctypes.data, nxt.ctypes.data), "das_verify_step")
        return acc, nxt

    def kv_commit(self, seq_ids, accept_lens, next_tokens):
        ids, a, t = _i32(seq_ids), _i32(accept_lens), _i32(next_tokens)
        _chk(lib().das_kv_commit(self.h, len(ids), ids.ctypes.data, a.ctypes.data, t.ctypes.data), "das_kv_commit")

    def kv_rollback(self, seq_ids):
        ids = _i32(seq_ids)
        _chk(lib().das_kv_rollback(self.h, len(ids), ids.ctypes.data), "das_kv_rollback")

    def seq_free(self, seq_ids):
        ids = _i32(seq_ids)
        _chk(lib().das_seq_free(self.h, len(ids), ids.ctypes.data), "das_seq_free")

    def seq_rewind(self, seq_ids, new_lens, pending_tokens):
        ids, l, t = _i32(seq_ids), _i32(new_lens), _i32(pending_tokens)
        _chk(lib().das_seq_rewind(self.h, len(ids), ids.ctypes.data, l.ctypes.data, t.ctypes.data), "das_seq_rewind")

    def seq_create(self, seq_id, ctx_len, pending):
        _chk(lib().das_seq_create(self.h, int(seq_id), int(ctx_len), int(pending)), "das_seq_create")

    def kv_import(self, seq_id, layer, first_pos, k, v):
        k = np.ascontiguousarray(k, dtype=np.uint16)
        v = np.ascontiguousarray(v, dtype=np.uint16)
        _chk(lib().das_kv_import(self.h, int(seq_id), int(layer), int(first_pos), k.shape[0], k.ctypes.data, v.ctypes.data),
             "das_kv_import")

    def kv_export(self, seq_id, layer, first_pos, n_pos):
        shp = (n_pos, self.cfg.n_kv_heads, self.cfg.head_dim)
        k, v = np.empty(shp, np.uint16), np.empty(shp, np.uint16)
        _chk(lib().das_kv_export(self.h, int(seq_id), int(layer), int(first_pos), int(n_pos), k.ctypes.data, v.ctypes.data),
             "das_kv_export")
        return k, v

    def kv_synth(self, seq_id, seed, seq_key):
        _chk(lib().das_kv_synth(self.h, int(seq_id), int(seed), int(seq_key)), "das_kv_synth")

    def keep_logits(self, on=True):
        """Make every later greedy pass write its fp32 logits (for debug_logits); by default the LM-head GEMM
        gathers the row argmax itself and the logits are never stored."""
        _chk(lib().das_debug_keep_logits(self.h, 1 if on else 0), "das_debug_keep_logits")

    def debug_num_rows(self):
        n = C.c_int32()
        _chk(lib().das_debug_num_rows(self.h, C.byref(n)), "das_debug_num_rows")
        return n.value

    def debug_logits(self, first_row=0, n_rows=None):
        if n_rows is None:
            n_rows = self.debug_num_rows() - first_row
        out = np.empty((n_rows, self.cfg.vocab), np.float32)
        _chk(lib().das_debug_logits(self.h, first_row, n_rows, out.ctypes.data), "das_debug_logits")
        return out

    def debug_row_argmax(self):
        out = np.empty(self.debug_num_rows(), np.int32)
        _chk(lib().das_debug_row_argmax(self.h, out.ctypes.data), "das_debug_row_argmax")
        return out

    def debug_seq(self, seq_id):
        c, p, s, n = C.c_int32(), C.c_int32(), C.c_int32(), C.c_int32()
        _chk(lib().das_debug_seq(self.h, int(seq_id), C.byref(c), C.byref(p), C.byref(s), None, C.byref(n)), "das_debug_seq")
        pages = np.empty(n.value, np.int32)
        _chk(lib().das_debug_seq(self.h, int(seq_id), None, None, None, pages.ctypes.data, None), "das_debug_seq")
        return dict(ctx_len=c.value, pending=p.value, state=s.value, pages=pages.tolist())

    def debug_kv_saturated(self):
        n = C.c_int64()
        _chk(lib().das_debug_kv_saturated(self.h, C.byref(n)), "das_debug_kv_saturated")
        return n.value

    def debug_free_pages(self):
        n = C.c_int64()
        _chk(lib().das_debug_free_pages(self.h, C.byref(n)), "das_debug_free_pages")
        return n.value

    def profile_enable(self, on=True):
        _chk(lib().das_profile_enable(self.h, 1 if on else 0), "das_profile_enable")

    def profile_reset(self):
        _chk(lib().das_profile_reset(self.h), "das_profile_reset")

    def profile_read(self):
        """{kernel class: (ms, launches)} since the last reset."""
        out = {}
        for i, name in enumerate(kernel_classes()):
            ms, n = C.c_double(), C.c_int64()
            _chk(lib().das_profile_read(self.h, i, C.byref(ms), C.byref(n)), "das_profile_read")
            out[name] = (ms.value, n.value)
        return out

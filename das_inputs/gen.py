"""ctypes front end of gen.c (weights, synthetic KV, uniforms, bf16 widening)."""
import ctypes as C
import os
import subprocess
import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libdas_inputs.so")
_lib = None


def build(force=True):
    """Compile gen.c into libdas_inputs.so next to this file."""
    src = os.path.join(_HERE, "gen.c")
    if not force and os.path.exists(_SO) and os.path.getmtime(_SO) >= os.path.getmtime(src):
        return _SO
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _SO, src, "-lm"])
    return _SO


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            build()
        lib = C.CDLL(_SO)
        lib.dasin_weight_count.restype = C.c_int64
        lib.dasin_weight_count.argtypes = [C.c_int32] * 7
        lib.dasin_weights_bf16.restype = None
        lib.dasin_weights_bf16.argtypes = [C.c_int32] * 7 + [C.c_uint64, C.c_double, C.c_double, C.c_void_p]
        lib.dasin_bf16_to_f32.restype = None
        lib.dasin_bf16_to_f32.argtypes = [C.c_void_p, C.c_void_p, C.c_int64]
        lib.dasin_f32_to_bf16.restype = None
        lib.dasin_f32_to_bf16.argtypes = [C.c_void_p, C.c_void_p, C.c_int64]
        lib.dasin_kv_synth.restype = None
        lib.dasin_kv_synth.argtypes = [C.c_uint64, C.c_uint64, C.c_int32, C.c_int32, C.c_int64, C.c_int64,
                                       C.c_int32, C.c_int32, C.c_void_p]
        lib.dasin_uniforms.restype = None
        lib.dasin_uniforms.argtypes = [C.c_uint64, C.c_int64, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
        lib.dasin_num_threads.restype = C.c_int32
        _lib = lib
    return _lib


def _dims(m):
    return (m.n_layers, m.d_model, m.n_q_heads, m.n_kv_heads, m.head_dim, m.d_ffn, m.vocab)


def weight_count(m):
    return int(_load().dasin_weight_count(*_dims(m)))


def weights_bf16(m, seed=0, sigma=0.02, gain_sigma=0.0):
    """Canonical bf16 weight blob (uint16 array) for model shape `m`."""
    out = np.empty(weight_count(m), dtype=np.uint16)
    _load().dasin_weights_bf16(*_dims(m), seed, float(sigma), float(gain_sigma), out.ctypes.data)
    return out


def bf16_to_f32(a):
    a = np.ascontiguousarray(a, dtype=np.uint16)
    out = np.empty(a.shape, dtype=np.float32)
    _load().dasin_bf16_to_f32(a.ctypes.data, out.ctypes.data, a.size)
    return out


def f32_to_bf16(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    out = np.empty(a.shape, dtype=np.uint16)
    _load().dasin_f32_to_bf16(a.ctypes.data, out.ctypes.data, a.size)
    return out


def kv_synth(seed, seq_key, layer, which, first_token, n_tokens, n_kv_heads, head_dim):
    """bf16 [n_tokens][n_kv_heads][head_dim] synthetic K (which=0) or V (which=1)."""
    out = np.empty((n_tokens, n_kv_heads, head_dim), dtype=np.uint16)
    _load().dasin_kv_synth(seed, seq_key, layer, which, first_token, n_tokens, n_kv_heads, head_dim,
                           out.ctypes.data)
    return out


def uniforms(seed, seq_keys, positions, stream):
    """fp32 uniforms in [0,1) keyed by (seed, sequence key, absolute position, stream)."""
    sk = np.ascontiguousarray(seq_keys, dtype=np.int64)
    ps = np.ascontiguousarray(positions, dtype=np.int64)
    out = np.empty(sk.shape, dtype=np.float32)
    _load().dasin_uniforms(seed, sk.size, sk.ctypes.data, ps.ctypes.data, stream, out.ctypes.data)
    return out


def num_threads():
    return int(_load().dasin_num_threads())

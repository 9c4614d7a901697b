"""ctypes front-end of the RanDeS CPU oracle -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this package.  It loads ``oracle/liboracle.so`` (plain C, built with gcc from
``randes_oracle.c``) and marshals numpy arrays; all arithmetic is in the C
file.  bf16 arrays travel as ``numpy.uint16`` bit patterns.

The layer description used here is a list of ``(rows, cols, group, flags)``
tuples; ``FLIP``/``SHUFFLE``/``SHIFT`` are the flag bits.
"""
import ctypes
import os
import subprocess

import numpy as np

F32, BF16 = 0, 1
FLIP, SHUFFLE, SHIFT = 1, 2, 4

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "randes_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force=False):
    """Compile the oracle with gcc (no fused contraction, no intrinsics)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
           "-std=c11", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


class _Layer(ctypes.Structure):
    _fields_ = [("rows", ctypes.c_int64), ("cols", ctypes.c_int64),
                ("group", ctypes.c_int32), ("flags", ctypes.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        u32p = ctypes.POINTER(ctypes.c_uint32)
        L.oracle_philox4x32_10.argtypes = [u32p, u32p, u32p]
        L.oracle_philox4x32_10.restype = None
        L.oracle_sign_bit.argtypes = [ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint64]
        L.oracle_sign_bit.restype = ctypes.c_uint32
        L.oracle_sign_mask.argtypes = [ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int64, ctypes.c_void_p]
        L.oracle_sign_mask.restype = None
        L.oracle_layer_perm.argtypes = [ctypes.c_uint64, ctypes.c_int32, ctypes.c_int32,
                                        ctypes.c_void_p, ctypes.c_void_p]
        L.oracle_layer_perm.restype = None
        L.oracle_bf16_to_f32.argtypes = [ctypes.c_uint16]
        L.oracle_bf16_to_f32.restype = ctypes.c_float
        L.oracle_f32_to_bf16.argtypes = [ctypes.c_float]
        L.oracle_f32_to_bf16.restype = ctypes.c_uint16
        L.oracle_source_table.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p,
                                          ctypes.c_int32, ctypes.c_void_p]
        L.oracle_source_table.restype = ctypes.c_int
        L.oracle_merge.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32,
                                   ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_int,
                                   ctypes.c_int]
        L.oracle_merge.restype = ctypes.c_int
        L.oracle_merge_weights.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                           ctypes.c_int32, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p,
                                           ctypes.c_int, ctypes.c_int]
        L.oracle_merge_weights.restype = ctypes.c_int
        L.oracle_retrieve.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int,
                                      ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64, ctypes.c_float,
                                      ctypes.c_void_p, ctypes.c_int, ctypes.c_int]
        L.oracle_retrieve.restype = ctypes.c_int
        L.oracle_lora.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                                  ctypes.c_int32, ctypes.c_double, ctypes.c_int, ctypes.c_void_p,
                                  ctypes.c_void_p]
        L.oracle_lora.restype = None
        L.oracle_lora_merge.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                        ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_double,
                                        ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
        L.oracle_lora_merge.restype = ctypes.c_int
        L.oracle_update.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int,
                                    ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64, ctypes.c_int,
                                    ctypes.c_int]
        L.oracle_update.restype = ctypes.c_int
        L.oracle_dot3.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int,
                                  ctypes.c_void_p]
        L.oracle_dot3.restype = None
        L.oracle_delta_stats.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_uint64,
                                         ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int, ctypes.c_void_p]
        L.oracle_delta_stats.restype = ctypes.c_int
        L.oracle_max_threads.argtypes = []
        L.oracle_max_threads.restype = ctypes.c_int
        _lib = L
    return _lib


# ---------------------------------------------------------------- marshalling
def _np_dtype(dtype):
    return np.float32 if dtype == F32 else np.uint16


def _layers_struct(layers):
    arr = (_Layer * len(layers))()
    for q, (rows, cols, group, flags) in enumerate(layers):
        arr[q] = _Layer(int(rows), int(cols), int(group), int(flags))
    return arr


def _check(a, dtype, count=None):
    assert isinstance(a, np.ndarray) and a.flags["C_CONTIGUOUS"], "need a C-contiguous numpy array"
    assert a.dtype == _np_dtype(dtype), (a.dtype, dtype)
    if count is not None:
        assert a.size == count, (a.size, count)
    return a


def _ptr_array(arrays):
    pa = (ctypes.c_void_p * len(arrays))()
    for q, a in enumerate(arrays):
        pa[q] = a.ctypes.data
    return pa


def _seed_array(seeds):
    return (ctypes.c_uint64 * len(seeds))(*[int(s) & 0xFFFFFFFFFFFFFFFF for s in seeds])


# ---------------------------------------------------------------- generator
def philox4x32_10(ctr, key):
    c = (ctypes.c_uint32 * 4)(*[int(x) & 0xFFFFFFFF for x in ctr])
    k = (ctypes.c_uint32 * 2)(*[int(x) & 0xFFFFFFFF for x in key])
    o = (ctypes.c_uint32 * 4)()
    lib().oracle_philox4x32_10(c, k, o)
    return [int(x) for x in o]


def sign_bit(seed, layer, col):
    return int(lib().oracle_sign_bit(int(seed) & 0xFFFFFFFFFFFFFFFF, int(layer), int(col)))


def sign_mask(seed, layer, cols):
    """uint8 array of length cols; 1 where the context matrix entry is -1."""
    out = np.zeros(int(cols), dtype=np.uint8)
    lib().oracle_sign_mask(int(seed) & 0xFFFFFFFFFFFFFFFF, int(layer), int(cols), out.ctypes.data)
    return out


def layer_perm(seed, group, group_size, return_keys=False):
    perm = np.zeros(int(group_size), dtype=np.int32)
    keys = np.zeros(int(group_size), dtype=np.uint64)
    lib().oracle_layer_perm(int(seed) & 0xFFFFFFFFFFFFFFFF, int(group), int(group_size),
                            perm.ctypes.data, keys.ctypes.data)
    return (perm, keys) if return_keys else perm


def source_table(layers, seeds):
    """int32 [n_tasks, n_layers]: layer of model i that lands in slot l."""
    out = np.zeros((len(seeds), len(layers)), dtype=np.int32)
    ls = _layers_struct(layers)
    sd = _seed_array(seeds)
    rc = lib().oracle_source_table(ls, len(layers), sd, len(seeds), out.ctypes.data)
    if rc != 0:
        raise ValueError("shape mismatch inside a shuffle group")
    return out


# ---------------------------------------------------------------- formats
def bf16_to_f32(bits):
    bits = np.asarray(bits, dtype=np.uint16)
    f = np.frompyfunc(lambda h: lib().oracle_bf16_to_f32(int(h)), 1, 1)
    return f(bits).astype(np.float32)


def f32_to_bf16(x):
    x = np.asarray(x, dtype=np.float32)
    f = np.frompyfunc(lambda v: lib().oracle_f32_to_bf16(float(v)), 1, 1)
    return f(x).astype(np.uint16)


# ---------------------------------------------------------------- the path
def merge(layers, deltas, seeds, delta_dtype=F32, merged_dtype=F32, n_threads=1):
    """deltas[i][l]: numpy array of model i's layer l (original position).
    Returns the list of superposed layers Delta_*[l]."""
    n_layers, n_tasks = len(layers), len(seeds)
    assert len(deltas) == n_tasks and all(len(d) == n_layers for d in deltas)
    flat = [_check(deltas[i][l], delta_dtype, layers[l][0] * layers[l][1])
            for i in range(n_tasks) for l in range(n_layers)]
    out = [np.zeros((layers[l][0], layers[l][1]), dtype=_np_dtype(merged_dtype)) for l in range(n_layers)]
    rc = lib().oracle_merge(_layers_struct(layers), n_layers, _ptr_array(flat), n_tasks,
                            _seed_array(seeds), delta_dtype, _ptr_array(out), merged_dtype, n_threads)
    if rc != 0:
        raise ValueError("shape mismatch inside a shuffle group")
    return out


def merge_weights(layers, weights, base, seeds, weight_dtype=F32, merged_dtype=F32, n_threads=1):
    """weights[i][l], base[l]: numpy arrays (original positions).  Deltas are formed on the fly."""
    n_layers, n_tasks = len(layers), len(seeds)
    flat = [_check(weights[i][l], weight_dtype, layers[l][0] * layers[l][1])
            for i in range(n_tasks) for l in range(n_layers)]
    b = [_check(base[l], weight_dtype, layers[l][0] * layers[l][1]) for l in range(n_layers)]
    out = [np.zeros((layers[l][0], layers[l][1]), dtype=_np_dtype(merged_dtype)) for l in range(n_layers)]
    rc = lib().oracle_merge_weights(_layers_struct(layers), n_layers, _ptr_array(flat), _ptr_array(b), n_tasks,
                                    _seed_array(seeds), weight_dtype, _ptr_array(out), merged_dtype, n_threads)
    if rc != 0:
        raise ValueError("shape mismatch inside a shuffle group")
    return out


def retrieve(layers, merged, base, seed, lam, merged_dtype=F32, base_dtype=F32, out_dtype=F32, n_threads=1):
    """Returns the list of retrieved layers hat Theta_i[l] (original positions)."""
    n_layers = len(layers)
    m = [_check(merged[l], merged_dtype, layers[l][0] * layers[l][1]) for l in range(n_layers)]
    b = [_check(base[l], base_dtype, layers[l][0] * layers[l][1]) for l in range(n_layers)]
    out = [np.zeros((layers[l][0], layers[l][1]), dtype=_np_dtype(out_dtype)) for l in range(n_layers)]
    rc = lib().oracle_retrieve(_layers_struct(layers), n_layers, _ptr_array(m), merged_dtype,
                               _ptr_array(b), base_dtype, int(seed) & 0xFFFFFFFFFFFFFFFF, float(lam),
                               _ptr_array(out), out_dtype, n_threads)
    if rc != 0:
        raise ValueError("shape mismatch inside a shuffle group")
    return out


def update(layers, merged, delta, seed, remove=False, merged_dtype=F32, delta_dtype=F32, n_threads=1):
    """In-place hot swap on ``merged`` (list of numpy arrays, modified)."""
    n_layers = len(layers)
    m = [_check(merged[l], merged_dtype, layers[l][0] * layers[l][1]) for l in range(n_layers)]
    d = [_check(delta[l], delta_dtype, layers[l][0] * layers[l][1]) for l in range(n_layers)]
    rc = lib().oracle_update(_layers_struct(layers), n_layers, _ptr_array(m), merged_dtype,
                             _ptr_array(d), delta_dtype, int(seed) & 0xFFFFFFFFFFFFFFFF,
                             1 if remove else 0, n_threads)
    if rc != 0:
        raise ValueError("shape mismatch inside a shuffle group")
    return merged


def lora(B, A, scale=1.0, ab_dtype=F32):
    """float64 (value, magnitude) of scale * B @ A; B rows x rank, A rank x cols."""
    rows, rank = B.shape
    rank2, cols = A.shape
    assert rank == rank2
    _check(B, ab_dtype)
    _check(A, ab_dtype)
    out = np.zeros((rows, cols), dtype=np.float64)
    mag = np.zeros((rows, cols), dtype=np.float64)
    lib().oracle_lora(B.ctypes.data, A.ctypes.data, rows, cols, rank, float(scale), ab_dtype,
                      out.ctypes.data, mag.ctypes.data)
    return out, mag


def lora_merge(layers, factors, seeds, scale=1.0, ab_dtype=F32):
    """factors[i][l] = (B, A) numpy arrays of model i, layer l (original position).
    Returns (values, magnitudes): lists of float64 arrays, one per slot layer."""
    n_layers, n_tasks = len(layers), len(seeds)
    Bs = [_check(factors[i][l][0], ab_dtype) for i in range(n_tasks) for l in range(n_layers)]
    As = [_check(factors[i][l][1], ab_dtype) for i in range(n_tasks) for l in range(n_layers)]
    rank = Bs[0].shape[1]
    out = [np.zeros((layers[l][0], layers[l][1]), dtype=np.float64) for l in range(n_layers)]
    mag = [np.zeros((layers[l][0], layers[l][1]), dtype=np.float64) for l in range(n_layers)]
    rc = lib().oracle_lora_merge(_layers_struct(layers), n_layers, _ptr_array(Bs), _ptr_array(As), rank, n_tasks,
                                 _seed_array(seeds), float(scale), ab_dtype, _ptr_array(out), _ptr_array(mag))
    if rc != 0:
        raise ValueError("shape mismatch inside a shuffle group")
    return out, mag


def dot3(a, b, dtype=F32):
    """(<a,b>, <a,a>, <b,b>) in float64."""
    _check(a, dtype)
    _check(b, dtype, a.size)
    out = (ctypes.c_double * 3)()
    lib().oracle_dot3(a.ctypes.data, b.ctypes.data, a.size, dtype, out)
    return float(out[0]), float(out[1]), float(out[2])


def delta_stats(layers, a, seed_a, b, seed_b, dtype=F32):
    """(<a',b'>, <a',a'>, <b',b'>) of two transformed deltas (lists of per-layer arrays)."""
    n_layers = len(layers)
    aa = [_check(a[l], dtype, layers[l][0] * layers[l][1]) for l in range(n_layers)]
    bb = [_check(b[l], dtype, layers[l][0] * layers[l][1]) for l in range(n_layers)]
    out = (ctypes.c_double * 3)()
    rc = lib().oracle_delta_stats(_layers_struct(layers), n_layers, _ptr_array(aa), int(seed_a) & 0xFFFFFFFFFFFFFFFF,
                                  _ptr_array(bb), int(seed_b) & 0xFFFFFFFFFFFFFFFF, dtype, out)
    if rc != 0:
        raise ValueError("shape mismatch inside a shuffle group")
    return float(out[0]), float(out[1]), float(out[2])


def max_threads():
    return int(lib().oracle_max_threads())

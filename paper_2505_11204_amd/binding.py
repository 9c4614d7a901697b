"""Thin Python binding of ``librandes.so`` (C ABI in ``include/randes.h``).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  PyTorch supplies device memory and streams.  There is no CPU
fallback: if the library is missing or a call fails, an exception is raised.

Names follow the C ABI: :func:`layer_perm`, :func:`source_table`,
:func:`sign_mask`, :func:`merge`, :func:`retrieve`, :func:`update`,
:func:`lora_materialize`, :func:`lora_materialize_batched`.

A layer list is a sequence of ``(rows, cols, group, flags)`` tuples.
"""
import ctypes
import os

import torch

F32, BF16 = 0, 1
FLIP, SHUFFLE, SHIFT = 1, 2, 4
MAX_TASKS = 128

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librandes.so")

# include/randes.h: the method's calls
EXPORTS = ["randes_layer_perm", "randes_source_table", "randes_sign_mask", "randes_merge", "randes_merge_weights",
           "randes_retrieve", "randes_retrieve_many", "randes_update", "randes_delta_stats", "randes_delta_stats_noalloc",
           "randes_lora_materialize",
           "randes_lora_materialize_batched", "randes_lora_merge", "randes_strerror", "randes_shutdown"]
# include/randes_bench.h: measurement aids
BENCH_EXPORTS = ["randes_set_tile_rows", "randes_set_tile_cols", "randes_set_fold", "randes_probe_stream"]
# include/randes_place.h: where stacks lie in device memory
PLACE_EXPORTS = ["randes_place_classify", "randes_place_classify_device", "randes_place_serving_layout"]
COPY_RATE_FN = ctypes.CFUNCTYPE(ctypes.c_double, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p)


class RandesError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("randes error %d: %s" % (code, text))
        self.code = code


class _Layer(ctypes.Structure):
    _fields_ = [("rows", ctypes.c_int64), ("cols", ctypes.c_int64),
                ("group", ctypes.c_int32), ("flags", ctypes.c_int32)]


_lib = None


def lib():
    """Load the library; raise if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("librandes.so is not built: run `python -m paper_2505_11204_amd.build` "
                           "(there is no fallback path)")
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, u64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64
    L.randes_layer_perm.argtypes = [u64, i32, i32, vp]
    L.randes_source_table.argtypes = [vp, i32, u64, vp]
    L.randes_sign_mask.argtypes = [u64, i32, i64, vp, vp]
    L.randes_merge.argtypes = [vp, i32, vp, i32, vp, ctypes.c_int, vp, ctypes.c_int, vp]
    L.randes_merge_weights.argtypes = [vp, i32, vp, vp, i32, vp, ctypes.c_int, vp, ctypes.c_int, vp]
    L.randes_retrieve.argtypes = [vp, i32, vp, ctypes.c_int, vp, ctypes.c_int, u64, ctypes.c_float,
                                  vp, ctypes.c_int, vp]
    L.randes_retrieve_many.argtypes = [vp, i32, vp, ctypes.c_int, vp, ctypes.c_int, i32, vp, vp,
                                       vp, ctypes.c_int, vp]
    L.randes_update.argtypes = [vp, i32, vp, ctypes.c_int, vp, ctypes.c_int, u64, i32, vp]
    L.randes_delta_stats.argtypes = [vp, i32, vp, u64, vp, u64, ctypes.c_int, vp, vp]
    L.randes_delta_stats_noalloc.argtypes = [vp, i32, vp, u64, vp, u64, ctypes.c_int, vp, vp]
    L.randes_lora_materialize.argtypes = [vp, vp, i64, i64, i32, ctypes.c_float, ctypes.c_int, vp,
                                          ctypes.c_int, vp]
    L.randes_lora_materialize_batched.argtypes = [i32, vp, vp, vp, vp, i32, ctypes.c_float, ctypes.c_int,
                                                  vp, ctypes.c_int, vp]
    L.randes_lora_merge.argtypes = [vp, i32, vp, vp, i32, i32, vp, ctypes.c_float, ctypes.c_int, vp, ctypes.c_int, vp]
    L.randes_strerror.argtypes = [ctypes.c_int]
    L.randes_strerror.restype = ctypes.c_char_p
    L.randes_shutdown.argtypes = []
    L.randes_set_tile_rows.argtypes = [i32, i32]
    L.randes_set_tile_cols.argtypes = [i32]
    L.randes_set_fold.argtypes = [i32]
    L.randes_probe_stream.argtypes = [vp, i32, vp, i64, i32, vp]
    L.randes_place_classify.argtypes = [i32, COPY_RATE_FN, vp, ctypes.c_double, i32, vp]
    L.randes_place_classify_device.argtypes = [vp, u64, i32, vp, vp]
    L.randes_place_serving_layout.argtypes = [vp, i32, u64, u64, i32, i32, vp, vp]
    for name in EXPORTS + BENCH_EXPORTS + PLACE_EXPORTS:
        if name != "randes_strerror":
            getattr(L, name).restype = ctypes.c_int
    _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise RandesError(rc, lib().randes_strerror(rc).decode("utf-8", "replace"))


def _u64(x):
    return int(x) & 0xFFFFFFFFFFFFFFFF


def dtype_code(t):
    if t == torch.float32:
        return F32
    if t == torch.bfloat16:
        return BF16
    raise TypeError("unsupported dtype %r (float32 and bfloat16 only)" % (t,))


def torch_dtype(code):
    return torch.float32 if code == F32 else torch.bfloat16


class LayerTable:
    """ctypes image of a layer list, built once and reused across calls."""

    def __init__(self, layers):
        self.layers = [tuple(int(x) for x in l) for l in layers]
        self.n = len(self.layers)
        self.array = (_Layer * max(self.n, 1))()
        for q, (rows, cols, group, flags) in enumerate(self.layers):
            self.array[q] = _Layer(rows, cols, group, flags)


def _layer_table(layers):
    return layers if isinstance(layers, LayerTable) else LayerTable(layers)


class PtrTable:
    """Host array of device pointers for a list of tensors (kept alive here)."""

    def __init__(self, tensors, layer_table=None, dtype=None):
        self.tensors = list(tensors)
        self.dtype = self.tensors[0].dtype if dtype is None else dtype
        self.array = (ctypes.c_void_p * max(len(self.tensors), 1))()
        for q, t in enumerate(self.tensors):
            if not t.is_cuda:
                raise ValueError("tensor %d is not on the GPU" % q)
            if not t.is_contiguous():
                raise ValueError("tensor %d is not contiguous" % q)
            if t.dtype != self.dtype:
                raise TypeError("tensor %d has dtype %r, expected %r" % (q, t.dtype, self.dtype))
            self.array[q] = t.data_ptr()
        if layer_table is not None:
            n = layer_table.n
            if len(self.tensors) % n != 0:
                raise ValueError("%d tensors for %d layers" % (len(self.tensors), n))
            for q, t in enumerate(self.tensors):
                rows, cols = layer_table.layers[q % n][:2]
                if t.numel() != rows * cols:
                    raise ValueError("tensor %d has %d elements, layer is %d x %d" % (q, t.numel(), rows, cols))

    @property
    def code(self):
        return dtype_code(self.dtype)


def _ptr_table(x, lt):
    return x if isinstance(x, PtrTable) else PtrTable(x, lt)


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


# ------------------------------------------------------------------ host-only calls
def layer_perm(seed, group, group_size):
    """sigma of one (model, group): list where entry k is the within-group index
    of the layer that lands in slot k."""
    out = (ctypes.c_int32 * max(int(group_size), 1))()
    _check(lib().randes_layer_perm(_u64(seed), int(group), int(group_size), out))
    return [int(x) for x in out[:int(group_size)]]


def source_table(layers, seed):
    """Entry l = layer of this model whose delta lands in slot l."""
    lt = _layer_table(layers)
    out = (ctypes.c_int32 * max(lt.n, 1))()
    _check(lib().randes_source_table(lt.array, lt.n, _u64(seed), out))
    return [int(x) for x in out[:lt.n]]


# ------------------------------------------------------------------ device calls
def sign_mask(seed, layer, cols, device="cuda", stream=None):
    """uint8 tensor of length cols on the GPU: 1 where the context matrix is -1."""
    out = torch.empty(int(cols), dtype=torch.uint8, device=device)
    _check(lib().randes_sign_mask(_u64(seed), int(layer), int(cols), ctypes.c_void_p(out.data_ptr()),
                                  _stream(stream)))
    return out


def alloc_like_layers(layers, dtype, device="cuda"):
    lt = _layer_table(layers)
    return [torch.empty((rows, cols), dtype=dtype, device=device) for (rows, cols, _, _) in lt.layers]


def merge(layers, deltas, seeds, merged=None, merged_dtype=None, stream=None):
    """compress: ``deltas`` is a list over models of lists over layers (original
    positions) or a PtrTable in model-major order.  Returns the list (or the
    PtrTable given) of superposed layers."""
    lt = _layer_table(layers)
    if not isinstance(deltas, PtrTable):
        flat = [t for per_model in deltas for t in per_model]
        if not flat:
            raise ValueError("no deltas given")
        deltas = PtrTable(flat, lt)
    n_tasks = len(deltas.tensors) // max(lt.n, 1)
    if n_tasks != len(seeds):
        raise ValueError("%d seeds for %d models" % (len(seeds), n_tasks))
    if merged is None:
        md = deltas.dtype if merged_dtype is None else merged_dtype
        merged = alloc_like_layers(lt, md, deltas.tensors[0].device)
    mt = _ptr_table(merged, lt)
    sd = (ctypes.c_uint64 * max(len(seeds), 1))(*[_u64(s) for s in seeds])
    _check(lib().randes_merge(lt.array, lt.n, deltas.array, n_tasks, sd, deltas.code,
                              mt.array, mt.code, _stream(stream)))
    return merged


def merge_weights(layers, weights, base, seeds, merged=None, merged_dtype=None, stream=None):
    """compress straight from fine-tuned weights and the base (deltas formed on the fly)."""
    lt = _layer_table(layers)
    if not isinstance(weights, PtrTable):
        flat = [t for per_model in weights for t in per_model]
        if not flat:
            raise ValueError("no weights given")
        weights = PtrTable(flat, lt)
    bt = _ptr_table(base, lt)
    if bt.dtype != weights.dtype:
        raise TypeError("weights and base must share a dtype")
    n_tasks = len(weights.tensors) // max(lt.n, 1)
    if n_tasks != len(seeds):
        raise ValueError("%d seeds for %d models" % (len(seeds), n_tasks))
    if merged is None:
        merged = alloc_like_layers(lt, weights.dtype if merged_dtype is None else merged_dtype, weights.tensors[0].device)
    mt = _ptr_table(merged, lt)
    sd = (ctypes.c_uint64 * max(len(seeds), 1))(*[_u64(s) for s in seeds])
    _check(lib().randes_merge_weights(lt.array, lt.n, weights.array, bt.array, n_tasks, sd, weights.code,
                                      mt.array, mt.code, _stream(stream)))
    return merged


def retrieve(layers, merged, base, seed, lam, out=None, out_dtype=None, stream=None):
    """retrieve one model: returns the list (or PtrTable) of its layers."""
    lt = _layer_table(layers)
    mt = _ptr_table(merged, lt)
    bt = _ptr_table(base, lt)
    if out is None:
        od = bt.dtype if out_dtype is None else out_dtype
        out = alloc_like_layers(lt, od, bt.tensors[0].device)
    ot = _ptr_table(out, lt)
    _check(lib().randes_retrieve(lt.array, lt.n, mt.array, mt.code, bt.array, bt.code, _u64(seed),
                                 ctypes.c_float(lam), ot.array, ot.code, _stream(stream)))
    return out


def retrieve_many(layers, merged, base, seeds, lams, outs=None, out_dtype=None, stream=None):
    """retrieve several models in one pass: returns one list of layers per request
    (or the PtrTable passed as ``outs``, which then holds request q's layer l at q * n_layers + l)."""
    lt = _layer_table(layers)
    mt = _ptr_table(merged, lt)
    bt = _ptr_table(base, lt)
    n = len(seeds)
    if len(lams) != n:
        raise ValueError("%d lambdas for %d seeds" % (len(lams), n))
    result = outs
    if outs is None:
        od = bt.dtype if out_dtype is None else out_dtype
        result = [alloc_like_layers(lt, od, bt.tensors[0].device) for _ in range(n)]
        outs = result
    if not isinstance(outs, PtrTable):
        flat = [t for per_request in outs for t in per_request]
        if not flat:
            raise ValueError("no requests given")
        outs = PtrTable(flat, lt)
    if len(outs.tensors) != n * lt.n:
        raise ValueError("outs holds %d tensors, expected %d" % (len(outs.tensors), n * lt.n))
    sd = (ctypes.c_uint64 * max(n, 1))(*[_u64(s) for s in seeds])
    la = (ctypes.c_float * max(n, 1))(*[float(x) for x in lams])
    _check(lib().randes_retrieve_many(lt.array, lt.n, mt.array, mt.code, bt.array, bt.code, n, sd, la,
                                      outs.array, outs.code, _stream(stream)))
    return result


def update(layers, merged, delta, seed, remove=False, stream=None):
    """hot swap: add (or remove) one model in place on ``merged``."""
    lt = _layer_table(layers)
    mt = _ptr_table(merged, lt)
    dt = _ptr_table(delta, lt)
    _check(lib().randes_update(lt.array, lt.n, mt.array, mt.code, dt.array, dt.code, _u64(seed),
                               1 if remove else 0, _stream(stream)))
    return merged


def delta_stats(layers, delta_a, seed_a, delta_b, seed_b, out=None, stream=None, noalloc=False):
    """(<a',b'>, <a',a'>, <b',b'>) of two transformed deltas as a float64 GPU tensor of 3.
    ``noalloc`` calls randes_delta_stats_noalloc (then ``out`` must be given: nothing is allocated)."""
    lt = _layer_table(layers)
    at, bt = _ptr_table(delta_a, lt), _ptr_table(delta_b, lt)
    if at.dtype != bt.dtype:
        raise TypeError("both deltas must share a dtype")
    if out is None:
        if noalloc:
            raise ValueError("the no-allocation call needs its output tensor")
        out = torch.empty(3, dtype=torch.float64, device=at.tensors[0].device)
    fn = lib().randes_delta_stats_noalloc if noalloc else lib().randes_delta_stats
    _check(fn(lt.array, lt.n, at.array, _u64(seed_a), bt.array, _u64(seed_b), at.code,
              ctypes.c_void_p(out.data_ptr()), _stream(stream)))
    return out


def lora_materialize(B, A, scale=1.0, out=None, out_dtype=None, stream=None):
    """delta = scale * B @ A on the matrix cores; B rows x rank, A rank x cols."""
    rows, rank = B.shape
    rank2, cols = A.shape
    if rank != rank2 or B.dtype != A.dtype:
        raise ValueError("B is %s %s, A is %s %s" % (tuple(B.shape), B.dtype, tuple(A.shape), A.dtype))
    if not (B.is_cuda and A.is_cuda and B.is_contiguous() and A.is_contiguous()):
        raise ValueError("B and A must be contiguous GPU tensors")
    if out is None:
        out = torch.empty((rows, cols), dtype=B.dtype if out_dtype is None else out_dtype, device=B.device)
    if not (out.is_cuda and out.is_contiguous() and out.numel() == rows * cols):
        raise ValueError("bad output tensor")
    _check(lib().randes_lora_materialize(ctypes.c_void_p(B.data_ptr()), ctypes.c_void_p(A.data_ptr()),
                                         rows, cols, rank, ctypes.c_float(scale), dtype_code(B.dtype),
                                         ctypes.c_void_p(out.data_ptr()), dtype_code(out.dtype),
                                         _stream(stream)))
    return out


class LoraBatch:
    """Marshalled arguments of a batched materialisation, built once and reused."""

    def __init__(self, Bs, As, outs=None, out_dtype=None):
        n = len(Bs)
        if n != len(As) or n < 1:
            raise ValueError("need as many A as B matrices, at least one")
        self.rank = int(Bs[0].shape[1])
        for B, A in zip(Bs, As):
            if B.shape[1] != self.rank or A.shape[0] != self.rank or B.dtype != Bs[0].dtype or A.dtype != Bs[0].dtype:
                raise ValueError("all adapters of a batch share rank and dtype")
        if outs is None:
            od = Bs[0].dtype if out_dtype is None else out_dtype
            outs = [torch.empty((B.shape[0], A.shape[1]), dtype=od, device=B.device) for B, A in zip(Bs, As)]
        self.n, self.outs = n, outs
        self.bt, self.at, self.ot = PtrTable(Bs), PtrTable(As), PtrTable(outs)
        self.rows = (ctypes.c_int64 * n)(*[int(B.shape[0]) for B in Bs])
        self.cols = (ctypes.c_int64 * n)(*[int(A.shape[1]) for A in As])
        for q, o in enumerate(outs):
            if o.numel() != self.rows[q] * self.cols[q]:
                raise ValueError("output %d has the wrong size" % q)

    def run(self, scale=1.0, stream=None):
        _check(lib().randes_lora_materialize_batched(self.n, self.bt.array, self.at.array, self.rows, self.cols,
                                                     self.rank, ctypes.c_float(scale), self.bt.code,
                                                     self.ot.array, self.ot.code, _stream(stream)))
        return self.outs


def lora_materialize_batched(Bs, As, scale=1.0, outs=None, out_dtype=None, stream=None):
    """Many adapters in one launch; all share rank and dtypes."""
    return LoraBatch(Bs, As, outs, out_dtype).run(scale, stream)


class LoraMerge:
    """Marshalled arguments of a fused LoRA compress, built once and reused."""

    def __init__(self, layers, factors, seeds, merged=None, merged_dtype=None):
        lt = _layer_table(layers)
        n_tasks = len(factors)
        if n_tasks != len(seeds) or n_tasks < 1:
            raise ValueError("%d seeds for %d models" % (len(seeds), n_tasks))
        Bs = [f[0] for per in factors for f in per]
        As = [f[1] for per in factors for f in per]
        if len(Bs) != n_tasks * lt.n:
            raise ValueError("need one (B, A) pair per model and layer")
        rank = int(Bs[0].shape[1])
        for q, (B, A) in enumerate(zip(Bs, As)):
            rows, cols = lt.layers[q % lt.n][:2]
            if tuple(B.shape) != (rows, rank) or tuple(A.shape) != (rank, cols) or A.dtype != Bs[0].dtype or B.dtype != Bs[0].dtype:
                raise ValueError("factor pair %d does not fit layer %d x %d at rank %d" % (q, rows, cols, rank))
        if merged is None:
            merged = alloc_like_layers(lt, Bs[0].dtype if merged_dtype is None else merged_dtype, Bs[0].device)
        self.lt, self.n_tasks, self.rank, self.merged = lt, n_tasks, rank, merged
        self.bt, self.at, self.mt = PtrTable(Bs), PtrTable(As), _ptr_table(merged, lt)
        self.sd = (ctypes.c_uint64 * n_tasks)(*[_u64(s) for s in seeds])

    def run(self, scale=1.0, stream=None):
        _check(lib().randes_lora_merge(self.lt.array, self.lt.n, self.bt.array, self.at.array, self.rank, self.n_tasks,
                                       self.sd, ctypes.c_float(scale), self.bt.code, self.mt.array, self.mt.code,
                                       _stream(stream)))
        return self.merged


def lora_merge(layers, factors, seeds, scale=1.0, merged=None, merged_dtype=None, stream=None):
    """Fused LoRA compress: ``factors[i][l] = (B, A)`` of model i, layer l (original
    position).  Returns the superposed dense layers, written once."""
    return LoraMerge(layers, factors, seeds, merged, merged_dtype).run(scale, stream)


def set_tile_rows(merge_rows=0, retrieve_rows=0):
    """Launch-shape knob of the calling thread for measurements (0 = default).  Results do not depend on it."""
    _check(lib().randes_set_tile_rows(int(merge_rows), int(retrieve_rows)))


def set_tile_cols(max_waves_along_columns=0):
    """Second launch-shape knob (4, 2, 1; 0 = default).  Results do not depend on it."""
    _check(lib().randes_set_tile_cols(int(max_waves_along_columns)))


def set_fold(enable=True):
    """Third launch-shape knob: fold rows of layers that leave lanes idle (default on).
    Results do not depend on it."""
    _check(lib().randes_set_fold(1 if enable else 0))


def probe_stream(inputs, output, write=True, stream=None):
    """Plain streaming probe (measurement aid): output = integer sum of the input
    streams, or loads only when ``write`` is false.  All tensors flat, equal byte size."""
    it = PtrTable(inputs)
    nbytes = inputs[0].numel() * inputs[0].element_size()
    for t in inputs:
        if t.numel() * t.element_size() != nbytes:
            raise ValueError("probe streams differ in size")
    if write and output.numel() * output.element_size() < nbytes:
        raise ValueError("probe output too small")
    _check(lib().randes_probe_stream(it.array, len(inputs), ctypes.c_void_p(output.data_ptr()), nbytes,
                                     1 if write else 0, _stream(stream)))


def shutdown():
    """Free the library's cached descriptor tables (synchronise streams first)."""
    _check(lib().randes_shutdown())

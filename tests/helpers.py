"""Shared test plumbing: move seeded inputs to the GPU library and to the CPU
oracle, and compare results.  No arithmetic of the method lives here."""
import numpy as np
import torch

from paper_2505_11204_amd import workloads as wl

NP = {"f32": np.float32, "bf16": np.uint16}
CODE = {"f32": 0, "bf16": 1}


def layers_of(stack):
    return [(l.rows, l.cols, l.group, l.flags) for l in stack]


def to_np(t):
    return wl.to_numpy(t)


def bits_equal(gpu_tensor, oracle_array, what=""):
    """Bit-for-bit comparison (f32 as uint32, bf16 as uint16)."""
    g = to_np(gpu_tensor)
    o = np.asarray(oracle_array)
    assert g.shape == o.shape or g.size == o.size, (what, g.shape, o.shape)
    gv = g.reshape(-1).view(np.uint32 if g.dtype == np.float32 else np.uint16)
    ov = o.reshape(-1).view(np.uint32 if o.dtype == np.float32 else np.uint16)
    bad = np.nonzero(gv != ov)[0]
    assert bad.size == 0, "%s: %d of %d elements differ, first at %d: gpu %r oracle %r" % (
        what, bad.size, gv.size, bad[0], g.reshape(-1)[bad[0]], o.reshape(-1)[bad[0]])


def bf16_ulp_distance(a_bits, b_bits):
    """Distance in bf16 units of last place between two uint16 bit patterns
    (finite values): map sign-magnitude to a monotone integer line."""
    def key(x):
        x = x.astype(np.int32)
        return np.where(x & 0x8000, -(x & 0x7FFF), x & 0x7FFF)
    return np.abs(key(a_bits) - key(b_bits))


def bf16_within_one_ulp(gpu_tensor, oracle_array, what=""):
    """The stated bar for bf16 outputs: within 1 bf16 ulp; returns the number
    of elements that are not bit-equal (expected 0)."""
    g = to_np(gpu_tensor).reshape(-1)
    o = np.asarray(oracle_array).reshape(-1)
    d = bf16_ulp_distance(g, o)
    assert d.max() <= 1, "%s: max bf16 ulp distance %d" % (what, d.max())
    return int((d != 0).sum())


def compare(gpu_tensor, oracle_array, what=""):
    """fp32: bit-exact.  bf16: within 1 ulp, and report/require bit equality."""
    if gpu_tensor.dtype == torch.float32:
        bits_equal(gpu_tensor, oracle_array, what)
    else:
        n_off = bf16_within_one_ulp(gpu_tensor, oracle_array, what)
        assert n_off == 0, "%s: %d bf16 elements differ by one ulp (expected bit equality)" % (what, n_off)


def cpu_inputs(stack, n_tasks, dtype, data_seed=1234, scales=None, delta_std=1e-3):
    """Seeded CPU tensors (the oracle's and, copied, the GPU's inputs)."""
    return wl.make_inputs(stack, n_tasks, dtype=dtype, device="cpu", data_seed=data_seed,
                          scales=scales, delta_std=delta_std)


def to_gpu(list_of_tensors):
    return [t.cuda() for t in list_of_tensors]


def np_lists(list_of_tensors):
    return [to_np(t) for t in list_of_tensors]


def gather_rows(views, row_sets):
    """Device tensors -> numpy arrays holding only the sampled rows of each layer."""
    out = []
    for v, rows in zip(views, row_sets):
        idx = torch.as_tensor(rows, device=v.device)
        out.append(to_np(v.index_select(0, idx)))
    return out

"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element
by element, on the same seeded inputs.  Bar: sign masks, permutations and f32
outputs bit-exact; bf16 outputs within 1 bf16 ulp (and in fact bit-equal, which
is asserted too, since both sides round the same binary32 value the same way)."""
import os

import numpy as np
import pytest
import torch

import oracle
from helpers import CODE, bits_equal, compare, cpu_inputs, layers_of, np_lists, to_gpu, to_np
from paper_2505_11204_amd import binding as rb
from paper_2505_11204_amd import workloads as wl
from paper_2505_11204_amd.workloads import FLIP, SHIFT, SHUFFLE, SRSF, Layer

pytestmark = pytest.mark.gpu

TD = {"f32": torch.float32, "bf16": torch.bfloat16}


@pytest.fixture(autouse=True)
def _default_tiles():
    rb.set_tile_rows(0, 0)
    rb.set_tile_cols(0)
    yield
    torch.cuda.synchronize()
    rb.set_tile_rows(0, 0)
    rb.set_tile_cols(0)


def ragged_stack():
    """Several tiles per layer at 16 rows per tile, ragged row and column tails,
    vector and element-wise layers, groups interleaved, singletons."""
    return [
        Layer(130, 1032, 0, SRSF), Layer(70, 520, 1, SRSF), Layer(130, 1032, 0, SRSF),
        Layer(257, 136, -1, FLIP), Layer(70, 520, 1, SRSF), Layer(130, 1032, 0, SRSF),
        Layer(5, 77, -1, FLIP), Layer(3, 1, -1, FLIP), Layer(1, 3000, -1, FLIP),
        Layer(33, 2048, 2, SRSF), Layer(33, 2048, 2, SRSF), Layer(19, 130, 3, SHUFFLE),
        Layer(19, 130, 3, SHUFFLE), Layer(19, 130, 3, SHUFFLE), Layer(64, 4104, -1, 0),
    ]


def run_both(stack, n_tasks, seeds, d_in, d_merged, d_base, d_out, lam, tasks_to_retrieve,
             data_seed=1234, scales=None):
    layers = layers_of(stack)
    base, deltas = cpu_inputs(stack, n_tasks, d_in, data_seed, scales)
    if d_base != d_in:
        base = [b.to(TD[d_base]) for b in base]
    g_merged = rb.merge(layers, [to_gpu(d) for d in deltas], seeds, merged_dtype=TD[d_merged])
    o_merged = oracle.merge(layers, [np_lists(d) for d in deltas], seeds, CODE[d_in], CODE[d_merged], n_threads=8)
    for l in range(len(stack)):
        compare(g_merged[l], o_merged[l], "merged layer %d" % l)
    g_base = to_gpu(base)
    for i in tasks_to_retrieve:
        g_out = rb.retrieve(layers, g_merged, g_base, seeds[i], lam, out_dtype=TD[d_out])
        o_out = oracle.retrieve(layers, o_merged, np_lists(base), seeds[i], lam,
                                CODE[d_merged], CODE[d_base], CODE[d_out], n_threads=8)
        for l in range(len(stack)):
            compare(g_out[l], o_out[l], "task %d layer %d" % (i, l))
    return g_merged, o_merged


# ------------------------------------------------------------------ generator
def test_sign_masks_bit_exact():
    for seed, layer, cols in [(0, 0, 128), (42, 0, 4096), (43, 17, 11008), (2**64 - 1, 225, 32000),
                              (0x123456789ABCDEF, 3, 1), (7, 1, 77), (7, 2, 129), (44, 9, 100003)]:
        g = rb.sign_mask(seed, layer, cols).cpu().numpy()
        assert np.array_equal(g, oracle.sign_mask(seed, layer, cols)), (seed, layer, cols)


def test_permutations_bit_exact():
    for seed in (0, 42, 43, 2**63):
        for group in (0, 6, 17):
            for G in (1, 4, 12, 24, 32):
                assert rb.layer_perm(seed, group, G) == oracle.layer_perm(seed, group, G).tolist()


# ------------------------------------------------------------------ the path
def test_tiny_config():
    # 4 tasks, 4 f32 matrices of 256 x 256, seeds 0..3, lambda = 1, merge then retrieve task 2
    run_both(wl.tiny(), 4, [0, 1, 2, 3], "f32", "f32", "f32", "f32", 1.0, [2])


@pytest.mark.parametrize("d_in,d_merged,d_base,d_out", [
    ("f32", "f32", "f32", "f32"), ("bf16", "bf16", "bf16", "bf16"), ("bf16", "f32", "bf16", "bf16"),
    ("f32", "bf16", "f32", "f32"), ("bf16", "bf16", "f32", "f32"), ("f32", "f32", "bf16", "bf16"),
    ("bf16", "f32", "f32", "bf16"), ("bf16", "bf16", "bf16", "f32")])
@pytest.mark.parametrize("n_tasks", [1, 3, 8, 9, 20])
def test_ragged_stack_all_dtypes(d_in, d_merged, d_base, d_out, n_tasks):
    rb.set_tile_rows(3, 5)
    rb.set_tile_cols(2 if n_tasks % 2 else 4)
    seeds = [42 + i for i in range(n_tasks)]
    run_both(ragged_stack(), n_tasks, seeds, d_in, d_merged, d_base, d_out, 0.3, [0, n_tasks - 1])


@pytest.mark.parametrize("n_tasks", [2, 4, 5, 6, 7])
def test_every_register_resident_task_count(n_tasks):
    rb.set_tile_cols(1 if n_tasks % 2 else 0)
    seeds = [1000 + 7 * i for i in range(n_tasks)]
    run_both(ragged_stack(), n_tasks, seeds, "bf16", "bf16", "bf16", "bf16", 1.0, [n_tasks // 2])
    run_both(ragged_stack(), n_tasks, seeds, "f32", "f32", "f32", "f32", 1.0, [n_tasks // 2])


@pytest.mark.parametrize("flags", [0, FLIP, SHUFFLE, SHIFT, FLIP | SHIFT])
def test_flag_variants(flags):
    stack = [Layer(40, 264, 0, flags)] * 5 + [Layer(9, 40, -1, flags & FLIP)]
    run_both(stack, 3, [5, 6, 7], "f32", "f32", "f32", "f32", 0.7, [1])
    run_both(stack, 3, [5, 6, 7], "bf16", "bf16", "bf16", "bf16", 0.7, [1])


def test_skip_rate_pattern():
    # only every 2nd layer of the repeated set is shuffled and flipped
    stack = [Layer(24, 256, 0, SRSF if k % 2 == 0 else 0) for k in range(8)]
    run_both(stack, 4, [42, 43, 44, 45], "f32", "f32", "f32", "f32", 1.0, [3])


@pytest.mark.parametrize("lam", [0.0, 0.1, 1.0, 2.0, -0.5])
def test_lambda_values(lam):
    stack = [Layer(20, 512, 0, SRSF)] * 3
    run_both(stack, 4, [1, 2, 3, 4], "f32", "f32", "f32", "f32", lam, [2])
    run_both(stack, 4, [1, 2, 3, 4], "bf16", "bf16", "bf16", "bf16", lam, [2])


def test_single_model_round_trip_is_exact_on_gpu():
    stack = [Layer(64, 1024, 0, SRSF)] * 4
    layers = layers_of(stack)
    base, deltas = cpu_inputs(stack, 1, "f32")
    gm = rb.merge(layers, [to_gpu(deltas[0])], [9])
    out = rb.retrieve(layers, gm, to_gpu(base), 9, 1.0)
    for l in range(4):
        assert torch.equal(out[l].cpu(), base[l] + deltas[0][l])


def test_launch_geometry_does_not_change_results():
    stack = ragged_stack()
    layers = layers_of(stack)
    base, deltas = cpu_inputs(stack, 8, "bf16")
    gd = [to_gpu(d) for d in deltas]
    gb = to_gpu(base)
    seeds = list(range(42, 50))
    ref_m = ref_o = None
    for tr, tc in ((0, 0), (1, 4), (2, 2), (3, 1), (4, 2), (7, 1), (1000, 4)):
        rb.set_tile_rows(tr, tr)
        rb.set_tile_cols(tc)
        m = rb.merge(layers, gd, seeds)
        o = rb.retrieve(layers, m, gb, seeds[3], 0.9)
        torch.cuda.synchronize()
        if ref_m is None:
            ref_m, ref_o = m, o
        else:
            for l in range(len(stack)):
                assert torch.equal(m[l].view(torch.int16), ref_m[l].view(torch.int16))
                assert torch.equal(o[l].view(torch.int16), ref_o[l].view(torch.int16))


def test_unaligned_layers_take_the_elementwise_path_with_equal_results():
    stack = [Layer(10, 264, 0, SRSF)] * 3
    layers = layers_of(stack)
    base, deltas = cpu_inputs(stack, 2, "f32")
    seeds = [3, 4]

    def shifted(t):  # same values at a 4-byte offset: not 16-byte aligned
        buf = torch.empty(t.numel() + 1, dtype=t.dtype, device="cuda")
        v = buf[1:].view(t.shape)
        v.copy_(t)
        return v
    gd = [[shifted(t) for t in d] for d in deltas]
    assert gd[0][0].data_ptr() % 16 != 0
    m = rb.merge(layers, gd, seeds)
    o_m = oracle.merge(layers, [np_lists(d) for d in deltas], seeds)
    for l in range(3):
        compare(m[l], o_m[l], "unaligned merge %d" % l)
    out = rb.retrieve(layers, m, [shifted(b) for b in base], 4, 1.0)
    o_out = oracle.retrieve(layers, o_m, np_lists(base), 4, 1.0)
    for l in range(3):
        compare(out[l], o_out[l], "unaligned retrieve %d" % l)


def test_in_place_retrieve_into_base():
    stack = [Layer(48, 512, 0, SRSF)] * 4
    layers = layers_of(stack)
    base, deltas = cpu_inputs(stack, 3, "bf16")
    seeds = [1, 2, 3]
    m = rb.merge(layers, [to_gpu(d) for d in deltas], seeds)
    gb = to_gpu(base)
    rb.retrieve(layers, m, gb, 2, 1.0, out=gb)
    o_m = oracle.merge(layers, [np_lists(d) for d in deltas], seeds, 1, 1)
    o_out = oracle.retrieve(layers, o_m, np_lists(base), 2, 1.0, 1, 1, 1)
    for l in range(4):
        compare(gb[l], o_out[l], "in-place %d" % l)


def test_special_values():
    # signed zeros, denormals, infinities, large magnitudes; NaN positions must agree
    stack = [Layer(4, 256, -1, FLIP)]
    layers = layers_of(stack)
    g = torch.Generator().manual_seed(5)
    K = 3
    deltas = []
    specials = torch.tensor([0.0, -0.0, 1e-45, -1e-45, 1e-39, 3e38, -3e38, float("inf"), float("-inf"),
                             float("nan"), 1.0, -1.0, 65504.0, 2.0 ** -126, 1.1754942e-38, 7.0])
    for i in range(K):
        x = torch.randn(4, 256, generator=g)
        idx = torch.randint(0, 16, (4, 256), generator=g)
        pick = torch.rand(4, 256, generator=g) < 0.5
        x = torch.where(pick, specials[idx], x)
        deltas.append([x])
    base = [torch.randn(4, 256, generator=g)]
    seeds = [11, 12, 13]
    for dt in ("f32", "bf16"):
        dd = [[t.to(TD[dt]) for t in d] for d in deltas]
        bb = [b.to(TD[dt]) for b in base]
        m = rb.merge(layers, [to_gpu(d) for d in dd], seeds)
        o_m = oracle.merge(layers, [np_lists(d) for d in dd], seeds, CODE[dt], CODE[dt])
        out = rb.retrieve(layers, m, to_gpu(bb), 12, 0.5)
        o_out = oracle.retrieve(layers, o_m, np_lists(bb), 12, 0.5, CODE[dt], CODE[dt], CODE[dt])
        for got, want in ((m[0], o_m[0]), (out[0], o_out[0])):
            gf = got.float().cpu().numpy()
            wf = oracle.bf16_to_f32(want) if dt == "bf16" else want
            assert np.array_equal(np.isnan(gf), np.isnan(wf))
            ok = ~np.isnan(wf)
            gb_, wb_ = to_np(got)[ok], np.asarray(want)[ok]
            assert np.array_equal(gb_.view(np.uint32 if dt == "f32" else np.uint16),
                                  wb_.view(np.uint32 if dt == "f32" else np.uint16))


@pytest.mark.parametrize("cols", [1024, 1021])
def test_bf16_rounding_at_every_boundary(cols):
    # binary32 -> bf16 on the way out of merge and retrieve, for every one of the 65536 high halves (every
    # exponent, NaNs, infinities and subnormals among them) with low halves at, next to and between the
    # ties.  1024 columns: 16-byte accesses; 1021: the element-wise kernels.
    lows = np.array([0x0000, 0x0001, 0x4000, 0x7fff, 0x8000, 0x8001, 0xc000, 0xffff], dtype=np.uint32)
    u = ((np.arange(65536, dtype=np.uint32)[:, None] << 16) | lows[None, :]).reshape(-1)
    rows = -(-u.size // cols)
    u = np.concatenate([u, u[:rows * cols - u.size]])
    x = torch.from_numpy(u.view(np.float32).reshape(rows, cols).copy())
    stack = [Layer(rows, cols, -1, FLIP)]
    layers = layers_of(stack)

    def same(got, want, what):
        gf, wf = got.float().cpu().numpy(), oracle.bf16_to_f32(want)
        assert np.array_equal(np.isnan(gf), np.isnan(wf)), what
        ok = ~np.isnan(wf)
        assert np.array_equal(to_np(got)[ok].view(np.uint16), np.asarray(want)[ok].view(np.uint16)), what

    m = rb.merge(layers, [to_gpu([x])], [77], merged_dtype=torch.bfloat16)
    o_m = oracle.merge(layers, [np_lists([x])], [77], CODE["f32"], CODE["bf16"])
    same(m[0], o_m[0], "merge")
    base = [torch.full((rows, cols), -0.0)]     # x + (-0) = x for every x, zeros of either sign included
    out = rb.retrieve(layers, to_gpu([x]), to_gpu(base), 77, 1.0, out_dtype=torch.bfloat16)
    o_out = oracle.retrieve(layers, np_lists([x]), np_lists(base), 77, 1.0, CODE["f32"], CODE["f32"], CODE["bf16"])
    same(out[0], o_out[0], "retrieve")


def test_empty_and_invalid_requests_are_rejected():
    stack = [Layer(8, 256, 0, SRSF)] * 2
    layers = layers_of(stack)
    base, deltas = cpu_inputs(stack, 2, "f32")
    gd = [to_gpu(d) for d in deltas]
    with pytest.raises(rb.RandesError):
        rb.merge(layers, gd, [1, 2], merged=gd[0])          # output aliases an input
    m = rb.merge(layers, gd, [1, 2])
    with pytest.raises(rb.RandesError):
        rb.retrieve(layers, m, to_gpu(base), 1, 1.0, out=m)  # out aliases the superposition
    with pytest.raises(rb.RandesError):
        rb.retrieve(layers, m, to_gpu(base), 1, float("nan"))
    with pytest.raises(rb.RandesError):
        rb.merge([(8, 256, 0, 3), (4, 512, 0, 3)], gd, [1, 2])  # group with mixed shapes
    with pytest.raises(ValueError):
        rb.merge(layers, [], [])                               # no models


def test_buffers_that_are_not_this_devices_memory_or_too_small_are_rejected():
    # checked against the runtime's records when the tables of an argument set are built: nothing is launched
    import ctypes
    lib = rb.lib()
    n_layers, K = 1, 2
    good = [torch.zeros(8, 256, device="cuda") for _ in range(K + 3)]
    layer = rb.LayerTable([(8, 256, -1, 1)])
    seeds = (ctypes.c_uint64 * K)(1, 2)

    def ptrs(*addresses):
        return (ctypes.c_void_p * len(addresses))(*addresses)
    host = np.zeros((8, 256), dtype=np.float32)       # ordinary host memory, unknown to HIP
    d0, d1, m = good[0].data_ptr(), good[1].data_ptr(), good[2].data_ptr()
    rc = lib.randes_merge(layer.array, n_layers, ptrs(d0, host.ctypes.data), K, seeds, 0, ptrs(m), 0, None)
    assert rc == -1 and "not memory known to HIP" in lib.randes_strerror(rc).decode()
    rc = lib.randes_retrieve(layer.array, n_layers, ptrs(m), 0, ptrs(host.ctypes.data), 0, ctypes.c_uint64(1),
                             ctypes.c_float(1.0), ptrs(good[3].data_ptr()), 0, None)
    assert rc == -1 and "not memory known to HIP" in lib.randes_strerror(rc).decode()
    # a delta of 64 MiB behind a layer of 96 MiB (the merged buffer does hold 96 MiB); of three such deltas at
    # least one lies where its claimed extent does not run into the merged buffer, which would be refused as overlap
    mib = 1 << 20
    torch.cuda.empty_cache()          # so that each tensor below is an allocation of its own size
    big_m = torch.zeros(96 * mib // 4, device="cuda")
    small = [torch.zeros(64 * mib // 4, device="cuda") for _ in range(3)]
    free = [t for t in small if t.data_ptr() + 96 * mib <= big_m.data_ptr() or t.data_ptr() >= big_m.data_ptr() + 96 * mib]
    assert free
    big = rb.LayerTable([(96 * mib // 4 // 4096, 4096, -1, 1)])
    one_seed = (ctypes.c_uint64 * 1)(7)
    rc = lib.randes_merge(big.array, n_layers, ptrs(free[0].data_ptr()), 1, one_seed, 0, ptrs(big_m.data_ptr()), 0, None)
    assert rc == -1 and "past its allocation" in lib.randes_strerror(rc).decode()
    torch.cuda.synchronize()
    assert float(big_m.abs().sum()) == 0.0
    torch.cuda.synchronize()
    assert all(float(t.abs().sum()) == 0.0 for t in good)     # nothing was written
    # the same pointers with their true shape are accepted
    assert lib.randes_merge(layer.array, n_layers, ptrs(d0, d1), K, seeds, 0, ptrs(m), 0, None) == 0
    torch.cuda.synchronize()


# ------------------------------------------------------------------ hot swap
@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_hot_swap(dt):
    stack = ragged_stack()
    layers = layers_of(stack)
    _, deltas = cpu_inputs(stack, 4, dt)
    seeds = [10, 11, 12, 13]
    gd = [to_gpu(d) for d in deltas]
    part = rb.merge(layers, gd[:3], seeds[:3])
    rb.update(layers, part, gd[3], seeds[3])
    o_part = oracle.merge(layers, [np_lists(d) for d in deltas[:3]], seeds[:3], CODE[dt], CODE[dt])
    oracle.update(layers, o_part, np_lists(deltas[3]), seeds[3], False, CODE[dt], CODE[dt])
    for l in range(len(stack)):
        compare(part[l], o_part[l], "hot add %d" % l)
    if dt == "f32":  # appending keeps the summation order: identical to a fresh merge of all four
        fresh = rb.merge(layers, gd, seeds)
        for l in range(len(stack)):
            assert torch.equal(part[l].view(torch.int32), fresh[l].view(torch.int32))
    rb.update(layers, part, gd[1], seeds[1], remove=True)
    oracle.update(layers, o_part, np_lists(deltas[1]), seeds[1], True, CODE[dt], CODE[dt])
    for l in range(len(stack)):
        compare(part[l], o_part[l], "hot remove %d" % l)


# ------------------------------------------------------------------ LoRA
@pytest.mark.parametrize("dt_ab,dt_out", [("bf16", "bf16"), ("bf16", "f32"), ("f32", "f32"), ("f32", "bf16")])
@pytest.mark.parametrize("rows,cols,rank", [(768, 768, 16), (70, 100, 16), (33, 129, 5), (64, 256, 40), (1, 1, 1)])
def test_lora_materialize(dt_ab, dt_out, rows, cols, rank):
    g = torch.Generator().manual_seed(rows * 1000 + cols + rank)
    B = (torch.randn(rows, rank, generator=g) * 0.01).to(TD[dt_ab])
    A = (torch.randn(rank, cols, generator=g) * 0.01).to(TD[dt_ab])
    scale = 2.0
    got = rb.lora_materialize(B.cuda(), A.cuda(), scale, out_dtype=TD[dt_out]).float().cpu().numpy().astype(np.float64)
    want, mag = oracle.lora(to_np(B), to_np(A), scale, CODE[dt_ab])
    # binary32 accumulation in any order: rank * 2^-24 * sum|B||A|; one more rounding for the
    # scale multiply; half a bf16 ulp (2^-9 relative) if the output is bf16
    tol = rank * 2.0 ** -24 * mag + 2.0 ** -23 * np.abs(want) + 1e-45
    if dt_out == "bf16":
        tol = tol + 2.0 ** -8 * np.abs(want) + 2.0 ** -133
    err = np.abs(got - want)
    assert (err <= tol).all(), (err.max(), tol[err > tol].min() if (err > tol).any() else None)


def test_lora_exact_cases_and_batched():
    # power-of-two valued factors: every product and partial sum is exact, so any order agrees exactly
    g = torch.Generator().manual_seed(3)
    B = (2.0 ** torch.randint(-3, 4, (96, 16), generator=g).float()) * (torch.randint(0, 2, (96, 16), generator=g) * 2 - 1)
    A = (2.0 ** torch.randint(-3, 4, (16, 160), generator=g).float()) * (torch.randint(0, 2, (16, 160), generator=g) * 2 - 1)
    want, _ = oracle.lora(B.numpy(), A.numpy(), 1.0, 0)
    for dt in ("bf16", "f32"):
        got = rb.lora_materialize(B.to(TD[dt]).cuda(), A.to(TD[dt]).cuda(), 1.0, out_dtype=torch.float32)
        assert np.array_equal(got.cpu().numpy().astype(np.float64), want)
    # identity-padded B copies A
    Bi = torch.zeros(40, 16)
    Bi[:16] = torch.eye(16)
    Ar = torch.randn(16, 72, generator=g).to(torch.bfloat16)
    got = rb.lora_materialize(Bi.to(torch.bfloat16).cuda(), Ar.cuda(), 1.0)
    assert torch.equal(got[:16].cpu(), Ar) and (got[16:] == 0).all()
    # batched = one by one
    Bs = [(torch.randn(r, 16, generator=g) * 0.01).to(torch.bfloat16).cuda() for r in (64, 70, 768)]
    As = [(torch.randn(16, c, generator=g) * 0.01).to(torch.bfloat16).cuda() for c in (128, 100, 768)]
    outs = rb.lora_materialize_batched(Bs, As, 0.5)
    for Bq, Aq, o in zip(Bs, As, outs):
        single = rb.lora_materialize(Bq, Aq, 0.5)
        assert torch.equal(o.view(torch.int16), single.view(torch.int16))


def test_lora_deltas_feed_the_merge_bit_exactly():
    # the GPU-materialised deltas are copied to the host and given to the oracle's merge,
    # so the merge itself stays bit-exact although B.A is only tolerance-checked
    stack = [Layer(768, 768, 0, SRSF)] * 3
    layers = layers_of(stack)
    K = 3
    factors = wl.make_lora_factors(stack, [0, 1, 2], K, rank=16, dtype="bf16", device="cuda")
    deltas = [[rb.lora_materialize(Bq, Aq, 1.0) for (Bq, Aq) in per] for per in factors]
    seeds = [42, 43, 44]
    m = rb.merge(layers, deltas, seeds)
    o_m = oracle.merge(layers, [[to_np(t) for t in per] for per in deltas], seeds, 1, 1, n_threads=8)
    for l in range(3):
        compare(m[l], o_m[l], "lora merge %d" % l)


def test_lora_then_merge_against_an_oracle_only_pipeline():
    # the same two steps with nothing of the GPU in the oracle's inputs: float64 products rounded
    # to bf16 on the host, merged by the oracle.  The GPU's deltas may differ from those by one
    # bf16 unit each (its products are binary32 sums in the hardware's order), so the merged
    # values agree to K such units plus the final rounding.
    stack = [Layer(96, 520, 0, SRSF)] * 3 + [Layer(40, 264, -1, FLIP)]
    layers = layers_of(stack)
    K = 4
    factors = wl.make_lora_factors(stack, list(range(len(stack))), K, rank=16, dtype="bf16", device="cuda")
    seeds = [42 + i for i in range(K)]
    deltas = [rb.lora_materialize_batched([f[0] for f in per], [f[1] for f in per], 1.0) for per in factors]
    got = rb.merge(layers, deltas, seeds)
    host_deltas, biggest = [], 0.0
    for per in factors:
        row = []
        for (Bq, Aq) in per:
            want, _ = oracle.lora(to_np(Bq), to_np(Aq), 1.0, 1)
            biggest = max(biggest, float(np.abs(want).max()))
            row.append(oracle.f32_to_bf16(want.astype(np.float32)))
        host_deltas.append(row)
    want_m = oracle.merge(layers, host_deltas, seeds, 1, 1, n_threads=8)
    for l in range(len(stack)):
        g = got[l].float().cpu().numpy().astype(np.float64)
        w = oracle.bf16_to_f32(want_m[l]).astype(np.float64)
        tol = K * 2.0 ** -7 * biggest + 2.0 ** -7 * np.abs(w)
        assert (np.abs(g - w) <= tol).all(), (l, np.abs(g - w).max())


@pytest.mark.parametrize("dt_ab,dt_out", [("bf16", "bf16"), ("bf16", "f32"), ("f32", "f32")])
@pytest.mark.parametrize("rank,n_tasks", [(16, 8), (5, 3), (40, 2)])
def test_fused_lora_merge(dt_ab, dt_out, rank, n_tasks):
    # sum_i (B_i A_i) D_i with the shuffle, written once: against the float64 oracle
    stack = [Layer(70, 520, 0, SRSF), Layer(64, 1032, 1, SRSF), Layer(70, 520, 0, SRSF), Layer(33, 77, -1, FLIP),
             Layer(64, 1032, 1, SRSF), Layer(70, 520, 0, SRSF)]
    layers = layers_of(stack)
    seeds = [42 + i for i in range(n_tasks)]
    factors = wl.make_lora_factors(stack, list(range(len(stack))), n_tasks, rank=rank, dtype=dt_ab, device="cpu")
    got = rb.lora_merge(layers, [[(B.cuda(), A.cuda()) for (B, A) in per] for per in factors], seeds, 0.5,
                        merged_dtype=TD[dt_out])
    want, mag = oracle.lora_merge(layers, [[(to_np(B), to_np(A)) for (B, A) in per] for per in factors], seeds, 0.5,
                                  CODE[dt_ab])
    for l in range(len(stack)):
        g = got[l].float().cpu().numpy().astype(np.float64)
        tol = n_tasks * rank * 2.0 ** -24 * mag[l] + 2.0 ** -23 * np.abs(want[l]) + 1e-45
        if dt_out == "bf16":
            tol = tol + 2.0 ** -8 * np.abs(want[l]) + 2.0 ** -133
        err = np.abs(g - want[l])
        assert (err <= tol).all(), (l, err.max())
    # and it agrees with materialise-then-merge up to the intermediate bf16 rounding of each L_i
    if dt_ab == "bf16" and dt_out == "bf16":
        gf = [[(B.cuda(), A.cuda()) for (B, A) in per] for per in factors]
        deltas = [[rb.lora_materialize(B, A, 0.5) for (B, A) in per] for per in gf]
        two_step = rb.merge(layers, deltas, seeds)
        for l in range(len(stack)):
            a, b = got[l].float(), two_step[l].float()
            # each of the n_tasks intermediate roundings is at most half a bf16 ulp of its own L_i
            bound = n_tasks * 2.0 ** -8 * max(d[l].float().abs().max().item() for d in deltas) + 2.0 ** -7 * b.abs().max().item()
            assert ((a - b).abs() <= bound).all()


@pytest.mark.parametrize("dt_out", ["bf16", "f32"])
@pytest.mark.parametrize("rank,n_tasks", [(16, 8), (16, 4), (16, 5), (16, 7), (32, 2), (32, 4), (64, 2), (16, 9)])
def test_fused_lora_merge_of_superpositions_with_wide_accesses(dt_out, rank, n_tasks):
    # Every matrix fit for 16-byte accesses (cols a multiple of 8, bf16 factors): products of 4 to 8 depth
    # slices take the kernel that keeps all fragments of A in registers while it walks down its band (long
    # walks of odd and even length, ragged last row blocks, bands wider than the matrix, slices short of 8),
    # (16, 9) with its 9 slices the streaming kernel with two row blocks per fetch.
    stack = [Layer(70, 520, 0, SRSF), Layer(1000, 264, 1, SRSF), Layer(70, 520, 0, SRSF), Layer(33, 8, -1, FLIP),
             Layer(1000, 264, 1, SRSF), Layer(1, 1032, -1, FLIP), Layer(2049, 256, -1, FLIP), Layer(70, 520, 0, SRSF)]
    layers = layers_of(stack)
    seeds = [1000 + 7 * i for i in range(n_tasks)]
    factors = wl.make_lora_factors(stack, list(range(len(stack))), n_tasks, rank=rank, dtype="bf16", device="cpu")
    got = rb.lora_merge(layers, [[(B.cuda(), A.cuda()) for (B, A) in per] for per in factors], seeds, 0.75,
                        merged_dtype=TD[dt_out])
    want, mag = oracle.lora_merge(layers, [[(to_np(B), to_np(A)) for (B, A) in per] for per in factors], seeds, 0.75,
                                  CODE["bf16"])
    for l in range(len(stack)):
        g = got[l].float().cpu().numpy().astype(np.float64)
        tol = n_tasks * rank * 2.0 ** -24 * mag[l] + 2.0 ** -23 * np.abs(want[l]) + 1e-45
        if dt_out == "bf16":
            tol = tol + 2.0 ** -8 * np.abs(want[l]) + 2.0 ** -133
        err = np.abs(g - want[l])
        assert (err <= tol).all(), (l, err.max())


@pytest.mark.parametrize("dt,dt_merged", [("f32", "f32"), ("bf16", "bf16"), ("bf16", "f32")])
@pytest.mark.parametrize("n_tasks", [1, 3, 4, 8, 11])
def test_merge_from_weights(dt, dt_merged, n_tasks):
    stack = ragged_stack()
    layers = layers_of(stack)
    seeds = [42 + i for i in range(n_tasks)]
    base, deltas = cpu_inputs(stack, n_tasks, "f32")
    weights = [[(b + d).to(TD[dt]) for b, d in zip(base, per)] for per in deltas]
    base = [b.to(TD[dt]) for b in base]
    got = rb.merge_weights(layers, [to_gpu(w) for w in weights], to_gpu(base), seeds, merged_dtype=TD[dt_merged])
    want = oracle.merge_weights(layers, [np_lists(w) for w in weights], np_lists(base), seeds,
                                CODE[dt], CODE[dt_merged], n_threads=8)
    for l in range(len(stack)):
        compare(got[l], want[l], "merge from weights, layer %d" % l)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_delta_stats(dt):
    stack = ragged_stack()
    layers = layers_of(stack)
    _, deltas = cpu_inputs(stack, 2, dt, delta_std=1.0)
    ga, gb = to_gpu(deltas[0]), to_gpu(deltas[1])
    na, nb = np_lists(deltas[0]), np_lists(deltas[1])
    for (sa, sb, lay) in ((42, 43, layers), (42, 42, layers), (1, 2, [(m, n, g, 0) for (m, n, g, _) in layers])):
        got = rb.delta_stats(lay, ga, sa, gb, sb).cpu().numpy()
        want = np.array(oracle.delta_stats(lay, na, sa, nb, sb, CODE[dt]))
        scale = np.sqrt(want[1] * want[2])
        assert np.all(np.abs(got - want) <= 1e-11 * scale), (got, want)
    # decorrelation: identical deltas under different seeds are nearly orthogonal, under equal seeds parallel
    # (on layers that all carry the flip; the ragged stack has an unflagged layer that stays correlated)
    flagged = [(64, 2048, 0, SRSF)] * 4
    _, fd = cpu_inputs([Layer(*l) for l in flagged], 1, dt, delta_std=1.0)
    gf = to_gpu(fd[0])
    c_diff = rb.delta_stats(flagged, gf, 42, gf, 43).cpu().numpy()
    c_same = rb.delta_stats(flagged, gf, 42, gf, 42).cpu().numpy()
    assert abs(c_same[0] / np.sqrt(c_same[1] * c_same[2]) - 1.0) < 1e-12
    assert abs(c_diff[0] / np.sqrt(c_diff[1] * c_diff[2])) < 0.05
    # reproducible bit for bit
    again = rb.delta_stats(flagged, gf, 42, gf, 43).cpu().numpy()
    assert np.array_equal(again.view(np.uint64), c_diff.view(np.uint64))


def test_factor_space_lora_superposition():
    # The paper superposes "LoRA weight vectors": the factors A and B themselves can be the layers of
    # the same merge / retrieve kernels (storage stays at adapter size); the dense update is then
    # materialised from the retrieved factors.  A factors form one group, B factors another.
    n_mod, rank, K = 6, 16, 3
    stack = []
    for _ in range(n_mod):
        stack.append(Layer(rank, 768, 0, SRSF))   # A: rank x cols
        stack.append(Layer(768, rank, 1, SRSF))   # B: rows x rank
    layers = layers_of(stack)
    seeds = [42, 43, 44]
    g = torch.Generator().manual_seed(7)
    factors = [[(torch.randn(l.rows, l.cols, generator=g) * 0.01).to(torch.bfloat16) for l in stack] for _ in range(K)]
    zero = [torch.zeros(l.rows, l.cols, dtype=torch.bfloat16) for l in stack]
    gm = rb.merge(layers, [to_gpu(f) for f in factors], seeds)
    om = oracle.merge(layers, [np_lists(f) for f in factors], seeds, 1, 1)
    for l in range(len(stack)):
        compare(gm[l], om[l], "factor merge %d" % l)
    got = rb.retrieve(layers, gm, to_gpu(zero), seeds[1], 1.0)
    want = oracle.retrieve(layers, om, np_lists(zero), seeds[1], 1.0, 1, 1, 1)
    for l in range(len(stack)):
        compare(got[l], want[l], "factor retrieve %d" % l)
    # dense update of module 2 from the retrieved factors, against the float64 product of the same factors
    A_hat, B_hat = got[4], got[5]
    dense = rb.lora_materialize(B_hat, A_hat, 1.0, out_dtype=torch.float32).cpu().numpy().astype(np.float64)
    ref, mag = oracle.lora(to_np(B_hat), to_np(A_hat), 1.0, 1)
    assert (np.abs(dense - ref) <= rank * 2.0 ** -24 * mag + 2.0 ** -23 * np.abs(ref) + 1e-45).all()
    # a single model comes back exactly
    g1 = rb.merge(layers, [to_gpu(factors[0])], [seeds[0]])
    back = rb.retrieve(layers, g1, to_gpu(zero), seeds[0], 1.0)
    for l in range(len(stack)):
        assert torch.equal(back[l].cpu().view(torch.int16), factors[0][l].view(torch.int16))


@pytest.mark.parametrize("rows,cols", [(3, 5_000_008), (1, 33_554_432), (300_000, 8), (2, 40_000_001), (70_001, 24)])
def test_extreme_shapes(rows, cols):
    # very wide (many generator blocks, offsets near the 32-bit in-tile limit) and very tall, thin layers
    stack = [Layer(rows, cols, -1, FLIP)]
    layers = layers_of(stack)
    base, deltas = cpu_inputs(stack, 2, "bf16")
    seeds = [5, 6]
    m = rb.merge(layers, [to_gpu(d) for d in deltas], seeds)
    om = oracle.merge(layers, [np_lists(d) for d in deltas], seeds, 1, 1, n_threads=8)
    compare(m[0], om[0], "extreme merge")
    out = rb.retrieve(layers, m, to_gpu(base), 6, 0.5)
    oo = oracle.retrieve(layers, om, np_lists(base), 6, 0.5, 1, 1, 1, n_threads=8)
    compare(out[0], oo[0], "extreme retrieve")


def aligned_stack():
    """Every layer on the vector path (cols a multiple of 8, 256-byte aligned allocations):
    ragged row tails, partly filled column tiles, two shuffle groups, a shifted group, singletons."""
    return [
        Layer(130, 1032, 0, SRSF), Layer(70, 520, 1, SRSF), Layer(130, 1032, 0, SRSF),
        Layer(257, 136, -1, FLIP), Layer(70, 520, 1, SRSF), Layer(130, 1032, 0, SRSF),
        Layer(1, 3000, -1, FLIP), Layer(33, 2048, 2, FLIP | SHIFT), Layer(33, 2048, 2, FLIP | SHIFT),
        Layer(33, 2048, 2, FLIP | SHIFT), Layer(64, 4104, -1, 0), Layer(9, 8, -1, FLIP),
    ]


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("n_req", [1, 2, 3, 5, 8, 11, 15])
def test_retrieve_many_equals_single_retrievals_and_the_oracle(dt, n_req):
    # 15 = 8 + 4 + 2 + 1 exercises every pass size; seeds repeat (several requests for one model)
    stack = aligned_stack()
    layers = layers_of(stack)
    K = 4
    seeds = [900 + i for i in range(K)]
    base, deltas = cpu_inputs(stack, K, dt)
    g_merged = rb.merge(layers, [to_gpu(d) for d in deltas], seeds)
    o_merged = oracle.merge(layers, [np_lists(d) for d in deltas], seeds, CODE[dt], CODE[dt], n_threads=8)
    g_base = to_gpu(base)
    req_seeds = [seeds[(3 * q + 1) % K] for q in range(n_req)]
    lams = [0.25 + 0.125 * q for q in range(n_req)]
    outs = rb.retrieve_many(layers, g_merged, g_base, req_seeds, lams)
    assert len(outs) == n_req
    for q in range(n_req):
        single = rb.retrieve(layers, g_merged, g_base, req_seeds[q], lams[q])
        want = oracle.retrieve(layers, o_merged, np_lists(base), req_seeds[q], lams[q],
                               CODE[dt], CODE[dt], CODE[dt], n_threads=8)
        for l in range(len(stack)):
            assert torch.equal(outs[q][l].view(torch.int16 if dt == "bf16" else torch.int32),
                               single[l].view(torch.int16 if dt == "bf16" else torch.int32))
            compare(outs[q][l], want[l], "request %d layer %d" % (q, l))


@pytest.mark.parametrize("case", ["ragged", "mixed_dtypes", "launch_shape"])
def test_retrieve_many_other_paths(case):
    # layers off the vector path, or stacks of different dtypes, are served request by request;
    # the launch-shape knob must not change the result of the one-pass kernel
    stack = ragged_stack() if case == "ragged" else aligned_stack()
    layers = layers_of(stack)
    K, dt = 3, "bf16"
    seeds = [77, 78, 79]
    base, deltas = cpu_inputs(stack, K, dt)
    d_merged = "f32" if case == "mixed_dtypes" else dt
    g_merged = rb.merge(layers, [to_gpu(d) for d in deltas], seeds, merged_dtype=TD[d_merged])
    o_merged = oracle.merge(layers, [np_lists(d) for d in deltas], seeds, CODE[dt], CODE[d_merged], n_threads=8)
    g_base = to_gpu(base)
    if case == "launch_shape":
        rb.set_tile_cols(1)
    req = [79, 77, 78, 77]
    lams = [1.0, 0.5, 2.0, 0.0]
    outs = rb.retrieve_many(layers, g_merged, g_base, req, lams)
    for q in range(len(req)):
        want = oracle.retrieve(layers, o_merged, np_lists(base), req[q], lams[q],
                               CODE[d_merged], CODE[dt], CODE[dt], n_threads=8)
        for l in range(len(stack)):
            compare(outs[q][l], want[l], "%s request %d layer %d" % (case, q, l))


def test_retrieve_many_rejects_overlapping_outputs():
    stack = aligned_stack()[:3]
    layers = layers_of(stack)
    base, deltas = cpu_inputs(stack, 2, "f32")
    g_merged = rb.merge(layers, [to_gpu(d) for d in deltas], [1, 2])
    g_base = to_gpu(base)
    one = rb.alloc_like_layers(layers, torch.float32)
    with pytest.raises(rb.RandesError):      # two requests into one output stack
        rb.retrieve_many(layers, g_merged, g_base, [1, 2], [1.0, 1.0], outs=[one, one])
    with pytest.raises(rb.RandesError):      # an output stack that is the base
        rb.retrieve_many(layers, g_merged, g_base, [1, 2], [1.0, 1.0], outs=[one, g_base])
    with pytest.raises(rb.RandesError):
        rb.retrieve_many(layers, g_merged, g_base, [1, 2], [1.0, float("nan")])


def test_plan_cache_eviction_and_reuse():
    # more distinct calls than the cache holds: old tables are dropped, results stay right, and a
    # call whose tables were dropped builds them again
    stack = [Layer(40, 264, 0, SRSF), Layer(40, 264, 0, SRSF), Layer(9, 77, -1, FLIP)]
    layers = layers_of(stack)
    base, deltas = cpu_inputs(stack, 2, "f32")
    seeds = [5, 6]
    g_d = [to_gpu(d) for d in deltas]
    g_merged = rb.merge(layers, g_d, seeds)
    o_merged = oracle.merge(layers, [np_lists(d) for d in deltas], seeds, 0, 0)
    g_base = to_gpu(base)
    out = rb.alloc_like_layers(layers, torch.float32)
    for rnd in range(2):
        for s in range(300):          # 300 different seeds = 300 different table sets; the cache keeps 256
            rb.retrieve(layers, g_merged, g_base, 1000 + s, 1.0, out=out)
            if s in (0, 141, 299):
                want = oracle.retrieve(layers, o_merged, np_lists(base), 1000 + s, 1.0, 0, 0, 0)
                for l in range(len(stack)):
                    compare(out[l], want[l], "round %d seed %d layer %d" % (rnd, s, l))
    again = rb.merge(layers, g_d, seeds)      # its tables were dropped long ago
    for l in range(len(stack)):
        compare(again[l], o_merged[l], "merged again %d" % l)


def test_tables_of_dropped_argument_sets_are_released_in_batches():
    # a loop over far more argument sets than the cache keeps must not grow device memory without bound,
    # and results stay right across the releases
    stack = [Layer(8, 256, g % 7, SRSF) for g in range(420)]
    layers = layers_of(stack)
    lt = rb.LayerTable(layers)
    base, deltas = cpu_inputs(stack, 1, "f32")
    gm, gb = to_gpu(deltas[0]), to_gpu(base)
    t_m, t_b = rb.PtrTable(gm, lt), rb.PtrTable(gb, lt)
    out = rb.alloc_like_layers(lt, torch.float32)
    t_o = rb.PtrTable(out, lt)
    want = {}
    for seed in (5, 2500, 7999):
        o = oracle.retrieve(layers, np_lists(gm), np_lists(gb), seed, 0.5)
        want[seed] = o
    torch.cuda.synchronize()
    free = [torch.cuda.mem_get_info()[0]]
    for seed in range(8000):
        rb.retrieve(lt, t_m, t_b, seed, 0.5, out=t_o)
        if seed in want:
            torch.cuda.synchronize()
            for l in (0, 211, 419):
                bits_equal(out[l], want[seed][l], "seed %d layer %d" % (seed, l))
        if seed % 500 == 499:
            torch.cuda.synchronize()
            free.append(torch.cuda.mem_get_info()[0])
    used = [(free[0] - f) >> 20 for f in free]
    print("device memory taken after every 500 argument sets (MiB):", used)
    # a set's tables are about 30 KB: 8000 sets would hold some 250 MiB if none were released; released in
    # batches of 64 MiB and more, what is held goes up and down and ends far below that
    assert max(used) < 160 and used[-1] < 160
    assert any(b < a for a, b in zip(used, used[1:])), "nothing was ever released"


def test_cached_calls_can_be_captured_in_a_graph():
    # once a call's tables are cached it only launches kernels, so it can be recorded into a HIP
    # graph; every replay must give what the eager call gives on the data of that moment
    stack = aligned_stack()
    layers = layers_of(stack)
    K, dt = 3, "bf16"
    seeds = [11, 12, 13]
    base, deltas = cpu_inputs(stack, K, dt)
    g_d = [to_gpu(d) for d in deltas]
    g_base = to_gpu(base)
    lt = rb.LayerTable(layers)
    t_d = rb.PtrTable([t for per in g_d for t in per], lt)
    merged = rb.alloc_like_layers(layers, TD[dt])
    out = rb.alloc_like_layers(layers, TD[dt])
    t_m, t_b, t_o = rb.PtrTable(merged, lt), rb.PtrTable(g_base, lt), rb.PtrTable(out, lt)
    stats = torch.zeros(3, dtype=torch.float64, device="cuda")
    t_d0, t_d1 = rb.PtrTable(g_d[0], lt), rb.PtrTable(g_d[1], lt)

    def run():
        rb.merge(lt, t_d, seeds, merged=t_m)
        rb.retrieve(lt, t_m, t_b, seeds[1], 0.5, out=t_o)
        rb.delta_stats(lt, t_d0, seeds[0], t_d1, seeds[1], out=stats)
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        run()                               # builds and caches the tables (the diagnostics' are per stream)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph.capture_begin()
        try:
            run()
        finally:
            graph.capture_end()
    torch.cuda.synchronize()
    for rnd in range(3):
        # new data in the same buffers, eager result first
        for per in g_d:
            for t in per:
                t.mul_(1.5 + rnd)
        run()
        torch.cuda.synchronize()
        want_m = [t.clone() for t in merged]
        want_o = [t.clone() for t in out]
        want_s = stats.clone()
        for t in merged + out:
            t.zero_()
        stats.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for l in range(len(stack)):
            assert torch.equal(merged[l].view(torch.int16), want_m[l].view(torch.int16)), (rnd, l)
            assert torch.equal(out[l].view(torch.int16), want_o[l].view(torch.int16)), (rnd, l)
        assert torch.equal(stats, want_s)
    # tables of recorded calls survive the cache's turnover: 300 other calls, then one more replay
    scratch = rb.alloc_like_layers(layers, TD[dt])
    for s_ in range(300):
        rb.retrieve(lt, t_m, t_b, 70000 + s_, 1.0, out=scratch)
    torch.cuda.synchronize()
    for t in merged + out:
        t.zero_()
    graph.replay()
    torch.cuda.synchronize()
    for l in range(len(stack)):
        assert torch.equal(merged[l].view(torch.int16), want_m[l].view(torch.int16)), l
        assert torch.equal(out[l].view(torch.int16), want_o[l].view(torch.int16)), l
    # and the eager result is the oracle's
    o_m = oracle.merge(layers, [[to_np(t) for t in per] for per in g_d], seeds, CODE[dt], CODE[dt], n_threads=8)
    for l in range(len(stack)):
        compare(merged[l], o_m[l], "graph replay, merged %d" % l)


@pytest.mark.parametrize("trial", range(int(os.environ.get("RANDES_RANDOM_TRIALS", "24"))))
def test_random_stacks_through_every_streaming_entry_point(trial):
    # randomly drawn stacks (shapes on and off the vector path, random groups and flags), model
    # counts, dtypes and scales; merge, retrieve, several retrievals per pass, hot add / remove and
    # merge-from-weights against the oracle
    rnd = np.random.RandomState(7000 + trial)
    shapes = [(rnd.randint(1, 70), int(rnd.choice([1, 7, 8, 64, 130, 136, 384, 520, 640, 768, 1032, 2056]))) for _ in range(3)]
    stack = []
    for _ in range(rnd.randint(1, 9)):
        g = int(rnd.randint(-1, 3))
        rows, cols = shapes[g] if g >= 0 else (rnd.randint(1, 40), int(rnd.choice([3, 8, 24, 100, 264])))
        flags = int(rnd.choice([0, FLIP, SHUFFLE, SRSF, SRSF, SRSF]))
        stack.append(Layer(int(rows), int(cols), g, flags))
    if rnd.rand() < 0.25:          # one group shifted instead of shuffled
        stack = [Layer(l.rows, l.cols, l.group, (l.flags & FLIP) | SHIFT) if l.group == 0 else l for l in stack]
    layers = layers_of(stack)
    K = int(rnd.randint(1, 11))
    d_in = str(rnd.choice(["f32", "bf16"]))
    d_merged = str(rnd.choice(["f32", "bf16"]))
    d_out = str(rnd.choice(["f32", "bf16"]))
    seeds = [int(s) for s in rnd.randint(0, 2 ** 31, size=K)]
    seeds[0] = (seeds[0] << 33) | 5          # both key halves in use
    lam = float(rnd.choice([1.0, 0.3, -0.75, 2.0]))
    gm, om = run_both(stack, K, seeds, d_in, d_merged, d_in, d_out, lam, sorted({0, K - 1}), data_seed=trial)
    base, deltas = cpu_inputs(stack, K, d_in, trial)
    g_base = to_gpu(base)
    # several retrievals in one pass
    n_req = int(rnd.randint(1, 6))
    req = [seeds[int(i)] for i in rnd.randint(0, K, size=n_req)]
    lams = [float(x) for x in rnd.choice([1.0, 0.5, 0.0, -1.25], size=n_req)]
    outs = rb.retrieve_many(layers, gm, g_base, req, lams, out_dtype=TD[d_out])
    for q in range(n_req):
        want = oracle.retrieve(layers, om, np_lists(base), req[q], lams[q], CODE[d_merged], CODE[d_in], CODE[d_out])
        for l in range(len(stack)):
            compare(outs[q][l], want[l], "trial %d request %d layer %d" % (trial, q, l))
    # hot add of a further model, then removal of the first
    _, extra = cpu_inputs(stack, 1, d_in, trial + 500)
    rb.update(layers, gm, to_gpu(extra[0]), 31337)
    oracle.update(layers, om, np_lists(extra[0]), 31337, False, CODE[d_merged], CODE[d_in])
    rb.update(layers, gm, to_gpu(deltas[0]), seeds[0], remove=True)
    oracle.update(layers, om, np_lists(deltas[0]), seeds[0], True, CODE[d_merged], CODE[d_in])
    for l in range(len(stack)):
        compare(gm[l], om[l], "trial %d after hot swap, layer %d" % (trial, l))
    # merge straight from weights (here: base + delta rounded to the storage dtype)
    weights = [[(b.float() + d.float()).to(TD[d_in]) for b, d in zip(base, per)] for per in deltas]
    gw = rb.merge_weights(layers, [to_gpu(w) for w in weights], g_base, seeds, merged_dtype=TD[d_merged])
    ow = oracle.merge_weights(layers, [np_lists(w) for w in weights], np_lists(base), seeds, CODE[d_in], CODE[d_merged])
    for l in range(len(stack)):
        compare(gw[l], ow[l], "trial %d merge from weights, layer %d" % (trial, l))


def folding_stack():
    """Layers whose rows are folded on the vector path (cols a multiple of 128 that leaves lanes of the
    column tiles idle), with row counts that divide by the fold factor, leave a remainder, or are too
    few to fold; groups of them are shuffled; one layer that never folds."""
    return [
        Layer(70, 768, 0, SRSF), Layer(70, 768, 0, SRSF), Layer(70, 768, 0, SRSF),
        Layer(7, 384, 1, SRSF), Layer(7, 384, 1, SRSF),
        Layer(1, 768, -1, FLIP), Layer(2, 640, -1, FLIP), Layer(3, 1152, -1, FLIP),
        Layer(9, 11008, -1, FLIP), Layer(33, 2048, -1, FLIP), Layer(5, 896, -1, 0), Layer(11, 1664, -1, FLIP),
    ]


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_folded_rows_match_the_oracle_and_the_unfolded_launch(dt):
    stack = folding_stack()
    layers = layers_of(stack)
    K = 3
    seeds = [3, (9 << 40) | 4, 5]
    try:
        rb.set_fold(True)
        gm, om = run_both(stack, K, seeds, dt, dt, dt, dt, 0.75, [0, 2])
        base, deltas = cpu_inputs(stack, K, dt)
        g_base, g_d = to_gpu(base), [to_gpu(d) for d in deltas]
        outs = rb.retrieve_many(layers, gm, g_base, [seeds[1], seeds[0]], [1.0, -0.5])
        stats = rb.delta_stats(layers, g_d[0], seeds[0], g_d[1], seeds[1]).cpu().numpy()
        weights = [[(b.float() + d.float()).to(TD[dt]) for b, d in zip(base, per)] for per in deltas]
        gw = rb.merge_weights(layers, [to_gpu(w) for w in weights], g_base, seeds)
        rb.update(layers, gm, g_d[1], seeds[1], remove=True)
        # the same calls with folding off: identical bits
        rb.set_fold(False)
        gm2 = rb.merge(layers, g_d, seeds)
        outs2 = rb.retrieve_many(layers, gm2, g_base, [seeds[1], seeds[0]], [1.0, -0.5])
        stats2 = rb.delta_stats(layers, g_d[0], seeds[0], g_d[1], seeds[1]).cpu().numpy()
        gw2 = rb.merge_weights(layers, [to_gpu(w) for w in weights], g_base, seeds)
        rb.update(layers, gm2, g_d[1], seeds[1], remove=True)
    finally:
        rb.set_fold(True)
    view = torch.int16 if dt == "bf16" else torch.int32
    for l in range(len(stack)):
        assert torch.equal(gm[l].view(view), gm2[l].view(view)), l
        assert torch.equal(gw[l].view(view), gw2[l].view(view)), l
        for q in range(2):
            assert torch.equal(outs[q][l].view(view), outs2[q][l].view(view)), (q, l)
    # the reduction's grouping changes with the tiling, its value to rounding does not
    np.testing.assert_allclose(stats, stats2, rtol=1e-12)
    for q, (sd, lam) in enumerate([(seeds[1], 1.0), (seeds[0], -0.5)]):
        want = oracle.retrieve(layers, om, np_lists(base), sd, lam, CODE[dt], CODE[dt], CODE[dt])
        for l in range(len(stack)):
            compare(outs[q][l], want[l], "folded, request %d layer %d" % (q, l))
    oracle.update(layers, om, np_lists(deltas[1]), seeds[1], True, CODE[dt], CODE[dt])
    ow = oracle.merge_weights(layers, [np_lists(w) for w in weights], np_lists(base), seeds, CODE[dt], CODE[dt])
    for l in range(len(stack)):
        compare(gm[l], om[l], "folded, after removal, layer %d" % l)
        compare(gw[l], ow[l], "folded, merge from weights, layer %d" % l)
    a = np.concatenate([x.astype(np.float64).ravel() for x in oracle.merge(layers, [np_lists(deltas[0])], [seeds[0]], CODE[dt], 0)])
    b = np.concatenate([x.astype(np.float64).ravel() for x in oracle.merge(layers, [np_lists(deltas[1])], [seeds[1]], CODE[dt], 0)])
    np.testing.assert_allclose(stats, [a @ b, a @ a, b @ b], rtol=1e-10)


def test_first_call_during_capture_is_refused_before_anything_is_recorded():
    # a call whose tables are not cached yet would have to allocate and copy: under capture it returns
    # RANDES_ENOTSUP and records nothing; after one eager call the same call records fine
    stack = aligned_stack()[:3]
    layers = layers_of(stack)
    base, deltas = cpu_inputs(stack, 2, "f32")
    g_d = [to_gpu(d) for d in deltas]
    merged = rb.alloc_like_layers(layers, torch.float32)
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    counter = torch.zeros(8, device="cuda")
    with torch.cuda.stream(side):
        graph.capture_begin()
        try:
            counter.add_(1.0)              # so that the recorded graph is not empty
            with pytest.raises(rb.RandesError) as err:
                rb.merge(layers, g_d, [901, 902], merged=merged)
        finally:
            graph.capture_end()
    assert err.value.code == -2 and "eagerly" in str(err.value)
    torch.cuda.synchronize()
    graph.replay()                         # the capture itself survived the refused call
    torch.cuda.synchronize()
    assert counter.tolist() == [1.0] * 8
    want = rb.merge(layers, g_d, [901, 902], merged=merged)       # eager: builds the tables
    torch.cuda.synchronize()
    want = [t.clone() for t in want]
    graph2 = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph2.capture_begin()
        try:
            rb.merge(layers, g_d, [901, 902], merged=merged)
        finally:
            graph2.capture_end()
    for t in merged:
        t.zero_()
    torch.cuda.synchronize()
    graph2.replay()
    torch.cuda.synchronize()
    for l in range(len(stack)):
        assert torch.equal(merged[l], want[l]), l


def test_concurrent_callers_on_their_own_streams():
    # several host threads, each with its own stream and output stack, share the library's table
    # cache: 320 distinct calls are live at once, more than the 256 it keeps, so table sets are dropped
    # and rebuilt while other threads launch
    import threading
    stack = aligned_stack()[:6]
    layers = layers_of(stack)
    K, dt = 3, "f32"
    seeds = [21, 22, 23]
    base, deltas = cpu_inputs(stack, K, dt)
    g_merged = rb.merge(layers, [to_gpu(d) for d in deltas], seeds)
    g_base = to_gpu(base)
    torch.cuda.synchronize()
    n_threads, n_calls = 4, 80
    outs = [rb.alloc_like_layers(layers, torch.float32) for _ in range(n_threads)]
    errors = []

    def worker(w):
        try:
            s = torch.cuda.Stream()
            for rnd in range(2):
                for c in range(n_calls):
                    rb.retrieve(layers, g_merged, g_base, 5000 + 100 * w + c, 1.0, out=outs[w], stream=s)
            s.synchronize()
        except Exception as e:        # noqa: BLE001
            errors.append(repr(e))
    threads = [threading.Thread(target=worker, args=(w,)) for w in range(n_threads)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    torch.cuda.synchronize()
    o_merged = oracle.merge(layers, [np_lists(d) for d in deltas], seeds, 0, 0)
    for w in range(n_threads):
        want = oracle.retrieve(layers, o_merged, np_lists(base), 5000 + 100 * w + n_calls - 1, 1.0, 0, 0, 0)
        for l in range(len(stack)):
            compare(outs[w][l], want[l], "thread %d layer %d" % (w, l))


def test_equal_delta_stats_calls_on_two_streams_do_not_share_partial_sums():
    # two host threads issue the same diagnostics call (same stacks, same seeds), each on its own stream,
    # many times over while the other runs: every result must be the one the call gives alone
    import threading
    stack = [Layer(900, 1032, 0, SRSF)] * 3 + [Layer(257, 136, -1, FLIP)]
    layers = layers_of(stack)
    _, deltas = cpu_inputs(stack, 2, "f32", delta_std=1.0)
    ga, gb = to_gpu(deltas[0]), to_gpu(deltas[1])
    alone = rb.delta_stats(layers, ga, 42, gb, 43).cpu().numpy()
    want = np.array(oracle.delta_stats(layers, np_lists(deltas[0]), 42, np_lists(deltas[1]), 43, 0))
    assert np.all(np.abs(alone - want) <= 1e-11 * np.sqrt(want[1] * want[2]))
    n_calls = 200
    results = [torch.zeros((n_calls, 3), dtype=torch.float64, device="cuda") for _ in range(2)]
    errors = []
    go = threading.Barrier(2)

    def worker(w):
        try:
            s = torch.cuda.Stream()
            go.wait()
            for c in range(n_calls):
                rb.delta_stats(layers, ga, 42, gb, 43, out=results[w][c], stream=s)
            s.synchronize()
        except Exception as e:        # noqa: BLE001
            errors.append(repr(e))
    threads = [threading.Thread(target=worker, args=(w,)) for w in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    torch.cuda.synchronize()
    for w in range(2):
        got = results[w].cpu().numpy()
        assert np.array_equal(got.view(np.uint64), np.tile(alone.view(np.uint64), (n_calls, 1))), w

"""CPU-only checks of the GPU library's host side: it loads, exports what the
header declares, its host-only entry points agree with the oracle, and bad
arguments come back as error codes before any GPU work."""
import ctypes
import os
import re

import pytest

import oracle
from paper_2505_11204_amd import binding as rb
from paper_2505_11204_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(rb.LIB_PATH):
        from paper_2505_11204_amd import build
        build.build(force=True)
    return rb.lib()


@pytest.mark.parametrize("header_name,exports", [("randes.h", rb.EXPORTS), ("randes_bench.h", rb.BENCH_EXPORTS),
                                                 ("randes_place.h", rb.PLACE_EXPORTS)])
def test_library_exports_every_declared_symbol(lib, header_name, exports):
    header = open(os.path.join(ROOT, "include", header_name)).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(randes_[a-z_]+)\s*\(", header))
    assert declared == set(exports)
    for name in declared:
        assert hasattr(lib, name), name


def test_the_method_header_holds_only_calls_that_cite_the_paper():
    # every declaration of randes.h is preceded by a comment naming the passage it implements (or, for the
    # housekeeping calls, saying what they are); measurement aids live in randes_bench.h
    header = open(os.path.join(ROOT, "include", "randes.h")).read()
    for name in rb.BENCH_EXPORTS:
        assert name not in header
    for name in rb.EXPORTS:
        if name in ("randes_strerror", "randes_shutdown", "randes_lora_materialize_batched", "randes_source_table",
                    "randes_delta_stats_noalloc"):     # the last one names the callers it is for instead
            continue
        decl = header.index("int %s(" % name)
        comment = header.rfind("/*", 0, decl)
        assert re.search(r"Sec\.|App\.", header[comment:decl]), name


def test_layer_perm_matches_oracle(lib):
    for seed in (0, 1, 42, 43, 2**64 - 1, 0x299F31D0A4093822):
        for group in (0, 1, 10):
            for G in (1, 2, 4, 12, 24, 32, 77):
                assert rb.layer_perm(seed, group, G) == oracle.layer_perm(seed, group, G).tolist()


@pytest.mark.parametrize("name", ["tiny", "vit_b32", "vit_l14", "t5_base", "llama_7b"])
def test_source_table_matches_oracle_on_the_benchmark_stacks(lib, name):
    stack = wl.STACKS[name]()
    layers = [(l.rows, l.cols, l.group, l.flags) for l in stack]
    for seed in (42, 49):
        want = oracle.source_table(layers, [seed])[0].tolist()
        assert rb.source_table(layers, seed) == want
        assert sorted(want) == list(range(len(layers)))
        for l, s in enumerate(want):  # only same-shape, same-group layers trade places
            assert layers[l][:3] == layers[s][:3]


def test_source_table_skip_rate_and_shift(lib):
    layers = [(1, 4, 0, (wl.SRSF if k % 2 == 0 else 0)) for k in range(8)] + [(1, 4, 3, wl.SHIFT)] * 5
    for seed in (5, 0, 1, 99, 2 ** 64 - 1, 42, 43):
        want = oracle.source_table(layers, [seed])[0].tolist()
        assert rb.source_table(layers, seed) == want
    assert rb.source_table(layers, 5)[8:] == [12, 8, 9, 10, 11]
    assert rb.source_table(layers, 1)[8:] == [11, 12, 8, 9, 10]


def test_stack_sizes():
    assert wl.n_elements(wl.tiny()) == 262144
    assert wl.n_elements(wl.vit_b32()) == 84934656
    assert wl.n_elements(wl.vit_l14()) == 301989888
    assert wl.n_elements(wl.t5_base()) == 247529472
    assert wl.n_elements(wl.llama_7b()) == 6738149376
    assert len(wl.t5_lora_targets(wl.t5_base())) == 72


def test_bad_arguments_are_error_codes_not_crashes(lib):
    L = rb._Layer
    one = (L * 1)(L(4, 4, 0, 3))
    ptr = (ctypes.c_void_p * 1)(0x1000)
    null = (ctypes.c_void_p * 1)(None)
    seeds = (ctypes.c_uint64 * 1)(1)
    EINVAL, ENOTSUP = -1, -2
    # merge
    assert lib.randes_merge(None, 1, ptr, 1, seeds, 0, ptr, 0, None) == EINVAL
    assert lib.randes_merge(one, 0, ptr, 1, seeds, 0, ptr, 0, None) == EINVAL
    assert lib.randes_merge(one, 1, ptr, 0, seeds, 0, ptr, 0, None) == EINVAL
    assert lib.randes_merge(one, 1, ptr, rb.MAX_TASKS + 1, seeds, 0, ptr, 0, None) == ENOTSUP
    assert lib.randes_merge(one, 1, ptr, 1, seeds, 7, ptr, 0, None) == EINVAL
    assert lib.randes_merge(one, 1, null, 1, seeds, 0, ptr, 0, None) == EINVAL
    assert lib.randes_merge(one, 1, ptr, 1, None, 0, ptr, 0, None) == EINVAL
    odd = (ctypes.c_void_p * 1)(0x1002)   # not a multiple of the f32 element size
    assert lib.randes_merge(one, 1, odd, 1, seeds, 0, ptr, 0, None) == EINVAL
    assert lib.randes_retrieve(one, 1, ptr, 0, ptr, 0, 1, ctypes.c_float(1.0), odd, 0, None) == EINVAL
    bad_rows = (L * 1)(L(0, 4, 0, 3))
    assert lib.randes_merge(bad_rows, 1, ptr, 1, seeds, 0, ptr, 0, None) == EINVAL
    bad_flag = (L * 1)(L(4, 4, 0, 64))
    assert lib.randes_merge(bad_flag, 1, ptr, 1, seeds, 0, ptr, 0, None) == EINVAL
    assert b"flag" in lib.randes_strerror(EINVAL)
    # retrieve: non-finite lambda
    assert lib.randes_retrieve(one, 1, ptr, 0, ptr, 0, 1, ctypes.c_float(float("nan")), ptr, 0, None) == EINVAL
    assert lib.randes_retrieve(one, 1, ptr, 0, ptr, 0, 1, ctypes.c_float(float("inf")), ptr, 0, None) == EINVAL
    assert lib.randes_retrieve(one, 1, ptr, 0, None, 0, 1, ctypes.c_float(1.0), ptr, 0, None) == EINVAL
    lam1 = (ctypes.c_float * 1)(1.0)
    assert lib.randes_retrieve_many(one, 1, ptr, 0, ptr, 0, 0, seeds, lam1, ptr, 0, None) == EINVAL
    assert lib.randes_retrieve_many(one, 1, ptr, 0, ptr, 0, 1, None, lam1, ptr, 0, None) == EINVAL
    assert lib.randes_retrieve_many(one, 1, ptr, 0, ptr, 0, 1, seeds, None, ptr, 0, None) == EINVAL
    assert lib.randes_retrieve_many(one, 1, ptr, 0, ptr, 0, 1, seeds, lam1, null, 0, None) == EINVAL
    assert lib.randes_retrieve_many(one, 1, ptr, 0, ptr, 0, 1, seeds, lam1, odd, 0, None) == EINVAL
    # out == merged == base: overlap is refused before anything is launched
    assert lib.randes_retrieve_many(one, 1, ptr, 0, ptr, 0, 1, seeds, lam1, ptr, 0, None) == EINVAL
    assert b"overlap" in lib.randes_strerror(EINVAL)
    # mismatched group shapes
    two = (L * 2)(L(4, 4, 0, 3), L(4, 8, 0, 3))
    out = (ctypes.c_int32 * 2)()
    assert lib.randes_source_table(two, 2, 1, out) == EINVAL
    assert b"shape" in lib.randes_strerror(EINVAL)
    # perm / mask / lora / knobs
    assert lib.randes_layer_perm(1, 0, 0, out) == EINVAL
    assert lib.randes_layer_perm(1, 0, 2, None) == EINVAL
    assert lib.randes_sign_mask(1, 0, 0, ptr, None) == EINVAL
    assert lib.randes_sign_mask(1, 0, 16, None, None) == EINVAL
    assert lib.randes_lora_materialize(None, ptr, 4, 4, 2, ctypes.c_float(1.0), 0, ptr, 0, None) == EINVAL
    assert lib.randes_lora_materialize(ptr, ptr, 4, 4, 0, ctypes.c_float(1.0), 0, ptr, 0, None) == EINVAL
    assert lib.randes_update(one, 1, ptr, 0, None, 0, 1, 0, None) == EINVAL
    # the fused front-ends, diagnostics and the probe
    assert lib.randes_merge_weights(one, 1, ptr, None, 1, seeds, 0, ptr, 0, None) == EINVAL
    assert lib.randes_merge_weights(one, 1, ptr, null, 1, seeds, 0, ptr, 0, None) == EINVAL
    assert lib.randes_merge_weights(None, 1, ptr, ptr, 1, seeds, 0, ptr, 0, None) == EINVAL
    assert lib.randes_delta_stats(one, 1, ptr, 1, ptr, 2, 0, None, None) == EINVAL
    assert lib.randes_delta_stats(one, 1, null, 1, ptr, 2, 0, ptr, None) == EINVAL
    assert lib.randes_delta_stats(one, 1, ptr, 1, ptr, 2, 9, ptr, None) == EINVAL
    assert lib.randes_lora_merge(one, 1, ptr, ptr, 0, 1, seeds, ctypes.c_float(1.0), 0, ptr, 0, None) == EINVAL
    assert lib.randes_lora_merge(one, 1, ptr, null, 4, 1, seeds, ctypes.c_float(1.0), 0, ptr, 0, None) == EINVAL
    assert lib.randes_lora_merge(one, 1, ptr, ptr, 4, rb.MAX_TASKS + 1, seeds, ctypes.c_float(1.0), 0, ptr, 0, None) == ENOTSUP
    assert lib.randes_lora_merge(one, 1, ptr, ptr, 4, 1, seeds, ctypes.c_float(float("nan")), 0, ptr, 0, None) == EINVAL
    assert lib.randes_lora_merge(one, 1, odd, ptr, 4, 1, seeds, ctypes.c_float(1.0), 0, ptr, 0, None) == EINVAL
    assert lib.randes_lora_merge(one, 1, ptr, ptr, 4, 1, seeds, ctypes.c_float(1.0), 0, odd, 0, None) == EINVAL
    assert lib.randes_lora_materialize(ctypes.c_void_p(0x1001), ptr, 4, 4, 2, ctypes.c_float(1.0), 1, ptr, 1, None) == EINVAL
    assert b"misaligned" in lib.randes_strerror(EINVAL)
    # LoRA outputs that alias a factor or each other are refused before anything is launched
    f1 = ctypes.c_float(1.0)
    pB, pA = ctypes.c_void_p(0x10000), ctypes.c_void_p(0x20000)
    assert lib.randes_lora_materialize(pB, pA, 4, 4, 2, f1, 0, pA, 0, None) == EINVAL          # out is A
    assert b"overlaps a factor" in lib.randes_strerror(EINVAL)
    assert lib.randes_lora_materialize(pB, pA, 4, 4, 2, f1, 0, ctypes.c_void_p(0x10000 + 16), 0, None) == EINVAL   # inside B
    two_b, two_a = (ctypes.c_void_p * 2)(0x10000, 0x11000), (ctypes.c_void_p * 2)(0x20000, 0x21000)
    dims = (ctypes.c_int64 * 2)(4, 4)
    same_out = (ctypes.c_void_p * 2)(0x30000, 0x30000 + 32)       # second output starts inside the first (64 bytes)
    assert lib.randes_lora_materialize_batched(2, two_b, two_a, dims, dims, 2, f1, 0, same_out, 0, None) == EINVAL
    assert b"overlap each other" in lib.randes_strerror(EINVAL)
    merged_is_b = (ctypes.c_void_p * 1)(0x10000)
    assert lib.randes_lora_merge(one, 1, two_b, two_a, 2, 1, seeds, f1, 0, merged_is_b, 0, None) == EINVAL
    assert b"overlaps a factor" in lib.randes_strerror(EINVAL)
    assert lib.randes_probe_stream(ptr, 0, ptr, 16384, 1, None) == EINVAL
    assert lib.randes_probe_stream(ptr, 9, ptr, 16384, 1, None) == EINVAL
    assert lib.randes_probe_stream(ptr, 1, ptr, 1000, 1, None) == EINVAL
    unaligned = (ctypes.c_void_p * 1)(0x1004)
    assert lib.randes_probe_stream(unaligned, 1, ptr, 16384, 1, None) == EINVAL
    assert lib.randes_set_tile_rows(-1, 0) == EINVAL
    assert lib.randes_set_tile_rows(0, 0) == 0
    assert lib.randes_set_tile_cols(3) == EINVAL
    assert lib.randes_set_tile_cols(0) == 0
    assert lib.randes_strerror(0) == b"ok"
    assert lib.randes_shutdown() == 0


def test_row_samplers_of_the_full_size_tests():
    # the bands hold every row of three 128-row ranges (whole tiles of at most 64 rows) and the scattered rows;
    # layers of one shape sample the same rows, whatever their place in the stack
    from paper_2505_11204_amd import workloads as wl
    rows = wl.tile_band_rows(11008)
    for start in (0, 5504 // 128 * 128, 11008 - 128):
        assert set(range(start, start + 128)) <= set(rows)
    assert set(wl.shadow_rows(11008, 16, 99)) <= set(rows)
    assert rows == sorted(set(rows)) and rows[0] == 0 and rows[-1] == 11007
    assert wl.tile_band_rows(100) == list(range(100))
    assert wl.tile_band_rows(4096) == wl.tile_band_rows(4096)

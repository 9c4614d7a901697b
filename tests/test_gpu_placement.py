"""The arena of the HBM placement on the device: chunk classification runs and
returns a label per chunk, and stacks placed inside the arena at the offsets of
a layout (here one that lies across a chunk boundary) give the oracle's results."""
import pytest
import torch

import oracle
from helpers import CODE, compare, layers_of, np_lists
from paper_2505_11204_amd import binding as rb
from paper_2505_11204_amd import placement as pl
from paper_2505_11204_amd import workloads as wl
from paper_2505_11204_amd.workloads import Layer

pytestmark = pytest.mark.gpu


def test_arena_classifies_and_holds_stacks():
    chunk = 64 << 20
    arena = pl.Arena(12 * chunk, chunk_bytes=chunk)
    assert arena.n_chunks == 12
    assert arena.copy_rate(0, 5) > 0
    labels = arena.classify()
    assert len(labels) == 12 and min(labels) == 0 and max(labels) <= 3
    assert sum(b - a for _, a, b in pl.runs_of(labels)) == 12

    stack = [Layer(96, 520, 0, 3), Layer(96, 520, 0, 3), Layer(96, 520, 0, 3), Layer(7, 1000, -1, 1)]
    layers = layers_of(stack)
    K, dtype, td = 3, "bf16", torch.bfloat16
    n = wl.stack_elements(stack, td)
    nbytes = (n * 2 + 255) // 256 * 256
    # the output stack straddles the boundary of chunks 3 and 4, as a layout would put it
    offs = {"base": 0, 0: nbytes, 1: 2 * nbytes, 2: 3 * nbytes, "merged": chunk, "out": 4 * chunk - nbytes // 2 // 256 * 256}
    base, deltas = wl.make_inputs(stack, K, dtype=dtype, device="cuda",
                                  place=lambda who: arena.flat(offs[who], n, td))
    plain_base, plain_deltas = wl.make_inputs(stack, K, dtype=dtype, device="cuda")
    for a, b in zip(base, plain_base):                    # placement does not change the values drawn
        assert torch.equal(a, b)
    _, merged = wl.alloc_stack(stack, td, "cuda", into=arena.flat(offs["merged"], n, td))
    _, out = wl.alloc_stack(stack, td, "cuda", into=arena.flat(offs["out"], n, td))
    seeds = [7, 8, 9]
    rb.merge(layers, deltas, seeds, merged=merged)
    rb.retrieve(layers, merged, base, seeds[1], 0.75, out=out)
    torch.cuda.synchronize()
    want_m = oracle.merge(layers, [np_lists(d) for d in deltas], seeds, CODE[dtype], CODE[dtype])
    want_o = oracle.retrieve(layers, want_m, np_lists(base), seeds[1], 0.75, CODE[dtype], CODE[dtype], CODE[dtype])
    for l in range(len(stack)):
        compare(merged[l], want_m[l], "merged %d" % l)
        compare(out[l], want_o[l], "out %d" % l)

    with pytest.raises(ValueError):
        arena.flat(128, 16, td)
    with pytest.raises(ValueError):
        arena.flat(12 * chunk - 256, 1024, td)
    with pytest.raises(ValueError):
        wl.alloc_stack(stack, td, "cuda", into=arena.flat(0, n + 128, td))

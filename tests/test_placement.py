"""Host logic of the HBM placement (include/randes_place.h through its binding): finding
address groups from copy rates and packing the stacks of a serving set-up into them.  The
rates here come from a model of the behaviour measured on the device (same group slow,
different groups fast, a little noise, a rare slow misread); no GPU is involved.  A second
implementation in plain Python (tests/placement_reference.py) must agree on random cases."""
import random

import pytest

import placement_reference as ref
from paper_2505_11204_amd import placement as pl

GIB = 1 << 30
STACK = 13476298752          # bytes of one Llama-7B-shaped bf16 stack


def rates_of(groups, noise=20.0, seed=0, outliers=0.02):
    rnd = random.Random(seed)

    def rate(r, w):
        v = (5780.0 if groups[r] == groups[w] else 6010.0) + rnd.uniform(-noise, noise)
        if rnd.random() < outliers:
            v -= 200.0
        return v
    return rate


def same_partition(truth, labels, slack=1):
    """Equal up to renaming, ignoring chunks within `slack` of a true boundary."""
    edges = [c for c in range(1, len(truth)) if truth[c] != truth[c - 1]]
    m = {}
    for c, (a, b) in enumerate(zip(truth, labels)):
        if any(abs(c - e) <= slack and c >= e - slack for e in edges):
            continue
        if m.setdefault(a, b) != b:
            return False
    return len(set(m.values())) == len(m)


@pytest.mark.parametrize("seed", range(6))
def test_three_contiguous_groups_are_found(seed):
    truth = [0] * 96 + [1] * 96 + [2] * 82
    labels = pl.classify_chunks(len(truth), rates_of(truth, seed=seed))
    assert same_partition(truth, labels)


@pytest.mark.parametrize("seed", range(6))
def test_groups_in_several_runs_are_found(seed):
    truth = list("X" * 64 + "Y" * 64 + "X" * 32 + "Z" * 32 + "Y" * 24 + "Z" * 32 + "Y" * 8 + "Z" * 22)
    labels = pl.classify_chunks(len(truth), rates_of(truth, seed=seed))
    assert same_partition(truth, labels)


def test_uniform_memory_is_one_group_and_gets_no_layout():
    rnd = random.Random(5)
    labels = pl.classify_chunks(64, lambda r, w: 6000.0 + rnd.uniform(-40, 40) - (200 if rnd.random() < 0.03 else 0))
    assert labels == [0] * 64
    assert pl.plan_serving_layout(labels, GIB, STACK, 8) is None


def test_runs_of():
    assert pl.runs_of([0, 0, 1, 1, 1, 0]) == [(0, 0, 2), (1, 2, 5), (0, 5, 6)]
    assert pl.runs_of([3]) == [(3, 0, 1)]


def check_layout(labels, lay, n_models):
    spans = [(lay["merged"], "merged"), (lay["base"], "base"), (lay["out"], "out")]
    spans += [(d, "delta") for d in lay["deltas"]]
    assert len(lay["deltas"]) == n_models
    # inside the allocation, 256-byte aligned, pairwise disjoint
    for off, _ in spans:
        assert off % 256 == 0 and 0 <= off and off + STACK <= len(labels) * GIB
    order = sorted(off for off, _ in spans)
    assert all(b - a >= STACK for a, b in zip(order, order[1:]))

    def groups_touched(off):
        return {labels[c] for c in range(off // GIB, (off + STACK - 1) // GIB + 1)}
    R = lay["read_group"]
    assert groups_touched(lay["merged"]) == {R} and groups_touched(lay["base"]) == {R}
    assert groups_touched(lay["out"]) == set(lay["write_groups"]) and R not in lay["write_groups"]
    # the output stack lies half and half across the boundary
    edge = next(c for c in range(lay["out"] // GIB, len(labels)) if labels[c] != labels[lay["out"] // GIB]) * GIB
    assert abs((edge - lay["out"]) - STACK / 2) <= 256
    for d in lay["deltas"]:
        assert R not in groups_touched(d)


def test_layout_on_contiguous_groups():
    labels = [1] * 96 + [0] * 96 + [2] * 82
    lay = pl.plan_serving_layout(labels, GIB, STACK, 8)
    check_layout(labels, lay, 8)


def test_layout_on_groups_in_several_runs():
    labels = [0] * 64 + [1] * 64 + [0] * 32 + [2] * 32 + [1] * 24 + [2] * 32 + [1] * 8 + [2] * 22
    lay = pl.plan_serving_layout(labels, GIB, STACK, 8)
    check_layout(labels, lay, 8)


def test_layout_with_more_output_stacks():
    labels = [1] * 96 + [0] * 96 + [2] * 82
    lay = pl.plan_serving_layout(labels, GIB, STACK, 8, n_more_outputs=3)
    check_layout(labels, lay, 8)
    spans = sorted([lay["merged"], lay["base"], lay["out"]] + lay["deltas"] + lay["more_outputs"])
    assert len(lay["more_outputs"]) == 3 and all(b - a >= STACK for a, b in zip(spans, spans[1:]))
    for off in lay["more_outputs"]:
        assert lay["read_group"] not in {labels[c] for c in range(off // GIB, (off + STACK - 1) // GIB + 1)}
    assert pl.plan_serving_layout(labels, GIB, STACK, 8, n_more_outputs=9) is None     # no room outside the read group


def test_layout_needs_room():
    labels = [0] * 20 + [1] * 20 + [2] * 20          # 60 GiB cannot hold eleven 12.55 GiB stacks
    assert pl.plan_serving_layout(labels, GIB, STACK, 8) is None
    assert pl.plan_serving_layout([0] * 96 + [1] * 96, GIB, STACK, 8) is None     # two groups only


def random_groups(rnd, n_chunks):
    """A random map of 1 to 4 groups in runs of 8 chunks and more."""
    n_groups = rnd.randint(1, 4)
    out = []
    while len(out) < n_chunks:
        out += [rnd.randrange(n_groups)] * rnd.randint(8, 80)
    return out[:n_chunks]


@pytest.mark.parametrize("seed", range(40))
def test_library_and_reference_agree_on_random_maps(seed):
    rnd = random.Random(1000 + seed)
    truth = random_groups(rnd, rnd.randint(2, 300))
    noise, outliers = rnd.choice([5.0, 20.0, 60.0]), rnd.choice([0.0, 0.02, 0.1])
    got = pl.classify_chunks(len(truth), rates_of(truth, noise=noise, seed=seed, outliers=outliers))
    want = ref.classify_chunks(len(truth), rates_of(truth, noise=noise, seed=seed, outliers=outliers))
    assert got == want
    assert pl.runs_of(got) == ref.runs_of(want)
    for stack, models, more in ((STACK, 8, 0), (STACK, 8, 3), (1 << 30, 20, 1), (3 << 28, 2, 0), (40 << 30, 1, 0)):
        assert pl.plan_serving_layout(got, GIB, stack, models, more) == ref.plan_serving_layout(want, GIB, stack, models, more)
    # the planners also agree on the true map and on maps nobody measured
    labels = [rnd.randrange(4) for _ in range(rnd.randint(1, 40))] if seed % 2 else truth
    assert pl.plan_serving_layout(labels, GIB, STACK // 4, 3, 1) == ref.plan_serving_layout(labels, GIB, STACK // 4, 3, 1)


def test_classification_options_and_errors():
    truth = [0] * 40 + [1] * 40 + [2] * 40 + [3] * 40
    clean = rates_of(truth, noise=1.0, outliers=0.0)
    assert len(set(pl.classify_chunks(160, clean))) == 4
    assert len(set(pl.classify_chunks(160, clean, max_groups=2))) == 2
    assert pl.classify_chunks(160, clean, min_separation=0.2) == [0] * 160          # 4 % apart is not 20 %
    assert pl.classify_chunks(1, clean) == [0]
    for max_groups in (2, 3):
        assert pl.classify_chunks(160, clean, max_groups=max_groups) == ref.classify_chunks(160, clean, max_groups=max_groups)
    with pytest.raises(ZeroDivisionError):                                           # the caller's exception comes back
        pl.classify_chunks(8, lambda r, w: 1 / 0)
    from paper_2505_11204_amd import binding as rb
    with pytest.raises(rb.RandesError):
        pl.classify_chunks(0, clean)
    with pytest.raises(rb.RandesError):
        pl.plan_serving_layout([0, 1, 2], GIB, 0, 1)


def test_benchmark_places_a_write_only_buffer_across_a_group_boundary():
    import os
    import sys
    from types import SimpleNamespace
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    import bench
    chunk = 1 << 30
    labels = [1] * 96 + [0] * 96 + [2] * 82
    fake = SimpleNamespace(arena=SimpleNamespace(chunk_bytes=chunk), labels=labels)
    nbytes = 679_477_248
    off = bench.across_a_boundary(fake, nbytes)
    assert off % 256 == 0
    assert off < 96 * chunk < off + nbytes                        # the first boundary lies inside the buffer
    assert abs((96 * chunk - off) - nbytes // 2) < 256            # half of it on either side
    # a boundary whose neighbouring runs are too short for half the buffer is passed over
    labels = [1] * 4 + [0] * 1 + [2] * 8 + [1] * 8
    fake = SimpleNamespace(arena=SimpleNamespace(chunk_bytes=chunk), labels=labels)
    off = bench.across_a_boundary(fake, 6 * chunk)
    assert off == 13 * chunk - 3 * chunk
    assert bench.across_a_boundary(SimpleNamespace(arena=SimpleNamespace(chunk_bytes=chunk), labels=[0] * 20), nbytes) is None
    assert bench.across_a_boundary(None, nbytes) is None

"""A second, independent implementation of the placement's host logic (finding address groups
from copy rates, packing stacks into them), in plain Python, for the tests to hold the library's
against.  Written first; the library's C++ follows the same description."""


def _align_up(x, a=256):
    return (x + a - 1) // a * a


def _two_medians(values):
    """Centres of a two-cluster split of a list of numbers (medians, so that a few
    outliers do not become a cluster of their own), or None if one cluster is empty."""
    vals = sorted(values)
    lo, hi = vals[len(vals) // 10], vals[-1 - len(vals) // 10]
    for _ in range(8):
        mid = 0.5 * (lo + hi)
        a = [v for v in vals if v < mid]
        b = [v for v in vals if v >= mid]
        if not a or not b:
            return None
        lo, hi = a[len(a) // 2], b[len(b) // 2]
    return lo, hi


def _middle_of_longest_run(chunks):
    best, cur = [], []
    for c in chunks:
        cur = cur + [c] if cur and c == cur[-1] + 1 else [c]
        if len(cur) > len(best):
            best = cur
    return best[len(best) // 2]


def classify_chunks(n_chunks, rate, min_separation=0.02, max_groups=4):
    """Label every chunk 0..n_chunks-1 with a group number.

    ``rate(r, w)`` is the measured rate of a copy that reads chunk r and writes chunk w.
    Chunks that copy slowly from a reference chunk are in its group, the others are
    not; the rest is split again from a new reference until the rates no longer fall
    into two clusters at least ``min_separation`` (relative) apart.  Groups come in long
    runs, so a majority vote over five neighbouring chunks removes single misreads.
    """
    label = [-1] * n_chunks
    rest, g = list(range(n_chunks)), 0
    while len(rest) > 1 and g < max_groups - 1:
        ref = _middle_of_longest_run(rest)
        rates = {c: rate(ref, c) for c in rest if c != ref}
        centres = _two_medians(list(rates.values()))
        if centres is None or (centres[1] - centres[0]) / centres[1] < min_separation:
            break
        mid = 0.5 * (centres[0] + centres[1])
        other = {c: (1 if v >= mid else 0) for c, v in rates.items()}
        other[ref] = 0
        voted = {}
        for c in rest:
            near = [other[x] for x in range(c - 2, c + 3) if x in other]
            voted[c] = 1 if 2 * sum(near) > len(near) else 0
        if min(sum(voted.values()), len(rest) - sum(voted.values())) < 3:
            break                                # not a group, a handful of misreads
        for c in rest:
            if voted[c] == 0:
                label[c] = g
        rest = [c for c in rest if voted[c] == 1]
        g += 1
    for c in rest:
        label[c] = g
    return label


def runs_of(labels):
    """Maximal runs of equal labels as (group, first_chunk, end_chunk) triples."""
    out, start = [], 0
    for c in range(1, len(labels) + 1):
        if c == len(labels) or labels[c] != labels[start]:
            out.append((labels[start], start, c))
            start = c
    return out


def plan_serving_layout(labels, chunk_bytes, stack_bytes, n_models, n_more_outputs=0):
    """Byte offsets of the stacks of one serving set-up inside the classified allocation.

    Returns ``{"merged", "base", "out", "deltas": [...], "more_outputs": [...], "read_group", "write_groups"}`` or
    None when the groups found do not allow the layout: the output stack lies across a
    boundary between two groups, half on either side; merged deltas and base lie in a
    third group; the models' deltas, then ``n_more_outputs`` further output stacks (for several
    retrievals in one pass), fill what is left of every group but that third.
    Every stack is contiguous and stays one chunk away from the other group boundaries,
    whose position is only known to one chunk.
    """
    rs = runs_of(labels)
    if len(set(labels)) < 3:
        return None
    half = _align_up(stack_bytes // 2)
    n = len(labels)

    def free_ranges(skip_boundary, out_span):
        """(group, lo, hi) byte ranges usable for whole stacks."""
        fr = []
        for i, (g, a, b) in enumerate(rs):
            lo = a * chunk_bytes + (chunk_bytes if a > 0 else 0)
            hi = b * chunk_bytes - (chunk_bytes if b < n else 0)
            if i == skip_boundary:          # run on the left of the straddled boundary
                hi = min(b * chunk_bytes, out_span[0])
            if i == skip_boundary + 1:      # run on its right
                lo = max(a * chunk_bytes, out_span[1])
            if hi > lo:
                fr.append([g, _align_up(lo), hi])
        return fr

    def take(fr, ok_group):
        for r in fr:
            if ok_group(r[0]) and r[1] + stack_bytes <= r[2]:
                off = r[1]
                r[1] = _align_up(off + stack_bytes)
                return off
        return None

    for i in range(len(rs) - 1):
        (g1, a1, b1), (g2, a2, b2) = rs[i], rs[i + 1]
        edge = b1 * chunk_bytes
        # half a stack and a chunk of margin on both sides of the boundary
        if (b1 - a1) * chunk_bytes < half + chunk_bytes or (b2 - a2) * chunk_bytes < half + chunk_bytes:
            continue
        out_off = edge - half
        out_span = (out_off, out_off + _align_up(stack_bytes))
        for read_group in sorted(set(labels) - {g1, g2}):
            fr = free_ranges(i, out_span)
            merged = take(fr, lambda g: g == read_group)
            base = take(fr, lambda g: g == read_group)
            deltas = [take(fr, lambda g: g != read_group) for _ in range(n_models)]
            more = [take(fr, lambda g: g != read_group) for _ in range(n_more_outputs)]
            if merged is None or base is None or any(d is None for d in deltas + more):
                continue
            return {"merged": merged, "base": base, "out": out_off, "deltas": deltas, "more_outputs": more,
                    "read_group": read_group, "write_groups": (g1, g2)}
    return None

"""Where the stacks of a serving set-up lie in HBM.

Measured on MI355X: device memory falls into a few large groups of addresses (96 GiB
each on the machines seen, contiguous or in runs of 8 GiB and more inside one big
allocation).  A copy whose read and write streams lie in the same group runs 3-5 %
slower than one whose streams lie in different groups, and the streaming kernels of
the method follow suit:

* retrieve is fastest when both read streams (merged deltas, base) share one group
  and the output stack is spread half and half over two other groups;
* merge is fastest when the merged stack shares its group with none of the deltas.

Nothing in the runtime reports the groups, so :func:`classify_chunks` finds them by
timing plain copies between chunks of one large allocation, and
:func:`plan_serving_layout` packs the stacks accordingly.  Both are pure functions of
their inputs; :class:`Arena` supplies the device memory and the timing.  Placement is
a property of the caller's allocations: the kernels take any pointers.
"""
import torch

from . import binding as rb

GIB = 1 << 30


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


def _align_up(x, a=256):
    return (x + a - 1) // a * a


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


class Arena:
    """One large device allocation, cut into chunks, with the copy timing that
    :func:`classify_chunks` needs and views for the stacks placed in it."""

    def __init__(self, nbytes, chunk_bytes=GIB, device="cuda"):
        if chunk_bytes % 16384:
            raise ValueError("chunk_bytes must be a multiple of 16384")
        self.chunk_bytes = chunk_bytes
        self.n_chunks = nbytes // chunk_bytes
        if self.n_chunks < 1:
            raise ValueError("arena smaller than one chunk")
        self.buf = torch.empty(self.n_chunks * chunk_bytes, dtype=torch.uint8, device=device)
        for c in range(self.n_chunks):          # touch every page before timing anything
            self.chunk(c).fill_(1)
        torch.cuda.synchronize(self.buf.device)

    def chunk(self, c):
        return self.buf[c * self.chunk_bytes:(c + 1) * self.chunk_bytes]

    def copy_rate(self, r, w, reps=4):
        """Best rate (bytes per ms) of a plain streaming copy reading chunk r, writing chunk w."""
        best = None
        for i in range(reps + 1):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            rb.probe_stream([self.chunk(r)], self.chunk(w), True)
            b.record()
            b.synchronize()
            if i:                                # the first launch warms up
                ms = a.elapsed_time(b)
                best = ms if best is None else min(best, ms)
        return 2.0 * self.chunk_bytes / best

    def classify(self):
        return classify_chunks(self.n_chunks, self.copy_rate)

    def flat(self, byte_offset, n_elements, dtype):
        """A 1-D tensor of ``dtype`` over the arena's bytes from ``byte_offset`` (256-aligned)."""
        if byte_offset % 256:
            raise ValueError("byte_offset must be a multiple of 256")
        eb = torch.empty((), dtype=dtype).element_size()
        end = byte_offset + n_elements * eb
        if end > self.buf.numel():
            raise ValueError("range past the end of the arena")
        return self.buf[byte_offset:end].view(dtype)


def main(argv=None):
    """Print what the classification finds on this machine, and the map of copy rates behind it
    (read chunk x write chunk at regular positions of one large allocation)."""
    import argparse
    ap = argparse.ArgumentParser(description=main.__doc__)
    ap.add_argument("--reserve-gib", type=int, default=12, help="device memory left outside the allocation")
    ap.add_argument("--step-gib", type=int, default=8, help="distance between the positions of the map")
    args = ap.parse_args(argv)
    rb.lib()
    free_bytes, total_bytes = torch.cuda.mem_get_info()
    arena = Arena(free_bytes - args.reserve_gib * GIB)
    labels = arena.classify()
    print("device memory %.1f GiB, allocation of %d chunks of 1 GiB" % (total_bytes / GIB, arena.n_chunks))
    print("group of every chunk: " + "".join(str(g) for g in labels))
    print("runs (group, first GiB, end GiB): " + ", ".join("(%d, %d, %d)" % r for r in runs_of(labels)))
    pos = list(range(0, arena.n_chunks - 1, args.step_gib))
    print("copy rate in units of 100 GB/s; rows: position of the chunk read (GiB), columns: of the chunk written")
    print("      " + " ".join("%3d" % p for p in pos))
    for r in pos:
        print("%4d: " % r + " ".join(" . " if r == w else "%3d" % round(arena.copy_rate(r, w) * 1e-8) for w in pos))
    return 0


if __name__ == "__main__":
    raise SystemExit(main())

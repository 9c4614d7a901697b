"""Where the stacks of a serving set-up lie in HBM.

Measured on MI355X: device memory falls into a few large groups of addresses (96 GiB
each on the machines seen, contiguous or in runs of 8 GiB and more inside one big
allocation).  A copy whose read and write streams lie in the same group runs 3-5 %
slower than one whose streams lie in different groups, and the streaming kernels of
the method follow suit:

* retrieve is fastest when both read streams (merged deltas, base) share one group
  and the output stack is spread half and half over two other groups;
* merge is fastest when the merged stack shares its group with none of the deltas.

Nothing in the runtime reports the groups, so the library finds them by timing plain
copies between chunks of one large allocation and packs the stacks accordingly
(``include/randes_place.h``); this module is the binding of those calls
(:func:`classify_chunks`, :func:`plan_serving_layout`, both pure functions of their
inputs) plus :class:`Arena`, which supplies the device memory.  Placement is a
property of the caller's allocations: the kernels take any pointers.
"""
import ctypes

import torch

from . import binding as rb

GIB = 1 << 30


def classify_chunks(n_chunks, rate, min_separation=0.02, max_groups=4):
    """Label every chunk 0..n_chunks-1 with a group number (``randes_place_classify``).

    ``rate(r, w)`` is the measured rate of a copy that reads chunk r and writes chunk w.
    Chunks that copy slowly from a reference chunk are in its group, the others are
    not; the rest is split again from a new reference until the rates no longer fall
    into two clusters at least ``min_separation`` (relative) apart.  Groups come in long
    runs, so a majority vote over five neighbouring chunks removes single misreads.
    """
    labels = (ctypes.c_int32 * n_chunks)()
    failure = []

    def call(r, w, _ctx):
        try:
            return float(rate(r, w))
        except Exception as e:          # an exception must not unwind through the C caller
            failure.append(e)
            return 0.0
    rb._check(rb.lib().randes_place_classify(n_chunks, rb.COPY_RATE_FN(call), None, float(min_separation),
                                             int(max_groups), labels))
    if failure:
        raise failure[0]
    return list(labels)


def runs_of(labels):
    """Maximal runs of equal labels as (group, first_chunk, end_chunk) triples."""
    out, start = [], 0
    for c in range(1, len(labels) + 1):
        if c == len(labels) or labels[c] != labels[start]:
            out.append((labels[start], start, c))
            start = c
    return out


def plan_serving_layout(labels, chunk_bytes, stack_bytes, n_models, n_more_outputs=0):
    """Byte offsets of the stacks of one serving set-up inside the classified allocation
    (``randes_place_serving_layout``).

    Returns ``{"merged", "base", "out", "deltas": [...], "more_outputs": [...], "read_group", "write_groups"}`` or
    None when the groups found do not allow the layout: the output stack lies across a
    boundary between two groups, half on either side; merged deltas and base lie in a
    third group; the models' deltas, then ``n_more_outputs`` further output stacks (for several
    retrievals in one pass), fill what is left of every group but that third.
    Every stack is contiguous and stays one chunk away from the other group boundaries,
    whose position is only known to one chunk.
    """
    n = len(labels)
    lab = (ctypes.c_int32 * n)(*labels)
    offs = (ctypes.c_uint64 * (3 + n_models + n_more_outputs))()
    groups = (ctypes.c_int32 * 3)()
    rc = rb.lib().randes_place_serving_layout(lab, n, int(chunk_bytes), int(stack_bytes), int(n_models),
                                              int(n_more_outputs), offs, groups)
    if rc == -2:        # RANDES_ENOTSUP: no such layout in these groups
        return None
    rb._check(rc)
    offs = list(offs)
    return {"merged": offs[0], "base": offs[1], "out": offs[2], "deltas": offs[3:3 + n_models],
            "more_outputs": offs[3 + n_models:], "read_group": groups[0], "write_groups": (groups[1], groups[2])}


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
        """Group of every chunk, from copies timed inside the library (``randes_place_classify_device``)."""
        labels = (ctypes.c_int32 * self.n_chunks)()
        rb._check(rb.lib().randes_place_classify_device(self.buf.data_ptr(), self.chunk_bytes, self.n_chunks,
                                                        rb._stream(None), labels))
        return list(labels)

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

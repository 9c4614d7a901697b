"""Synthetic weight stacks and seeded input generators.

This module serves both the GPU library's tests/benchmark and the CPU oracle's
tests.  It holds none of the method's arithmetic: only layer shapes, shuffle
groups and random fills.  Shapes stand in for the checkpoints the paper
evaluates on (CLIP-ViT-B/32, CLIP-ViT-L/14, Flan-T5-base with and without
LoRA; Sec. "Experiments") plus a 7B decoder stack; the checkpoints themselves
are never needed.

A stack is a list of ``(rows, cols, group, flags)`` tuples, one per parameter
matrix, in model order (block-major).  ``group`` collects the layers of one
type across blocks (Sec. 4.3: only same-type layers are shuffled); ``-1`` marks
input/output layers that belong to no group.
"""
from collections import namedtuple

import torch

FLIP, SHUFFLE, SHIFT = 1, 2, 4
SRSF = FLIP | SHUFFLE

Layer = namedtuple("Layer", "rows cols group flags")


def _blocks(n_blocks, shapes, first_group=0, flags=SRSF):
    out = []
    for _ in range(n_blocks):
        for j, (m, n) in enumerate(shapes):
            out.append(Layer(m, n, first_group + j, flags))
    return out


def tiny(flags=SRSF):
    """4 fp32 matrices of 256 x 256 in one group."""
    return _blocks(4, [(256, 256)], flags=flags)


def vit_b32(flags=SRSF):
    """12 blocks, d = 768: qkv, proj, fc1, fc2 (84.9 M elements)."""
    return _blocks(12, [(768, 2304), (768, 768), (768, 3072), (3072, 768)], flags=flags)


def vit_l14(flags=SRSF):
    """24 blocks, d = 1024, MLP 4096 (302 M elements)."""
    return _blocks(24, [(1024, 3072), (1024, 1024), (1024, 4096), (4096, 1024)], flags=flags)


def t5_base(flags=SRSF, embeddings=True):
    """12 encoder + 12 decoder blocks, d = 768, d_ff = 2048, gated FFN; two
    32128 x 768 input/output matrices as singletons (247.5 M elements)."""
    attn = [(768, 768)] * 4
    ffn = [(768, 2048), (768, 2048), (2048, 768)]
    enc = _blocks(12, attn + ffn, first_group=0, flags=flags)
    dec = _blocks(12, attn + attn + ffn, first_group=7, flags=flags)
    io = [Layer(32128, 768, -1, flags & FLIP)] * 2 if embeddings else []
    return io[:1] + enc + dec + io[1:]


def llama_7b(flags=SRSF, n_blocks=32, embeddings=True):
    """32 blocks, d = 4096, ffn 11008 (q, k, v, o, gate, up, down); two
    32000 x 4096 input/output matrices as singletons (6.738 G elements)."""
    shapes = [(4096, 4096)] * 4 + [(4096, 11008)] * 2 + [(11008, 4096)]
    io = [Layer(32000, 4096, -1, flags & FLIP)] * 2 if embeddings else []
    return io[:1] + _blocks(n_blocks, shapes, flags=flags) + io[1:]


STACKS = {"tiny": tiny, "vit_b32": vit_b32, "vit_l14": vit_l14, "t5_base": t5_base, "llama_7b": llama_7b}


def t5_lora_targets(stack):
    """Indices of the layers that carry rank-16 adapters in the LoRA variant:
    the q and v projections (768 x 768) of all 36 attention modules.  The paper
    does not say which modules carry adapters; this is a stated choice."""
    picks = []
    for idx, layer in enumerate(stack):
        if layer.group in (0, 2, 7, 9, 11, 13):  # enc q, v; dec self q, v; dec cross q, v
            picks.append(idx)
    return picks


def n_elements(stack):
    return sum(l.rows * l.cols for l in stack)


def torch_dtype(name):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def _aligned(count, elem_bytes, align=256):
    per = align // elem_bytes
    return (count + per - 1) // per * per


def stack_elements(stack, dtype):
    """Elements of the flat buffer of :func:`alloc_stack` (layers padded to 256 bytes)."""
    eb = torch.empty((), dtype=dtype).element_size()
    return sum(_aligned(l.rows * l.cols, eb) for l in stack)


def alloc_stack(stack, dtype, device, into=None):
    """One flat buffer holding every layer (each 256-byte aligned), plus the
    list of per-layer 2-D views into it.  ``into`` is a flat tensor of
    :func:`stack_elements` elements to use instead of a new allocation."""
    eb = torch.empty((), dtype=dtype).element_size()
    offs, total = [], 0
    for l in stack:
        offs.append(total)
        total += _aligned(l.rows * l.cols, eb)
    if into is not None:
        if into.dtype != dtype or into.dim() != 1 or into.numel() != total:
            raise ValueError("`into` must be a flat %s tensor of %d elements" % (dtype, total))
        flat = into
    else:
        flat = torch.empty(total, dtype=dtype, device=device)
    views = [flat[o:o + l.rows * l.cols].view(l.rows, l.cols) for o, l in zip(offs, stack)]
    return flat, views


def fill_normal(flat, std, generator):
    """In-place N(0, std^2) fill, drawn in fp32 and rounded by torch to the
    buffer's dtype.  Chunked so the fp32 temporary stays small."""
    step = 1 << 28
    for s in range(0, flat.numel(), step):
        part = flat[s:s + step]
        tmp = torch.empty(part.numel(), dtype=torch.float32, device=flat.device)
        tmp.normal_(0.0, std, generator=generator)
        part.copy_(tmp)
    return flat


def task_scales(n_tasks, data_seed, low=0.5, high=2.0):
    """Per-task delta scale c_i ~ U[low, high], drawn once per task."""
    g = torch.Generator(device="cpu")
    g.manual_seed(data_seed + 7919)
    return (low + (high - low) * torch.rand(n_tasks, generator=g, dtype=torch.float64)).tolist()


def make_inputs(stack, n_tasks, dtype="f32", device="cpu", data_seed=1234,
                base_std=0.02, delta_std=1e-3, scales=None, with_base=True, flats=None,
                place=None):
    """Seeded synthetic base weights and deltas.

    Returns ``(base_views, delta_views)`` where ``delta_views[i][l]`` is model
    i's delta for layer l in its original position.  base ~ N(0, base_std^2),
    delta_i ~ N(0, (delta_std * scales[i])^2), i.i.d.; values are rounded to
    ``dtype`` by torch.  The same (device, seed) always gives the same bits.
    If ``flats`` is a list, the flat backing buffers (base first, then one per
    model) are appended to it.  ``place("base")`` / ``place(i)``, if given,
    returns the flat tensor a stack is to live in (see :func:`alloc_stack`);
    the values drawn do not depend on it.
    """
    td = torch_dtype(dtype)
    g = torch.Generator(device=device)
    g.manual_seed(data_seed)
    base = None
    if with_base:
        bflat, base = alloc_stack(stack, td, device, into=place("base") if place else None)
        fill_normal(bflat, base_std, g)
        if flats is not None:
            flats.append(bflat)
    deltas = []
    for i in range(n_tasks):
        dflat, dviews = alloc_stack(stack, td, device, into=place(i) if place else None)
        fill_normal(dflat, delta_std * (scales[i] if scales else 1.0), g)
        deltas.append(dviews)
        if flats is not None:
            flats.append(dflat)
    return base, deltas


def make_lora_factors(stack, targets, n_tasks, rank=16, dtype="bf16", device="cpu",
                      data_seed=4321, std=0.01):
    """A (rank x cols) and B (rows x rank) ~ N(0, std^2) for each target layer
    of each task: ``factors[i][t] = (B, A)``."""
    td = torch_dtype(dtype)
    g = torch.Generator(device=device)
    g.manual_seed(data_seed)
    out = []
    for _ in range(n_tasks):
        per = []
        for t in targets:
            l = stack[t]
            B = torch.empty(l.rows, rank, dtype=torch.float32, device=device).normal_(0.0, std, generator=g).to(td)
            A = torch.empty(rank, l.cols, dtype=torch.float32, device=device).normal_(0.0, std, generator=g).to(td)
            per.append((B, A))
        out.append(per)
    return out


def to_numpy(t):
    """CPU tensor -> numpy array the oracle accepts (bf16 as uint16 bits)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view("uint16")
    return t.numpy()


def from_numpy(a, dtype):
    """Inverse of :func:`to_numpy`."""
    if dtype == "bf16":
        return torch.from_numpy(a.view("int16").copy()).view(torch.bfloat16)
    return torch.from_numpy(a.copy())


def shadow_rows(rows, n_pick, seed):
    """Row indices to sample from a layer for full-size parity: the first and
    last rows, rows around multiples of 128 (tile edges), and a few seeded random
    ones; sorted and unique.  Depends on ``rows`` and ``seed`` only, so layers
    that can trade places in a shuffle sample the same rows."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed + rows)
    fixed = [0, 1, 2, 3, 127, 128, 129, rows // 2, rows - 129, rows - 128, rows - 2, rows - 1]
    rnd = torch.randint(0, rows, (max(n_pick - len(fixed), 0),), generator=g).tolist()
    picks = sorted({r for r in fixed + rnd if 0 <= r < rows})
    return picks


def tile_band_rows(rows, band=128, seed=99):
    """Row indices for denser full-size parity: every row of the first ``band`` rows, of a band
    in the middle (starting at a multiple of ``band``) and of the last ``band`` rows, plus the
    scattered rows of :func:`shadow_rows`.  The streaming kernels cut a layer into tiles of at
    most 64 rows that span a column range, so each band holds at least one whole row of tiles
    from its first to its last column, with its neighbours' edges.  Depends on ``rows`` and
    ``seed`` only, like :func:`shadow_rows`."""
    mid = (rows // 2) // band * band
    picks = set(shadow_rows(rows, 16, seed))
    for start in (0, mid, rows - band):
        picks.update(r for r in range(start, start + band) if 0 <= r < rows)
    return sorted(picks)

"""CPU-only pins of the oracle's generator: Philox core, sign masks, layer
permutations, bf16 conversion.  Nothing here touches the GPU library."""
import os

import numpy as np
import pytest
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _kat():
    rows = []
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w = [int(x, 16) for x in line.split()]
            rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_philox_known_answers():
    rows = _kat()
    assert len(rows) == 3
    for ctr, key, want in rows:
        assert oracle.philox4x32_10(ctr, key) == want


def test_philox_is_a_bijection_of_the_counter_on_a_sample():
    # a counter-based generator is a keyed bijection of the counter: distinct
    # counters under one key never collide
    outs = {tuple(oracle.philox4x32_10([c, 5, 0, 0], [1, 2])) for c in range(4096)}
    assert len(outs) == 4096


def test_sign_bits_of_seed0_layer0_are_the_bits_of_the_zero_vector_answer():
    # seed 0, layer 0, columns 0..127 use counter (0,0,0,0) and key (0,0): the
    # published all-zero known answer.  Column c reads bit (c mod 32) of word
    # (c / 32), least significant bit first.
    words = _kat()[0][2]
    mask = oracle.sign_mask(0, 0, 128)
    for c in range(128):
        assert mask[c] == (words[c // 32] >> (c % 32)) & 1
    # spot values written out by hand from 0x6627e8d5 = ...1101 0101 and 0x9b00dbd8 = 1001 1011 ...
    assert list(mask[0:8]) == [1, 0, 1, 0, 1, 0, 1, 1]
    assert mask[127] == 1 and mask[126] == 0 and mask[125] == 0 and mask[124] == 1


def test_sign_bits_key_is_the_64_bit_seed_split_low_high():
    # the all-ones known answer: counter words (col/128, layer) = (2^32-1, 2^32-1)
    # cannot be reached with counter words 2, 3 = 0, so pin the key split with the
    # third vector's key instead, through the permutation keys' path below; here
    # check that low and high seed halves are not interchangeable.
    a = oracle.sign_mask(0x00000001_00000000, 3, 256)
    b = oracle.sign_mask(0x00000000_00000001, 3, 256)
    assert (a != b).any()
    want = oracle.philox4x32_10([1, 3, 0, 0], [0, 1])
    for c in range(128, 256):
        assert a[c] == (want[(c // 32) % 4] >> (c % 32)) & 1


def test_sign_mask_is_a_function_of_seed_layer_column_only():
    long = oracle.sign_mask(42, 7, 5000)
    for cols in (1, 3, 77, 128, 130, 4096):
        assert (oracle.sign_mask(42, 7, cols) == long[:cols]).all()
    for c in (0, 1, 127, 128, 129, 4999):
        assert oracle.sign_bit(42, 7, c) == long[c]


def test_sign_mask_is_balanced_and_masks_are_pairwise_independent():
    # Sec. 4.4: diagonal entries are +1 or -1 with equal probability.
    n = 1 << 20
    a = oracle.sign_mask(42, 0, n)
    frac = a.mean()
    assert abs(frac - 0.5) < 4.0 / (2.0 * np.sqrt(n))
    for seed, layer in ((43, 0), (42, 1), (0xFFFFFFFFFFFFFFFF, 0)):
        b = oracle.sign_mask(seed, layer, n)
        agree = (a == b).mean()
        assert abs(agree - 0.5) < 4.0 / (2.0 * np.sqrt(n))
    # lag-1 serial correlation of the +-1 sequence is ~ N(0, 1/n)
    s = 1.0 - 2.0 * a.astype(np.float64)
    assert abs((s[1:] * s[:-1]).mean()) < 4.0 / np.sqrt(n)


def test_flip_is_an_involution_and_preserves_norm():
    # D^2 = I and ||Delta D||_F = ||Delta||_F (D orthogonal, Sec. 4).
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 300)).astype(np.float32)
    s = oracle.sign_mask(9, 2, 300)
    d = np.where(s == 1, np.float32(-1), np.float32(1))
    y = x * d
    assert (y * d == x).all()
    assert np.sum(y.astype(np.float64) ** 2) == np.sum(x.astype(np.float64) ** 2)


# ------------------------------------------------------------------ permutations
@pytest.mark.parametrize("G", [1, 2, 3, 4, 12, 24, 32, 100])
def test_layer_perm_is_a_bijection(G):
    for seed in (0, 1, 42, 2**63 + 5):
        for group in (0, 1, 6):
            p = oracle.layer_perm(seed, group, G)
            assert sorted(p.tolist()) == list(range(G))
    assert oracle.layer_perm(5, 0, 1).tolist() == [0]


def test_layer_perm_is_the_stable_argsort_of_its_keys():
    p, keys = oracle.layer_perm(42, 3, 12, return_keys=True)
    assert p.tolist() == np.argsort(keys, kind="stable").tolist()
    # keys come from counter (k, group, 1, 0) under key (seed low, seed high)
    for k in (0, 5, 11):
        o = oracle.philox4x32_10([k, 3, 1, 0], [42, 0])
        assert int(keys[k]) == (o[0] << 32) | o[1]
    # and by hand for a tiny case: print, sort by eye
    p4, k4 = oracle.layer_perm(0, 0, 4, return_keys=True)
    order = sorted(range(4), key=lambda k: int(k4[k]))
    assert p4.tolist() == order


def test_layer_perm_key_uses_both_seed_halves_third_known_answer():
    # counter (k=0x243f6a88, group=0x85a308d3, 1, 0) is not reachable with a small
    # group, so pin the key split with a direct evaluation of the third vector's key
    seed = (0x299F31D0 << 32) | 0xA4093822
    _, keys = oracle.layer_perm(seed, 2, 3, return_keys=True)
    o = oracle.philox4x32_10([1, 2, 1, 0], [0xA4093822, 0x299F31D0])
    assert int(keys[1]) == (o[0] << 32) | o[1]


def test_layer_perm_is_uniform_over_s4():
    # chi-square over the 24 outcomes of G = 4 across 24 000 seeds
    counts = {}
    n = 24000
    for seed in range(n):
        t = tuple(oracle.layer_perm(seed, 0, 4).tolist())
        counts[t] = counts.get(t, 0) + 1
    assert len(counts) == 24
    exp = n / 24.0
    chi2 = sum((c - exp) ** 2 / exp for c in counts.values())
    assert chi2 < 60.0  # 23 dof: P(chi2 > 60) ~ 4e-5


def test_perm_and_sign_streams_are_disjoint_and_group_dependent():
    a = oracle.layer_perm(42, 0, 32).tolist()
    b = oracle.layer_perm(42, 1, 32).tolist()
    c = oracle.layer_perm(43, 0, 32).tolist()
    assert a != b and a != c and b != c


# ------------------------------------------------------------------ bf16
def test_bf16_round_to_nearest_even_matches_torch():
    g = torch.Generator().manual_seed(0)
    x = torch.randn(20000, generator=g) * torch.logspace(-30, 30, 20000)
    special = torch.tensor([0.0, -0.0, 1.0, -1.0, float("inf"), float("-inf"),
                            1.00390625, 1.01171875,   # exact ties: 1 + 2^-8 (to even: down), 1 + 3*2^-8 (up)
                            3.3895314e38, 3.4028235e38,  # rounds to inf
                            1e-45, 9.18e-41, -9.18e-41])  # denormals
    x = torch.cat([x, special])
    want = x.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = oracle.f32_to_bf16(x.numpy())
    assert (got == want).all()
    back = oracle.bf16_to_f32(got)
    assert (back.view(np.uint32) == (got.astype(np.uint32) << 16)).all()
    assert (back == x.to(torch.bfloat16).float().numpy()).all()


def test_bf16_ties_and_nan_by_hand():
    tie_down = np.array([0x3F808000], dtype=np.uint32).view(np.float32)  # mantissa lsb 0 -> stays
    tie_up = np.array([0x3F818000], dtype=np.uint32).view(np.float32)    # mantissa lsb 1 -> up
    assert oracle.f32_to_bf16(tie_down)[0] == 0x3F80
    assert oracle.f32_to_bf16(tie_up)[0] == 0x3F82
    above = np.array([0x3F808001], dtype=np.uint32).view(np.float32)
    assert oracle.f32_to_bf16(above)[0] == 0x3F81
    nan = np.array([0x7FA00001, 0xFF800001], dtype=np.uint32).view(np.float32)
    out = oracle.f32_to_bf16(nan)
    assert (out & 0x7FC0 == 0x7FC0).all() and out[1] & 0x8000
    big = np.array([0x7F7FFFFF], dtype=np.uint32).view(np.float32)
    assert oracle.f32_to_bf16(big)[0] == 0x7F80

"""CPU-only pins of the oracle's merge / retrieve / hot-swap / LoRA /
diagnostics against closed forms, invariants, dense brute force and library
routines.  Nothing here touches the GPU library."""
import numpy as np
import pytest

import oracle
from oracle import BF16, F32, FLIP, SHIFT, SHUFFLE

SRSF = FLIP | SHUFFLE


def _ints(rng, shape, lim=64):
    return rng.integers(-lim, lim + 1, size=shape).astype(np.float32)


def _small_model():
    # two groups (3 layers of 2x5, 2 layers of 3x4) interleaved, one singleton
    return [(2, 5, 0, SRSF), (3, 4, 1, SRSF), (2, 5, 0, SRSF), (2, 2, -1, FLIP),
            (3, 4, 1, SRSF), (2, 5, 0, SRSF)]


def _dense_O(layers, seed):
    """Explicit d x d matrix of the transform O_i = (column sign flip keyed by
    slot) o (block permutation), acting on the layer-major, row-major
    flattening of a delta (Sec. 4: Theta_* = Theta_0 + lambda sum_i O_i Delta_i)."""
    sizes = [m * n for (m, n, _, _) in layers]
    offs = np.concatenate([[0], np.cumsum(sizes)])
    d = int(offs[-1])
    # block permutation P: slot l <- layer src(l)
    src = list(range(len(layers)))
    groups = {}
    for l, (_, _, g, fl) in enumerate(layers):
        if g >= 0 and (fl & SHUFFLE):
            groups.setdefault(g, []).append(l)
    for g, members in groups.items():
        sigma = oracle.layer_perm(seed, g, len(members))
        for k, l in enumerate(members):
            src[l] = members[int(sigma[k])]
    P = np.zeros((d, d))
    for l in range(len(layers)):
        for e in range(sizes[l]):
            P[offs[l] + e, offs[src[l]] + e] = 1.0
    # sign flip S: entry (l, r, c) scaled by D^l_cc
    diag = np.ones(d)
    for l, (m, n, _, fl) in enumerate(layers):
        if fl & FLIP:
            s = 1.0 - 2.0 * oracle.sign_mask(seed, l, n).astype(np.float64)
            diag[offs[l]:offs[l + 1]] = np.tile(s, m)
    return np.diag(diag) @ P, offs


def _flatten(arrs):
    return np.concatenate([a.reshape(-1).astype(np.float64) for a in arrs])


def test_merge_and_retrieve_equal_dense_orthogonal_brute_force():
    layers = _small_model()
    rng = np.random.default_rng(1)
    seeds = [42, 43, 44]
    deltas = [[_ints(rng, (m, n)) for (m, n, _, _) in layers] for _ in seeds]
    base = [_ints(rng, (m, n)) for (m, n, _, _) in layers]
    Os = []
    for s in seeds:
        O, offs = _dense_O(layers, s)
        assert np.array_equal(O.T @ O, np.eye(O.shape[0]))  # orthogonal
        Os.append(O)
    want_star = sum(O @ _flatten(d) for O, d in zip(Os, deltas))
    merged = oracle.merge(layers, deltas, seeds)
    assert np.array_equal(_flatten(merged), want_star)
    lam = 0.5
    for i, s in enumerate(seeds):
        want = _flatten(base) + lam * (Os[i].T @ want_star)
        got = oracle.retrieve(layers, merged, base, s, lam)
        assert np.array_equal(_flatten(got), want)
        # Sec. 4, expansion of hat Theta_i: (1-lam) Theta_0 + lam Theta_i + lam sum_{j != i} O_i^-1 O_j Delta_j
        theta_i = _flatten(base) + _flatten(deltas[i])
        interf = sum(Os[i].T @ (Os[j] @ _flatten(deltas[j])) for j in range(len(seeds)) if j != i)
        assert np.array_equal(_flatten(got), (1 - lam) * _flatten(base) + lam * theta_i + lam * interf)


def test_single_model_retrieval_is_base_plus_delta_exactly():
    layers = [(4, 130, 0, SRSF)] * 5 + [(3, 7, -1, FLIP)]
    rng = np.random.default_rng(2)
    delta = [rng.standard_normal((m, n)).astype(np.float32) * 1e-3 for (m, n, _, _) in layers]
    base = [rng.standard_normal((m, n)).astype(np.float32) * 0.02 for (m, n, _, _) in layers]
    merged = oracle.merge(layers, [delta], [7])
    out = oracle.retrieve(layers, merged, base, 7, 1.0)
    for l in range(len(layers)):
        assert np.array_equal(out[l], base[l] + delta[l])  # fl(b + d): one rounding
    # lambda = 0 gives the base bit for bit
    out0 = oracle.retrieve(layers, merged, base, 7, 0.0)
    for l in range(len(layers)):
        assert np.array_equal(out0[l].view(np.uint32), base[l].view(np.uint32))
    # general lambda: correctly rounded value of b + lam * d, checked in float64
    lam = np.float32(0.3)
    outl = oracle.retrieve(layers, merged, base, 7, float(lam))
    for l in range(len(layers)):
        exact = base[l].astype(np.float64) + np.float64(lam) * delta[l].astype(np.float64)
        assert np.array_equal(outl[l], exact.astype(np.float32))


def test_no_flags_is_task_arithmetic_in_task_order():
    # identity context matrices reduce RanDeS to task arithmetic (Sec. 3 eq. for Theta_*^TA)
    layers = [(6, 33, 0, 0)] * 3
    rng = np.random.default_rng(3)
    K = 5
    deltas = [[rng.standard_normal((6, 33)).astype(np.float32) for _ in layers] for _ in range(K)]
    merged = oracle.merge(layers, deltas, list(range(K)))
    for l in range(3):
        acc = np.zeros((6, 33), dtype=np.float32)
        for i in range(K):
            acc = acc + deltas[i][l]
        assert np.array_equal(merged[l], acc)
    # order matters in binary32: the reversed order differs somewhere, so the test above does pin the order
    acc_rev = np.zeros((6, 33), dtype=np.float32)
    for i in reversed(range(K)):
        acc_rev = acc_rev + deltas[i][0]
    assert not np.array_equal(acc_rev, merged[0])


def test_shuffle_only_moves_whole_layers_within_the_group():
    layers = [(2, 3, 0, SHUFFLE)] * 6 + [(2, 3, 1, SHUFFLE)] * 2
    deltas = [[np.full((2, 3), 10.0 * l + 1, dtype=np.float32) for l in range(8)]]
    merged = oracle.merge(layers, deltas, [11])
    sigma0 = oracle.layer_perm(11, 0, 6)
    sigma1 = oracle.layer_perm(11, 1, 2)
    for k in range(6):
        assert (merged[k] == 10.0 * sigma0[k] + 1).all()      # slot k <- layer sigma(k)
    for k in range(2):
        assert (merged[6 + k] == 10.0 * (6 + sigma1[k]) + 1).all()
    src = oracle.source_table(layers, [11])
    assert src[0].tolist() == [int(s) for s in sigma0] + [6 + int(s) for s in sigma1]
    # retrieve undoes it: slot k goes back to layer sigma(k)
    zero = [np.zeros((2, 3), dtype=np.float32) for _ in range(8)]
    out = oracle.retrieve(layers, merged, zero, 11, 1.0)
    for l in range(8):
        assert (out[l] == deltas[0][l]).all()


def test_group_shape_mismatch_is_rejected():
    with pytest.raises(ValueError):
        oracle.source_table([(2, 3, 0, SRSF), (3, 2, 0, SRSF)], [1])


def test_unflagged_members_stay_in_place_and_shift_moves_each_model_by_its_own_distance():
    # skip-rate pattern: only every 2nd layer of the group is a target
    layers = [(1, 4, 0, SRSF if k % 2 == 0 else 0) for k in range(8)]
    src = oracle.source_table(layers, [5])[0]
    assert [src[k] for k in range(1, 8, 2)] == [1, 3, 5, 7]
    sigma = oracle.layer_perm(5, 0, 4)
    assert [src[k] for k in range(0, 8, 2)] == [2 * int(s) for s in sigma]
    # layer shifting (App. "Dynamics between Layer Shuffling and Random Sign Flips"): model `seed` moves
    # (seed mod G) + 1 slots deeper, the deepest layers wrapping to the front.  Written out by hand, G = 5:
    layers = [(1, 4, 0, SHIFT)] * 5
    src = oracle.source_table(layers, [0, 1, 5, 99, 2 ** 64 - 1])
    assert src[0].tolist() == [4, 0, 1, 2, 3]     # seed 0: one slot deeper, the last layer wraps to slot 0
    assert src[1].tolist() == [3, 4, 0, 1, 2]     # seed 1: two slots
    assert src[2].tolist() == [4, 0, 1, 2, 3]     # seed 5 = 0 mod 5: one slot again
    assert src[3].tolist() == [0, 1, 2, 3, 4]     # seed 99 = 4 mod 5: five slots = none
    assert src[4].tolist() == [4, 0, 1, 2, 3]     # 2^64 - 1 = 0 mod 5
    # a shift common to all models would only relabel the slots; per-model distances move two models
    # against each other: retrieving model 0 leaves model 1's layers one slot out of place
    rng = np.random.default_rng(5)
    d0 = [_ints(rng, (1, 4)) for _ in layers]
    d1 = [_ints(rng, (1, 4)) for _ in layers]
    zero = [np.zeros((1, 4), np.float32) for _ in layers]
    merged = oracle.merge(layers, [d0, d1], [0, 1])
    got = oracle.retrieve(layers, merged, zero, 0, 1.0)
    for t in range(5):
        assert np.array_equal(got[t], d0[t] + d1[(t - 1) % 5])


def test_integer_inputs_sum_exactly_in_any_order():
    layers = [(8, 260, 0, SRSF)] * 4
    rng = np.random.default_rng(4)
    K = 16
    seeds = list(range(100, 100 + K))
    deltas = [[_ints(rng, (8, 260), 1024) for _ in layers] for _ in range(K)]
    merged = oracle.merge(layers, deltas, seeds)
    src = oracle.source_table(layers, seeds)
    for l in range(4):
        acc = np.zeros((8, 260), dtype=np.int64)
        for i in reversed(range(K)):
            s = 1 - 2 * oracle.sign_mask(seeds[i], l, 260).astype(np.int64)
            acc += deltas[i][src[i, l]].astype(np.int64) * s[None, :]
        assert np.array_equal(merged[l].astype(np.int64), acc)


def test_second_model_zero_returns_first_model():
    layers = [(5, 40, 0, SRSF)] * 3
    rng = np.random.default_rng(5)
    d1 = [rng.standard_normal((5, 40)).astype(np.float32) for _ in layers]
    d2 = [np.zeros((5, 40), dtype=np.float32) for _ in layers]
    base = [rng.standard_normal((5, 40)).astype(np.float32) for _ in layers]
    merged = oracle.merge(layers, [d1, d2], [1, 2])
    lam = 0.75
    out = oracle.retrieve(layers, merged, base, 1, lam)
    for l in range(3):
        exact = base[l].astype(np.float64) + 0.75 * d1[l].astype(np.float64)
        assert np.array_equal(out[l], exact.astype(np.float32))


def test_negative_zero_column_sums_to_positive_zero():
    layers = [(1, 4, -1, 0)]
    nz = np.full((1, 4), -0.0, dtype=np.float32)
    merged = oracle.merge(layers, [[nz], [nz.copy()]], [0, 1])
    assert (merged[0].view(np.uint32) == 0).all()  # accumulation starts at +0


def test_cross_task_residual_shrinks_like_inverse_sqrt_n():
    # Worst-case correlated deltas (all identical, rows constant): after retrieval of task 0 the
    # interference sum_{j != 0} Delta D_j D_0 has cosine ~ 1/sqrt(n) with Delta and relative norm
    # 1/sqrt(K-1) of the aligned sum (Sec. 3 norm identity with cos -> 0; Sec. 4 decorrelation).
    K = 9
    seeds = list(range(42, 42 + K))
    ns = [2 ** p for p in range(8, 15)]
    rms_cos, rel_norm = [], []
    for n in ns:
        cos = []
        for layer in range(24):
            masks = [1.0 - 2.0 * oracle.sign_mask(s, layer, n).astype(np.float64) for s in seeds]
            for j in range(1, K):
                cos.append(np.mean(masks[j] * masks[0]))  # cos(Delta D_j D_0, Delta) for Delta = ones
        rms_cos.append(np.sqrt(np.mean(np.square(cos))))
        masks = [1.0 - 2.0 * oracle.sign_mask(s, 0, n).astype(np.float64) for s in seeds]
        interf = sum(masks[j] * masks[0] for j in range(1, K))
        rel_norm.append(np.linalg.norm(interf) / ((K - 1) * np.sqrt(n)))
    slope = np.polyfit(np.log(ns), np.log(rms_cos), 1)[0]
    assert abs(slope + 0.5) < 0.1
    for n, c in zip(ns, rms_cos):
        assert 0.7 / np.sqrt(n) < c < 1.4 / np.sqrt(n)
    for r in rel_norm[2:]:
        assert abs(r - 1.0 / np.sqrt(K - 1)) < 0.08
    # the same through the real path: merge K copies of one delta, retrieve task 0
    n = 4096
    layers = [(2, n, -1, FLIP)]
    delta = [np.ones((2, n), dtype=np.float32)]
    merged = oracle.merge(layers, [delta] * K, seeds)
    out = oracle.retrieve(layers, merged, [np.zeros((2, n), dtype=np.float32)], seeds[0], 1.0)
    resid = out[0].astype(np.float64) - 1.0
    ab, aa, bb = oracle.dot3(resid.astype(np.float32), delta[0])
    assert abs(ab / np.sqrt(aa * bb)) < 4.0 / np.sqrt(n)
    assert abs(np.sqrt(aa / bb) - np.sqrt(K - 1)) < 0.08 * np.sqrt(K - 1) * 2


def test_interference_norm_identity():
    # || lam sum_{j != i} Delta_j ||^2 = lam^2 ( sum ||Delta_j||^2 + 2 sum_{l<j} ||Delta_l|| ||Delta_j|| cos )
    rng = np.random.default_rng(6)
    vs = [rng.standard_normal(500).astype(np.float32) for _ in range(4)]
    lam = 0.3
    total = sum(v.astype(np.float64) for v in vs)
    lhs = (lam ** 2) * float(total @ total)
    rhs = 0.0
    for a in range(4):
        _, aa, _ = oracle.dot3(vs[a], vs[a])
        rhs += aa
        for b in range(a + 1, 4):
            ab, aa2, bb = oracle.dot3(vs[a], vs[b])
            cos = ab / np.sqrt(aa2 * bb)
            rhs += 2.0 * np.sqrt(aa2) * np.sqrt(bb) * cos
    assert abs(lhs - lam ** 2 * rhs) < 1e-9 * lhs
    ab, aa, bb = oracle.dot3(vs[0], vs[1])
    assert abs(ab - float(vs[0].astype(np.float64) @ vs[1].astype(np.float64))) < 1e-9


def test_bf16_path_widens_exactly_and_rounds_once():
    layers = [(3, 136, 0, SRSF)] * 2
    rng = np.random.default_rng(7)
    K = 3
    seeds = [1, 2, 3]
    d32 = [[rng.standard_normal((3, 136)).astype(np.float32) * 1e-3 for _ in layers] for _ in range(K)]
    d16 = [[oracle.f32_to_bf16(x) for x in per] for per in d32]
    dback = [[oracle.bf16_to_f32(x) for x in per] for per in d16]
    m32 = oracle.merge(layers, dback, seeds, F32, F32)
    m16 = oracle.merge(layers, d16, seeds, BF16, BF16)
    mmix = oracle.merge(layers, d16, seeds, BF16, F32)
    for l in range(2):
        assert np.array_equal(mmix[l], m32[l])
        assert np.array_equal(m16[l], oracle.f32_to_bf16(m32[l]))
    base16 = [oracle.f32_to_bf16(rng.standard_normal((3, 136)).astype(np.float32) * 0.02) for _ in layers]
    out16 = oracle.retrieve(layers, m16, base16, 2, 0.8, BF16, BF16, BF16)
    out32 = oracle.retrieve(layers, [oracle.bf16_to_f32(x) for x in m16],
                            [oracle.bf16_to_f32(x) for x in base16], 2, 0.8, F32, F32, F32)
    for l in range(2):
        assert np.array_equal(out16[l], oracle.f32_to_bf16(out32[l]))


def test_hot_add_equals_fresh_merge_and_remove_undoes_it_on_integers():
    layers = [(4, 70, 0, SRSF)] * 3 + [(2, 9, -1, FLIP)]
    rng = np.random.default_rng(8)
    K = 4
    seeds = [10, 11, 12, 13]
    deltas = [[rng.standard_normal((m, n)).astype(np.float32) for (m, n, _, _) in layers] for _ in range(K)]
    fresh = oracle.merge(layers, deltas, seeds)
    part = oracle.merge(layers, deltas[:3], seeds[:3])
    oracle.update(layers, part, deltas[3], seeds[3], remove=False)
    for l in range(len(layers)):
        assert np.array_equal(part[l], fresh[l])  # appending last keeps the summation order
    ideltas = [[_ints(rng, (m, n)) for (m, n, _, _) in layers] for _ in range(K)]
    full = oracle.merge(layers, ideltas, seeds)
    oracle.update(layers, full, ideltas[1], seeds[1], remove=True)
    want = oracle.merge(layers, [ideltas[0], ideltas[2], ideltas[3]], [10, 12, 13])
    for l in range(len(layers)):
        assert np.array_equal(full[l], want[l])


def test_lora_matches_float64_matmul_and_special_cases():
    rng = np.random.default_rng(9)
    B = (rng.standard_normal((40, 16)) * 0.01).astype(np.float32)
    A = (rng.standard_normal((16, 50)) * 0.01).astype(np.float32)
    val, mag = oracle.lora(B, A, 2.0)
    want = 2.0 * (B.astype(np.float64) @ A.astype(np.float64))
    assert np.allclose(val, want, rtol=0, atol=1e-18 + 1e-15 * np.abs(want).max())
    assert np.allclose(mag, 2.0 * (np.abs(B).astype(np.float64) @ np.abs(A).astype(np.float64)))
    # rank 1 is an outer product: exact in float64 for float32 inputs
    val1, _ = oracle.lora(B[:, :1].copy(), A[:1].copy(), 1.0)
    assert np.array_equal(val1, np.outer(B[:, 0].astype(np.float64), A[0].astype(np.float64)))
    # B = [I; 0] copies A's rows
    Bi = np.zeros((20, 16), dtype=np.float32)
    Bi[:16] = np.eye(16, dtype=np.float32)
    vali, _ = oracle.lora(Bi, A, 1.0)
    assert np.array_equal(vali[:16], A.astype(np.float64)) and (vali[16:] == 0).all()
    # a transposed operand would fail this non-square case
    B2 = np.arange(6, dtype=np.float32).reshape(3, 2)
    A2 = np.arange(8, dtype=np.float32).reshape(2, 4)
    v2, _ = oracle.lora(B2, A2, 1.0)
    assert v2.tolist() == [[4, 5, 6, 7], [12, 17, 22, 27], [20, 29, 38, 47]]
    # bf16 operands widen exactly
    B16, A16 = oracle.f32_to_bf16(B), oracle.f32_to_bf16(A)
    v16, _ = oracle.lora(B16, A16, 1.0, BF16)
    assert np.allclose(v16, oracle.bf16_to_f32(B16).astype(np.float64) @ oracle.bf16_to_f32(A16).astype(np.float64),
                       rtol=1e-14, atol=0)


def test_fused_lora_merge_equals_explicit_matrix_products():
    # sum_i (B_i A_i) D_i with the shuffle: against numpy float64 products, explicit diagonal
    # matrices and the permutations drawn separately
    layers = [(6, 9, 0, SRSF)] * 3 + [(4, 5, -1, FLIP)]
    rng = np.random.default_rng(11)
    seeds = [7, 8, 9]
    rank = 3
    factors = [[(rng.standard_normal((m, rank)).astype(np.float32), rng.standard_normal((rank, n)).astype(np.float32))
                for (m, n, _, _) in layers] for _ in seeds]
    got, mag = oracle.lora_merge(layers, factors, seeds, 0.5)
    for l, (m, n, g, fl) in enumerate(layers):
        want = np.zeros((m, n))
        wmag = np.zeros((m, n))
        for i, s in enumerate(seeds):
            t = l if g < 0 else int(oracle.layer_perm(s, g, 3)[l])   # group members are layers 0, 1, 2
            B, A = factors[i][t]
            D = np.diag(1.0 - 2.0 * oracle.sign_mask(s, l, n).astype(np.float64))
            want += B.astype(np.float64) @ A.astype(np.float64) @ D
            wmag += np.abs(B).astype(np.float64) @ np.abs(A).astype(np.float64)
        assert np.allclose(got[l], 0.5 * want, rtol=1e-13, atol=1e-15)
        assert np.allclose(mag[l], 0.5 * wmag, rtol=1e-13)
    # one model, no flags: the plain adapter product
    one, _ = oracle.lora_merge([(6, 9, -1, 0)], [[factors[0][0]]], [1], 1.0)
    ref, _ = oracle.lora(factors[0][0][0], factors[0][0][1], 1.0)
    assert np.array_equal(one[0], ref)


def test_threads_do_not_change_the_result():
    layers = [(37, 129, 0, SRSF)] * 3
    rng = np.random.default_rng(10)
    seeds = [1, 2, 3, 4]
    deltas = [[rng.standard_normal((37, 129)).astype(np.float32) for _ in layers] for _ in seeds]
    a = oracle.merge(layers, deltas, seeds, n_threads=1)
    b = oracle.merge(layers, deltas, seeds, n_threads=4)
    for l in range(3):
        assert np.array_equal(a[l].view(np.uint32), b[l].view(np.uint32))


def test_merge_from_weights_equals_merge_of_float32_deltas():
    # Delta_i = Theta_i - Theta_0 (Sec. 3), formed in binary32: identical to merging the numpy
    # float32 differences; for bf16 weights the difference is NOT rounded back to bf16
    layers = [(5, 40, 0, SRSF)] * 3 + [(2, 9, -1, FLIP)]
    rng = np.random.default_rng(12)
    seeds = [3, 4, 5]
    base = [rng.standard_normal((m, n)).astype(np.float32) * 0.02 for (m, n, _, _) in layers]
    weights = [[b + rng.standard_normal(b.shape).astype(np.float32) * 1e-3 for b in base] for _ in seeds]
    deltas = [[w - b for w, b in zip(per, base)] for per in weights]
    a = oracle.merge_weights(layers, weights, base, seeds)
    b_ = oracle.merge(layers, deltas, seeds)
    for l in range(len(layers)):
        assert np.array_equal(a[l].view(np.uint32), b_[l].view(np.uint32))
    base16 = [oracle.f32_to_bf16(x) for x in base]
    w16 = [[oracle.f32_to_bf16(x) for x in per] for per in weights]
    d32 = [[oracle.bf16_to_f32(w) - oracle.bf16_to_f32(b) for w, b in zip(per, base16)] for per in w16]
    a16 = oracle.merge_weights(layers, w16, base16, seeds, BF16, BF16)
    b16 = oracle.merge(layers, d32, seeds, F32, BF16)
    for l in range(len(layers)):
        assert np.array_equal(a16[l], b16[l])
    # the base that is subtracted is the one of the SOURCE layer (it travels with the shuffle):
    # with every model equal to the base the result is exactly zero whatever the permutation
    z = oracle.merge_weights(layers, [base, base], base, [1, 2])
    for l in range(len(layers)):
        assert (z[l] == 0).all()


def test_delta_stats_against_numpy_and_the_merge_itself():
    layers = [(4, 33, 0, SRSF)] * 3 + [(3, 10, -1, FLIP)]
    rng = np.random.default_rng(13)
    a = [rng.standard_normal((m, n)).astype(np.float32) for (m, n, _, _) in layers]
    b = [rng.standard_normal((m, n)).astype(np.float32) for (m, n, _, _) in layers]
    sa, sb = 21, 22
    ab, aa, bb = oracle.delta_stats(layers, a, sa, b, sb)
    # explicit: transformed copies through the single-model merge (already pinned), then numpy
    ta = oracle.merge(layers, [a], [sa])
    tb = oracle.merge(layers, [b], [sb])
    fa = np.concatenate([x.reshape(-1).astype(np.float64) for x in ta])
    fb = np.concatenate([x.reshape(-1).astype(np.float64) for x in tb])
    assert abs(ab - fa @ fb) < 1e-10 and abs(aa - fa @ fa) < 1e-10 and abs(bb - fb @ fb) < 1e-10
    # orthogonal transforms keep norms: same as the untransformed norms
    ra = np.concatenate([x.reshape(-1).astype(np.float64) for x in a])
    assert abs(aa - ra @ ra) < 1e-10
    # the same transform on both sides keeps the inner product (O_i^T O_i = I)
    ab_same, _, _ = oracle.delta_stats(layers, a, sa, b, sa)
    rb_ = np.concatenate([x.reshape(-1).astype(np.float64) for x in b])
    assert abs(ab_same - ra @ rb_) < 1e-10
    # no flags: plain inner products
    plain = [(m, n, g, 0) for (m, n, g, _) in layers]
    ab0, aa0, bb0 = oracle.delta_stats(plain, a, sa, b, sb)
    assert abs(ab0 - ra @ rb_) < 1e-10
    # Sec. 3 norm identity through these sums: ||a' + b'||^2 = aa + bb + 2 ab
    m2 = oracle.merge(layers, [a, b], [sa, sb])
    fm = np.concatenate([x.reshape(-1).astype(np.float64) for x in m2])
    assert abs(fm @ fm - (aa + bb + 2 * ab)) < 1e-4 * (aa + bb)   # merge rounds to float32

"""Pins for the CPU oracle's prune (Alg. 1 and the pruning functions of Sec. III-B).

None of the expectations below is produced by the oracle itself: they come from
the paper's worked example, from brute-force enumeration of all keep-sets with
keys computed here by other means (float comparison instead of bit patterns,
Python integers for the hash), from closed forms and from invariants.
"""
import itertools
import os

import numpy as np
import pytest

import oracle
from paper_2202_00774_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
RANKERS = (oracle.RANDOM, oracle.GREEDY, oracle.GREEDY_ADJUSTED)


# ------------------------------------------------------------------ helpers

def store(x, dtype):
    """float values -> storage array of the dtype (values used here are exact in bf16)."""
    x = np.asarray(x, dtype=np.float32)
    return wl.f32_to_bf16_bits(x) if dtype == oracle.BF16 else x


def load(a):
    return wl.bf16_bits_to_f32(a) if a.dtype == np.uint16 else a


def py_hash(seed, e):
    """The counter hash with Python integers (Sec. III-B gives no generator; this is the build's definition)."""
    M = 0xFFFFFFFF
    x, y, s0, s1 = e & M, (e >> 32) & M, seed & M, (seed >> 32) & M
    v = 0xA54FF53A ^ (x >> 2) ^ ((s0 * 0x9E3779B9) & M) ^ ((y * 0xBB67AE85) & M) ^ ((s1 * 0x510E527F) & M)
    v ^= v >> 16
    v = (v * 0x6A09E667) & M
    v ^= v >> 15
    v = (v * 0xBB67AE85) & M
    v ^= v >> 16
    rot = 8 * (x & 3)           # one mixed word per aligned quad of elements, one byte rotation of it per element
    return ((v << rot) | (v >> (32 - rot))) & M & 0xFFFFFFF0   # a key is 28 bits wide: the low four are cleared


def brute_force_keep(keys, n):
    """The unique n-subset S with (key_j, -j) > (key_j', -j') for every j in S, j' not in S.

    Enumerates all C(m, n) subsets and asserts that exactly one qualifies.
    """
    m = len(keys)
    found = []
    for S in itertools.combinations(range(m), n):
        inside = set(S)
        ok = all((keys[j], -j) > (keys[jp], -jp) for j in S for jp in range(m) if jp not in inside)
        if ok:
            found.append(S)
    assert len(found) == 1, (keys, n, found)
    return found[0]


def kept_positions(idx_row, n):
    return [tuple(int(v) for v in idx_row[g * n:(g + 1) * n]) for g in range(len(idx_row) // n)]


# ------------------------------------------------- the paper's worked example

def read_example():
    vals = {}
    with open(os.path.join(GOLDEN, "paper_magnitude_example.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *rest = line.split()
            vals[k] = [float(v) for v in rest]
    return vals["group"], int(vals["n"][0]), vals["pruned"]


@pytest.mark.parametrize("dtype", [oracle.F32, oracle.BF16])
def test_paper_worked_example(dtype):
    group, n, expect = read_example()
    pruned, vals, idx = oracle.prune(store([group], dtype), n, len(group), oracle.GREEDY)
    assert load(pruned)[0].tolist() == expect
    assert idx[0].tolist() == [1, 2]
    assert load(vals)[0].tolist() == [7.0, -3.0]


@pytest.mark.parametrize("dtype", [oracle.F32, oracle.BF16])
def test_paper_example_rescaled(dtype):
    """Rescaled Magnitude on the same group: |.|_1 = 13, kept 10, so the kept values become 7*1.3, -3*1.3."""
    group, n, _ = read_example()
    pruned, vals, idx = oracle.prune(store([group], dtype), n, 4, oracle.GREEDY_ADJUSTED)
    assert idx[0].tolist() == [1, 2]
    out = load(pruned)[0].astype(np.float64)
    assert out[0] == 0 and out[3] == 0
    ulp = 2.0 ** -23 if dtype == oracle.F32 else 2.0 ** -8
    assert abs(out[1] - 9.1) <= 9.1 * ulp and abs(out[2] + 3.9) <= 3.9 * ulp
    # the exact bit patterns follow from s = fl32(13/10) and one rounding of the product
    s = np.float32(13.0) / np.float32(10.0)
    assert s.view(np.uint32) == 0x3FA66666
    if dtype == oracle.F32:
        assert pruned.view(np.uint32)[0].tolist() == [0, 0x41119999, 0xC0799999, 0]
    else:
        assert pruned[0].tolist() == [0, 0x4112, 0xC07A, 0]


# ---------------------------------------------------------- greedy keep-set

ALPHABET = [-2.0, -1.0, -0.0, 0.0, 1.0, 2.0]


@pytest.mark.parametrize("dtype", [oracle.F32, oracle.BF16])
@pytest.mark.parametrize("n", [1, 2, 3, 4])
def test_greedy_exhaustive_groups_of_four(dtype, n):
    groups = np.array(list(itertools.product(ALPHABET, repeat=4)), dtype=np.float32)  # 1296 groups
    dO = store(groups, dtype)
    before = dO.copy()
    pruned, vals, idx = oracle.prune(dO, n, 4, oracle.GREEDY)
    assert np.array_equal(dO, before)
    for row in range(groups.shape[0]):
        keys = [abs(float(v)) for v in groups[row]]           # float compare; -0.0 and 0.0 tie
        S = brute_force_keep(keys, n)
        assert tuple(idx[row].tolist()) == S
        expect = np.zeros(4, np.float32)
        expect[list(S)] = groups[row, list(S)]
        # bit compare: kept -0.0 stays -0.0, dropped slots are +0.0
        assert np.array_equal(store(expect, dtype).view(np.uint8), pruned[row].view(np.uint8))
        # among all subsets, S has the largest sum of magnitudes, and is the first such in lexicographic order
        best = max(sum(keys[j] for j in T) for T in itertools.combinations(range(4), n))
        firsts = [T for T in itertools.combinations(range(4), n) if sum(keys[j] for j in T) == best]
        assert S == firsts[0]


@pytest.mark.parametrize("dtype", [oracle.F32, oracle.BF16])
@pytest.mark.parametrize("n,m", [(2, 8), (4, 8), (1, 8), (2, 16), (4, 16), (3, 5), (7, 7), (4, 32), (16, 32), (2, 2), (1, 1)])
def test_greedy_bruteforce_random_groups(dtype, n, m):
    rng = np.random.default_rng(100 * m + n)
    count = 300 if m <= 16 else 4
    groups = rng.choice(np.array(ALPHABET + [0.5, -0.5, 3.0], np.float32), size=(count, m))
    pruned, vals, idx = oracle.prune(store(groups.reshape(count // 2, 2 * m), dtype), n, m, oracle.GREEDY)
    idx = idx.reshape(count, n)
    for row in range(count):
        keys = [abs(float(v)) for v in groups[row]]
        if m <= 16:
            S = brute_force_keep(keys, n)
        else:  # C(32,16) is too many subsets: use the sorted order instead
            S = tuple(sorted(sorted(range(m), key=lambda j: (-keys[j], j))[:n]))
        assert tuple(idx[row].tolist()) == S


def test_greedy_hand_cases():
    cases = [([0, 0, 5, 0], (0, 2)), ([-2, 2, 2, -2], (0, 1)), ([0, 0, 0, 0], (0, 1)), ([1, 2, 3, 4], (2, 3)),
             ([4, 3, 2, 1], (0, 1)), ([-0.0, 0.0, -0.0, 1], (0, 3))]
    for dtype in (oracle.F32, oracle.BF16):
        for g, S in cases:
            _, _, idx = oracle.prune(store([g], dtype), 2, 4, oracle.GREEDY)
            assert tuple(idx[0].tolist()) == S, (g, dtype)


def test_greedy_uses_bit_pattern_order_for_tiny_and_infinite_values():
    """Subnormals are ranked by their true magnitude (no flush to zero); infinity outranks every finite value."""
    tiny = np.array([1e-45, 3e-45, 0.0, 1e-44], np.float32)           # fp32 subnormals
    _, _, idx = oracle.prune(tiny[None], 2, 4, oracle.GREEDY)
    assert idx[0].tolist() == [1, 3]
    big = np.array([np.inf, 3e38, -np.inf, 1.0], np.float32)
    _, _, idx = oracle.prune(big[None], 2, 4, oracle.GREEDY)
    assert idx[0].tolist() == [0, 2]
    bf = np.array([0x0001, 0x8003, 0x0000, 0x0002], np.uint16)        # bf16 subnormals, one negative
    _, _, idx = oracle.prune(bf[None], 2, 4, oracle.GREEDY)
    assert idx[0].tolist() == [1, 3]


# ------------------------------------------------------------- structure

@pytest.mark.parametrize("ranker", RANKERS)
@pytest.mark.parametrize("dtype", [oracle.F32, oracle.BF16])
@pytest.mark.parametrize("n,m", [(2, 4), (2, 8), (2, 16), (4, 8), (4, 32), (1, 4), (3, 4)])
def test_structure_invariants(ranker, dtype, n, m):
    dO = wl.laplace_with_zeros((7, 5, 3 * m * 2), 1e-3, 0.3, seed=m * 10 + n, dtype=dtype)
    before = dO.copy()
    pruned, vals, idx = oracle.prune(dO, n, m, ranker, seed=9)
    assert np.array_equal(dO, before)                          # dL/dO survives: it is needed for dL/dW
    rows = dO.size // dO.shape[-1]
    C = dO.shape[-1]
    G = C // m
    idxg = idx.reshape(rows, G, n).astype(np.int64)
    assert idxg.max() < m
    assert np.all(np.diff(idxg, axis=2) > 0) or n == 1        # strictly ascending inside a group
    # scattering the compact form reproduces the dense-shaped form, bit for bit
    scat = np.zeros((rows, G, m), dO.dtype)
    np.put_along_axis(scat, idxg, vals.reshape(rows, G, n), axis=2)
    assert np.array_equal(scat.reshape(dO.shape).view(np.uint8), pruned.view(np.uint8))
    # at most n nonzeros in every group of m
    nz = (load(pruned).reshape(rows, G, m) != 0).sum(axis=2)
    assert nz.max() <= n
    if ranker != oracle.GREEDY_ADJUSTED:                        # kept values are bit copies
        src = np.take_along_axis(dO.reshape(rows, G, m), idxg, axis=2)
        assert np.array_equal(src.view(np.uint8), vals.reshape(rows, G, n).view(np.uint8))


@pytest.mark.parametrize("ranker", RANKERS)
@pytest.mark.parametrize("dtype", [oracle.F32, oracle.BF16])
def test_n_equals_m_is_identity(ranker, dtype):
    dO = wl.laplace_with_zeros((33, 64), 1e-3, 0.3, seed=5, dtype=dtype)
    pruned, vals, idx = oracle.prune(dO, 8, 8, ranker, seed=3)
    # an exact zero (of either sign) times the scale 1 is itself; everything is kept
    assert np.array_equal(load(pruned), load(dO))
    assert np.array_equal(idx.reshape(-1, 8), np.tile(np.arange(8, dtype=np.uint8), (33 * 8, 1)))
    if ranker != oracle.GREEDY_ADJUSTED:
        assert np.array_equal(pruned, dO)


def test_rejects_bad_arguments():
    dO = np.zeros((2, 12), np.float32)
    for n, m in ((0, 4), (5, 4), (2, 5), (2, 64)):
        with pytest.raises(ValueError):
            oracle.prune(dO, n, m, oracle.GREEDY)


def test_empty_tensor():
    pruned, vals, idx = oracle.prune(np.zeros((0, 16), np.float32), 2, 4, oracle.GREEDY)
    assert pruned.shape == (0, 16) and vals.shape == (0, 8) and idx.shape == (0, 8)


# ---------------------------------------------------------------- random

def test_hash_matches_stored_vectors_and_python_integers():
    with open(os.path.join(GOLDEN, "hash_vectors.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            seed, e, h = line.split()
            assert oracle.hash32(int(seed), int(e)) == int(h, 16)
            assert py_hash(int(seed), int(e)) == int(h, 16)
    rng = np.random.default_rng(7)
    for _ in range(2000):
        seed = int(rng.integers(0, 2 ** 63)) * 2 + int(rng.integers(0, 2))
        e = int(rng.integers(0, 2 ** 63)) * 2 + int(rng.integers(0, 2))
        assert oracle.hash32(seed, e) == py_hash(seed, e)


def test_random_first_groups_from_stored_vectors():
    """With seed 0 the stored hash values (the byte rotations of 0x20179656 for elements 0-3 and of 0x69A5D3E6 for 4-7, low four
    bits cleared) make row 0 keep {2,3} in group 0 and {2,3} in group 1 at 2:4, {6,7} at 2:8."""
    dO = np.arange(16, dtype=np.float32)[None]
    _, _, idx = oracle.prune(dO, 2, 4, oracle.RANDOM, seed=0)
    assert idx[0, :4].tolist() == [2, 3, 2, 3]
    _, _, idx = oracle.prune(dO, 2, 8, oracle.RANDOM, seed=0)
    assert idx[0, :2].tolist() == [6, 7]


@pytest.mark.parametrize("dtype", [oracle.F32, oracle.BF16])
@pytest.mark.parametrize("n,m", [(2, 4), (2, 8), (3, 8), (2, 16)])
def test_random_keep_set_is_top_n_of_hash_over_flat_index(dtype, n, m):
    rows, C = 9, 4 * m
    dO = wl.laplace_with_zeros((rows, C), 1.0, 0.3, seed=1, dtype=dtype)
    seed = 0x1234_5678_9ABC_DEF0
    pruned, vals, idx = oracle.prune(dO, n, m, oracle.RANDOM, seed=seed)
    idx = idx.reshape(rows, C // m, n)
    for i in range(rows):
        for g in range(C // m):
            keys = [py_hash(seed, i * C + g * m + j) for j in range(m)]
            assert tuple(idx[i, g].tolist()) == brute_force_keep(keys, n)
    # the values play no part: a different tensor gives the same positions
    other = wl.laplace_with_zeros((rows, C), 1.0, 0.0, seed=2, dtype=dtype)
    _, _, idx2 = oracle.prune(other, n, m, oracle.RANDOM, seed=seed)
    assert np.array_equal(idx2.reshape(idx.shape), idx)
    # and another seed gives other positions
    _, _, idx3 = oracle.prune(other, n, m, oracle.RANDOM, seed=seed + 1)
    assert not np.array_equal(idx3.reshape(idx.shape), idx)


def test_random_is_uniform_over_subsets():
    """Chi-square test: each of the C(4,2)=6 keep-sets of a 2:4 group is equally likely; also 2:8 (28 sets)."""
    for n, m, groups in ((2, 4, 60000), (2, 8, 84000)):
        dO = np.zeros((groups // 10, 10 * m), np.float32)
        _, _, idx = oracle.prune(dO, n, m, oracle.RANDOM, seed=42)
        sets, counts = np.unique(idx.reshape(-1, n), axis=0, return_counts=True)
        k = len(list(itertools.combinations(range(m), n)))
        assert len(sets) == k
        expected = groups / k
        chi2 = float(((counts - expected) ** 2 / expected).sum())
        # 99.99 % quantile of chi-square with k-1 degrees of freedom: 25.7 (5 dof), 63.2 (27 dof)
        assert chi2 < (25.7 if k == 6 else 63.2), chi2


def test_random_independent_of_row_shape():
    """The flat element index is row*C + channel, so reshaping rows (same C) changes nothing."""
    dO = wl.laplace_with_zeros((6, 4, 32), 1.0, 0.2, seed=3, dtype=oracle.BF16)
    a = oracle.prune(dO, 2, 8, oracle.RANDOM, seed=5)[0]
    b = oracle.prune(dO.reshape(24, 32), 2, 8, oracle.RANDOM, seed=5)[0]
    assert np.array_equal(a.reshape(24, 32), b)


# --------------------------------------------------------------- adjusted

@pytest.mark.parametrize("dtype", [oracle.F32, oracle.BF16])
@pytest.mark.parametrize("n,m", [(2, 4), (2, 8), (2, 16), (4, 8), (4, 32)])
def test_adjusted_invariants(dtype, n, m):
    rows, C = 64, 4 * m
    dO = wl.laplace_with_zeros((rows, C), 1e-3, 0.3, seed=77 + m, dtype=dtype)
    g_pruned, g_vals, g_idx = oracle.prune(dO, n, m, oracle.GREEDY)
    a_pruned, a_vals, a_idx = oracle.prune(dO, n, m, oracle.GREEDY_ADJUSTED)
    assert np.array_equal(g_idx, a_idx)                       # Sec. III-C: both prune the same elements
    x = np.abs(wl.to_f64(dO)).reshape(rows, C // m, m)
    kept = np.abs(wl.to_f64(g_pruned)).reshape(rows, C // m, m)
    out = np.abs(wl.to_f64(a_pruned)).reshape(rows, C // m, m)
    S, T, U = x.sum(2), kept.sum(2), out.sum(2)
    live = T > 0
    # the L1 norm of every group is preserved up to the rounding of the scale and of each product
    eps = 2.0 ** -22 if dtype == oracle.F32 else 2.0 ** -8
    assert np.all(np.abs(U[live] - S[live]) <= eps * (m + 2) * S[live])
    assert np.all(U[~live] == 0)
    # the implied scale lies in [1, m/n]: the kept are the n largest of m
    scale = U[live] / T[live]
    assert scale.min() >= 1 - eps * 4 and scale.max() <= m / n * (1 + eps * 4)
    # signs never change and every kept value moves by the same factor (within rounding)
    assert np.all(np.sign(wl.to_f64(a_pruned)) == np.sign(wl.to_f64(g_pruned)))
    ratio = np.abs(wl.to_f64(a_vals)) / np.maximum(np.abs(wl.to_f64(g_vals)), 1e-300)
    ratio = ratio.reshape(rows, C // m, n)
    nzk = np.abs(wl.to_f64(g_vals)).reshape(rows, C // m, n) > 0
    group_scale = (S / np.where(T > 0, T, 1))[:, :, None]
    assert np.all(np.abs(ratio - group_scale)[nzk] <= 4 * eps * group_scale.repeat(n, 2)[nzk])


def test_adjusted_exact_small_cases():
    """Cases whose scale and products are exact in binary: the result is known without rounding."""
    # |.|_1 = 8, kept 4 -> s = 2 ; |.|_1 = 6, kept 4 -> 1.5 ; nothing to rescale when the dropped are zero
    cases = [([2, -2, 2, 2], [4, -4, 0, 0]), ([1, 3, -1, 1], [1.5, 4.5, 0, 0]), ([0, 5, 0, -7], [0, 5, 0, -7]),
             ([0, 0, 0, 0], [0, 0, 0, 0]), ([0.5, 0, 0, 0], [0.5, 0, 0, 0])]
    for dtype in (oracle.F32, oracle.BF16):
        for g, expect in cases:
            pruned, _, _ = oracle.prune(store([g], dtype), 2, 4, oracle.GREEDY_ADJUSTED)
            assert load(pruned)[0].tolist() == [float(v) for v in expect], (g, dtype)


def test_adjusted_fp32_summation_order_is_ascending():
    """Sums are taken left to right in fp32: 2^24 + 1 + 1 stays 2^24, but 1 + 1 + 2^24 is 2^24 + 2."""
    big = np.float32(2.0 ** 24)
    a = np.array([[big, 1, 1, 0]], np.float32)       # total = fl(fl(2^24+1)+1) = 2^24, kept = fl(2^24+1) = 2^24 -> s = 1
    b = np.array([[1, 1, big, 0]], np.float32)       # total = 2^24+2, kept (positions 0 and 2) = fl(1+2^24) = 2^24
    pa = oracle.prune(a, 2, 4, oracle.GREEDY_ADJUSTED)[0]
    pb = oracle.prune(b, 2, 4, oracle.GREEDY_ADJUSTED)[0]
    assert pa[0].tolist() == [float(big), 1.0, 0.0, 0.0]
    s = np.float32(np.float32(2.0 ** 24 + 2) / big)
    assert pb[0].tolist() == [float(np.float32(1) * s), 0.0, float(big * s), 0.0]


def test_adjusted_bf16_rounds_to_nearest_even():
    # group [1, 1, 0.5, 0.00390625*?]: choose s so that the product falls exactly between two bf16 values.
    # x = 1 + 2^-7 (bf16), |.|_1 = x + x/... simpler: s = 1.5 exactly with x = 1 + 2^-7 -> x*s = 1.5 + 1.5*2^-7
    # = 1.51171875 = 1.5 + 2^-7 + 2^-8: halfway between 1.5078125 (odd mantissa) and 1.515625 (even) -> even.
    x = 1.0 + 2.0 ** -7
    g = [x, x, x, 0.0]                              # total 3x, kept 2x -> s = 1.5
    pruned, _, _ = oracle.prune(store([g], oracle.BF16), 2, 4, oracle.GREEDY_ADJUSTED)
    out = load(pruned)[0]
    assert out.tolist() == [1.515625, 1.515625, 0.0, 0.0]
    assert oracle.float_to_bf16(1.51171875) == oracle.float_to_bf16(1.515625)
    assert oracle.bf16_to_float(oracle.float_to_bf16(1.50390625)) == 1.5     # the other tie goes down to even


def test_bf16_conversion_against_exhaustive_definition():
    """Round-to-nearest-even bf16 of a float is the nearest of its two bf16 neighbours, even mantissa on ties."""
    rng = np.random.default_rng(0)
    xs = np.concatenate([rng.standard_normal(3000).astype(np.float32) * np.float32(1e-3),
                         np.array([1.0, 1.00390625, 1.001953125, 3.3895314e38, 1e-40, 0.0, -0.0], np.float32)])
    for x in xs:
        u = int(np.float32(x).view(np.uint32))
        lo = u & 0xFFFF0000
        hi = lo + 0x10000
        flo, fhi = (np.uint32(v).view(np.float32).astype(np.float64) for v in (lo, hi & 0xFFFFFFFF))
        dlo, dhi = abs(float(x) - flo), abs(fhi - float(x))
        want = lo if dlo < dhi or (dlo == dhi and (lo >> 16) % 2 == 0) else hi
        assert oracle.float_to_bf16(float(x)) == (want >> 16) & 0xFFFF
    assert np.array_equal(wl.f32_to_bf16_bits(xs), np.array([oracle.float_to_bf16(float(x)) for x in xs], np.uint16))

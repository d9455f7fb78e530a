"""Property tests of the oracle (CPU only): facts that the definitions of Sec. II-C and Alg. 2 fix for ANY input,
checked on inputs drawn by hypothesis.  None of them re-types an oracle formula: each compares the oracle with
what the definition implies directly (a full sort, exact integer arithmetic, a vector with one non-zero).
"""
import numpy as np
from hypothesis import given, settings, strategies as st

import oracle
from oracle import Oracle
from paper_2210_07454_amd import inputs

P = 2147483647
floats32 = st.floats(width=32, allow_nan=False, allow_infinity=False)


@settings(max_examples=150, deadline=None)
@given(st.lists(st.one_of(floats32, st.sampled_from([0.0, -0.0, 1.0, -1.0, 2.5, -2.5])), min_size=1, max_size=60),
       st.data())
def test_topk_is_the_head_of_the_full_sort(values, data):
    # Top-k by magnitude, ties to the smaller coordinate, result ascending: the first k of the sort by
    # (-|x|, index), whatever the values (signed zeros and repeated magnitudes included)
    est = np.array(values, dtype=np.float32)
    k = data.draw(st.integers(1, len(values)))
    order = sorted(range(len(values)), key=lambda l: (-abs(float(est[l])), l))
    want = np.sort(np.array(order[:k], dtype=np.int32))
    assert np.array_equal(Oracle("f32").topk(est, k), want)


@settings(max_examples=60, deadline=None)
@given(st.integers(1, 400), st.integers(1, 8), st.integers(1, 97), st.integers(0, 2 ** 31 - 1), st.integers(-5, 5))
def test_sketch_is_linear_on_integer_vectors(d, r, c, seed, alpha):
    # Eq. (3): S(alpha a + b) = alpha S(a) + S(b); with small integers every sum is exact in fp32
    rng = np.random.default_rng(seed)
    hp = inputs.hash_params(r, seed=seed % 1000)
    a = rng.integers(-50, 51, d).astype(np.float32)
    b = rng.integers(-50, 51, d).astype(np.float32)
    o = Oracle("f32")
    lhs = o.sketch((alpha * a + b).astype(np.float32), hp, c)
    assert np.array_equal(lhs, alpha * o.sketch(a, hp, c) + o.sketch(b, hp, c))


@settings(max_examples=80, deadline=None)
@given(st.integers(1, 300), st.integers(1, 10), st.integers(1, 64), st.integers(0, 10 ** 6),
       st.floats(min_value=-1e6, max_value=1e6, width=32).filter(lambda x: x != 0.0), st.data())
def test_one_nonzero_coordinate_is_recovered_exactly(d, r, c, seed, x, data):
    # Sec. II-C: a vector with a single non-zero x at l puts s_j(l) x into one cell per row; every row's
    # estimate of l is then s_j(l)^2 x = x, and so is their median.  Any other coordinate reads, per row,
    # either an empty cell (0) or that same cell (+x or -x): nothing else can come out.
    l = data.draw(st.integers(0, d - 1))
    hp = inputs.hash_params(r, seed=seed % 1000)
    u = np.zeros(d, np.float32)
    u[l] = np.float32(x)
    o = Oracle("f32")
    S = o.sketch(u, hp, c)
    assert np.count_nonzero(S) == r                  # one cell per row
    bkt, sgn = oracle.hash_dump(hp, c, d)
    for j in range(r):
        assert S[j, bkt[j, l]] == np.float32(sgn[j, l]) * np.float32(x)
    est = o.unsketch(S, None, d, hp)
    assert est[l] == np.float32(x)
    assert set(np.abs(est).tolist()) <= {0.0, abs(float(np.float32(x)))}


@settings(max_examples=100, deadline=None)
@given(st.lists(floats32, min_size=1, max_size=50), st.data())
def test_refine_keeps_the_largest_exact_values_among_the_candidates(values, data):
    # Sec. III-A second round: of the candidates, the k_out with the largest exact magnitude (ties to the
    # smaller coordinate), returned with their coordinates ascending
    n = len(values)
    cand = np.sort(np.array(data.draw(st.lists(st.integers(0, 10_000), min_size=n, max_size=n, unique=True)),
                            dtype=np.int32))
    delta = np.array(values, dtype=np.float32)
    k_out = data.draw(st.integers(1, n))
    order = sorted(range(n), key=lambda q: (-abs(float(delta[q])), int(cand[q])))[:k_out]
    keep = sorted(order, key=lambda q: int(cand[q]))
    idx, val = Oracle("f32").refine(cand, delta, k_out)
    assert np.array_equal(idx, cand[keep]) and np.array_equal(val, delta[keep])


@settings(max_examples=100, deadline=None)
@given(st.integers(1, P - 1), st.integers(0, P - 1), st.integers(0, P - 2), st.integers(1, 2 ** 31 - 2))
def test_hash_is_the_affine_map_modulo_the_mersenne_prime(a, b, l, c):
    y = (a * l + b) % P                              # Python integers: no overflow to get wrong
    assert oracle.hash_y(a, b, l) == y
    assert oracle.bucket(a, b, l, c) == y % c

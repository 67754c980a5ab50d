"""Pins of the oracle's functions for chunks that follow earlier context (no GPU)."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_worked_scores_with_context.txt")


def _parse_num(tok):
    if tok.startswith("ln"):
        return math.log(float(tok[2:]))
    return float(Fraction(tok))


def test_golden_hand_worked_examples_with_context():
    n_cases = 0
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        head, ks, exp = [p.strip() for p in line.split("|")]
        _, P, N, n, qv = head.split()
        P, N, n, qv = int(P), int(N), int(n), float(qv)
        k = np.array([_parse_num(t) for t in ks.split()]).reshape(P + N, 1, 1)
        q = np.full((N, 1, 1), qv)
        want = np.array([_parse_num(t) for t in exp.split()])
        got = oracle.importance_scores_with_context(q, k, [0, N], [0, P + N], n_obs=n, scale=1.0)
        np.testing.assert_allclose(got, want, rtol=1e-14, atol=0)
        n_cases += 1
    assert n_cases == 5


def _batch(rng, Ps, Ns, Hq=4, Hkv=2, D=8):
    cq = np.concatenate([[0], np.cumsum(Ns)])
    ck = np.concatenate([[0], np.cumsum(np.add(Ps, Ns))])
    q = rng.standard_normal((cq[-1], Hq, D))
    k = rng.standard_normal((ck[-1], Hkv, D))
    return q, k, cq, ck


def test_without_earlier_tokens_it_is_the_plain_score():
    rng = np.random.default_rng(0)
    Ns = [1, 17, 0, 300, 64]
    q, k, cq, ck = _batch(rng, [0] * len(Ns), Ns)
    got = oracle.importance_scores_with_context(q, k, cq, ck, n_obs=32)
    want = oracle.importance_scores(q, k, cq, n_obs=32)
    np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("P,N,n", [(100, 50, 16), (7, 300, 128), (513, 1, 128), (64, 64, 200), (1000, 130, 128)])
def test_chunk_scores_are_the_tail_of_the_whole_sequence_scores(P, N, n):
    """A chunk of N tokens after P earlier ones, window n <= N or n > N: the scores are those of
    the sequence so far, scored as one sequence with the window min(n, N), at the chunk's tokens."""
    rng = np.random.default_rng(P + N)
    Hq, Hkv, D = 6, 2, 16
    k = rng.standard_normal((P + N, Hkv, D))
    q_chunk = rng.standard_normal((N, Hq, D))
    q_whole = np.concatenate([np.full((P, Hq, D), np.nan), q_chunk])     # earlier queries are never read
    whole = oracle.importance_scores(q_whole, k, [0, P + N], n_obs=min(n, N))
    got = oracle.importance_scores_with_context(q_chunk, k, [0, N], [0, P + N], n_obs=n)
    np.testing.assert_allclose(got, whole[P:], rtol=1e-13, atol=0)
    # the chunk's share of the attention mass plus the earlier tokens' share is the whole
    assert abs(got.sum() + whole[:P].sum() - 1.0) < 1e-12


@pytest.mark.parametrize("P,N,n", [(5, 3, 2), (200, 128, 128), (1000, 40, 128), (3, 700, 64)])
def test_harmonic_closed_form_with_context(P, N, n):
    """Q = 0: the row at position p spreads 1/(p+1) over keys 0..p, so chunk token i gets
    (1/n_eff) * sum over window positions p >= P+i of 1/(p+1)."""
    rng = np.random.default_rng(3)
    Hq, Hkv, D = 4, 2, 8
    q = np.zeros((N, Hq, D))
    k = rng.standard_normal((P + N, Hkv, D))
    got = oracle.importance_scores_with_context(q, k, [0, N], [0, P + N], n_obs=n)
    n_eff, L = min(n, N), P + N
    want = [float(sum(Fraction(1, p + 1) for p in range(max(P + i, L - n_eff), L)) / n_eff) for i in range(N)]
    np.testing.assert_allclose(got, want, rtol=1e-13)


def test_softmax_library_routine_single_row():
    """n = 1, one head: the chunk scores are the tail of scipy's softmax of the last row's logits."""
    from scipy.special import softmax
    rng = np.random.default_rng(4)
    P, N, D = 37, 20, 8
    q = rng.standard_normal((N, 1, D))
    k = rng.standard_normal((P + N, 1, D))
    got = oracle.importance_scores_with_context(q, k, [0, N], [0, P + N], n_obs=1)
    want = softmax((k[:, 0, :] @ q[-1, 0, :]) / math.sqrt(D))[P:]
    np.testing.assert_allclose(got, want, rtol=1e-13)


def test_batch_is_the_concatenation_of_its_requests():
    rng = np.random.default_rng(5)
    Ps, Ns = [0, 40, 300, 5, 129], [64, 1, 200, 0, 77]
    q, k, cq, ck = _batch(rng, Ps, Ns)
    got = oracle.importance_scores_with_context(q, k, cq, ck, n_obs=64)
    for r in range(len(Ns)):
        one = oracle.importance_scores_with_context(q[cq[r]:cq[r + 1]], k[ck[r]:ck[r + 1]], [0, Ns[r]],
                                                    [0, Ps[r] + Ns[r]], n_obs=64)
        np.testing.assert_array_equal(got[cq[r]:cq[r + 1]], one)


def test_sinks_inside_the_chunk():
    assert list(oracle.sinks_in_chunk([0, 10, 20, 30], [0, 10, 25, 200], 8)) == [8, 3, 0]


def test_selection_with_context_forces_only_the_sinks_that_fall_in_the_chunk():
    rng = np.random.default_rng(6)
    Ps, Ns = [0, 100, 1000], [700, 700, 700]
    cq = np.concatenate([[0], np.cumsum(Ns)])
    ck = np.concatenate([[0], np.cumsum(np.add(Ps, Ns))])
    s = rng.random(cq[-1]).astype(np.float32)
    s[cq[1]:cq[1] + 128] = 0.0          # would-be sinks of request 1: only the first 28 are forced
    s[cq[2]:cq[2] + 128] = 0.0          # request 2 has no sink in its chunk
    kept, new_cu = oracle.select_tokens_with_context(s, cq, ck, [0.25] * 3, block_size=64, n_obs=128, n_sink=128)
    kept = set(int(x) for x in kept)
    assert all(cq[0] + i in kept for i in range(128))
    assert all(cq[1] + i in kept for i in range(28))
    # block 0 of request 1 (64 tokens, 28 forced, k = max(16, 28) = 28): nothing but the sinks
    assert sum(1 for i in range(64) if cq[1] + i in kept) == 28
    # request 2, block 0: 16 kept by the index rule among all-zero scores
    assert [i for i in range(64) if cq[2] + i in kept] == list(range(16))
    # the last n tokens of every chunk are kept
    for r in range(3):
        assert all(cq[r + 1] - 1 - i in kept for i in range(128))
    # per request it is select_tokens with the reduced sink count
    for r, A in enumerate([128, 28, 0]):
        idx, ncu = oracle.select_tokens(s[cq[r]:cq[r + 1]], [0, Ns[r]], [0.25], block_size=64, n_obs=128, n_sink=A)
        assert ncu[1] == new_cu[r + 1] - new_cu[r]
        assert set(int(x) + int(cq[r]) for x in idx) <= kept


def test_gather_paged_keys_hand_case_and_round_trip():
    """Eq. 16 indexing.  Blocks of 2 rows; request 0 has 3 keys in physical blocks 2 and 0,
    request 1 has 2 keys in block 3: written out by hand."""
    cache = np.arange(10 * 1).reshape(10, 1).astype(np.float64)      # row i holds the value i
    table = np.array([[2, 0], [3, -1]])
    got = oracle.gather_paged_keys(cache, [0, 3, 5], table, 2)
    np.testing.assert_array_equal(got[:, 0], [4, 5, 0, 6, 7])
    # the generator's layout read back is the packed tensor (its own, independent, writer)
    import workloads
    rng = np.random.default_rng(8)
    ck = np.array([0, 37, 37, 100, 164])
    k = rng.standard_normal((164, 2, 4))
    cache, table = workloads.make_paged_cache(k, ck, 16, seed=3)
    np.testing.assert_array_equal(oracle.gather_paged_keys(cache, ck, table, 16), k)
    assert len(set(table[table >= 0].tolist())) == (table >= 0).sum()        # no block used twice


def test_top_p_with_context_differs_from_the_plain_rule_only_in_the_sinks():
    rng = np.random.default_rng(11)
    Ns, Ps = [700, 300, 64, 1000], [0, 50, 500, 127]
    cq = np.concatenate([[0], np.cumsum(Ns)])
    ck = np.concatenate([[0], np.cumsum(np.add(Ns, Ps))])
    s = (rng.random(cq[-1]) ** 6).astype(np.float32)
    tp = np.array([0.9, 0.5, 0.99, 0.7], np.float32)
    kept, new_cu = oracle.select_tokens_top_p_with_context(s, cq, ck, tp, block_size=64, n_obs=32, n_sink=128)
    kept = set(int(x) for x in kept)
    # no earlier tokens anywhere: the plain rule
    k0, n0 = oracle.select_tokens_top_p_with_context(s, cq, cq, tp, block_size=64, n_obs=32, n_sink=128)
    k1, n1 = oracle.select_tokens_top_p(s, cq, tp, block_size=64, n_obs=32, n_sink=128)
    np.testing.assert_array_equal(k0, k1)
    np.testing.assert_array_equal(n0, n1)
    for r, (N, P) in enumerate(zip(Ns, Ps)):
        A = max(0, 128 - P)
        # what the block rule keeps does not depend on the sinks; the forced tokens do
        plain, _ = oracle.select_tokens_top_p(s[cq[r]:cq[r + 1]], [0, N], [tp[r]], block_size=64, n_obs=32, n_sink=0)
        want = set(int(x) + int(cq[r]) for x in plain) | set(int(cq[r]) + i for i in range(min(A, N)))
        assert {t for t in kept if cq[r] <= t < cq[r + 1]} == want
        assert new_cu[r + 1] - new_cu[r] == len(want)


def _lse_of_window_rows(q, k, cq, ck, n_obs, scale=None):
    """Normalisers of the window rows from a library routine (scipy's logsumexp); other rows NaN."""
    from scipy.special import logsumexp
    T, Hq, D = q.shape
    group = Hq // k.shape[1]
    scale = 1.0 / math.sqrt(D) if scale is None else scale
    lse = np.full((Hq, T), np.nan)
    for r in range(len(cq) - 1):
        N, L = cq[r + 1] - cq[r], ck[r + 1] - ck[r]
        for j in range(N - min(n_obs, N), N):
            vis = L - N + j + 1                                    # keys 0 .. P + j
            for h in range(Hq):
                logits = scale * (k[ck[r]:ck[r] + vis, h // group, :] @ q[cq[r] + j, h, :])
                lse[h, cq[r] + j] = logsumexp(logits)
    return lse


def test_scores_from_exact_normalisers_are_the_two_pass_scores():
    rng = np.random.default_rng(12)
    Ps, Ns = [0, 40, 300, 5], [64, 1, 200, 77]
    q, k, cq, ck = _batch(rng, Ps, Ns)
    lse = _lse_of_window_rows(q, k, cq, ck, 32)
    got = oracle.importance_scores_from_lse(q, k, lse, cq, ck, n_obs=32)
    want = oracle.importance_scores_with_context(q, k, cq, ck, n_obs=32)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=0)
    # without earlier tokens: the plain scores
    q2, k2, cq2, _ = _batch(rng, [0, 0], [100, 9])
    lse2 = _lse_of_window_rows(q2, k2, cq2, cq2, 16)
    np.testing.assert_allclose(oracle.importance_scores_from_lse(q2, k2, lse2, cq2, cq2, n_obs=16),
                               oracle.importance_scores(q2, k2, cq2, n_obs=16), rtol=1e-12, atol=0)


def test_scores_from_normalisers_hand_case_and_scaling():
    """One head, D = 1, scale 1, q = 1, keys ln1, ln2, ln3, window of two rows: the normalisers are
    ln 3 and ln 6, the weights [1/3, 2/3, 0] and [1/6, 2/6, 3/6], the scores [1/4, 1/2, 1/4].
    A normaliser that is too large by ln 2 halves that row's weights."""
    q = np.ones((3, 1, 1))
    k = np.log(np.array([1.0, 2.0, 3.0])).reshape(3, 1, 1)
    lse = np.array([[np.nan, math.log(3.0), math.log(6.0)]])
    got = oracle.importance_scores_from_lse(q, k, lse, [0, 3], [0, 3], n_obs=2, scale=1.0)
    np.testing.assert_allclose(got, [1 / 4, 1 / 2, 1 / 4], rtol=1e-14)
    lse[0, 2] += math.log(2.0)
    got = oracle.importance_scores_from_lse(q, k, lse, [0, 3], [0, 3], n_obs=2, scale=1.0)
    np.testing.assert_allclose(got, [(1 / 3 + 1 / 12) / 2, (2 / 3 + 2 / 12) / 2, (3 / 12) / 2], rtol=1e-14)


def test_partial_sums_of_head_shards_add_up_to_the_scores():
    """Eq. 15: with the heads split over ranks (each rank its query heads and their kv heads), the
    ranks' sums add up to n_eff * Hq times the score of the whole model."""
    rng = np.random.default_rng(15)
    Ps, Ns = [0, 40, 300], [64, 1, 200]
    cq = np.concatenate([[0], np.cumsum(Ns)])
    ck = np.concatenate([[0], np.cumsum(np.add(Ps, Ns))])
    Hq, Hkv, D = 8, 4, 8
    q = rng.standard_normal((cq[-1], Hq, D))
    k = rng.standard_normal((ck[-1], Hkv, D))
    whole = oracle.importance_scores_with_context(q, k, cq, ck, n_obs=32)
    parts = [oracle.importance_sums(q[:, 2 * t:2 * t + 2], k[:, t:t + 1], cq, ck, n_obs=32) for t in range(4)]
    got = oracle.scores_from_partial_sums(parts, cq, n_obs=32, total_q_heads=Hq)
    np.testing.assert_allclose(got, whole, rtol=1e-13, atol=0)
    # one rank with all heads: its sums are the scores times rows times heads
    all_heads = oracle.importance_sums(q, k, cq, ck, n_obs=32)
    for r in range(3):
        n_eff = min(32, Ns[r])
        np.testing.assert_allclose(all_heads[cq[r]:cq[r + 1]], whole[cq[r]:cq[r + 1]] * n_eff * Hq, rtol=1e-13)
    # hand case: one head, weights 1:2:3 over two rows -> column sums [1/2, 1, 1/2]
    qh = np.ones((3, 1, 1))
    kh = np.log(np.array([1.0, 2.0, 3.0])).reshape(3, 1, 1)
    np.testing.assert_allclose(oracle.importance_sums(qh, kh, [0, 3], [0, 3], n_obs=2, scale=1.0), [1 / 2, 1.0, 1 / 2], rtol=1e-14)

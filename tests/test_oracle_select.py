"""Pins for the oracle's block partition, forced keeps, key encoding, block-local
top-k, compaction/scatter, and the paper's block-level top-p rule."""
import itertools
import math
import struct

import numpy as np
import pytest

import oracle
import workloads


# ----------------------------------------------------------------------------- phi (Eq. 14)
def test_phi_is_monotone_on_special_and_random_floats():
    rng = np.random.default_rng(0)
    specials = np.array([-np.inf, -3.4028235e38, -1.0, -1e-38, -1e-45, -0.0, 0.0, 1e-45, 1e-38,
                         2.0 ** -64, 1.0, 3.4028235e38, np.inf], dtype=np.float32)
    rnd = rng.standard_normal(4096).astype(np.float32) * np.float32(10.0) ** rng.integers(-30, 30, 4096).astype(np.float32)
    x = np.unique(np.concatenate([specials, rnd]))          # sorted ascending, -0.0/+0.0 collapse
    p = oracle.phi(x).astype(np.int64)
    assert (np.diff(p) > 0).all()
    # -0.0 sorts directly below +0.0 (sign taken from the sign bit)
    assert oracle.phi(np.float32(-0.0)) + 1 == oracle.phi(np.float32(0.0))


def test_phi_matches_bit_definition():
    for v in [0.0, 1.0, 0.5, 1e-20, -1.0, -2.5]:
        bits = struct.unpack("<I", struct.pack("<f", v))[0]
        want = bits ^ (0xFFFFFFFF if v < 0 else 0x80000000)
        assert int(oracle.phi(np.float32(v))) == want


def test_packed_key_order_is_forced_then_score_then_lower_index():
    s = np.array([0.5, 0.5, 0.9, 0.0, 0.9, 0.1], dtype=np.float32)
    forced = np.array([0, 0, 0, 1, 0, 0], dtype=bool)
    keys = oracle.packed_keys(s, forced, 8)
    order = list(np.argsort(keys)[::-1])
    assert order == [3, 2, 4, 0, 1, 5]


# ----------------------------------------------------------------------------- counts
def test_kept_count_values_of_the_five_configs():
    assert oracle.kept_count(64, 0, np.float32(0.5)) == 32
    assert oracle.kept_count(128, 0, np.float32(0.3)) == 39      # 0.3f * 128 = 38.400002 -> 39
    assert oracle.kept_count(128, 0, np.float32(0.25)) == 32
    assert oracle.kept_count(64, 0, np.float32(0.4)) == 26       # 0.4f * 64 = 25.600000381 -> 26
    assert oracle.kept_count(64, 0, np.float32(1.0)) == 64
    assert oracle.kept_count(7, 0, np.float32(1e-6)) == 1        # never zero
    assert oracle.kept_count(64, 50, np.float32(0.5)) == 50      # forced tokens fill the quota first
    assert oracle.kept_count(5, 5, np.float32(0.2)) == 5


def test_total_kept_of_full_size_configs_closed_form():
    """Config 1: 64 blocks of 64: 2 sink blocks + 2 window blocks fully kept, 60 x 32.
    Config 2: 256 blocks of 128: 1 + 1 fully kept, 254 x 39.  Config 4: 1024 blocks: 2 x 128 + 1022 x 32."""
    assert oracle.plan([0, 4096], [0.5], block_size=64, n_obs=128, n_sink=128)[-1] == 4 * 64 + 60 * 32 == 2176
    assert oracle.plan([0, 32768], [0.3], block_size=128, n_obs=128, n_sink=128)[-1] == 2 * 128 + 254 * 39 == 10162
    assert oracle.plan([0, 131072], [0.25], block_size=128, n_obs=128, n_sink=128)[-1] == 2 * 128 + 1022 * 32 == 32960


def test_forced_mask():
    m = oracle.forced_mask(10, 3, 2)
    assert list(np.nonzero(m)[0]) == [0, 1, 7, 8, 9]
    assert oracle.forced_mask(5, 128, 128).all()
    assert oracle.forced_mask(256, 128, 128).all()
    assert not oracle.forced_mask(257, 128, 128).all()


# ----------------------------------------------------------------------------- brute force
def _brute_force_block(scores, forced, k):
    """All k-subsets; best = most forced tokens, then largest score sum under exact
    rational arithmetic, then lexicographically smallest index tuple."""
    from fractions import Fraction
    best, best_key = None, None
    for sub in itertools.combinations(range(len(scores)), k):
        key = (-sum(int(forced[i]) for i in sub), -sum(Fraction(float(scores[i])) for i in sub), sub)
        if best_key is None or key < best_key:
            best, best_key = sub, key
    return list(best)


@pytest.mark.parametrize("seed", range(12))
def test_selection_against_subset_enumeration(seed):
    rng = np.random.default_rng(seed)
    G = 8
    N = int(rng.integers(1, 40))
    n_obs, n_sink = int(rng.integers(0, 5)), int(rng.integers(0, 5))
    rho = np.float32(rng.uniform(0.05, 1.0))
    kind = seed % 4
    if kind == 0:
        s = rng.random(N).astype(np.float32)
    elif kind == 1:
        s = rng.integers(0, 3, N).astype(np.float32) / 4          # many exact ties
    elif kind == 2:
        s = np.zeros(N, dtype=np.float32)                         # all-zero block
    else:
        s = np.full(N, 0.25, dtype=np.float32)                    # all-equal block
    kept, new_cu = oracle.select_tokens(s, [0, N], [rho], block_size=G, n_obs=n_obs, n_sink=n_sink)
    f = oracle.forced_mask(N, n_obs, n_sink)
    want = []
    for lo in range(0, N, G):
        hi = min(N, lo + G)
        kg = oracle.kept_count(hi - lo, int(f[lo:hi].sum()), rho)
        want += [lo + i for i in _brute_force_block(s[lo:hi], f[lo:hi], kg)]
    assert list(kept) == want
    assert new_cu[-1] == len(want)


def test_selection_equals_tuple_sort_on_random_blocks():
    rng = np.random.default_rng(100)
    for _ in range(30):
        G = int(rng.choice([32, 64, 128]))
        N = int(rng.integers(1, 700))
        s = (rng.random(N) ** 8).astype(np.float32)
        s[rng.random(N) < 0.3] = 0.0
        rho = np.float32(rng.uniform(0.1, 1.0))
        kept, _ = oracle.select_tokens(s, [0, N], [rho], block_size=G, n_obs=100, n_sink=50)
        f = oracle.forced_mask(N, 100, 50)
        want = []
        for lo in range(0, N, G):
            hi = min(N, lo + G)
            kg = oracle.kept_count(hi - lo, int(f[lo:hi].sum()), rho)
            order = sorted(range(lo, hi), key=lambda i: (not f[i], -float(s[i]), i))
            want += sorted(order[:kg])
        assert list(kept) == want


# ----------------------------------------------------------------------------- invariants
def _random_batch(rng, R=6, maxlen=500):
    lengths = rng.integers(0, maxlen, R)
    lengths[rng.integers(0, R)] = 1
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    T = int(cu[-1])
    s = (rng.random(T) ** 6).astype(np.float32)
    ratio = rng.uniform(0.1, 1.0, R).astype(np.float32)
    return cu, s, ratio


@pytest.mark.parametrize("G", [32, 64, 128])
def test_kept_idx_shape_counts_and_forced(G):
    rng = np.random.default_rng(G)
    cu, s, ratio = _random_batch(rng)
    kept, new_cu = oracle.select_tokens(s, cu, ratio, block_size=G, n_obs=128, n_sink=128)
    assert (np.diff(kept) > 0).all() and kept.dtype == np.int32
    assert kept.min() >= 0 and kept.max() < cu[-1]
    np.testing.assert_array_equal(new_cu, oracle.plan(cu, ratio, block_size=G, n_obs=128, n_sink=128))
    keptset = set(kept.tolist())
    for r in range(len(cu) - 1):
        N = cu[r + 1] - cu[r]
        inside = kept[(kept >= cu[r]) & (kept < cu[r + 1])]
        assert len(inside) == new_cu[r + 1] - new_cu[r]
        counts = oracle.block_kept_counts(int(N), G, 128, 128, ratio[r])
        for g, kg in enumerate(counts):
            lo = cu[r] + g * G
            assert ((inside >= lo) & (inside < lo + G)).sum() == kg
        for i in np.nonzero(oracle.forced_mask(int(N), 128, 128))[0]:
            assert int(cu[r] + i) in keptset
        if N <= 256:
            assert len(inside) == N


def test_identity_at_keep_ratio_one():
    rng = np.random.default_rng(3)
    cu, s, _ = _random_batch(rng)
    kept, new_cu = oracle.select_tokens(s, cu, np.ones(len(cu) - 1, np.float32), block_size=64, n_obs=128, n_sink=128)
    np.testing.assert_array_equal(kept, np.arange(cu[-1], dtype=np.int32))
    np.testing.assert_array_equal(new_cu, cu)
    h = rng.integers(0, 65536, (cu[-1], 16)).astype(np.uint16)
    p = rng.integers(0, 1 << 30, cu[-1]).astype(np.int32)
    ho, po = oracle.compact(h, p, kept)
    np.testing.assert_array_equal(ho, h)
    np.testing.assert_array_equal(po, p)


def test_gather_scatter_round_trips():
    rng = np.random.default_rng(4)
    cu, s, ratio = _random_batch(rng)
    T = int(cu[-1])
    kept, _ = oracle.select_tokens(s, cu, ratio, block_size=32, n_obs=16, n_sink=8)
    h = rng.integers(0, 65536, (T, 24)).astype(np.uint16)
    hc, _ = oracle.compact(h, np.arange(T, dtype=np.int32), kept)
    np.testing.assert_array_equal(oracle.scatter(hc, kept, h), h)
    mask = np.zeros(T, bool)
    mask[kept] = True
    np.testing.assert_array_equal(oracle.scatter(hc, kept, np.zeros_like(h)), h * mask[:, None])
    x = rng.integers(0, 65536, hc.shape).astype(np.uint16)
    back, _ = oracle.compact(oracle.scatter(x, kept, h), np.arange(T, dtype=np.int32), kept)
    np.testing.assert_array_equal(back, x)
    # rows that were dropped keep their old state (Eq. 8)
    out = oracle.scatter(x, kept, h)
    np.testing.assert_array_equal(out[~mask], h[~mask])


def test_varlen_batch_equals_concatenated_single_runs():
    rng = np.random.default_rng(5)
    cu, s, ratio = _random_batch(rng, R=7)
    kept, new_cu = oracle.select_tokens(s, cu, ratio, block_size=64, n_obs=128, n_sink=128)
    parts = []
    for r in range(len(cu) - 1):
        a, b = int(cu[r]), int(cu[r + 1])
        kr, nc = oracle.select_tokens(s[a:b], [0, b - a], ratio[r:r + 1], block_size=64, n_obs=128, n_sink=128)
        parts.append(kr + a)
        assert nc[-1] == new_cu[r + 1] - new_cu[r]
    np.testing.assert_array_equal(kept, np.concatenate(parts))


def test_end_to_end_small_shrunk_configs_are_consistent():
    """sparsify() on shrunk versions of the five workloads: structure invariants hold together."""
    for idx, shrink in [(1, 8), (2, 64), (3, 64), (4, 256), (5, 16)]:
        w = workloads.make_config(idx, shrink=shrink, hidden_dim=32)
        q = workloads.bf16_bits_to_f32(w.q)
        k = workloads.bf16_bits_to_f32(w.k)
        out = oracle.sparsify(q, k, w.hidden, w.pos, w.cu_seqlens, w.keep_ratio,
                              block_size=w.block_size, n_obs=w.n_obs, n_sink=w.n_sink)
        assert (np.diff(out["kept_idx"]) > 0).all()
        np.testing.assert_array_equal(out["new_cu_seqlens"],
                                      oracle.plan(w.cu_seqlens, w.keep_ratio, block_size=w.block_size,
                                                  n_obs=w.n_obs, n_sink=w.n_sink))
        np.testing.assert_array_equal(out["hidden_out"], w.hidden[out["kept_idx"]])
        np.testing.assert_array_equal(out["pos_out"], w.pos[out["kept_idx"]])
        for r in range(w.num_seqs):
            a, b = w.cu_seqlens[r], w.cu_seqlens[r + 1]
            assert abs(out["scores64"][a:b].sum() - 1.0) < 1e-10


def test_higher_score_never_loses_to_lower_score_in_same_block():
    rng = np.random.default_rng(6)
    N, G = 1000, 64
    s = rng.random(N).astype(np.float32)
    kept, _ = oracle.select_tokens(s, [0, N], [np.float32(0.3)], block_size=G, n_obs=0, n_sink=0)
    mask = np.zeros(N, bool)
    mask[kept] = True
    for lo in range(0, N, G):
        blk = slice(lo, min(N, lo + G))
        if (~mask[blk]).any():
            assert s[blk][mask[blk]].min() >= s[blk][~mask[blk]].max()


# ----------------------------------------------------------------------------- paper's top-p rule (Eq. 5-6)
def test_top_p_keeps_minimal_prefix_with_mass_at_least_p():
    rng = np.random.default_rng(7)
    N, G = 1000, 64
    o = rng.random(N) ** 10
    o /= o.sum()
    for p in [0.5, 0.9, 0.99]:
        mask = oracle.select_blocks_top_p(o, p, block_size=G, n_obs=0, n_sink=0)
        b = oracle.block_mass(o, N, G)
        kb = np.array([mask[lo] for lo in range(0, N, G)])
        assert b[kb].sum() >= p * b.sum() - 1e-15            # Eq. 6: dropped mass <= 1 - p
        # minimal: dropping the smallest kept block falls below p
        assert b[kb].sum() - b[kb].min() < p * b.sum()
        # greedy: every kept block outweighs every dropped block
        if (~kb).any():
            assert b[kb].min() >= b[~kb].max()


def test_top_p_forces_sinks_and_window_and_p1_keeps_all_positive_mass():
    rng = np.random.default_rng(8)
    N, G = 700, 32
    o = rng.random(N)
    o[100:400] = 0.0
    o /= o.sum()
    m = oracle.select_blocks_top_p(o, 0.3, block_size=G, n_obs=50, n_sink=20)
    assert m[:20].all() and m[-50:].all()
    m1 = oracle.select_blocks_top_p(o, 1.0, block_size=G, n_obs=0, n_sink=0)
    b = oracle.block_mass(o, N, G)
    for g, lo in enumerate(range(0, N, G)):
        if b[g] > 0:
            assert m1[lo]


# ----------------------------------------------------------------------------- top-p on quantised scores
def _brute_force_top_p(mass, p):
    """Smallest k, then (descending mass, lower index first) prefix -- by enumeration of k."""
    nb = len(mass)
    order = sorted(range(nb), key=lambda g: (-float(mass[g]), g))
    total = 0.0
    for g in order:
        total += float(mass[g])
    run = 0.0
    for k, g in enumerate(order, 1):
        run += float(mass[g])
        if run >= float(np.float32(p)) * total:
            return set(order[:k])
    return set(order)


@pytest.mark.parametrize("seed", range(6))
def test_quantised_top_p_blocks_against_enumeration(seed):
    rng = np.random.default_rng(100 + seed)
    nb = int(rng.integers(1, 40))
    mass = (rng.random(nb) ** 6).astype(np.float32)
    if seed % 2:
        mass[rng.integers(0, nb, size=nb // 2)] = mass[0]      # ties
    if seed == 3:
        mass[:] = 0.0                                            # nothing to go by: first block only
    for p in [0.1, 0.5, 0.9, 0.99, 1.0]:
        keep = oracle.top_p_kept_blocks(mass, p)
        assert set(np.nonzero(keep)[0]) == _brute_force_top_p(mass, p)
        kept_mass = float(mass[keep].astype(np.float64).sum())
        assert kept_mass >= float(np.float32(p)) * float(mass.astype(np.float64).sum()) * (1 - 1e-12)   # Eq. 6
        if keep.sum() > 1:   # minimal: without its lightest kept block the set misses p
            assert kept_mass - float(mass[keep].min()) < float(np.float32(p)) * float(mass.astype(np.float64).sum())


def test_chunked_running_sum_against_exact_rationals_and_its_shape():
    """The running sum that the top-p threshold is taken on: exact where every partial sum is
    representable (checked against rational arithmetic at every position, across chunk borders),
    the plain sequential sum up to one chunk, never decreasing, within n * 2^-53 of the exact sum
    otherwise -- and a hand case in which the two-level shape shows: a chunk's small values are
    added among themselves before they meet the large earlier total."""
    from fractions import Fraction
    rng = np.random.default_rng(21)
    # (a) dyadic values with few significant bits: every partial sum is exact in double
    v = (rng.integers(0, 1 << 12, size=300) / 1024.0).astype(np.float32)
    run = oracle.chunked_running_sum(v)
    exact, acc = [], Fraction(0)
    for x in v:
        acc += Fraction(float(x))
        exact.append(acc)
    assert all(Fraction(float(r)) == e for r, e in zip(run, exact))
    # (b) up to one chunk: the sequential double sum, bit for bit
    w = (rng.random(64) ** 9).astype(np.float32)
    np.testing.assert_array_equal(oracle.chunked_running_sum(w), np.add.accumulate(w.astype(np.float64)))
    # (c) random heavy-tailed values over several chunks: monotone, close to exact, last = total
    z = np.exp(rng.standard_normal(1000) * 8 - 20).astype(np.float32)
    run = oracle.chunked_running_sum(z)
    assert (np.diff(run) >= 0).all() and len(run) == 1000
    acc = Fraction(0)
    for k, x in enumerate(z):
        acc += Fraction(float(x))
        assert abs(Fraction(float(run[k])) - acc) <= acc * Fraction(k + 1, 2 ** 53)
    # (d) hand case: 1, then 63 zeros | 64 values of 2^-54.  One after the other each 2^-54 would be
    # rounded away against 1 (ties to even); inside their chunk they add up to 2^-48 first.
    h = np.zeros(128, np.float32)
    h[0] = 1.0
    h[64:] = 2.0 ** -54
    run = oracle.chunked_running_sum(h)
    assert run[63] == 1.0 and run[64] == 1.0 and run[127] == 1.0 + 2.0 ** -48
    assert np.add.accumulate(h.astype(np.float64))[-1] == 1.0          # (the sequential sum differs)
    assert len(oracle.chunked_running_sum(np.zeros(0, np.float32))) == 0


def test_top_p_threshold_across_chunk_borders_against_exact_rationals():
    """More blocks than one chunk of the running sum, masses whose sums are exact: the kept set is
    the one rational arithmetic gives, for thresholds that fall before, on and after a chunk border."""
    from fractions import Fraction
    rng = np.random.default_rng(22)
    nb = 200
    mass = (rng.integers(1, 1 << 10, size=nb) / 256.0).astype(np.float32)
    order = sorted(range(nb), key=lambda g: (-float(mass[g]), g))
    total = sum(Fraction(float(m)) for m in mass)
    for p in [0.05, 0.3, 0.5, 0.75, 0.9, 0.999, 1.0]:
        thr = Fraction(float(np.float32(p))) * total
        # (p * total in double, as the oracle takes it, equals the rational product here: few bits)
        acc, want = Fraction(0), None
        for k, g in enumerate(order, 1):
            acc += Fraction(float(mass[g]))
            if acc >= Fraction(float(np.float32(p)) * float(total)):
                want = set(order[:k])
                break
        keep = oracle.top_p_kept_blocks(mass, p)
        assert set(np.nonzero(keep)[0]) == want, p
    ks = [int(oracle.top_p_kept_blocks(mass, p).sum()) for p in (0.3, 0.5, 0.75, 0.9)]
    assert ks == sorted(ks) and ks[0] < 64 < ks[-1]          # thresholds on both sides of the first border


def test_block_mass_f32_is_the_rounded_exact_sum():
    rng = np.random.default_rng(9)
    s = (rng.random(1000) ** 8).astype(np.float32)
    b = oracle.block_mass_f32(s, 1000, 64)
    from fractions import Fraction
    for g, lo in enumerate(range(0, 1000, 64)):
        exact = sum(Fraction(float(v)) for v in s[lo:lo + 64])
        assert abs(Fraction(float(b[g])) - exact) <= Fraction(float(np.spacing(b[g]))) / 2 + exact * Fraction(1, 2 ** 50)
    assert len(b) == 16 and b.dtype == np.float32


def test_top_p_block_keys_order():
    b = np.array([0.5, 0.25, 0.5, 0.0, 1.0], dtype=np.float32)
    order = np.argsort(oracle.top_p_block_keys(b))[::-1]
    assert list(order) == [4, 0, 2, 1, 3]          # descending mass, equal masses: lower block first


def test_select_tokens_top_p_shape_forced_and_consistency_with_fp64_rule():
    rng = np.random.default_rng(10)
    lengths = [700, 0, 64, 1, 333]
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    o = rng.random(cu[-1]) ** 12
    for r in range(len(lengths)):
        if lengths[r]:
            o[cu[r]:cu[r + 1]] /= o[cu[r]:cu[r + 1]].sum()
    s32 = oracle.quantise_scores(o)
    top_p = np.array([0.9, 0.5, 0.99, 0.7, 0.6], dtype=np.float32)
    G, n, A = 32, 40, 8
    kept, new_cu = oracle.select_tokens_top_p(s32, cu, top_p, block_size=G, n_obs=n, n_sink=A)
    assert (np.diff(kept) > 0).all() and kept.dtype == np.int32
    assert new_cu[-1] == len(kept) and new_cu[0] == 0
    for r, N in enumerate(lengths):
        mine = kept[new_cu[r]:new_cu[r + 1]] - cu[r]
        assert ((mine >= 0) & (mine < max(N, 1))).all()
        if N == 0:
            assert len(mine) == 0
            continue
        mask = np.zeros(N, bool)
        mask[mine] = True
        assert mask[:A].all() and mask[max(0, N - n):].all()                 # sinks and window
        # non-forced tokens are kept or dropped block by block
        f = oracle.forced_mask(N, n, A)
        for lo in range(0, N, G):
            blk = mask[lo:lo + G][~f[lo:lo + G]]
            assert blk.all() or not blk.any()
        # same decision as the fp64 statement of the rule (scores here are far from any tie)
        ref = oracle.select_blocks_top_p(s32[cu[r]:cu[r + 1]].astype(np.float64), float(top_p[r]),
                                         block_size=G, n_obs=n, n_sink=A)
        np.testing.assert_array_equal(mask, ref)
    # p = 1 keeps every block of positive mass
    kept1, _ = oracle.select_tokens_top_p(s32, cu, np.ones(5, np.float32), block_size=G, n_obs=0, n_sink=0)
    m1 = np.zeros(cu[-1], bool)
    m1[kept1] = True
    for r, N in enumerate(lengths):
        for lo in range(0, N, G):
            blk = slice(cu[r] + lo, cu[r] + min(N, lo + G))
            if s32[blk].sum() > 0:
                assert m1[blk].all()


# ----------------------------------------------------------------------------- index maps across drop layers
def test_compose_index_identities_and_two_level_round_trip():
    rng = np.random.default_rng(11)
    T, d = 500, 6
    H = rng.standard_normal((T, d)).astype(np.float32)
    idx1 = np.sort(rng.choice(T, size=300, replace=False)).astype(np.int32)        # first drop
    idx2 = np.sort(rng.choice(300, size=120, replace=False)).astype(np.int32)      # second drop, on the compacted stream
    idx3 = np.sort(rng.choice(120, size=50, replace=False)).astype(np.int32)
    c12 = oracle.compose_index(idx1, idx2)
    assert c12.dtype == np.int32 and (np.diff(c12) > 0).all() and set(c12) <= set(idx1)   # nested, still ascending
    np.testing.assert_array_equal(oracle.compose_index(np.arange(T), idx1), idx1)          # identity on the left
    np.testing.assert_array_equal(oracle.compose_index(idx1, np.arange(300)), idx1)        # ... and on the right
    np.testing.assert_array_equal(oracle.compose_index(oracle.compose_index(idx1, idx2), idx3),
                                  oracle.compose_index(idx1, oracle.compose_index(idx2, idx3)))   # associative
    # compacting twice == compacting once through the composed map
    h1, _ = oracle.compact(H, np.arange(T), idx1)
    h2, _ = oracle.compact(h1, np.arange(300), idx2)
    h12, _ = oracle.compact(H, np.arange(T), c12)
    np.testing.assert_array_equal(h2, h12)
    # reconstitution through two levels == one scatter through the composed map (dropped rows keep their state)
    new2 = h2 + 1.0
    lvl1 = oracle.scatter(new2, idx2, h1)
    full_two_step = oracle.scatter(lvl1, idx1, H)
    full_direct = oracle.scatter(new2, c12, H)
    np.testing.assert_array_equal(full_two_step, full_direct)
    np.testing.assert_array_equal(oracle.retained_lengths([0, 5, 5, 12]), [5, 0, 7])


# ----------------------------------------------------------------------------- serving-side metadata
def test_kv_slot_mapping_and_seqused_small_cases():
    # two requests, KV blocks of 4 slots; request 0 kept positions 0,1,5,6; request 1 kept 2,9
    bt = np.array([[7, 3, 0], [2, 5, 9]], dtype=np.int32)
    slots = oracle.kv_slot_mapping([0, 1, 5, 6, 2, 9], [0, 4, 6], bt, 4)
    np.testing.assert_array_equal(slots, [28, 29, 13, 14, 10, 37])   # 7*4+0, 7*4+1, 3*4+1, 3*4+2, 2*4+2, 9*4+1
    # identity block table and no drop: slot == position offset by the request's base
    N = 37
    bt = np.arange(10, dtype=np.int32)[None, :]
    np.testing.assert_array_equal(oracle.kv_slot_mapping(np.arange(N), [0, N], bt, 4), np.arange(N))
    # distinct tokens of a request never share a slot when its block table has distinct blocks
    rng = np.random.default_rng(12)
    bt = rng.permutation(64).astype(np.int32).reshape(2, 32)
    pos = np.concatenate([np.sort(rng.choice(500, 200, replace=False)), np.sort(rng.choice(500, 123, replace=False))])
    s = oracle.kv_slot_mapping(pos, [0, 200, 323], bt, 16)
    assert len(set(s.tolist())) == 323
    np.testing.assert_array_equal(oracle.seqused([100, 7], [1030, 9], [1024, 8]), [106, 8])


def test_seqused_per_layer_hand_worked_history():
    """Eq. 17 on a history worked by hand: 6 layers, drops at layers 1 and 3.  Request 0: prompt of
    1000 tokens, 400 kept at layer 1, 150 at layer 3, 5 tokens decoded since; request 1: prompt of
    8, nothing dropped (8, 8), 1 token decoded.  Layers up to and including the first drop layer
    see the whole prompt; a drop takes effect in the layers after it."""
    got = oracle.seqused_per_layer([1, 3], [[400, 8], [150, 8]], [1005, 9], [1000, 8], 6)
    np.testing.assert_array_equal(got, [[1005, 9], [1005, 9], [405, 9], [405, 9], [155, 9], [155, 9]])
    # no drop events: every layer sees the whole KV length
    got = oracle.seqused_per_layer([], np.zeros((0, 2)), [1005, 9], [1000, 8], 3)
    np.testing.assert_array_equal(got, [[1005, 9]] * 3)
    # each layer agrees with the single-layer form, and lengths never grow with depth
    rng = np.random.default_rng(13)
    orig = rng.integers(100, 5000, size=7)
    hist = np.sort(rng.integers(1, 100, size=(3, 7)), axis=0)[::-1] * orig // 100 + 1
    hist = np.minimum.accumulate(np.minimum(hist, orig), axis=0)
    kv = orig + rng.integers(0, 50, size=7)
    table = oracle.seqused_per_layer([0, 4, 9], hist, kv, orig, 12)
    for layer in range(12):
        k = max([i for i, lk in enumerate([0, 4, 9]) if lk < layer], default=None)
        s = orig if k is None else hist[k]
        np.testing.assert_array_equal(table[layer], oracle.seqused(s, kv, orig))
    assert (np.diff(table.astype(np.int64), axis=0) <= 0).all()


def test_keep_mask_hand_case_and_agreement_with_the_selection():
    np.testing.assert_array_equal(oracle.keep_mask([0, 3, 4, 9], 11), [1, 0, 0, 1, 1, 0, 0, 0, 0, 1, 0])
    np.testing.assert_array_equal(oracle.keep_mask([], 3), [0, 0, 0])
    rng = np.random.default_rng(14)
    cu = np.array([0, 300, 300, 1000])
    s32 = rng.random(1000).astype(np.float32)
    kept, new_cu = oracle.select_tokens(s32, cu, [0.3, 0.5, 0.7], block_size=64, n_obs=32, n_sink=8)
    m = oracle.keep_mask(kept, 1000)
    assert int(m.sum()) == len(kept) == new_cu[-1]
    np.testing.assert_array_equal(np.nonzero(m)[0], kept)                       # the list is the mask's support, ascending
    for r in range(3):
        assert int(m[cu[r]:cu[r + 1]].sum()) == new_cu[r + 1] - new_cu[r]

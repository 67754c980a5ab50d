"""GPU parity: every C-ABI entry point against the fp64 CPU oracle on the same
seeded inputs.  Integer, index and byte outputs must be bit-exact; scores agree
within 1e-2 relative (bf16 inputs) plus the 2^-64 floor."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_06221_amd as up
import workloads
from gpu_util import DeviceBatch, dev_bf16, host_bits, oracle_run, score_margin_report

pytestmark = pytest.mark.gpu

SCORE_RTOL = 1e-2          # bf16 inputs (tolerance stated for this build)
SCORE_ATOL = 2.0 ** -64    # the floor


def _say(*a):
    print(*a, flush=True)


# ----------------------------------------------------------------------------- compact / scatter
@pytest.mark.parametrize("d,dtype", [(8, "bf16"), (24, "bf16"), (1024, "bf16"), (4096, "bf16"), (5120, "bf16"),
                                      (520, "bf16"), (4, "f32"), (1000, "f32")])
def test_compact_and_scatter_are_bit_exact(d, dtype):
    _say("compact/scatter d", d, dtype)
    rng = np.random.default_rng(d)
    T = 3000
    mask = rng.random(T) < 0.37
    mask[[0, T - 1]] = True
    kept = np.nonzero(mask)[0].astype(np.int32)
    K = len(kept)
    pos = rng.integers(0, 1 << 30, T).astype(np.int32)
    if dtype == "bf16":
        h = rng.integers(0, 65536, (T, d)).astype(np.uint16)
        hd = dev_bf16(h)
        out = torch.zeros((K + 8, d), dtype=torch.bfloat16, device="cuda")
        hdt = up.UP_BF16
        to_host = host_bits
    else:
        h = rng.integers(0, 1 << 32, (T, d), dtype=np.uint64).astype(np.uint32)
        hd = torch.from_numpy(h.view(np.int32)).cuda()
        out = torch.zeros((K + 8, d), dtype=torch.int32, device="cuda")
        hdt = up.UP_F32
        to_host = lambda t: t.cpu().numpy().view(np.uint32)
    p = up.make_params(num_seqs=1, total_tokens=T, block_size=64, hidden_dim=d, hidden_dtype=hdt)
    kd = torch.from_numpy(kept).cuda()
    pd = torch.from_numpy(pos).cuda()
    po = torch.full((K + 8,), -5, dtype=torch.int32, device="cuda")
    up.uniprefill_compact(p, hd, pd, kd, K, out, po)
    torch.cuda.synchronize()
    want_h, want_p = oracle.compact(h, pos, kept)
    np.testing.assert_array_equal(to_host(out[:K]), want_h)
    np.testing.assert_array_equal(po[:K].cpu().numpy(), want_p)
    assert (po[K:] == -5).all() and (out[K:] == 0).all()
    # scatter into a different full tensor: kept rows replaced, others untouched
    full = rng.integers(0, 60000, (T, d)).astype(h.dtype)
    fd = dev_bf16(full) if dtype == "bf16" else torch.from_numpy(full.view(np.int32)).cuda()
    up.uniprefill_scatter(p, out, kd, K, fd)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_host(fd), oracle.scatter(want_h, kept, full))
    # no position ids: both NULL is legal
    up.uniprefill_compact(p, hd, None, kd, K, out, None)
    torch.cuda.synchronize()


def test_compact_with_padded_row_stride_and_empty_selection():
    rng = np.random.default_rng(0)
    T, d, stride = 500, 64, 96
    h = rng.integers(0, 65536, (T, stride)).astype(np.uint16)
    kept = np.arange(0, T, 3, dtype=np.int32)
    p = up.make_params(num_seqs=1, total_tokens=T, block_size=32, hidden_dim=d, hidden_row_stride=stride)
    out = torch.zeros((len(kept), stride), dtype=torch.bfloat16, device="cuda")
    up.uniprefill_compact(p, dev_bf16(h), None, torch.from_numpy(kept).cuda(), len(kept), out, None)
    got = host_bits(out)
    np.testing.assert_array_equal(got[:, :d], h[kept, :d])
    assert (got[:, d:] == 0).all()          # bytes beyond hidden_dim are never written
    up.uniprefill_compact(p, dev_bf16(h), None, torch.from_numpy(kept).cuda(), 0, out, None)
    torch.cuda.synchronize()


def test_counted_copies_never_write_past_the_capacity():
    """The row count on the device may exceed the capacity the caller sized its buffers for
    (a stale or foreign counter): the copies stop at the capacity, whose launch is rounded up to
    whole work-groups (4 rows, 256 index entries)."""
    _say("counted copies clamp to the capacity")
    rng = np.random.default_rng(7)
    T, d, cap = 300, 64, 37                                  # 37 % 4 != 0
    h = rng.integers(0, 65536, (T, d)).astype(np.uint16)
    pos = rng.integers(0, 1 << 20, T).astype(np.int32)
    kept = np.sort(rng.choice(T, 64, replace=False)).astype(np.int32)
    p = up.make_params(num_seqs=1, total_tokens=T, block_size=32, hidden_dim=d)
    count = torch.tensor([50], dtype=torch.int32, device="cuda")     # more than the capacity
    out = torch.full((cap + 8, d), -7.0, dtype=torch.bfloat16, device="cuda")
    pos_out = torch.full((cap + 8,), -77, dtype=torch.int32, device="cuda")
    kd = torch.from_numpy(kept).cuda()
    up.uniprefill_compact_counted(p, dev_bf16(h), torch.from_numpy(pos).cuda(), kd, count, cap, out, pos_out)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host_bits(out[:cap]), oracle.compact(h, pos, kept[:cap])[0])
    np.testing.assert_array_equal(pos_out[:cap].cpu().numpy(), pos[kept[:cap]])
    assert (out[cap:] == -7.0).all() and (pos_out[cap:] == -77).all()
    # index-map composition: capacity 37 of a 256-entry launch, device count above it
    outer = rng.integers(0, 1 << 20, T).astype(np.int32)
    composed = torch.full((cap + 300,), -77, dtype=torch.int32, device="cuda")
    up.uniprefill_compose_index(torch.from_numpy(outer).cuda(), T, kd, count, cap, composed)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(composed[:cap].cpu().numpy(), oracle.compose_index(outer, kept[:cap]))
    assert (composed[cap:] == -77).all()
    # a device count below the capacity still wins
    count.fill_(5)
    out.fill_(-7.0)
    up.uniprefill_compact_counted(p, dev_bf16(h), None, kd, count, cap, out, None)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host_bits(out[:5]), h[kept[:5]])
    assert (out[5:] == -7.0).all()


# ----------------------------------------------------------------------------- select
def _select_case(rng, G, n_obs, n_sink, R, maxlen, kind):
    lengths = rng.integers(0, maxlen, R)
    lengths[rng.integers(0, R)] = 1
    lengths[rng.integers(0, R)] = 0
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    T = int(cu[-1])
    if kind == "random":
        s = (rng.random(T) ** 6).astype(np.float32)
    elif kind == "ties":
        s = (rng.integers(0, 4, T) / 8).astype(np.float32)
    elif kind == "zeros":
        s = np.zeros(T, np.float32)
    else:  # heavy tail with floored zeros and denormal-range values
        s = np.exp(rng.standard_normal(T) * 30 - 40).astype(np.float32)
        s[rng.random(T) < 0.5] = 0.0
    ratio = rng.uniform(0.05, 1.0, R).astype(np.float32)
    ratio[0] = 1.0
    return cu, s, ratio


@pytest.mark.parametrize("G", [32, 64, 128])
@pytest.mark.parametrize("kind", ["random", "ties", "zeros", "heavy"])
def test_select_is_bit_exact_on_given_scores(G, kind):
    _say("select", G, kind)
    rng = np.random.default_rng(G * 7 + len(kind))
    for n_obs, n_sink, R, maxlen in [(128, 128, 9, 2000), (16, 8, 30, 300), (1, 0, 5, 700), (512, 200, 6, 3000)]:
        cu, s, ratio = _select_case(rng, G, n_obs, n_sink, R, maxlen, kind)
        T = int(cu[-1])
        p = up.make_params(num_seqs=R, total_tokens=T, block_size=G, n_obs=n_obs, n_sink=n_sink)
        want_idx, want_cu = oracle.select_tokens(s, cu, ratio, block_size=G, n_obs=n_obs, n_sink=n_sink)
        K = len(want_idx)
        kept = torch.full((K + 16,), -3, dtype=torch.int32, device="cuda")
        new_cu = torch.full((R + 1 + 16,), -3, dtype=torch.int32, device="cuda")
        up.uniprefill_select(p, torch.from_numpy(s).cuda(), torch.from_numpy(cu).cuda(), cu,
                             torch.from_numpy(ratio).cuda(), ratio, kept, new_cu)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(new_cu[:R + 1].cpu().numpy(), want_cu)
        np.testing.assert_array_equal(kept[:K].cpu().numpy(), want_idx)
        assert (kept[K:] == -3).all() and (new_cu[R + 1:] == -3).all()


def test_select_many_sequences_prefix_scan():
    """More than 1024 sequences: the device-side offsets scan in several rounds."""
    rng = np.random.default_rng(5)
    R = 2500
    lengths = rng.integers(0, 70, R)
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    T = int(cu[-1])
    s = rng.random(T).astype(np.float32)
    ratio = rng.uniform(0.1, 1.0, R).astype(np.float32)
    p = up.make_params(num_seqs=R, total_tokens=T, block_size=32, n_obs=4, n_sink=2)
    want_idx, want_cu = oracle.select_tokens(s, cu, ratio, block_size=32, n_obs=4, n_sink=2)
    kept = torch.zeros(len(want_idx), dtype=torch.int32, device="cuda")
    new_cu = torch.zeros(R + 1, dtype=torch.int32, device="cuda")
    up.uniprefill_select(p, torch.from_numpy(s).cuda(), torch.from_numpy(cu).cuda(), cu,
                         torch.from_numpy(ratio).cuda(), ratio, kept, new_cu)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(new_cu.cpu().numpy(), want_cu)
    np.testing.assert_array_equal(kept.cpu().numpy(), want_idx)


# ----------------------------------------------------------------------------- score
def _q_f32(w):
    """q as the oracle reads it: only window rows are upcast (the rest is NaN filler)."""
    from gpu_util import _LazyQ
    return _LazyQ(w.q)


def _score_close(got, want32):
    want = want32.astype(np.float64)
    err = np.abs(got.astype(np.float64) - want)
    ok = err <= SCORE_RTOL * want + SCORE_ATOL
    return ok.all(), (err / np.maximum(want, 1e-300))[want > 0].max() if (want > 0).any() else 0.0


@pytest.mark.parametrize("case", [
    dict(lengths=[700], Hq=8, Hkv=8, n_obs=128),
    dict(lengths=[1, 5, 130, 0, 257, 1000, 64], Hq=8, Hkv=2, n_obs=128),
    dict(lengths=[3000, 2], Hq=32, Hkv=8, n_obs=128),
    dict(lengths=[1500], Hq=40, Hkv=8, n_obs=128),
    dict(lengths=[900, 77], Hq=4, Hkv=4, n_obs=32),
    dict(lengths=[600], Hq=2, Hkv=1, n_obs=512),
    dict(lengths=[2100], Hq=16, Hkv=2, n_obs=200),
    dict(lengths=[3000, 500], Hq=2, Hkv=2, n_obs=1024),       # the largest window
    dict(lengths=[1300, 1, 70], Hq=6, Hkv=2, n_obs=1),        # a single query row
])
def test_scores_match_oracle(case):
    _say("score", case)
    w = workloads.make_custom(name="score", seed=11, lengths=case["lengths"], keep_ratio=[0.5] * len(case["lengths"]),
                              hidden_dim=8, num_q_heads=case["Hq"], num_kv_heads=case["Hkv"], block_size=64,
                              n_obs=case["n_obs"])
    b = DeviceBatch(w)
    b.score()
    got = b.results()["scores"]
    want = oracle.quantise_scores(oracle.importance_scores(
        _q_f32(w), workloads.bf16_bits_to_f32(w.k), w.cu_seqlens, n_obs=w.n_obs))
    ok, worst = _score_close(got, want)
    _say("  worst relative score error", worst)
    assert ok
    assert b.canaries_intact()
    for r in range(w.num_seqs):
        a, e = w.cu_seqlens[r], w.cu_seqlens[r + 1]
        if e > a:
            assert abs(float(got[a:e].astype(np.float64).sum()) - 1.0) < 1e-4


@pytest.mark.parametrize("n_obs,Hq,Hkv", [(128, 8, 2), (200, 6, 2), (32, 4, 4)])
def test_scores_many_short_sequences_use_the_wide_work_groups(n_obs, Hq, Hkv):
    """230+ sequences push the launch geometry to 512-key work-groups (16 waves) although every
    sequence is short: lengths around the tile, unit and key-block boundaries, empty ones included."""
    special = [0, 1, 2, 31, 32, 33, 63, 127, 128, 129, 255, 256, 257, 383, 511, 512, 513, 640, 1023, 1024, 1025, 1500]
    rng = np.random.default_rng(5)
    lengths = special + [int(x) for x in rng.integers(1, 700, size=230 - len(special))]
    rng.shuffle(lengths)
    _say("score many sequences", n_obs, Hq, Hkv, "T", sum(lengths))
    w = workloads.make_custom(name="many", seed=21, lengths=lengths, keep_ratio=[0.4] * len(lengths),
                              hidden_dim=8, num_q_heads=Hq, num_kv_heads=Hkv, block_size=64, n_obs=n_obs)
    assert w.total_tokens // 512 + w.num_seqs >= 224      # the geometry this test is about
    b = DeviceBatch(w)
    b.score()
    got = b.results()["scores"]
    want = oracle.quantise_scores(oracle.importance_scores(
        _q_f32(w), workloads.bf16_bits_to_f32(w.k), w.cu_seqlens, n_obs=w.n_obs))
    ok, worst = _score_close(got, want)
    _say("  worst relative score error", worst)
    assert ok
    assert b.canaries_intact()


def test_fused_many_short_sequences_bit_exact():
    rng = np.random.default_rng(6)
    lengths = [0, 1, 33, 127, 129, 300, 511, 512, 513, 1025, 2049] + [int(x) for x in rng.integers(1, 900, size=225)]
    _say("fused many sequences T", sum(lengths))
    ratios = [float(x) for x in rng.uniform(0.2, 0.9, size=len(lengths))]
    w = workloads.make_custom(name="manyf", seed=22, lengths=lengths, keep_ratio=ratios, hidden_dim=64,
                              num_q_heads=8, num_kv_heads=2, block_size=128, n_obs=128)
    assert w.total_tokens // 512 + w.num_seqs >= 224
    b = DeviceBatch(w)
    b.fused()
    _assert_fused_exact(w, b, oracle_run(w))


# fp32 operands: tolerance stated for this build; what the arithmetic gives is derived in the design notes
SCORE_RTOL_F32 = 1e-5


def _f32_operands(w, seed):
    """float32 q and k that are not bf16-representable; q rows outside the window are NaN."""
    rng = np.random.default_rng(seed)
    k = rng.standard_normal(w.k.shape, dtype=np.float32)
    q = np.full(w.q.shape, np.nan, dtype=np.float32)
    for r in range(w.num_seqs):
        a, e = int(w.cu_seqlens[r]), int(w.cu_seqlens[r + 1])
        n_eff = min(w.n_obs, e - a)
        q[e - n_eff:e] = rng.standard_normal((n_eff,) + w.q.shape[1:], dtype=np.float32)
    return q, k


@pytest.mark.parametrize("case", [
    dict(lengths=[700], Hq=8, Hkv=8, n_obs=128),
    dict(lengths=[1, 5, 130, 0, 257, 1000, 64], Hq=8, Hkv=2, n_obs=128),
    dict(lengths=[2100, 300], Hq=12, Hkv=4, n_obs=200),
])
def test_scores_from_fp32_operands_match_oracle(case):
    _say("score fp32", case)
    w = workloads.make_custom(name="f32", seed=12, lengths=case["lengths"], keep_ratio=[0.5] * len(case["lengths"]),
                              hidden_dim=8, num_q_heads=case["Hq"], num_kv_heads=case["Hkv"], block_size=64,
                              n_obs=case["n_obs"])
    q32, k32 = _f32_operands(w, 31)
    b = DeviceBatch(w, qk_f32=(q32, k32))
    b.score()
    got = b.results()["scores"].astype(np.float64)
    want = oracle.quantise_scores(oracle.importance_scores(q32, k32, w.cu_seqlens, n_obs=w.n_obs)).astype(np.float64)
    err = np.abs(got - want)
    worst = (err / np.maximum(want, 1e-300))[want > 0].max()
    _say("  worst relative score error", worst)
    assert (err <= SCORE_RTOL_F32 * want + SCORE_ATOL).all()
    assert b.canaries_intact()


def test_fused_from_fp32_operands_bit_exact():
    _say("fused fp32")
    w = workloads.make_custom(name="f32f", seed=13, lengths=[1500, 40, 777], keep_ratio=[0.3, 0.5, 0.7],
                              hidden_dim=64, num_q_heads=8, num_kv_heads=2, block_size=64, n_obs=128)
    q32, k32 = _f32_operands(w, 32)
    b = DeviceBatch(w, qk_f32=(q32, k32))
    b.fused()
    ref = oracle.sparsify(q32, k32, w.hidden, w.pos, w.cu_seqlens, w.keep_ratio, block_size=w.block_size,
                          n_obs=w.n_obs, n_sink=w.n_sink)
    res = b.results()
    err = np.abs(res["scores"].astype(np.float64) - ref["scores"].astype(np.float64))
    assert (err <= SCORE_RTOL_F32 * ref["scores"] + SCORE_ATOL).all()
    np.testing.assert_array_equal(res["new_cu_seqlens"], ref["new_cu_seqlens"])
    np.testing.assert_array_equal(res["kept_idx"], ref["kept_idx"])
    np.testing.assert_array_equal(res["pos_out"], ref["pos_out"])
    np.testing.assert_array_equal(res["hidden_out"], ref["hidden_out"])
    assert b.canaries_intact()


def _many_lengths(seed, count):
    special = [0, 1, 2, 31, 32, 33, 127, 128, 129, 255, 256, 257, 511, 512, 513, 1023, 1025, 1500]
    rng = np.random.default_rng(seed)
    lengths = special + [int(x) for x in rng.integers(1, 700, size=count - len(special))]
    rng.shuffle(lengths)
    return lengths


@pytest.mark.parametrize("head_dim", [64, 256])
@pytest.mark.parametrize("case", [
    dict(lengths=[1, 5, 130, 0, 257, 1000, 64], Hq=8, Hkv=2, n_obs=128),
    dict(lengths=[2100, 300], Hq=12, Hkv=4, n_obs=200),
    dict(lengths=[5000], Hq=4, Hkv=1, n_obs=32),
    dict(lengths="many", Hq=8, Hkv=2, n_obs=128),
])
def test_scores_head_dims_64_and_256_match_oracle(head_dim, case):
    """Head dimensions other than 128: four (64) or sixteen (256) matrix steps per tile, the
    latter in 256-key work-groups only; "many" reaches the 512-key work-groups for 64."""
    lengths = _many_lengths(7, 230) if case["lengths"] == "many" else case["lengths"]
    _say("score head_dim", head_dim, case if case["lengths"] != "many" else "many sequences")
    w = workloads.make_custom(name="hd", seed=14, lengths=lengths, keep_ratio=[0.5] * len(lengths),
                              hidden_dim=8, num_q_heads=case["Hq"], num_kv_heads=case["Hkv"], block_size=64,
                              n_obs=case["n_obs"], head_dim=head_dim)
    b = DeviceBatch(w)
    b.score()
    got = b.results()["scores"]
    want = oracle.quantise_scores(oracle.importance_scores(
        _q_f32(w), workloads.bf16_bits_to_f32(w.k), w.cu_seqlens, n_obs=w.n_obs))
    ok, worst = _score_close(got, want)
    _say("  worst relative score error", worst)
    assert ok
    assert b.canaries_intact()


@pytest.mark.parametrize("head_dim", [64, 256])
def test_fused_head_dims_64_and_256_bit_exact(head_dim):
    _say("fused head_dim", head_dim)
    w = workloads.make_custom(name="hdf", seed=15, lengths=[3000, 40, 777, 9000], keep_ratio=[0.3, 0.5, 0.7, 0.25],
                              hidden_dim=64, num_q_heads=8, num_kv_heads=2, block_size=64, n_obs=128,
                              head_dim=head_dim)
    b = DeviceBatch(w)
    b.fused()
    _assert_fused_exact(w, b, oracle_run(w))


def test_scores_from_fp32_operands_head_dim_64():
    _say("score fp32 head_dim 64")
    w = workloads.make_custom(name="f32hd", seed=16, lengths=[1, 130, 0, 700, 2100], keep_ratio=[0.5] * 5,
                              hidden_dim=8, num_q_heads=8, num_kv_heads=2, block_size=64, n_obs=128, head_dim=64)
    q32, k32 = _f32_operands(w, 33)
    b = DeviceBatch(w, qk_f32=(q32, k32))
    b.score()
    got = b.results()["scores"].astype(np.float64)
    want = oracle.quantise_scores(oracle.importance_scores(q32, k32, w.cu_seqlens, n_obs=w.n_obs)).astype(np.float64)
    err = np.abs(got - want)
    _say("  worst relative score error", (err / np.maximum(want, 1e-300))[want > 0].max())
    assert (err <= SCORE_RTOL_F32 * want + SCORE_ATOL).all()
    assert b.canaries_intact()


def test_scores_custom_scale_and_heavy_tail():
    _say("score heavy tail")
    w = workloads.make_custom(name="ht", seed=3, lengths=[4000], keep_ratio=[0.25], hidden_dim=8,
                              num_q_heads=8, num_kv_heads=2, block_size=128, k_row_lognormal=True)
    for scale in [0.0, 0.03]:
        b = DeviceBatch(w, softmax_scale=scale)
        b.score()
        got = b.results()["scores"]
        want = oracle.quantise_scores(oracle.importance_scores(
            _q_f32(w), workloads.bf16_bits_to_f32(w.k), w.cu_seqlens, n_obs=w.n_obs, scale=scale or None))
        ok, worst = _score_close(got, want)
        _say("  scale", scale, "worst relative score error", worst, "zeros", int((want == 0).sum()))
        assert ok
        # the floor is applied identically except within rounding of the floor itself
        assert ((got == 0) != (want == 0)).sum() <= 2


# ----------------------------------------------------------------------------- fused, small
def _assert_fused_exact(w, b, ref):
    res = b.results()
    np.testing.assert_array_equal(res["new_cu_seqlens"], ref["new_cu_seqlens"])
    ok, worst = _score_close(res["scores"], ref["scores"])
    margin = score_margin_report(ref, w)
    _say(f"  {w.name}: T={w.total_tokens} kept={len(ref['kept_idx'])} worst score rel err {worst:.3e} "
         f"min selection margin {margin:.3e}")
    assert ok
    diff = np.nonzero(res["kept_idx"] != ref["kept_idx"])[0]
    assert len(diff) == 0, f"{len(diff)} kept indices differ (first at {diff[:5]})"
    np.testing.assert_array_equal(res["pos_out"], ref["pos_out"])
    np.testing.assert_array_equal(res["hidden_out"], ref["hidden_out"])
    assert b.canaries_intact()


@pytest.mark.parametrize("idx,shrink", [(1, 4), (2, 16), (3, 16), (4, 32), (5, 8)])
def test_fused_shrunk_configs_bit_exact(idx, shrink):
    _say("fused shrunk", idx, shrink)
    w = workloads.make_config(idx, shrink=shrink, hidden_dim=256)
    b = DeviceBatch(w)
    b.fused()
    _assert_fused_exact(w, b, oracle_run(w))


def test_fused_without_scores_and_repeatability():
    _say("fused determinism")
    w = workloads.make_config(3, shrink=32, hidden_dim=128)
    b = DeviceBatch(w)
    b.fused(want_scores=False)
    first = b.results()
    assert (first["scores"] == -7.0).all()        # scores_out = NULL: never written
    ref = oracle_run(w)
    np.testing.assert_array_equal(first["kept_idx"], ref["kept_idx"])
    np.testing.assert_array_equal(first["hidden_out"], ref["hidden_out"])
    b.fused(want_scores=True)
    s1 = b.results()["scores"].copy()
    for _ in range(100):       # the same call a hundred times: the same bits every time (no float atomics, fixed orders)
        b.fused(want_scores=True)
        again = b.results()
        np.testing.assert_array_equal(again["kept_idx"], first["kept_idx"])
        np.testing.assert_array_equal(again["hidden_out"], first["hidden_out"])
        np.testing.assert_array_equal(again["scores"].view(np.uint32), s1.view(np.uint32))


def test_sequences_kept_whole_are_not_scored_when_no_scores_are_wanted():
    """Decode rows and short requests (every token a sink or in the window) are kept verbatim by the
    forced-retention rule; with scores_out = NULL the call must not even read their q and k --
    they are poisoned with NaN here -- and the other sequences must come out as the oracle says."""
    _say("sequences kept whole: not scored")
    lengths = [1, 1, 3000, 256, 1, 200, 0, 1300, 255, 1]
    ratio = [0.5, 1.0, 0.3, 0.25, 0.4, 0.6, 0.5, 0.45, 0.2, 0.3]
    w = workloads.make_custom(name="forced", seed=33, lengths=lengths, keep_ratio=ratio, hidden_dim=128,
                              num_q_heads=8, num_kv_heads=4, block_size=64, n_obs=128, n_sink=128)
    ref = oracle_run(w)
    q, k = w.q.copy(), w.k.copy()
    cu = w.cu_seqlens
    for r, N in enumerate(lengths):
        if N <= 256:
            q[cu[r]:cu[r + 1]] = 0x7FC0
            k[cu[r]:cu[r + 1]] = 0x7FC0
    w.q, w.k = q, k
    b = DeviceBatch(w)
    b.fused(want_scores=False)
    res = b.results()
    np.testing.assert_array_equal(res["new_cu_seqlens"], ref["new_cu_seqlens"])
    np.testing.assert_array_equal(res["kept_idx"], ref["kept_idx"])
    np.testing.assert_array_equal(res["hidden_out"], ref["hidden_out"])
    np.testing.assert_array_equal(res["pos_out"], ref["pos_out"])
    assert b.canaries_intact()
    for r, N in enumerate(lengths):          # ... and those sequences are there whole
        if N <= 256:
            got = res["kept_idx"][ref["new_cu_seqlens"][r]:ref["new_cu_seqlens"][r + 1]]
            np.testing.assert_array_equal(got, np.arange(cu[r], cu[r + 1]))


def test_fused_with_fp32_hidden_rows_and_padded_row_strides():
    """The fused call with every row stride larger than the row (q, k and hidden are views into wider
    buffers) and hidden states in float32: indices, rows and positions bit for bit, scores in tolerance;
    the padding of the outputs is never written."""
    _say("fused: fp32 hidden rows, padded strides")
    w = workloads.make_custom(name="strides", seed=44, lengths=[2500, 70, 1100], keep_ratio=[0.3, 0.5, 0.6],
                              hidden_dim=96, num_q_heads=8, num_kv_heads=2, block_size=64, n_obs=128)
    ref = oracle_run(w)
    T, Hq, Hkv, D, d = w.total_tokens, 8, 2, 128, 96
    rng = np.random.default_rng(5)
    qs, ks, hs = Hq * D + 64, Hkv * D + 8, d + 12             # row strides in elements (multiples of 16 bytes)
    q_wide = np.full((T, qs), 0x7FC0, np.uint16); q_wide[:, :Hq * D] = w.q.reshape(T, -1)
    k_wide = np.full((T, ks), 0x7FC0, np.uint16); k_wide[:, :Hkv * D] = w.k.reshape(T, -1)
    hidden_f32 = rng.standard_normal((T, d)).astype(np.float32)
    h_wide = np.full((T, hs), np.nan, np.float32); h_wide[:, :d] = hidden_f32
    p = up.make_params(num_seqs=w.num_seqs, total_tokens=T, block_size=64, n_obs=128, n_sink=128, num_q_heads=Hq,
                       num_kv_heads=Hkv, head_dim=D, hidden_dim=d, q_row_stride=qs, k_row_stride=ks,
                       hidden_row_stride=hs, hidden_dtype=up.UP_F32)
    cu_host = np.ascontiguousarray(w.cu_seqlens, np.int32)
    ratio_host = np.ascontiguousarray(w.keep_ratio, np.float32)
    _, new_cu_plan, K, ws_bytes = up.uniprefill_plan(p, cu_host, ratio_host)
    assert K == len(ref["kept_idx"])
    out = torch.full((K + 8, hs), -7.0, dtype=torch.float32, device="cuda")
    pos_out = torch.full((K + 8,), -77, dtype=torch.int32, device="cuda")
    kept = torch.full((K + 8,), -77, dtype=torch.int32, device="cuda")
    new_cu = torch.full((w.num_seqs + 1 + 8,), -77, dtype=torch.int32, device="cuda")
    scores = torch.full((T + 8,), -7.0, dtype=torch.float32, device="cuda")
    workspace = torch.empty(ws_bytes + 256, dtype=torch.uint8, device="cuda")
    up.uniprefill_fused(p, dev_bf16(q_wide), dev_bf16(k_wide), torch.from_numpy(h_wide).cuda(), torch.from_numpy(w.pos).cuda(),
                        torch.from_numpy(cu_host).cuda(), cu_host, torch.from_numpy(ratio_host).cuda(), ratio_host, out,
                        pos_out, kept, new_cu, scores, workspace, ws_bytes)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(kept[:K].cpu().numpy(), ref["kept_idx"])
    np.testing.assert_array_equal(new_cu[:w.num_seqs + 1].cpu().numpy(), ref["new_cu_seqlens"])
    np.testing.assert_array_equal(pos_out[:K].cpu().numpy(), ref["pos_out"])
    got = out.cpu().numpy()
    np.testing.assert_array_equal(got[:K, :d].view(np.uint32), hidden_f32[ref["kept_idx"]].view(np.uint32))
    assert (got[:K, d:] == -7.0).all() and (got[K:] == -7.0).all()          # padding and canary rows untouched
    assert (kept[K:] == -77).all() and (pos_out[K:] == -77).all() and (scores[T:] == -7.0).all()
    want = ref["scores"].astype(np.float64)
    assert (np.abs(scores[:T].cpu().numpy() - want) <= SCORE_RTOL * want + SCORE_ATOL).all()


def test_fused_identity_at_ratio_one_and_varlen_concat():
    _say("fused identity / concat")
    rng = np.random.default_rng(9)
    lengths = [300, 1, 0, 1029, 257]
    w = workloads.make_custom(name="id", seed=9, lengths=lengths, keep_ratio=[1.0] * 5, hidden_dim=64,
                              num_q_heads=8, num_kv_heads=2, block_size=64)
    b = DeviceBatch(w)
    b.fused()
    res = b.results()
    np.testing.assert_array_equal(res["kept_idx"], np.arange(w.total_tokens, dtype=np.int32))
    np.testing.assert_array_equal(res["hidden_out"], w.hidden)
    np.testing.assert_array_equal(res["new_cu_seqlens"], w.cu_seqlens)
    # varlen batch == concatenation of single-sequence runs
    w2 = workloads.make_custom(name="cat", seed=10, lengths=lengths, keep_ratio=[0.3, 0.5, 0.5, 0.2, 0.6],
                               hidden_dim=64, num_q_heads=8, num_kv_heads=2, block_size=64)
    b2 = DeviceBatch(w2)
    b2.fused()
    whole = b2.results()
    parts = []
    for r in range(5):
        a, e = int(w2.cu_seqlens[r]), int(w2.cu_seqlens[r + 1])
        if e == a:
            continue
        w1 = workloads.Workload(name="one", block_size=64, n_obs=128, n_sink=128, num_q_heads=8, num_kv_heads=2,
                                head_dim=128, hidden_dim=64, cu_seqlens=np.array([0, e - a], np.int32),
                                keep_ratio=w2.keep_ratio[r:r + 1], hidden=w2.hidden[a:e], q=w2.q[a:e],
                                k=w2.k[a:e], pos=w2.pos[a:e])
        b1 = DeviceBatch(w1)
        b1.fused()
        parts.append(b1.results()["kept_idx"] + a)
    np.testing.assert_array_equal(whole["kept_idx"], np.concatenate(parts))


# ----------------------------------------------------------------------------- fused, full size
@pytest.mark.parametrize("idx", [1, 2, 5, 3, 4])
def test_fused_full_size_configs_bit_exact(idx):
    """The five workloads at full size, in the launch configuration the benchmark times."""
    _say("fused full", idx)
    w = workloads.make_config(idx)
    _say("  generated", w.name, "T =", w.total_tokens)
    b = DeviceBatch(w)
    b.fused()
    torch.cuda.synchronize()
    _say("  gpu done; running oracle")
    ref = oracle_run(w)
    _assert_fused_exact(w, b, ref)


def test_fused_128k_shape_with_plain_normal_keys_bit_exact():
    """The headline workload's shape (one 131072-token sequence, 40/8 heads, block 128, ratio 0.25) with
    plain N(0,1) keys instead of the lognormal-scaled ones: on the headline data every block's
    boundary falls among floored zeros (the index rule decides), here the score ranking decides every
    block, at the same launch configuration.  The margin is printed."""
    _say("fused 128k shape, plain keys")
    w = workloads.make_custom(name="c4_shape_plain_keys", seed=77, lengths=[131072], keep_ratio=[0.25], hidden_dim=512,
                              num_q_heads=40, num_kv_heads=8, block_size=128)
    b = DeviceBatch(w)
    b.fused()
    torch.cuda.synchronize()
    ref = oracle_run(w)
    _assert_fused_exact(w, b, ref)
    margin = score_margin_report(ref, w)
    assert np.isfinite(margin) and margin > 0          # blocks whose boundary is decided by the scores exist
    nz = int(np.count_nonzero(ref["scores"]))
    _say(f"  non-zero scores {nz} of {w.total_tokens}, smallest selection margin {margin:.3g}")
    assert nz == w.total_tokens


# ----------------------------------------------------------------------------- block-level top-p (Eq. 4-6)
def _top_p_buffers(w):
    p = up.make_params(num_seqs=w.num_seqs, total_tokens=w.total_tokens, block_size=w.block_size, n_obs=w.n_obs,
                       n_sink=w.n_sink, num_q_heads=w.num_q_heads, num_kv_heads=w.num_kv_heads,
                       head_dim=w.head_dim, hidden_dim=w.hidden_dim)
    cu_host = np.ascontiguousarray(w.cu_seqlens, dtype=np.int32)
    _, _, _, ws_bytes = up.uniprefill_plan(p, cu_host, np.full(w.num_seqs, 0.5, np.float32))
    T, pad = w.total_tokens, 64
    return dict(p=p, cu_host=cu_host, cu=torch.from_numpy(cu_host).cuda(), ws_bytes=ws_bytes,
                workspace=torch.empty(ws_bytes + 256, dtype=torch.uint8, device="cuda"),
                kept_idx=torch.full((T + pad,), -77, dtype=torch.int32, device="cuda"),
                new_cu=torch.full((w.num_seqs + 1 + pad,), -77, dtype=torch.int32, device="cuda"))


@pytest.mark.parametrize("G", [32, 64, 128])
@pytest.mark.parametrize("kind", ["random", "ties", "zeros", "heavy"])
def test_select_top_p_is_bit_exact_on_given_scores(G, kind):
    _say("top-p select", G, kind)
    lengths = [1000, 0, 1, G, G + 1, 5000, 77, 3 * G - 1]
    rng = np.random.default_rng(40 + G)
    w = workloads.make_custom(name="tp", seed=5, lengths=lengths, keep_ratio=[0.5] * len(lengths), hidden_dim=8,
                              num_q_heads=2, num_kv_heads=1, block_size=G, n_obs=48, n_sink=20)
    T = w.total_tokens
    if kind == "random":
        s = rng.random(T).astype(np.float32)
    elif kind == "ties":
        s = rng.integers(0, 3, size=T).astype(np.float32) * np.float32(0.125)
    elif kind == "zeros":
        s = np.zeros(T, np.float32)
    else:
        s = (rng.random(T) ** 30).astype(np.float32)
        s[rng.random(T) < 0.5] = 0.0
    top_p = rng.choice(np.array([0.3, 0.9, 0.99, 1.0], np.float32), size=len(lengths)).astype(np.float32)
    want_idx, want_cu = oracle.select_tokens_top_p(s, w.cu_seqlens, top_p, block_size=G, n_obs=w.n_obs, n_sink=w.n_sink)
    b = _top_p_buffers(w)
    up.uniprefill_select_top_p(b["p"], torch.from_numpy(s).cuda(), b["cu"], b["cu_host"], torch.from_numpy(top_p).cuda(),
                               top_p, b["kept_idx"], b["new_cu"], b["workspace"], b["ws_bytes"])
    torch.cuda.synchronize()
    np.testing.assert_array_equal(b["new_cu"][:w.num_seqs + 1].cpu().numpy(), want_cu)
    np.testing.assert_array_equal(b["kept_idx"][:len(want_idx)].cpu().numpy(), want_idx)
    assert (b["kept_idx"][len(want_idx):] == -77).all() and (b["new_cu"][w.num_seqs + 1:] == -77).all()


def test_select_top_p_long_sequence_and_many_sequences():
    rng = np.random.default_rng(44)
    lengths = [131072] + [int(x) for x in rng.integers(0, 300, size=300)]
    _say("top-p select long + many, T", sum(lengths))
    w = workloads.make_custom(name="tpl", seed=6, lengths=lengths, keep_ratio=[0.5] * len(lengths), hidden_dim=8,
                              num_q_heads=2, num_kv_heads=1, block_size=32, n_obs=128, n_sink=128)
    s = (rng.random(w.total_tokens) ** 20).astype(np.float32)
    top_p = rng.uniform(0.5, 1.0, size=len(lengths)).astype(np.float32)
    want_idx, want_cu = oracle.select_tokens_top_p(s, w.cu_seqlens, top_p, block_size=32, n_obs=128, n_sink=128)
    b = _top_p_buffers(w)
    up.uniprefill_select_top_p(b["p"], torch.from_numpy(s).cuda(), b["cu"], b["cu_host"], torch.from_numpy(top_p).cuda(),
                               top_p, b["kept_idx"], b["new_cu"], b["workspace"], b["ws_bytes"])
    torch.cuda.synchronize()
    np.testing.assert_array_equal(b["new_cu"][:w.num_seqs + 1].cpu().numpy(), want_cu)
    np.testing.assert_array_equal(b["kept_idx"][:len(want_idx)].cpu().numpy(), want_idx)


def test_select_top_p_one_million_tokens_at_block_32():
    """32768 blocks in one sequence (1 M tokens at G = 32, the paper's smallest block at its longest
    context and beyond): the blocks are ordered across the chip and the running sum is formed chunk by
    chunk; bit for bit the oracle's selection."""
    _say("top-p select, 1M tokens, G = 32")
    rng = np.random.default_rng(45)
    T = 1 << 20
    w = workloads.make_custom(name="tp1m", seed=6, lengths=[T], keep_ratio=[0.5], hidden_dim=8, num_q_heads=2,
                              num_kv_heads=1, block_size=32, n_obs=128, n_sink=128)
    s = (rng.random(T) ** 24).astype(np.float32)
    s[rng.random(T) < 0.3] = 0.0
    top_p = np.array([0.97], np.float32)
    want_idx, want_cu = oracle.select_tokens_top_p(s, w.cu_seqlens, top_p, block_size=32, n_obs=128, n_sink=128)
    b = _top_p_buffers(w)
    up.uniprefill_select_top_p(b["p"], torch.from_numpy(s).cuda(), b["cu"], b["cu_host"], torch.from_numpy(top_p).cuda(),
                               top_p, b["kept_idx"], b["new_cu"], b["workspace"], b["ws_bytes"])
    torch.cuda.synchronize()
    np.testing.assert_array_equal(b["new_cu"][:2].cpu().numpy(), want_cu)
    np.testing.assert_array_equal(b["kept_idx"][:len(want_idx)].cpu().numpy(), want_idx)
    assert 0 < len(want_idx) < T and (b["kept_idx"][len(want_idx):] == -77).all()


@pytest.mark.parametrize("idx", [2, 4])
def test_fused_top_p_full_size_configs(idx):
    """The paper's own rule (p = 0.99) end to end on the 32768- and the 131072-token workload at full
    size: the selection is the oracle's rule on the scores the GPU produced, bit for bit, and equals the
    selection of the fp64-scored oracle; rows and positions are the gathered ones."""
    _say("fused top-p, full size", idx)
    w = workloads.make_config(idx)
    top_p = np.full(w.num_seqs, 0.99, np.float32)
    b = _top_p_buffers(w)
    T, d = w.total_tokens, w.hidden_dim
    q, k, hidden = dev_bf16(w.q), dev_bf16(w.k), dev_bf16(w.hidden)
    pos = torch.from_numpy(w.pos).cuda()
    hidden_out = torch.full((T + 8, d), -7.0, dtype=torch.bfloat16, device="cuda")
    pos_out = torch.full((T + 8,), -77, dtype=torch.int32, device="cuda")
    scores = torch.empty(T, dtype=torch.float32, device="cuda")
    up.uniprefill_fused_top_p(b["p"], q, k, hidden, pos, b["cu"], b["cu_host"], torch.from_numpy(top_p).cuda(), top_p,
                              hidden_out, pos_out, b["kept_idx"], b["new_cu"], scores, b["workspace"], b["ws_bytes"])
    torch.cuda.synchronize()
    got_scores = scores.cpu().numpy()
    got_cu = b["new_cu"][:w.num_seqs + 1].cpu().numpy()
    total = int(got_cu[-1])
    got_idx = b["kept_idx"][:total].cpu().numpy()
    want_idx, want_cu = oracle.select_tokens_top_p(got_scores, w.cu_seqlens, top_p, block_size=w.block_size,
                                                   n_obs=w.n_obs, n_sink=w.n_sink)
    np.testing.assert_array_equal(got_cu, want_cu)
    np.testing.assert_array_equal(got_idx, want_idx)
    ref = oracle_run(w)
    ok, worst = _score_close(got_scores, ref["scores"])
    assert ok
    ref_idx, ref_cu = oracle.select_tokens_top_p(ref["scores"], w.cu_seqlens, top_p, block_size=w.block_size,
                                                 n_obs=w.n_obs, n_sink=w.n_sink)
    _say(f"  kept {total} of {T}; worst score error {worst:.3g}")
    np.testing.assert_array_equal(ref_cu, got_cu)
    np.testing.assert_array_equal(ref_idx, got_idx)
    np.testing.assert_array_equal(host_bits(hidden_out[:total]), w.hidden[got_idx])
    np.testing.assert_array_equal(pos_out[:total].cpu().numpy(), w.pos[got_idx])
    assert (hidden_out[total:] == -7.0).all() and (pos_out[total:] == -77).all() and (b["kept_idx"][total:] == -77).all()


def test_fused_top_p_matches_oracle_end_to_end():
    _say("fused top-p")
    w = workloads.make_custom(name="ftp", seed=14, lengths=[3000, 150, 0, 1111], keep_ratio=[0.5] * 4,
                              hidden_dim=64, num_q_heads=8, num_kv_heads=2, block_size=64, n_obs=128)
    top_p = np.array([0.9, 0.99, 0.5, 0.8], np.float32)
    b = _top_p_buffers(w)
    T, d = w.total_tokens, w.hidden_dim
    q, k, hidden = dev_bf16(w.q), dev_bf16(w.k), dev_bf16(w.hidden)
    pos = torch.from_numpy(w.pos).cuda()
    hidden_out = torch.full((T + 8, d), -7.0, dtype=torch.bfloat16, device="cuda")
    pos_out = torch.full((T + 8,), -77, dtype=torch.int32, device="cuda")
    scores = torch.empty(T, dtype=torch.float32, device="cuda")
    up.uniprefill_fused_top_p(b["p"], q, k, hidden, pos, b["cu"], b["cu_host"], torch.from_numpy(top_p).cuda(), top_p,
                              hidden_out, pos_out, b["kept_idx"], b["new_cu"], scores, b["workspace"], b["ws_bytes"])
    torch.cuda.synchronize()
    got_scores = scores.cpu().numpy()
    got_cu = b["new_cu"][:w.num_seqs + 1].cpu().numpy()
    total = int(got_cu[-1])
    got_idx = b["kept_idx"][:total].cpu().numpy()
    # the selection is the oracle's rule applied to the scores the GPU produced (bit for bit) ...
    want_idx, want_cu = oracle.select_tokens_top_p(got_scores, w.cu_seqlens, top_p, block_size=w.block_size,
                                                   n_obs=w.n_obs, n_sink=w.n_sink)
    np.testing.assert_array_equal(got_cu, want_cu)
    np.testing.assert_array_equal(got_idx, want_idx)
    # ... the scores are the oracle's within tolerance, and on this input so is the selection
    ref_scores = oracle.quantise_scores(oracle.importance_scores(_q_f32(w), workloads.bf16_bits_to_f32(w.k),
                                                                w.cu_seqlens, n_obs=w.n_obs))
    ok, worst = _score_close(got_scores, ref_scores)
    assert ok
    ref_idx, ref_cu = oracle.select_tokens_top_p(ref_scores, w.cu_seqlens, top_p, block_size=w.block_size,
                                                 n_obs=w.n_obs, n_sink=w.n_sink)
    _say("  kept", total, "of", T, "worst score error", worst, "same set as the fp64-scored oracle:",
         bool(np.array_equal(ref_idx, got_idx)))
    np.testing.assert_array_equal(ref_cu, got_cu)
    np.testing.assert_array_equal(ref_idx, got_idx)
    # compaction with the count on the device
    want_h, want_p = oracle.compact(w.hidden, w.pos, got_idx)
    np.testing.assert_array_equal(host_bits(hidden_out[:total]), want_h)
    np.testing.assert_array_equal(pos_out[:total].cpu().numpy(), want_p)
    assert (hidden_out[total:] == -7.0).all() and (pos_out[total:] == -77).all()
    assert (b["kept_idx"][total:] == -77).all()


# ----------------------------------------------------------------------------- two drops in a row
def test_second_drop_on_the_compacted_stream_and_composed_scatter():
    """Drop twice (top-k, then top-p on the compacted stream), compose the index maps on the device
    and reconstitute the full batch with one scatter: all bit-exact against the oracle."""
    _say("two drops")
    rng = np.random.default_rng(50)
    w = workloads.make_custom(name="two", seed=15, lengths=[2000, 300, 900], keep_ratio=[0.5, 0.6, 0.4],
                              hidden_dim=64, num_q_heads=4, num_kv_heads=2, block_size=64, n_obs=128)
    T = w.total_tokens
    s1 = rng.random(T).astype(np.float32)
    idx1, cu1 = oracle.select_tokens(s1, w.cu_seqlens, w.keep_ratio, block_size=64, n_obs=128, n_sink=128)
    n1 = len(idx1)
    s2 = (rng.random(n1) ** 8).astype(np.float32)                 # scores of the next drop layer, on the compacted stream
    top_p = np.array([0.7, 0.9, 0.8], np.float32)
    idx2, cu2 = oracle.select_tokens_top_p(s2, cu1, top_p, block_size=64, n_obs=128, n_sink=128)
    want = oracle.compose_index(idx1, idx2)
    # device: second selection on the compacted geometry (cu1), then the composition with the count on the device
    p2 = up.make_params(num_seqs=w.num_seqs, total_tokens=n1, block_size=64, n_obs=128, n_sink=128, num_q_heads=4,
                        num_kv_heads=2, head_dim=128, hidden_dim=64)
    cu1_host = np.ascontiguousarray(cu1, dtype=np.int32)
    _, _, _, ws_bytes = up.uniprefill_plan(p2, cu1_host, np.full(3, 0.5, np.float32))
    workspace = torch.empty(ws_bytes + 256, dtype=torch.uint8, device="cuda")
    idx1_dev = torch.from_numpy(idx1).cuda()
    idx2_dev = torch.full((n1,), -1, dtype=torch.int32, device="cuda")
    cu2_dev = torch.empty(4, dtype=torch.int32, device="cuda")
    up.uniprefill_select_top_p(p2, torch.from_numpy(s2).cuda(), torch.from_numpy(cu1_host).cuda(), cu1_host,
                               torch.from_numpy(top_p).cuda(), top_p, idx2_dev, cu2_dev, workspace, ws_bytes)
    composed = torch.full((n1 + 16,), -77, dtype=torch.int32, device="cuda")
    up.uniprefill_compose_index(idx1_dev, n1, idx2_dev, cu2_dev[3:], n1, composed)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(cu2_dev.cpu().numpy(), cu2)
    n2 = int(cu2[-1])
    np.testing.assert_array_equal(composed[:n2].cpu().numpy(), want)
    assert (composed[n2:] == -77).all()
    # reconstitution (Eq. 8) straight from the innermost stream
    hidden = dev_bf16(w.hidden)
    inner_rows = torch.from_numpy(rng.standard_normal((n2, 64)).astype(np.float32)).cuda().to(torch.bfloat16)
    p1 = up.make_params(num_seqs=w.num_seqs, total_tokens=T, block_size=64, hidden_dim=64)
    full = hidden.clone()
    up.uniprefill_scatter(p1, inner_rows, composed, n2, full)
    torch.cuda.synchronize()
    want_full = oracle.scatter(host_bits(inner_rows), want, w.hidden)
    np.testing.assert_array_equal(host_bits(full), want_full)


# ----------------------------------------------------------------------------- seeded random geometries
@pytest.mark.parametrize("seed", range(24))
def test_fused_random_geometries_bit_exact(seed):
    """Random batch shapes, head layouts, block sizes, window and sink sizes: the launch geometry
    (key-block size, head split, edge classes) must never show in the result."""
    rng = np.random.default_rng(1000 + seed)
    R = int(rng.integers(1, 9))
    lengths = [int(x) for x in rng.choice([0, 1, 17, 64, 129, 300, 512, 777, 1500, 2600, 4100], size=R)]
    if sum(lengths) == 0:
        lengths[0] = 333
    Hkv = int(rng.choice([1, 2, 4, 8]))
    Hq = Hkv * int(rng.choice([1, 2, 4, 5]))
    G = int(rng.choice([32, 64, 128]))
    n_obs = int(rng.choice([16, 100, 128, 256, 384]))
    n_sink = int(rng.choice([0, 4, 128, 200]))
    ratios = [float(x) for x in rng.uniform(0.05, 1.0, size=R)]
    _say("random geometry", seed, dict(lengths=lengths, Hq=Hq, Hkv=Hkv, G=G, n_obs=n_obs, n_sink=n_sink))
    w = workloads.make_custom(name=f"rnd{seed}", seed=2000 + seed, lengths=lengths, keep_ratio=ratios, hidden_dim=32,
                              num_q_heads=Hq, num_kv_heads=Hkv, block_size=G, n_obs=n_obs, n_sink=n_sink)
    b = DeviceBatch(w)
    b.fused()
    _assert_fused_exact(w, b, oracle_run(w))


# ----------------------------------------------------------------------------- the fused call, phase by phase
@pytest.mark.parametrize("lengths", [[3000, 40, 777], [40000]])
def test_fused_phases_one_by_one_equal_the_fused_call(lengths):
    """Enqueuing the five phases separately is exactly uniprefill_fused (both launch geometries:
    shared key blocks for the small batch, one work-group per key block for the long sequence)."""
    _say("phases", lengths)
    w = workloads.make_custom(name="ph", seed=16, lengths=lengths, keep_ratio=[0.3] * len(lengths), hidden_dim=64,
                              num_q_heads=4, num_kv_heads=2, block_size=64, n_obs=128)
    a = DeviceBatch(w)
    a.fused()
    want = a.results()
    b = DeviceBatch(w)
    args = (b.p, b.q, b.k, b.hidden, b.pos, b.cu, b.cu_host, b.ratio, b.ratio_host, b.hidden_out, b.pos_out,
            b.kept_idx, b.new_cu, b.scores, b.workspace, b.ws_bytes)
    for mask in (up.UP_PHASE_PLAN, up.UP_PHASE_ROW_STATS, up.UP_PHASE_MERGE_STATS, up.UP_PHASE_SWEEP_SELECT,
                 up.UP_PHASE_GATHER):
        up.uniprefill_fused_phases(*args, mask)
    got = b.results()
    for key in want:
        np.testing.assert_array_equal(got[key], want[key], err_msg=key)
    assert b.canaries_intact()
    assert up.uniprefill_fused_phases(*args, 64, check=False) == up.UP_ERR_RANGE


@pytest.mark.parametrize("lengths", [[3000, 40, 777, 0, 129], [40000]])
def test_gather_riding_in_the_selecting_kernel_equals_the_fused_call(lengths):
    """UP_PHASE_GATHER_IN_SELECT (the kernel that selects copies its rows; no gather launch) gives the
    fused call's outputs exactly, in both launch geometries and with sequences kept whole."""
    _say("gather in select", lengths)
    w = workloads.make_custom(name="gis", seed=18, lengths=lengths, keep_ratio=[0.37] * len(lengths), hidden_dim=200,
                              num_q_heads=4, num_kv_heads=2, block_size=64, n_obs=128, n_sink=4)
    a = DeviceBatch(w)
    a.fused()
    want = a.results()
    _assert_fused_exact(w, a, oracle_run(w))
    for with_scores in (True, False):      # (without scores the sequences kept whole are not scored)
        b = DeviceBatch(w)
        args = (b.p, b.q, b.k, b.hidden, b.pos, b.cu, b.cu_host, b.ratio, b.ratio_host, b.hidden_out, b.pos_out,
                b.kept_idx, b.new_cu, b.scores if with_scores else None, b.workspace, b.ws_bytes)
        up.uniprefill_fused_phases(*args, up.UP_PHASE_ALL | up.UP_PHASE_GATHER_IN_SELECT)
        got = b.results()
        for key in want:
            if key == "scores" and not with_scores:
                continue
            np.testing.assert_array_equal(got[key], want[key], err_msg=key)
        assert b.canaries_intact()


def test_slot_mapping_of_a_compacted_stream():
    _say("slot mapping")
    rng = np.random.default_rng(60)
    w = workloads.make_custom(name="slots", seed=17, lengths=[1000, 0, 333, 64], keep_ratio=[0.3, 0.5, 0.6, 1.0],
                              hidden_dim=8, num_q_heads=2, num_kv_heads=1, block_size=64, n_obs=32, n_sink=8,
                              pos_offsets=[0, 0, 5, 100])
    scores = rng.random(w.total_tokens).astype(np.float32)
    idx, new_cu = oracle.select_tokens(scores, w.cu_seqlens, w.keep_ratio, block_size=64, n_obs=32, n_sink=8)
    _, pos_kept = oracle.compact(w.hidden, w.pos, idx)
    B, max_blocks = 16, 80
    block_table = rng.permutation(4 * max_blocks).astype(np.int32).reshape(4, max_blocks)
    want = oracle.kv_slot_mapping(pos_kept, new_cu, block_table, B)
    n = len(idx)
    slots = torch.full((n + 8,), -77, dtype=torch.int64, device="cuda")
    up.uniprefill_slot_mapping(torch.from_numpy(pos_kept).cuda(), torch.from_numpy(new_cu).cuda(), 4,
                               torch.from_numpy(block_table).cuda(), max_blocks, B, n + 8, slots)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(slots[:n].cpu().numpy(), want)
    assert (slots[n:] == -77).all()


# ---- tokens that follow earlier context (chunked prefill: the keys of earlier tokens are cached)

def _score_oracle_ctx(w, q=None, k=None):
    return oracle.quantise_scores(oracle.importance_scores_with_context(
        _q_f32(w) if q is None else q, workloads.bf16_bits_to_f32(w.k) if k is None else k,
        w.cu_seqlens, w.cu_seqlens_k, n_obs=w.n_obs))


@pytest.mark.parametrize("case", [
    dict(lengths=[700], earlier=[300], Hq=8, Hkv=2, n_obs=128),
    dict(lengths=[1, 5, 130, 0, 257, 1000, 64], earlier=[0, 1000, 77, 50, 512, 3, 2048], Hq=8, Hkv=2, n_obs=128),
    dict(lengths=[64], earlier=[5000], Hq=4, Hkv=4, n_obs=128),
    dict(lengths=[2100, 300], earlier=[513, 4096], Hq=12, Hkv=4, n_obs=200),
    dict(lengths=[1500, 1500], earlier=[0, 1], Hq=40, Hkv=8, n_obs=128),
    dict(lengths="many", earlier="many", Hq=8, Hkv=2, n_obs=128),
    dict(lengths=[900, 77, 1], earlier=[100, 1000, 700], Hq=4, Hkv=2, n_obs=32, head_dim=64),
    dict(lengths=[900, 77, 1], earlier=[100, 1000, 700], Hq=4, Hkv=2, n_obs=32, head_dim=256),
])
def test_scores_with_earlier_context_match_oracle(case):
    if case["lengths"] == "many":
        lengths = _many_lengths(8, 230)
        earlier = [int(x) for x in np.random.default_rng(9).integers(0, 600, size=len(lengths))]
    else:
        lengths, earlier = case["lengths"], case["earlier"]
    _say("score with context", {k: v for k, v in case.items() if v != "many"}, "T", sum(lengths), "Tk", sum(lengths) + sum(earlier))
    w = workloads.make_custom(name="ctx", seed=17, lengths=lengths, keep_ratio=[0.5] * len(lengths), hidden_dim=8,
                              num_q_heads=case["Hq"], num_kv_heads=case["Hkv"], block_size=64, n_obs=case["n_obs"],
                              head_dim=case.get("head_dim", 128), earlier=earlier)
    b = DeviceBatch(w)
    b.score()
    got = b.results()["scores"]
    ok, worst = _score_close(got, _score_oracle_ctx(w))
    _say("  worst relative score error", worst)
    assert ok
    assert b.canaries_intact()


def test_scores_with_earlier_context_from_fp32_operands():
    _say("score with context fp32")
    w = workloads.make_custom(name="ctx32", seed=18, lengths=[700, 1, 300], keep_ratio=[0.5] * 3, hidden_dim=8,
                              num_q_heads=8, num_kv_heads=2, block_size=64, n_obs=128, earlier=[300, 999, 0])
    q32, k32 = _f32_operands(w, 34)
    b = DeviceBatch(w, qk_f32=(q32, k32))
    b.score()
    got = b.results()["scores"].astype(np.float64)
    want = _score_oracle_ctx(w, q32, k32).astype(np.float64)
    err = np.abs(got - want)
    _say("  worst relative score error", (err / np.maximum(want, 1e-300))[want > 0].max())
    assert (err <= SCORE_RTOL_F32 * want + SCORE_ATOL).all()
    assert b.canaries_intact()


@pytest.mark.parametrize("case", [
    dict(lengths=[3000, 40, 777, 9000], earlier=[1000, 0, 64, 12345], ratios=[0.3, 0.5, 0.7, 0.25], G=64),
    dict(lengths=[8129, 8190, 1, 1, 4000], earlier=[8192, 100, 5000, 0, 17], ratios=[0.4, 0.4, 0.4, 0.4, 0.2], G=128),
    dict(lengths=[20000], earlier=[45000], ratios=[0.3], G=32),
])
def test_fused_with_earlier_context_bit_exact(case):
    _say("fused with context", case)
    w = workloads.make_custom(name="ctxf", seed=19, lengths=case["lengths"], keep_ratio=case["ratios"],
                              hidden_dim=64, num_q_heads=8, num_kv_heads=2, block_size=case["G"], n_obs=128,
                              earlier=case["earlier"])
    b = DeviceBatch(w)
    b.fused()
    _assert_fused_exact(w, b, oracle_run(w))


def test_chunked_entry_with_equal_offsets_equals_the_plain_entry():
    """cu_seqlens_k == cu_seqlens: no earlier context; every output equals the plain entry's, bit for bit
    (the column sums take the route through the workspace, the arithmetic is the same)."""
    _say("chunked == plain without context")
    w = workloads.make_custom(name="ctx0", seed=20, lengths=[3000, 0, 40, 5000], keep_ratio=[0.3, 0.5, 0.5, 0.6],
                              hidden_dim=64, num_q_heads=8, num_kv_heads=2, block_size=64, n_obs=128)
    plain = DeviceBatch(w)
    plain.fused()
    want = plain.results()
    w.cu_seqlens_k = w.cu_seqlens.copy()
    chunked = DeviceBatch(w)
    chunked.fused()
    got = chunked.results()
    for key in want:
        np.testing.assert_array_equal(got[key], want[key], err_msg=key)
    assert chunked.canaries_intact()


def test_select_with_earlier_context_on_given_scores():
    _say("select with context")
    rng = np.random.default_rng(23)
    lengths, earlier = [700, 64, 1, 3000, 129], [100, 0, 5000, 127, 128]
    w = workloads.make_custom(name="ctxs", seed=21, lengths=lengths, keep_ratio=[0.25, 0.5, 0.5, 0.1, 0.9],
                              hidden_dim=8, num_q_heads=2, num_kv_heads=1, block_size=64, n_obs=128, earlier=earlier)
    scores = rng.random(w.total_tokens).astype(np.float32)
    scores[rng.random(w.total_tokens) < 0.3] = 0.0        # ties
    b = DeviceBatch(w)
    b.select(torch.from_numpy(scores).cuda())
    res = b.results()
    kept, new_cu = oracle.select_tokens_with_context(scores, w.cu_seqlens, w.cu_seqlens_k, w.keep_ratio,
                                                     block_size=64, n_obs=128, n_sink=w.n_sink)
    np.testing.assert_array_equal(res["new_cu_seqlens"], new_cu)
    np.testing.assert_array_equal(res["kept_idx"], kept)
    np.testing.assert_array_equal(b.new_cu_plan, new_cu)
    assert b.canaries_intact()


@pytest.mark.parametrize("dtype", [np.int64, np.int32])
def test_compact_column_of_position_ids(dtype):
    """64-bit (and 32-bit) per-token columns follow the kept indices like the hidden rows (Eq. 7);
    with a count on the device only that many entries are written."""
    _say("compact column", dtype.__name__)
    rng = np.random.default_rng(31)
    T = 100003
    column = rng.integers(-2**40 if dtype == np.int64 else -2**30, 2**40 if dtype == np.int64 else 2**30, size=T).astype(dtype)
    kept = np.sort(rng.choice(T, size=33333, replace=False)).astype(np.int32)
    want, _ = oracle.compact(column, column, kept)
    col_d, kept_d = torch.from_numpy(column).cuda(), torch.from_numpy(kept).cuda()
    out = torch.full((len(kept) + 64,), -77, dtype=col_d.dtype, device="cuda")
    up.uniprefill_compact_column(col_d, column.itemsize, kept_d, len(kept), None, out)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out[:len(kept)].cpu().numpy(), want)
    assert bool((out[len(kept):] == -77).all())
    # count on the device, smaller than the capacity
    out.fill_(-77)
    count = torch.tensor([1000], dtype=torch.int32, device="cuda")
    up.uniprefill_compact_column(col_d, column.itemsize, kept_d, len(kept), count, out)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out[:1000].cpu().numpy(), want[:1000])
    assert bool((out[1000:] == -77).all())


def test_seqused_per_layer_matches_oracle():
    """Eq. 17 from a drop history made by two real drops on the device: the retained lengths are the
    differences of each drop's new_cu_seqlens."""
    _say("seqused")
    rng = np.random.default_rng(41)
    R, num_layers, drop_layers = 700, 36, [0, 7, 20]
    orig = rng.integers(1, 30000, size=R).astype(np.int32)
    hist = np.zeros((3, R), np.int32)
    cur = orig.astype(np.int64)
    for k in range(3):
        cur = np.maximum(1, cur * rng.integers(20, 100, size=R) // 100)
        hist[k] = cur
    kv = (orig + rng.integers(0, 2000, size=R)).astype(np.int32)
    out = torch.full((num_layers * R + 64,), -77, dtype=torch.int32, device="cuda")
    up.uniprefill_seqused(drop_layers, torch.from_numpy(hist).cuda(), torch.from_numpy(kv).cuda(),
                          torch.from_numpy(orig).cuda(), R, num_layers, out)
    torch.cuda.synchronize()
    want = oracle.seqused_per_layer(drop_layers, hist, kv, orig, num_layers)
    np.testing.assert_array_equal(out[:num_layers * R].cpu().numpy().reshape(num_layers, R), want)
    assert bool((out[num_layers * R:] == -77).all())
    # no drop events at all
    up.uniprefill_seqused([], None, torch.from_numpy(kv).cuda(), torch.from_numpy(orig).cuda(), R, 2, out)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out[:2 * R].cpu().numpy().reshape(2, R), np.stack([kv, kv]))


def test_fused_call_replayed_from_a_hip_graph():
    """The fused call allocates nothing, never synchronises and records no memset, so a caller can
    capture it in a HIP graph.  Replays with new inputs written into the captured buffers between
    them (and eager work and synchronisations in between) must each equal the eager result."""
    _say("fused under graph capture")
    ws = [workloads.make_custom(name=f"g{i}", seed=50 + i, lengths=[3000, 40, 777], keep_ratio=[0.3, 0.5, 0.7],
                                hidden_dim=64, num_q_heads=8, num_kv_heads=2, block_size=64, n_obs=128)
          for i in range(3)]
    b = DeviceBatch(ws[0])
    b.fused()                                     # warm-up outside the capture (module load)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            b.fused()
    torch.cuda.synchronize()
    for rep, w in enumerate(ws + ws[:1]):
        # new inputs into the captured buffers; outputs poisoned
        b.q.copy_(dev_bf16(w.q)); b.k.copy_(dev_bf16(w.k)); b.hidden.copy_(dev_bf16(w.hidden))
        b.pos.copy_(torch.from_numpy(w.pos).cuda())
        b.hidden_out.fill_(-7.0); b.kept_idx.fill_(-77); b.pos_out.fill_(-77); b.scores.fill_(-7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = b.results()
        eager = DeviceBatch(w)
        eager.fused()
        want = eager.results()
        for key in want:
            np.testing.assert_array_equal(got[key], want[key], err_msg=f"replay {rep}: {key}")
        assert b.canaries_intact()


@pytest.mark.parametrize("seed", range(24))
def test_fused_random_geometries_with_context_and_head_dims_bit_exact(seed):
    """Like the random geometries above, with a random amount of earlier context per request
    (none for some) and head dimensions 64 / 128 / 256."""
    rng = np.random.default_rng(3000 + seed)
    R = int(rng.integers(1, 7))
    lengths = [int(x) for x in rng.choice([0, 1, 17, 64, 129, 300, 512, 777, 1500, 2600], size=R)]
    if sum(lengths) == 0:
        lengths[0] = 333
    earlier = [int(x) for x in rng.choice([0, 0, 1, 63, 128, 511, 512, 513, 1000, 3000, 7000], size=R)]
    Hkv = int(rng.choice([1, 2, 4, 8]))
    Hq = Hkv * int(rng.choice([1, 2, 4]))
    G = int(rng.choice([32, 64, 128]))
    n_obs = int(rng.choice([16, 100, 128, 256]))
    n_sink = int(rng.choice([0, 4, 128, 200]))
    head_dim = int(rng.choice([64, 128, 256]))
    ratios = [float(x) for x in rng.uniform(0.05, 1.0, size=R)]
    _say("random geometry with context", seed, dict(lengths=lengths, earlier=earlier, Hq=Hq, Hkv=Hkv, G=G, n_obs=n_obs,
                                                    n_sink=n_sink, head_dim=head_dim))
    w = workloads.make_custom(name=f"rndc{seed}", seed=4000 + seed, lengths=lengths, keep_ratio=ratios, hidden_dim=32,
                              num_q_heads=Hq, num_kv_heads=Hkv, block_size=G, n_obs=n_obs, n_sink=n_sink,
                              head_dim=head_dim, earlier=earlier)
    b = DeviceBatch(w)
    b.fused()
    _assert_fused_exact(w, b, oracle_run(w))


@pytest.mark.parametrize("kv_block", [16, 256])
def test_paged_keys_equal_packed_keys(kv_block):
    """Keys read through a block table out of a paged cache (random physical blocks, unused rows NaN):
    the scores match the oracle on the keys gathered by Eq. 16, and the fused results are those of
    the chunked entry on the packed keys, bit for bit."""
    _say("paged keys, KV block", kv_block)
    lengths, earlier = [3000, 40, 777, 1, 5000], [1000, 0, 64, 4097, 12345]
    w = workloads.make_custom(name="paged", seed=23, lengths=lengths, keep_ratio=[0.3, 0.5, 0.7, 0.5, 0.25],
                              hidden_dim=64, num_q_heads=8, num_kv_heads=2, block_size=64, n_obs=128, earlier=earlier)
    cache, table = workloads.make_paged_cache(w.k, w.cu_seqlens_k, kv_block, seed=5)
    packed = DeviceBatch(w)
    packed.fused()
    want = packed.results()
    paged = DeviceBatch(w, paged=(cache, table, kv_block))
    paged.fused()
    got = paged.results()
    for key in want:
        np.testing.assert_array_equal(got[key], want[key], err_msg=key)
    assert paged.canaries_intact()
    # and against the oracle, reading the cache itself
    k_read = oracle.gather_paged_keys(cache, w.cu_seqlens_k, table, kv_block)
    ref = oracle.quantise_scores(oracle.importance_scores_with_context(
        _q_f32(w), workloads.bf16_bits_to_f32(k_read), w.cu_seqlens, w.cu_seqlens_k, n_obs=w.n_obs))
    paged.scores.fill_(-7.0)
    paged.score()
    ok, worst = _score_close(paged.results()["scores"], ref)
    _say("  worst relative score error", worst)
    assert ok


def test_fused_one_million_tokens_bit_exact():
    """One sequence of 2^20 tokens (2048 key blocks, 8192 selection blocks): row slots, key-block
    slots and byte offsets far beyond the benchmark sizes."""
    _say("fused 1M tokens")
    w = workloads.make_custom(name="1m", seed=61, lengths=[1 << 20], keep_ratio=[0.2], hidden_dim=64,
                              num_q_heads=8, num_kv_heads=2, block_size=128, n_obs=128)
    b = DeviceBatch(w)
    b.fused()
    _assert_fused_exact(w, b, oracle_run(w))


def test_fused_three_thousand_sequences_bit_exact():
    """A continuous batch of 3000 short requests (empty ones and single tokens among them): the plan
    scans the sequences 1024 (or 256) at a time, and every slot search runs over 3000 offsets."""
    rng = np.random.default_rng(62)
    lengths = [int(x) for x in rng.integers(0, 260, size=3000)]
    lengths[:6] = [0, 1, 1, 0, 259, 128]
    ratios = [float(x) for x in rng.uniform(0.1, 1.0, size=3000)]
    _say("fused 3000 sequences, T", sum(lengths))
    w = workloads.make_custom(name="3k", seed=63, lengths=lengths, keep_ratio=ratios, hidden_dim=32,
                              num_q_heads=4, num_kv_heads=2, block_size=32, n_obs=16, n_sink=4)
    b = DeviceBatch(w)
    b.fused()
    _assert_fused_exact(w, b, oracle_run(w))


@pytest.mark.parametrize("paged", [False, True])
def test_fused_top_p_with_earlier_context(paged):
    """The paper's top-p rule on chunks that follow earlier context, keys packed or in a paged cache."""
    _say("fused top-p with context, paged" if paged else "fused top-p with context")
    lengths, earlier = [3000, 150, 0, 1111, 64], [500, 0, 77, 4000, 100]
    w = workloads.make_custom(name="ftpc", seed=24, lengths=lengths, keep_ratio=[0.5] * 5, hidden_dim=64,
                              num_q_heads=8, num_kv_heads=2, block_size=64, n_obs=128, earlier=earlier)
    top_p = np.array([0.9, 0.99, 0.5, 0.8, 0.7], np.float32)
    b = _top_p_buffers(w)
    cu_k_host = np.ascontiguousarray(w.cu_seqlens_k, dtype=np.int32)
    cu_k = torch.from_numpy(cu_k_host).cuda()
    _, _, _, ws_bytes = up.uniprefill_plan_chunked(b["p"], b["cu_host"], cu_k_host, np.full(w.num_seqs, 0.5, np.float32))
    workspace = torch.empty(ws_bytes + 256, dtype=torch.uint8, device="cuda")
    T, d = w.total_tokens, w.hidden_dim
    table_dev, stride, B = None, 0, 16
    k_bits = w.k
    if paged:
        k_bits, table = workloads.make_paged_cache(w.k, w.cu_seqlens_k, B, seed=6)
        table_dev, stride = torch.from_numpy(table).cuda(), table.shape[1]
    q, k, hidden = dev_bf16(w.q), dev_bf16(k_bits), dev_bf16(w.hidden)
    pos = torch.from_numpy(w.pos).cuda()
    hidden_out = torch.full((T + 8, d), -7.0, dtype=torch.bfloat16, device="cuda")
    pos_out = torch.full((T + 8,), -77, dtype=torch.int32, device="cuda")
    scores = torch.empty(T, dtype=torch.float32, device="cuda")
    up.uniprefill_fused_top_p_chunked(b["p"], q, k, hidden, pos, b["cu"], b["cu_host"], cu_k, cu_k_host, table_dev,
                                      stride, B, torch.from_numpy(top_p).cuda(), top_p, hidden_out, pos_out,
                                      b["kept_idx"], b["new_cu"], scores, workspace, ws_bytes)
    torch.cuda.synchronize()
    got_scores = scores.cpu().numpy()
    got_cu = b["new_cu"][:w.num_seqs + 1].cpu().numpy()
    total = int(got_cu[-1])
    got_idx = b["kept_idx"][:total].cpu().numpy()
    ref_scores = oracle.quantise_scores(oracle.importance_scores_with_context(
        _q_f32(w), workloads.bf16_bits_to_f32(w.k), w.cu_seqlens, w.cu_seqlens_k, n_obs=w.n_obs))
    ok, worst = _score_close(got_scores, ref_scores)
    assert ok
    # the selection is the oracle's rule on the scores the GPU produced, and on this input also on the oracle's
    for sc in (got_scores, ref_scores):
        want_idx, want_cu = oracle.select_tokens_top_p_with_context(sc, w.cu_seqlens, w.cu_seqlens_k, top_p,
                                                                    block_size=w.block_size, n_obs=w.n_obs, n_sink=w.n_sink)
        np.testing.assert_array_equal(got_cu, want_cu)
        np.testing.assert_array_equal(got_idx, want_idx)
    _say("  kept", total, "of", T, "worst score error", worst)
    want_h, want_p = oracle.compact(w.hidden, w.pos, got_idx)
    np.testing.assert_array_equal(host_bits(hidden_out[:total]), want_h)
    np.testing.assert_array_equal(pos_out[:total].cpu().numpy(), want_p)
    assert (hidden_out[total:] == -7.0).all() and (pos_out[total:] == -77).all()
    assert (b["kept_idx"][total:] == -77).all()
    # the stand-alone selection on the same scores
    b["kept_idx"].fill_(-77)
    up.uniprefill_select_top_p_chunked(b["p"], scores, b["cu"], b["cu_host"], cu_k, cu_k_host, torch.from_numpy(top_p).cuda(),
                                       top_p, b["kept_idx"], b["new_cu"], workspace, ws_bytes)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(b["kept_idx"][:total].cpu().numpy(), got_idx)


def test_keep_mask_from_the_index_list():
    _say("keep mask")
    w = workloads.make_custom(name="mask", seed=25, lengths=[3000, 0, 40, 5000, 1], keep_ratio=[0.3, 0.5, 0.5, 0.6, 1.0],
                              hidden_dim=64, num_q_heads=8, num_kv_heads=2, block_size=64, n_obs=128)
    b = DeviceBatch(w)
    b.fused()
    res = b.results()
    T, K = w.total_tokens, b.total_kept
    mask = torch.full((T + 64,), 7, dtype=torch.uint8, device="cuda")
    up.uniprefill_keep_mask(b.kept_idx, K, None, T, mask)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(mask[:T].cpu().numpy(), oracle.keep_mask(res["kept_idx"], T))
    assert bool((mask[T:] == 7).all())
    # the count on the device (as after a top-p selection), smaller than the capacity
    mask.fill_(7)
    up.uniprefill_keep_mask(b.kept_idx, K, torch.tensor([100], dtype=torch.int32, device="cuda"), T, mask)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(mask[:T].cpu().numpy(), oracle.keep_mask(res["kept_idx"][:100], T))
    # an empty list: every byte is written with zero
    up.uniprefill_keep_mask(b.kept_idx, 0, None, T, mask)
    torch.cuda.synchronize()
    assert int(mask[:T].sum()) == 0


# ---- the rows' normalisers handed in (the log-sum-exp an attention kernel returns)

def _window_lse_f32(w):
    """float32 [Hq, T]: log-sum-exp of every window row's visible logits (fp64, scipy), rounded to
    float; entries of other rows are NaN (never read).  An input of the entry under test."""
    from scipy.special import logsumexp
    q = _q_f32(w)
    k = workloads.bf16_bits_to_f32(w.k).astype(np.float64)
    cq = w.cu_seqlens
    ck = w.cu_seqlens_k if w.cu_seqlens_k is not None else w.cu_seqlens
    Hq, group = w.num_q_heads, w.num_q_heads // w.num_kv_heads
    scale = 1.0 / np.sqrt(w.head_dim)
    lse = np.full((Hq, w.total_tokens), np.nan, dtype=np.float32)
    for r in range(w.num_seqs):
        N, L = int(cq[r + 1] - cq[r]), int(ck[r + 1] - ck[r])
        n_eff = min(w.n_obs, N)
        if n_eff == 0:
            continue
        Qw = q[int(cq[r + 1]) - n_eff:int(cq[r + 1])].astype(np.float64)
        for h in range(Hq):
            S = scale * (Qw[:, h, :] @ k[int(ck[r]):int(ck[r + 1]), h // group, :].T)
            for j in range(n_eff):
                lse[h, int(cq[r + 1]) - n_eff + j] = logsumexp(S[j, :L - n_eff + j + 1])
    return lse


@pytest.mark.parametrize("case", [
    dict(lengths=[3000, 40, 777, 9000], earlier=None),
    dict(lengths=[3000, 40, 0, 777, 5000], earlier=[1000, 0, 50, 64, 12345]),
    dict(lengths=[3000, 40, 0, 777, 5000], earlier=[1000, 0, 50, 64, 12345], paged=16),
    dict(lengths=[40000], earlier=None),
])
def test_fused_with_given_normalisers_bit_exact(case):
    _say("fused from lse", case)
    R = len(case["lengths"])
    w = workloads.make_custom(name="lse", seed=26, lengths=case["lengths"], keep_ratio=[0.3, 0.5, 0.7, 0.25, 0.4][:R],
                              hidden_dim=64, num_q_heads=8, num_kv_heads=2, block_size=64, n_obs=128,
                              earlier=case["earlier"])
    lse = _window_lse_f32(w)
    paged = None
    if case.get("paged"):
        cache, table = workloads.make_paged_cache(w.k, w.cu_seqlens_k, case["paged"], seed=7)
        paged = (cache, table, case["paged"])
    b = DeviceBatch(w, paged=paged)
    b.fused_lse(torch.from_numpy(lse).cuda())
    res = b.results()
    # the oracle reads the same float32 normalisers
    ck = w.cu_seqlens_k if w.cu_seqlens_k is not None else w.cu_seqlens
    o = oracle.importance_scores_from_lse(_q_f32(w), workloads.bf16_bits_to_f32(w.k), lse, w.cu_seqlens, ck, n_obs=w.n_obs)
    s32 = oracle.quantise_scores(o)
    ok, worst = _score_close(res["scores"], s32)
    _say("  worst relative score error", worst)
    assert ok
    if w.cu_seqlens_k is not None:
        kept, new_cu = oracle.select_tokens_with_context(s32, w.cu_seqlens, w.cu_seqlens_k, w.keep_ratio, block_size=w.block_size,
                                                         n_obs=w.n_obs, n_sink=w.n_sink)
    else:
        kept, new_cu = oracle.select_tokens(s32, w.cu_seqlens, w.keep_ratio, block_size=w.block_size, n_obs=w.n_obs,
                                            n_sink=w.n_sink)
    np.testing.assert_array_equal(res["new_cu_seqlens"], new_cu)
    np.testing.assert_array_equal(res["kept_idx"], kept)
    h_out, p_out = oracle.compact(w.hidden, w.pos, kept)
    np.testing.assert_array_equal(res["hidden_out"], h_out)
    np.testing.assert_array_equal(res["pos_out"], p_out)
    assert b.canaries_intact()
    # and the two-pass call on the same batch keeps the same tokens (the normalisers were exact to float rounding)
    two = DeviceBatch(w, paged=paged)
    two.fused()
    np.testing.assert_array_equal(two.results()["kept_idx"], res["kept_idx"])


def test_score_and_top_p_with_given_normalisers():
    """uniprefill_score_lse and uniprefill_fused_top_p_lse on chunks after earlier context: the scores
    are the oracle's from the same float normalisers; the top-p selection is the oracle's rule on them."""
    _say("score / fused top-p from lse")
    lengths, earlier = [3000, 150, 0, 1111, 64], [500, 0, 77, 4000, 100]
    w = workloads.make_custom(name="lsetp", seed=27, lengths=lengths, keep_ratio=[0.5] * 5, hidden_dim=64,
                              num_q_heads=8, num_kv_heads=2, block_size=64, n_obs=128, earlier=earlier)
    lse = _window_lse_f32(w)
    lse_dev = torch.from_numpy(lse).cuda()
    top_p = np.array([0.9, 0.99, 0.5, 0.8, 0.7], np.float32)
    b = DeviceBatch(w)
    T, d = w.total_tokens, w.hidden_dim
    up.uniprefill_score_lse(b.p, b.q, b.k, lse_dev, T, b.cu, b.cu_host, b.cu_k, b.cu_k_host, None, 0, 16, b.scores,
                            b.workspace, b.ws_bytes)
    got_scores = b.results()["scores"]
    ref = oracle.quantise_scores(oracle.importance_scores_from_lse(_q_f32(w), workloads.bf16_bits_to_f32(w.k), lse,
                                                                   w.cu_seqlens, w.cu_seqlens_k, n_obs=w.n_obs))
    ok, worst = _score_close(got_scores, ref)
    _say("  worst relative score error", worst)
    assert ok and b.canaries_intact()
    kept = torch.full((T + 64,), -77, dtype=torch.int32, device="cuda")
    ncu = torch.full((w.num_seqs + 1,), -77, dtype=torch.int32, device="cuda")
    hout = torch.full((T + 8, d), -7.0, dtype=torch.bfloat16, device="cuda")
    pout = torch.full((T + 8,), -77, dtype=torch.int32, device="cuda")
    sc = torch.empty(T, dtype=torch.float32, device="cuda")
    up.uniprefill_fused_top_p_lse(b.p, b.q, b.k, lse_dev, T, b.hidden, b.pos, b.cu, b.cu_host, b.cu_k, b.cu_k_host, None, 0,
                                  16, torch.from_numpy(top_p).cuda(), top_p, hout, pout, kept, ncu, sc, b.workspace,
                                  b.ws_bytes)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(sc.cpu().numpy(), got_scores)
    for scores in (got_scores, ref):
        want_idx, want_cu = oracle.select_tokens_top_p_with_context(scores, w.cu_seqlens, w.cu_seqlens_k, top_p,
                                                                    block_size=w.block_size, n_obs=w.n_obs, n_sink=w.n_sink)
        np.testing.assert_array_equal(ncu.cpu().numpy(), want_cu)
        np.testing.assert_array_equal(kept[:int(want_cu[-1])].cpu().numpy(), want_idx)
    total = int(ncu[-1].item())
    wh, wp = oracle.compact(w.hidden, w.pos, kept[:total].cpu().numpy())
    np.testing.assert_array_equal(host_bits(hout[:total]), wh)
    np.testing.assert_array_equal(pout[:total].cpu().numpy(), wp)
    assert (kept[total:] == -77).all() and (pout[total:] == -77).all()


def test_batches_without_tokens():
    """Every request empty: legal; nothing but the plan is launched and new_cu_seqlens is all zero.
    Also a batch whose requests have cached keys but bring no token."""
    _say("empty batches")
    for earlier in (None, [100, 0, 7]):
        w = workloads.make_custom(name="none", seed=28, lengths=[0, 0, 0], keep_ratio=[0.5] * 3, hidden_dim=64,
                                  num_q_heads=8, num_kv_heads=2, block_size=64, n_obs=128, earlier=earlier)
        assert w.total_tokens == 0
        b = DeviceBatch(w)
        assert b.total_kept == 0
        b.fused()
        res = b.results()
        np.testing.assert_array_equal(res["new_cu_seqlens"], [0, 0, 0, 0])
        assert res["kept_idx"].size == 0 and b.canaries_intact()
        b.new_cu.fill_(-77)
        b.score()
        b.select(b.scores)
        np.testing.assert_array_equal(b.results()["new_cu_seqlens"], [0, 0, 0, 0])
        assert b.canaries_intact()
        # the per-token arrays and the workspace may be NULL when there is no token
        b.new_cu.fill_(-77)
        if earlier is None:
            up.uniprefill_fused(b.p, None, None, None, None, b.cu, b.cu_host, b.ratio, b.ratio_host, None, None, None,
                                b.new_cu, None, None, 0)
        else:
            up.uniprefill_fused_chunked(b.p, None, None, None, None, b.cu, b.cu_host, b.cu_k, b.cu_k_host, b.ratio,
                                        b.ratio_host, None, None, None, b.new_cu, None, None, 0)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(b.new_cu[:4].cpu().numpy(), [0, 0, 0, 0])
        b.new_cu.fill_(-77)
        up.uniprefill_fused_top_p_lse(b.p, None, None, torch.zeros(8, dtype=torch.float32, device="cuda"), 0, None, None,
                                      b.cu, b.cu_host, b.cu_k if earlier else None, b.cu_k_host if earlier else None,
                                      None, 0, 16, b.ratio, b.ratio_host, None, None, None, b.new_cu, None, None, 0)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(b.new_cu[:4].cpu().numpy(), [0, 0, 0, 0])
        assert up.uniprefill_compact(b.p, None, None, None, 0, None, None) == up.UP_OK
        assert up.uniprefill_scatter(b.p, None, None, 0, None) == up.UP_OK
    # no request at all
    p0 = up.make_params(num_seqs=0, total_tokens=0, block_size=64, num_q_heads=8, num_kv_heads=2, hidden_dim=64)
    cu0_host = np.zeros(1, np.int32)
    cu0 = torch.zeros(1, dtype=torch.int32, device="cuda")
    out0 = torch.full((4,), -77, dtype=torch.int32, device="cuda")
    up.uniprefill_fused(p0, None, None, None, None, cu0, cu0_host, None, None, None, None, None, out0, None, None, 0)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out0.cpu().numpy(), [0, -77, -77, -77])


@pytest.mark.parametrize("earlier", [None, [700, 0, 64]])
def test_tensor_parallel_shares_add_up_to_the_single_device_result(earlier):
    """Eq. 15 on one device: the heads are split over four ranks (two query heads and their kv head
    each, read as views into the full rows), every rank leaves its partial sums, the sums are
    combined in rank order, and the scores and the selection are those of the whole model."""
    _say("tensor-parallel shares", earlier)
    lengths = [3000, 40, 2500]
    Hq, Hkv, D, ranks = 8, 4, 128, 4
    w = workloads.make_custom(name="tp", seed=29, lengths=lengths, keep_ratio=[0.3, 0.5, 0.4], hidden_dim=64,
                              num_q_heads=Hq, num_kv_heads=Hkv, block_size=64, n_obs=128, earlier=earlier)
    T = w.total_tokens
    whole = DeviceBatch(w)
    q_all, k_all = whole.q, whole.k
    p_rank = up.make_params(num_seqs=w.num_seqs, total_tokens=T, block_size=w.block_size, n_obs=w.n_obs, n_sink=w.n_sink,
                            num_q_heads=Hq // ranks, num_kv_heads=Hkv // ranks, head_dim=D, hidden_dim=w.hidden_dim,
                            q_row_stride=Hq * D, k_row_stride=Hkv * D)
    cu_k_host = whole.cu_k_host if earlier else None
    cu_k = whole.cu_k if earlier else None
    if earlier:
        _, _, _, ws_bytes = up.uniprefill_plan_chunked(p_rank, whole.cu_host, cu_k_host, whole.ratio_host)
    else:
        _, _, _, ws_bytes = up.uniprefill_plan(p_rank, whole.cu_host, whole.ratio_host)
    workspace = torch.empty(ws_bytes + 256, dtype=torch.uint8, device="cuda")
    partials = torch.full((ranks, T + 8), -7.0, dtype=torch.float64, device="cuda")
    for t in range(ranks):
        q_view = q_all[:, t * (Hq // ranks):, :]          # the rank's heads start here; the row stride stays the full row
        k_view = k_all[:, t * (Hkv // ranks):, :]
        up.uniprefill_score_partial(p_rank, q_view, k_view, whole.cu, whole.cu_host, cu_k, cu_k_host, partials[t],
                                    workspace, ws_bytes)
    torch.cuda.synchronize()
    assert bool((partials[:, T:] == -7.0).all())
    # every rank's sums against the oracle's for that share
    kf = workloads.bf16_bits_to_f32(w.k)
    ck = w.cu_seqlens_k if earlier else w.cu_seqlens
    refs = []
    for t in range(ranks):
        ref = oracle.importance_sums(_ShardQ(w.q, t * (Hq // ranks), Hq // ranks), kf[:, t:t + 1, :], w.cu_seqlens, ck, n_obs=w.n_obs)
        refs.append(ref)
        got = partials[t, :T].cpu().numpy()
        assert (np.abs(got - ref) <= 1e-5 * ref + 2.0 ** -64).all()
    scores = torch.full((T + 64,), -7.0, dtype=torch.float32, device="cuda")
    up.uniprefill_scores_from_partials(partials, ranks, T + 8, whole.cu, w.num_seqs, T, w.n_obs, Hq, scores)
    torch.cuda.synchronize()
    want = oracle.quantise_scores(oracle.scores_from_partial_sums(refs, w.cu_seqlens, n_obs=w.n_obs, total_q_heads=Hq))
    ok, worst = _score_close(scores[:T].cpu().numpy(), want)
    _say("  worst relative score error", worst)
    assert ok and bool((scores[T:] == -7.0).all())
    # the selection on the combined scores is the single-device selection
    whole.fused()
    single = whole.results()
    whole.kept_idx.fill_(-77)
    whole.select(scores[:T])
    np.testing.assert_array_equal(whole.results()["kept_idx"], single["kept_idx"])
    np.testing.assert_array_equal(single["kept_idx"], oracle_run(w)["kept_idx"])


class _ShardQ:
    """Window rows of a head shard of w.q, upcast on demand (the oracle slices rows only)."""

    def __init__(self, bits, h0, nh):
        self.bits, self.h0, self.nh = bits, h0, nh
        self.shape = (bits.shape[0], nh, bits.shape[2])

    def __getitem__(self, item):
        return workloads.bf16_bits_to_f32(self.bits[item][:, self.h0:self.h0 + self.nh, :])

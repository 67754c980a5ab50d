"""CPU-only tests of the C-ABI boundary: the library loads, exports every declared
symbol, rejects bad arguments on the host before any launch, and its closed-form
plan agrees with the oracle's block-by-block counts."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2605_06221_amd as up

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _params(**kw):
    base = dict(num_seqs=1, total_tokens=1000, block_size=64, num_q_heads=8, num_kv_heads=2, hidden_dim=256)
    base.update(kw)
    return up.make_params(**base)


def test_library_exports_every_symbol_declared_in_the_header():
    header = open(os.path.join(ROOT, "include", "uniprefill.h")).read()
    declared = set(re.findall(r"\b(uniprefill_\w+)\s*\(", header))
    assert declared == set(up.EXPORTS)
    lib = ctypes.CDLL(up.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_status_strings():
    seen = {up.status_string(i) for i in range(9)}
    assert len(seen) == 9 and up.status_string(0) == "ok"
    assert up.status_string(99) == "unknown status"


def test_params_struct_layout_matches_header():
    # 9 int32, pad to 8, 3 int64, float, 2 int32  -> 40 + 24 + 12 = 76 -> padded to 80
    assert ctypes.sizeof(up.up_params) == 80
    assert up.up_params.q_row_stride.offset == 40
    assert up.up_params.softmax_scale.offset == 64


@pytest.mark.parametrize("seed", range(6))
def test_plan_matches_oracle_counts(seed):
    rng = np.random.default_rng(seed)
    R = int(rng.integers(1, 40))
    lengths = rng.integers(0, 3000, R)
    lengths[rng.integers(0, R)] = int(rng.integers(0, 3))
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    ratio = rng.uniform(0.01, 1.0, R).astype(np.float32)
    ratio[rng.integers(0, R)] = 1.0
    G = int(rng.choice([32, 64, 128]))
    n_obs = int(rng.choice([1, 17, 32, 128, 512]))
    n_sink = int(rng.choice([0, 5, 128, 200, 5000]))
    p = _params(num_seqs=R, total_tokens=int(cu[-1]), block_size=G, n_obs=n_obs, n_sink=n_sink)
    st, new_cu, total, ws = up.uniprefill_plan(p, cu, ratio)
    want = oracle.plan(cu, ratio, block_size=G, n_obs=n_obs, n_sink=n_sink)
    np.testing.assert_array_equal(new_cu, want)
    assert total == want[-1] and ws > 0 and ws % 256 == 0


def test_plan_totals_of_the_named_workloads():
    for T, G, rho, want in [(4096, 64, 0.5, 2176), (32768, 128, 0.3, 10162), (131072, 128, 0.25, 32960)]:
        p = _params(total_tokens=T, block_size=G)
        _, new_cu, total, _ = up.uniprefill_plan(p, np.array([0, T], np.int32), np.array([rho], np.float32))
        assert total == want and new_cu[1] == want


def test_plan_handles_empty_batches():
    p = _params(num_seqs=0, total_tokens=0)
    st, new_cu, total, ws = up.uniprefill_plan(p, np.array([0], np.int32), np.zeros(0, np.float32))
    assert st == up.UP_OK and total == 0 and list(new_cu) == [0]
    p = _params(num_seqs=3, total_tokens=0)
    st, new_cu, total, _ = up.uniprefill_plan(p, np.zeros(4, np.int32), np.ones(3, np.float32))
    assert st == up.UP_OK and total == 0


def test_plan_rejects_bad_arguments():
    cu = np.array([0, 1000], np.int32)
    ratio = np.array([0.5], np.float32)
    plan = lambda p, c=cu, r=ratio: up.uniprefill_plan(p, c, r, check=False)[0]
    assert plan(_params()) == up.UP_OK
    assert plan(_params(block_size=48)) == up.UP_ERR_RANGE
    assert plan(_params(n_obs=0)) == up.UP_ERR_RANGE
    assert plan(_params(n_obs=4096)) == up.UP_ERR_RANGE
    assert plan(_params(n_sink=-1)) == up.UP_ERR_RANGE
    assert plan(_params(head_dim=64)) == up.UP_OK
    assert plan(_params(head_dim=256)) == up.UP_OK
    assert plan(_params(head_dim=96)) == up.UP_ERR_UNSUPPORTED
    assert plan(_params(head_dim=256, qk_dtype=up.UP_F32)) == up.UP_ERR_UNSUPPORTED
    assert plan(_params(num_q_heads=6, num_kv_heads=4)) == up.UP_ERR_UNSUPPORTED
    assert plan(_params(qk_dtype=up.UP_F32)) == up.UP_OK
    assert plan(_params(qk_dtype=7)) == up.UP_ERR_UNSUPPORTED
    assert plan(_params(qk_dtype=up.UP_F32, q_row_stride=8 * 128 + 2)) == up.UP_ERR_ALIGN
    assert plan(_params(softmax_scale=-1.0)) == up.UP_ERR_RANGE
    assert plan(_params(softmax_scale=float("nan"))) == up.UP_ERR_RANGE
    assert plan(_params(q_row_stride=8 * 128 + 4)) == up.UP_ERR_ALIGN
    assert plan(_params(q_row_stride=128)) == up.UP_ERR_SHAPE
    assert plan(_params(total_tokens=999)) == up.UP_ERR_SHAPE
    assert plan(_params(), np.array([1, 1000], np.int32)) == up.UP_ERR_SHAPE
    assert plan(_params(num_seqs=2), np.array([0, 1200, 1000], np.int32), np.array([0.5, 0.5], np.float32)) == up.UP_ERR_SHAPE
    for bad in [0.0, -0.1, 1.0001, float("nan")]:
        assert plan(_params(), cu, np.array([bad], np.float32)) == up.UP_ERR_RANGE
    st = up.lib().uniprefill_plan(None, up.ptr(cu), up.ptr(ratio), None, None, None)
    assert st == up.UP_ERR_NULL
    st = up.lib().uniprefill_plan(ctypes.byref(_params()), None, up.ptr(ratio), None, None, None)
    assert st == up.UP_ERR_NULL
    st = up.lib().uniprefill_plan(ctypes.byref(_params()), up.ptr(cu), None, None, None, None)
    assert st == up.UP_ERR_NULL
    with pytest.raises(up.UniPrefillError):
        up.uniprefill_plan(_params(block_size=5), cu, ratio)


def test_device_entries_reject_bad_arguments_before_any_launch():
    """Argument errors come back synchronously; with no GPU in the process this also
    proves that nothing was launched."""
    cu = np.array([0, 1000], np.int32)
    ratio = np.array([0.5], np.float32)
    fake = 0x1000                       # aligned non-null stand-in, never dereferenced
    odd = 0x1008
    p = _params()
    L = up.lib()
    B = ctypes.byref
    v = ctypes.c_void_p
    # compact / scatter
    assert L.uniprefill_compact(B(p), None, None, v(fake), 10, v(fake), None, None) == up.UP_ERR_NULL
    assert L.uniprefill_compact(B(p), v(fake), v(fake), v(fake), 10, v(fake), None, None) == up.UP_ERR_NULL
    assert L.uniprefill_compact(B(p), v(odd), None, v(fake), 10, v(fake), None, None) == up.UP_ERR_ALIGN
    assert L.uniprefill_compact(B(p), v(fake), None, v(fake), -1, v(fake), None, None) == up.UP_ERR_RANGE
    assert L.uniprefill_compact(B(p), v(fake), None, v(fake), 1001, v(fake), None, None) == up.UP_ERR_RANGE
    assert L.uniprefill_compact(B(_params(hidden_dim=100)), v(fake), None, v(fake), 1, v(fake), None, None) == up.UP_ERR_ALIGN
    assert L.uniprefill_compact(B(_params(hidden_dtype=7)), v(fake), None, v(fake), 1, v(fake), None, None) == up.UP_ERR_UNSUPPORTED
    assert L.uniprefill_compact(B(_params(hidden_row_stride=128)), v(fake), None, v(fake), 1, v(fake), None, None) == up.UP_ERR_SHAPE
    assert L.uniprefill_scatter(B(p), v(fake), None, 10, v(fake), None) == up.UP_ERR_NULL
    assert L.uniprefill_scatter(B(p), v(fake), v(fake), 10, v(odd), None) == up.UP_ERR_ALIGN
    # zero rows: legal, launches nothing
    assert L.uniprefill_compact(B(p), v(fake), None, v(fake), 0, v(fake), None, None) == up.UP_OK
    assert L.uniprefill_scatter(B(p), v(fake), v(fake), 0, v(fake), None) == up.UP_OK
    # select
    assert L.uniprefill_select(B(p), None, v(fake), up.ptr(cu), v(fake), up.ptr(ratio), v(fake), v(fake), None) == up.UP_ERR_NULL
    assert L.uniprefill_select(B(p), v(fake), v(fake), None, v(fake), up.ptr(ratio), v(fake), v(fake), None) == up.UP_ERR_NULL
    bad_ratio = np.array([1.5], np.float32)
    assert L.uniprefill_select(B(p), v(fake), v(fake), up.ptr(cu), v(fake), up.ptr(bad_ratio), v(fake), v(fake), None) == up.UP_ERR_RANGE
    bad_cu = np.array([0, 999], np.int32)
    assert L.uniprefill_select(B(p), v(fake), v(fake), up.ptr(bad_cu), v(fake), up.ptr(ratio), v(fake), v(fake), None) == up.UP_ERR_SHAPE
    # score
    assert L.uniprefill_score(B(p), v(fake), None, v(fake), up.ptr(cu), v(fake), v(fake), 1 << 30, None) == up.UP_ERR_NULL
    assert L.uniprefill_score(B(p), v(fake), v(odd), v(fake), up.ptr(cu), v(fake), v(fake), 1 << 30, None) == up.UP_ERR_ALIGN
    assert L.uniprefill_score(B(p), v(fake), v(fake), v(fake), up.ptr(cu), v(fake), None, 0, None) == up.UP_ERR_WORKSPACE
    assert L.uniprefill_score(B(p), v(fake), v(fake), v(fake), up.ptr(cu), v(fake), v(fake), 16, None) == up.UP_ERR_WORKSPACE
    assert L.uniprefill_score(B(p), v(fake), v(fake), v(fake), up.ptr(cu), v(fake), v(0x1010), 1 << 30, None) == up.UP_ERR_ALIGN
    assert L.uniprefill_score(B(_params(head_dim=96)), v(fake), v(fake), v(fake), up.ptr(cu), v(fake), v(fake), 1 << 30, None) == up.UP_ERR_UNSUPPORTED
    # fused
    args = [v(fake)] * 4 + [v(fake), up.ptr(cu), v(fake), up.ptr(ratio)] + [v(fake)] * 4 + [None, v(fake), 16, None]
    assert L.uniprefill_fused(B(p), *args) == up.UP_ERR_WORKSPACE
    args[0] = None
    assert L.uniprefill_fused(B(p), *args) == up.UP_ERR_NULL


def test_top_p_entries_reject_bad_arguments_before_any_launch():
    cu = np.array([0, 1000], np.int32)
    top_p = np.array([0.9], np.float32)
    fake, odd = 0x1000, 0x1008
    p = _params()
    L = up.lib()
    B = ctypes.byref
    v = ctypes.c_void_p
    big = 1 << 30
    sel = lambda *a: L.uniprefill_select_top_p(B(p), *a)
    assert sel(None, v(fake), up.ptr(cu), v(fake), up.ptr(top_p), v(fake), v(fake), v(fake), big, None) == up.UP_ERR_NULL
    assert sel(v(fake), v(fake), None, v(fake), up.ptr(top_p), v(fake), v(fake), v(fake), big, None) == up.UP_ERR_NULL
    assert sel(v(fake), v(fake), up.ptr(cu), v(fake), None, v(fake), v(fake), v(fake), big, None) == up.UP_ERR_NULL
    for bad in [0.0, 1.5, float("nan")]:
        assert sel(v(fake), v(fake), up.ptr(cu), v(fake), up.ptr(np.array([bad], np.float32)), v(fake), v(fake),
                   v(fake), big, None) == up.UP_ERR_RANGE
    assert sel(v(fake), v(fake), up.ptr(cu), v(fake), up.ptr(top_p), v(fake), v(fake), None, 0, None) == up.UP_ERR_WORKSPACE
    assert sel(v(fake), v(fake), up.ptr(cu), v(fake), up.ptr(top_p), v(fake), v(fake), v(fake), 8, None) == up.UP_ERR_WORKSPACE
    assert sel(v(fake), v(fake), up.ptr(cu), v(fake), up.ptr(top_p), v(fake), v(fake), v(0x1010), big, None) == up.UP_ERR_ALIGN
    # a sequence with more blocks than the kernels order (65536)
    p_long = _params(total_tokens=32 * 65536 + 1, block_size=32)
    cu_long = np.array([0, 32 * 65536 + 1], np.int32)
    assert L.uniprefill_select_top_p(B(p_long), v(fake), v(fake), up.ptr(cu_long), v(fake), up.ptr(top_p), v(fake),
                                     v(fake), v(fake), big, None) == up.UP_ERR_UNSUPPORTED
    # compact with the count on the device
    cc = lambda *a: L.uniprefill_compact_counted(B(p), *a)
    assert cc(v(fake), None, v(fake), None, 10, v(fake), None, None) == up.UP_ERR_NULL
    assert cc(v(fake), None, v(fake), v(fake), 1001, v(fake), None, None) == up.UP_ERR_RANGE
    assert cc(v(fake), None, v(fake), v(fake), -1, v(fake), None, None) == up.UP_ERR_RANGE
    assert cc(v(odd), None, v(fake), v(fake), 10, v(fake), None, None) == up.UP_ERR_ALIGN
    assert cc(v(fake), v(fake), v(fake), v(fake), 10, v(fake), None, None) == up.UP_ERR_NULL
    assert cc(v(fake), None, v(fake), v(fake), 0, v(fake), None, None) == up.UP_OK
    # fused: every check of the three steps before the first launch
    args = [v(fake)] * 4 + [v(fake), up.ptr(cu), v(fake), up.ptr(top_p)] + [v(fake)] * 4 + [v(fake), v(fake), 16, None]
    assert L.uniprefill_fused_top_p(B(p), *args) == up.UP_ERR_WORKSPACE
    args[12] = None          # the score buffer is required here
    assert L.uniprefill_fused_top_p(B(p), *args) == up.UP_ERR_NULL


def test_compose_index_rejects_bad_arguments():
    L, v, fake = up.lib(), ctypes.c_void_p, 0x1000
    assert L.uniprefill_compose_index(None, 10, v(fake), None, 5, v(fake), None) == up.UP_ERR_NULL
    assert L.uniprefill_compose_index(v(fake), 10, v(fake), None, 11, v(fake), None) == up.UP_ERR_RANGE
    assert L.uniprefill_compose_index(v(fake), -1, v(fake), None, 0, v(fake), None) == up.UP_ERR_RANGE
    assert L.uniprefill_compose_index(v(fake), 10, v(fake), None, 0, v(fake), None) == up.UP_OK


def test_slot_mapping_rejects_bad_arguments():
    L, v, fake = up.lib(), ctypes.c_void_p, 0x1000
    assert L.uniprefill_slot_mapping(None, v(fake), 2, v(fake), 8, 16, 10, v(fake), None) == up.UP_ERR_NULL
    assert L.uniprefill_slot_mapping(v(fake), v(fake), 2, v(fake), 8, 0, 10, v(fake), None) == up.UP_ERR_RANGE
    assert L.uniprefill_slot_mapping(v(fake), v(fake), -1, v(fake), 8, 16, 10, v(fake), None) == up.UP_ERR_RANGE
    assert L.uniprefill_slot_mapping(v(fake), v(fake), 2, v(fake), 8, 16, 0, v(fake), None) == up.UP_OK


def test_plan_chunked_matches_oracle_and_rejects_bad_offsets():
    import oracle
    rng = np.random.default_rng(9)
    for _ in range(30):
        R = int(rng.integers(1, 9))
        Ns = rng.integers(0, 900, size=R)
        Ps = rng.integers(0, 400, size=R) * (rng.random(R) < 0.7)
        G = int(rng.choice([32, 64, 128]))
        n_obs, n_sink = int(rng.choice([16, 128, 200])), int(rng.choice([0, 4, 128]))
        cu = np.concatenate([[0], np.cumsum(Ns)]).astype(np.int32)
        cu_k = np.concatenate([[0], np.cumsum(Ns + Ps)]).astype(np.int32)
        ratio = rng.uniform(0.05, 1.0, size=R).astype(np.float32)
        p = _params(num_seqs=R, total_tokens=int(cu[-1]), block_size=G, n_obs=n_obs, n_sink=n_sink)
        st, new_cu, total, ws = up.uniprefill_plan_chunked(p, cu, cu_k, ratio)
        assert st == up.UP_OK and ws > 0
        sinks = oracle.sinks_in_chunk(cu, cu_k, n_sink)
        want = np.zeros(R + 1, np.int64)
        for r in range(R):
            want[r + 1] = want[r] + sum(oracle.block_kept_counts(int(Ns[r]), G, n_obs, int(sinks[r]), ratio[r]))
        np.testing.assert_array_equal(new_cu, want)
        assert total == want[-1]
        # equal offsets: the plain plan
        st2, new_cu2, total2, _ = up.uniprefill_plan_chunked(p, cu, cu, ratio)
        _, new_cu3, total3, _ = up.uniprefill_plan(p, cu, ratio)
        np.testing.assert_array_equal(new_cu2, new_cu3)
        assert total2 == total3
    cu = np.array([0, 100, 300], np.int32)
    ratio = np.array([0.5, 0.5], np.float32)
    p = _params(num_seqs=2, total_tokens=300)
    plan = lambda ck: up.uniprefill_plan_chunked(p, cu, ck, ratio, check=False)[0]
    assert plan(np.array([0, 100, 300], np.int32)) == up.UP_OK
    assert plan(np.array([0, 1000, 1200], np.int32)) == up.UP_OK
    assert plan(np.array([0, 99, 400], np.int32)) == up.UP_ERR_SHAPE      # fewer keys than tokens
    assert plan(np.array([5, 105, 305], np.int32)) == up.UP_ERR_SHAPE     # does not start at zero
    assert up.lib().uniprefill_plan_chunked(ctypes.byref(p), up.ptr(cu), None, up.ptr(ratio), None, None,
                                            None) == up.UP_ERR_NULL


def test_compact_column_rejects_bad_arguments():
    L = up.lib()
    fake = ctypes.c_void_p(0x1000)
    call = lambda col, eb, idx, cap, out: L.uniprefill_compact_column(col, eb, idx, ctypes.c_int64(cap), None, out, None)
    assert call(fake, 2, fake, 10, fake) == up.UP_ERR_UNSUPPORTED
    assert call(fake, 8, fake, -1, fake) == up.UP_ERR_RANGE
    assert call(fake, 8, fake, 0, fake) == up.UP_OK            # nothing to do, nothing launched
    assert call(None, 8, fake, 10, fake) == up.UP_ERR_NULL
    assert call(fake, 8, None, 10, fake) == up.UP_ERR_NULL
    assert call(fake, 8, fake, 10, None) == up.UP_ERR_NULL
    assert call(ctypes.c_void_p(0x1004), 8, fake, 10, fake) == up.UP_ERR_ALIGN
    assert call(fake, 4, fake, 10, ctypes.c_void_p(0x1002)) == up.UP_ERR_ALIGN


def test_seqused_rejects_bad_arguments():
    L = up.lib()
    fake = ctypes.c_void_p(0x1000)
    layers = lambda *v: up.ptr(np.array(v, np.int32))
    call = lambda lay, nd, ret, kv, orig, R, nl, out: L.uniprefill_seqused(lay, nd, ret, kv, orig, R, nl, out, None)
    assert call(layers(1, 3), 2, fake, fake, fake, 0, 6, fake) == up.UP_OK           # no request: nothing launched
    assert call(layers(3, 1), 2, fake, fake, fake, 4, 6, fake) == up.UP_ERR_RANGE    # not ascending
    assert call(layers(1, 1), 2, fake, fake, fake, 4, 6, fake) == up.UP_ERR_RANGE
    assert call(layers(-1), 1, fake, fake, fake, 4, 6, fake) == up.UP_ERR_RANGE
    assert call(None, 2, fake, fake, fake, 4, 6, fake) == up.UP_ERR_NULL
    assert call(layers(1, 3), 2, None, fake, fake, 4, 6, fake) == up.UP_ERR_NULL
    assert call(layers(1, 3), 2, fake, None, fake, 4, 6, fake) == up.UP_ERR_NULL
    assert call(layers(1, 3), 2, fake, fake, fake, 4, 6, None) == up.UP_ERR_NULL
    assert call(layers(1, 3), -1, fake, fake, fake, 4, 6, fake) == up.UP_ERR_RANGE
    assert call(layers(*range(65)), 65, fake, fake, fake, 4, 6, fake) == up.UP_ERR_UNSUPPORTED
    assert call(layers(1), 1, fake, fake, fake, 4, 70000, fake) == up.UP_ERR_RANGE


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                         text=True, timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr and res.stdout.strip() == ""


def test_paged_entries_reject_bad_block_tables():
    L = up.lib()
    fake = ctypes.c_void_p(0x1000)
    cu = np.array([0, 100, 300], np.int32)
    cu_k = np.array([0, 1000, 1200], np.int32)
    p = _params(num_seqs=2, total_tokens=300)
    odd = ctypes.c_void_p(0x1010)      # a workspace that is not 256-aligned: the last check before any launch
    def score(table, stride, B):
        return L.uniprefill_score_paged(ctypes.byref(p), fake, fake, fake, up.ptr(cu), fake, up.ptr(cu_k), table,
                                        ctypes.c_int64(stride), B, fake, odd, ctypes.c_size_t(1 << 30), None)
    assert score(None, 64, 16) == up.UP_ERR_NULL
    assert score(fake, 64, 0) == up.UP_ERR_RANGE
    assert score(fake, 62, 16) == up.UP_ERR_SHAPE          # 1000 keys need 63 blocks of 16
    assert score(fake, -1, 16) == up.UP_ERR_RANGE
    # the table is long enough with 63 entries: the next complaint is the workspace's alignment
    assert score(fake, 63, 16) == up.UP_ERR_ALIGN


def test_keep_mask_rejects_bad_arguments():
    L = up.lib()
    fake = ctypes.c_void_p(0x1000)
    call = lambda idx, cap, T, out: L.uniprefill_keep_mask(idx, ctypes.c_int64(cap), None, ctypes.c_int64(T), out, None)
    assert call(fake, 5, 0, fake) == up.UP_ERR_RANGE        # more kept rows than tokens
    assert call(fake, -1, 10, fake) == up.UP_ERR_RANGE
    assert call(fake, 0, 0, fake) == up.UP_OK               # nothing to do, nothing launched
    assert call(fake, 5, 10, None) == up.UP_ERR_NULL
    assert call(None, 5, 10, fake) == up.UP_ERR_NULL


def test_fused_lse_rejects_bad_arguments():
    L = up.lib()
    fake = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1010)
    cu = np.array([0, 100, 300], np.int32)
    cu_k = np.array([0, 1000, 1200], np.int32)
    ratio = np.array([0.5, 0.5], np.float32)
    p = _params(num_seqs=2, total_tokens=300)
    def call(lse=fake, stride=300, ckd=None, ckh=None, table=None, ws=odd):
        return L.uniprefill_fused_lse(ctypes.byref(p), fake, fake, lse, ctypes.c_int64(stride), fake, None, fake, up.ptr(cu),
                                      ckd, ckh, table, ctypes.c_int64(64), 16, fake, up.ptr(ratio), fake, None, fake, fake,
                                      None, ws, ctypes.c_size_t(1 << 30), None)
    assert call(lse=None) == up.UP_ERR_NULL
    assert call(lse=ctypes.c_void_p(0x1002)) == up.UP_ERR_ALIGN
    assert call(ckd=fake) == up.UP_ERR_NULL                       # device offsets without the host copy
    assert call(table=fake) == up.UP_ERR_NULL                     # a block table without key counts
    assert call(stride=299) == up.UP_ERR_SHAPE                    # heads of lse overlap
    assert call(ckd=fake, ckh=up.ptr(np.array([0, 99, 400], np.int32))) == up.UP_ERR_SHAPE
    assert call(ckd=fake, ckh=up.ptr(cu_k), table=fake) == up.UP_ERR_ALIGN    # all fine up to the odd workspace
    assert call() == up.UP_ERR_ALIGN


def test_scores_from_partials_rejects_bad_arguments():
    L = up.lib()
    fake = ctypes.c_void_p(0x1000)
    call = lambda parts, n, stride, T, heads, out: L.uniprefill_scores_from_partials(parts, n, ctypes.c_int64(stride), fake, 2, T,
                                                                                      128, heads, out, None)
    assert call(fake, 0, 100, 100, 8, fake) == up.UP_ERR_RANGE
    assert call(fake, 2, 99, 100, 8, fake) == up.UP_ERR_RANGE       # the parts would overlap
    assert call(fake, 2, 100, 100, 0, fake) == up.UP_ERR_RANGE
    assert call(fake, 2, 100, 0, 8, fake) == up.UP_OK               # nothing to do, nothing launched
    assert call(None, 2, 100, 100, 8, fake) == up.UP_ERR_NULL
    assert call(fake, 2, 100, 100, 8, None) == up.UP_ERR_NULL
    assert call(ctypes.c_void_p(0x1004), 2, 100, 100, 8, fake) == up.UP_ERR_ALIGN


def test_every_export_declares_its_argument_types():
    """No entry point is left to ctypes' default int conversion (which would truncate a
    size_t or an int64 argument to 32 bits)."""
    L = up.lib()
    for name in up.EXPORTS:
        fn = getattr(L, name)
        assert fn.argtypes is not None, name
    header = open(os.path.join(ROOT, "include", "uniprefill.h")).read()
    # the number of declared parameters equals the number of argtypes
    for name in up.EXPORTS:
        m = re.search(r"\b" + name + r"\s*\(([^;]*?)\)\s*;", header, re.S)
        assert m, name
        n_params = len([a for a in m.group(1).split(",") if a.strip()])
        assert n_params == len(getattr(L, name).argtypes), (name, n_params, len(getattr(L, name).argtypes))


def test_a_short_workspace_is_refused_through_every_wrapper_that_takes_one():
    """Sizes of 2 GiB and more reach the library intact (size_t), and a workspace that is too
    small comes back as UP_ERR_WORKSPACE through the chunked, paged and lse wrappers too."""
    cu = np.array([0, 1000], np.int32)
    cu_k = np.array([0, 3000], np.int32)
    ratio = np.array([0.5], np.float32)
    fake = 0x1000
    table = 0x2000
    p = _params()
    W = up.UP_ERR_WORKSPACE
    big = (1 << 32) + 16            # would read as 16 if truncated to 32 bits: the library must see the real size
    for ws_bytes in (16,):            # (only refusals are exercised: a call that passed every check would launch)
        assert up.uniprefill_score_chunked(p, fake, fake, fake, cu, fake, cu_k, fake, fake, ws_bytes, stream=0, check=False) == W
        assert up.uniprefill_score_paged(p, fake, fake, fake, cu, fake, cu_k, table, 256, 16, fake, fake, ws_bytes,
                                         stream=0, check=False) == W
        assert up.uniprefill_fused_chunked(p, fake, fake, fake, None, fake, cu, fake, cu_k, fake, ratio, fake, None, fake,
                                           fake, None, fake, ws_bytes, stream=0, check=False) == W
        assert up.uniprefill_fused_paged(p, fake, fake, fake, None, fake, cu, fake, cu_k, table, 256, 16, fake, ratio, fake,
                                         None, fake, fake, None, fake, ws_bytes, stream=0, check=False) == W
        assert up.uniprefill_score_lse(p, fake, fake, fake, 1000, fake, cu, None, None, None, 0, 16, fake, fake, ws_bytes,
                                       stream=0, check=False) == W
        assert up.uniprefill_fused_lse(p, fake, fake, fake, 1000, fake, None, fake, cu, None, None, None, 0, 16, fake, ratio,
                                       fake, None, fake, fake, None, fake, ws_bytes, stream=0, check=False) == W
        assert up.uniprefill_score_partial(p, fake, fake, fake, cu, None, None, fake, fake, ws_bytes, stream=0,
                                           check=False) == W
        assert up.uniprefill_select_top_p_chunked(p, fake, fake, cu, fake, cu_k, fake, ratio, fake, fake, fake, 8,
                                                  stream=0, check=False) == W
    # a size above 4 GiB is not truncated on its way in: with a misaligned workspace pointer the
    # call gets past the size check (truncated it would fail it) and is refused for the alignment
    assert up.uniprefill_score_chunked(p, fake, fake, fake, cu, fake, cu_k, fake, 0x1010, big, stream=0,
                                       check=False) == up.UP_ERR_ALIGN


def test_fused_static_refuses_what_its_scratch_cannot_hold():
    """The call that allocates nothing checks its arguments and the size of its static scratch
    buffer on the host, before it touches the device."""
    fake = 0x1000
    # 3000 short sequences of 350 tokens: the plan asks for more than the static buffer
    R = 3000
    cu = (np.arange(R + 1) * 350).astype(np.int32)
    ratio = np.full(R, 0.5, np.float32)
    p = _params(num_seqs=R, total_tokens=int(cu[-1]), num_q_heads=32, num_kv_heads=8, hidden_dim=256)
    _, _, _, ws = up.uniprefill_plan(p, cu, ratio)
    assert ws > up.STATIC_SCRATCH_BYTES
    call = lambda p_, cu_, ratio_: up.uniprefill_fused_static(p_, fake, fake, fake, None, fake, cu_, fake, ratio_, fake, None,
                                                              fake, fake, None, stream=0, check=False)
    assert call(p, cu, ratio) == up.UP_ERR_SCRATCH
    # argument errors come first, as in the other entries
    small = _params()
    cu1 = np.array([0, 1000], np.int32)
    assert call(small, np.array([0, 999], np.int32), np.array([0.5], np.float32)) == up.UP_ERR_SHAPE
    assert call(small, cu1, np.array([1.5], np.float32)) == up.UP_ERR_RANGE
    assert call(_params(head_dim=96), cu1, np.array([0.5], np.float32)) == up.UP_ERR_UNSUPPORTED
    with pytest.raises(up.UniPrefillError, match="static scratch"):
        up.uniprefill_fused_static(p, fake, fake, fake, None, fake, cu, fake, ratio, fake, None, fake, fake, None, stream=0)

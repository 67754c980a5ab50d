"""GPU test of the entry point that allocates nothing (uniprefill_fused_static): its outputs
equal those of uniprefill_fused bit for bit, on two calls in a row through the C ABI, the
second with a smaller batch (the static scratch buffer then still holds the first call's
contents), and the device's free memory does not change across a call."""
import numpy as np
import pytest
import torch

import paper_2605_06221_amd as up
import workloads
from gpu_util import DeviceBatch, oracle_run

pytestmark = pytest.mark.gpu


def _fused_static(b, want_scores=True):
    return up.uniprefill_fused_static(b.p, b.q, b.k, b.hidden, b.pos, b.cu, b.cu_host, b.ratio, b.ratio_host,
                                      b.hidden_out, b.pos_out, b.kept_idx, b.new_cu,
                                      b.scores if want_scores else None)


def _same(a, b):
    ra, rb = a.results(), b.results()
    for key in ("kept_idx", "new_cu_seqlens", "hidden_out", "pos_out"):
        np.testing.assert_array_equal(ra[key], rb[key], err_msg=key)
    # the same kernels on the same inputs: the scores are the same bits
    np.testing.assert_array_equal(ra["scores"].view(np.uint32), rb["scores"].view(np.uint32))
    assert a.canaries_intact() and b.canaries_intact()
    return rb


def test_fused_static_equals_fused_on_two_calls_in_a_row():
    print("no-alloc entry: first call, 5 sequences, 23.7k tokens", flush=True)
    big = workloads.make_custom(name="static_big", seed=91, lengths=[9000, 1, 5000, 700, 9000],
                                keep_ratio=[0.3, 0.5, 0.45, 1.0, 0.2], hidden_dim=512, num_q_heads=16, num_kv_heads=4,
                                block_size=64)
    a, b = DeviceBatch(big), DeviceBatch(big)
    assert a.ws_bytes <= up.STATIC_SCRATCH_BYTES
    a.fused()
    _fused_static(b)
    _same(a, b)

    print("no-alloc entry: second call, smaller batch, other shape", flush=True)
    small = workloads.make_custom(name="static_small", seed=92, lengths=[1500, 300, 2100], keep_ratio=[0.5, 0.25, 0.4],
                                  hidden_dim=256, num_q_heads=8, num_kv_heads=8, block_size=128)
    c, d = DeviceBatch(small), DeviceBatch(small)
    c.fused()
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    _fused_static(d)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before        # nothing was allocated or freed
    got = _same(c, d)
    # ... and both equal the oracle (indices, rows, positions bit for bit; scores within 1e-2 relative)
    ref = oracle_run(small)
    np.testing.assert_array_equal(got["kept_idx"], ref["kept_idx"])
    np.testing.assert_array_equal(got["new_cu_seqlens"], ref["new_cu_seqlens"])
    np.testing.assert_array_equal(got["hidden_out"], ref["hidden_out"])
    np.testing.assert_array_equal(got["pos_out"], ref["pos_out"])
    want = ref["scores"].astype(np.float64)
    assert (np.abs(got["scores"] - want) <= 1e-2 * want + 2.0 ** -64).all()

    print("no-alloc entry: scores not wanted; a batch without tokens", flush=True)
    e = DeviceBatch(small)
    _fused_static(e, want_scores=False)
    re = e.results()
    np.testing.assert_array_equal(re["kept_idx"], ref["kept_idx"])
    np.testing.assert_array_equal(re["hidden_out"], ref["hidden_out"])
    assert (e.scores == -7.0).all()
    empty = workloads.make_custom(name="static_empty", seed=93, lengths=[0, 0], keep_ratio=[0.5, 0.5], hidden_dim=256,
                                  num_q_heads=8, num_kv_heads=8, block_size=128)
    f = DeviceBatch(empty)
    _fused_static(f)
    assert (f.results()["new_cu_seqlens"] == 0).all() and f.canaries_intact()

"""Helpers for the GPU parity tests: move a seeded workload to the device and call
the C ABI through the thin binding.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

import paper_2605_06221_amd as up


def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    """uint16 bf16 bit patterns -> bf16 tensor on the GPU (bit-exact)."""
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def host_bits(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor -> uint16 bit patterns on the host."""
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


class DeviceBatch:
    """A workload resident in HBM plus output buffers sized by uniprefill_plan."""

    def __init__(self, w, softmax_scale: float = 0.0, canary: bool = True, qk_f32=None, paged=None):
        """qk_f32 = (q, k) float32 arrays of the workload's shapes: score from those instead of
        the workload's bf16 tensors (the fp32 operand path).
        paged = (k_cache bits, block_table, kv_block_size): the keys sit in a paged cache."""
        self.w = w
        self.cu_host = np.ascontiguousarray(w.cu_seqlens, dtype=np.int32)
        self.ratio_host = np.ascontiguousarray(w.keep_ratio, dtype=np.float32)
        self.p = up.make_params(
            num_seqs=w.num_seqs, total_tokens=w.total_tokens, block_size=w.block_size, n_obs=w.n_obs,
            n_sink=w.n_sink, num_q_heads=w.num_q_heads, num_kv_heads=w.num_kv_heads, head_dim=w.head_dim,
            hidden_dim=w.hidden_dim, softmax_scale=softmax_scale,
            qk_dtype=up.UP_BF16 if qk_f32 is None else up.UP_F32)
        self.ctx = w.cu_seqlens_k is not None      # the requests follow earlier context
        if self.ctx:
            self.cu_k_host = np.ascontiguousarray(w.cu_seqlens_k, dtype=np.int32)
            self.cu_k = torch.from_numpy(self.cu_k_host).cuda()
            _, self.new_cu_plan, self.total_kept, self.ws_bytes = up.uniprefill_plan_chunked(
                self.p, self.cu_host, self.cu_k_host, self.ratio_host)
        else:
            _, self.new_cu_plan, self.total_kept, self.ws_bytes = up.uniprefill_plan(self.p, self.cu_host, self.ratio_host)
        T, d = w.total_tokens, w.hidden_dim
        if qk_f32 is None:
            self.q = dev_bf16(w.q)
            self.k = dev_bf16(w.k)
        else:
            self.q = torch.from_numpy(np.ascontiguousarray(qk_f32[0], dtype=np.float32)).cuda()
            self.k = torch.from_numpy(np.ascontiguousarray(qk_f32[1], dtype=np.float32)).cuda()
        self.paged = None
        if paged is not None:
            self.k = dev_bf16(paged[0])
            self.paged = (torch.from_numpy(np.ascontiguousarray(paged[1], dtype=np.int32)).cuda(), int(paged[1].shape[1]),
                          int(paged[2]))
        self.hidden = dev_bf16(w.hidden)
        self.pos = torch.from_numpy(w.pos).cuda()
        self.cu = torch.from_numpy(self.cu_host).cuda()
        self.ratio = torch.from_numpy(self.ratio_host).cuda()
        self.workspace = torch.empty(self.ws_bytes + 256, dtype=torch.uint8, device="cuda")
        self.pad = 64 if canary else 0     # canary rows/entries after every output
        K = self.total_kept
        self.hidden_out = torch.full((K + self.pad, d), -7.0, dtype=torch.bfloat16, device="cuda")
        self.pos_out = torch.full((K + self.pad,), -77, dtype=torch.int32, device="cuda")
        self.kept_idx = torch.full((K + self.pad,), -77, dtype=torch.int32, device="cuda")
        self.new_cu = torch.full((w.num_seqs + 1 + self.pad,), -77, dtype=torch.int32, device="cuda")
        self.scores = torch.full((T + self.pad,), -7.0, dtype=torch.float32, device="cuda")

    # ---- entry points -------------------------------------------------------
    def fused(self, want_scores=True, stream=None):
        if self.paged is not None:
            return up.uniprefill_fused_paged(self.p, self.q, self.k, self.hidden, self.pos, self.cu, self.cu_host,
                                             self.cu_k, self.cu_k_host, self.paged[0], self.paged[1], self.paged[2],
                                             self.ratio, self.ratio_host, self.hidden_out, self.pos_out,
                                             self.kept_idx, self.new_cu, self.scores if want_scores else None,
                                             self.workspace, self.ws_bytes, stream=stream)
        if self.ctx:
            return up.uniprefill_fused_chunked(self.p, self.q, self.k, self.hidden, self.pos, self.cu, self.cu_host,
                                               self.cu_k, self.cu_k_host, self.ratio, self.ratio_host,
                                               self.hidden_out, self.pos_out, self.kept_idx, self.new_cu,
                                               self.scores if want_scores else None, self.workspace,
                                               self.ws_bytes, stream=stream)
        return up.uniprefill_fused(self.p, self.q, self.k, self.hidden, self.pos, self.cu, self.cu_host,
                                   self.ratio, self.ratio_host, self.hidden_out, self.pos_out, self.kept_idx,
                                   self.new_cu, self.scores if want_scores else None, self.workspace,
                                   self.ws_bytes, stream=stream)

    def fused_lse(self, lse_dev, want_scores=True):
        """The fused call with the rows' normalisers given (lse_dev: float [Hq, T] on the device)."""
        table, stride, B = self.paged if self.paged is not None else (None, 0, 16)
        return up.uniprefill_fused_lse(self.p, self.q, self.k, lse_dev, int(lse_dev.shape[1]), self.hidden, self.pos,
                                       self.cu, self.cu_host, self.cu_k if self.ctx else None,
                                       self.cu_k_host if self.ctx else None, table, stride, B, self.ratio,
                                       self.ratio_host, self.hidden_out, self.pos_out, self.kept_idx, self.new_cu,
                                       self.scores if want_scores else None, self.workspace, self.ws_bytes)

    def score(self):
        if self.paged is not None:
            return up.uniprefill_score_paged(self.p, self.q, self.k, self.cu, self.cu_host, self.cu_k, self.cu_k_host,
                                             self.paged[0], self.paged[1], self.paged[2], self.scores,
                                             self.workspace, self.ws_bytes)
        if self.ctx:
            return up.uniprefill_score_chunked(self.p, self.q, self.k, self.cu, self.cu_host, self.cu_k,
                                               self.cu_k_host, self.scores, self.workspace, self.ws_bytes)
        return up.uniprefill_score(self.p, self.q, self.k, self.cu, self.cu_host, self.scores,
                                   self.workspace, self.ws_bytes)

    def select(self, scores_dev):
        if self.ctx:
            return up.uniprefill_select_chunked(self.p, scores_dev, self.cu, self.cu_host, self.cu_k, self.cu_k_host,
                                                self.ratio, self.ratio_host, self.kept_idx, self.new_cu)
        return up.uniprefill_select(self.p, scores_dev, self.cu, self.cu_host, self.ratio, self.ratio_host,
                                    self.kept_idx, self.new_cu)

    # ---- results ------------------------------------------------------------
    def results(self):
        torch.cuda.synchronize()
        K, R, T = self.total_kept, self.w.num_seqs, self.w.total_tokens
        return {
            "kept_idx": self.kept_idx[:K].cpu().numpy(),
            "new_cu_seqlens": self.new_cu[:R + 1].cpu().numpy(),
            "hidden_out": host_bits(self.hidden_out[:K]),
            "pos_out": self.pos_out[:K].cpu().numpy(),
            "scores": self.scores[:T].cpu().numpy(),
        }

    def canaries_intact(self):
        torch.cuda.synchronize()
        if not self.pad:
            return True
        K, R, T = self.total_kept, self.w.num_seqs, self.w.total_tokens
        return bool((self.hidden_out[K:] == -7.0).all() and (self.pos_out[K:] == -77).all()
                    and (self.kept_idx[K:] == -77).all() and (self.new_cu[R + 1:] == -77).all()
                    and (self.scores[T:] == -7.0).all())


def oracle_run(w, scale=None):
    """The oracle's end-to-end result for a workload (imports the oracle lazily)."""
    import oracle
    import workloads
    qf = _LazyQ(w.q)      # the oracle slices only the window rows; upcast those on demand
    kf = workloads.bf16_bits_to_f32(w.k)
    if w.cu_seqlens_k is not None:
        return oracle.sparsify_with_context(qf, kf, w.hidden, w.pos, w.cu_seqlens, w.cu_seqlens_k, w.keep_ratio,
                                            block_size=w.block_size, n_obs=w.n_obs, n_sink=w.n_sink, scale=scale)
    return oracle.sparsify(qf, kf, w.hidden, w.pos, w.cu_seqlens, w.keep_ratio, block_size=w.block_size,
                           n_obs=w.n_obs, n_sink=w.n_sink, scale=scale)


class _LazyQ:
    """Array-like view of w.q that upcasts bf16 bits to float32 only for the rows read."""

    def __init__(self, bits):
        self.bits = bits
        self.shape = bits.shape

    def __getitem__(self, item):
        import workloads
        return workloads.bf16_bits_to_f32(self.bits[item])


def score_margin_report(res_oracle, w):
    """Smallest relative gap, over all blocks, between the last kept and the first
    dropped non-forced oracle score (fp64), ignoring exact ties of quantised scores."""
    import oracle
    o = res_oracle["scores64"]
    s32 = res_oracle["scores"]
    kept = np.zeros(w.total_tokens, bool)
    kept[res_oracle["kept_idx"]] = True
    best = np.inf
    cu = w.cu_seqlens
    sinks = [w.n_sink] * w.num_seqs if w.cu_seqlens_k is None else oracle.sinks_in_chunk(cu, w.cu_seqlens_k, w.n_sink)
    for r in range(w.num_seqs):
        N = int(cu[r + 1] - cu[r])
        f = oracle.forced_mask(N, w.n_obs, int(sinks[r]))
        for lo in range(0, N, w.block_size):
            sl = slice(int(cu[r]) + lo, int(cu[r]) + min(N, lo + w.block_size))
            kk = kept[sl] & ~f[lo:lo + w.block_size]
            dd = ~kept[sl]
            if kk.any() and dd.any():
                a = o[sl][kk].min()
                b = o[sl][dd].max()
                a32 = s32[sl][kk].min()
                b32 = s32[sl][dd].max()
                if a32 != b32 and a > 0:
                    best = min(best, (a - b) / a)
    return best

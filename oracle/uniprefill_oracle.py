"""CPU oracle for the UniPrefill block-wise token-sparsification operator.

TEST INFRASTRUCTURE ONLY.  This is a plain, slow, fp64 numpy statement of what
the operator computes.  Only the test-suite, the smoke check and the benchmark's
``cpu_baseline`` leg may import it; the product path never does, and it shares
no code with the HIP kernels.

What is computed, step by step (paper section / equation in brackets):

1. token importance [Token Importance Estimation, Eq. 2-3; kernel-design
   paragraph of "Fused Kernel and vLLM Integration"]: for every sequence of the
   packed batch, every query head and each of the last n query rows, the
   causal softmax over the *whole* visible key sequence of q.k/sqrt(d_k);
   the per-token score is the mean of those attention weights over the n rows
   and over the heads.
2. quantisation: the score is carried as a 32-bit float (the key encoding of
   Eq. 14 acts on float bits); means below 2**-64 are floored to +0 so that
   fp32 underflow is a *defined* tie rather than an accident.
3. block partition [Token Importance Estimation: non-overlapping blocks of G
   tokens per sequence, ragged tail] and forced retention of the first A
   tokens and the last n tokens [Top-p Token Selection, last sentence; expansion
   kernel in the kernel-design paragraph].
4. block-local top-k by keep ratio (the selection rule of this build's target;
   the paper's own block-level top-p rule is ``select_blocks_top_p`` in fp64 and
   ``select_tokens_top_p`` on the quantised scores, below),
   ordered with the packed integer key of Eq. 14, index complemented so that a
   descending order prefers the lower index among equal scores.
5. compaction of hidden states / position ids onto the kept rows [Sparsity
   Propagation, Eq. 7] and the inverse scatter [Eq. 8].

6. chunks that follow earlier context (chunked prefill, keys of earlier tokens
   cached): ``importance_scores_with_context`` and the selection with the sinks
   that fall inside the chunk; pinned by hand-worked rationals, the harmonic
   closed form, a library softmax, and by being the tail of the whole-sequence
   scores (tests/test_oracle_context.py).

Pins (see tests/test_oracle_*.py): softmax row sums, harmonic closed form for
Q = 0, a library attention routine with V = I, shift/permutation invariances,
exact kept counts, brute-force subset enumeration, identity at ratio 1,
gather/scatter round trips, varlen == concatenation, monotonicity of phi.
End-to-end model accuracy (RULER) is **parity unpinned**: it needs the dataset
and model weights, which are not available.
"""
from __future__ import annotations

import math

import numpy as np

SCORE_FLOOR = 2.0 ** -64


# --------------------------------------------------------------------------- #
# 1. token importance  (Eq. 2, Eq. 3; causal mask per the kernel-design text)
# --------------------------------------------------------------------------- #
def importance_scores(q, k, cu_seqlens, *, n_obs, scale=None):
    """Per-token importance o_i in float64 (not yet quantised).

    q : [T, Hq, D] float array (only the last min(n_obs, N_r) rows of each
        sequence are read), k : [T, Hkv, D] float array, cu_seqlens : [R+1].
    Query head h reads kv head h // (Hq // Hkv).
    """
    k = np.asarray(k)                       # q is only sliced (window rows), never read whole
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    assert k.shape[0] == T and k.shape[2] == D and Hq % Hkv == 0
    group = Hq // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(D)          # Eq. 2: logits divided by sqrt(d_k)
    o = np.zeros(T, dtype=np.float64)
    for r in range(len(cu) - 1):
        c0, c1 = int(cu[r]), int(cu[r + 1])
        N = c1 - c0
        if N == 0:
            continue
        n_eff = min(int(n_obs), N)
        Kr = k[c0:c1].astype(np.float64)                 # [N, Hkv, D]
        Qw = np.asarray(q[c1 - n_eff:c1], dtype=np.float64)   # [n_eff, Hq, D]
        qpos = np.arange(N - n_eff, N)                   # local position of each query row
        visible = np.arange(N)[None, :] <= qpos[:, None]  # key i visible to row j iff i <= j
        colsum = np.zeros(N, dtype=np.float64)
        for h in range(Hq):
            S = scale * (Qw[:, h, :] @ Kr[:, h // group, :].T)   # partial GEMM, [n_eff, N]
            S[~visible] = -np.inf
            S -= S.max(axis=1, keepdims=True)
            P = np.exp(S)
            P /= P.sum(axis=1, keepdims=True)            # softmax over the complete key sequence
            colsum += P.sum(axis=0)
        o[c0:c1] = colsum / (n_eff * Hq)                 # Eq. 3 mean over rows; mean over heads
    return o


def quantise_scores(o):
    """fp64 score -> the fp32 value selection sees; values below 2**-64 become +0."""
    o = np.asarray(o, dtype=np.float64)
    out = o.astype(np.float32)
    out[o < SCORE_FLOOR] = np.float32(0.0)
    return out


# --------------------------------------------------------------------------- #
# 2. order-preserving key encoding  (Eq. 14)
# --------------------------------------------------------------------------- #
def phi(x):
    """Monotone map from float32 to uint32: flip the sign bit of non-negative
    floats, flip all bits of negative floats (sign taken from the sign bit)."""
    bits = np.asarray(x, dtype=np.float32).view(np.uint32)
    neg = (bits >> np.uint32(31)) == 1
    return np.where(neg, bits ^ np.uint32(0xFFFFFFFF), bits ^ np.uint32(0x80000000)).astype(np.uint32)


def packed_keys(scores_f32, forced, block_size):
    """(phi(score) << 32) | (G-1-local_index) for the tokens of one block.

    Forced tokens take the all-ones upper word, above every finite score.  The
    paper packs the plain index; the index is complemented here so that the
    descending sort breaks score ties toward the lower index."""
    s = np.asarray(scores_f32, dtype=np.float32)
    L = s.shape[0]
    hi = phi(s).astype(np.uint64)
    hi = np.where(np.asarray(forced, dtype=bool), np.uint64(0xFFFFFFFF), hi)
    lo = (np.uint64(block_size - 1) - np.arange(L, dtype=np.uint64))
    return (hi << np.uint64(32)) | lo


# --------------------------------------------------------------------------- #
# 3. block partition, forced tokens, kept counts
# --------------------------------------------------------------------------- #
def forced_mask(N, n_obs, n_sink):
    """True for the first A tokens and the last n tokens of a length-N sequence."""
    i = np.arange(N)
    return (i < n_sink) | (i >= N - n_obs)


def kept_count(L, F, rho):
    """Tokens kept in a block of L tokens, F of them forced, at keep ratio rho.

    rho is a float32 widened to double; rho*L is then exact, so the ceiling is
    unambiguous."""
    want = math.ceil(float(np.float32(rho)) * L)
    want = min(L, max(1, want))
    return max(want, F)


def block_kept_counts(N, block_size, n_obs, n_sink, rho):
    """k_g for every block of one sequence."""
    f = forced_mask(N, n_obs, n_sink)
    out = []
    for lo in range(0, N, block_size):
        hi = min(N, lo + block_size)
        out.append(kept_count(hi - lo, int(f[lo:hi].sum()), rho))
    return out


def plan(cu_seqlens, keep_ratio, *, block_size, n_obs, n_sink):
    """Closed-form output layout: new_cu_seqlens (int32 [R+1])."""
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    new_cu = np.zeros(len(cu), dtype=np.int32)
    for r in range(len(cu) - 1):
        N = int(cu[r + 1] - cu[r])
        new_cu[r + 1] = new_cu[r] + sum(block_kept_counts(N, block_size, n_obs, n_sink, keep_ratio[r]))
    return new_cu


# --------------------------------------------------------------------------- #
# 4. block-local top-k selection
# --------------------------------------------------------------------------- #
def select_tokens(scores_f32, cu_seqlens, keep_ratio, *, block_size, n_obs, n_sink):
    """kept_idx (int32, ascending global packed row ids) and new_cu_seqlens."""
    s = np.asarray(scores_f32, dtype=np.float32)
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    kept = []
    new_cu = np.zeros(len(cu), dtype=np.int32)
    for r in range(len(cu) - 1):
        c0, c1 = int(cu[r]), int(cu[r + 1])
        N = c1 - c0
        f = forced_mask(N, n_obs, n_sink)
        count = 0
        for lo in range(0, N, block_size):
            hi = min(N, lo + block_size)
            fb = f[lo:hi]
            kg = kept_count(hi - lo, int(fb.sum()), keep_ratio[r])
            keys = packed_keys(s[c0 + lo:c0 + hi], fb, block_size)
            order = np.argsort(keys, kind="stable")[::-1]          # descending, keys are unique
            chosen = np.sort(order[:kg])
            kept.append((c0 + lo + chosen).astype(np.int32))
            count += kg
        new_cu[r + 1] = new_cu[r] + count
    kept_idx = np.concatenate(kept) if kept else np.zeros(0, dtype=np.int32)
    return kept_idx.astype(np.int32), new_cu


# --------------------------------------------------------------------------- #
# 5. compaction and its inverse  (Eq. 7, Eq. 8)
# --------------------------------------------------------------------------- #
def compact(hidden, pos, kept_idx):
    """Rows of hidden / entries of pos at kept_idx (bit copies)."""
    idx = np.asarray(kept_idx, dtype=np.int64)
    return np.asarray(hidden)[idx].copy(), np.asarray(pos)[idx].copy()


def scatter(hidden_compact, kept_idx, hidden_full):
    """Write compact rows back at kept_idx; every other row keeps its old state."""
    out = np.array(hidden_full, copy=True)
    out[np.asarray(kept_idx, dtype=np.int64)] = np.asarray(hidden_compact)
    return out


# --------------------------------------------------------------------------- #
# whole path
# --------------------------------------------------------------------------- #
def sparsify(q, k, hidden, pos, cu_seqlens, keep_ratio, *, block_size, n_obs, n_sink, scale=None):
    """score -> quantise -> select -> compact.  Returns a dict of all products."""
    o = importance_scores(q, k, cu_seqlens, n_obs=n_obs, scale=scale)
    s32 = quantise_scores(o)
    kept_idx, new_cu = select_tokens(s32, cu_seqlens, keep_ratio,
                                     block_size=block_size, n_obs=n_obs, n_sink=n_sink)
    h_out, p_out = compact(hidden, pos, kept_idx)
    return {"scores64": o, "scores": s32, "kept_idx": kept_idx, "new_cu_seqlens": new_cu,
            "hidden_out": h_out, "pos_out": p_out}


# --------------------------------------------------------------------------- #
# the paper's own selection rule (block-level top-p, Eq. 4-5) -- next row
# --------------------------------------------------------------------------- #
def block_mass(o, N, block_size):
    """Attention mass captured by each block (sum of token scores; a constant
    1/G factor would cancel in the ratio of Eq. 5)."""
    return np.array([o[lo:min(N, lo + block_size)].sum() for lo in range(0, N, block_size)],
                    dtype=np.float64)


def select_blocks_top_p(o_seq, p, *, block_size, n_obs, n_sink):
    """Token keep-mask of one sequence under Eq. 5: the minimal prefix of
    score-sorted blocks whose cumulative mass reaches p of the total, lifted to
    tokens, with sinks and the query window always kept."""
    o_seq = np.asarray(o_seq, dtype=np.float64)
    N = o_seq.shape[0]
    b = block_mass(o_seq, N, block_size)
    order = np.argsort(-b, kind="stable")                # descending, ties to the lower block
    csum = np.cumsum(b[order])
    total = csum[-1]
    kstar = int(np.searchsorted(csum, p * total, side="left")) + 1
    kstar = min(kstar, len(b))
    keep_block = np.zeros(len(b), dtype=bool)
    keep_block[order[:kstar]] = True
    mask = np.repeat(keep_block, block_size)[:N]
    return mask | forced_mask(N, n_obs, n_sink)


# --------------------------------------------------------------------------- #
# block-level top-p on the quantised scores: the form a kernel can match bit for bit
# --------------------------------------------------------------------------- #
def block_mass_f32(scores_f32, N, block_size):
    """Block masses as 32-bit floats (the key encoding of Eq. 14 acts on float bits): the
    fp32 token scores of a block added one after the other in double, rounded once."""
    s = np.asarray(scores_f32, dtype=np.float32).astype(np.float64)
    out = []
    for lo in range(0, N, block_size):
        acc = 0.0
        for v in s[lo:min(N, lo + block_size)]:
            acc += float(v)
        out.append(np.float32(acc))
    return np.array(out, dtype=np.float32)


def top_p_block_keys(mass_f32):
    """(phi(mass) << 32) | (nb-1-g): the packed word of Eq. 14 for blocks, block index
    complemented so that a descending order puts the lower block first among equal masses."""
    b = np.asarray(mass_f32, dtype=np.float32)
    nb = b.shape[0]
    return (phi(b).astype(np.uint64) << np.uint64(32)) | (np.uint64(nb - 1) - np.arange(nb, dtype=np.uint64))


TOP_P_CHUNK = 64      # positions per chunk of the running sum below


def chunked_running_sum(values_f32):
    """Running sum in double of float32 values taken in the given order, in a fixed two-level
    shape (the paper thresholds "a cumulative sum" and states no precision, Eq. 5): the positions
    are cut into chunks of 64; inside a chunk the sum runs from zero, one addition after the
    other; the chunks' totals are added one after the other; the running sum at a position is
    (the sum of the earlier chunks' totals) + (its sum inside its chunk).  Up to 64 values this
    is the plain sequential sum.  Pure-Python loops: every addition is spelled out."""
    v = [float(x) for x in np.asarray(values_f32, dtype=np.float32)]
    run = []
    offset = 0.0                                  # total of the earlier chunks
    for lo in range(0, len(v), TOP_P_CHUNK):
        inside = 0.0
        for x in v[lo:lo + TOP_P_CHUNK]:
            inside = inside + x
            run.append(offset + inside)
        offset = offset + inside
    return np.array(run, dtype=np.float64)


def top_p_kept_blocks(mass_f32, p):
    """Boolean keep flag per block under Eq. 5: blocks in descending key order, running sum
    of their masses in double in that order (``chunked_running_sum``), k* the first
    position where the running sum reaches p times the total (the last running sum).  p is a
    float32 widened to double."""
    b = np.asarray(mass_f32, dtype=np.float32)
    nb = b.shape[0]
    order = np.argsort(top_p_block_keys(b), kind="stable")[::-1]
    run = chunked_running_sum(b[order])
    thr = float(np.float32(p)) * float(run[-1])
    kstar = int(np.count_nonzero(run < thr)) + 1                   # run is non-decreasing (masses >= 0)
    kstar = min(kstar, nb)
    keep = np.zeros(nb, dtype=bool)
    keep[order[:kstar]] = True
    return keep


def select_tokens_top_p(scores_f32, cu_seqlens, top_p, *, block_size, n_obs, n_sink):
    """kept_idx (ascending packed row ids) and new_cu_seqlens under the paper's rule:
    whole blocks chosen by cumulative mass (Eq. 4-5), sinks and query window always kept
    (last sentence of "Top-p Token Selection"; expansion kernel of the kernel-design paragraph)."""
    s = np.asarray(scores_f32, dtype=np.float32)
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    kept = []
    new_cu = np.zeros(len(cu), dtype=np.int32)
    for r in range(len(cu) - 1):
        c0, c1 = int(cu[r]), int(cu[r + 1])
        N = c1 - c0
        if N == 0:
            new_cu[r + 1] = new_cu[r]
            continue
        keep_block = top_p_kept_blocks(block_mass_f32(s[c0:c1], N, block_size), top_p[r])
        mask = np.repeat(keep_block, block_size)[:N] | forced_mask(N, n_obs, n_sink)
        idx = np.nonzero(mask)[0]
        kept.append((c0 + idx).astype(np.int32))
        new_cu[r + 1] = new_cu[r] + len(idx)
    kept_idx = np.concatenate(kept) if kept else np.zeros(0, dtype=np.int32)
    return kept_idx.astype(np.int32), new_cu


# --------------------------------------------------------------------------- #
# index maps across drop layers ("Sparsity Propagation Across All Layers")
# --------------------------------------------------------------------------- #
def keep_mask(kept_idx, total_tokens):
    """The token keep mask M in {0,1}^T that the index list stands for ("Top-p Token Selection";
    expansion kernel of the kernel-design paragraph): 1 at the kept packed rows."""
    m = np.zeros(int(total_tokens), dtype=np.uint8)
    for i in np.asarray(kept_idx, dtype=np.int64):
        m[i] = 1
    return m


def compose_index(outer_idx, inner_idx):
    """Index map of two successive drops: inner_idx selects rows of the stream that
    outer_idx had compacted, so row t of the twice-compacted stream is packed row
    outer_idx[inner_idx[t]] of the original batch (retained sets are nested: a token
    dropped at one layer stays out of every later layer)."""
    outer = np.asarray(outer_idx, dtype=np.int64)
    inner = np.asarray(inner_idx, dtype=np.int64)
    return outer[inner].astype(np.int32)


def retained_lengths(new_cu_seqlens):
    """Per-request retained length after a drop (the s_k^r of the drop history used for the
    per-layer KV length during decode)."""
    return np.diff(np.asarray(new_cu_seqlens, dtype=np.int64)).astype(np.int32)


# --------------------------------------------------------------------------- #
# serving-side metadata of a compacted stream ("vLLM scheduler integration")
# --------------------------------------------------------------------------- #
def kv_slot_mapping(pos_kept, new_cu_seqlens, block_table, kv_block_size):
    """Physical KV-cache slot of every retained token (Eq. 16): token i of request r at
    logical position p goes to block_table[r, p // B] * B + p % B."""
    pos = np.asarray(pos_kept, dtype=np.int64)
    cu = np.asarray(new_cu_seqlens, dtype=np.int64)
    bt = np.asarray(block_table, dtype=np.int64)
    B = int(kv_block_size)
    out = np.zeros(pos.shape[0], dtype=np.int64)
    for r in range(len(cu) - 1):
        for i in range(int(cu[r]), int(cu[r + 1])):
            p = int(pos[i])
            out[i] = bt[r, p // B] * B + p % B
    return out


def seqused(retained_len_at_last_drop, kv_len, orig_len):
    """KV length a layer sees during decode (Eq. 17): the length retained by the last drop
    before that layer plus the tokens appended since prefill."""
    s = np.asarray(retained_len_at_last_drop, dtype=np.int64)
    return (s + (np.asarray(kv_len, dtype=np.int64) - np.asarray(orig_len, dtype=np.int64))).astype(np.int32)


def seqused_per_layer(drop_layers, retained, kv_len, orig_len, num_layers):
    """Eq. 17 for every layer: int32 [num_layers, R].  ``drop_layers`` are the layers l_k of the drop
    events (ascending), ``retained[k][r]`` the length s_k^r request r kept at event k.  Layer l sees
    the length kept by the last event at a layer strictly before l -- the whole prompt if there is
    none -- plus the tokens appended since prefill."""
    drop_layers = [int(x) for x in drop_layers]
    kv = np.asarray(kv_len, dtype=np.int64)
    orig = np.asarray(orig_len, dtype=np.int64)
    retained = np.asarray(retained, dtype=np.int64).reshape(len(drop_layers), orig.shape[0])
    out = np.zeros((int(num_layers), orig.shape[0]), dtype=np.int32)
    for layer in range(int(num_layers)):
        before = [k for k, lk in enumerate(drop_layers) if lk < layer]
        s = retained[max(before)] if before else orig
        out[layer] = s + (kv - orig)
    return out


# --------------------------------------------------------------------------- #
# chunks that follow earlier context  (chunked prefill: keys of earlier tokens are cached)
# --------------------------------------------------------------------------- #
# The paper scores whole prompts; its serving integration (Fused Kernel and vLLM Integration)
# runs under continuous batching, where a long prompt arrives in chunks and the keys of the
# earlier chunks sit in the KV cache.  The reading taken here: the tokens of a chunk get the
# scores they would get if the sequence so far (earlier tokens + chunk) were scored with the
# window taken from the chunk's last min(n, N) tokens; selection blocks start at the chunk's
# first token; a chunk token is a sink when its position in the sequence so far is below A.
def importance_scores_with_context(q, k, cu_seqlens_q, cu_seqlens_k, *, n_obs, scale=None):
    """Per-token importance (float64) of the chunk tokens of every request.

    q : [T, Hq, D], the chunk tokens (only the last min(n_obs, N_r) rows of each request are
    read); k : [Tk, Hkv, D], for request r the keys of its P_r earlier tokens followed by the
    keys of its N_r chunk tokens (P_r + N_r = cu_seqlens_k[r+1] - cu_seqlens_k[r]).
    Chunk row j sits at position P_r + j and sees keys 0 .. P_r + j; the softmax runs over all
    of them (Eq. 2); chunk token i receives the mean weight of key P_r + i (Eq. 3)."""
    k = np.asarray(k)
    cq = np.asarray(cu_seqlens_q, dtype=np.int64)
    ck = np.asarray(cu_seqlens_k, dtype=np.int64)
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    assert k.shape[2] == D and Hq % Hkv == 0 and len(cq) == len(ck)
    group = Hq // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(D)
    o = np.zeros(T, dtype=np.float64)
    for r in range(len(cq) - 1):
        c0, c1 = int(cq[r]), int(cq[r + 1])
        k0, k1 = int(ck[r]), int(ck[r + 1])
        N, L = c1 - c0, k1 - k0
        P = L - N
        assert P >= 0
        if N == 0:
            continue
        n_eff = min(int(n_obs), N)
        Kr = k[k0:k1].astype(np.float64)                       # [L, Hkv, D]
        Qw = np.asarray(q[c1 - n_eff:c1], dtype=np.float64)    # [n_eff, Hq, D]
        qpos = np.arange(L - n_eff, L)                         # position of each window row
        visible = np.arange(L)[None, :] <= qpos[:, None]
        colsum = np.zeros(L, dtype=np.float64)
        for h in range(Hq):
            S = scale * (Qw[:, h, :] @ Kr[:, h // group, :].T)   # [n_eff, L]
            S[~visible] = -np.inf
            S -= S.max(axis=1, keepdims=True)
            W = np.exp(S)
            W /= W.sum(axis=1, keepdims=True)                  # over earlier and chunk keys alike
            colsum += W.sum(axis=0)
        o[c0:c1] = colsum[P:] / (n_eff * Hq)
    return o


def importance_scores_from_lse(q, k, lse, cu_seqlens_q, cu_seqlens_k, *, n_obs, scale=None):
    """The same scores when the softmax normaliser of every row is handed in instead of computed:
    ``lse[h, t]`` is the natural logarithm of the sum of exp(scale * <q_t, k_i>) over the keys that
    token t of head h sees (what an attention kernel returns next to its output).  The weight of
    key i for window row j is then exp(scale * <q_j, k_i> - lse[h, j]) (Eq. 2), and the score is
    the mean over rows and heads (Eq. 3).  ``cu_seqlens_k`` as in importance_scores_with_context
    (pass cu_seqlens_q when there is no earlier context); only the window rows of lse are read."""
    k = np.asarray(k)
    lse = np.asarray(lse, dtype=np.float64)
    cq = np.asarray(cu_seqlens_q, dtype=np.int64)
    ck = np.asarray(cu_seqlens_k, dtype=np.int64)
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    group = Hq // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(D)
    o = np.zeros(T, dtype=np.float64)
    for r in range(len(cq) - 1):
        c0, c1 = int(cq[r]), int(cq[r + 1])
        k0, k1 = int(ck[r]), int(ck[r + 1])
        N, L = c1 - c0, k1 - k0
        P = L - N
        if N == 0:
            continue
        n_eff = min(int(n_obs), N)
        Kr = k[k0:k1].astype(np.float64)
        Qw = np.asarray(q[c1 - n_eff:c1], dtype=np.float64)
        qpos = np.arange(L - n_eff, L)
        visible = np.arange(L)[None, :] <= qpos[:, None]
        colsum = np.zeros(L, dtype=np.float64)
        for h in range(Hq):
            S = scale * (Qw[:, h, :] @ Kr[:, h // group, :].T)
            W = np.exp(S - lse[h, c1 - n_eff:c1][:, None])
            W[~visible] = 0.0
            colsum += W.sum(axis=0)
        o[c0:c1] = colsum[P:] / (n_eff * Hq)
    return o


def importance_sums(q, k, cu_seqlens_q, cu_seqlens_k, *, n_obs, scale=None):
    """What one tensor-parallel rank contributes (section "Tensor parallelism", Eq. 15): the
    attention weights of Eq. 2 summed over the window rows and over the query heads given (the
    rank's share), not yet divided by anything.  Same arguments as importance_scores_with_context."""
    k = np.asarray(k)
    cq = np.asarray(cu_seqlens_q, dtype=np.int64)
    ck = np.asarray(cu_seqlens_k, dtype=np.int64)
    T, Hq, D = q.shape
    group = Hq // k.shape[1]
    if scale is None:
        scale = 1.0 / math.sqrt(D)
    out = np.zeros(T, dtype=np.float64)
    for r in range(len(cq) - 1):
        c0, c1, k0, k1 = int(cq[r]), int(cq[r + 1]), int(ck[r]), int(ck[r + 1])
        N, L = c1 - c0, k1 - k0
        if N == 0:
            continue
        n_eff = min(int(n_obs), N)
        Kr = k[k0:k1].astype(np.float64)
        Qw = np.asarray(q[c1 - n_eff:c1], dtype=np.float64)
        visible = np.arange(L)[None, :] <= np.arange(L - n_eff, L)[:, None]
        colsum = np.zeros(L, dtype=np.float64)
        for h in range(Hq):
            S = scale * (Qw[:, h, :] @ Kr[:, h // group, :].T)
            S[~visible] = -np.inf
            S -= S.max(axis=1, keepdims=True)
            W = np.exp(S)
            W /= W.sum(axis=1, keepdims=True)
            colsum += W.sum(axis=0)
        out[c0:c1] = colsum[L - N:]
    return out


def scores_from_partial_sums(partials, cu_seqlens, *, n_obs, total_q_heads):
    """Eq. 15 followed by the means of Eq. 3: the ranks' sums added (in rank order), divided by
    the window rows and by the query heads of all ranks; float64, not yet quantised."""
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    total = np.zeros(int(cu[-1]), dtype=np.float64)
    for part in partials:
        total = total + np.asarray(part, dtype=np.float64)
    o = np.zeros_like(total)
    for r in range(len(cu) - 1):
        N = int(cu[r + 1] - cu[r])
        if N:
            o[cu[r]:cu[r + 1]] = total[cu[r]:cu[r + 1]] / (min(int(n_obs), N) * int(total_q_heads))
    return o


def gather_paged_keys(k_cache, cu_seqlens_k, block_table, kv_block_size):
    """Keys of every request read out of a paged KV cache into the packed layout that
    ``importance_scores_with_context`` takes: key i of request r is row
    block_table[r, i // B] * B + i % B of the cache (the indexing of Eq. 16)."""
    cache = np.asarray(k_cache)
    ck = np.asarray(cu_seqlens_k, dtype=np.int64)
    bt = np.asarray(block_table, dtype=np.int64)
    B = int(kv_block_size)
    out = np.empty((int(ck[-1]),) + cache.shape[1:], dtype=cache.dtype)
    for r in range(len(ck) - 1):
        for i in range(int(ck[r + 1] - ck[r])):
            out[ck[r] + i] = cache[bt[r, i // B] * B + i % B]
    return out


def sinks_in_chunk(cu_seqlens_q, cu_seqlens_k, n_sink):
    """Number of sink tokens inside each request's chunk: max(0, A - P_r)."""
    cq = np.asarray(cu_seqlens_q, dtype=np.int64)
    ck = np.asarray(cu_seqlens_k, dtype=np.int64)
    P = (ck[1:] - ck[:-1]) - (cq[1:] - cq[:-1])
    return np.maximum(0, int(n_sink) - P)


def select_tokens_with_context(scores_f32, cu_seqlens_q, cu_seqlens_k, keep_ratio, *, block_size, n_obs, n_sink):
    """Block-local top-k over the chunk tokens: ``select_tokens`` request by request, with the
    sinks that fall inside the chunk."""
    s = np.asarray(scores_f32, dtype=np.float32)
    cq = np.asarray(cu_seqlens_q, dtype=np.int64)
    A = sinks_in_chunk(cu_seqlens_q, cu_seqlens_k, n_sink)
    kept = []
    new_cu = np.zeros(len(cq), dtype=np.int32)
    for r in range(len(cq) - 1):
        c0, c1 = int(cq[r]), int(cq[r + 1])
        idx, ncu = select_tokens(s[c0:c1], [0, c1 - c0], [keep_ratio[r]], block_size=block_size,
                                 n_obs=n_obs, n_sink=int(A[r]))
        kept.append(idx.astype(np.int64) + c0)
        new_cu[r + 1] = new_cu[r] + ncu[1]
    kept_idx = np.concatenate(kept) if kept else np.zeros(0, dtype=np.int64)
    return kept_idx.astype(np.int32), new_cu


def select_tokens_top_p_with_context(scores_f32, cu_seqlens_q, cu_seqlens_k, top_p, *, block_size, n_obs, n_sink):
    """The paper's block-level top-p rule over the chunk tokens: ``select_tokens_top_p`` request by
    request with the sinks that fall inside the chunk.  The threshold is p times the mass of the
    chunk's own blocks (the earlier tokens were decided when they were a chunk)."""
    s = np.asarray(scores_f32, dtype=np.float32)
    cq = np.asarray(cu_seqlens_q, dtype=np.int64)
    A = sinks_in_chunk(cu_seqlens_q, cu_seqlens_k, n_sink)
    kept = []
    new_cu = np.zeros(len(cq), dtype=np.int32)
    for r in range(len(cq) - 1):
        c0, c1 = int(cq[r]), int(cq[r + 1])
        idx, ncu = select_tokens_top_p(s[c0:c1], [0, c1 - c0], [top_p[r]], block_size=block_size,
                                       n_obs=n_obs, n_sink=int(A[r]))
        kept.append(idx.astype(np.int64) + c0)
        new_cu[r + 1] = new_cu[r] + ncu[1]
    kept_idx = np.concatenate(kept) if kept else np.zeros(0, dtype=np.int64)
    return kept_idx.astype(np.int32), new_cu


def sparsify_with_context(q, k, hidden, pos, cu_seqlens_q, cu_seqlens_k, keep_ratio, *, block_size, n_obs,
                          n_sink, scale=None):
    """score -> quantise -> select -> compact for chunks that follow earlier context."""
    o = importance_scores_with_context(q, k, cu_seqlens_q, cu_seqlens_k, n_obs=n_obs, scale=scale)
    s32 = quantise_scores(o)
    kept_idx, new_cu = select_tokens_with_context(s32, cu_seqlens_q, cu_seqlens_k, keep_ratio,
                                                  block_size=block_size, n_obs=n_obs, n_sink=n_sink)
    h_out, p_out = compact(hidden, pos, kept_idx)
    return {"scores64": o, "scores": s32, "kept_idx": kept_idx, "new_cu_seqlens": new_cu,
            "hidden_out": h_out, "pos_out": p_out}

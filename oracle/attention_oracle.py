"""CPU oracle for shared-prompt (DualKV) attention.  TEST INFRASTRUCTURE ONLY.

Plain numpy fp64.  It shares no code with the HIP path and must never be
imported by the product package: only tests, the smoke check and the
benchmark's cpu_baseline leg call it.

What it computes is the *definition*, not the tiled algorithm: every response
is explicitly replicated next to a private copy of the prompt (the standard
packing, Eq. 1), ordinary causal softmax attention (Eq. 2) and its textbook
backward are evaluated per (sequence, head) on the dense score matrix, and the
results are mapped back to the single-prompt layout:

  * O_d, LSE_d, dQ_d, dK_d, dV_d  = response rows of replica i;
  * O_c, LSE_c                    = prompt rows (identical in every replica,
                                    Sec. 2.2 "prompt invariance");
  * total dK_c, dV_c              = sum over the N replicas of the prompt rows
                                    of dK^(i), dV^(i) (Eq. 6 and the gradient
                                    equivalence theorem, App. A.5).

Conventions fixed here where the paper is silent:
  * diagonal inclusive: row at logical position t sees keys 0..t (App. A.3);
  * sliding window W>0: row t sees keys j with t-W < j <= t, i.e. exactly W keys
    once t >= W-1 (App. F "attends only the last W logical keys");
  * GQA: query head h reads KV head h // (H/H_k);
  * LSE is the natural log of sum_j exp(scale * q.k_j) over visible keys
    (Alg. 3, last line);
  * upstream gradient of replica i is [dO_c^(i); dO_d^(i)] with
    sum_i dO_c^(i) = dO_c (App. A.5); ``ctx_grad_owner`` chooses the split.

Pins (tests/test_oracle_*.py): closed forms (zero keys -> running mean and
log-count, two-key logistic, key-shift invariance), central finite differences
of all gradients, an autograd evaluation of the same loss, explicit-loop
evaluation of Eq. 4 in the single-prompt layout, finite differences with
respect to the *shared* K_c/V_c, the row samplers' O / LSE / dQ against the dense
pass, and hand-written examples of the two packings and their position ids.
"""
from __future__ import annotations

import numpy as np


# --------------------------------------------------------------------------
# single sequence, dense definition (Eq. 2)
# --------------------------------------------------------------------------
def visibility(S: int, window: int = 0, row0: int = 0, nrows: int | None = None) -> np.ndarray:
    """Boolean (nrows, S) mask: entry [a, j] is True iff row t=row0+a sees key j."""
    if nrows is None:
        nrows = S - row0
    t = np.arange(row0, row0 + nrows)[:, None]
    j = np.arange(S)[None, :]
    vis = j <= t
    if window and window > 0:
        vis &= j > t - window
    return vis


def attn_fwd_seq(q, k, v, scale, window=0):
    """Causal softmax attention of one sequence.

    q: (S, H, d); k, v: (S, H_k, d) fp64.  Returns o (S, H, d), lse (H, S).
    """
    S, H, d = q.shape
    Hk = k.shape[1]
    G = H // Hk
    o = np.zeros((S, H, d))
    lse = np.zeros((H, S))
    if S == 0:
        return o, lse
    vis = visibility(S, window)
    for h in range(H):
        kv = h // G
        s = scale * (q[:, h, :] @ k[:, kv, :].T)
        s = np.where(vis, s, -np.inf)
        m = s.max(axis=1, keepdims=True)
        e = np.exp(s - m)
        l = e.sum(axis=1, keepdims=True)
        lse[h] = (m + np.log(l))[:, 0]
        o[:, h, :] = (e / l) @ v[:, kv, :]
    return o, lse


def attn_bwd_seq(q, k, v, do, scale, window=0):
    """Textbook backward of attn_fwd_seq for upstream gradient do (S, H, d).

    A = softmax(S);  dV = A^T dO;  dP = dO V^T;  D = rowsum(A * dP);
    dS = A * (dP - D);  dQ = scale dS K;  dK = scale dS^T Q  (Alg. 1 without tiling).
    dK, dV are summed over the query heads of each KV group.
    """
    S, H, d = q.shape
    Hk = k.shape[1]
    G = H // Hk
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    if S == 0:
        return dq, dk, dv
    vis = visibility(S, window)
    for h in range(H):
        kv = h // G
        s = scale * (q[:, h, :] @ k[:, kv, :].T)
        s = np.where(vis, s, -np.inf)
        m = s.max(axis=1, keepdims=True)
        e = np.exp(s - m)
        a = e / e.sum(axis=1, keepdims=True)
        dv[:, kv, :] += a.T @ do[:, h, :]
        dp = do[:, h, :] @ v[:, kv, :].T
        dd = (a * dp).sum(axis=1, keepdims=True)
        ds = a * (dp - dd)
        dq[:, h, :] = scale * (ds @ k[:, kv, :])
        dk[:, kv, :] += scale * (ds.T @ q[:, h, :])
    return dq, dk, dv


# --------------------------------------------------------------------------
# shared-prompt group via explicit replication
# --------------------------------------------------------------------------
def replicate(P, cu, x_c, x_d, i):
    """Rows of replica i in the standard packing: [x_c ; x_d^(i)]."""
    return np.concatenate([x_c[:P], x_d[cu[i]:cu[i + 1]]], axis=0)


def dualkv_forward(q_c, k_c, v_c, q_d, k_d, v_d, cu, scale, window=0):
    """O and LSE of both calls from N replicated causal passes.

    Returns dict(o_c (P,H,d), lse_c (H,P), o_d (T,H,d), lse_d (H,T)).
    Asserts that the prompt rows agree across replicas.
    """
    P = q_c.shape[0]
    N = len(cu) - 1
    T, H, d = q_d.shape
    o_d = np.zeros((T, H, d))
    lse_d = np.zeros((H, T))
    o_c = lse_c = None
    for i in range(N):
        o, lse = attn_fwd_seq(replicate(P, cu, q_c, q_d, i), replicate(P, cu, k_c, k_d, i),
                              replicate(P, cu, v_c, v_d, i), scale, window)
        o_d[cu[i]:cu[i + 1]] = o[P:]
        lse_d[:, cu[i]:cu[i + 1]] = lse[:, P:]
        if o_c is None:
            o_c, lse_c = o[:P].copy(), lse[:, :P].copy()
        else:
            # identical up to the BLAS blocking of differently sized score matrices
            assert np.allclose(o_c, o[:P], rtol=1e-12, atol=1e-12)
            assert np.allclose(lse_c, lse[:, :P], rtol=1e-12, atol=1e-12)
    if o_c is None:  # N == 0 cannot happen (N >= 1); kept for clarity
        o_c, lse_c = np.zeros((P, H, d)), np.zeros((H, P))
    return dict(o_c=o_c, lse_c=lse_c, o_d=o_d, lse_d=lse_d)


def dualkv_backward(q_c, k_c, v_c, q_d, k_d, v_d, cu, scale, do_c, do_d, window=0,
                    ctx_grad_owner=0):
    """Gradients from N replicated backward passes.

    Replica ``ctx_grad_owner`` carries the whole prompt-row upstream gradient
    do_c, the others carry zero there (any split with the same sum is
    equivalent by linearity of the backward in dO).  ``ctx_grad_owner`` may also
    be an (N,) array of weights summing to one.

    Returns dict with dq_c, dq_d, dk_c, dv_c (totals), dk_d, dv_d.
    """
    P = q_c.shape[0]
    N = len(cu) - 1
    w = np.zeros(N)
    if np.ndim(ctx_grad_owner) == 0:
        w[int(ctx_grad_owner)] = 1.0
    else:
        w[:] = np.asarray(ctx_grad_owner, dtype=np.float64)
    dq_c = np.zeros_like(q_c)
    dk_c = np.zeros_like(k_c)
    dv_c = np.zeros_like(v_c)
    dq_d = np.zeros_like(q_d)
    dk_d = np.zeros_like(k_d)
    dv_d = np.zeros_like(v_d)
    for i in range(N):
        do = np.concatenate([w[i] * do_c[:P], do_d[cu[i]:cu[i + 1]]], axis=0)
        dq, dk, dv = attn_bwd_seq(replicate(P, cu, q_c, q_d, i), replicate(P, cu, k_c, k_d, i),
                                  replicate(P, cu, v_c, v_d, i), do, scale, window)
        dq_c += dq[:P]
        dk_c += dk[:P]
        dv_c += dv[:P]
        dq_d[cu[i]:cu[i + 1]] = dq[P:]
        dk_d[cu[i]:cu[i + 1]] = dk[P:]
        dv_d[cu[i]:cu[i + 1]] = dv[P:]
    return dict(dq_c=dq_c, dq_d=dq_d, dk_c=dk_c, dv_c=dv_c, dk_d=dk_d, dv_d=dv_d)


def dualkv_reference(q_c, k_c, v_c, q_d, k_d, v_d, cu, scale, do_c, do_d, window=0):
    """Everything the four library entry points return, per call.

    * ``call1``: dq_c, dk_c, dv_c produced by the prompt self-attention backward
      alone (response upstream gradient set to zero);
    * ``call2``: dq_d, dk_c, dv_c, dk_d, dv_d produced by the response rows alone
      (prompt upstream gradient set to zero);
    * ``total``: sum of both for the shared K_c, V_c.
    """
    fwd = dualkv_forward(q_c, k_c, v_c, q_d, k_d, v_d, cu, scale, window)
    z_c, z_d = np.zeros_like(do_c), np.zeros_like(do_d)
    g1 = dualkv_backward(q_c, k_c, v_c, q_d, k_d, v_d, cu, scale, do_c, z_d, window)
    g2 = dualkv_backward(q_c, k_c, v_c, q_d, k_d, v_d, cu, scale, z_c, do_d, window)
    out = dict(fwd)
    out["call1"] = dict(dq_c=g1["dq_c"], dk_c=g1["dk_c"], dv_c=g1["dv_c"])
    out["call2"] = dict(dq_d=g2["dq_d"], dk_c=g2["dk_c"], dv_c=g2["dv_c"],
                        dk_d=g2["dk_d"], dv_d=g2["dv_d"])
    out["total"] = dict(dk_c=g1["dk_c"] + g2["dk_c"], dv_c=g1["dv_c"] + g2["dv_c"])
    return out


# --------------------------------------------------------------------------
# row / column samples at sizes where the dense pass is too slow
# --------------------------------------------------------------------------
def _keys_of_row(P, cu, x_c, x_d, i, r, kv):
    """Keys (or values) visible candidates of response row r of sequence i: [x_c; x_d^(i)[0..r]]."""
    return np.concatenate([x_c[:P, kv, :], x_d[cu[i]:cu[i] + r + 1, kv, :]], axis=0)


def response_row(q_d, k_c, v_c, k_d, v_d, cu, scale, i, r, h, window=0, do_row=None):
    """One response query row (sequence i, row r, head h) straight from Eq. 4.

    Returns (o (d,), lse, dq (d,) or None).
    """
    P = k_c.shape[0]
    G = q_d.shape[1] // k_c.shape[1]
    kv = h // G
    q = q_d[cu[i] + r, h, :]
    K = _keys_of_row(P, cu, k_c, k_d, i, r, kv)
    V = _keys_of_row(P, cu, v_c, v_d, i, r, kv)
    t = P + r
    s = scale * (K @ q)
    if window and window > 0:
        j = np.arange(t + 1)
        s = np.where(j > t - window, s, -np.inf)
    m = s.max()
    e = np.exp(s - m)
    l = e.sum()
    a = e / l
    o = a @ V
    lse = m + np.log(l)
    dq = None
    if do_row is not None:
        dp = V @ do_row
        ds = a * (dp - a @ dp)
        dq = scale * (ds @ K)
    return o, lse, dq


def prompt_row(q_c, k_c, v_c, scale, t, h, window=0, do_row=None):
    """One prompt query row (position t, head h) of the context self-attention (Eq. 3)."""
    G = q_c.shape[1] // k_c.shape[1]
    kv = h // G
    q = q_c[t, h, :]
    K = k_c[:t + 1, kv, :]
    V = v_c[:t + 1, kv, :]
    s = scale * (K @ q)
    if window and window > 0:
        j = np.arange(t + 1)
        s = np.where(j > t - window, s, -np.inf)
    m = s.max()
    e = np.exp(s - m)
    l = e.sum()
    a = e / l
    o = a @ V
    dq = None
    if do_row is not None:
        dp = V @ do_row
        ds = a * (dp - a @ dp)
        dq = scale * (ds @ K)
    return o, m + np.log(l), dq


def key_columns_call2(q_d, k_c, v_c, k_d, v_d, cu, scale, do_d, kv, ctx_keys, dec_keys,
                      window=0, rows=None, progress=None):
    """Call-2 dK/dV at chosen key positions of KV head ``kv``.

    ctx_keys: array of prompt positions j; dec_keys: list of (i, j) response key
    positions.  ``rows``: optional list of (i, r) response rows that carry a
    non-zero upstream gradient (all rows if None) -- rows with dO == 0 contribute
    nothing, so the caller may restrict the sum to them.

    Every contributing row needs its own softmax normaliser and D, so the cost is
    one dense row evaluation per (row, head of the group).
    Returns dk_c (len(ctx_keys), d), dv_c, dk_d (len(dec_keys), d), dv_d.
    """
    P = k_c.shape[0]
    N = len(cu) - 1
    H = q_d.shape[1]
    G = H // k_c.shape[1]
    d = q_d.shape[2]
    ctx_keys = np.asarray(ctx_keys, dtype=np.int64)
    dk_c = np.zeros((len(ctx_keys), d))
    dv_c = np.zeros((len(ctx_keys), d))
    dk_d = np.zeros((len(dec_keys), d))
    dv_d = np.zeros((len(dec_keys), d))
    dec_by_seq = {}
    for n, (i, j) in enumerate(dec_keys):
        dec_by_seq.setdefault(int(i), []).append((n, int(j)))
    if rows is None:
        rows_by_seq = {i: np.arange(cu[i + 1] - cu[i]) for i in range(N)}
    else:
        rows_by_seq = {}
        for (i, r) in rows:
            rows_by_seq.setdefault(int(i), []).append(int(r))
        rows_by_seq = {i: np.asarray(sorted(v)) for i, v in rows_by_seq.items()}
    for i in sorted(rows_by_seq):
        rr = rows_by_seq[i]
        if len(rr) == 0:
            continue
        Ri = int(cu[i + 1] - cu[i])
        K = np.concatenate([k_c[:P, kv, :], k_d[cu[i]:cu[i + 1], kv, :]], axis=0)
        V = np.concatenate([v_c[:P, kv, :], v_d[cu[i]:cu[i + 1], kv, :]], axis=0)
        t = P + rr[:, None]
        j = np.arange(P + Ri)[None, :]
        vis = j <= t
        if window and window > 0:
            vis &= j > t - window
        for g in range(G):
            h = kv * G + g
            q = q_d[cu[i] + rr, h, :]
            do = do_d[cu[i] + rr, h, :]
            s = np.where(vis, scale * (q @ K.T), -np.inf)
            m = s.max(axis=1, keepdims=True)
            e = np.exp(s - m)
            a = e / e.sum(axis=1, keepdims=True)
            dp = do @ V.T
            ds = a * (dp - (a * dp).sum(axis=1, keepdims=True))
            dv_c += a[:, ctx_keys].T @ do
            dk_c += scale * (ds[:, ctx_keys].T @ q)
            for (n, jj) in dec_by_seq.get(i, []):
                dv_d[n] += a[:, P + jj] @ do
                dk_d[n] += scale * (ds[:, P + jj] @ q)
        if progress is not None:
            progress(i)
    return dk_c, dv_c, dk_d, dv_d


# --------------------------------------------------------------------------
# counting helpers (exact visible-pair counts; Sec. 2 FLOP expressions)
# --------------------------------------------------------------------------
def visible_pairs_call1(P, window=0):
    """Visible (query, key) pairs per head of the prompt self-attention."""
    t = np.arange(P, dtype=np.int64)
    n = t + 1
    if window and window > 0:
        n = np.minimum(n, window)
    return int(n.sum())


def visible_pairs_call2(P, resp_lens, window=0):
    """Visible pairs per head of all response rows (prompt keys + own causal keys)."""
    tot = 0
    for R in resp_lens:
        t = P + np.arange(int(R), dtype=np.int64)
        n = t + 1
        if window and window > 0:
            n = np.minimum(n, window)
        tot += int(n.sum())
    return tot


def visible_pairs_replicated(P, resp_lens, window=0):
    """Visible pairs per head of the N-copy baseline (Eq. 2): sum_i causal pairs of length P+R_i."""
    return sum(visible_pairs_call1(P + int(R), window) for R in resp_lens)


# --------------------------------------------------------------------------
# next-token map of the single-prompt packing (Sec. 2.3, "shared prompt logits")
# --------------------------------------------------------------------------
def next_token_pairs_replicated(P, cu):
    """Set of (predicting packed row, predicted packed row) pairs, from the definition: in every replica
    [prompt ; response i] of the standard packing, row s predicts row s + 1; rows are then renamed to the
    single-prompt packing (prompt row j -> j for every replica, response i row r -> P + cu[i] + r)."""
    pairs = set()
    for i in range(len(cu) - 1):
        R = int(cu[i + 1] - cu[i])
        packed = list(range(P)) + [P + int(cu[i]) + r for r in range(R)]
        for s in range(P + R - 1):
            pairs.add((packed[s], packed[s + 1]))
    return pairs



# --------------------------------------------------------------------------
# the two packings as data movement (Eq. 1 <-> Eq. 5) and their position ids (App. A.2)
# --------------------------------------------------------------------------
def replicated_layout(P, cu, x_c, x_d):
    """Standard packing (Eq. 1) of per-token records: [prompt, resp_1 | prompt, resp_2 | ...].

    x_c: (P, ...) prompt records, x_d: (T, ...) packed response records, cu: (N+1,) response offsets.
    Returns (x_rep, cu_rep): sequence i occupies rows cu_rep[i]:cu_rep[i+1] = its own prompt copy (P rows)
    followed by its R_i response rows.
    """
    n = len(cu) - 1
    parts = []
    cu_rep = np.zeros(n + 1, dtype=np.int32)
    for i in range(n):
        parts.append(x_c[:P])
        parts.append(x_d[cu[i]:cu[i + 1]])
        cu_rep[i + 1] = cu_rep[i] + P + (cu[i + 1] - cu[i])
    return np.concatenate(parts, axis=0), cu_rep


def single_prompt_layout(P, cu, x_rep):
    """Inverse of replicated_layout (Eq. 5): [prompt | resp_1 | ... | resp_N], the prompt taken from
    sequence 0's copy."""
    n = len(cu) - 1
    parts = [x_rep[:P]]
    off = 0
    for i in range(n):
        R = int(cu[i + 1] - cu[i])
        parts.append(x_rep[off + P:off + P + R])
        off += P + R
    return np.concatenate(parts, axis=0)


def position_ids_replicated(P, cu):
    """Logical position of every row of the standard packing: 0 .. P+R_i-1 inside each sequence."""
    return np.concatenate([np.arange(P + int(cu[i + 1] - cu[i])) for i in range(len(cu) - 1)]).astype(np.int64)


def position_ids_single_prompt(P, cu):
    """Logical position of every row of the single-prompt packing: prompt row j -> j, row r of any
    response -> P + r (the position it has in its own replica; App. A.2)."""
    return np.concatenate([np.arange(P)] +
                          [P + np.arange(int(cu[i + 1] - cu[i])) for i in range(len(cu) - 1)]).astype(np.int64)

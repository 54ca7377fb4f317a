"""CPU oracle for the Cartridge hot path -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

Plain numpy, fp64 everywhere, full score rows materialised, no tiling, no
online softmax, no code shared with the HIP library.  Only tests, the smoke
check and the benchmark's cpu_baseline leg may import this module; the product
path never routes through it.

What each function follows (arxiv 2506.06266):

* attn_fwd / attn_bwd -- Eq. 1 (Sec. 2.3, causal softmax attention) evaluated
  over the cache ordering of Sec. 3.2 ("Cartridge KV cache": the p trainable
  pairs (z_k, z_v) first, then the sequence's own pairs).  Every query sees all
  p prefix slots; the own part is causal, j <= i, as Eq. 1's sum over j = 1..i.
  The backward pass is the analytic gradient of that definition; Sec. 3.2
  trains Z by back-propagating into the key and value vectors with the model
  frozen, so dZ sums every query of every sequence in the batch.
  attn_varlen_fwd / attn_varlen_bwd -- the same over a packed batch of
  sequences of different lengths (Fig. "Scaling Self-Study compute" trains on batches
  of 64 conversations of at most 1024 tokens; the paper does not say how they are
  laid out: packing instead of padding is this build's choice).
* distill_kl -- Eq. 3 (Sec. 4.2), the KL divergence from the teacher's to the
  student's next-token distribution, restricted to the teacher entries that
  were recorded (App. A.2 "Training Objective": top output probabilities are
  collected at data-generation time).
* distill_kl_rest_bucket -- the same divergence with the unrecorded vocabulary
  kept as one extra outcome on both sides (a proper KL of (k+1)-outcome
  distributions); ntp_cross_entropy -- the next-token objective Sec. 4.2
  compares context distillation with (ablated in Sec. 5.3), with an ignore
  label.
* teacher_topk -- App. A.2: the teacher's top output probabilities, recorded
  at data-generation time (what distill_kl consumes).
* decode -- Sec. 2.3 (decode: one new query over the whole cache) with the
  cache of Sec. 3.3 (a cartridge is served as a cached prefix of length p).
  decode_composed -- the same over several cartridges concatenated (Sec. 5.4,
  composition without retraining) and / or a different cartridge per request
  (the serving protocol of App. A.3, "Throughput measurement details").

Readings where the paper is silent (listed in the design notes as well):
scale is 1/sqrt(head_dim) per head unless given; query head h reads KV head
h // (Hq // Hkv); teacher entries with a negative index are ignored.

Parity pins: every function here is pinned by tests/test_oracle_*.py against
closed forms, textbook special cases written independently in the tests,
brute-force loops on tiny inputs and central finite differences.
"""
from __future__ import annotations

import math
from typing import Optional, Tuple

import numpy as np

__all__ = ["attn_fwd", "attn_bwd", "distill_kl", "distill_kl_rest_bucket", "ntp_cross_entropy", "decode", "decode_composed", "teacher_topk", "attn_varlen_fwd", "attn_varlen_bwd"]


def _f64(x) -> np.ndarray:
    return np.asarray(x, dtype=np.float64)


def _visible(S: int, p: int) -> np.ndarray:
    """[S, p+S] boolean: column j of the concatenated cache is visible to query row i.

    Prefix columns (j < p) are always visible; own column p + t is visible iff t <= i
    (Sec. 3.2 cache ordering, Eq. 1 causal sum)."""
    vis = np.ones((S, p + S), dtype=bool)
    own = np.tril(np.ones((S, S), dtype=bool))
    vis[:, p:] = own
    return vis


def _probs(q_bh: np.ndarray, keys: np.ndarray, vis: np.ndarray, scale: float):
    """Softmax weights of Eq. 1 for one (sequence, query head): returns (P [S, p+S], lse [S])."""
    s = scale * (q_bh @ keys.T)
    s = np.where(vis, s, -np.inf)
    m = s.max(axis=1, keepdims=True)
    e = np.exp(s - m)
    l = e.sum(axis=1, keepdims=True)
    return e / l, (m + np.log(l))[:, 0]


def attn_fwd(q, k_own, v_own, z_k, z_v, scale: Optional[float] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Cartridge attention forward.

    q [B,S,Hq,d]; k_own, v_own [B,S,Hkv,d]; z_k, z_v [Hkv,p,d] (p may be 0).
    Returns o [B,S,Hq,d] and lse [B,Hq,S] (log of the softmax denominator of each row)."""
    q, k_own, v_own, z_k, z_v = map(_f64, (q, k_own, v_own, z_k, z_v))
    B, S, Hq, d = q.shape
    Hkv, p = z_k.shape[0], z_k.shape[1]
    G = Hq // Hkv
    assert Hq == G * Hkv and k_own.shape == (B, S, Hkv, d) and z_v.shape == (Hkv, p, d)
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    vis = _visible(S, p)
    o = np.zeros((B, S, Hq, d))
    lse = np.zeros((B, Hq, S))
    for b in range(B):
        for h in range(Hq):
            hk = h // G
            keys = np.concatenate([z_k[hk], k_own[b, :, hk]], axis=0)
            vals = np.concatenate([z_v[hk], v_own[b, :, hk]], axis=0)
            P, lse[b, h] = _probs(q[b, :, h], keys, vis, scale)
            o[b, :, h] = P @ vals
    return o, lse


def attn_bwd(q, k_own, v_own, z_k, z_v, d_o, scale: Optional[float] = None):
    """Gradient of sum(o * d_o) with respect to every input of attn_fwd.

    Returns (d_q [B,S,Hq,d], d_k_own, d_v_own [B,S,Hkv,d], d_z_k, d_z_v [Hkv,p,d]).
    With P the softmax weights, D_i = dO_i . O_i, dP = dO V^T, dS = P * (dP - D):
    dQ = scale dS K, dK = scale dS^T Q, dV = P^T dO.  Key/value gradients sum over the
    query heads of a group; for the prefix rows they also sum over the whole batch."""
    q, k_own, v_own, z_k, z_v, d_o = map(_f64, (q, k_own, v_own, z_k, z_v, d_o))
    B, S, Hq, d = q.shape
    Hkv, p = z_k.shape[0], z_k.shape[1]
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    vis = _visible(S, p)
    d_q = np.zeros_like(q)
    d_k_own = np.zeros_like(k_own)
    d_v_own = np.zeros_like(v_own)
    d_z_k = np.zeros_like(z_k)
    d_z_v = np.zeros_like(z_v)
    for b in range(B):
        for h in range(Hq):
            hk = h // G
            keys = np.concatenate([z_k[hk], k_own[b, :, hk]], axis=0)
            vals = np.concatenate([z_v[hk], v_own[b, :, hk]], axis=0)
            P, _ = _probs(q[b, :, h], keys, vis, scale)
            o = P @ vals
            g = d_o[b, :, h]
            D = (g * o).sum(axis=1, keepdims=True)
            dP = g @ vals.T
            dS = P * (dP - D)
            d_q[b, :, h] = scale * (dS @ keys)
            d_keys = scale * (dS.T @ q[b, :, h])
            d_vals = P.T @ g
            d_z_k[hk] += d_keys[:p]
            d_z_v[hk] += d_vals[:p]
            d_k_own[b, :, hk] += d_keys[p:]
            d_v_own[b, :, hk] += d_vals[p:]
    return d_q, d_k_own, d_v_own, d_z_k, d_z_v


def distill_kl(logits, teacher_idx, teacher_logp, scale: float = 1.0):
    """Context-distillation loss over recorded teacher entries and its gradient.

    logits [N,V]; teacher_idx [N,k] integer (entries < 0 are ignored); teacher_logp [N,k].
    Per row: t_j = exp(logp_j), log s = logits - logsumexp(logits),
    KL_n = sum_j t_j (logp_j - log s[idx_j]);  loss = scale * sum_n KL_n.
    d loss / d logits[n,v] = scale * (M_n s_nv - t_nv), M_n = sum_j t_j, t_nv = t_j at v = idx_j.
    Returns (loss, d_logits [N,V], row_kl [N])."""
    z = _f64(logits)
    idx = np.asarray(teacher_idx, dtype=np.int64)
    lp = _f64(teacher_logp)
    N, V = z.shape
    m = z.max(axis=1, keepdims=True)
    lse = m + np.log(np.exp(z - m).sum(axis=1, keepdims=True))
    log_s = z - lse
    s = np.exp(log_s)
    row_kl = np.zeros(N)
    d_logits = np.zeros((N, V))
    for n in range(N):
        M = 0.0
        for j in range(idx.shape[1]):
            v = idx[n, j]
            if v < 0:
                continue
            t = math.exp(lp[n, j])
            row_kl[n] += t * (lp[n, j] - log_s[n, v])
            d_logits[n, v] -= t
            M += t
        d_logits[n] += M * s[n]
    return scale * row_kl.sum(), scale * d_logits, row_kl


def distill_kl_rest_bucket(logits, teacher_idx, teacher_logp, scale: float = 1.0):
    """The same loss with the unrecorded vocabulary kept as one extra outcome.

    Eq. 3 is a KL divergence between full distributions while App. A.2 records only the teacher's
    top entries.  Here the k recorded tokens and "every other token" form a (k+1)-outcome
    distribution on both sides: teacher (t_1..t_k, 1 - M), student (s_idx_1..s_idx_k, 1 - S_K)
    with M = sum_j t_j and S_K = sum_j s_idx_j, and the row value is their KL divergence
    KL_n = sum_j t_j (log t_j - log s_idx_j) + (1 - M) (log(1 - M) - log(1 - S_K))  (>= 0).
    d KL_n / d logits[v] = s_v - t_v on the recorded tokens and s_v (M - S_K) / (1 - S_K) elsewhere.
    Entries with a negative index are ignored.  Returns (loss, d_logits [N,V], row_kl [N])."""
    z = _f64(logits)
    idx = np.asarray(teacher_idx, dtype=np.int64)
    lp = _f64(teacher_logp)
    N, V = z.shape
    m = z.max(axis=1, keepdims=True)
    lse = m + np.log(np.exp(z - m).sum(axis=1, keepdims=True))
    log_s = z - lse
    s = np.exp(log_s)
    row_kl = np.zeros(N)
    d_logits = np.zeros((N, V))
    for n in range(N):
        on = np.zeros(V, dtype=bool)
        M = 0.0
        S_K = 0.0
        for j in range(idx.shape[1]):
            v = idx[n, j]
            if v < 0:
                continue
            t = math.exp(lp[n, j])
            row_kl[n] += t * (lp[n, j] - log_s[n, v])
            d_logits[n, v] = s[n, v] - t
            on[v] = True
            M += t
            S_K += s[n, v]
        rest_t = 1.0 - M
        rest_s = s[n, ~on].sum()            # 1 - S_K without the cancellation
        if rest_t > 1e-12:                  # below that the teacher's mass is 1 up to rounding
            row_kl[n] += rest_t * (math.log(rest_t) - math.log(rest_s)) if rest_s > 0.0 else math.inf
        if rest_s > 0.0:
            d_logits[n, ~on] = s[n, ~on] * (M - S_K) / rest_s
    return scale * row_kl.sum(), scale * d_logits, row_kl


def ntp_cross_entropy(logits, labels, scale: float = 1.0):
    """Next-token cross-entropy (the objective Sec. 4.2 compares context distillation with).

    logits [N,V]; labels [N] integer, rows with a negative label are ignored (no loss, zero
    gradient).  row_n = -log softmax(logits_n)[label_n]; loss = scale * sum_n row_n;
    d loss / d logits = scale * (softmax - onehot).  Returns (loss, d_logits [N,V], row [N])."""
    z = _f64(logits)
    lab = np.asarray(labels, dtype=np.int64)
    N, V = z.shape
    row = np.zeros(N)
    d_logits = np.zeros((N, V))
    for n in range(N):
        if lab[n] < 0:
            continue
        zn = z[n] - z[n].max()
        log_s = zn - math.log(np.exp(zn).sum())
        row[n] = -log_s[lab[n]]
        d_logits[n] = np.exp(log_s)
        d_logits[n, lab[n]] -= 1.0
    return scale * row.sum(), scale * d_logits, row


def decode(q, z_k, z_v, k_own, v_own, cu_lens, scale: Optional[float] = None):
    """One query token per request over [shared cartridge ; the request's own KV].

    q [B,Hq,d]; z_k, z_v [Hkv,p,d]; k_own, v_own [T,Hkv,d] ragged, request b owns rows
    cu_lens[b] .. cu_lens[b+1]-1 (the current token's own key/value is the last of them), all
    visible.  Returns o [B,Hq,d] and lse [B,Hq]."""
    q, z_k, z_v, k_own, v_own = map(_f64, (q, z_k, z_v, k_own, v_own))
    cu = np.asarray(cu_lens, dtype=np.int64)
    B, Hq, d = q.shape
    Hkv = z_k.shape[0]
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    o = np.zeros((B, Hq, d))
    lse = np.zeros((B, Hq))
    for b in range(B):
        for h in range(Hq):
            hk = h // G
            keys = np.concatenate([z_k[hk], k_own[cu[b]:cu[b + 1], hk]], axis=0)
            vals = np.concatenate([z_v[hk], v_own[cu[b]:cu[b + 1], hk]], axis=0)
            s = scale * (keys @ q[b, h])
            m = s.max()
            e = np.exp(s - m)
            l = e.sum()
            o[b, h] = (e / l) @ vals
            lse[b, h] = m + math.log(l)
    return o, lse


def decode_composed(q, shared, pool_k, pool_v, cart_id, k_own, v_own, cu_lens, scale: Optional[float] = None):
    """Decode step over composed cartridges (Sec. 5.4: independently trained cartridges are
    concatenated without retraining; App. A.3's throughput protocol serves a different cartridge
    per request).

    Request b attends over, in cache order: every shared segment (z_k, z_v) of `shared`, each
    [Hkv,p_s,d]; then its private cartridge pool_k[cart_id[b]], pool_v[cart_id[b]] ([Hkv,p_c,d];
    none when cart_id[b] < 0 or the pool is None); then its own rows of k_own / v_own.  All
    visible.  Returns o [B,Hq,d] and lse [B,Hq]."""
    q, k_own, v_own = map(_f64, (q, k_own, v_own))
    shared = [(_f64(a), _f64(b_)) for a, b_ in shared]
    cu = np.asarray(cu_lens, dtype=np.int64)
    B, Hq, d = q.shape
    Hkv = k_own.shape[1]
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    o = np.zeros((B, Hq, d))
    lse = np.zeros((B, Hq))
    for b in range(B):
        for h in range(Hq):
            hk = h // G
            ks = [zk[hk] for zk, _ in shared]
            vs = [zv[hk] for _, zv in shared]
            if pool_k is not None and cart_id is not None and int(cart_id[b]) >= 0:
                ks.append(_f64(pool_k[int(cart_id[b]), hk]))
                vs.append(_f64(pool_v[int(cart_id[b]), hk]))
            ks.append(k_own[cu[b]:cu[b + 1], hk])
            vs.append(v_own[cu[b]:cu[b + 1], hk])
            keys, vals = np.concatenate(ks, axis=0), np.concatenate(vs, axis=0)
            s = scale * (keys @ q[b, h])
            m = s.max()
            e = np.exp(s - m)
            l = e.sum()
            o[b, h] = (e / l) @ vals
            lse[b, h] = m + math.log(l)
    return o, lse


def teacher_topk(logits, k: int):
    """The records App. A.2 says are collected while the teacher generates: at every position the
    k most probable next tokens and their log-probabilities.

    logits [N,V] -> idx [N,k] int64, logp [N,k], each row by descending probability; among equal
    logits the lower token index comes first (so the result is unique)."""
    z = _f64(logits)
    N, V = z.shape
    idx = np.zeros((N, k), dtype=np.int64)
    logp = np.zeros((N, k))
    for n in range(N):
        m = z[n].max()
        lse = m + math.log(np.exp(z[n] - m).sum())
        order = sorted(range(V), key=lambda v: (-z[n, v], v))[:k]
        idx[n] = order
        logp[n] = z[n, order] - lse
    return idx, logp


def attn_varlen_fwd(q, k_own, v_own, z_k, z_v, cu_seqlens, scale: Optional[float] = None):
    """attn_fwd over a packed batch of sequences of different lengths (the training batches of
    Fig. "Scaling Self-Study compute": 64 conversations of at most 1024 tokens; the paper is silent on
    their layout, concatenating them instead of padding is this build's choice).

    q [T,Hq,d]; k_own, v_own [T,Hkv,d]; sequence b owns rows cu_seqlens[b] .. cu_seqlens[b+1]-1 and
    attends over [Z ; its own rows, causally] exactly as a batch of one in attn_fwd.
    Returns o [T,Hq,d] and lse [Hq,T]."""
    q, k_own, v_own = map(_f64, (q, k_own, v_own))
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    T, Hq, d = q.shape
    o = np.zeros((T, Hq, d))
    lse = np.zeros((Hq, T))
    for b in range(len(cu) - 1):
        sl = slice(cu[b], cu[b + 1])
        ob, lb = attn_fwd(q[None, sl], k_own[None, sl], v_own[None, sl], z_k, z_v, scale)
        o[sl] = ob[0]
        lse[:, sl] = lb[0]
    return o, lse


def attn_varlen_bwd(q, k_own, v_own, z_k, z_v, d_o, cu_seqlens, scale: Optional[float] = None):
    """Gradient of attn_varlen_fwd: per sequence as attn_bwd; the prefix gradients add up over the
    sequences of the packed batch.  Returns (d_q, d_k_own, d_v_own [packed], d_z_k, d_z_v)."""
    q, k_own, v_own, d_o = map(_f64, (q, k_own, v_own, d_o))
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    d_q, d_k, d_v = np.zeros_like(q), np.zeros_like(k_own), np.zeros_like(v_own)
    d_zk, d_zv = np.zeros_like(_f64(z_k)), np.zeros_like(_f64(z_v))
    for b in range(len(cu) - 1):
        sl = slice(cu[b], cu[b + 1])
        g = attn_bwd(q[None, sl], k_own[None, sl], v_own[None, sl], z_k, z_v, d_o[None, sl], scale)
        d_q[sl], d_k[sl], d_v[sl] = g[0][0], g[1][0], g[2][0]
        d_zk += g[3]
        d_zv += g[4]
    return d_q, d_k, d_v, d_zk, d_zv

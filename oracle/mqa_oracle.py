"""Float64 CPU oracle for multi-query / multi-head attention decoding.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
HIP kernels are checked against.  It shares no code with them and nothing in
the product path may import it; only tests, the smoke check and the
benchmark's CPU-baseline leg call it.

Everything is numpy float64.  Each function states the passage of the paper
(arXiv 1911.02150) it writes out.  The paper's method is exact attention with
the heads dimension removed from K and V, so the oracle is that definition:
contractions ("broadcast, multiply, sum", Section 2.1) and a softmax over the
memory positions, with no blocking or fusion of the method's steps.  The
contractions are numpy matrix products / einsum(optimize=True), which hand the
sum to the BLAS and so leave the order of a float64 sum to it: results move by
a few 1e-16 relative between summation orders, and the pins that compare two
float64 routes allow 1e-15..1e-12 for that reason.

Readings taken where the paper's listings are silent or garbled:
  * Section 2.4 / Section 3 incremental listings project an undefined `M` and
    return an undefined `O`: read as the step input `x` and the heads' outputs
    `o` (self-attention: the new memory row comes from the current input).
  * The Section 3 incremental listing concatenates on axis 2 of a [b,m,k]
    tensor; its declared result [b,m+1,k] fixes the position axis as axis 1.
  * No 1/sqrt(k) logit scale (Section 2.2 note): `scale` defaults to 1.
  * softmax runs over the last (memory position) axis, per (sequence, head).
  * The new token attends to itself (logits use the concatenated K).
  * A sequence with no valid position yields a zero output row.
  * The growing concat is kept as an in-place append into a capacity-sized
    buffer with per-sequence lengths (the alternative named in the Section 4.3
    footnote); rows at and beyond the length are never read.
  * Cache number format is not stated by the paper; a bf16 cache stores each
    new row rounded float32 -> bf16, round-to-nearest-even.

Parity pins (tests/test_oracle_*.py): brute-force enumeration on tiny shapes,
softmax against scipy, weights sum to one, MQA == MHA with shared K/V,
incremental == causally masked batched attention, closed forms (one position,
zero query, dominant logit, shift and permutation invariance, convex hull,
a window as a shortened cache, a window of one position, beams as
separate sequences with materialised memories, moving a row between the shared and the
own part),
torch float64 scaled-dot-product attention as an independent routine, split
and recombine of the softmax state, NaN rows beyond the length, and bf16
rounding against torch's cast.  No function here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------
# Section 2.1: softmax and single-query dot-product attention
# --------------------------------------------------------------------------
def softmax64(z, axis=-1):
    """softmax over `axis` (Section 2.1, `weights = softmax(logits)`)."""
    z = np.asarray(z, dtype=F64)
    e = np.exp(z - np.max(z, axis=axis, keepdims=True))
    return e / np.sum(e, axis=axis, keepdims=True)


def dot_product_attention(q, K, V):
    """Section 2.1 `DotProductAttention`: q [k], K [m,k], V [m,v] -> y [v]."""
    q, K, V = (np.asarray(a, dtype=F64) for a in (q, K, V))
    logits = np.einsum("k,mk->m", q, K)
    weights = softmax64(logits)
    return np.einsum("m,mv->v", weights, V)


# --------------------------------------------------------------------------
# Sections 2.2, 2.3 and 3: whole attention layers, written as loops over the
# (sequence, head) pairs around the Section 2.1 function.  Every pair is an
# independent dot-product attention: head j queries with x . P_q[j], reads the
# memory through (M . P_k[j], M . P_v[j]) -- multi-query: through the one shared
# (M . P_k, M . P_v), Section 3 -- and adds its output vector times P_o[j]^T
# (P_o is [h,d,v]: model width before value width) into the layer output.
# --------------------------------------------------------------------------
def _masked_attention(Q, K, V, mask=None):
    """Section 2.1 attention for several queries over one memory: Q [n,k], K [m,k], V [m,v] and an
    additive mask [n,m] (0 or -inf, Section 2.3) -> [n,v]."""
    logits = Q @ K.T
    if mask is not None:
        logits = logits + mask
    return softmax64(logits) @ V


def _layer(X, M, mask, P_q, P_k, P_v, P_o, shared_kv, kv_round=None):
    """Y [b,n,d] for X [b,n,d] against M [b,m,d]; mask [b,h,n,m] or None.  shared_kv: P_k [d,k],
    P_v [d,v] (multi-query); else P_k [h,d,k], P_v [h,d,v] (multi-head)."""
    X, M, P_q, P_k, P_v, P_o = (np.asarray(a, dtype=F64) for a in (X, M, P_q, P_k, P_v, P_o))
    if mask is not None:
        mask = np.asarray(mask, dtype=F64)
    rnd = (lambda a: a) if kv_round is None else kv_round
    b, n, d = X.shape
    h = P_q.shape[0]
    Y = np.zeros((b, n, d), dtype=F64)
    for i in range(b):
        if shared_kv:
            K_i, V_i = rnd(M[i] @ P_k), rnd(M[i] @ P_v)              # one K, V for every head (Section 3)
        for j in range(h):
            if not shared_kv:
                K_i, V_i = rnd(M[i] @ P_k[j]), rnd(M[i] @ P_v[j])    # this head's K, V (Section 2.2)
            o_ij = _masked_attention(X[i] @ P_q[j], K_i, V_i, None if mask is None else mask[i, j])
            Y[i] += o_ij @ P_o[j].T
    return Y


def multihead_attention(x, M, P_q, P_k, P_v, P_o):
    """Section 2.2 `MultiheadAttention`: x [d], M [m,d], P_q/P_k [h,d,k],
    P_v/P_o [h,d,v] -> y [d]."""
    x, M = np.asarray(x, dtype=F64), np.asarray(M, dtype=F64)
    return _layer(x[None, None, :], M[None], None, P_q, P_k, P_v, P_o, shared_kv=False)[0, 0]


def multiquery_attention(x, M, P_q, P_k, P_v, P_o):
    """The Section 2.2 layer under the Section 3 rule (K, V, P_k, P_v lose the heads
    dimension): P_k [d,k], P_v [d,v]."""
    x, M = np.asarray(x, dtype=F64), np.asarray(M, dtype=F64)
    return _layer(x[None, None, :], M[None], None, P_q, P_k, P_v, P_o, shared_kv=True)[0, 0]


def causal_mask(b, h, n, m=None):
    """Additive mask of Section 2.3: 0 where position j <= i, -inf elsewhere."""
    m = n if m is None else m
    i = np.arange(n)[:, None]
    j = np.arange(m)[None, :]
    mask = np.where(j <= i, 0.0, -np.inf)
    return np.broadcast_to(mask, (b, h, n, m)).copy()


def multihead_attention_batched(X, M, mask, P_q, P_k, P_v, P_o, kv_round=None):
    """Section 2.3 `MultiheadAttentionBatched`: X [b,n,d], M [b,m,d],
    mask [b,h,n,m] -> Y [b,n,d].  `kv_round`, if given, is applied to K and V
    (used to mirror a reduced-precision cache)."""
    return _layer(X, M, mask, P_q, P_k, P_v, P_o, shared_kv=False, kv_round=kv_round)


def multiquery_attention_batched(X, M, mask, P_q, P_k, P_v, P_o, kv_round=None):
    """Section 3 `MultiqueryAttentionBatched`: as above with one K [m,k] and one V [m,v] per
    sequence, P_k [d,k], P_v [d,v]."""
    return _layer(X, M, mask, P_q, P_k, P_v, P_o, shared_kv=True, kv_round=kv_round)


# --------------------------------------------------------------------------
# the pieces of one incremental step (Section 2.4 and Section 3 listings)
# --------------------------------------------------------------------------
def project_q(x, P_q):
    """q = einsum('bd,hdk->bhk') (first line of both incremental listings)."""
    return np.einsum("bd,hdk->bhk", np.asarray(x, dtype=F64), np.asarray(P_q, dtype=F64), optimize=True)


def project_kv(x, P):
    """Multi-query new row: einsum('bd,dk->bk') (Section 3 incremental listing)."""
    return np.einsum("bd,dk->bk", np.asarray(x, dtype=F64), np.asarray(P, dtype=F64), optimize=True)


def project_kv_mh(x, P):
    """Multi-head new rows: einsum('bd,hdk->bhk') (Section 2.4 listing)."""
    return np.einsum("bd,hdk->bhk", np.asarray(x, dtype=F64), np.asarray(P, dtype=F64), optimize=True)


def project_o(o, P_o):
    """y = einsum('bhv,hdv->bd') (last line of both incremental listings;
    note P_o is [h,d,v], model width before value width)."""
    return np.einsum("bhv,hdv->bd", np.asarray(o, dtype=F64), np.asarray(P_o, dtype=F64), optimize=True)


def round_to_bf16(a):
    """float -> nearest bfloat16 (ties to even) via float32, returned as
    float64 holding the exactly representable value.  NaN stays NaN."""
    f = np.ascontiguousarray(np.asarray(a, dtype=F64).astype(np.float32))
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    r = ((u + np.uint64(0x7FFF) + lsb) >> np.uint64(16)) << np.uint64(16)
    out = r.astype(np.uint32).view(np.float32).astype(F64)
    return np.where(np.isnan(f), np.nan, out).reshape(np.shape(a))


def round_to_f32(a):
    return np.asarray(a, dtype=F64).astype(np.float32).astype(F64)


_CACHE_ROUND = {"f64": lambda a: np.asarray(a, dtype=F64), "f32": round_to_f32, "bf16": round_to_bf16}


def append_kv(K, V, k_new, v_new, lens, cache="f64"):
    """In-place form of the listings' concat: write the new row at position
    lens[i] of sequence i, then lens[i] += 1.  K is [b,cap,k] (multi-query,
    k_new [b,k]) or [b,h,cap,k] (multi-head, k_new [b,h,k]); same for V.
    A sequence already at capacity is left untouched."""
    rnd = _CACHE_ROUND[cache]
    k_new, v_new = rnd(k_new), rnd(v_new)
    cap = K.shape[-2]
    for i in range(K.shape[0]):
        L = int(lens[i])
        if L >= cap:
            continue
        K[i, ..., L, :] = k_new[i]
        V[i, ..., L, :] = v_new[i]
        lens[i] = L + 1


def mqa_decode_weights(q, K, lens, scale=1.0):
    """softmax weights of the Section 3 step: list over sequences of [h, len_i]."""
    q, K = np.asarray(q, dtype=F64), np.asarray(K, dtype=F64)
    out = []
    for i in range(q.shape[0]):
        L = int(lens[i])
        if L == 0:
            out.append(np.zeros((q.shape[1], 0)))
            continue
        logits = scale * np.einsum("hk,mk->hm", q[i], K[i, :L], optimize=True)
        out.append(softmax64(logits))
    return out


def mqa_decode(q, K, V, lens, scale=1.0, window=None):
    """Attention part of `MultiquerySelfAttentionIncremental` (Section 3):
    logits = einsum('bhk,bmk->bhm'), softmax over m, o = einsum('bhm,bmv->bhv'),
    restricted per sequence to its first lens[i] positions.
    q [b,h,k], K [b,cap,k], V [b,cap,v] -> o [b,h,v].
    `window` = W gives the "local" variant of Section 4.1: only the current position
    and the W-1 before it, i.e. positions [max(0, lens[i]-W), lens[i])."""
    q, K, V = (np.asarray(a, dtype=F64) for a in (q, K, V))
    b, h, _ = q.shape
    o = np.zeros((b, h, V.shape[-1]), dtype=F64)
    for i in range(b):
        L = int(lens[i])
        if L == 0:
            continue
        lo = 0 if window is None else max(0, L - int(window))
        logits = scale * np.einsum("hk,mk->hm", q[i], K[i, lo:L], optimize=True)
        weights = softmax64(logits)
        o[i] = np.einsum("hm,mv->hv", weights, V[i, lo:L], optimize=True)
    return o


def mqa_prefill(q, K, V, lens, scale=1.0):
    """Attention of the Section 3 batched listing (`MultiqueryAttentionBatched`) for n consecutive
    queries per sequence against a cache that already holds their rows, with the causal mask of
    Section 2.3: q [b,n,h,k]; query j of sequence i sits at position lens[i]-n+j and attends to
    positions 0..lens[i]-n+j.  Returns o [b,n,h,v]."""
    q, K, V = (np.asarray(a, dtype=F64) for a in (q, K, V))
    b, n, h, _ = q.shape
    o = np.zeros((b, n, h, V.shape[-1]), dtype=F64)
    for i in range(b):
        L = int(lens[i])
        pos = L - n + np.arange(n)                                   # positions of the n queries
        logits = scale * np.einsum("nhk,mk->hnm", q[i], K[i, :L], optimize=True)
        mask = np.where(np.arange(L)[None, :] <= pos[:, None], 0.0, -np.inf)      # [n, L]
        weights = softmax64(logits + mask[None])
        o[i] = np.einsum("hnm,mv->nhv", weights, V[i, :L], optimize=True)
    return o


def mqa_decode_beams(q, K_src, V_src, lens_src, K_beam, V_beam, lens_beam, scale=1.0):
    """Beam search decoding (Section 4.1 decodes with beam 4; Table 2's last column) of the
    Section 3 step when the `beam` hypotheses of a source share their first positions (the source
    or prompt) and differ only in the positions each hypothesis produced itself.  The memory of
    hypothesis (i, e) is, by definition, the rows K_src[i, :lens_src[i]] followed by
    K_beam[i, e, :lens_beam[i, e]] (likewise V); the step is plain dot-product attention over it.
    q [b,beam,h,k], K_src [b,cap_s,k], V_src [b,cap_s,v], K_beam [b,beam,cap_t,k],
    V_beam [b,beam,cap_t,v], lens_beam [b,beam] -> o [b,beam,h,v]."""
    q, K_src, V_src, K_beam, V_beam = (np.asarray(a, dtype=F64) for a in (q, K_src, V_src, K_beam, V_beam))
    lens_beam = np.asarray(lens_beam).reshape(q.shape[0], q.shape[1])
    b, beam, h, _ = q.shape
    o = np.zeros((b, beam, h, V_src.shape[-1]), dtype=F64)
    for i in range(b):
        Ls = int(lens_src[i])
        for e in range(beam):
            Lt = int(lens_beam[i, e])
            Kmem = np.concatenate([K_src[i, :Ls], K_beam[i, e, :Lt]], axis=0)
            Vmem = np.concatenate([V_src[i, :Ls], V_beam[i, e, :Lt]], axis=0)
            if Kmem.shape[0] == 0:
                continue
            for j in range(h):
                o[i, e, j] = dot_product_attention(scale * q[i, e, j], Kmem, Vmem)
    return o


def beam_reorder_kv(K, V, lens, parent):
    """Cache bookkeeping of beam search: after a step, hypothesis slot r continues hypothesis
    parent[r] (slots are numbered over all sources, r = i*beam + e), so it takes over that
    hypothesis' rows and length.  K [n,cap,k] (or [n,h,cap,k]), lens [n], parent [n] ->
    (K', V', lens').  Rows at and beyond the length are never read; they are returned as zeros."""
    K, V = np.asarray(K), np.asarray(V)
    lens, parent = np.asarray(lens), np.asarray(parent)
    K2, V2 = np.zeros_like(K), np.zeros_like(V)
    lens2 = lens[parent].copy()
    for r in range(K.shape[0]):
        L = int(lens2[r])
        K2[r, ..., :L, :] = K[parent[r], ..., :L, :]
        V2[r, ..., :L, :] = V[parent[r], ..., :L, :]
    return K2, V2, lens2


def mha_prefill(q, K, V, lens, scale=1.0):
    """Attention of the Section 2.3 batched listing (`MultiheadAttentionBatched`) with its causal
    mask, for n consecutive queries per sequence against per-head caches that already hold their
    rows: q [b,h,n,k], K [b,h,cap,k], V [b,h,cap,v]; query j of sequence i sits at position
    lens[i]-n+j and attends to positions 0..lens[i]-n+j of its own head.  Returns o [b,h,n,v]."""
    q, K, V = (np.asarray(a, dtype=F64) for a in (q, K, V))
    b, h, n, _ = q.shape
    o = np.zeros((b, h, n, V.shape[-1]), dtype=F64)
    for i in range(b):
        L = int(lens[i])
        pos = L - n + np.arange(n)
        mask = np.where(np.arange(L)[None, :] <= pos[:, None], 0.0, -np.inf)      # [n, L]
        for j in range(h):
            logits = scale * np.einsum("nk,mk->nm", q[i, j], K[i, j, :L], optimize=True)
            o[i, j] = np.einsum("nm,mv->nv", softmax64(logits + mask), V[i, j, :L], optimize=True)
    return o


def mha_decode(q, K, V, lens, scale=1.0, window=None):
    """Attention part of `MultiheadSelfAttentionIncremental` (Section 2.4):
    logits = einsum('bhk,bhmk->bhm'), softmax, o = einsum('bhm,bhmv->bhv').
    q [b,h,k], K [b,h,cap,k], V [b,h,cap,v] -> o [b,h,v].  `window` as in mqa_decode."""
    q, K, V = (np.asarray(a, dtype=F64) for a in (q, K, V))
    b, h, _ = q.shape
    o = np.zeros((b, h, V.shape[-1]), dtype=F64)
    for i in range(b):
        L = int(lens[i])
        if L == 0:
            continue
        lo = 0 if window is None else max(0, L - int(window))
        logits = scale * np.einsum("hk,hmk->hm", q[i], K[i, :, lo:L], optimize=True)
        weights = softmax64(logits)
        o[i] = np.einsum("hm,hmv->hv", weights, V[i, :, lo:L], optimize=True)
    return o


def mqa_incremental_step(x, K, V, lens, P_q, P_k, P_v, P_o, cache="f64", scale=1.0):
    """`MultiquerySelfAttentionIncremental` (Section 3) on capacity buffers:
    project q and the new K/V row, append (mutates K, V, lens), attend over all
    positions including the new one, project out.  Returns (y [b,d], o, q)."""
    q = project_q(x, P_q)
    append_kv(K, V, project_kv(x, P_k), project_kv(x, P_v), lens, cache)
    o = mqa_decode(q, K, V, lens, scale)
    return project_o(o, P_o), o, q


def mha_incremental_step(x, K, V, lens, P_q, P_k, P_v, P_o, cache="f64", scale=1.0):
    """`MultiheadSelfAttentionIncremental` (Section 2.4) on capacity buffers."""
    q = project_q(x, P_q)
    append_kv(K, V, project_kv_mh(x, P_k), project_kv_mh(x, P_v), lens, cache)
    o = mha_decode(q, K, V, lens, scale)
    return project_o(o, P_o), o, q


# --------------------------------------------------------------------------
# splitting the softmax over disjoint position ranges and recombining
# (follows from the Section 2.1 softmax definition; the GPU path's second pass)
# --------------------------------------------------------------------------
def partial_state(q_i, K_i, V_i, lo, hi, scale=1.0):
    """For one sequence and positions [lo,hi): per head the maximum logit, the
    sum of exp(logit - max) and the un-normalised weighted sum of V rows."""
    h = q_i.shape[0]
    if hi <= lo:
        return np.full((h,), -np.inf), np.zeros((h,)), np.zeros((h, V_i.shape[-1]))
    logits = scale * np.einsum("hk,mk->hm", np.asarray(q_i, F64), np.asarray(K_i[lo:hi], F64))
    mx = logits.max(axis=1)
    e = np.exp(logits - mx[:, None])
    return mx, e.sum(axis=1), np.einsum("hm,mv->hv", e, np.asarray(V_i[lo:hi], F64))


def combine_partials(states):
    """Merge partial states (max_i, sum_i, acc_i): M = max max_i,
    L = sum_i sum_i e^{max_i - M}, o = sum_i acc_i e^{max_i - M} / L."""
    mx = np.stack([s[0] for s in states])            # [S,h]
    M = mx.max(axis=0)
    if np.all(np.isneginf(M)):
        return np.zeros_like(states[0][2])
    w = np.exp(mx - np.where(np.isneginf(M), 0.0, M)[None])   # [S,h]
    L = np.sum(w * np.stack([s[1] for s in states]), axis=0)
    acc = np.sum(w[:, :, None] * np.stack([s[2] for s in states]), axis=0)
    with np.errstate(invalid="ignore", divide="ignore"):
        o = acc / L[:, None]
    return np.where(L[:, None] > 0, o, 0.0)

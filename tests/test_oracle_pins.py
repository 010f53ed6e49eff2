"""Pins for the float64 oracle: everything here runs on the CPU and checks the
oracle against facts fixed by the paper or by mathematics, never against
itself.  A dropped term, wrong sign, wrong axis or transposed operand in any
oracle function fails at least one of these."""
import math
import os

import numpy as np
import pytest
import scipy.special
import torch

from oracle import brute_force as bf
from oracle import mqa_oracle as orc

HERE = os.path.dirname(os.path.abspath(__file__))


def _rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------- brute force
@pytest.mark.parametrize("seed", range(12))
def test_decode_matches_enumeration(seed):
    g = _rng(seed)
    b, h, m = g.integers(1, 3), g.integers(1, 4), g.integers(1, 6)
    k, v = g.integers(1, 5), g.integers(1, 5)
    q = g.normal(size=(b, h, k)) * 2
    K = g.normal(size=(b, m, k))
    V = g.normal(size=(b, m, v))
    lens = g.integers(0, m + 1, size=b)
    scale = float(g.choice([1.0, 0.37]))
    got = orc.mqa_decode(q, K, V, lens, scale)
    ref = np.array(bf.mqa_decode_bf(q.tolist(), K.tolist(), V.tolist(), lens.tolist(), scale))
    assert np.max(np.abs(got - ref)) <= 1e-14
    Kh = g.normal(size=(b, h, m, k))
    Vh = g.normal(size=(b, h, m, v))
    got = orc.mha_decode(q, Kh, Vh, lens, scale)
    ref = np.array(bf.mha_decode_bf(q.tolist(), Kh.tolist(), Vh.tolist(), lens.tolist(), scale))
    assert np.max(np.abs(got - ref)) <= 1e-14


@pytest.mark.parametrize("seed", range(6))
def test_projections_match_enumeration(seed):
    g = _rng(100 + seed)
    b, h, d, k, v = g.integers(1, 3), g.integers(1, 4), g.integers(1, 6), g.integers(1, 5), g.integers(1, 5)
    x = g.normal(size=(b, d))
    P_q, P_k = g.normal(size=(h, d, k)), g.normal(size=(d, k))
    P_o, o = g.normal(size=(h, d, v)), g.normal(size=(b, h, v))
    assert np.allclose(orc.project_q(x, P_q), bf.project_q_bf(x.tolist(), P_q.tolist()), atol=1e-14, rtol=0)
    assert np.allclose(orc.project_kv(x, P_k), bf.project_kv_bf(x.tolist(), P_k.tolist()), atol=1e-14, rtol=0)
    assert np.allclose(orc.project_o(o, P_o), bf.project_o_bf(o.tolist(), P_o.tolist()), atol=1e-14, rtol=0)
    # multi-head K projection is the multi-query one applied per head
    P_kh = g.normal(size=(h, d, k))
    got = orc.project_kv_mh(x, P_kh)
    for j in range(h):
        assert np.allclose(got[:, j], bf.project_kv_bf(x.tolist(), P_kh[j].tolist()), atol=1e-14, rtol=0)


def test_output_projection_orientation():
    """P_o is [h,d,v]: a one-hot P_o[j,t,c] routes o[:,j,c] to y[:,t]."""
    h, d, v = 3, 5, 4
    o = _rng(1).normal(size=(2, h, v))
    P_o = np.zeros((h, d, v))
    P_o[2, 4, 1] = 1.0
    y = orc.project_o(o, P_o)
    expect = np.zeros((2, d))
    expect[:, 4] = o[:, 2, 1]
    assert np.array_equal(y, expect)


# ---------------------------------------------------------------- worked example
def test_hand_worked_example():
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "two_position_example.txt"))
            if l.strip() and not l.startswith("#")]
    K = np.array([[[0.0], [1.0]]])
    V = np.array([[[4.0, -8.0], [8.0, 0.0]]])
    q = np.array([[[math.log(3)], [0.0], [-math.log(3)]]])
    o = orc.mqa_decode(q, K, V, [2])
    w = orc.mqa_decode_weights(q, K, [2])[0]
    for r in rows:
        j = int(r[0])
        assert np.allclose(w[j], [float(r[1]), float(r[2])], atol=1e-15, rtol=0)
        assert np.allclose(o[0, j], [float(r[3]), float(r[4])], atol=1e-14, rtol=0)
    # the single-query function of Section 2.1 gives the same numbers
    assert np.allclose(orc.dot_product_attention(q[0, 0], K[0], V[0]), [7.0, -2.0], atol=1e-14, rtol=0)


# ---------------------------------------------------------------- softmax
def test_softmax_against_scipy_and_normalisation():
    g = _rng(3)
    z = g.normal(size=(4, 7, 33)) * 20
    w = orc.softmax64(z)
    assert np.max(np.abs(w - scipy.special.softmax(z, axis=-1))) <= 1e-15
    assert np.all(w >= 0)
    for row in w.reshape(-1, 33):
        assert abs(math.fsum(row.tolist()) - 1.0) <= 1e-15
    # huge logits do not overflow
    w = orc.softmax64(np.array([1000.0, 1000.0, -1000.0]))
    assert np.allclose(w, [0.5, 0.5, 0.0], atol=1e-16, rtol=0)


def test_decode_weights_sum_to_one():
    g = _rng(4)
    q, K = g.normal(size=(3, 5, 8)) * 3, g.normal(size=(3, 40, 8))
    lens = [40, 17, 1]
    for i, w in enumerate(orc.mqa_decode_weights(q, K, lens)):
        assert w.shape == (5, lens[i])
        assert np.all(w >= 0)
        for row in w:
            assert abs(math.fsum(row.tolist()) - 1.0) <= 1e-15


# ---------------------------------------------------------------- MQA == MHA with shared K/V
def test_mqa_equals_mha_with_shared_kv():
    g = _rng(5)
    b, h, m, k, v = 3, 6, 19, 8, 5
    q = g.normal(size=(b, h, k))
    K, V = g.normal(size=(b, m, k)), g.normal(size=(b, m, v))
    lens = [19, 7, 1]
    Kh = np.repeat(K[:, None], h, axis=1)
    Vh = np.repeat(V[:, None], h, axis=1)
    assert np.max(np.abs(orc.mqa_decode(q, K, V, lens) - orc.mha_decode(q, Kh, Vh, lens))) <= 1e-15


def test_layer_level_mqa_equals_mha_with_replicated_projections():
    g = _rng(6)
    h, d, m, k, v = 4, 10, 9, 3, 5
    x, M = g.normal(size=(d,)), g.normal(size=(m, d))
    P_q, P_o = g.normal(size=(h, d, k)), g.normal(size=(h, d, v))
    P_k, P_v = g.normal(size=(d, k)), g.normal(size=(d, v))
    y_mq = orc.multiquery_attention(x, M, P_q, P_k, P_v, P_o)
    y_mh = orc.multihead_attention(x, M, P_q, np.repeat(P_k[None], h, 0), np.repeat(P_v[None], h, 0), P_o)
    assert np.max(np.abs(y_mq - y_mh)) <= 1e-13
    # one head: multi-head, multi-query and the single-query function coincide
    q = np.einsum("d,dk->k", x, P_q[0])
    y1 = orc.dot_product_attention(q, M @ P_k, M @ P_v) @ P_o[0].T
    assert np.max(np.abs(orc.multiquery_attention(x, M, P_q[:1], P_k, P_v, P_o[:1]) - y1)) <= 1e-13


# ---------------------------------------------------------------- incremental == batched causal
@pytest.mark.parametrize("cache", ["f64", "bf16"])
def test_incremental_equals_causal_batched(cache):
    g = _rng(7)
    b, n, d, h, k, v = 2, 9, 12, 3, 4, 5
    X = g.normal(size=(b, n, d))
    P_q, P_o = g.normal(size=(h, d, k)) / 3, g.normal(size=(h, d, v))
    P_k, P_v = g.normal(size=(d, k)) / 3, g.normal(size=(d, v))
    P_kh, P_vh = g.normal(size=(h, d, k)) / 3, g.normal(size=(h, d, v))
    rnd = None if cache == "f64" else orc.round_to_bf16
    mask = orc.causal_mask(b, h, n)

    K, V = np.full((b, n, k), np.nan), np.full((b, n, v), np.nan)
    lens = np.zeros(b, dtype=np.int64)
    ys = [orc.mqa_incremental_step(X[:, t], K, V, lens, P_q, P_k, P_v, P_o, cache)[0] for t in range(n)]
    Y = orc.multiquery_attention_batched(X, X, mask, P_q, P_k, P_v, P_o, kv_round=rnd)
    assert np.max(np.abs(np.stack(ys, 1) - Y)) <= 1e-12
    assert list(lens) == [n] * b

    K, V = np.full((b, h, n, k), np.nan), np.full((b, h, n, v), np.nan)
    lens = np.zeros(b, dtype=np.int64)
    ys = [orc.mha_incremental_step(X[:, t], K, V, lens, P_q, P_kh, P_vh, P_o, cache)[0] for t in range(n)]
    Y = orc.multihead_attention_batched(X, X, mask, P_q, P_kh, P_vh, P_o, kv_round=rnd)
    assert np.max(np.abs(np.stack(ys, 1) - Y)) <= 1e-12


def test_batched_matches_single_query_listing():
    """Section 2.3 / Section 3 batched forms with an all-zero mask reduce to the
    one-query listings of Section 2.2 applied per (sequence, position)."""
    g = _rng(8)
    b, n, m, d, h, k, v = 2, 3, 4, 6, 2, 3, 2
    X, M = g.normal(size=(b, n, d)), g.normal(size=(b, m, d))
    P_q, P_o = g.normal(size=(h, d, k)), g.normal(size=(h, d, v))
    P_k, P_v = g.normal(size=(d, k)), g.normal(size=(d, v))
    P_kh, P_vh = g.normal(size=(h, d, k)), g.normal(size=(h, d, v))
    zero = np.zeros((b, h, n, m))
    Yq = orc.multiquery_attention_batched(X, M, zero, P_q, P_k, P_v, P_o)
    Yh = orc.multihead_attention_batched(X, M, zero, P_q, P_kh, P_vh, P_o)
    for i in range(b):
        for t in range(n):
            assert np.allclose(Yq[i, t], orc.multiquery_attention(X[i, t], M[i], P_q, P_k, P_v, P_o), atol=1e-13, rtol=0)
            assert np.allclose(Yh[i, t], orc.multihead_attention(X[i, t], M[i], P_q, P_kh, P_vh, P_o), atol=1e-13, rtol=0)


def test_causal_mask_values():
    mk = orc.causal_mask(1, 1, 3)[0, 0]
    assert np.array_equal(mk == 0, np.tril(np.ones((3, 3), bool)))
    assert np.all(np.isneginf(mk[~np.tril(np.ones((3, 3), bool))]))


# ---------------------------------------------------------------- closed forms
def test_closed_forms():
    g = _rng(9)
    b, h, m, k, v = 2, 4, 23, 6, 5
    q, K, V = g.normal(size=(b, h, k)), g.normal(size=(b, m, k)), g.normal(size=(b, m, v))
    full = [m, m]
    # one valid position: output is that V row for every head
    o = orc.mqa_decode(q, K, V, [1, 1])
    assert np.array_equal(o, np.repeat(V[:, :1], h, axis=1))
    # zero query (or zero keys): uniform weights -> mean of the valid V rows
    o = orc.mqa_decode(np.zeros_like(q), K, V, [m, 10])
    assert np.allclose(o[0], V[0].mean(0)[None].repeat(h, 0), atol=1e-15, rtol=0)
    assert np.allclose(o[1], V[1, :10].mean(0)[None].repeat(h, 0), atol=1e-15, rtol=0)
    o = orc.mqa_decode(q, np.zeros_like(K), V, full)
    assert np.allclose(o[0, 2], V[0].mean(0), atol=1e-15, rtol=0)
    # one dominant logit: output approaches that V row, error <= (L-1) e^{-gap} max|V| * 2
    K2 = K.copy()
    K2[0, 5] = 40.0 * q[0, 1] / (q[0, 1] @ q[0, 1])
    o = orc.mqa_decode(q, K2, V, full)
    logits = K2[0] @ q[0, 1]
    gap = logits[5] - np.max(np.delete(logits, 5))
    assert gap > 20
    assert np.max(np.abs(o[0, 1] - V[0, 5])) <= 2 * (m - 1) * math.exp(-gap) * np.max(np.abs(V))
    # adding one vector u to every key shifts all logits of a head equally: no change
    u = g.normal(size=(k,))
    assert np.max(np.abs(orc.mqa_decode(q, K + u, V, full) - orc.mqa_decode(q, K, V, full))) <= 1e-13
    # joint permutation of the (K,V) rows: no change
    p = g.permutation(m)
    assert np.max(np.abs(orc.mqa_decode(q, K[:, p], V[:, p], full) - orc.mqa_decode(q, K, V, full))) <= 1e-14
    # outputs lie in the convex hull of the V rows, coordinate-wise
    o = orc.mqa_decode(q * 3, K, V, [m, 7])
    assert np.all(o[0] <= V[0].max(0) + 1e-15) and np.all(o[0] >= V[0].min(0) - 1e-15)
    assert np.all(o[1] <= V[1, :7].max(0) + 1e-15) and np.all(o[1] >= V[1, :7].min(0) - 1e-15)
    # head independence and sequence independence
    q2 = q.copy()
    q2[:, 0] += 1.0
    o1, o2 = orc.mqa_decode(q, K, V, full), orc.mqa_decode(q2, K, V, full)
    assert np.array_equal(o1[:, 1:], o2[:, 1:]) and not np.allclose(o1[:, 0], o2[:, 0])
    # scale multiplies the logits: same as scaling q
    assert np.max(np.abs(orc.mqa_decode(q, K, V, full, scale=0.25) - orc.mqa_decode(0.25 * q, K, V, full))) <= 1e-14
    assert np.max(np.abs(orc.mha_decode(q, np.repeat(K[:, None], h, 1), np.repeat(V[:, None], h, 1), full, scale=0.25)
                         - orc.mqa_decode(0.25 * q, K, V, full))) <= 1e-14
    # empty sequence -> zeros
    assert np.array_equal(orc.mqa_decode(q, K, V, [0, 3])[0], np.zeros((h, v)))


def test_mha_heads_use_their_own_kv():
    g = _rng(10)
    b, h, m, k, v = 2, 3, 11, 4, 6
    q = g.normal(size=(b, h, k))
    K, V = g.normal(size=(b, h, m, k)), g.normal(size=(b, h, m, v))
    o = orc.mha_decode(q, K, V, [m, 5])
    for i, L in enumerate([m, 5]):
        for j in range(h):
            assert np.allclose(o[i, j], orc.dot_product_attention(q[i, j], K[i, j, :L], V[i, j, :L]), atol=1e-15, rtol=0)


# ---------------------------------------------------------------- independent library routine
def test_against_torch_sdpa_float64():
    g = _rng(11)
    b, h, m, k, v = 3, 5, 37, 16, 16
    q, K, V = g.normal(size=(b, h, k)), g.normal(size=(b, m, k)), g.normal(size=(b, m, v))
    tq = torch.from_numpy(q)[:, :, None, :]
    tK = torch.from_numpy(K)[:, None].expand(b, h, m, k)
    tV = torch.from_numpy(V)[:, None].expand(b, h, m, v)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tK, tV, scale=1.0)[:, :, 0].numpy()
    assert np.max(np.abs(orc.mqa_decode(q, K, V, [m] * b) - ref)) <= 1e-13
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tK, tV, scale=0.5)[:, :, 0].numpy()
    assert np.max(np.abs(orc.mqa_decode(q, K, V, [m] * b, scale=0.5) - ref)) <= 1e-13


# ---------------------------------------------------------------- masking by length
def test_rows_beyond_length_are_never_read():
    g = _rng(12)
    b, h, cap, k, v = 3, 2, 12, 4, 4
    q, K, V = g.normal(size=(b, h, k)), g.normal(size=(b, cap, k)), g.normal(size=(b, cap, v))
    lens = [12, 5, 0]
    ref = orc.mqa_decode(q, K, V, lens)
    Kp, Vp = K.copy(), V.copy()
    for i, L in enumerate(lens):
        Kp[i, L:], Vp[i, L:] = np.nan, np.nan
    got = orc.mqa_decode(q, Kp, Vp, lens)
    assert np.array_equal(got, ref) and not np.any(np.isnan(got))
    Kh, Vh = np.repeat(Kp[:, None], h, 1), np.repeat(Vp[:, None], h, 1)
    assert np.max(np.abs(orc.mha_decode(q, Kh, Vh, lens) - ref)) <= 1e-15


# ---------------------------------------------------------------- split + combine
@pytest.mark.parametrize("seed", range(5))
def test_split_combine_reproduces_unsplit(seed):
    g = _rng(20 + seed)
    h, L, k, v = 3, 50, 8, 6
    q, K, V = g.normal(size=(h, k)) * 4, g.normal(size=(L, k)), g.normal(size=(L, v))
    cuts = np.sort(g.choice(np.arange(0, L + 1), size=4))
    bounds = [0, *cuts.tolist(), L]         # may contain empty ranges
    states = [orc.partial_state(q, K, V, lo, hi) for lo, hi in zip(bounds[:-1], bounds[1:])]
    ref = orc.mqa_decode(q[None], K[None], V[None], [L])[0]
    assert np.max(np.abs(orc.combine_partials(states) - ref)) <= 1e-14
    empty = [orc.partial_state(q, K, V, 3, 3)]
    assert np.array_equal(orc.combine_partials(empty), np.zeros((h, v)))


# ---------------------------------------------------------------- append and bf16
def test_bf16_rounding_matches_torch():
    g = _rng(13)
    x = np.concatenate([
        g.normal(size=20000) * np.exp(g.normal(size=20000) * 8),
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40, -1e-40, np.inf, -np.inf]),
        (np.arange(0x3F800000, 0x3F800000 + 0x40000, 0x4000, dtype=np.uint32) + 0x8000).view(np.float32),  # exact ties
    ]).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    got = orc.round_to_bf16(x)
    assert np.array_equal(got, ref)
    assert np.isnan(orc.round_to_bf16(np.array([np.nan]))[0])


def test_append_semantics():
    b, cap, k, v = 3, 4, 2, 3
    K, V = np.full((b, cap, k), np.nan), np.full((b, cap, v), np.nan)
    lens = np.array([0, 2, 4])
    k_new = np.array([[1.0, 2.0], [3.0, 4.0], [5.0, 6.0]]) + 2.0 ** -12
    v_new = np.arange(9.0).reshape(3, 3)
    orc.append_kv(K, V, k_new, v_new, lens, cache="bf16")
    assert list(lens) == [1, 3, 4]                       # full sequence untouched
    assert np.array_equal(K[0, 0], [1.0, 2.0]) and np.array_equal(K[1, 2], [3.0, 4.0])
    assert np.array_equal(V[1, 2], [3.0, 4.0, 5.0])
    assert np.all(np.isnan(K[2])) and np.all(np.isnan(K[0, 1:])) and np.all(np.isnan(K[1, [0, 1, 3]]))
    # float32 cache keeps float32 rounding only
    K32, V32 = np.zeros((1, 2, 2)), np.zeros((1, 2, 3))
    l32 = np.array([1])
    orc.append_kv(K32, V32, k_new[:1], v_new[:1], l32, cache="f32")
    assert np.array_equal(K32[0, 1], k_new[0].astype(np.float32).astype(np.float64)) and l32[0] == 2
    # multi-head layout
    Kh, Vh = np.zeros((1, 2, 3, 2)), np.zeros((1, 2, 3, 3))
    lh = np.array([1])
    orc.append_kv(Kh, Vh, np.arange(4.0).reshape(1, 2, 2), np.arange(6.0).reshape(1, 2, 3), lh, cache="f64")
    assert np.array_equal(Kh[0, :, 1], [[0, 1], [2, 3]]) and np.array_equal(Vh[0, 1, 1], [3, 4, 5]) and lh[0] == 2
    assert np.all(Kh[0, :, [0, 2]] == 0)


# ---------------------------------------------------------------- local window (Section 4.1)
def test_window_is_a_shortened_cache():
    g = _rng(30)
    b, h, m, k, v = 3, 4, 40, 6, 5
    q, K, V = g.normal(size=(b, h, k)), g.normal(size=(b, m, k)), g.normal(size=(b, m, v))
    lens = [40, 13, 3]
    for W in (1, 5, 32, 100):
        got = orc.mqa_decode(q, K, V, lens, window=W)
        for i, L in enumerate(lens):
            lo = max(0, L - W)
            ref = orc.mqa_decode(q[i:i + 1], K[i:i + 1, lo:L], V[i:i + 1, lo:L], [L - lo])    # the pinned full form
            assert np.max(np.abs(got[i] - ref[0])) <= 1e-15
        assert np.max(np.abs(got - np.array(bf.mqa_decode_bf(q.tolist(), K.tolist(), V.tolist(), lens, 1.0, W)))) <= 1e-14
    # a window of one position returns the newest V row; a window longer than the cache changes nothing
    assert np.array_equal(orc.mqa_decode(q, K, V, lens, window=1)[1], np.repeat(V[1, 12:13], h, 0))
    assert np.array_equal(orc.mqa_decode(q, K, V, lens, window=64), orc.mqa_decode(q, K, V, lens))
    Kh, Vh = np.repeat(K[:, None], h, 1), np.repeat(V[:, None], h, 1)
    assert np.max(np.abs(orc.mha_decode(q, Kh, Vh, lens, window=5) - orc.mqa_decode(q, K, V, lens, window=5))) <= 1e-15


# ---------------------------------------------------------------- prompt attention (causal, batched)
def test_prefill_equals_stepwise_decode_and_batched_listing():
    g = _rng(31)
    b, n, h, k, v, d = 2, 7, 3, 4, 5, 6
    prefix = [0, 4]                                  # positions already in the cache before the n new ones
    cap = n + 4
    K, V = g.normal(size=(b, cap, k)), g.normal(size=(b, cap, v))
    q = g.normal(size=(b, n, h, k))
    lens = [prefix[0] + n, prefix[1] + n]
    got = orc.mqa_prefill(q, K, V, lens, scale=0.7)
    for i in range(b):
        for j in range(n):                           # one query at a time through the pinned decode step
            ref = orc.mqa_decode(q[i:i + 1, j], K[i:i + 1], V[i:i + 1], [prefix[i] + j + 1], scale=0.7)
            assert np.max(np.abs(got[i, j] - ref[0])) <= 1e-14
    # whole layer: projections + prefill attention == the Section 3 batched listing with a causal mask
    X = g.normal(size=(b, n, d))
    P_q, P_o = g.normal(size=(h, d, k)), g.normal(size=(h, d, v))
    P_k, P_v = g.normal(size=(d, k)), g.normal(size=(d, v))
    Kc = np.einsum("bnd,dk->bnk", X, P_k)
    Vc = np.einsum("bnd,dv->bnv", X, P_v)
    Q = np.einsum("bnd,hdk->bnhk", X, P_q)
    o = orc.mqa_prefill(Q, Kc, Vc, [n, n])
    Y = np.einsum("bnhv,hdv->bnd", o, P_o)
    ref = orc.multiquery_attention_batched(X, X, orc.causal_mask(b, h, n), P_q, P_k, P_v, P_o)
    assert np.max(np.abs(Y - ref)) <= 1e-12


def test_mha_prefill_pins():
    g = _rng(33)
    b, n, h, k, v, d = 2, 6, 3, 4, 5, 7
    prefix = [0, 3]
    cap = n + 4
    K, V = g.normal(size=(b, h, cap, k)), g.normal(size=(b, h, cap, v))
    q = g.normal(size=(b, h, n, k))
    lens = [prefix[0] + n, prefix[1] + n]
    got = orc.mha_prefill(q, K, V, lens, scale=1.3)
    for i in range(b):
        for j in range(n):                           # one query at a time through the pinned multi-head step
            ref = orc.mha_decode(q[i:i + 1, :, j], K[i:i + 1], V[i:i + 1], [prefix[i] + j + 1], scale=1.3)
            assert np.max(np.abs(got[i, :, j] - ref[0])) <= 1e-14
    # every head reading the same K/V: the multi-query prefill (other q layout)
    Ks, Vs = K[:, 0], V[:, 0]
    same = orc.mha_prefill(q, np.repeat(Ks[:, None], h, 1), np.repeat(Vs[:, None], h, 1), lens)
    assert np.max(np.abs(same.transpose(0, 2, 1, 3) - orc.mqa_prefill(q.transpose(0, 2, 1, 3), Ks, Vs, lens))) <= 1e-14
    # whole layer == the Section 2.3 batched listing with a causal mask
    X = g.normal(size=(b, n, d))
    P_q, P_k, P_v, P_o = (g.normal(size=(h, d, e)) for e in (k, k, v, v))
    Q = np.einsum("bnd,hdk->bhnk", X, P_q)
    Kc = np.einsum("bnd,hdk->bhnk", X, P_k)
    Vc = np.einsum("bnd,hdv->bhnv", X, P_v)
    Y = np.einsum("bhnv,hdv->bnd", orc.mha_prefill(Q, Kc, Vc, [n, n]), P_o)
    ref = orc.multihead_attention_batched(X, X, orc.causal_mask(b, h, n), P_q, P_k, P_v, P_o)
    assert np.max(np.abs(Y - ref)) <= 1e-12


# ---------------------------------------------------------------- beam search (Section 4.1, Table 2 last column)
def _beam_case(seed, b=3, beam=4, h=2, cap_s=7, cap_t=5, k=3, v=4):
    g = _rng(seed)
    q = g.normal(size=(b, beam, h, k)) * 2
    Ks, Vs = g.normal(size=(b, cap_s, k)), g.normal(size=(b, cap_s, v))
    Kt, Vt = g.normal(size=(b, beam, cap_t, k)), g.normal(size=(b, beam, cap_t, v))
    ls = g.integers(0, cap_s + 1, size=b)
    lt = g.integers(0, cap_t + 1, size=(b, beam))
    return q, Ks, Vs, ls, Kt, Vt, lt


@pytest.mark.parametrize("seed", range(6))
def test_beams_equal_separate_sequences_with_materialised_memories(seed):
    """Every hypothesis as its own sequence whose memory holds a private copy of the shared rows
    followed by its own: the multi-query step over those b*beam sequences (pinned above, and the
    pure-Python enumeration) must give the same outputs."""
    q, Ks, Vs, ls, Kt, Vt, lt = _beam_case(seed)
    b, beam, h, k = q.shape
    cap = Ks.shape[1] + Kt.shape[2]
    K = np.full((b * beam, cap, k), np.nan)
    V = np.full((b * beam, cap, Vs.shape[-1]), np.nan)
    lens = np.zeros(b * beam, dtype=int)
    for i in range(b):
        for e in range(beam):
            r = i * beam + e
            K[r, :ls[i]], V[r, :ls[i]] = Ks[i, :ls[i]], Vs[i, :ls[i]]
            K[r, ls[i]:ls[i] + lt[i, e]], V[r, ls[i]:ls[i] + lt[i, e]] = Kt[i, e, :lt[i, e]], Vt[i, e, :lt[i, e]]
            lens[r] = ls[i] + lt[i, e]
    got = orc.mqa_decode_beams(q, Ks, Vs, ls, Kt, Vt, lt, scale=0.7)
    flat = orc.mqa_decode(q.reshape(b * beam, h, k), K, V, lens, scale=0.7)
    assert np.max(np.abs(got.reshape(flat.shape) - flat)) <= 1e-14
    enum = np.array(bf.mqa_decode_bf(q.reshape(b * beam, h, k).tolist(), np.nan_to_num(K).tolist(),
                                     np.nan_to_num(V).tolist(), lens.tolist(), scale=0.7))
    assert np.max(np.abs(got.reshape(enum.shape) - enum)) <= 1e-12


def test_beams_special_cases():
    q, Ks, Vs, ls, Kt, Vt, lt = _beam_case(11)
    b, beam, h, k = q.shape
    # no own positions: all hypotheses of a source are extra heads over the shared memory
    zero = np.zeros_like(lt)
    ls1 = np.maximum(ls, 1)
    got = orc.mqa_decode_beams(q, Ks, Vs, ls1, Kt, Vt, zero)
    ref = orc.mqa_decode(q.reshape(b, beam * h, k), Ks, Vs, ls1)
    assert np.max(np.abs(got.reshape(ref.shape) - ref)) <= 1e-14
    # no shared positions: b*beam independent sequences
    got = orc.mqa_decode_beams(q, Ks, Vs, np.zeros_like(ls), Kt, Vt, lt)
    ref = orc.mqa_decode(q.reshape(b * beam, h, k), Kt.reshape(b * beam, -1, k), Vt.reshape(b * beam, -1, Vt.shape[-1]),
                         lt.reshape(-1))
    assert np.max(np.abs(got.reshape(ref.shape) - ref)) <= 1e-14
    # attention does not care which part a row sits in: move the last shared row of source 0 to
    # the end of every hypothesis' own part
    ls2, lt2 = ls.copy(), lt.copy()
    ls2[0], lt2[0] = 3, 2
    base = orc.mqa_decode_beams(q, Ks, Vs, ls2, Kt, Vt, lt2)
    Kt3, Vt3, ls3, lt3 = Kt.copy(), Vt.copy(), ls2.copy(), lt2.copy()
    Kt3[0, :, 2], Vt3[0, :, 2] = Ks[0, 2], Vs[0, 2]
    ls3[0], lt3[0] = 2, 3
    moved = orc.mqa_decode_beams(q, Ks, Vs, ls3, Kt3, Vt3, lt3)
    assert np.max(np.abs(base - moved)) <= 1e-14
    # nothing to attend to: zeros
    assert not orc.mqa_decode_beams(q, Ks, Vs, np.zeros_like(ls), Kt, Vt, zero).any()


def test_beam_reorder_semantics():
    g = _rng(5)
    n, cap, k = 8, 6, 3
    K, V = g.normal(size=(n, cap, k)), g.normal(size=(n, cap, 2))
    lens = np.array([0, 1, 6, 3, 2, 5, 4, 6])
    parent = np.array([2, 2, 1, 0, 7, 7, 7, 3])      # slots may be dropped (4, 5, 6) or duplicated
    K2, V2, lens2 = orc.beam_reorder_kv(K, V, lens, parent)
    assert lens2.tolist() == [6, 6, 1, 0, 6, 6, 6, 3]
    for r in range(n):
        for t in range(lens2[r]):
            assert K2[r, t].tolist() == K[parent[r], t].tolist() and V2[r, t].tolist() == V[parent[r], t].tolist()
    # identity permutation keeps every valid row; a step after the reorder sees the parent's memory
    K3, V3, lens3 = orc.beam_reorder_kv(K, V, lens, np.arange(n))
    q = g.normal(size=(n, 2, k))
    assert np.array_equal(orc.mqa_decode(q, K3, V3, lens3), orc.mqa_decode(q, K, V, lens))
    assert np.array_equal(orc.mqa_decode(q, K2, V2, lens2)[4], orc.mqa_decode(q[4:5], K[7:8], V[7:8], lens[7:8])[0])
    # multi-head caches [n, h, cap, k]
    Kh = g.normal(size=(n, 2, cap, k))
    Kh2, _, _ = orc.beam_reorder_kv(Kh, Kh, lens, parent)
    assert np.array_equal(Kh2[0, :, :6], Kh[2, :, :6]) and np.array_equal(Kh2[7, 1, :3], Kh[3, 1, :3])

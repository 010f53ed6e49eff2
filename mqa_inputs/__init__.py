"""Seeded synthetic inputs for the multi-query-attention decode path.

This module is the only code shared by the CPU oracle's tests and the HIP
path's tests / benchmark.  It draws random tensors, packs them in the layouts
the paper uses (Section 2.4 and Section 3 listings: q [b,h,k], multi-query
K [b,m,k] / V [b,m,v], multi-head K [b,h,m,k] / V [b,h,m,v], P_q/P_o
[h,d,k]/[h,d,v], P_k/P_v [d,k]/[d,v]) and converts number formats.  It holds
none of the method's arithmetic: no projection, no logits, no softmax, no
cache append.

Random numbers: numpy ``Generator(Philox(key=[seed, stream]))`` with
``seed = 191102150 + config index`` and one ``stream`` number per tensor (and
per sequence for the large tensors, so they can be produced piecewise).
bfloat16 tensors are carried as ``uint16`` bit patterns; the float32 -> bf16
conversion of *inputs* is done by torch's CPU cast (round-to-nearest-even).

Workload shapes follow the paper's experimental set-up (Section 4.1 and 4.3:
d_model 1024, h 8, d_k = d_v 128, 128 sequences per core, 128 + 128 tokens)
plus a long-context bandwidth probe and a ragged batch; the datasets the paper
used (WMT14, LM1B) are not needed for timing and are not reproduced.
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

SEED_BASE = 191102150

# stream numbers (second Philox key word) for the tensors of a workload
_S_X, _S_M, _S_V, _S_PQ, _S_PK, _S_PV, _S_PO, _S_LENS, _S_PICK, _S_PK_MH, _S_PV_MH = range(11)
_S_PER_SEQ = 1 << 20        # per-sequence streams start here
_S_MH = 1 << 30             # multi-head twins of per-sequence streams


def rng(config_index: int, stream: int = 0) -> np.random.Generator:
    """Counter-based generator for (workload, tensor)."""
    key = np.array([SEED_BASE + int(config_index), int(stream)], dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


# --------------------------------------------------------------------------
# number-format plumbing (inputs only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 array -> uint16 bf16 bit patterns (torch CPU cast, RNE)."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> the float32 values they denote (exact)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(bits).astype(np.float64)


def bits_to_torch_bf16(bits: np.ndarray) -> torch.Tensor:
    """uint16 bit patterns -> torch.bfloat16 CPU tensor sharing the values."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16)


def _normal(g: np.random.Generator, shape, std: float = 1.0) -> np.ndarray:
    a = g.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


# --------------------------------------------------------------------------
# workload table (index = position in the benchmark's config list, 1-based)
# --------------------------------------------------------------------------
CONFIGS = {
    1: dict(name="single_step_fp32", b=1, d=1024, h=8, k=128, v=128, m=128, cache="f32"),
    2: dict(name="incremental_b128", b=128, d=1024, h=8, k=128, v=128, steps=128, cap=128, cache="bf16"),
    3: dict(name="decoder_stack", b=128, d=1024, h=8, k=128, v=128, layers=6, d_ff=4096,
            vocab=32768, prompt=128, gen=128, cap=256, cache="bf16"),
    4: dict(name="long_context_probe", b=64, h=32, k=128, v=128, m=8192, cap=8192, cache="bf16"),
    5: dict(name="ragged_large_batch", b=512, h=64, k=128, v=128, cap=4096, cache="bf16",
            outlier_fraction=0.01, outlier_boost=30.0),
}


def config1(d=1024, h=8, k=128, v=128, m=128):
    """One query against a memory of m vectors, everything float32.

    Every entry is N(0,1)/sqrt(d).  Returns x [1,d], M [1,m,d], P_q [h,d,k],
    P_k [d,k], P_v [d,v], P_o [h,d,v] and the multi-head twins P_k_mh [h,d,k],
    P_v_mh [h,d,v].
    """
    s = 1.0 / math.sqrt(d)
    return dict(
        x=_normal(rng(1, _S_X), (1, d), s),
        M=_normal(rng(1, _S_M), (1, m, d), s),
        P_q=_normal(rng(1, _S_PQ), (h, d, k), s),
        P_k=_normal(rng(1, _S_PK), (d, k), s),
        P_v=_normal(rng(1, _S_PV), (d, v), s),
        P_o=_normal(rng(1, _S_PO), (h, d, v), s),
        P_k_mh=_normal(rng(1, _S_PK_MH), (h, d, k), s),
        P_v_mh=_normal(rng(1, _S_PV_MH), (h, d, v), s),
    )


def config2(b=128, d=1024, h=8, k=128, v=128, steps=128):
    """Incremental decoding of one layer: X [b,steps,d] ~ N(0,1), one row per
    sequence per step; projections ~ N(0, 1/d) (std 1/sqrt(d)), float32."""
    s = 1.0 / math.sqrt(d)
    return dict(
        X=_normal(rng(2, _S_X), (b, steps, d)),
        P_q=_normal(rng(2, _S_PQ), (h, d, k), s),
        P_k=_normal(rng(2, _S_PK), (d, k), s),
        P_v=_normal(rng(2, _S_PV), (d, v), s),
        P_o=_normal(rng(2, _S_PO), (h, d, v), s),
        P_k_mh=_normal(rng(2, _S_PK_MH), (h, d, k), s),
        P_v_mh=_normal(rng(2, _S_PV_MH), (h, d, v), s),
    )


def config3_weights(layers=6, d=1024, h=8, k=128, v=128, d_ff=4096, vocab=32768, max_pos=256,
                    multi_head=False):
    """Random decoder-only stack: embeddings N(0,1), matrices N(0, 1/fan_in)."""
    cfg = 3
    w = dict(
        E=_normal(rng(cfg, 100), (vocab, d)),
        pos=_normal(rng(cfg, 101), (max_pos, d)),
        layers=[],
    )
    for l in range(layers):
        base = 200 + 20 * l + (10 if multi_head else 0)
        kv_shape_k = (h, d, k) if multi_head else (d, k)
        kv_shape_v = (h, d, v) if multi_head else (d, v)
        w["layers"].append(dict(
            P_q=_normal(rng(cfg, base + 0), (h, d, k), 1.0 / math.sqrt(d)),
            P_k=_normal(rng(cfg, base + 1), kv_shape_k, 1.0 / math.sqrt(d)),
            P_v=_normal(rng(cfg, base + 2), kv_shape_v, 1.0 / math.sqrt(d)),
            P_o=_normal(rng(cfg, base + 3), (h, d, v), 1.0 / math.sqrt(h * v)),
            W1=_normal(rng(cfg, base + 4), (d, d_ff), 1.0 / math.sqrt(d)),
            W2=_normal(rng(cfg, base + 5), (d_ff, d), 1.0 / math.sqrt(d_ff)),
        ))
    return w


def config3_prompts(b=128, prompt=128, vocab=32768):
    return rng(3, _S_X).integers(0, vocab, size=(b, prompt), dtype=np.int64)


def config4_q(b=64, h=32, k=128):
    """q [b,h,k] float32 ~ N(0,1)/sqrt(k)."""
    return _normal(rng(4, _S_X), (b, h, k), 1.0 / math.sqrt(k))


def _kv_block_bits(cfg, stream, shape):
    return f32_to_bf16_bits(_normal(rng(cfg, stream), shape))


def config4_kv(b=64, m=8192, k=128, v=128, threads=8):
    """Multi-query cache: K [b,m,k], V [b,m,v] bf16 bits ~ N(0,1), drawn per
    sequence so that they can be produced piecewise and in parallel."""
    K = np.empty((b, m, k), dtype=np.uint16)
    V = np.empty((b, m, v), dtype=np.uint16)

    def fill(i):
        K[i] = _kv_block_bits(4, _S_PER_SEQ + 2 * i, (m, k))
        V[i] = _kv_block_bits(4, _S_PER_SEQ + 2 * i + 1, (m, v))

    with ThreadPoolExecutor(max_workers=threads) as ex:
        list(ex.map(fill, range(b)))
    return K, V


def config4_kv_mh_block(i, j, m=8192, k=128, v=128):
    """Multi-head twin: K[i,j] [m,k] and V[i,j] [m,v] bf16 bits for sequence i, head j."""
    s = _S_MH + 2 * (i * 4096 + j)
    return _kv_block_bits(4, s, (m, k)), _kv_block_bits(4, s + 1, (m, v))


def config5(b=512, h=64, k=128, v=128, cap=4096, outlier_fraction=0.01, outlier_boost=30.0,
            poison=True):
    """Ragged batch.  lens ~ U{1..cap}; q ~ N(0,1)/sqrt(k); K,V ~ N(0,1) in the
    valid rows.  For `outlier_fraction` of the valid (sequence, position) pairs
    one head is chosen and K[i,j,:] gets `outlier_boost` * q[i,head,:]/|q[i,head,:]|^2
    added before the bf16 rounding, which lifts that head's dot product with the
    row by `outlier_boost`.  Rows at and beyond lens[i] hold NaN when `poison`.
    Returns q, K_bits, V_bits, lens (int32).
    """
    lens = rng(5, _S_LENS).integers(1, cap + 1, size=(b,), dtype=np.int64).astype(np.int32)
    q = _normal(rng(5, _S_X), (b, h, k), 1.0 / math.sqrt(k))
    nan_bits = np.uint16(0x7FC0)
    K = np.full((b, cap, k), nan_bits if poison else 0, dtype=np.uint16)
    V = np.full((b, cap, v), nan_bits if poison else 0, dtype=np.uint16)
    for i in range(b):
        L = int(lens[i])
        Ki = _normal(rng(5, _S_PER_SEQ + 3 * i), (L, k))
        Vi = _normal(rng(5, _S_PER_SEQ + 3 * i + 1), (L, v))
        g = rng(5, _S_PER_SEQ + 3 * i + 2)
        pick = np.nonzero(g.random(L) < outlier_fraction)[0]
        heads = g.integers(0, h, size=pick.shape[0])
        for j, hh in zip(pick, heads):
            qv = q[i, hh].astype(np.float64)
            Ki[j] += (outlier_boost * qv / float(qv @ qv)).astype(np.float32)
        K[i, :L] = f32_to_bf16_bits(Ki)
        V[i, :L] = f32_to_bf16_bits(Vi)
    return q, K, V, lens


def random_case(seed, b, h, cap, k, v, cache="bf16", lens="full", multi_head=False,
                q_std=None, kv_std=1.0, poison=True):
    """A free-form seeded decode case for parity tests.

    Returns dict(q [b,h,k] f32, K, V (uint16 bits for cache 'bf16', float32 for
    'f32'; [b,cap,k] or [b,h,cap,k]), lens int32 [b]).  `lens` is 'full',
    'ragged' (uniform in 1..cap), 'with_zero' (ragged with some zeros) or an
    explicit sequence.  Rows at and beyond lens[i] are NaN when `poison`.
    """
    cfg = 1000 + int(seed)
    if q_std is None:
        q_std = 1.0 / math.sqrt(k)
    q = _normal(rng(cfg, _S_X), (b, h, k), q_std)
    kshape = (b, h, cap, k) if multi_head else (b, cap, k)
    vshape = (b, h, cap, v) if multi_head else (b, cap, v)
    K = _normal(rng(cfg, _S_M), kshape, kv_std)
    V = _normal(rng(cfg, _S_V), vshape, kv_std)
    if isinstance(lens, str):
        if lens == "full":
            L = np.full((b,), cap, dtype=np.int32)
        elif lens == "ragged":
            L = rng(cfg, _S_LENS).integers(1, cap + 1, size=(b,)).astype(np.int32)
        elif lens == "with_zero":
            L = rng(cfg, _S_LENS).integers(0, cap + 1, size=(b,)).astype(np.int32)
            L[:: max(1, b // 3)] = 0
        else:
            raise ValueError(lens)
    else:
        L = np.asarray(lens, dtype=np.int32).reshape(b)
    if poison:
        for i in range(b):
            K[i, ..., int(L[i]):, :] = np.nan
            V[i, ..., int(L[i]):, :] = np.nan
    if cache == "bf16":
        K = f32_to_bf16_bits(K)
        V = f32_to_bf16_bits(V)
    elif cache != "f32":
        raise ValueError(cache)
    return dict(q=q, K=K, V=V, lens=L)


def beam_case(seed, b, beam, h, cap_src, cap_own, k, v, cache="bf16", lens_src="ragged", lens_own="ragged",
              poison=True):
    """A seeded beam-search step: `beam` hypotheses per source share the source's rows and own the
    rows they produced (the shape of the paper's beam-4 translation decoding: a source / prompt of
    up to cap_src positions, up to cap_own generated ones).

    Returns dict(q [b,beam,h,k] f32, K_src [b,cap_src,k], V_src, lens_src [b] int32,
    K_own [b,beam,cap_own,k], V_own, lens_own [b*beam] int32); caches as in random_case.
    `lens_*`: 'full', 'ragged' (uniform in 1..cap, own part uniform in 0..cap) or explicit."""
    cfg = 2000 + int(seed)
    q = _normal(rng(cfg, _S_X), (b, beam, h, k), 1.0 / math.sqrt(k))
    K_src = _normal(rng(cfg, _S_M), (b, cap_src, k))
    V_src = _normal(rng(cfg, _S_V), (b, cap_src, v))
    K_own = _normal(rng(cfg, _S_PK), (b, beam, cap_own, k))
    V_own = _normal(rng(cfg, _S_PV), (b, beam, cap_own, v))

    def lens_of(spec, n, cap, lowest, stream):
        if isinstance(spec, str):
            if spec == "full":
                return np.full((n,), cap, dtype=np.int32)
            if spec == "ragged":
                return rng(cfg, stream).integers(lowest, cap + 1, size=(n,)).astype(np.int32)
            raise ValueError(spec)
        return np.asarray(spec, dtype=np.int32).reshape(n)

    ls = lens_of(lens_src, b, cap_src, 1, _S_LENS)
    lo = lens_of(lens_own, b * beam, cap_own, 0, _S_PICK)
    if poison:
        for i in range(b):
            K_src[i, int(ls[i]):] = np.nan
            V_src[i, int(ls[i]):] = np.nan
            for e in range(beam):
                K_own[i, e, int(lo[i * beam + e]):] = np.nan
                V_own[i, e, int(lo[i * beam + e]):] = np.nan
    if cache == "bf16":
        K_src, V_src, K_own, V_own = (f32_to_bf16_bits(a) for a in (K_src, V_src, K_own, V_own))
    elif cache != "f32":
        raise ValueError(cache)
    return dict(q=q, K_src=K_src, V_src=V_src, lens_src=ls, K_own=K_own, V_own=V_own, lens_own=lo)


def cache_as_f64(a: np.ndarray) -> np.ndarray:
    """Cache tensor (uint16 bf16 bits or float32) -> float64 with the same values."""
    if a.dtype == np.uint16:
        return bf16_bits_to_f64(a)
    return a.astype(np.float64)

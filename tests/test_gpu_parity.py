"""Parity of the HIP path (through the C ABI) with the float64 oracle, element
by element on the same seeded inputs.

Tolerances (the build's stated bar): float32 cache: max |g - r| <= 1e-5;
bf16 cache with float32 accumulation: max |g - r| <= 2e-2 and
max |g - r| / max |r| <= 1e-2, per tensor.  The cache values are rounded to
bf16 on the host and the same rounded values go to both sides, so the
comparison measures the GPU's arithmetic, not the quantisation.
"""
import numpy as np
import pytest
import torch

import mqa_inputs as mi
from oracle import mqa_oracle as orc

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def m():
    import paper_1911_02150_amd as lib
    lib.load_library()
    return lib


def to_dev_cache(a):
    if a.dtype == np.uint16:
        return mi.bits_to_torch_bf16(a).to(DEV)
    return torch.from_numpy(a).to(DEV)


def check(got, ref, cache, what=""):
    got = got.detach().cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = float(np.max(np.abs(got - ref))) if ref.size else 0.0
    scale = float(np.max(np.abs(ref))) if ref.size else 1.0
    if cache == "f32":
        assert err <= 1e-5, f"{what}: max abs err {err:.3e} > 1e-5"
    else:
        assert err <= 2e-2, f"{what}: max abs err {err:.3e} > 2e-2"
        assert err <= 1e-2 * max(scale, 1e-30), f"{what}: rel err {err / scale:.3e} > 1e-2"
    return err


def run_case(m, c, multi_head, scale=1.0, tuning=None):
    q = torch.from_numpy(c["q"]).to(DEV)
    K, V = to_dev_cache(c["K"]), to_dev_cache(c["V"])
    lens = torch.from_numpy(c["lens"]).to(DEV)
    fn = m.mha_decode_step if multi_head else m.mqa_decode_step
    o = fn(q, K, V, lens, scale=scale, tuning=tuning)
    torch.cuda.synchronize()
    ofn = orc.mha_decode if multi_head else orc.mqa_decode
    ref = ofn(c["q"], mi.cache_as_f64(c["K"]), mi.cache_as_f64(c["V"]), c["lens"], scale)
    return o, ref


# ----------------------------------------------------------------- MFMA kernel, bf16, k = v = 128
MFMA_CASES = [
    # (seed, b, h, cap, lens, splits)
    (1, 3, 8, 128, "full", 0),
    (2, 2, 32, 300, "ragged", 0),          # several tiles + ragged tail
    (3, 5, 1, 97, "ragged", 0),
    (4, 2, 20, 1000, "ragged", 3),         # h not a multiple of 16, forced split
    (5, 3, 64, 515, "with_zero", 2),       # four head blocks, empty sequences
    (6, 1, 72, 260, "full", 1),            # more than 64 heads: two head groups
    (7, 4, 16, 2048, "ragged", 7),
    (8, 2, 32, 4100, "full", 0),           # heuristics choose the split
    (9, 6, 8, 33, [1, 2, 31, 32, 33, 17], 0),
    (10, 2, 40, 64, "with_zero", 2),
    (11, 1, 8, 4096, "ragged", 64),        # the maximum number of ranges: the merge folds 8 batches of slots
    (12, 2, 32, 2500, "ragged", 20),
    (13, 1, 32, 40000, "ragged", 0),       # one long sequence: the heuristics spread it over up to 256 ranges
    (14, 3, 8, 3000, "with_zero", 24),     # many slots per row with empty sequences and unwritten ranges
    (15, 4, 8, 1, "full", 0),              # a cache of one position: the output is that V row
    (16, 2, 8, 7, [7, 3], 0),
]


@pytest.mark.parametrize("seed,b,h,cap,lens,splits", MFMA_CASES)
def test_mqa_decode_bf16(m, seed, b, h, cap, lens, splits):
    c = mi.random_case(seed, b, h, cap, 128, 128, cache="bf16", lens=lens)
    tuning = dict(splits=splits, kernel=2) if splits else dict(kernel=2)
    o, ref = run_case(m, c, False, tuning=tuning)
    err = check(o, ref, "bf16", f"mqa bf16 seed {seed}")
    print(f"mqa bf16 case {seed}: max abs err {err:.2e}")


@pytest.mark.parametrize("flags", [1, 2, 3])
def test_mqa_decode_bf16_reduced_terms(m, flags):
    """The faster single-term variants still meet the bf16 tolerance on the bandwidth-probe distribution."""
    c = mi.random_case(40 + flags, 2, 32, 1024, 128, 128, cache="bf16", lens="ragged")
    o, ref = run_case(m, c, False, tuning=dict(kernel=2, flags=flags, splits=2))
    check(o, ref, "bf16", f"flags {flags}")


def test_mqa_decode_bf16_large_logits_and_scale(m):
    # un-scaled queries (logits of std ~ sqrt(128)) and an explicit scale factor
    c = mi.random_case(11, 3, 8, 200, 128, 128, cache="bf16", lens="ragged", q_std=1.0)
    o, ref = run_case(m, c, False)
    check(o, ref, "bf16", "unit-variance q")
    o, ref = run_case(m, c, False, scale=0.25)
    check(o, ref, "bf16", "scale 0.25")


@pytest.mark.parametrize("seed,b,h,cap,lens,splits", [
    (21, 2, 8, 128, "full", 0), (22, 2, 5, 300, "ragged", 2), (23, 3, 3, 70, "with_zero", 0),
])
def test_mha_decode_bf16(m, seed, b, h, cap, lens, splits):
    c = mi.random_case(seed, b, h, cap, 128, 128, cache="bf16", lens=lens, multi_head=True)
    o, ref = run_case(m, c, True, tuning=dict(splits=splits) if splits else None)
    check(o, ref, "bf16", f"mha bf16 seed {seed}")


def test_mqa_equals_mha_on_shared_kv_gpu(m):
    """Section 3: multi-query is multi-head with every head reading the same K/V."""
    c = mi.random_case(24, 2, 6, 150, 128, 128, cache="bf16", lens="ragged")
    q = torch.from_numpy(c["q"]).to(DEV)
    K, V = to_dev_cache(c["K"]), to_dev_cache(c["V"])
    lens = torch.from_numpy(c["lens"]).to(DEV)
    o1 = m.mqa_decode_step(q, K, V, lens)
    Kh = K[:, None].expand(2, 6, 150, 128).contiguous()
    Vh = V[:, None].expand(2, 6, 150, 128).contiguous()
    o2 = m.mha_decode_step(q, Kh, Vh, lens)
    assert float((o1 - o2).abs().max()) <= 1e-5


# ----------------------------------------------------------------- generic kernel
GENERIC_CASES = [
    # (seed, b, h, cap, k, v, cache, lens, splits, multi_head)
    (31, 1, 8, 128, 128, 128, "f32", "full", 0, False),
    (32, 3, 5, 200, 64, 32, "f32", "ragged", 0, False),
    (33, 2, 11, 700, 40, 72, "f32", "with_zero", 3, False),
    (34, 2, 9, 130, 256, 256, "f32", "ragged", 0, False),
    (35, 2, 4, 90, 64, 64, "bf16", "ragged", 0, False),
    (36, 2, 3, 300, 128, 128, "f32", "ragged", 2, True),
    (37, 2, 3, 65, 16, 8, "bf16", "full", 0, True),
]


@pytest.mark.parametrize("seed,b,h,cap,k,v,cache,lens,splits,mh", GENERIC_CASES)
def test_decode_generic(m, seed, b, h, cap, k, v, cache, lens, splits, mh):
    c = mi.random_case(seed, b, h, cap, k, v, cache=cache, lens=lens, multi_head=mh)
    o, ref = run_case(m, c, mh, tuning=dict(splits=splits, kernel=1))
    check(o, ref, cache, f"generic seed {seed}")


def test_generic_matches_mfma_kernel(m):
    c = mi.random_case(38, 2, 8, 400, 128, 128, cache="bf16", lens="ragged")
    o1, ref = run_case(m, c, False, tuning=dict(kernel=1))
    o2, _ = run_case(m, c, False, tuning=dict(kernel=2))
    check(o1, ref, "bf16"), check(o2, ref, "bf16")


def test_two_phase_calls_equal_one_call(m):
    c = mi.random_case(39, 2, 32, 2048, 128, 128, cache="bf16", lens="ragged")
    q = torch.from_numpy(c["q"]).to(DEV)
    K, V = to_dev_cache(c["K"]), to_dev_cache(c["V"])
    lens = torch.from_numpy(c["lens"]).to(DEV)
    tn = dict(splits=4)
    o1 = m.mqa_decode_step(q, K, V, lens, tuning=tn)
    ws = torch.empty(m.mqa_decode_workspace_bytes(2, 32, 2048, 128), dtype=torch.uint8, device=DEV)
    o2 = torch.full_like(o1, float("nan"))
    m.mqa_decode_partials(q, K, V, lens, o2, ws, tuning=tn)
    m.mqa_decode_combine(lens, o2, 2048, 128, m.MQA_BF16, ws, tuning=tn)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2)


# ----------------------------------------------------------------- append
@pytest.mark.parametrize("cache,mh", [("bf16", False), ("bf16", True), ("f32", False), ("f32", True)])
def test_append_bit_exact(m, cache, mh):
    g = mi.rng(2000, 1 + int(mh))
    b, h, cap, k, v = 5, 3, 6, 16, 24
    hk = h if mh else 1
    shape_k = (b, h, cap, k) if mh else (b, cap, k)
    shape_v = (b, h, cap, v) if mh else (b, cap, v)
    lens0 = np.array([0, 3, 6, 5, 1], dtype=np.int32)           # sequence 2 is full
    k_new = g.standard_normal((b, hk, k), dtype=np.float32) * np.float32(3)
    v_new = g.standard_normal((b, hk, v), dtype=np.float32)
    k_new[0, 0, :4] = [1.00390625, 1.01171875, -0.0, 3e-41]      # ties to even, signed zero, subnormal
    tdt = torch.bfloat16 if cache == "bf16" else torch.float32
    K = torch.zeros(shape_k, dtype=tdt, device=DEV)
    V = torch.zeros(shape_v, dtype=tdt, device=DEV)
    lens = torch.from_numpy(lens0.copy()).to(DEV)
    kn = torch.from_numpy(k_new if mh else k_new[:, 0]).contiguous().to(DEV)
    vn = torch.from_numpy(v_new if mh else v_new[:, 0]).contiguous().to(DEV)
    m.mqa_append_kv(K, V, kn, vn, lens)
    torch.cuda.synchronize()
    Kr, Vr = np.zeros(shape_k), np.zeros(shape_v)
    lr = lens0.astype(np.int64)
    orc.append_kv(Kr, Vr, k_new if mh else k_new[:, 0], v_new if mh else v_new[:, 0], lr, cache)
    assert np.array_equal(lens.cpu().numpy(), lr)
    assert np.array_equal(K.double().cpu().numpy(), Kr)
    assert np.array_equal(V.double().cpu().numpy(), Vr)
    assert np.array_equal(np.signbit(K.double().cpu().numpy()), np.signbit(Kr))


# ----------------------------------------------------------------- projections
@pytest.mark.parametrize("rows,d,h,kv", [(1, 1024, 8, 128), (128, 1024, 8, 128), (37, 72, 3, 40), (5, 8, 1, 8),
                                         (3000, 1032, 8, 136),      # LDS-tiled kernel, 128x128 tiles, ragged edges
                                         (1000, 1032, 8, 136),      # the same with 64x64 tiles
                                         (130, 264, 64, 128),       # few rows, very wide output
                                         (100, 2056, 16, 128),      # long contraction, ragged rows and tail: 16x64 tiles
                                         # the other tile shapes of the split-contraction kernel (RB x CB blocks of 16x16):
                                         (40, 2560, 20, 128),       # 32x32 tiles, both weight layouts
                                         (40, 264, 1, 1296),        # 32x16 tiles, N contiguous (N = 81 x 16)
                                         (40, 1296, 2, 64),         # 32x16 tiles, C contiguous
                                         (100, 2568, 2, 64),        # 32x64 tiles, C contiguous, ragged last column tile
                                         (128, 1024, 1, 4104)])     # 32x64 tiles, N contiguous, 8 columns in the last tile; contraction tail
def test_projections(m, rows, d, h, kv):
    g = mi.rng(3000, rows + d)
    x = g.standard_normal((rows, d), dtype=np.float32)
    P_q = g.standard_normal((h, d, kv), dtype=np.float32) / np.float32(np.sqrt(d))
    P_k = g.standard_normal((d, kv), dtype=np.float32) / np.float32(np.sqrt(d))
    o = g.standard_normal((rows, h, kv), dtype=np.float32)
    P_o = g.standard_normal((h, d, kv), dtype=np.float32) / np.float32(np.sqrt(h * kv))
    dx, dPq, dPk, do, dPo = (torch.from_numpy(a).to(DEV) for a in (x, P_q, P_k, o, P_o))
    got = m.mqa_project_qkvo(m.MQA_PROJ_Q, dx, dPq)
    assert np.max(np.abs(got.cpu().numpy() - orc.project_q(x, P_q))) <= 1e-5
    # the new K / V rows are accumulated in float64 and rounded once: the float32 result is the oracle's
    # float64 value rounded to float32 (two float64 sums in different orders can straddle a float32
    # rounding boundary about once in 1e7 elements: at most a stray last-place difference is allowed)
    for mode, P, ref in ((m.MQA_PROJ_KV_MH, dPq, orc.project_kv_mh(x, P_q)), (m.MQA_PROJ_KV, dPk, orc.project_kv(x, P_k))):
        got = m.mqa_project_qkvo(mode, dx, P).cpu().numpy()
        want = ref.astype(np.float32)
        differ = got != want
        assert differ.sum() <= 1 and np.all(np.abs(got - want) <= np.spacing(np.abs(want))), f"mode {mode}: {differ.sum()} differ"
    got = m.mqa_project_qkvo(m.MQA_PROJ_LINEAR, dx, dPk)
    assert np.max(np.abs(got.cpu().numpy() - orc.project_kv(x, P_k))) <= 1e-5
    got = m.mqa_project_qkvo(m.MQA_PROJ_O, do, dPo)
    assert np.max(np.abs(got.cpu().numpy() - orc.project_o(o, P_o))) <= 1e-5
    # epilogues: relu on the way out, and accumulation into what the output holds (a residual stream)
    got = m.mqa_project_qkvo_ex(m.MQA_PROJ_LINEAR, dx, dPk, epilogue=m.MQA_EPI_RELU)
    assert np.max(np.abs(got.cpu().numpy() - np.maximum(orc.project_kv(x, P_k), 0))) <= 1e-5
    assert float(got.min()) >= 0.0
    res = g.standard_normal((rows, d), dtype=np.float32)
    acc = torch.from_numpy(res.copy()).to(DEV)
    m.mqa_project_qkvo_ex(m.MQA_PROJ_O, do, dPo, out=acc, epilogue=m.MQA_EPI_ADD)
    assert np.max(np.abs(acc.cpu().numpy() - (res + orc.project_o(o, P_o)))) <= 1e-5
    acc = torch.from_numpy(res[:, :kv].copy()).to(DEV) if kv <= d else None
    if acc is not None:
        for mode in (m.MQA_PROJ_LINEAR, m.MQA_PROJ_KV):
            acc = torch.from_numpy(res[:, :kv].copy()).to(DEV)
            m.mqa_project_qkvo_ex(mode, dx, dPk, out=acc, epilogue=m.MQA_EPI_ADD)
            assert np.max(np.abs(acc.cpu().numpy() - (res[:, :kv] + orc.project_kv(x, P_k)))) <= 1e-5


# ----------------------------------------------------------------- workload 1: one float32 step against a memory
def test_config1_single_step_fp32(m):
    c = mi.config1()
    h, d, k = c["P_q"].shape
    mem = c["M"].shape[1]
    x = torch.from_numpy(c["x"]).to(DEV)
    M = torch.from_numpy(c["M"][0]).to(DEV)
    lens = torch.full((1,), mem, dtype=torch.int32, device=DEV)
    # multi-query
    q = m.mqa_project_qkvo(m.MQA_PROJ_Q, x, torch.from_numpy(c["P_q"]).to(DEV))
    K = m.mqa_project_qkvo(m.MQA_PROJ_KV, M, torch.from_numpy(c["P_k"]).to(DEV))[None]
    V = m.mqa_project_qkvo(m.MQA_PROJ_KV, M, torch.from_numpy(c["P_v"]).to(DEV))[None]
    o = m.mqa_decode_step(q, K.contiguous(), V.contiguous(), lens)
    y = m.mqa_project_qkvo(m.MQA_PROJ_O, o, torch.from_numpy(c["P_o"]).to(DEV))
    ref = orc.multiquery_attention(c["x"][0], c["M"][0], c["P_q"], c["P_k"], c["P_v"], c["P_o"])
    err = check(y[0], ref, "f32", "config 1 multi-query y")
    print(f"config 1 multi-query: max abs err {err:.2e}, max |y| {np.abs(ref).max():.2e}")
    # multi-head twin
    Kh = m.mqa_project_qkvo(m.MQA_PROJ_KV_MH, M, torch.from_numpy(c["P_k_mh"]).to(DEV))     # [m,h,k]
    Vh = m.mqa_project_qkvo(m.MQA_PROJ_KV_MH, M, torch.from_numpy(c["P_v_mh"]).to(DEV))
    Kh = Kh.permute(1, 0, 2).contiguous()[None]
    Vh = Vh.permute(1, 0, 2).contiguous()[None]
    o = m.mha_decode_step(q, Kh, Vh, lens)
    y = m.mqa_project_qkvo(m.MQA_PROJ_O, o, torch.from_numpy(c["P_o"]).to(DEV))
    ref = orc.multihead_attention(c["x"][0], c["M"][0], c["P_q"], c["P_k_mh"], c["P_v_mh"], c["P_o"])
    check(y[0], ref, "f32", "config 1 multi-head y")


# ----------------------------------------------------------------- workload 2: incremental decoding, every step
def _row_view(cache, t, multi_head):
    return cache[:, :, t] if multi_head else cache[:, t]


def _check_appended_row(got_row, ref_row, exact_row, what):
    """The row a step appends is the projection (both sides: a float64 sum of exact products)
    rounded to float32 and then to bf16, so the two caches are expected to agree bit for bit.
    Returns how many elements differ; a differing element must still be a valid rounding (as
    close to the oracle's unrounded float64 value as the oracle's own rounding, within 1e-6)."""
    got = got_row.double().cpu().numpy()
    differs = got != ref_row
    assert np.all(np.abs(got - exact_row) <= np.abs(ref_row - exact_row) + 1e-6), f"{what}: invalid rounding"
    return int(differs.sum())


@pytest.mark.parametrize("multi_head", [False, True])
def test_config2_incremental(m, multi_head):
    """128 sequences decoded for 128 steps (projections -> append -> attention
    -> output projection), free running: no value ever flows from one side to the
    other.  Every step: the appended bf16 rows equal the oracle's rows bit for bit,
    and o and y are compared with the stated tolerance.  The stacked y equal one
    causally masked parallel call of the oracle (Section 2.3 / Section 3 batched
    listings)."""
    b, steps = 128, 128
    c = mi.config2(b=b, steps=steps)
    h, d, k = c["P_q"].shape
    v = c["P_o"].shape[2]
    Pk_np, Pv_np = (c["P_k_mh"], c["P_v_mh"]) if multi_head else (c["P_k"], c["P_v"])
    P_q, P_k, P_v, P_o = (torch.from_numpy(a).to(DEV) for a in (c["P_q"], Pk_np, Pv_np, c["P_o"]))
    kshape = (b, h, steps, k) if multi_head else (b, steps, k)
    vshape = (b, h, steps, v) if multi_head else (b, steps, v)
    nan = float("nan")
    K = torch.full(kshape, nan, dtype=torch.bfloat16, device=DEV)
    V = torch.full(vshape, nan, dtype=torch.bfloat16, device=DEV)
    lens = torch.zeros(b, dtype=torch.int32, device=DEV)
    Kr, Vr = np.full(kshape, np.nan), np.full(vshape, np.nan)
    lr = np.zeros(b, dtype=np.int64)
    X = torch.from_numpy(c["X"]).to(DEV)
    kv_mode = m.MQA_PROJ_KV_MH if multi_head else m.MQA_PROJ_KV
    okv = orc.project_kv_mh if multi_head else orc.project_kv
    step_fn = orc.mha_incremental_step if multi_head else orc.mqa_incremental_step
    dec = m.mha_decode_step if multi_head else m.mqa_decode_step
    ys, worst_o, worst_y, flips = [], 0.0, 0.0, 0
    for t in range(steps):
        x = X[:, t].contiguous()
        q = m.mqa_project_qkvo(m.MQA_PROJ_Q, x, P_q)
        kn = m.mqa_project_qkvo(kv_mode, x, P_k)
        vn = m.mqa_project_qkvo(kv_mode, x, P_v)
        m.mqa_append_kv(K, V, kn, vn, lens)
        y_ref, o_ref, _ = step_fn(c["X"][:, t], Kr, Vr, lr, c["P_q"], Pk_np, Pv_np, c["P_o"], cache="bf16")
        flips += _check_appended_row(_row_view(K, t, multi_head), _row_view(Kr, t, multi_head),
                                     okv(c["X"][:, t], Pk_np), f"step {t} K row")
        flips += _check_appended_row(_row_view(V, t, multi_head), _row_view(Vr, t, multi_head),
                                     okv(c["X"][:, t], Pv_np), f"step {t} V row")
        o = dec(q, K, V, lens)
        y = m.mqa_project_qkvo(m.MQA_PROJ_O, o, P_o)
        worst_o = max(worst_o, check(o, o_ref, "bf16", f"step {t} o"))
        worst_y = max(worst_y, check(y, y_ref, "bf16", f"step {t} y"))
        ys.append(y.cpu().numpy())
    assert np.array_equal(lens.cpu().numpy(), np.full(b, steps))
    assert flips == 0, f"{flips} cached elements differ from the oracle's cache"
    assert np.array_equal(K.double().cpu().numpy(), Kr) and np.array_equal(V.double().cpu().numpy(), Vr)
    # stacked incremental outputs == one causally masked parallel call (first 8 sequences)
    nb = 8
    mask = orc.causal_mask(nb, h, steps)
    fn = orc.multihead_attention_batched if multi_head else orc.multiquery_attention_batched
    Y = fn(c["X"][:nb], c["X"][:nb], mask, c["P_q"], Pk_np, Pv_np, c["P_o"], kv_round=orc.round_to_bf16)
    got = np.stack(ys, axis=1)[:nb].astype(np.float64)
    err = np.max(np.abs(got - Y))
    assert err <= 2e-2 and err <= 1e-2 * np.max(np.abs(Y))
    print(f"config 2 {'mha' if multi_head else 'mqa'}: worst o err {worst_o:.2e}, worst y err {worst_y:.2e}, "
          f"vs parallel {err:.2e}, cached elements differing from the oracle's {flips}")


@pytest.mark.parametrize("multi_head", [False, True])
def test_config2_free_running_fused(m, multi_head):
    """The same loop through the fused launch (q, new K/V rows and the append in one call, the
    lengths alternating between two arrays), free running for all 128 steps: the caches equal
    the oracle's bit for bit and o meets the stated tolerance with no allowance."""
    b, steps = 128, 128
    c = mi.config2(b=b, steps=steps)
    h, d, k = c["P_q"].shape
    v = c["P_o"].shape[2]
    Pk_np, Pv_np = (c["P_k_mh"], c["P_v_mh"]) if multi_head else (c["P_k"], c["P_v"])
    P_q, P_k, P_v = (torch.from_numpy(a).to(DEV) for a in (c["P_q"], Pk_np, Pv_np))
    kshape = (b, h, steps, k) if multi_head else (b, steps, k)
    K = torch.zeros(kshape, dtype=torch.bfloat16, device=DEV)
    V = torch.zeros(kshape[:-1] + (v,), dtype=torch.bfloat16, device=DEV)
    lens, lens_next = torch.zeros(b, dtype=torch.int32, device=DEV), torch.zeros(b, dtype=torch.int32, device=DEV)
    Kr, Vr = np.zeros(kshape), np.zeros(kshape[:-1] + (v,))
    lr = np.zeros(b, dtype=np.int64)
    X = torch.from_numpy(c["X"]).to(DEV)
    step_fn = orc.mha_incremental_step if multi_head else orc.mqa_incremental_step
    dec = m.mha_decode_step if multi_head else m.mqa_decode_step
    worst = 0.0
    for t in range(steps):
        q = m.mqa_project_append_qkv(X[:, t].contiguous(), P_q, P_k, P_v, K, V, lens, lens_next)
        lens, lens_next = lens_next, lens
        o = dec(q, K, V, lens)
        _, o_ref, _ = step_fn(c["X"][:, t], Kr, Vr, lr, c["P_q"], Pk_np, Pv_np, c["P_o"], cache="bf16")
        worst = max(worst, check(o, o_ref, "bf16", f"free-running step {t} o"))
    assert np.array_equal(lens.cpu().numpy(), lr)
    assert np.array_equal(K.double().cpu().numpy(), Kr) and np.array_equal(V.double().cpu().numpy(), Vr)
    print(f"config 2 free running, fused launch, {'mha' if multi_head else 'mqa'}: worst o err {worst:.2e}")


# ----------------------------------------------------------------- robustness of the boundary
def test_lengths_outside_capacity_are_clamped(m):
    """lens values outside [0, cap] are clamped by the kernels (the host cannot see them)."""
    c = mi.random_case(50, 4, 8, 160, 128, 128, cache="bf16", lens="full", poison=False)
    q = torch.from_numpy(c["q"]).to(DEV)
    K, V = to_dev_cache(c["K"]), to_dev_cache(c["V"])
    lens = torch.tensor([160, 1000, -5, 77], dtype=torch.int32, device=DEV)
    for tuning in (dict(kernel=2), dict(kernel=2, splits=3), dict(kernel=1), dict(kernel=1, splits=2)):
        o = m.mqa_decode_step(q, K, V, lens, tuning=tuning)
        ref = orc.mqa_decode(c["q"], mi.cache_as_f64(c["K"]), mi.cache_as_f64(c["V"]), [160, 160, 0, 77])
        check(o, ref, "bf16", f"clamped lens {tuning}")
        assert float(o[2].abs().max()) == 0.0


def test_decode_step_in_a_hip_graph(m):
    """The library neither allocates nor synchronises, so a whole step (append + attention)
    can be captured in a HIP graph; every replay must equal the eager result."""
    b, h, cap = 8, 32, 2048
    c = mi.random_case(51, b, h, cap, 128, 128, cache="bf16", lens="ragged", poison=False)
    q = torch.from_numpy(c["q"]).to(DEV)
    K, V = to_dev_cache(c["K"]), to_dev_cache(c["V"])
    lens0 = torch.from_numpy(np.minimum(c["lens"], cap - 8)).to(DEV)
    g = mi.rng(1051, 3)
    kn = torch.from_numpy(g.standard_normal((b, 128), dtype=np.float32)).to(DEV)
    vn = torch.from_numpy(g.standard_normal((b, 128), dtype=np.float32)).to(DEV)
    ws = torch.empty(m.mqa_decode_workspace_bytes(b, h, cap, 128), dtype=torch.uint8, device=DEV)
    o = torch.empty((b, h, 128), dtype=torch.float32, device=DEV)

    def eager(lens):
        m.mqa_append_kv(K, V, kn, vn, lens)
        return m.mqa_decode_step(q, K, V, lens, o=torch.empty_like(o), workspace=ws).clone()

    lens = lens0.clone()
    expect = [eager(lens) for _ in range(3)]            # three steps, each one position longer
    K2, V2 = to_dev_cache(c["K"]), to_dev_cache(c["V"])  # fresh caches for the captured run
    lens = lens0.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            m.mqa_append_kv(K2, V2, kn, vn, lens, stream=side)
            m.mqa_decode_step(q, K2, V2, lens, o=o, workspace=ws, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    lens.copy_(lens0)                                    # the capture itself ran nothing
    for i in range(3):
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(o, expect[i]), f"replay {i} differs from the eager step"
        _ = (q * 2).sum().item()                         # unrelated eager work between replays
    assert torch.equal(lens, lens0 + 3)


# ----------------------------------------------------------------- local attention (Section 4.1 variant)
@pytest.mark.parametrize("window", [1, 31, 32, 33, 100, 5000])
def test_mqa_decode_window_bf16(m, window):
    lens = [1, 2, 31, 32, 33, 64, 65, 97, 300, 301, 0, 255]
    c = mi.random_case(60, len(lens), 8, 301, 128, 128, cache="bf16", lens=lens)
    q = torch.from_numpy(c["q"]).to(DEV)
    K, V = to_dev_cache(c["K"]), to_dev_cache(c["V"])
    dl = torch.from_numpy(c["lens"]).to(DEV)
    o = m.mqa_decode_step_window(q, K, V, dl, window)
    ref = orc.mqa_decode(c["q"], mi.cache_as_f64(c["K"]), mi.cache_as_f64(c["V"]), c["lens"], window=window)
    check(o, ref, "bf16", f"window {window}")
    if window >= 301:
        assert torch.equal(o, m.mqa_decode_step(q, K, V, dl))


def test_decode_window_other_paths(m):
    # long window over a long cache: the ranges are split and merged (few sequences, many CUs)
    c = mi.random_case(61, 2, 32, 3000, 128, 128, cache="bf16", lens=[3000, 1777])
    q = torch.from_numpy(c["q"]).to(DEV)
    K, V = to_dev_cache(c["K"]), to_dev_cache(c["V"])
    dl = torch.from_numpy(c["lens"]).to(DEV)
    for window in (1024, 1500):
        o = m.mqa_decode_step_window(q, K, V, dl, window)
        ref = orc.mqa_decode(c["q"], mi.cache_as_f64(c["K"]), mi.cache_as_f64(c["V"]), c["lens"], window=window)
        check(o, ref, "bf16", f"long window {window}")
    # full sequences whose window is a multiple of the range length: the last range of every sequence starts
    # at the capacity (nothing to do there, and nothing may be read there -- the last sequence ends the buffer)
    c = mi.random_case(64, 2, 8, 4096, 128, 128, cache="bf16", lens=[4096, 4096], poison=False)
    S, chunk, _ = m.mqa_decode_plan(2, 8, 4096, 128, 128, m.MQA_BF16, window=1024)
    assert S > 1 and 1024 % chunk == 0 and S * chunk > 1024
    dl = torch.from_numpy(c["lens"]).to(DEV)
    o = m.mqa_decode_step_window(torch.from_numpy(c["q"]).to(DEV), to_dev_cache(c["K"]), to_dev_cache(c["V"]), dl, 1024)
    check(o, orc.mqa_decode(c["q"], mi.cache_as_f64(c["K"]), mi.cache_as_f64(c["V"]), c["lens"], window=1024), "bf16",
          "window ending at the capacity")
    # float32 cache (generic kernel) and the multi-head layout
    c = mi.random_case(62, 3, 5, 130, 64, 32, cache="f32", lens=[130, 40, 7])
    o = m.mqa_decode_step_window(torch.from_numpy(c["q"]).to(DEV), to_dev_cache(c["K"]), to_dev_cache(c["V"]),
                                 torch.from_numpy(c["lens"]).to(DEV), 32)
    check(o, orc.mqa_decode(c["q"], c["K"].astype(np.float64), c["V"].astype(np.float64), c["lens"], window=32), "f32", "generic window")
    c = mi.random_case(63, 2, 3, 90, 128, 128, cache="bf16", lens=[90, 33], multi_head=True)
    o = m.mha_decode_step_window(torch.from_numpy(c["q"]).to(DEV), to_dev_cache(c["K"]), to_dev_cache(c["V"]),
                                 torch.from_numpy(c["lens"]).to(DEV), 32)
    check(o, orc.mha_decode(c["q"], mi.cache_as_f64(c["K"]), mi.cache_as_f64(c["V"]), c["lens"], window=32), "bf16", "mha window")


# ----------------------------------------------------------------- prompt attention (causal, many queries at once)
@pytest.mark.parametrize("b,n,h,prefix", [(2, 5, 8, 0), (3, 33, 8, 17), (2, 128, 8, 0), (1, 64, 3, 100), (2, 40, 32, 9)])
def test_prefill_attention(m, b, n, h, prefix):
    cap = prefix + n + 7
    g = mi.rng(4000 + n, b)
    q = g.standard_normal((b, n, h, 128), dtype=np.float32) / np.float32(np.sqrt(128)) * np.float32(3)
    c = mi.random_case(70 + n, b, 1, cap, 128, 128, cache="bf16", lens=[prefix + n] * b)
    K, V = to_dev_cache(c["K"]), to_dev_cache(c["V"])
    lens = torch.from_numpy(c["lens"]).to(DEV)
    o = m.mqa_prefill_attention(torch.from_numpy(q).to(DEV), K, V, lens)
    ref = orc.mqa_prefill(q, mi.cache_as_f64(c["K"]), mi.cache_as_f64(c["V"]), c["lens"])
    check(o, ref, "bf16", f"prefill b={b} n={n} h={h} prefix={prefix}")
    # the same rows through n single-token decode steps
    j = n // 2
    step = m.mqa_decode_step(torch.from_numpy(np.ascontiguousarray(q[:, j])).to(DEV), K, V,
                             torch.full((b,), prefix + j + 1, dtype=torch.int32, device=DEV))
    assert float((step - o[:, j]).abs().max()) <= 1e-4


@pytest.mark.parametrize("b,n,h,prefix", [(2, 5, 8, 0), (2, 50, 3, 21), (1, 128, 8, 0)])
def test_mha_prefill_attention(m, b, n, h, prefix):
    cap = prefix + n + 5
    g = mi.rng(4200 + n, b)
    q = g.standard_normal((b, h, n, 128), dtype=np.float32) / np.float32(np.sqrt(128)) * np.float32(3)
    c = mi.random_case(80 + n, b, h, cap, 128, 128, cache="bf16", lens=[prefix + n] * b, multi_head=True)
    K, V = to_dev_cache(c["K"]), to_dev_cache(c["V"])
    lens = torch.from_numpy(c["lens"]).to(DEV)
    o = m.mha_prefill_attention(torch.from_numpy(q).to(DEV), K, V, lens)
    ref = orc.mha_prefill(q, mi.cache_as_f64(c["K"]), mi.cache_as_f64(c["V"]), c["lens"])
    check(o, ref, "bf16", f"mha prefill b={b} n={n} h={h} prefix={prefix}")
    j = n // 2                                          # the same rows through a single-token multi-head step
    step = m.mha_decode_step(torch.from_numpy(np.ascontiguousarray(q[:, :, j])).to(DEV), K, V,
                             torch.full((b,), prefix + j + 1, dtype=torch.int32, device=DEV))
    assert float((step - o[:, :, j]).abs().max()) <= 1e-4


def test_prefill_prompt_then_decode(m):
    """A prompt written with one bulk append and attended in one call, then a decode step on top:
    the cache and lengths the prefill leaves are what the incremental path continues from."""
    b, n, h, d, cap = 4, 48, 8, 256, 64
    g = mi.rng(4100, 0)
    X = g.standard_normal((b, n + 1, d), dtype=np.float32)
    P_q = g.standard_normal((h, d, 128), dtype=np.float32) / np.float32(np.sqrt(d))
    P_k = g.standard_normal((d, 128), dtype=np.float32) / np.float32(np.sqrt(d))
    P_v = g.standard_normal((d, 128), dtype=np.float32) / np.float32(np.sqrt(d))
    dX = torch.from_numpy(X).to(DEV)
    dPq, dPk, dPv = (torch.from_numpy(a).to(DEV) for a in (P_q, P_k, P_v))
    K = torch.full((b, cap, 128), float("nan"), dtype=torch.bfloat16, device=DEV)
    V = torch.full((b, cap, 128), float("nan"), dtype=torch.bfloat16, device=DEV)
    lens = torch.zeros(b, dtype=torch.int32, device=DEV)
    rows = dX[:, :n].reshape(b * n, d).contiguous()
    q = m.mqa_project_qkvo(m.MQA_PROJ_Q, rows, dPq).view(b, n, h, 128)
    kn = m.mqa_project_qkvo(m.MQA_PROJ_KV, rows, dPk).view(b, n, 128)
    vn = m.mqa_project_qkvo(m.MQA_PROJ_KV, rows, dPv).view(b, n, 128)
    m.mqa_append_kv_rows(K, V, kn, vn, lens)
    assert np.array_equal(lens.cpu().numpy(), np.full(b, n))
    assert torch.equal(K[:, :n], kn.to(torch.bfloat16)) and torch.isnan(K[:, n:].float()).all()
    o = m.mqa_prefill_attention(q, K, V, lens)
    # oracle on the GPU's own rounded cache rows would be an input from the HIP path: use the oracle's rows instead
    Kr, Vr = np.zeros((b, cap, 128)), np.zeros((b, cap, 128))
    lr = np.zeros(b, dtype=np.int64)
    for t in range(n):
        orc.append_kv(Kr, Vr, orc.project_kv(X[:, t], P_k), orc.project_kv(X[:, t], P_v), lr, cache="bf16")
    K[:, :n].copy_(torch.from_numpy(Kr[:, :n]).to(torch.bfloat16))      # oracle -> GPU, near-ties aside the same rows
    V[:, :n].copy_(torch.from_numpy(Vr[:, :n]).to(torch.bfloat16))
    o = m.mqa_prefill_attention(q, K, V, lens)
    Q = np.einsum("bnd,hdk->bnhk", X[:, :n].astype(np.float64), P_q.astype(np.float64))
    check(o, orc.mqa_prefill(Q, Kr, Vr, lr), "bf16", "prefill after bulk append")
    # one more token through the incremental path
    x = dX[:, n].contiguous()
    m.mqa_append_kv(K, V, m.mqa_project_qkvo(m.MQA_PROJ_KV, x, dPk), m.mqa_project_qkvo(m.MQA_PROJ_KV, x, dPv), lens)
    o1 = m.mqa_decode_step(m.mqa_project_qkvo(m.MQA_PROJ_Q, x, dPq), K, V, lens)
    orc.append_kv(Kr, Vr, orc.project_kv(X[:, n], P_k), orc.project_kv(X[:, n], P_v), lr, cache="bf16")
    K[:, n].copy_(torch.from_numpy(Kr[:, n]).to(torch.bfloat16))
    V[:, n].copy_(torch.from_numpy(Vr[:, n]).to(torch.bfloat16))
    o1 = m.mqa_decode_step(m.mqa_project_qkvo(m.MQA_PROJ_Q, x, dPq), K, V, lens)
    check(o1, orc.mqa_decode(orc.project_q(X[:, n], P_q), Kr, Vr, lr), "bf16", "decode after prefill")
    # a sequence without room for the whole prompt is left untouched
    lens2 = torch.tensor([cap - 3, 0, 0, 0], dtype=torch.int32, device=DEV)
    K2 = torch.zeros_like(K)
    m.mqa_append_kv_rows(K2, torch.zeros_like(V), kn, vn, lens2)
    assert lens2.cpu().tolist() == [cap - 3, n, n, n] and float(K2[0].float().abs().max()) == 0.0


# ----------------------------------------------------------------- longest-first scheduling of ragged batches
@pytest.mark.parametrize("b,h,cap,multi_head,splits", [(1030, 8, 96, False, 0), (515, 40, 160, False, 0), (5, 8, 300, False, 0),
                                                       (131, 8, 70, True, 0), (300, 16, 256, False, 4),
                                                       (300, 64, 200, False, 0), (1100, 48, 130, False, 0), (257, 33, 40, False, 0),
                                                       (1024, 64, 70, False, 0), (700, 64, 100, False, 0)])
def test_longest_first_schedule_changes_no_result(m, b, h, cap, multi_head, splits):
    """Large batches are started longest sequence first (a ranking pass orders the groups; the grid
    is padded to a multiple of 8 groups); forced here on small ones.  With more than 32 heads and
    more sequences than compute units, one workgroup per compute unit goes over several ranked
    sequences (2, 3 and 5 turns here, some of them empty sequences), ranking up to 1024 sequences
    itself and taking the ranking pass's order beyond that.  Outputs must equal the
    oracle's and be bit-identical to the unscheduled launch and to one workgroup per sequence."""
    c = mi.random_case(40 + b, b, h, cap, 128, 128, cache="bf16", lens="with_zero", multi_head=multi_head)
    tn = dict(splits=splits) if splits else {}
    o, ref = run_case(m, c, multi_head, tuning=dict(tn, flags=64))
    check(o, ref, "bf16", f"scheduled b={b} h={h}")
    o_plain, _ = run_case(m, c, multi_head, tuning=dict(tn, flags=32))
    assert torch.equal(o, o_plain)
    o_each, _ = run_case(m, c, multi_head, tuning=dict(tn, flags=64 | 1024))
    assert torch.equal(o, o_each)
    o_launch, _ = run_case(m, c, multi_head, tuning=dict(tn, flags=64 | 2048))      # ranked by the separate launch
    assert torch.equal(o, o_launch)


@pytest.mark.parametrize("pattern", ["all_equal", "two_values", "one_short"])
def test_ranking_inside_the_kernel_with_equal_lengths(m, pattern):
    """Every workgroup of the persistent form ranks the sequences for itself; equal lengths must be
    ranked the same way by all of them (else a sequence is done twice and another not at all)."""
    b, h, cap = 600, 64, 64
    lens = np.full(b, cap, dtype=np.int32)
    if pattern == "two_values":
        lens[::2] = 17
        lens[5] = 0
    elif pattern == "one_short":
        lens[333] = 3
    c = mi.random_case(77, b, h, cap, 128, 128, cache="bf16", lens=lens)
    o, ref = run_case(m, c, False, tuning=dict(flags=64))
    check(o, ref, "bf16", f"ranked in the kernel, {pattern}")
    o_each, _ = run_case(m, c, False, tuning=dict(flags=64 | 1024))
    assert torch.equal(o, o_each)


# ----------------------------------------------------------------- q, K row, V row and the append in one launch
@pytest.mark.parametrize("b,d,h,k,v,cap,cache,mh", [
    (128, 1024, 8, 128, 128, 40, "bf16", False),      # workload 2's shape: 16x64 tiles
    (128, 1024, 8, 128, 128, 40, "bf16", True),       # ... multi-head: 32x64 tiles
    (40, 136, 26, 48, 16, 5, "f32", False),           # k, v share only a factor 16: 32x16 tiles
    (40, 136, 78, 32, 32, 5, "bf16", False),          # k = v = 32: 32x32 tiles
    (512, 256, 8, 128, 64, 9, "bf16", False),
    (5, 72, 3, 48, 16, 7, "f32", False),
    (33, 136, 4, 32, 32, 5, "f32", True),
    (1024, 264, 8, 128, 128, 6, "bf16", False),       # large batch: the LDS-tiled kernel, 64x64 tiles
    (2500, 264, 8, 128, 128, 4, "bf16", False),       # ... 128x128 tiles, ragged row edge
    (1400, 136, 4, 64, 64, 5, "f32", True),           # ... multi-head rows
])
def test_fused_qkv_projection_and_append(m, b, d, h, k, v, cap, cache, mh):
    g = mi.rng(3300, b + d)
    x = g.standard_normal((b, d), dtype=np.float32)
    P_q = g.standard_normal((h, d, k), dtype=np.float32) / np.float32(np.sqrt(d))
    P_k = g.standard_normal((h, d, k) if mh else (d, k), dtype=np.float32) / np.float32(np.sqrt(d))
    P_v = g.standard_normal((h, d, v) if mh else (d, v), dtype=np.float32) / np.float32(np.sqrt(d))
    lens = g.integers(0, cap + 1, size=b).astype(np.int32)
    lens[0], lens[b - 1] = cap, 0                      # one sequence at capacity: untouched
    tdt = torch.bfloat16 if cache == "bf16" else torch.float32
    kshape = (b, h, cap, k) if mh else (b, cap, k)
    K = torch.full(kshape, 3.0, dtype=tdt, device=DEV)
    V = torch.full(kshape[:-1] + (v,), 3.0, dtype=tdt, device=DEV)
    lens_in = torch.from_numpy(lens).to(DEV)
    lens_out = torch.full((b,), -7, dtype=torch.int32, device=DEV)
    q = m.mqa_project_append_qkv(*(torch.from_numpy(a).to(DEV) for a in (x, P_q, P_k, P_v)), K, V, lens_in, lens_out)
    torch.cuda.synchronize()
    assert np.max(np.abs(q.cpu().numpy() - orc.project_q(x, P_q))) <= 1e-5
    assert np.array_equal(lens_out.cpu().numpy(), np.where(lens < cap, lens + 1, lens))
    assert np.array_equal(lens_in.cpu().numpy(), lens)
    k_exact = orc.project_kv_mh(x, P_k) if mh else orc.project_kv(x, P_k)
    v_exact = orc.project_kv_mh(x, P_v) if mh else orc.project_kv(x, P_v)
    rnd = orc.round_to_bf16 if cache == "bf16" else orc.round_to_f32
    for got, exact in ((K.double().cpu().numpy(), k_exact), (V.double().cpu().numpy(), v_exact)):
        for i in range(b):
            L = int(lens[i])
            rows = np.delete(got[i], L, axis=-2) if L < cap else got[i]
            assert (rows == 3.0).all(), "a row other than the appended one was written"
            if L < cap:
                new = got[i, ..., L, :]
                # the stored value is the oracle's: float64 sum -> float32 -> cache type
                assert np.array_equal(new, rnd(exact[i])), f"sequence {i}: appended row differs from the oracle's"
    # the same through the separate calls: bit for bit
    K2, V2 = torch.full_like(K, 3.0), torch.full_like(V, 3.0)
    l2 = lens_in.clone()
    mode = m.MQA_PROJ_KV_MH if mh else m.MQA_PROJ_KV
    dx = torch.from_numpy(x).to(DEV)
    m.mqa_append_kv(K2, V2, m.mqa_project_qkvo(mode, dx, torch.from_numpy(P_k).to(DEV)),
                    m.mqa_project_qkvo(mode, dx, torch.from_numpy(P_v).to(DEV)), l2)
    assert torch.equal(l2, lens_out)
    assert torch.equal(K2, K) and torch.equal(V2, V)

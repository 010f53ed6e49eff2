"""Parity at the full workload sizes, in the launch configuration the benchmark
times (library heuristics, no tuning): every output row of every sequence is
compared with the float64 oracle, which takes the sequences a few at a time.
Properties that hold at any size (order of the positions, the convex hull of
the V rows, agreement of the two kernels) are checked on top."""
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


def _tol_bf16(got, ref, what):
    err = float(np.max(np.abs(got - ref)))
    assert np.isfinite(got).all(), what
    assert err <= 2e-2 and err <= 1e-2 * float(np.max(np.abs(ref))), f"{what}: max abs err {err:.3e}"
    return err


def test_long_context_probe_mqa_full_size(m):
    """b=64, m=8192, h=32, k=v=128, bf16 K/V, all lengths full (268 MB of K/V)."""
    cfg = mi.CONFIGS[4]
    b, h, cap, k, v = cfg["b"], cfg["h"], cfg["cap"], cfg["k"], cfg["v"]
    q_np = mi.config4_q(b, h, k)
    K_np, V_np = mi.config4_kv(b=b, m=cap, k=k, v=v, threads=8)
    q = torch.from_numpy(q_np).to(DEV)
    K, V = mi.bits_to_torch_bf16(K_np).to(DEV), mi.bits_to_torch_bf16(V_np).to(DEV)
    lens = torch.full((b,), cap, dtype=torch.int32, device=DEV)
    assert m.mqa_decode_num_splits(b, h, cap, k, v, m.MQA_BF16) == 4
    o = m.mqa_decode_step(q, K, V, lens)
    torch.cuda.synchronize()
    got = o.cpu().numpy().astype(np.float64)
    err = 0.0
    for i0 in range(0, b, 8):            # all 64 sequences, 8 at a time (the float64 copies are 128 MiB per batch)
        sl = slice(i0, i0 + 8)
        ref = orc.mqa_decode(q_np[sl], mi.bf16_bits_to_f64(K_np[sl]), mi.bf16_bits_to_f64(V_np[sl]), [cap] * 8)
        err = max(err, _tol_bf16(got[sl], ref, f"long-context probe, sequences {i0}..{i0 + 7}"))
    # every output is a convex combination of its sequence's V rows
    Vf = V.float()
    assert bool((o <= Vf.amax(dim=1)[:, None, :] + 1e-4).all()) and bool((o >= Vf.amin(dim=1)[:, None, :] - 1e-4).all())
    assert np.isfinite(got).all()
    print(f"long-context probe MQA: max abs err over all {b} sequences {err:.2e}")
    # a property that holds at any size (Section 2.1: a weighted sum over the memory positions does not
    # depend on their order): the same rows of K and V in another order give the same outputs, on all
    # 64 sequences, although every tile, range and wave then holds different positions
    perm = torch.from_numpy(mi.rng(4, 997).permutation(cap)).to(DEV)
    o_perm = m.mqa_decode_step(q, K[:, perm].contiguous(), V[:, perm].contiguous(), lens)
    torch.cuda.synchronize()
    assert float((o_perm - o).abs().max()) <= 1e-5


def test_long_context_probe_mha_full_size(m):
    """The multi-head twin: K, V [64,32,8192,128] bf16, 8 GiB.  The blocks K[i,j], V[i,j] are
    copies of 8 seeded host-generated blocks (block (i*h+j) % 8), so any (i,j) output can be
    checked against the oracle at the cost of one [8192,128] block."""
    cfg = mi.CONFIGS[4]
    b, h, cap, k, v = cfg["b"], cfg["h"], cfg["cap"], cfg["k"], cfg["v"]
    npool = 8
    pool = [mi.config4_kv_mh_block(0, p_, m=cap, k=k, v=v) for p_ in range(npool)]
    Kp = torch.stack([mi.bits_to_torch_bf16(kb) for kb, _ in pool]).to(DEV)
    Vp = torch.stack([mi.bits_to_torch_bf16(vb) for _, vb in pool]).to(DEV)
    K = torch.empty((b, h, cap, k), dtype=torch.bfloat16, device=DEV)
    V = torch.empty((b, h, cap, v), dtype=torch.bfloat16, device=DEV)
    idx = (torch.arange(b * h, device=DEV) % npool).view(b, h)
    for i in range(b):
        K[i].copy_(Kp[idx[i]])
        V[i].copy_(Vp[idx[i]])
    q_np = mi.config4_q(b, h, k)
    q = torch.from_numpy(q_np).to(DEV)
    lens = torch.full((b,), cap, dtype=torch.int32, device=DEV)
    o = m.mha_decode_step(q, K, V, lens)
    torch.cuda.synchronize()
    got = o.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    # all 2048 (sequence, head) pairs: the pairs that hold a copy of pool block p_ are that block's memory
    # queried by their 256 q rows (the oracle's multi-query step with one sequence of 256 heads)
    worst = 0.0
    flat_q, flat_got = q_np.reshape(b * h, k), got.reshape(b * h, v)
    for p_ in range(npool):
        who = np.arange(p_, b * h, npool)
        kb, vb = pool[p_]
        ref = orc.mqa_decode(flat_q[who][None], mi.bf16_bits_to_f64(kb)[None], mi.bf16_bits_to_f64(vb)[None], [cap])[0]
        worst = max(worst, _tol_bf16(flat_got[who], ref, f"mha pairs holding block {p_}"))
    i, j = 37, 5                       # and one pair through the Section 2.1 function itself
    kb, vb = pool[(i * h + j) % npool]
    _tol_bf16(got[i, j], orc.dot_product_attention(q_np[i, j], mi.bf16_bits_to_f64(kb), mi.bf16_bits_to_f64(vb)), "mha (37,5)")
    print(f"long-context probe MHA: max abs err over all {b * h} (sequence, head) pairs {worst:.2e}")


def test_ragged_large_batch_full_size(m):
    """b=512, h=64, cap=4096, lens ~ U[1,4096], 1 % of the logits lifted by +30, NaN beyond the lengths."""
    cfg = mi.CONFIGS[5]
    b, h, cap, k, v = cfg["b"], cfg["h"], cfg["cap"], cfg["k"], cfg["v"]
    q_np, K_np, V_np, lens_np = mi.config5(b, h, k, v, cap, cfg["outlier_fraction"], cfg["outlier_boost"])
    q = torch.from_numpy(q_np).to(DEV)
    K, V = mi.bits_to_torch_bf16(K_np).to(DEV), mi.bits_to_torch_bf16(V_np).to(DEV)
    lens = torch.from_numpy(lens_np).to(DEV)
    o = m.mqa_decode_step(q, K, V, lens)
    torch.cuda.synchronize()
    got = o.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all(), "NaN rows beyond the length leaked into the output"
    err = 0.0
    for i0 in range(0, b, 16):           # all 512 sequences, 16 at a time
        sl = slice(i0, i0 + 16)
        Kf, Vf = mi.bf16_bits_to_f64(K_np[sl]), mi.bf16_bits_to_f64(V_np[sl])
        ref = orc.mqa_decode(q_np[sl], Kf, Vf, lens_np[sl])
        err = max(err, _tol_bf16(got[sl], ref, f"ragged batch, sequences {i0}..{i0 + 15}"))
    # the generic kernel (plain float32 FMAs through LDS, no code in common with the MFMA kernel) agrees on
    # all 512 x 64 output rows
    o_gen = m.mqa_decode_step(q, K, V, lens, tuning=dict(kernel=1))
    torch.cuda.synchronize()
    # (with 64 heads the MFMA path keeps the softmax weights as single bf16 terms: 2^-9 relative each, up to
    # ~4e-3 on an output of a short sequence; the generic kernel is plain float32)
    assert bool(torch.isfinite(o_gen).all()) and float((o_gen - o).abs().max()) <= 1e-2
    o_two = m.mqa_decode_step(q, K, V, lens, tuning=dict(flags=128))        # two-term weights: float32-level agreement
    torch.cuda.synchronize()
    assert float((o_gen - o_two).abs().max()) <= 1e-4
    # the forced-large logits are present in the sample: some softmax rows are sharply peaked
    longest = [int(np.argmax(lens_np))]
    w = orc.mqa_decode_weights(q_np[longest], mi.bf16_bits_to_f64(K_np[longest]), lens_np[longest])[0]
    print(f"ragged batch: lens {lens_np.min()}..{lens_np.max()}, max abs err over all {b} sequences {err:.2e}, "
          f"largest single weight in the longest sequence {w.max():.3f}")

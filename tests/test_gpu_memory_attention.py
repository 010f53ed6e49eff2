"""Encoder-decoder ("memory") multi-query attention as its own call pair: the memory is projected
once into the cache (mqa_project_memory_kv), every decoding step attends to it with fixed lengths
(mqa_memory_decode_step).  Checked against the oracle's one-query layer functions (Section 2.2
listing and the Section 3 rule) at the single-step float32 workload's shape and at the decoder
stack's shape (128 sequences, 128 source positions, bf16 cache), with padded memories and with
the four hypotheses of a beam sharing a source."""
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


def test_single_query_against_a_memory_fp32(m):
    """Workload 1's shape: x [d] against M [128,d], float32 cache; y against the Section 2.2 / Section 3
    one-query layer, 1e-5."""
    c = mi.config1()
    h, d, k = c["P_q"].shape
    v = c["P_o"].shape[2]
    mem = c["M"].shape[1]
    dM = torch.from_numpy(c["M"]).to(DEV)                                     # [1,m,d]
    K = torch.full((1, mem + 3, k), float("nan"), dtype=torch.float32, device=DEV)
    V = torch.full((1, mem + 3, v), float("nan"), dtype=torch.float32, device=DEV)
    lens = torch.zeros(1, dtype=torch.int32, device=DEV)
    m.mqa_project_memory_kv(dM, torch.from_numpy(c["P_k"]).to(DEV), torch.from_numpy(c["P_v"]).to(DEV), K, V, lens)
    assert int(lens[0]) == mem and bool(torch.isnan(K[0, mem:]).all())
    q = m.mqa_project_qkvo(m.MQA_PROJ_Q, torch.from_numpy(c["x"]).to(DEV), torch.from_numpy(c["P_q"]).to(DEV))
    o = m.mqa_memory_decode_step(q.view(1, 1, h, k), K, V, lens)
    y = m.mqa_project_qkvo(m.MQA_PROJ_O, o.view(1, h, v), torch.from_numpy(c["P_o"]).to(DEV))
    ref = orc.multiquery_attention(c["x"][0], c["M"][0], c["P_q"], c["P_k"], c["P_v"], c["P_o"])
    err = float(np.max(np.abs(y[0].cpu().numpy() - ref)))
    assert err <= 1e-5, err
    # multi-head memory: per-head caches through the same projection call, then the multi-head step
    Kh = torch.zeros((1, h, mem, k), dtype=torch.float32, device=DEV)
    Vh = torch.zeros((1, h, mem, v), dtype=torch.float32, device=DEV)
    m.mqa_project_memory_kv(dM, torch.from_numpy(c["P_k_mh"]).to(DEV), torch.from_numpy(c["P_v_mh"]).to(DEV), Kh, Vh, lens)
    y = m.mqa_project_qkvo(m.MQA_PROJ_O, m.mha_decode_step(q, Kh, Vh, lens), torch.from_numpy(c["P_o"]).to(DEV))
    ref = orc.multihead_attention(c["x"][0], c["M"][0], c["P_q"], c["P_k_mh"], c["P_v_mh"], c["P_o"])
    assert float(np.max(np.abs(y[0].cpu().numpy() - ref))) <= 1e-5


@pytest.mark.parametrize("queries", [1, 4])
def test_memory_attention_at_the_decoder_stack_shape(m, queries):
    """b=128 sources of 128 positions (padded: valid lengths 1..128), d=1024, h=8, k=v=128, bf16 cache; one
    query per memory (greedy) or four (a beam).  The cache rows equal the oracle's bit for bit; o and y meet the
    bf16 bar; y also equals the one-query layer function on the valid rows of each memory."""
    b, mem, d, h, k, v = 128, 128, 1024, 8, 128, 128
    g = mi.rng(2400, queries)
    s = np.float32(d ** -0.5)
    M = g.standard_normal((b, mem, d), dtype=np.float32)
    x = g.standard_normal((b, queries, d), dtype=np.float32)
    P_q = g.standard_normal((h, d, k), dtype=np.float32) * s
    P_k = g.standard_normal((d, k), dtype=np.float32) * s
    P_v = g.standard_normal((d, v), dtype=np.float32) * s
    P_o = g.standard_normal((h, d, v), dtype=np.float32) * np.float32((h * v) ** -0.5)
    mlen = g.integers(1, mem + 1, size=b).astype(np.int32)
    mlen[0], mlen[1] = mem, 1
    K = torch.zeros((b, mem, k), dtype=torch.bfloat16, device=DEV)
    V = torch.zeros((b, mem, v), dtype=torch.bfloat16, device=DEV)
    lens = torch.full((b,), -1, dtype=torch.int32, device=DEV)
    m.mqa_project_memory_kv(torch.from_numpy(M).to(DEV), torch.from_numpy(P_k).to(DEV), torch.from_numpy(P_v).to(DEV),
                            K, V, lens, mem_lens=torch.from_numpy(mlen).to(DEV))
    Kr = orc.round_to_bf16(orc.project_kv(M.reshape(b * mem, d), P_k)).reshape(b, mem, k)
    Vr = orc.round_to_bf16(orc.project_kv(M.reshape(b * mem, d), P_v)).reshape(b, mem, v)
    assert np.array_equal(lens.cpu().numpy(), mlen)
    assert np.array_equal(K.double().cpu().numpy(), Kr) and np.array_equal(V.double().cpu().numpy(), Vr)
    q = m.mqa_project_qkvo(m.MQA_PROJ_Q, torch.from_numpy(x).to(DEV).view(b * queries, d), torch.from_numpy(P_q).to(DEV))
    o = m.mqa_memory_decode_step(q.view(b, queries, h, k), K, V, lens)
    y = m.mqa_project_qkvo(m.MQA_PROJ_O, o.view(b * queries, h, v), torch.from_numpy(P_o).to(DEV)).view(b, queries, d)
    torch.cuda.synchronize()
    q_ref = orc.project_q(x.reshape(b * queries, d), P_q).reshape(b, queries * h, k)
    o_ref = orc.mqa_decode(q_ref, Kr, Vr, mlen)                                  # queries*h heads over one K/V
    y_ref = orc.project_o(o_ref.reshape(b * queries, h, v), P_o).reshape(b, queries, d)
    for got, ref, what in ((o.view(b, queries * h, v), o_ref, "o"), (y, y_ref, "y")):
        err = float(np.max(np.abs(got.cpu().numpy().astype(np.float64) - ref)))
        assert err <= 2e-2 and err <= 1e-2 * float(np.max(np.abs(ref))), (what, err)
    # the layer function itself on a few memories (its K/V rounded like the cache)
    for i in (0, 1, 77):
        L = int(mlen[i])
        for e in range(queries):
            ref = orc.multiquery_attention_batched(x[i, e][None, None], M[i, :L][None], None, P_q, P_k, P_v, P_o,
                                                   kv_round=orc.round_to_bf16)[0, 0]
            err = float(np.max(np.abs(y[i, e].cpu().numpy() - ref)))
            assert err <= 2e-2 and err <= 1e-2 * float(np.max(np.abs(ref))), (i, e, err)

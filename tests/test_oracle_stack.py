"""Pins for the oracle's decoder stack: stepping it token by token must equal a
parallel evaluation of the same model built from torch's float64 library
routines (layer_norm, linear, relu, causal scaled_dot_product_attention)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import mqa_inputs as mi
from oracle import decoder_stack as ods


def torch_parallel_logits(w, tokens, multi_head):
    E, pos = torch.from_numpy(w["E"]).double(), torch.from_numpy(w["pos"]).double()
    b, n = tokens.shape
    d = E.shape[1]
    x = E[torch.from_numpy(tokens)] + pos[:n][None]
    for lw in w["layers"]:
        P_q, P_k, P_v, P_o, W1, W2 = (torch.from_numpy(lw[k_]).double() for k_ in ("P_q", "P_k", "P_v", "P_o", "W1", "W2"))
        h = P_q.shape[0]
        hx = F.layer_norm(x, (d,), eps=1e-6)
        q = torch.einsum("bnd,hdk->bhnk", hx, P_q)
        if multi_head:
            K = torch.einsum("bnd,hdk->bhnk", hx, P_k)
            V = torch.einsum("bnd,hdv->bhnv", hx, P_v)
        else:
            K = torch.einsum("bnd,dk->bnk", hx, P_k)[:, None].expand(b, h, n, -1)
            V = torch.einsum("bnd,dv->bnv", hx, P_v)[:, None].expand(b, h, n, -1)
        o = F.scaled_dot_product_attention(q, K, V, is_causal=True, scale=1.0)
        x = x + torch.einsum("bhnv,hdv->bnd", o, P_o)
        x = x + F.linear(F.relu(F.linear(F.layer_norm(x, (d,), eps=1e-6), W1.T)), W2.T)
    return (F.layer_norm(x, (d,), eps=1e-6) @ E.T).numpy()


@pytest.mark.parametrize("multi_head", [False, True])
def test_incremental_stack_equals_parallel_torch_model(multi_head):
    w = mi.config3_weights(layers=2, d=32, h=4, k=8, v=8, d_ff=64, vocab=50, max_pos=16, multi_head=multi_head)
    b, n = 3, 9
    tokens = mi.rng(3, 77).integers(0, 50, size=(b, n))
    ref = torch_parallel_logits(w, tokens, multi_head)
    st = ods.OracleStack(w, b, cap=n, multi_head=multi_head, cache="f64")
    for t in range(n):
        logits = st.step(tokens[:, t], t)
        assert np.max(np.abs(logits - ref[:, t])) <= 1e-10
    assert all(int(x) == n for l in st.lens for x in l)


def test_layernorm_and_greedy():
    g = np.random.default_rng(5)
    x = g.normal(size=(4, 33)) * 3 + 1
    ref = F.layer_norm(torch.from_numpy(x), (33,), eps=1e-6).numpy()
    assert np.max(np.abs(ods.layernorm(x) - ref)) <= 1e-14
    assert list(ods.greedy_token(np.array([[1.0, 3.0, 3.0, 2.0], [5.0, 5.0, 5.0, 5.0], [-1.0, -2.0, -0.5, -0.5]]))) == [1, 0, 2]

"""Float64 oracle of the decoder-only stack around the attention step.

TEST INFRASTRUCTURE ONLY (see mqa_oracle.py).  The paper describes its models in
prose only (Section 4.1: layers, d_model, d_ff, h, d_k = d_v, learned positional
embeddings, embedding tied to the output layer); the reading taken here:
pre-layernorm residual blocks  x += Attn(LN(x)),  x += relu(LN(x) W1) W2,  a
final layernorm, logits = x E^T, no biases, layernorm gain 1 / bias 0 /
eps 1e-6 (biased variance), greedy token = lowest index among the largest logits.
Pins (tests/test_oracle_stack.py): torch's float64 layer_norm, linear, relu and
causal scaled_dot_product_attention run over the whole sequence in parallel.
"""
from __future__ import annotations

import numpy as np

from . import mqa_oracle as orc

F64 = np.float64


def layernorm(x, eps=1e-6):
    x = np.asarray(x, dtype=F64)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps)


def feed_forward(x, W1, W2):
    return np.maximum(layernorm(x) @ np.asarray(W1, F64), 0.0) @ np.asarray(W2, F64)


def greedy_token(logits):
    """Lowest index among the largest logits of each row (numpy argmax does exactly that)."""
    return np.argmax(logits, axis=-1)


class OracleStack:
    def __init__(self, weights, batch, cap, multi_head, cache="bf16"):
        self.w, self.b, self.cap, self.multi_head, self.cache = weights, batch, cap, multi_head, cache
        self.E = np.asarray(weights["E"], F64)
        self.pos = np.asarray(weights["pos"], F64)
        self.layers = [{k: np.asarray(v, F64) for k, v in lw.items()} for lw in weights["layers"]]
        h, d, k = self.layers[0]["P_q"].shape
        v = self.layers[0]["P_o"].shape[2]
        kshape = (batch, h, cap, k) if multi_head else (batch, cap, k)
        vshape = (batch, h, cap, v) if multi_head else (batch, cap, v)
        self.K = [np.zeros(kshape) for _ in self.layers]
        self.V = [np.zeros(vshape) for _ in self.layers]
        self.lens = [np.zeros(batch, dtype=np.int64) for _ in self.layers]

    def embed(self, tokens, t):
        return self.E[np.asarray(tokens)] + self.pos[t][None, :]

    def attention(self, l, x):
        """One incremental attention step of layer l on LN(x); returns y and the unrounded new rows."""
        w = self.layers[l]
        hx = layernorm(x)
        step = orc.mha_incremental_step if self.multi_head else orc.mqa_incremental_step
        proj = orc.project_kv_mh if self.multi_head else orc.project_kv
        rows = (proj(hx, w["P_k"]), proj(hx, w["P_v"]))
        y, _, _ = step(hx, self.K[l], self.V[l], self.lens[l], w["P_q"], w["P_k"], w["P_v"], w["P_o"], cache=self.cache)
        return y, rows

    def step(self, tokens, t):
        x = self.embed(tokens, t)
        for l, w in enumerate(self.layers):
            x = x + self.attention(l, x)[0]
            x = x + feed_forward(x, w["W1"], w["W2"])
        return layernorm(x) @ self.E.T

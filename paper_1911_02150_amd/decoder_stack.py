"""Incremental decoding of a decoder-only stack whose attention is the library's
multi-query (or multi-head) decode step.  Pure glue: every operation is a call
into the HIP library; torch only holds the device buffers.

Stack (the model family of the paper's Section 4.1, random weights): token
embedding + learned positional embedding; per layer  x += Attn(LN(x)),
x += relu(LN(x) W1) W2;  final LN; logits = x E^T (embedding tied to the output
layer); no biases; layernorm gain 1, bias 0, eps 1e-6.
"""
from __future__ import annotations

import torch

from . import binding as B


class DecoderStack:
    def __init__(self, weights: dict, batch: int, cap: int, multi_head: bool, device="cuda:0",
                 cache_dtype=torch.bfloat16):
        dev = torch.device(device)
        self.dev, self.b, self.cap, self.multi_head = dev, batch, cap, multi_head
        self.E = torch.from_numpy(weights["E"]).to(dev)
        self.pos = torch.from_numpy(weights["pos"]).to(dev)
        self.layers = [{k: torch.from_numpy(v).to(dev) for k, v in lw.items()} for lw in weights["layers"]]
        h, d, k = self.layers[0]["P_q"].shape
        v = self.layers[0]["P_o"].shape[2]
        self.h, self.d, self.k, self.v = h, d, k, v
        kshape = (batch, h, cap, k) if multi_head else (batch, cap, k)
        vshape = (batch, h, cap, v) if multi_head else (batch, cap, v)
        self.K = [torch.zeros(kshape, dtype=cache_dtype, device=dev) for _ in self.layers]
        self.V = [torch.zeros(vshape, dtype=cache_dtype, device=dev) for _ in self.layers]
        self.lens = [torch.zeros(batch, dtype=torch.int32, device=dev) for _ in self.layers]
        self._lens_next = [torch.zeros(batch, dtype=torch.int32, device=dev) for _ in self.layers]

    # -- pieces, so that a test can look between them
    def embed(self, tokens: torch.Tensor, t: int) -> torch.Tensor:
        positions = torch.full((self.b,), t, dtype=torch.int32, device=self.dev)
        return B.mqa_stack_embed(tokens.to(torch.int32), positions, self.E, self.pos)

    def attention_append(self, l: int, x: torch.Tensor):
        """LN, projections of q and the new K/V rows, append.  Returns q and the float32 rows."""
        w = self.layers[l]
        hx = B.mqa_stack_layernorm(x)
        q = B.mqa_project_qkvo(B.MQA_PROJ_Q, hx, w["P_q"])
        mode = B.MQA_PROJ_KV_MH if self.multi_head else B.MQA_PROJ_KV
        kn = B.mqa_project_qkvo(mode, hx, w["P_k"])
        vn = B.mqa_project_qkvo(mode, hx, w["P_v"])
        B.mqa_append_kv(self.K[l], self.V[l], kn, vn, self.lens[l])
        return q, kn, vn

    def attention_append_fused(self, l: int, x: torch.Tensor) -> torch.Tensor:
        """LN, then q and the append of the new K/V rows in one launch.  Returns q."""
        w = self.layers[l]
        hx = B.mqa_stack_layernorm(x)
        q = B.mqa_project_append_qkv(hx, w["P_q"], w["P_k"], w["P_v"], self.K[l], self.V[l], self.lens[l],
                                     self._lens_next[l])
        self.lens[l], self._lens_next[l] = self._lens_next[l], self.lens[l]      # the lengths alternate between two arrays
        return q

    def attention_attend(self, l: int, q: torch.Tensor) -> torch.Tensor:
        """Attention over the cache and the output projection.  Returns y."""
        dec = B.mha_decode_step if self.multi_head else B.mqa_decode_step
        o = dec(q, self.K[l], self.V[l], self.lens[l])
        return B.mqa_project_qkvo(B.MQA_PROJ_O, o, self.layers[l]["P_o"])

    def feed_forward(self, l: int, x: torch.Tensor) -> torch.Tensor:
        w = self.layers[l]
        hx = B.mqa_stack_layernorm(x)
        u = B.mqa_project_qkvo(B.MQA_PROJ_LINEAR, hx, w["W1"])
        B.mqa_stack_relu(u)
        return B.mqa_project_qkvo(B.MQA_PROJ_LINEAR, u, w["W2"])

    def logits(self, x: torch.Tensor) -> torch.Tensor:
        hx = B.mqa_stack_layernorm(x)
        return B.mqa_project_qkvo(B.MQA_PROJ_O, hx.view(self.b, 1, self.d), self.E.view(1, -1, self.d))

    # -- one decoding step for the whole stack: per layer 8 launches (layernorm, fused q/K/V + append,
    #    attention (+ merge), output projection added into x, layernorm, W1 with relu, W2 added into x)
    def step(self, tokens: torch.Tensor, t: int) -> torch.Tensor:
        x = self.embed(tokens, t)
        dec = B.mha_decode_step if self.multi_head else B.mqa_decode_step
        for l, w in enumerate(self.layers):
            q = self.attention_append_fused(l, x)
            o = dec(q, self.K[l], self.V[l], self.lens[l])
            B.mqa_project_qkvo_ex(B.MQA_PROJ_O, o, w["P_o"], out=x, epilogue=B.MQA_EPI_ADD)
            u = B.mqa_project_qkvo_ex(B.MQA_PROJ_LINEAR, B.mqa_stack_layernorm(x), w["W1"], epilogue=B.MQA_EPI_RELU)
            B.mqa_project_qkvo_ex(B.MQA_PROJ_LINEAR, u, w["W2"], out=x, epilogue=B.MQA_EPI_ADD)
        return self.logits(x)

    # -- a whole prompt at once (multi-query only): bulk append + fused causal attention per layer
    def prefill(self, prompts: torch.Tensor) -> torch.Tensor:
        """prompts [b,n] int32, caches empty.  Returns the logits of the last prompt position [b,vocab]."""
        if self.multi_head:
            raise NotImplementedError("prefill is built for the multi-query cache")
        b, n = prompts.shape
        positions = torch.arange(n, dtype=torch.int32, device=self.dev).repeat(b)
        x = B.mqa_stack_embed(prompts.reshape(-1).to(torch.int32).contiguous(), positions, self.E, self.pos)   # [b*n,d]
        for l, w in enumerate(self.layers):
            hx = B.mqa_stack_layernorm(x)
            q = B.mqa_project_qkvo(B.MQA_PROJ_Q, hx, w["P_q"]).view(b, n, self.h, self.k)
            kn = B.mqa_project_qkvo(B.MQA_PROJ_KV, hx, w["P_k"]).view(b, n, self.k)
            vn = B.mqa_project_qkvo(B.MQA_PROJ_KV, hx, w["P_v"]).view(b, n, self.v)
            B.mqa_append_kv_rows(self.K[l], self.V[l], kn, vn, self.lens[l])
            o = B.mqa_prefill_attention(q, self.K[l], self.V[l], self.lens[l])
            B.mqa_project_qkvo_ex(B.MQA_PROJ_O, o.view(b * n, self.h, self.v), w["P_o"], out=x, epilogue=B.MQA_EPI_ADD)
            u = B.mqa_project_qkvo_ex(B.MQA_PROJ_LINEAR, B.mqa_stack_layernorm(x), w["W1"], epilogue=B.MQA_EPI_RELU)
            B.mqa_project_qkvo_ex(B.MQA_PROJ_LINEAR, u, w["W2"], out=x, epilogue=B.MQA_EPI_ADD)
        last = x.view(b, n, self.d)[:, n - 1].contiguous()
        return self.logits(last)

    def greedy(self, logits: torch.Tensor) -> torch.Tensor:
        return B.mqa_stack_argmax(logits)

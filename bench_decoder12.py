#!/usr/bin/env python3
"""Decoder harness around the attention library: the benchmark contract's fifth configuration.

A 12-layer pre-LayerNorm decoder (d_model 768, 12 heads of 64, MLP 3072 with GELU, vocabulary
50257, learned positions, LM head tied to the token embedding, random-init bf16 weights N(0, 0.02))
run forward on B=8, N=4096 random token ids.  Everything except attention is a PyTorch-ROCm op
(embedding, LayerNorm, GEMMs, GELU: they are not the product); attention is one
gformer_attn_fwd call per layer (window 256, 2 of the 12 heads windowed: the 3/16 ratio of
section IV-D rounded to whole heads) on strided views of the fused QKV projection, i.e. the
paper's [B, N, H, E] storage of section III-A passed through strides, with no transposes or
copies around the call.  The script reports the attention share of the layer time.

    python bench_decoder12.py [--layers 12] [--batch 8] [--seq 4096] [--steps 5]

Prints one JSON line.  bench.py embeds the same measurement as `modes.decoder12`.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
from dataclasses import dataclass

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


@dataclass(frozen=True)
class DecoderConfig:
    layers: int = 12
    d_model: int = 768
    heads: int = 12
    d_head: int = 64
    d_mlp: int = 3072
    vocab: int = 50257
    max_pos: int = 4096
    window: int = 256
    n_sparse_heads: int = 2
    init_std: float = 0.02
    seed: int = 1005


def init_weights(cfg: DecoderConfig, dtype, device):
    """Seeded N(0, init_std) weights (LayerNorm gains 1, all biases 0), drawn on the CPU so that
    the same values can be handed to a reference model."""
    import torch
    g = torch.Generator().manual_seed(cfg.seed)

    def w(*shape):
        return (torch.randn(*shape, generator=g) * cfg.init_std).to(dtype).to(device)

    W = {"wte": w(cfg.vocab, cfg.d_model), "wpe": w(cfg.max_pos, cfg.d_model), "layers": []}
    for _ in range(cfg.layers):
        W["layers"].append({"w_qkv": w(cfg.d_model, 3 * cfg.d_model), "w_o": w(cfg.d_model, cfg.d_model),
                            "w_1": w(cfg.d_model, cfg.d_mlp), "w_2": w(cfg.d_mlp, cfg.d_model)})
    return W


class Decoder:
    """Forward pass only.  `attention(q, k, v, out)` receives [B, H, N, d] views (strided) and
    fills `out`; the default is the library."""

    def __init__(self, cfg: DecoderConfig, weights, attention=None):
        self.cfg, self.W = cfg, weights
        self.attention = attention or self._library_attention
        self.attn_events = []   # (start, end) per layer when timing is on
        self.layer_events = []
        self.timing = False

    def _library_attention(self, q, k, v, out):
        from paper_2412_19829_amd import binding as gb
        gb.gformer_attn_fwd(q, k, v, out, self.cfg.window, self.cfg.n_sparse_heads)

    def forward(self, ids):
        import torch
        import torch.nn.functional as F
        cfg = self.cfg
        B, N = ids.shape
        H, d, D = cfg.heads, cfg.d_head, cfg.d_model
        x = self.W["wte"][ids] + self.W["wpe"][:N]
        ones = torch.ones(D, dtype=x.dtype, device=x.device)
        zeros = torch.zeros(D, dtype=x.dtype, device=x.device)
        q_scale = 1.0 / math.sqrt(d)
        for L in self.W["layers"]:
            if self.timing:
                ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
                ev[0].record()
            h = F.layer_norm(x, (D,), ones, zeros)
            qkv = (h.reshape(B * N, D) @ L["w_qkv"]).view(B, N, 3, H, d)
            qkv[:, :, 0].mul_(q_scale)   # Q pre-scaled: softmax_scale stays 1, as in the other workloads
            q, k, v = (qkv[:, :, i].permute(0, 2, 1, 3) for i in range(3))   # [B, H, N, d] views
            attn = torch.empty((B, N, H, d), dtype=x.dtype, device=x.device)
            if self.timing:
                ev[1].record()
            self.attention(q, k, v, attn.permute(0, 2, 1, 3))
            if self.timing:
                ev[2].record()
            x = x + (attn.view(B * N, D) @ L["w_o"]).view(B, N, D)
            h = F.layer_norm(x, (D,), ones, zeros)
            x = x + (F.gelu(h.reshape(B * N, D) @ L["w_1"]) @ L["w_2"]).view(B, N, D)
            if self.timing:
                ev[3].record()
                self.attn_events.append((ev[1], ev[2]))
                self.layer_events.append((ev[0], ev[3]))
        x = F.layer_norm(x, (D,), ones, zeros)
        return x.reshape(B * N, D) @ self.W["wte"].t()


def measure(layers=12, batch=8, seq=4096, steps=5, warmup=2):
    """Times the forward pass on cuda:0; returns the dict that is printed / embedded."""
    import torch
    from paper_2412_19829_amd import binding as gb
    gb.lib()
    cfg = DecoderConfig(layers=layers, max_pos=seq)
    dev = torch.device("cuda:0")
    W = init_weights(cfg, torch.bfloat16, dev)
    model = Decoder(cfg, W)
    g = torch.Generator().manual_seed(cfg.seed + 1)
    ids = torch.randint(0, cfg.vocab, (batch, seq), generator=g).to(dev)
    for _ in range(warmup):
        model.forward(ids)
    torch.cuda.synchronize()
    model.timing = True
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0.record()
    for _ in range(steps):
        logits = model.forward(ids)
    t1.record()
    torch.cuda.synchronize()
    assert bool(torch.isfinite(logits.float()).all())
    attn_ms = sum(a.elapsed_time(b) for a, b in model.attn_events) / len(model.attn_events)
    layer_ms = sum(a.elapsed_time(b) for a, b in model.layer_events) / len(model.layer_events)
    fwd_ms = t0.elapsed_time(t1) / steps
    return {"workload": f"decoder12: {cfg.layers} pre-LN layers, d_model={cfg.d_model}, {cfg.heads} heads x {cfg.d_head}, "
                        f"MLP {cfg.d_mlp} GELU, vocab {cfg.vocab}, B={batch} N={seq}, window={cfg.window}, "
                        f"n_sparse_heads={cfg.n_sparse_heads}, bf16 weights N(0,{cfg.init_std})",
            "attention_ms_per_layer": round(attn_ms, 4), "layer_ms": round(layer_ms, 4),
            "attention_share_of_layer": round(attn_ms / layer_ms, 4),
            "forward_ms": round(fwd_ms, 3), "tokens_per_s": round(batch * seq / (fwd_ms * 1e-3), 1),
            "steps": steps,
            "note": "attention = gformer_attn_fwd on strided [B,N,H,E] views of the fused QKV projection; "
                    "all other ops are PyTorch-ROCm library ops; event pairs per layer add launch gaps "
                    "to both figures"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--layers", type=int, default=12)
    ap.add_argument("--batch", type=int, default=8)
    ap.add_argument("--seq", type=int, default=4096)
    ap.add_argument("--steps", type=int, default=5)
    args = ap.parse_args()
    import torch
    if not torch.cuda.is_available():
        print("bench_decoder12.py: no GPU visible; there is no CPU path", file=sys.stderr)
        return 2
    print(json.dumps(measure(args.layers, args.batch, args.seq, args.steps)))
    return 0


if __name__ == "__main__":
    sys.exit(main())

"""The decoder harness of the benchmark contract's fifth configuration at reduced size: the same
model code on the GPU (attention = the library) against the CPU in fp64 with the oracle as
attention, same seeded weights and token ids."""
from __future__ import annotations

import numpy as np
import pytest

import bench_decoder12 as bd
from oracle import cpu_oracle as co


def _oracle_attention(cfg):
    def attention(q, k, v, out):
        import torch
        qn, kn, vn = (np.ascontiguousarray(t.detach().numpy(), dtype=np.float64) for t in (q, k, v))
        out.copy_(torch.from_numpy(co.attn_fwd(qn, kn, vn, cfg.window, cfg.n_sparse_heads)))
    return attention


SMALL = bd.DecoderConfig(layers=3, d_model=128, heads=2, d_head=64, d_mlp=256, vocab=500, max_pos=200,
                         window=48, n_sparse_heads=1, seed=77)


def test_decoder_config_is_the_contract_shape():
    cfg = bd.DecoderConfig()
    assert (cfg.layers, cfg.d_model, cfg.heads, cfg.d_head, cfg.d_mlp, cfg.vocab) == (12, 768, 12, 64, 3072, 50257)
    assert cfg.window == 256 and cfg.init_std == 0.02 and cfg.heads * cfg.d_head == cfg.d_model


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_reduced_decoder_matches_the_model_with_the_oracle_as_attention(dtype):
    import torch
    cfg = SMALL
    B, N = 2, 200
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    W_gpu = bd.init_weights(cfg, tdt, torch.device("cuda:0"))
    # the reference sees the very values the device holds (bf16 weights are rounded once)
    W_ref = {"wte": W_gpu["wte"].double().cpu(), "wpe": W_gpu["wpe"].double().cpu(),
             "layers": [{k: t.double().cpu() for k, t in L.items()} for L in W_gpu["layers"]]}
    ids = torch.randint(0, cfg.vocab, (B, N), generator=torch.Generator().manual_seed(5))
    got = bd.Decoder(cfg, W_gpu).forward(ids.cuda()).double().cpu().numpy()
    ref = bd.Decoder(cfg, W_ref, attention=_oracle_attention(cfg)).forward(ids).numpy()
    assert np.isfinite(got).all()
    rel = np.sqrt(((got - ref) ** 2).sum(-1)) / np.sqrt((ref ** 2).sum(-1))
    # fp32: fp32 GEMMs and LayerNorms over 128..256 terms, three layers.  bf16: every activation
    # is rounded to bf16 (2^-9) between ops, a dozen times per layer on the residual branch.
    bar = 2e-5 if dtype == "f32" else 3e-2
    assert float(rel.max()) <= bar, f"{dtype}: worst logit row rel-L2 {rel.max():.3e}"

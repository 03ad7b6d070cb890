"""Shapes and sizes of the synthetic workloads against what the paper prints."""
import os

import numpy as np
import pytest

from paper_2406_16793_amd import partition, workloads

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")

# counts derived by hand from the configuration text (tensors, params, blocks)
EXPECTED = {
    "tiny": (19, 2_098_432, 5_653),
    "gpt2_small": (99, 124_373_760, 115_130),
    "llama2_7b": (291, 6_738_415_616, 1_163_841),
    "llama3_8b": (291, 8_030_261_248, 1_470_273),
    "llama2_13b": (363, 13_015_864_320, 1_787_601),
}


@pytest.mark.parametrize("name", list(EXPECTED))
def test_counts(name):
    wl = workloads.get(name)
    assert (len(wl.specs), wl.n_params, wl.n_blocks) == EXPECTED[name]
    for s in wl.specs:
        assert s.numel % s.block_numel == 0


def test_table1_memory():
    """Table 1 (Section 2.4): the paper quotes parameter counts rounded to 0.01 B,
    times 8 bytes for AdamW; Adam-mini is half of it because v shrinks by >= 99.9 %."""
    with open(os.path.join(GOLDEN, "table1_memory_gb.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    for name, adamw_gb, mini_gb in rows:
        wl = workloads.get(name)
        billions = round(wl.n_params / 1e9, 2)
        assert abs(billions * 8 - float(adamw_gb)) < 5e-3
        mini_bytes = 4 * wl.n_params + 4 * wl.n_blocks
        assert abs(mini_bytes / 1e9 - float(mini_gb)) < 0.02
        # Section 2.3: >= 99.9 % of Adam's v removed on mainstream LLM shapes
        assert wl.n_blocks / wl.n_params <= 1e-3


def test_block_shapes_follow_partition_rules():
    wl = workloads.get("llama3_8b")
    by_name = {s.name: s for s in wl.specs}
    assert by_name["embed.weight"].block_numel == 4096                     # by token
    assert by_name["output.weight"].block_numel == 4096
    assert by_name["layers.0.attn.query.weight"].block_numel == 128 * 4096  # by head
    assert by_name["layers.0.attn.query.weight"].n_blocks == 32
    assert by_name["layers.0.attn.key.weight"].n_blocks == 8               # per KV head
    assert by_name["layers.0.attn.value.weight"].n_blocks == 1024          # by output neuron
    assert by_name["layers.0.attn.proj.weight"].block_numel == 4096
    assert by_name["layers.0.mlp.down.weight"].block_numel == 14336
    assert by_name["layers.0.norm1.weight"].n_blocks == 1                  # whole tensor
    assert by_name["layers.0.norm1.weight"].wd_scale == 0.0
    whole = partition.partition_whole([(s.name, s.shape) for s in wl.specs[:5]])
    assert all(s.n_blocks == 1 for s in whole)
    assert all(s.block_numel == 1 for s in partition.as_adamw(wl.specs[:5]))
    v2 = partition.block_numel_for("layers.0.attn.value.weight", (1024, 4096), 32, 8, value_whole=True)
    assert v2 == 1024 * 4096


def test_gradients_are_seeded_and_shaped():
    import torch
    wl = workloads.get("tiny")
    k = 0
    spec = wl.specs[k]
    a = torch.empty(spec.numel, dtype=torch.float32)
    b = torch.empty(spec.numel, dtype=torch.float32)
    workloads.fill_grad(a, spec, wl, k, 3)
    workloads.fill_grad(b, spec, wl, k, 3)
    assert torch.equal(a, b)
    workloads.fill_grad(b, spec, wl, k, 4)
    assert not torch.equal(a, b)
    rows = a.view(spec.shape)
    zero_rows = (rows == 0).all(dim=1)
    assert bool(zero_rows[0]) and 0.03 < zero_rows.float().mean() < 0.2     # ~10 % of embedding rows
    rms = rows[~zero_rows].pow(2).mean(dim=1).sqrt().log()
    assert abs(float(rms.mean()) - np.log(1e-3)) < 0.2 and 0.8 < float(rms.std()) < 1.2
    # bf16 output is the round-to-nearest-even of the same fp32 draw
    wl2 = workloads.get("llama2_7b")
    spec2 = partition.TensorSpec("layers.0.attn.value.weight", (8, 64), 64)
    h = torch.empty(spec2.numel, dtype=torch.bfloat16)
    f = torch.empty(spec2.numel, dtype=torch.float32)
    workloads.fill_grad(h, spec2, wl2, 5, 1)
    workloads.fill_grad(f, spec2, wl2, 5, 1)
    assert torch.equal(h, f.to(torch.bfloat16))


def test_partition_rules_on_common_parameter_names():
    """Algorithm 3's keywords plus the spellings of widely used checkpoints."""
    f = partition.block_numel_for
    d, h, kv, ff, vocab = 512, 8, 2, 1376, 1000
    hd = d // h
    cases = [
        ("model.embed_tokens.weight", (vocab, d), d),                      # by token
        ("lm_head.weight", (vocab, d), d),
        ("model.layers.3.self_attn.q_proj.weight", (d, d), hd * d),        # by head
        ("model.layers.3.self_attn.k_proj.weight", (kv * hd, d), hd * d),  # by KEY head (GQA)
        ("model.layers.3.self_attn.v_proj.weight", (kv * hd, d), d),       # by output neuron
        ("model.layers.3.self_attn.o_proj.weight", (d, d), d),
        ("model.layers.3.mlp.gate_proj.weight", (ff, d), d),
        ("model.layers.3.mlp.down_proj.weight", (d, ff), ff),
        ("model.layers.3.input_layernorm.weight", (d,), d),                # whole tensor
        ("model.norm.weight", (d,), d),
        ("layers.0.attention.wq.weight", (d, d), hd * d),
        ("layers.0.attention.wk.weight", (kv * hd, d), hd * d),
        ("layers.0.attention.wo.weight", (d, d), d),
        ("layers.0.feed_forward.w2.weight", (d, ff), ff),
        ("tok_embeddings.weight", (vocab, d), d),
        ("output.weight", (vocab, d), d),
        ("some.conv.kernel", (16, 3, 3, 3), 16 * 27),                      # no rule: one block
    ]
    for name, shape, want in cases:
        assert f(name, shape, n_heads=h, n_kv_heads=kv) == want, name
    with pytest.raises(ValueError):
        f("attn.query.weight", (d + 1, d), n_heads=h)
    t = partition.transposed(partition.TensorSpec("embed.weight", (vocab, d), d))
    assert t.shape == (d, vocab) and t.block_numel == d and t.strided and t.n_blocks == vocab
    with pytest.raises(ValueError):
        partition.transposed(partition.TensorSpec("q", (d, d), hd * d))

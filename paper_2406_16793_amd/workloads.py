"""Seeded synthetic workloads: tensor lists of the benchmark configurations and
the gradient / parameter generators that feed BOTH the HIP library and the CPU
oracle.  Nothing of the optimizer's arithmetic lives here.

The paper trains on OpenWebText / C4 (Section 3, Appendix D); an optimizer step
only sees tensor shapes and gradient statistics, so seeded synthetic tensors of
the published model shapes stand in for those runs.  Gradient rows differ in
scale because all entries of a row of dL/dW share one back-propagated error term
(Appendix C, "Why using average v as learning rates").

Recipe (per tensor k, step t, all from torch.Generator(seed ^ hash(k, t))):
    sigma_r = exp(N(ln 1e-3, 1)) per outermost-dimension row r
    g[r,:]  = sigma_r * N(0,1)                      ("normal")
            = sigma_r * N(0,1) / sqrt(chi2_3 / 3)   ("student_t3", heavy tails)
    embedding tensors: each row is all-zero with probability zero_row_prob,
    row 0 always (tokens absent from the batch), when zero_row_prob > 0
    bf16 gradients: drawn in fp32, rounded to nearest-even once.
    params: N(0, 0.02^2) for matrices, 1.0 for 1-D gains; m = v = 0.
Values are generated on ONE device and copied to the other side, never drawn
twice (host and device generators differ).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

from .partition import TensorSpec, partition_transformer

SEED_BASE = 0xAD4A0000


@dataclass
class Workload:
    name: str
    config_id: int
    specs: List[TensorSpec]
    grad_dtype: str                 # "f32" | "bf16"
    steps: int
    grad_dist: str = "normal"       # "normal" | "student_t3"
    zero_row_prob: float = 0.0      # applied to tensors listed in zero_row_tensors
    zero_row_tensors: Tuple[int, ...] = ()
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.95
    eps: float = 1e-8
    weight_decay: float = 0.1
    rtol: float = 1e-5

    @property
    def seed(self) -> int:
        return SEED_BASE + self.config_id

    @property
    def n_params(self) -> int:
        return sum(s.numel for s in self.specs)

    @property
    def n_blocks(self) -> int:
        return sum(s.n_blocks for s in self.specs)

    def algorithmic_bytes_per_step(self) -> int:
        """read g + read/write m + read/write param, plus read/write of each v scalar."""
        gb = 2 if self.grad_dtype == "bf16" else 4
        return self.n_params * (gb + 16) + 8 * self.n_blocks


def _llama_shapes(n_layers, d_model, n_heads, n_kv_heads, d_ff, vocab, gated=True, tied=False):
    hd = d_model // n_heads
    names = [("embed.weight", (vocab, d_model))]
    for i in range(n_layers):
        p = "layers.%d." % i
        names += [(p + "attn.query.weight", (n_heads * hd, d_model)),
                  (p + "attn.key.weight", (n_kv_heads * hd, d_model)),
                  (p + "attn.value.weight", (n_kv_heads * hd, d_model)),
                  (p + "attn.proj.weight", (d_model, n_heads * hd))]
        if gated:
            names += [(p + "mlp.gate.weight", (d_ff, d_model)), (p + "mlp.up.weight", (d_ff, d_model)),
                      (p + "mlp.down.weight", (d_model, d_ff))]
        else:
            names += [(p + "mlp.up.weight", (d_ff, d_model)), (p + "mlp.down.weight", (d_model, d_ff))]
        names += [(p + "norm1.weight", (d_model,)), (p + "norm2.weight", (d_model,))]
    names.append(("final_norm.weight", (d_model,)))
    if not tied:
        names.append(("output.weight", (vocab, d_model)))
    return names


def _embedding_indices(specs: Sequence[TensorSpec]) -> Tuple[int, ...]:
    return tuple(i for i, s in enumerate(specs) if s.name.startswith("embed"))


def tiny() -> Workload:
    """Config 1: 2 layers, d_model 256, 4 heads (head_dim 64), MLP 1024 (not gated),
    vocab 1024, untied embedding/output, RMSNorm gains; fp32 grads; 10 % zero
    embedding rows; 10 steps.  19 tensors, 2,098,432 params, 5,653 blocks."""
    specs = partition_transformer(_llama_shapes(2, 256, 4, 4, 1024, 1024, gated=False), n_heads=4)
    return Workload("tiny", 1, specs, "f32", 10, zero_row_prob=0.10, zero_row_tensors=_embedding_indices(specs))


def gpt2_small() -> Workload:
    """Config 2: GPT-2-small shape, 12 layers, d_model 768, 12 heads, MLP 3072,
    vocab 50304, tied embedding split by token; fused QKV passed as three 768x768
    tensors; plus (not fixed by the configuration, chosen here) a learned 1024x768
    position table and 25 LayerNorm gains as whole-tensor blocks, no biases.
    fp32 grads; 20 steps.  99 tensors, 124,373,760 params, 115,130 blocks."""
    names = [("embed.wte.weight", (50304, 768)), ("wpe.weight", (1024, 768))]
    for i in range(12):
        p = "h.%d." % i
        names += [(p + "attn.query.weight", (768, 768)), (p + "attn.key.weight", (768, 768)),
                  (p + "attn.value.weight", (768, 768)), (p + "attn.proj.weight", (768, 768)),
                  (p + "mlp.fc.weight", (3072, 768)), (p + "mlp.proj.weight", (768, 3072)),
                  (p + "ln_1.weight", (768,)), (p + "ln_2.weight", (768,))]
    names.append(("ln_f.weight", (768,)))
    specs = partition_transformer(names, n_heads=12)
    return Workload("gpt2_small", 2, specs, "f32", 20, zero_row_prob=0.10,
                    zero_row_tensors=_embedding_indices(specs))


def gpt2_small_bf16() -> Workload:
    """GPT-2-small shape with bf16 gradients (an extra configuration, not one of the five benchmark ones): its 64x768 query / key
    head blocks carry 96 KB of gradient each, the case served by the LDS-staged kernel."""
    wl = gpt2_small()
    wl.name, wl.config_id, wl.grad_dtype, wl.rtol = "gpt2_small_bf16", 6, "bf16", 5e-3
    return wl


def gpt2_small_whole() -> Workload:
    """GPT-2-small tensors under the paper's "Partition for non-Transformers" (Appendix B):
    every tensor is ONE block (38.6 M elements for the embedding), fp32 gradients.  Not one of the
    five benchmark configurations; it exercises the multi-workgroup path on whole-tensor blocks."""
    from .partition import partition_whole
    wl = gpt2_small()
    wl.specs = partition_whole([(s.name, s.shape) for s in wl.specs])
    wl.name, wl.config_id, wl.steps = "gpt2_small_whole", 7, 5
    return wl


def llama2_7b_whole() -> Workload:
    """Llama-2-7B tensors with every tensor as ONE block ("Partition for non-Transformers" applied
    to a large model: blocks of 16.8 M to 131 M elements), bf16 gradients.  Not one of the five
    benchmark configurations; everything goes through the multi-workgroup path."""
    from .partition import partition_whole
    wl = llama2_7b()
    wl.specs = partition_whole([(s.name, s.shape) for s in wl.specs])
    wl.name, wl.config_id, wl.steps = "llama2_7b_whole", 11, 3
    return wl


def llama2_7b_value_whole() -> Workload:
    """Llama-2-7B shape with the appendix's value "strategy II": each value matrix is one
    16.8 M-element block instead of 4096 row blocks.  Not one of the five benchmark configurations."""
    specs = partition_transformer(_llama_shapes(32, 4096, 32, 32, 11008, 32000), n_heads=32, value_whole=True)
    return Workload("llama2_7b_value_whole", 8, specs, "bf16", 5, rtol=5e-3)


def llama2_7b_lora() -> Workload:
    """Rank-128 LoRA adapters on the seven linear maps of every Llama-2-7B layer: 448 small
    matrices A [128, in] and B [out, 128], partitioned by output neuron (rows of 4096 / 11008 /
    128 elements), no weight decay, bf16 gradients.  Not one of the five benchmark configurations; it stresses
    the multi-tensor packing and launch overhead rather than bandwidth."""
    r, d, f = 128, 4096, 11008
    names = []
    for i in range(32):
        pre = "layers.%d." % i
        for nm, (out_f, in_f) in (("attn.query", (d, d)), ("attn.key", (d, d)), ("attn.value", (d, d)),
                                  ("attn.proj", (d, d)), ("mlp.gate", (f, d)), ("mlp.up", (f, d)),
                                  ("mlp.down", (d, f))):
            names.append((pre + nm + ".lora_A.mlp", (r, in_f)))     # "mlp" keyword: split by output neuron
            names.append((pre + nm + ".lora_B.mlp", (out_f, r)))
    specs = [TensorSpec(n, tuple(sh), sh[1], 0.0) for n, sh in names]
    return Workload("llama2_7b_lora", 9, specs, "bf16", 5, weight_decay=0.0, rtol=5e-3)


def llama2_7b_embed_t() -> Workload:
    """Llama-2-7B shape whose embedding and output matrices are stored transposed ([4096, 32000]),
    so their per-token blocks are the columns of the stored matrix (the re-ordering case of the
    paper's Appendix D).  Not one of the five benchmark configurations."""
    from .partition import transposed
    wl = llama2_7b()
    wl.specs = [transposed(s) if (s.name.startswith("embed") or s.name.startswith("output")) else s
                for s in wl.specs]
    wl.name, wl.config_id, wl.steps = "llama2_7b_embed_t", 10, 5
    return wl


def llama2_7b() -> Workload:
    """Config 3: 32 layers, d_model 4096, 32 heads (head_dim 128), SwiGLU MLP 11008,
    vocab 32000; fp32 params and m, bf16 grads; 10 steps.  291 tensors,
    6,738,415,616 params, 1,163,841 blocks."""
    specs = partition_transformer(_llama_shapes(32, 4096, 32, 32, 11008, 32000), n_heads=32)
    return Workload("llama2_7b", 3, specs, "bf16", 10, rtol=5e-3)


def llama3_8b() -> Workload:
    """Config 4: 32 layers, d_model 4096, 32 query heads / 8 key-value heads (key
    blocks per KV head, 128x4096), MLP 14336, vocab 128256; bf16 grads with 30 %
    zero embedding rows; 10 steps.  291 tensors, 8,030,261,248 params."""
    specs = partition_transformer(_llama_shapes(32, 4096, 32, 8, 14336, 128256), n_heads=32, n_kv_heads=8)
    return Workload("llama3_8b", 4, specs, "bf16", 10, zero_row_prob=0.30,
                    zero_row_tensors=_embedding_indices(specs), rtol=5e-3)


def llama2_13b() -> Workload:
    """Config 5: 40 layers, d_model 5120, 40 heads (head_dim 128), MLP 13824, vocab
    32000; fp32 params, m and grads (~156 GB resident); Student-t(3) grads with
    lognormal row scale; 5 steps.  363 tensors, 13,015,864,320 params."""
    specs = partition_transformer(_llama_shapes(40, 5120, 40, 40, 13824, 32000), n_heads=40)
    return Workload("llama2_13b", 5, specs, "f32", 5, grad_dist="student_t3")


WORKLOADS = {"tiny": tiny, "gpt2_small": gpt2_small, "gpt2_small_bf16": gpt2_small_bf16,
             "gpt2_small_whole": gpt2_small_whole, "llama2_7b_whole": llama2_7b_whole, "llama2_7b_value_whole": llama2_7b_value_whole,
             "llama2_7b_lora": llama2_7b_lora, "llama2_7b_embed_t": llama2_7b_embed_t, "llama2_7b": llama2_7b,
             "llama3_8b": llama3_8b, "llama2_13b": llama2_13b}


def get(name: str) -> Workload:
    return WORKLOADS[name]()


# ----------------------------------------------------------------------------
# value generators (torch, any device)
# ----------------------------------------------------------------------------
def _generator(device, seed: int, tensor: int, step: int):
    import torch
    g = torch.Generator(device=device)
    # one stream per (seed, tensor, step), folded into 63 bits
    g.manual_seed(((int(seed) * 1000003 + int(tensor)) * 1000003 + int(step)) & (2 ** 63 - 1))
    return g


def init_param(spec: TensorSpec, seed: int, tensor: int, device="cpu"):
    """fp32 initial parameter values of one tensor (flat)."""
    import torch
    if len(spec.shape) < 2:
        return torch.ones(spec.numel, dtype=torch.float32, device=device)
    gen = _generator(device, seed, tensor, 0)
    p = torch.empty(spec.numel, dtype=torch.float32, device=device)
    p.normal_(0.0, 0.02, generator=gen)
    return p


def fill_grad(out, spec: TensorSpec, wl: Workload, tensor: int, step: int, row_chunk: int = 0) -> None:
    """Write the gradient of (tensor, step) into `out` (flat torch tensor of
    spec.numel elements, float32 or bfloat16, on any device), in place."""
    import torch
    device = out.device
    gen = _generator(device, wl.seed, tensor, step)
    rows = int(spec.shape[0]) if len(spec.shape) >= 2 else 1
    cols = spec.numel // rows
    sigma = torch.empty(rows, dtype=torch.float32, device=device).normal_(generator=gen)
    sigma = torch.exp(sigma - 6.907755278982137)            # ln 1e-3
    if wl.zero_row_prob > 0.0 and tensor in wl.zero_row_tensors:
        keep = torch.rand(rows, dtype=torch.float32, device=device, generator=gen) >= wl.zero_row_prob
        keep[0] = False
        sigma = sigma * keep.to(torch.float32)
    # generate in row slabs so the fp32 temporaries stay small next to a bf16 output
    slab = rows if row_chunk <= 0 else row_chunk
    out2 = out.view(rows, cols)
    for r0 in range(0, rows, slab):
        r1 = min(rows, r0 + slab)
        z = torch.empty((r1 - r0, cols), dtype=torch.float32, device=device).normal_(generator=gen)
        if wl.grad_dist == "student_t3":
            chi = torch.zeros_like(z)
            for _ in range(3):
                n = torch.empty_like(z).normal_(generator=gen)
                chi.addcmul_(n, n)
            z.div_(torch.sqrt(chi / 3.0))
        z.mul_(sigma[r0:r1, None])
        out2[r0:r1].copy_(z)                                  # fp32 -> bf16 rounds to nearest even


def torch_grad_dtype(wl: Workload):
    import torch
    return torch.bfloat16 if wl.grad_dtype == "bf16" else torch.float32

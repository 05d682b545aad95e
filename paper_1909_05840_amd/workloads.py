"""Seeded synthetic inputs and the BERT tensor shapes they take.

This module holds no quantizer or matmul arithmetic: it only draws random tensors and lists
shapes, so that the HIP path and the CPU checker can be fed identical bytes.  Everything is
generated on the host with a seeded ``torch.Generator`` and returned as CPU tensors.

The paper evaluates BERT-base fine-tuned on SST-2, MNLI, CoNLL-03 and SQuAD (Sec. 4, App.
"Datasets"); those datasets and checkpoints are not used.  The tensors below only take BERT's
layer shapes (Sec. 3.3: d = 768, 12 heads of 64, 128 groups of 6 output neurons; Table 6 lists
7.1 M parameters per encoder layer and a 23.8 M embedding) and stand in for them.
"""
import torch

# (name, N = output neurons, K = input features)
BERT_BASE_LINEARS = (("qkv", 2304, 768), ("attn_out", 768, 768), ("ffn_up", 3072, 768), ("ffn_down", 768, 3072))
BERT_LARGE_LINEARS = (("qkv", 3072, 1024), ("attn_out", 1024, 1024), ("ffn_up", 4096, 1024), ("ffn_down", 1024, 4096))
BERT_BASE = {"hidden": 768, "heads": 12, "layers": 12, "linears": BERT_BASE_LINEARS}
BERT_LARGE = {"hidden": 1024, "heads": 16, "layers": 24, "linears": BERT_LARGE_LINEARS, "vocab": 30522}
WEIGHT_BITS = (2, 3, 4, 8)
GROUPS = 128
ACT_CLIP = 6.0

# Per-encoder-layer weight bits printed in the paper's appendix (Table 6: 2/3-bit mixed
# precision, Table 7: 2/4-bit mixed precision), encoder layers 1..12 in order.
PAPER_BITS_2_3 = {
    "SST-2": (2, 2, 2, 3, 3, 3, 3, 3, 3, 2, 2, 2),
    "MNLI": (2, 2, 2, 2, 3, 3, 3, 3, 2, 2, 2, 2),
    "CoNLL-03": (2, 3, 3, 3, 3, 2, 2, 2, 2, 2, 2, 2),
    "SQuAD": (2, 2, 2, 3, 3, 3, 3, 3, 3, 2, 2, 2),
}
PAPER_BITS_2_4 = {
    "SST-2": (2, 2, 4, 4, 4, 2, 4, 4, 4, 2, 2, 2),
    "MNLI": (2, 2, 2, 4, 4, 4, 4, 4, 2, 2, 2, 2),
    "CoNLL-03": (2, 2, 2, 4, 4, 4, 4, 4, 2, 2, 2, 2),
    "SQuAD": (2, 2, 2, 4, 4, 4, 4, 4, 2, 2, 2, 2),
}


def _gen(seed):
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    return g


def weight(N, K, seed, std=0.04, outlier_frac=0.001, outlier_scale=10.0):
    """fp32 master weight: N(0, std^2) with a fraction of entries multiplied by outlier_scale."""
    g = _gen(seed)
    W = torch.randn(N, K, generator=g, dtype=torch.float32) * std
    if outlier_frac > 0:
        mask = torch.rand(N, K, generator=g) < outlier_frac
        W = torch.where(mask, W * outlier_scale, W)
    return W.contiguous()


def weight_uniform(N, K, seed, lo=-1.0, hi=1.0):
    """Outlier-free tensor, uniform on [lo, hi): every code and packing position gets used."""
    g = _gen(seed)
    return (torch.rand(N, K, generator=g, dtype=torch.float32) * (hi - lo) + lo).contiguous()


def activation(T, K, seed, std=1.0):
    g = _gen(seed)
    return (torch.randn(T, K, generator=g, dtype=torch.float32) * std).contiguous()


def grad_output_bf16(T, N, seed, std=1e-2):
    """Upstream gradient as bfloat16; returned as a torch.bfloat16 CPU tensor."""
    g = _gen(seed)
    return (torch.randn(T, N, generator=g, dtype=torch.float32) * std).to(torch.bfloat16).contiguous()


def bf16_bits(t):
    """uint16 bit patterns (numpy) of a bfloat16 CPU tensor."""
    import numpy as np
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def layer_bits(n_layers, seed):
    """Stand-in for the Hessian-ranked assignment: one width per layer drawn from {2,3,4,8}."""
    g = _gen(seed)
    idx = torch.randint(0, len(WEIGHT_BITS), (n_layers,), generator=g)
    return tuple(WEIGHT_BITS[i] for i in idx.tolist())


def embedding_table(V, d, seed, std=0.02):
    g = _gen(seed)
    return (torch.randn(V, d, generator=g, dtype=torch.float32) * std).contiguous()


def token_ids(n, V, seed):
    g = _gen(seed)
    return torch.randint(0, V, (n,), generator=g, dtype=torch.int64)


def config_seed(config_index, tensor_index):
    """Seed rule: 1000*config + tensor; configuration 1 (index 0) starts at seed 0."""
    return 1000 * int(config_index) + int(tensor_index)

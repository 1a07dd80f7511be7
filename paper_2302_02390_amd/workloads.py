"""Seeded synthetic inputs and tensor shapes for the QSDP codec workloads.

This module holds no part of the method's arithmetic: only shapes of GPT-style
parameter vectors (Section 6.1 of the paper trains GPT models of 125M, 350M and
1.3B parameters) and random value generators. It is the one module that both the
GPU library's tests/benchmark and the CPU oracle's tests use.

Values stand in for trained weights and real gradients, which need the paper's
dataset and training run: weights ~ 0.02*N(0,1); gradients ~ 1e-3*N(0,1) or
1e-3*Student-t(nu=3) (heavy tails stretch a bucket's [min,max], the effect
bucketing is there to contain).
"""
from collections import namedtuple

import torch

VOCAB = 50257
N_CTX = 2048  # the paper does not state the context length; < 0.5 % of any size

GPTShape = namedtuple("GPTShape", "name layers d")
GPT_125M = GPTShape("gpt-125m", 12, 768)
GPT_350M = GPTShape("gpt-350m", 24, 1024)
GPT_1P3B = GPTShape("gpt-1.3b", 24, 2048)


def block_tensors(d):
    """(name, numel) of the tensors of one transformer block, in storage order."""
    return [
        ("ln1_w", d), ("ln1_b", d),
        ("qkv_w", 3 * d * d), ("qkv_b", 3 * d),
        ("proj_w", d * d), ("proj_b", d),
        ("ln2_w", d), ("ln2_b", d),
        ("fc_w", 4 * d * d), ("fc_b", 4 * d),
        ("fc2_w", 4 * d * d), ("fc2_b", d),
    ]


def block_numel(d):
    return sum(s for _, s in block_tensors(d))


def model_tensors(shape, n_ctx=N_CTX):
    """(name, numel) of every tensor of the model, in flat-vector order."""
    out = [("wte", VOCAB * shape.d), ("wpe", n_ctx * shape.d)]
    for layer in range(shape.layers):
        out += [(f"h{layer}.{name}", s) for name, s in block_tensors(shape.d)]
    out += [("ln_f_w", shape.d), ("ln_f_b", shape.d)]
    return out


def model_numel(shape, n_ctx=N_CTX):
    return sum(s for _, s in model_tensors(shape, n_ctx))


def _generator(device, seed):
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    return gen


def weights(n, seed, device="cpu", std=0.02):
    """fp32[n] ~ std * N(0,1)."""
    gen = _generator(device, seed)
    out = torch.empty(n, dtype=torch.float32, device=device)
    out.normal_(0.0, std, generator=gen)
    return out


def grads_normal(n, seed, device="cpu", std=1e-3):
    """fp32[n] ~ std * N(0,1)."""
    return weights(n, seed, device, std)


def grads_student_t3(n, seed, device="cpu", scale=1e-3, chunk=1 << 26):
    """fp32[n] ~ scale * t_3, built as N(0,1) / sqrt(chi2_3 / 3) chunk by chunk."""
    gen = _generator(device, seed)
    out = torch.empty(n, dtype=torch.float32, device=device)
    for s in range(0, n, chunk):
        m = min(chunk, n - s)
        z = torch.empty(m, dtype=torch.float32, device=device).normal_(generator=gen)
        chi = torch.zeros(m, dtype=torch.float32, device=device)
        for _ in range(3):
            w = torch.empty(m, dtype=torch.float32, device=device).normal_(generator=gen)
            chi.addcmul_(w, w)
        out[s:s + m] = z / torch.sqrt(chi / 3.0) * scale
        del z, chi, w
    return out

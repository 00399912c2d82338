"""Seeded tensor generators (torch CPU).  No attention arithmetic lives here."""
import numpy as np
import torch


def seq_len(scales):
    return int(sum(int(s) * int(s) for s in scales))


def _lq(scales, q_scales):
    if q_scales is None:
        return seq_len(scales)
    return int(sum(int(s) * int(s) for s in scales[q_scales[0]:q_scales[1]]))


def make_qkv(scales, batch, heads, head_dim, dtype, seed, input_scale=1.0, q_scales=None):
    """Q [B,H,Lq,D], K, V [B,H,L,D] as CPU torch tensors of `dtype` ("f32"|"bf16").

    Draws fp32 N(0,1) in the order Q, K, V from torch.Generator(seed), multiplies
    by input_scale, casts once.
    """
    g = torch.Generator(device="cpu").manual_seed(int(seed))
    L, Lq = seq_len(scales), _lq(scales, q_scales)
    q = torch.randn(batch, heads, Lq, head_dim, generator=g, dtype=torch.float32)
    k = torch.randn(batch, heads, L, head_dim, generator=g, dtype=torch.float32)
    v = torch.randn(batch, heads, L, head_dim, generator=g, dtype=torch.float32)
    if input_scale != 1.0:
        q, k, v = q * input_scale, k * input_scale, v * input_scale
    if dtype == "bf16":
        q, k, v = q.to(torch.bfloat16), k.to(torch.bfloat16), v.to(torch.bfloat16)
    elif dtype != "f32":
        raise ValueError(dtype)
    return q, k, v


def make_workload_qkv(w):
    return make_qkv(w.scales, w.batch, w.heads, w.head_dim, w.dtype, w.seed, w.input_scale,
                    w.q_scales)


def make_cfg_share(heads, n_scales, seed, p=0.5):
    """uint8 [H, K] table: 1 where the uncond rows reuse the cond output."""
    g = torch.Generator(device="cpu").manual_seed(int(seed) + 100)
    return (torch.rand(heads, n_scales, generator=g) < p).to(torch.uint8)


def make_attn_map(scales, n_samples, heads, seed, sigma=(0.05, 0.4), noise=0.3):
    """Synthetic post-softmax attention maps [N, H, L, L] (float32), standing in for the
    reference maps that the paper collects from training images: block-causal across
    scales, each row a noisy bump around the query's own image position (positions taken as
    cell centres in the unit square, so no part of the method's window arithmetic enters),
    head h with its own width between sigma[0] and sigma[1], every row normalised to sum 1."""
    g = np.random.default_rng(seed)
    pos, scale_of = [], []
    for k, s in enumerate(scales):
        c = (np.arange(s) + 0.5) / s
        yy, xx = np.meshgrid(c, c, indexing="ij")
        pos.append(np.stack([yy.ravel(), xx.ravel()], axis=1))
        scale_of.append(np.full(s * s, k))
    pos, scale_of = np.concatenate(pos), np.concatenate(scale_of)
    L = len(pos)
    d2 = ((pos[:, None, :] - pos[None, :, :]) ** 2).sum(-1)
    causal = scale_of[None, :] <= scale_of[:, None]
    out = np.empty((n_samples, heads, L, L), dtype=np.float32)
    for h in range(heads):
        sg = sigma[0] + (sigma[1] - sigma[0]) * (h / max(heads - 1, 1))
        base = np.exp(-d2 / (2 * sg * sg))
        for n in range(n_samples):
            w = base * np.exp(noise * g.standard_normal((L, L))) * causal
            out[n, h] = (w / w.sum(axis=1, keepdims=True)).astype(np.float32)
    return torch.from_numpy(out)


def bf16_bits(t):
    """numpy uint16 view of a CPU bf16 tensor's bit patterns (no copy of values)."""
    assert t.dtype == torch.bfloat16 and t.device.type == "cpu"
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def to_oracle_array(t):
    """What the oracle consumes for tensor t: f32 array or bf16 bit patterns."""
    if t.dtype == torch.bfloat16:
        return bf16_bits(t)
    return t.contiguous().numpy()

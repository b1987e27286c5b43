"""Seeded synthetic KV caches shaped like the paper's workloads.

Serves both the GPU library's tests/benchmark and the CPU oracle; it holds none of the
method's arithmetic (no quantization, packing or coding), only the input recipe:

  V ~ N(0, 1)
  K ~ N(0, 1) * s[layer, head, channel],  s ~ LogNormal(0, 1), and 4 of the head_dim
      channels of every (layer, head) multiplied by 20 (outlier channels)

stored as fp16 or bf16 in [layer][kv][head][token][dim] order (kv: 0 = K, 1 = V), or in
a vLLM-style paged pool [layer][kv][phys_block][block_tokens][head][dim] addressed through
a block table that is a seeded random permutation.  These stand in for the real-model KV
of the paper's evaluation (section 7.1), which needs weights and datasets that are not
available here.  Values depend on (seed, layer) and on the device type that draws them;
a test always feeds the same tensor to both sides.
"""
import torch

OUTLIER_CHANNELS = 4
OUTLIER_GAIN = 20.0


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def channel_scales(seed, layers, heads, head_dim, device="cpu"):
    """[layers, heads, head_dim] float32 K channel scales (always drawn on the CPU)."""
    g = _gen(seed * 1000003 + 17, "cpu")
    s = torch.exp(torch.randn(layers, heads, head_dim, generator=g))
    pick = torch.rand(layers, heads, head_dim, generator=g).argsort(dim=-1)[..., :OUTLIER_CHANNELS]
    gain = torch.ones(layers, heads, head_dim)
    gain.scatter_(-1, pick, OUTLIER_GAIN)
    return (s * gain).to(device)


def make_layer(seed, layer, scales_l, heads, head_dim, tokens, dtype, device):
    """One layer, [2, heads, tokens, head_dim]."""
    g = _gen(seed * 7919 + layer * 104729 + 1, device)
    x = torch.randn(2, heads, tokens, head_dim, generator=g, device=device, dtype=torch.float32)
    x[0] *= scales_l[:, None, :]
    return x.to(dtype)


def make_kv(seed, layers, heads, head_dim, tokens, dtype=torch.float16, device="cpu"):
    """Contiguous cache [layers, 2, heads, tokens, head_dim]."""
    out = torch.empty(layers, 2, heads, tokens, head_dim, dtype=dtype, device=device)
    s = channel_scales(seed, layers, heads, head_dim, device)
    for l in range(layers):
        out[l] = make_layer(seed, l, s[l], heads, head_dim, tokens, dtype, device)
    return out


def block_table(seed, num_blocks, num_phys_blocks=None, device="cpu"):
    """Seeded random permutation of the physical blocks (first num_blocks entries), int32."""
    num_phys_blocks = num_phys_blocks or num_blocks
    g = _gen(seed * 31 + 5, "cpu")
    return torch.randperm(num_phys_blocks, generator=g)[:num_blocks].to(torch.int32).to(device)


def to_paged(x, table, block_tokens, num_phys_blocks):
    """Scatter a contiguous cache [L, 2, H, T, D] into a pool [L, 2, P, block_tokens, H, D]."""
    L, two, H, T, D = x.shape
    nb = -(-T // block_tokens)
    pool = torch.zeros(L, two, num_phys_blocks, block_tokens, H, D, dtype=x.dtype, device=x.device)
    idx = table.to(torch.int64).to(x.device)
    for l in range(L):
        xl = x[l]
        if nb * block_tokens != T:
            pad = torch.zeros(two, H, nb * block_tokens - T, D, dtype=x.dtype, device=x.device)
            xl = torch.cat([xl, pad], dim=2)
        xl = xl.reshape(two, H, nb, block_tokens, D).permute(0, 2, 3, 1, 4)
        pool[l, :, idx] = xl
    return pool


def from_paged(pool, table, tokens):
    """Gather a pool back into the contiguous order [L, 2, H, tokens, D]."""
    L, two, P, bt, H, D = pool.shape
    idx = table.to(torch.int64).to(pool.device)
    x = pool[:, :, idx]                                   # [L, 2, nb, bt, H, D]
    x = x.permute(0, 1, 4, 2, 3, 5).reshape(L, two, H, -1, D)
    return x[:, :, :, :tokens].contiguous()


def make_paged(seed, layers, heads, head_dim, tokens, dtype=torch.float16, device="cpu",
               block_tokens=16, num_phys_blocks=None):
    """Paged cache built layer by layer (never holds a second full copy). Returns (pool, table)."""
    nb = -(-tokens // block_tokens)
    num_phys_blocks = num_phys_blocks or nb
    table = block_table(seed, nb, num_phys_blocks, device)
    pool = torch.zeros(layers, 2, num_phys_blocks, block_tokens, heads, head_dim, dtype=dtype,
                       device=device)
    s = channel_scales(seed, layers, heads, head_dim, device)
    idx = table.to(torch.int64)
    for l in range(layers):
        xl = make_layer(seed, l, s[l], heads, head_dim, nb * block_tokens, dtype, device)
        if nb * block_tokens != tokens:
            xl[:, :, tokens:] = 0
        pool[l, :, idx] = xl.reshape(2, heads, nb, block_tokens, head_dim).permute(0, 2, 3, 1, 4)
    return pool, table


def request_lengths(seed, n, lo, hi):
    """n integer lengths uniform in [lo, hi]."""
    g = _gen(seed * 131 + 3, "cpu")
    return [int(v) for v in torch.randint(lo, hi + 1, (n,), generator=g)]


def as_u16(x):
    """Bit patterns of a 16-bit float CPU tensor as a numpy uint16 array (shares memory)."""
    import numpy as np
    return x.view(torch.int16).numpy().view(np.uint16)

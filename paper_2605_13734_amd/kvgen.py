"""Seeded synthetic KV caches shaped like the paper's workloads.

Serves both the GPU library's tests/benchmark and the CPU oracle; it holds none of the
method's arithmetic (no quantization, packing or coding), only the input recipe:

  V ~ N(0, 1)
  K ~ N(0, 1) * s[layer, head, channel],  s ~ LogNormal(0, 1), and 4 of the head_dim
      channels of every (layer, head) multiplied by 20 (outlier channels)

The normal variates come from a counter-based generator: element (layer, kv, head, token,
channel) of seed s is a function of those six numbers alone -- two rounds of a 64-bit integer
mixer give 16 bytes whose sum, centred and scaled, is the variate (a sum of 16 uniform bytes:
mean 0, variance 1, tails to +-6.9) -- in integer arithmetic and single IEEE float32
operations only.  So a tensor does not depend on the device that makes it or on its length: a
shorter sequence is the prefix of a longer one, and the benchmark's inputs can be rebuilt anywhere.

stored as fp16 or bf16 in [layer][kv][head][token][dim] order (kv: 0 = K, 1 = V), or in
a vLLM-style paged pool [layer][kv][phys_block][block_tokens][head][dim] addressed through
a block table that is a seeded random permutation.  These stand in for the real-model KV
of the paper's evaluation (section 7.1), which needs weights and datasets that are not
available here.  A test always feeds the same tensor to both sides.
"""
import torch

OUTLIER_CHANNELS = 4
OUTLIER_GAIN = 20.0


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def channel_scales(seed, layers, heads, head_dim, device="cpu"):
    """[layers, heads, head_dim] float32 K channel scales (always computed on the CPU, from the
    (layer, head, channel) numbers alone)."""
    idx = torch.arange(layers * heads * head_dim, dtype=torch.int64).reshape(layers, heads, head_dim)
    s = torch.exp(normal_at(seed * 1000003 + 17, idx))
    pick = _mix(idx + _s64(int(seed) * 0xD1B54A32D192ED03 + 29)).argsort(dim=-1)[..., :OUTLIER_CHANNELS]
    gain = torch.ones(layers, heads, head_dim)
    gain.scatter_(-1, pick, OUTLIER_GAIN)
    return (s * gain).to(device)


def _s64(v):
    """A 64-bit pattern as the signed integer torch's int64 holds."""
    v &= (1 << 64) - 1
    return v - (1 << 64) if v >> 63 else v


def _mix(z):
    """One round of a 64-bit finalizer (xor-shifts and odd multipliers; int64 arithmetic wraps)."""
    z = (z ^ ((z >> 30) & ((1 << 34) - 1))) * _s64(0xBF58476D1CE4E5B9)
    z = (z ^ ((z >> 27) & ((1 << 37) - 1))) * _s64(0x94D049BB133111EB)
    return z ^ ((z >> 31) & ((1 << 33) - 1))


def _byte_sum(h):
    """Sum of the eight bytes of every int64 of h."""
    x = (h & 0x00FF00FF00FF00FF) + ((h >> 8) & 0x00FF00FF00FF00FF)
    x = (x & 0x0000FFFF0000FFFF) + ((x >> 16) & 0x0000FFFF0000FFFF)
    return (x & 0xFFFFFFFF) + ((x >> 32) & 0xFFFFFFFF)


_IH_MEAN = 16 * 127.5
_IH_STD = (16 * (256.0 ** 2 - 1) / 12) ** 0.5


def normal_at(seed, index):
    """float32 variates for the int64 element numbers `index` (any shape, any device)."""
    h = _mix(index + _s64(int(seed) * 0x9E3779B97F4A7C15 + 0x632BE59BD9B4E019))
    total = _byte_sum(h) + _byte_sum(_mix(h + _s64(0x9E3779B97F4A7C15)))
    return (total - int(_IH_MEAN)).to(torch.float32) * torch.tensor(1.0 / _IH_STD, dtype=torch.float32).item()


def make_layer(seed, layer, scales_l, heads, head_dim, tokens, dtype, device, first_token=0):
    """One layer, [2, heads, tokens, head_dim]."""
    lead = (layer * 2 + torch.arange(2, device=device, dtype=torch.int64)[:, None] ) * heads \
        + torch.arange(heads, device=device, dtype=torch.int64)[None, :]                          # [2, heads]
    inner = torch.arange(first_token * head_dim, (first_token + tokens) * head_dim, device=device, dtype=torch.int64)
    x = normal_at(seed, (lead << 39)[:, :, None] + inner[None, None, :]).reshape(2, heads, tokens, head_dim)
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

"""Seeded synthetic inputs shaped like the paper's Open-Sora-2.0 workloads.

The paper evaluates on activations of Open-Sora 1.0 / 2.0 (Sec. 4.1; 3072
channels, tokens = latent frames x spatial positions).  Neither the models nor
their activations are available, so these generators stand in for them: same
shapes, heavy tails, per-frame scale drift and a few outlier channels (the
"channel-wise outliers" of Sec. 3.3).  This module holds no quantizer
arithmetic; the CPU oracle and the GPU library both consume what it returns.

Every tensor is generated in fp32 with torch's generator on the requested
device, in fixed 1024-row chunks each seeded from (seed, chunk index), then
rounded to bf16 (round-to-nearest-even).  A tensor generated with fewer rows
is therefore a prefix of the full one.  Values depend on the device type (CPU
and GPU generators differ); whoever generates a tensor hands the same bits to
both the oracle and the library.
"""

import math

import numpy as np
import torch

from .formatbook import range_buckets

CHUNK_ROWS = 1024

# name -> (rows, cols)
CONFIG_SHAPES = {
    "cfg1": (1024, 3072),
    "cfg2": (16384, 3072),
    "cfg3": (16384, 3072),
    "cfg4": (16384, 3072),
    "cfg5": (65536, 12288),
    "cfg5_weight": (12288, 3072),
}


def _gen(device, seed, chunk):
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1000003 + int(chunk)) & 0x7FFFFFFFFFFFFFFF)
    return g


def _student_t3(shape, device, g):
    z = torch.randn(shape, device=device, generator=g)
    chi = torch.zeros(shape, device=device)
    for _ in range(3):
        n = torch.randn(shape, device=device, generator=g)
        chi.addcmul_(n, n)
    return z * torch.rsqrt(chi / 3.0)


def _outlier_channels(cols, frac, seed):
    """floor(frac*cols) distinct channel indices, drawn on the CPU so they do
    not depend on the device."""
    k = int(math.floor(frac * cols))
    rng = np.random.default_rng([int(seed), 0xC0])
    return np.sort(rng.choice(cols, size=k, replace=False))


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor -> uint16 numpy array of its bit patterns (host copy)."""
    assert t.dtype == torch.bfloat16
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def bits_to_bf16(bits: np.ndarray, device="cpu") -> torch.Tensor:
    """uint16 bit patterns -> bf16 tensor on device."""
    a = np.ascontiguousarray(bits, dtype=np.uint16).view(np.int16)
    return torch.from_numpy(a).view(torch.bfloat16).to(device)


def gaussian_outlier(rows=1024, cols=3072, seed=1, device="cpu"):
    """cfg1: N(0,1), 1 % of the channels scaled by 50."""
    out = torch.empty((rows, cols), dtype=torch.bfloat16, device=device)
    ch = torch.from_numpy(_outlier_channels(cols, 0.01, seed)).to(device)
    for c, r0 in enumerate(range(0, rows, CHUNK_ROWS)):
        r1 = min(rows, r0 + CHUNK_ROWS)
        g = _gen(device, seed, c)
        x = torch.randn((CHUNK_ROWS, cols), device=device, generator=g)[: r1 - r0]
        x[:, ch] *= 50.0
        out[r0:r1] = x.to(torch.bfloat16)
    return out


def vdit_activation(rows=16384, cols=3072, seed=2, device="cpu",
                    outlier_frac=0.005, outlier_scale=100.0, frame_rows=1024):
    """cfg2 / cfg3 / cfg5: Student-t (nu=3) elements, one scale per latent
    frame drawn from U[0.5, 2], outlier channels scaled by 100."""
    out = torch.empty((rows, cols), dtype=torch.bfloat16, device=device)
    ch = torch.from_numpy(_outlier_channels(cols, outlier_frac, seed)).to(device)
    n_frames = (rows + frame_rows - 1) // frame_rows
    frng = np.random.default_rng([int(seed), 0xF0])
    fscale = torch.from_numpy(frng.uniform(0.5, 2.0, size=max(n_frames, 1)).astype(np.float32)).to(device)
    for c, r0 in enumerate(range(0, rows, CHUNK_ROWS)):
        r1 = min(rows, r0 + CHUNK_ROWS)
        g = _gen(device, seed, c)
        x = _student_t3((CHUNK_ROWS, cols), device, g)[: r1 - r0]
        frame = torch.arange(r0, r1, device=device) // frame_rows
        x *= fscale[frame][:, None]
        x[:, ch] *= outlier_scale
        out[r0:r1] = x.to(torch.bfloat16)
    return out


def mixture_activation(rows=16384, cols=3072, seed=4, device="cpu", n_components=64):
    """cfg4: every token belongs to one of 64 Gaussian components (its
    semantic group): x = mu_c[channel] + sigma_c * N(0,1).  Returns the tensor
    and the int32 component index of every row."""
    prng = np.random.default_rng([int(seed), 0xA0])
    mu = torch.from_numpy(prng.standard_normal((n_components, cols)).astype(np.float32)).to(device)
    sigma = torch.from_numpy(prng.uniform(0.5, 2.0, size=n_components).astype(np.float32)).to(device)
    comp_np = prng.integers(0, n_components, size=rows).astype(np.int32)
    comp = torch.from_numpy(comp_np).to(device)
    out = torch.empty((rows, cols), dtype=torch.bfloat16, device=device)
    for c, r0 in enumerate(range(0, rows, CHUNK_ROWS)):
        r1 = min(rows, r0 + CHUNK_ROWS)
        g = _gen(device, seed, c)
        z = torch.randn((CHUNK_ROWS, cols), device=device, generator=g)[: r1 - r0]
        k = comp[r0:r1].long()
        out[r0:r1] = (mu[k] + sigma[k][:, None] * z).to(torch.bfloat16)
    return out, comp_np


def seda_sub_formatbooks(formatbook, n_groups=64, seed=4):
    """Per group an 8-dialect sub-formatbook: one DID drawn uniformly from each
    dynamic-range bucket of the formatbook (Sec. 3.4), ascending.  uint8
    [n_groups][8]."""
    buckets = range_buckets(formatbook)
    rng = np.random.default_rng([int(seed), 0x5D])
    sub = np.zeros((n_groups, 8), dtype=np.uint8)
    for gidx in range(n_groups):
        for r in range(8):
            sub[gidx, r] = rng.choice(buckets[r])
    return sub


def layernorm_affine(cols=3072, seed=6):
    """Per-channel scale and shift of a LayerNorm in front of a quantized linear layer (in a DiT block the
    conditioning supplies them: gamma = 1 + scale, beta = shift): gamma = 1 + 0.1 N(0,1), beta = 0.1 N(0,1),
    float32 [cols] each."""
    prng = np.random.default_rng([int(seed), 0xB0])
    gamma = (1.0 + 0.1 * prng.standard_normal(cols)).astype(np.float32)
    beta = (0.1 * prng.standard_normal(cols)).astype(np.float32)
    return gamma, beta


def weight_matrix(rows=12288, cols=3072, seed=5, device="cpu", std=0.02):
    """cfg5 weight: N(0, std^2), blocks along the contiguous (reduction) dim."""
    out = torch.empty((rows, cols), dtype=torch.bfloat16, device=device)
    for c, r0 in enumerate(range(0, rows, CHUNK_ROWS)):
        r1 = min(rows, r0 + CHUNK_ROWS)
        g = _gen(device, seed + 7919, c)
        x = torch.randn((CHUNK_ROWS, cols), device=device, generator=g)[: r1 - r0]
        out[r0:r1] = (x * std).to(torch.bfloat16)
    return out


def salient_rows_from_attention(tokens, frac=0.05, heads=24, seed=3, device="cpu",
                                window=None, chunk=1024):
    """Synthetic stand-in for the attention-guided salient-token choice of
    Sec. 3.3: logits ~ N(0,1) per head, row softmax, summed over query rows
    and heads to a per-key score; the floor(frac*tokens) best keys (ties to the
    lower index) sorted ascending, int32.  With `window` set, a query attends
    only to the `window` keys of its own frame (used when tokens^2 logits are
    impractical).  Logits are generated and reduced chunk by chunk."""
    score = torch.zeros(tokens, dtype=torch.float64, device=device)
    for h in range(heads):
        if window is None:
            for c, r0 in enumerate(range(0, tokens, chunk)):
                r1 = min(tokens, r0 + chunk)
                g = _gen(device, seed * 131 + h, c)
                logits = torch.randn((chunk, tokens), device=device, generator=g)[: r1 - r0]
                score += torch.softmax(logits, dim=-1).sum(dim=0).double()
        else:
            for c, r0 in enumerate(range(0, tokens, window)):
                r1 = min(tokens, r0 + window)
                g = _gen(device, seed * 131 + h, c)
                logits = torch.randn((window, window), device=device, generator=g)[: r1 - r0, : r1 - r0]
                score[r0:r1] += torch.softmax(logits, dim=-1).sum(dim=0).double()
    n_sal = int(math.floor(frac * tokens))
    s = score.cpu().numpy()
    order = np.lexsort((np.arange(tokens), -s))  # by score descending, then index ascending
    return np.sort(order[:n_sal]).astype(np.int32)


def attention_qk(groups, tokens, dim, seed=7, device="cpu", salient_frac=0.03):
    """Synthetic query / key projections of one attention layer: bf16 [groups][tokens][dim] each, N(0, 1) with a
    common per-group direction mixed in (tokens of a frame resemble each other) and a few tokens per group with
    three times the norm (the ones an attention-guided choice should find)."""
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) * 7919 + 17)
    out = []
    for _ in range(2):
        x = torch.randn((groups, tokens, dim), device=device, generator=g)
        x += 0.5 * torch.randn((groups, 1, dim), device=device, generator=g)
        big = torch.rand((groups, tokens, 1), device=device, generator=g) < salient_frac
        x = torch.where(big, 3.0 * x, x)
        out.append(x.to(torch.bfloat16))
    return out[0], out[1]


def edge_case_tensor(cols=256, seed=11):
    """A small uint16 (bf16 bit pattern) tensor exercising the degenerate
    inputs: all-zero and all-negative-zero blocks, subnormals, values at and
    around the exponent clamps, +/-Inf, NaNs, a block of equal values, exact
    half-way points between integers, and a single huge outlier."""
    assert cols % 32 == 0 and cols >= 64
    rng = np.random.default_rng([int(seed), 0xED])
    rows = []

    def row(fill):
        r = np.empty(cols, dtype=np.uint16)
        r[:] = fill
        return r

    base = rng.standard_normal(cols).astype(np.float32)

    def f2b(a):
        u = np.asarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
        return (((u + 0x7FFF + ((u >> 16) & 1)) >> 16) & 0xFFFF).astype(np.uint16)

    rows.append(row(0x0000))                                   # all +0
    rows.append(row(0x8000))                                   # all -0
    r = f2b(base); r[::7] = 0x8000; rows.append(r)             # -0 scattered
    rows.append(rng.integers(0, 0x80, cols).astype(np.uint16))  # positive subnormals
    rows.append((rng.integers(0, 0x80, cols) | 0x8000).astype(np.uint16))  # negative subnormals
    r = rng.integers(0x0001, 0x0300, cols).astype(np.uint16)   # subnormals + tiniest normals
    r[1::2] |= 0x8000; rows.append(r)
    rows.append(rng.integers(0x0080, 0x0400, cols).astype(np.uint16))      # around lower clamp
    r = rng.integers(0x7E00, 0x7F80, cols).astype(np.uint16)   # largest finite
    r[::3] |= 0x8000; rows.append(r)
    r = f2b(base); r[5] = 0x7F80; r[40] = 0xFF80; rows.append(r)           # +/-Inf
    r = f2b(base); r[3] = 0x7FC0; r[33] = 0xFFC1; r[34] = 0x7F81; rows.append(r)  # NaNs
    r = row(0x7FC0); r[cols // 2:] = f2b(base)[cols // 2:]; rows.append(r)  # all-NaN blocks
    r = row(0x7FC0); r[7] = 0x3F80; r[39] = 0x7F80; rows.append(r)        # NaN + one value
    rows.append(row(0x3F80))                                   # all 1.0
    rows.append(row(0xC170))                                   # all -15.0
    half = (np.arange(cols) % 31).astype(np.float32) * 0.5     # exact k/2 grid, max 15
    rows.append(f2b(half))
    r = f2b(half); r[1::2] |= 0x8000; rows.append(r)
    r = f2b(base * 1e-3); r[17] = f2b(np.float32(3.0e4)); rows.append(r)   # one huge outlier
    r = f2b(base * 1e30); rows.append(r)
    r = f2b(base * 1e-30); rows.append(r)
    quarter = ((np.arange(cols) % 64).astype(np.float32) * 0.25)           # k/4 grid: bin midpoints
    rows.append(f2b(quarter))
    return np.stack(rows).astype(np.uint16)

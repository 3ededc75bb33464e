"""Seeded synthetic inputs for the codec (tests, smoke check and benchmark).

This module holds none of the codec's arithmetic: it only draws random numbers
and casts them to the storage formats, so that the CPU oracle and the HIP
library can be fed the same bytes.  The tensors stand in for the paper's real
workloads (BF16/FP8 model weights, consecutive BF16 checkpoints, FP8 K/V
caches, MXFP4 weights: Sec. 4.1 - 4.4), none of which ship with this
repository.

All casts are written with integer/float tensor ops so that they give the same
bytes on the CPU and on the GPU.  Random draws come from a torch.Generator on
the chosen device; the CPU and the GPU generator give different streams, so
one run must take both sides' input from the same device (and copy it).
"""
import math

import torch

FMT_BF16, FMT_FP8_E4M3, FMT_FP4_E2M1_MX = 1, 2, 3


# ----------------------------------------------------------------- casts

def bf16_bits(x):
    """float32 -> BF16 bit patterns (int16 tensor), round to nearest even."""
    b = x.contiguous().view(torch.int32)
    r = (b + 0x7FFF + ((b >> 16) & 1)) >> 16
    return r.to(torch.int16)


def bf16_to_f32(bits):
    return (bits.to(torch.int32) << 16).view(torch.float32)


def e4m3_bits(x):
    """float32 -> OCP FP8 E4M3 ("fn": bias 7, max 448, no inf) bytes, RNE, saturating."""
    x = x.contiguous().clamp(-448.0, 448.0)
    b = x.view(torch.int32)
    sign = (b >> 24) & 0x80
    mag = b & 0x7FFFFFFF
    # normal range: keep 3 mantissa bits of the float32 pattern, round half to even
    norm = ((mag + 0x7FFFF + ((mag >> 20) & 1)) >> 20) - ((127 - 7) << 3)
    # below 2^-6 the grid is uniform with step 2^-9
    sub = torch.round(x.abs() * 512.0).to(torch.int32)
    code = torch.where(x.abs() < 2.0 ** -6, sub, norm).clamp(0, 0x7E)
    return (sign | code).to(torch.uint8)


def e5m2_bits(x):
    """float32 -> FP8 E5M2 (bias 15, 2 mantissa bits, IEEE-like) bytes, RNE, saturating at 57344."""
    x = x.contiguous().clamp(-57344.0, 57344.0)
    b = x.view(torch.int32)
    sign = (b >> 24) & 0x80
    mag = b & 0x7FFFFFFF
    norm = ((mag + 0xFFFFF + ((mag >> 21) & 1)) >> 21) - ((127 - 15) << 2)
    sub = torch.round(x.abs() * 65536.0).to(torch.int32)          # below 2^-14 the grid is uniform with step 2^-16
    code = torch.where(x.abs() < 2.0 ** -14, sub, norm).clamp(0, 0x7B)
    return (sign | code).to(torch.uint8)


def mxfp4_bits(x):
    """float32 [.., 32*k] -> (packed E2M1 bytes, E8M0 scale bytes), OCP MX rule.

    One scale per 32 contiguous elements: 2^(floor(log2 amax) - 2); elements are
    RNE onto {0, .5, 1, 1.5, 2, 3, 4, 6}, saturating.  Element 2i is the low
    nibble of byte i."""
    flat = x.contiguous().reshape(-1, 32)
    amax = flat.abs().amax(dim=1)
    e = ((amax.view(torch.int32) >> 23) & 0xFF) - 127 - 2
    e = torch.where(amax > 0, e, torch.full_like(e, -127)).clamp(-127, 127)
    scale = (e + 127).to(torch.uint8)
    v = flat * torch.exp2(-e.to(torch.float32)).unsqueeze(1)
    code = e2m1_codes(v)
    code = code.reshape(-1, 2)
    packed = (code[:, 0] | (code[:, 1] << 4)).to(torch.uint8)
    return packed, scale


def e4m3_to_f32(bits):
    """OCP FP8 E4M3 bytes -> float32 (exact)."""
    b = bits.to(torch.int32)
    e, m = (b >> 3) & 0xF, b & 7
    mag = torch.where(e > 0, (1.0 + m.to(torch.float32) / 8.0) * torch.exp2((e - 7).to(torch.float32)), m.to(torch.float32) * 2.0 ** -9)
    return torch.where((b & 0x80) != 0, -mag, mag)


def e2m1_codes(v):
    """float32 -> E2M1 codes (sign in bit 3), RNE onto {0, .5, 1, 1.5, 2, 3, 4, 6}, saturating."""
    a = v.abs()
    code = torch.where(a < 1.0, torch.round(a * 2.0),
           torch.where(a < 2.0, 2.0 + torch.round((a - 1.0) * 2.0),
           torch.where(a < 4.0, 4.0 + torch.round(a - 2.0), 6.0 + torch.round((a - 4.0) * 0.5))))
    return code.clamp(0, 7).to(torch.int32) | ((v.contiguous().view(torch.int32) >> 28) & 0x8)


def nvfp4_bits(x):
    """float32 [.., 16*k] -> (packed E2M1 bytes, E4M3 scale bytes): one FP8 scale per 16 contiguous
    elements (Sec. 3.4).  The block scale is amax/6 divided by a per-tensor factor that maps the largest
    block scale to 448, cast to E4M3; the elements are RNE onto the E2M1 grid after division by the scale
    as stored.  Element 2i is the low nibble of byte i."""
    flat = x.contiguous().reshape(-1, 16)
    block = flat.abs().amax(dim=1) / 6.0
    tensor_scale = block.max().clamp_min(1e-30) / 448.0
    scale = e4m3_bits(block / tensor_scale)
    dec = e4m3_to_f32(scale) * tensor_scale
    v = torch.where(dec.unsqueeze(1) > 0, flat / dec.clamp_min(1e-30).unsqueeze(1), torch.zeros_like(flat))
    code = e2m1_codes(v).reshape(-1, 2)
    return (code[:, 0] | (code[:, 1] << 4)).to(torch.uint8), scale


# ------------------------------------------------------------- generators

def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _seed(config, index):
    return (config * 1000003 + index * 7919 + 12345) & 0x7FFFFFFF


def bf16_weight(n, device="cpu", seed=0, std=0.02):
    """Config 1: BF16 tensor of n values N(0, std)."""
    g = _gen(device, seed)
    return bf16_bits(torch.randn(n, generator=g, device=device) * std)


def fp8_weight(n, device="cpu", seed=0, std=0.02, outlier_frac=1e-3, outlier_gain=20.0):
    """Config 2: one FP8 weight tensor.  N(0, std), a Bernoulli(outlier_frac) subset
    scaled by outlier_gain, per-tensor scale mapping amax to 448, E4M3 RNE."""
    g = _gen(device, seed)
    x = torch.randn(n, generator=g, device=device) * std
    mask = torch.rand(n, generator=g, device=device) < outlier_frac
    x = torch.where(mask, x * outlier_gain, x)
    x = x * (448.0 / x.abs().max())
    return e4m3_bits(x)


def fp8_e5m2_weight(n, device="cpu", seed=0, std=0.02, outlier_frac=1e-3, outlier_gain=20.0):
    """The FP8 weight recipe of config 2 cast to E5M2 instead (per-tensor scale mapping amax to 57344)."""
    g = _gen(device, seed)
    x = torch.randn(n, generator=g, device=device) * std
    mask = torch.rand(n, generator=g, device=device) < outlier_frac
    x = torch.where(mask, x * outlier_gain, x)
    x = x * (57344.0 / x.abs().max())
    return e5m2_bits(x)


# per decoder layer of an 8B-class model: (name, rows, cols)
LAYER_8B = [("q", 4096, 4096), ("k", 4096, 1024), ("v", 4096, 1024), ("o", 4096, 4096),
            ("gate", 4096, 14336), ("up", 4096, 14336), ("down", 14336, 4096)]


def fp8_weight_set(n_layers=32, device="cpu", shrink=1, e5m2=False):
    """Config 2: yields (name, uint8 tensor) for every tensor of the set.
    shrink divides both matrix dimensions (tests use a reduced set); e5m2 casts to E5M2 instead of E4M3."""
    i = 0
    for layer in range(n_layers):
        for name, r, c in LAYER_8B:
            n = (r // shrink) * (c // shrink)
            yield "L%d.%s" % (layer, name), (fp8_e5m2_weight if e5m2 else fp8_weight)(n, device, _seed(2, i))
            i += 1


def mxfp4_weight(rows, cols, device="cpu", seed=0, std=0.015):
    """Config 3: one MXFP4 matrix -> (packed element bytes, scale bytes)."""
    g = _gen(device, seed)
    x = torch.randn(rows * cols, generator=g, device=device) * std
    return mxfp4_bits(x)


def nvfp4_weight(rows, cols, device="cpu", seed=0, std=0.015):
    """One NVFP4 matrix -> (packed element bytes, E4M3 scale bytes, one per 16 elements)."""
    g = _gen(device, seed)
    x = torch.randn(rows * cols, generator=g, device=device) * std
    return nvfp4_bits(x)


def bf16_checkpoint_pair(n, device="cpu", seed=0, std=0.02, step_std=1e-4):
    """Config 4: W0 ~ N(0, std) in BF16 and W1 = bf16(W0 + N(0, step_std))."""
    g = _gen(device, seed)
    w0 = bf16_bits(torch.randn(n, generator=g, device=device) * std)
    w1 = bf16_bits(bf16_to_f32(w0) + torch.randn(n, generator=g, device=device) * step_std)
    return w0, w1


def _kv_values(batch, heads, tokens, head_dim, device, seed):
    """(K, V) as float32, shape [batch, heads, tokens, head_dim]: V ~ N(0,1); K ~ N(0,1) with 4 fixed
    outlier channels per head at std 10 plus a slow drift 0.1*sin(t/512)."""
    g = _gen(device, seed)
    shape = (batch, heads, tokens, head_dim)
    v = torch.randn(shape, generator=g, device=device)
    k = torch.randn(shape, generator=g, device=device)
    sigma = torch.ones(heads, head_dim, device=device)
    for h in range(heads):
        ch = torch.randperm(head_dim, generator=g, device=device)[:4]
        sigma[h, ch] = 10.0
    t = torch.arange(tokens, device=device, dtype=torch.float32)
    k = k * sigma.view(1, heads, 1, head_dim) + 0.1 * torch.sin(t / 512.0).view(1, 1, tokens, 1)
    return k, v


def bf16_kv_pair(batch=4, heads=8, tokens=8192, head_dim=128, device="cpu", seed=0):
    """One layer's (K, V) cache in BF16 (int16 bit patterns), same distributions as fp8_kv_pair, unscaled."""
    k, v = _kv_values(batch, heads, tokens, head_dim, device, seed)
    return bf16_bits(k), bf16_bits(v)


def fp8_kv_pair(batch=4, heads=8, tokens=8192, head_dim=128, device="cpu", seed=0):
    """Config 5: one layer's (K, V) cache as E4M3 bytes, shape [batch, heads, tokens, head_dim].
    V ~ N(0,1).  K ~ N(0,1) with 4 fixed outlier channels per head at std 10 plus a slow
    drift 0.1*sin(t/512).  A scale per (batch, head) slice maps its amax to 448."""
    g = _gen(device, seed)
    shape = (batch, heads, tokens, head_dim)
    v = torch.randn(shape, generator=g, device=device)
    k = torch.randn(shape, generator=g, device=device)
    sigma = torch.ones(heads, head_dim, device=device)
    for h in range(heads):
        ch = torch.randperm(head_dim, generator=g, device=device)[:4]
        sigma[h, ch] = 10.0
    t = torch.arange(tokens, device=device, dtype=torch.float32)
    k = k * sigma.view(1, heads, 1, head_dim) + 0.1 * torch.sin(t / 512.0).view(1, 1, tokens, 1)
    out = []
    for x in (k, v):
        amax = x.abs().amax(dim=(2, 3), keepdim=True)
        out.append(e4m3_bits(x * (448.0 / amax)))
    return out[0], out[1]


def page_sample(n_pages, frac=0.25, device="cpu", seed=0):
    """Config 5: a seeded sample without replacement of page ids, in random order."""
    g = _gen(device, seed)
    k = int(math.floor(n_pages * frac))
    return torch.randperm(n_pages, generator=g, device=device)[:k].to(torch.int32)

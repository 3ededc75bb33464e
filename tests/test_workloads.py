"""The input generators: casts against torch's own, and the ratios the Gaussian
workloads must give (closed form), which also pins the oracle's stats."""
import math

import numpy as np
import torch

from oracle import zc_oracle as o
from paper_2508_19263_amd import workloads as wl


def test_bf16_cast_matches_torch():
    g = torch.Generator().manual_seed(0)
    x = torch.randn(200000, generator=g) * torch.exp2(torch.randint(-30, 30, (200000,), generator=g).float())
    assert torch.equal(wl.bf16_bits(x), x.to(torch.bfloat16).view(torch.int16))
    assert torch.equal(wl.bf16_to_f32(wl.bf16_bits(x)), x.to(torch.bfloat16).float())


def test_e4m3_cast_matches_torch_and_saturates():
    g = torch.Generator().manual_seed(1)
    x = torch.randn(300000, generator=g) * torch.exp2(torch.randint(-12, 9, (300000,), generator=g).float())
    x = x.clamp(-448, 448)
    assert torch.equal(wl.e4m3_bits(x), x.to(torch.float8_e4m3fn).view(torch.uint8))
    # every representable value maps to itself; ties go to even; overflow saturates
    allv = torch.arange(256, dtype=torch.uint8)
    keep = (allv & 0x7F) != 0x7F
    vals = allv.view(torch.float8_e4m3fn).float()[keep]
    assert torch.equal(wl.e4m3_bits(vals) & 0x7F, allv[keep] & 0x7F)
    assert wl.e4m3_bits(torch.tensor([1e9, -1e9, 464.0, 1.0625, 1.1875, 2.0 ** -10, 3 * 2.0 ** -10])).tolist() == \
        [0x7E, 0xFE, 0x7E, 0x38, 0x3A, 0x00, 0x02]


def test_mxfp4_cast():
    # block amax 6.0 -> shared exponent floor(log2 6) - 2 = 0 -> scale byte 127, values on the grid
    grid = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]
    x = torch.tensor(grid + [-v for v in grid] + [0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 7.0] + [0.0] * 8)
    packed, scale = wl.mxfp4_bits(x)
    assert scale.tolist() == [127]
    codes = []
    for b in packed.tolist():
        codes += [b & 0xF, b >> 4]
    assert codes[:8] == list(range(8)) and codes[8:16] == [8 + i for i in range(8)]
    # ties to even code: .25->0, .75->1.0(2), 1.25->1.0(2), 1.75->2.0(4), 2.5->2(4), 3.5->4(6), 5->4(6), 7->6(7)
    assert codes[16:24] == [0, 2, 2, 4, 4, 6, 6, 7]
    # scaling: amax 0.02 -> floor(log2 0.02) = -6 -> e = -8 -> byte 119; 0.02/2^-8 = 5.12 -> 6.0? no: 5.12 rounds to 6 (step 2: 4 or 6; 5.12 > 5)
    packed, scale = wl.mxfp4_bits(torch.tensor([0.02] + [0.0] * 31))
    assert scale.tolist() == [119] and packed[0].item() == 7


def gaussian_exponent_pmf(sigma, bias, ebits, mbits, scale=1.0):
    """P(exponent field = k) for x ~ N(0, sigma) after scaling and RNE to a format
    with the given bias: the binade [2^(k-bias), 2^(k+1-bias)) shifted down by half an ulp."""
    Phi = lambda t: 0.5 * (1 + math.erf(t / math.sqrt(2)))
    emax = (1 << ebits) - 1
    edges = []
    for k in range(emax + 2):
        if k == 0:
            edges.append(0.0)
        else:
            lo = 2.0 ** (max(k, 1) - bias)
            ulp_below = 2.0 ** (max(k - 1, 1) - bias - mbits)
            edges.append(lo - ulp_below / 2)
    pmf = []
    for k in range(emax + 1):
        hi = edges[k + 1] if k < emax else float("inf")
        pmf.append(2 * (Phi(hi / (sigma * scale)) - Phi(edges[k] / (sigma * scale))))
    return np.array(pmf)


def test_config1_bf16_ratios_match_closed_form():
    # Config 1: BF16, N(0, 0.02).  The exponent histogram follows from the normal CDF; the
    # optimal code for the expected histogram gives the expected ratio.
    n = 1 << 20
    x = wl.bf16_weight(n, seed=0)
    st = o.stats(x.numpy(), n, o.params(o.BF16, 65536))
    pmf = gaussian_exponent_pmf(0.02, 127, 8, 7)
    hist = np.array(st.field[0].hist[:256], float)
    assert abs(hist / n - pmf).max() < 2e-3
    exp_len = o.code_lengths(np.maximum(np.round(pmf * 1e12), 0).astype(np.uint64).tolist(), 16)
    mask = exp_len > 0
    expect = float((pmf[mask] * exp_len[mask]).sum()) / 8
    assert abs(st.field[0].ratio_payload - expect) < 3e-3
    assert 0.31 < st.field[0].ratio_payload < 0.34          # paper: BF16 total "up to 62%"
    assert st.field[1].ratio_payload > 0.99                  # sign+mantissa does not compress
    assert abs(st.ratio_payload_total - (st.field[0].ratio_payload + st.field[1].ratio_payload) / 2) < 1e-12
    H = st.field[0].entropy_bits
    assert H <= st.field[0].mean_code_len < H + 1
    assert st.field[0].max_len <= 16
    assert st.container_bytes >= st.ratio_payload_total * st.raw_bytes
    assert st.ratio_container_total < st.ratio_payload_total + 0.01


def test_fp8_fp4_kv_ratios_are_in_the_expected_ranges():
    # Sec. 4.2: exponent compresses, mantissa hardly; Sec. 3.4/4.4: FP4 elements do not
    # compress, the scale stream does.
    n = 1 << 20
    st = o.stats(wl.fp8_weight(n, seed=1).numpy(), n, o.params(o.FP8_E4M3, 262144))
    assert 0.6 < st.field[0].ratio_payload < 0.7 and st.field[1].ratio_payload > 0.99
    assert 0.80 < st.ratio_payload_total < 0.85
    for f in range(2):
        H = st.field[f].entropy_bits
        assert H <= st.field[f].mean_code_len < H + 1
    p, s = wl.mxfp4_weight(256, 4096, seed=2)
    st = o.stats(p.numpy(), 256 * 4096, o.params(o.FP4_E2M1_MX, 262144), scales=s.numpy())
    assert st.field[0].ratio_payload > 0.95 and st.field[1].ratio_payload > 0.99
    assert st.field[2].ratio_payload < 0.25
    assert st.raw_bytes == 256 * 4096 // 2 + 256 * 4096 // 32
    k, v = wl.fp8_kv_pair(batch=1, heads=2, tokens=512, seed=3)
    for t in (k, v):
        st = o.stats(t.numpy().reshape(-1), t.numel(), o.params(o.FP8_E4M3, 2048, streams=8))
        assert 0.55 < st.field[0].ratio_payload < 0.8


def test_generators_are_seeded():
    assert torch.equal(wl.fp8_weight(1000, seed=5), wl.fp8_weight(1000, seed=5))
    assert not torch.equal(wl.fp8_weight(1000, seed=5), wl.fp8_weight(1000, seed=6))
    ids = wl.page_sample(1024, 0.25, seed=1)
    assert len(ids) == 256 and len(set(ids.tolist())) == 256


def test_nvfp4_generator():
    # E4M3 decode is the inverse of the cast on every finite code, and the generator's blocks are 16 wide
    codes = torch.arange(256, dtype=torch.uint8)
    finite = (codes & 0x7F) != 0x7F
    assert torch.equal(wl.e4m3_bits(wl.e4m3_to_f32(codes[finite])), codes[finite])
    assert wl.e4m3_to_f32(torch.tensor([0x38, 0x7E, 0x01, 0xB8], dtype=torch.uint8)).tolist() == [1.0, 448.0, 2.0 ** -9, -1.0]
    packed, scale = wl.nvfp4_weight(64, 512, seed=1)
    assert packed.numel() == 64 * 512 // 2 and scale.numel() == 64 * 512 // 16 and int(scale.max()) == 0x7E
    # dequantised values stay close to a fresh draw of the same seed (block-scaled 4-bit grid: coarse check)
    g = torch.Generator().manual_seed(1)
    x = torch.randn(64 * 512, generator=g) * 0.015
    lo, hi = (packed & 0xF).to(torch.int64), (packed >> 4).to(torch.int64)
    grid = torch.tensor([0, .5, 1, 1.5, 2, 3, 4, 6, -0., -.5, -1, -1.5, -2, -3, -4, -6])
    vals = torch.stack([grid[lo], grid[hi]], dim=1).reshape(-1, 16)
    ts = (x.reshape(-1, 16).abs().amax(dim=1) / 6.0).max() / 448.0
    deq = vals * (wl.e4m3_to_f32(scale) * ts).unsqueeze(1)
    assert float((deq.reshape(-1) - x).abs().max()) < 0.25 * float(x.abs().max())
    # the MX generator still gives the same bytes after sharing the E2M1 cast
    p2, s2 = wl.mxfp4_weight(8, 64, seed=2)
    assert p2.numel() == 256 and s2.numel() == 16


def test_e5m2_cast_matches_torch():
    g = torch.Generator().manual_seed(5)
    x = torch.randn(200000, generator=g) * torch.exp2(torch.randint(-18, 15, (200000,), generator=g).float())
    x = x.clamp(-57344.0, 57344.0)
    assert torch.equal(wl.e5m2_bits(x), x.to(torch.float8_e5m2).view(torch.uint8))
    w = wl.fp8_e5m2_weight(4096, seed=3)
    assert w.dtype == torch.uint8 and int((w & 0x7F).max()) == 0x7B

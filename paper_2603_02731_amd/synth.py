"""Seeded synthetic inputs shaped like the paper's workloads.

This module serves both the CPU oracle's tests and the GPU path, and therefore holds
none of the method's arithmetic: it only draws random activations and puts them into
the *input* format of the conversions, DeepSeek-V3-style blockwise FP8 (E4M3 bytes with
one FP32 scale per 1x128 tile, scale = amax/448).  The E4M3 cast is PyTorch's.

The paper measures on activations of its 236B / 671B training runs (section 4.3), which
are not available; the generators stand in for them with DeepSeek-V3 sizes (hidden 7168,
expert intermediate 2048), heavy tails and outlier channels.
"""
import math

import torch

E4M3_MAX = 448.0


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def fp8_blockwise_quantize(v):
    """float32 [M,K] -> (uint8 E4M3 bytes [M,K], float32 scales [M,K/128]); scale = amax/448."""
    M, K = v.shape
    assert K % 128 == 0
    t = v.float().reshape(M, K // 128, 128)
    amax = t.abs().amax(dim=-1, keepdim=True)
    s = amax / E4M3_MAX
    safe = torch.where(s > 0, s, torch.ones_like(s))
    y = torch.clamp(t / safe, -E4M3_MAX, E4M3_MAX)
    x8 = y.to(torch.float8_e4m3fn).view(torch.uint8).reshape(M, K)
    return x8.contiguous(), s.reshape(M, K // 128).contiguous()


def tiny_roundtrip_fp8(seed=0, M=256, K=512):
    """Config 1: BF16 randn, 2% of columns x50, FP8-quantized; then 1% of the 32-blocks
    zeroed, and E4M3 subnormals and +-448 written at seeded positions.  CPU tensors."""
    g = _gen(seed, "cpu")
    v = torch.randn(M, K, generator=g, dtype=torch.float32).to(torch.bfloat16).float()
    n_out = max(1, int(round(0.02 * K)))
    cols = torch.randperm(K, generator=g)[:n_out]
    v[:, cols] *= 50.0
    x8, s = fp8_blockwise_quantize(v)
    nblk = M * K // 32
    zero_blocks = torch.randperm(nblk, generator=g)[: max(1, nblk // 100)]
    xb = x8.reshape(nblk, 32)
    xb[zero_blocks] = 0
    x8 = xb.reshape(M, K)
    flat = x8.reshape(-1)
    n_special = max(16, M * K // 256)
    pos = torch.randperm(M * K, generator=g)[: 2 * n_special]
    sub = torch.randint(1, 8, (n_special,), generator=g, dtype=torch.int64)
    sgn = torch.randint(0, 2, (n_special,), generator=g, dtype=torch.int64) * 0x80
    flat[pos[:n_special]] = (sub | sgn).to(torch.uint8)
    big = torch.randint(0, 2, (n_special,), generator=g, dtype=torch.int64) * 0x80 + 0x7E
    flat[pos[n_special:]] = big.to(torch.uint8)
    return flat.reshape(M, K).contiguous(), s


def student_t_fp8(M, K=7168, seed=0, device="cpu", df=3, outlier_frac=0.01, outlier_gain=100.0,
                  chunk_rows=4096):
    """Configs 2 and 5: Student-t(df) activations, 1% outlier channels x100, FP8-quantized."""
    g = _gen(seed, device)
    n_out = max(1, int(round(outlier_frac * K)))
    cols = torch.randperm(K, generator=g, device=device)[:n_out]
    gain = torch.ones(K, device=device)
    gain[cols] = outlier_gain
    x8 = torch.empty(M, K, dtype=torch.uint8, device=device)
    s = torch.empty(M, K // 128, dtype=torch.float32, device=device)
    for r0 in range(0, M, chunk_rows):
        r1 = min(M, r0 + chunk_rows)
        z = torch.randn(r1 - r0, K, generator=g, device=device)
        chi = torch.zeros_like(z)
        for _ in range(df):
            chi += torch.randn(r1 - r0, K, generator=g, device=device) ** 2
        v = z / torch.sqrt(chi / df) * gain
        x8[r0:r1], s[r0:r1] = fp8_blockwise_quantize(v)
    return x8, s


def swiglu_fp8(M, K=2048, seed=0, device="cpu", chunk_rows=8192):
    """Config 3: expert-FFN activations silu(a)*b, a,b ~ N(0,1), FP8-quantized."""
    g = _gen(seed, device)
    x8 = torch.empty(M, K, dtype=torch.uint8, device=device)
    s = torch.empty(M, K // 128, dtype=torch.float32, device=device)
    for r0 in range(0, M, chunk_rows):
        r1 = min(M, r0 + chunk_rows)
        a = torch.randn(r1 - r0, K, generator=g, device=device)
        b = torch.randn(r1 - r0, K, generator=g, device=device)
        x8[r0:r1], s[r0:r1] = fp8_blockwise_quantize(torch.nn.functional.silu(a) * b)
    return x8, s


def expert_offsets(seed=0, num_experts=32, total_tokens=65536, zipf_a=1.2, pad_to=128):
    """Config 4: token counts ~ multinomial(total, p_e), p_e proportional to rank^-a under a
    seeded permutation, each padded up to a multiple of pad_to.
    Returns (int32 offsets [E+1] of the padded layout, int64 true counts [E])."""
    g = _gen(seed, "cpu")
    ranks = torch.randperm(num_experts, generator=g).double() + 1.0
    p = ranks.pow(-zipf_a)
    p = p / p.sum()
    draws = torch.multinomial(p, total_tokens, replacement=True, generator=g)
    counts = torch.bincount(draws, minlength=num_experts)
    padded = ((counts + pad_to - 1) // pad_to) * pad_to
    off = torch.zeros(num_experts + 1, dtype=torch.int64)
    off[1:] = torch.cumsum(padded, 0)
    assert int(off[-1]) < 2 ** 31
    return off.to(torch.int32), counts


def zero_padding_rows(x8, s, offsets, counts):
    """Zero the padding rows of every expert slice (rows past the expert's true count)."""
    for e in range(len(counts)):
        lo = int(offsets[e]) + int(counts[e])
        hi = int(offsets[e + 1])
        x8[lo:hi] = 0
        s[lo:hi] = 0
    return x8, s


def routing_indices(seed=0, num_tokens=65536, top_k=8, device="cpu"):
    """Config 5: every token is sent to top_k experts; a seeded shuffle stands for the
    order in which the dispatch lays the copies out.  int32 [num_tokens*top_k]."""
    g = _gen(seed, device)
    idx = torch.arange(num_tokens, device=device, dtype=torch.int32).repeat_interleave(top_k)
    perm = torch.randperm(num_tokens * top_k, generator=g, device=device)
    return idx[perm].contiguous()


def random_mxfp4(M, K, seed=0, scale_center=127, scale_spread=4, nan_scale_frac=0.0, device="cpu"):
    """Stress input for the MXFP4-source conversions: uniform random nibbles and scale
    bytes uniform in [center-spread, center+spread] (clamped to [0,254]); optionally a
    fraction of NaN (0xFF) scale bytes."""
    g = _gen(seed, device)
    q = torch.randint(0, 256, (M, K // 2), generator=g, device=device, dtype=torch.int64).to(torch.uint8)
    lo = max(0, scale_center - scale_spread)
    hi = min(254, scale_center + scale_spread)
    sf = torch.randint(lo, hi + 1, (M, K // 32), generator=g, device=device, dtype=torch.int64).to(torch.uint8)
    if nan_scale_frac > 0:
        mask = torch.rand(M, K // 32, generator=g, device=device) < nan_scale_frac
        sf[mask] = 0xFF
    return q, sf


def payload_bytes(M, K):
    """Closed-form payloads (section 3.2): FP8 = M*K + 4*M*K/128, MXFP4 = M*K/2 + M*K/32."""
    return {"fp8": M * K + (M * K // 128) * 4, "mxfp4": M * K // 2 + M * K // 32}


__all__ = [n for n in dir() if not n.startswith("_") and n not in ("math", "torch")]

"""Seeded synthetic inputs for the SpeCache decode step.

Serves both the GPU path and the CPU oracle.  Holds only random draws and
rounding to the cache's 16-bit type: no quantiser, score, selection or
attention arithmetic lives here.

Recipe (stands in for the paper's LongBench / PG19 workloads, which need
datasets and trained weights): keys and values i.i.d. N(0,1); four key
channels per KV head scaled by 10 (the channel outliers that motivate
per-channel key quantisation, Section 2.1); queries q ~ N(0,1) and the
speculative query q' = q + 0.1 N(0,1); all rounded to the cache dtype.
Tensors are returned as raw uint16 bit patterns (numpy has no bfloat16).
Random numbers come from numpy's counter-based Philox generator keyed by
(seed, tensor id).
"""
import numpy as np

FP16, BF16 = 0, 1
_T_K, _T_V, _T_Q, _T_DQ, _T_SPEC, _T_OUTLIER, _T_STEP = range(7)


def _rng(seed, tensor_id, sub=0):
    return np.random.Generator(np.random.Philox(key=[(seed << 8) | tensor_id, sub]))


def to_bits(x, dtype):
    """Round float32 values to the 16-bit dtype (nearest even); return uint16 patterns."""
    x = np.ascontiguousarray(x, np.float32)
    if dtype == FP16:
        return x.astype(np.float16).view(np.uint16)
    u = x.view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def from_bits(bits, dtype):
    """Exact float32 values of uint16 patterns."""
    bits = np.ascontiguousarray(bits, np.uint16)
    if dtype == FP16:
        return bits.view(np.float16).astype(np.float32)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def outlier_channels(seed, B, Hkv, D, n_outlier=4):
    """Channel ids of the scaled key channels, one draw per (batch, KV head): [B, Hkv, n_outlier]."""
    rng = _rng(seed, _T_OUTLIER)
    out = np.empty((B, Hkv, n_outlier), np.int64)
    for b in range(B):
        for h in range(Hkv):
            out[b, h] = np.sort(rng.choice(D, size=n_outlier, replace=False))
    return out


def make_kv(seed, B, Hkv, S, D, dtype, n_outlier=4, outlier_scale=10.0, sub=0):
    """K, V as uint16 [B, Hkv, S, D]."""
    k = _rng(seed, _T_K, sub).standard_normal((B, Hkv, S, D), dtype=np.float32)
    v = _rng(seed, _T_V, sub).standard_normal((B, Hkv, S, D), dtype=np.float32)
    if n_outlier:
        ch = outlier_channels(seed, B, Hkv, D, n_outlier)
        for b in range(B):
            for h in range(Hkv):
                k[b, h][:, ch[b, h]] *= np.float32(outlier_scale)
    return to_bits(k, dtype), to_bits(v, dtype)


def make_queries(seed, B, Hq, D, dtype, n_rows=2, sub=0):
    """q as uint16 [B, Hq, n_rows, D]; row 0 = current query, row 1 = speculative query."""
    q = _rng(seed, _T_Q, sub).standard_normal((B, Hq, D), dtype=np.float32)
    rows = [q]
    if n_rows == 2:
        dq = _rng(seed, _T_DQ, sub).standard_normal((B, Hq, D), dtype=np.float32)
        rows.append(q + np.float32(0.1) * dq)
    return to_bits(np.stack(rows, axis=2), dtype)


def make_spec_kv(seed, B, Hkv, D, dtype, sub=0):
    """Transient (k_spec, v_spec) of the speculative token: uint16 [B, Hkv, 1, D] each."""
    r = _rng(seed, _T_SPEC, sub).standard_normal((2, B, Hkv, 1, D), dtype=np.float32)
    return to_bits(r[0], dtype), to_bits(r[1], dtype)


def make_step_kv(seed, step, B, Hkv, D, dtype, n_outlier=4, outlier_scale=10.0):
    """The (k, v) pair appended at decode step `step`: uint16 [B, Hkv, 1, D] each."""
    r = _rng(seed, _T_STEP, step).standard_normal((2, B, Hkv, 1, D), dtype=np.float32)
    k, v = r[0], r[1]
    if n_outlier:
        ch = outlier_channels(seed, B, Hkv, D, n_outlier)
        for b in range(B):
            for h in range(Hkv):
                k[b, h][:, ch[b, h]] *= np.float32(outlier_scale)
    return to_bits(k, dtype), to_bits(v, dtype)


# ---- the same recipe drawn on the GPU (full-size benchmark inputs) ------------

def torch_dtype(dtype):
    import torch
    return torch.float16 if dtype == FP16 else torch.bfloat16


def make_kv_device(seed, B, Hkv, S, D, dtype, n_outlier=4, outlier_scale=10.0, device="cuda"):
    """K, V as 16-bit tensors [B, Hkv, S, D] on the device, drawn with torch's seeded generator."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    k = torch.randn((B, Hkv, S, D), generator=gen, device=device, dtype=torch.float32)
    if n_outlier:
        ch = outlier_channels(seed, B, Hkv, D, n_outlier)
        scale = torch.ones((B, Hkv, 1, D), device=device)
        for b in range(B):
            for h in range(Hkv):
                scale[b, h, 0, torch.as_tensor(ch[b, h], device=device)] = outlier_scale
        k *= scale
    k = k.to(torch_dtype(dtype))
    v = torch.randn((B, Hkv, S, D), generator=gen, device=device, dtype=torch.float32).to(torch_dtype(dtype))
    return k, v


def make_queries_device(seed, n, B, Hq, D, dtype, device="cuda"):
    """n query tensors [n, B, Hq, 2, D]: row 0 = q ~ N(0,1), row 1 = q + 0.1 N(0,1)."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(seed + 7919)
    q = torch.randn((n, B, Hq, 1, D), generator=gen, device=device, dtype=torch.float32)
    dq = torch.randn((n, B, Hq, 1, D), generator=gen, device=device, dtype=torch.float32)
    return torch.cat([q, q + 0.1 * dq], dim=3).to(torch_dtype(dtype)).contiguous()


def bits_of(t):
    """uint16 numpy view of a 16-bit torch tensor (copied to the host)."""
    import torch
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)

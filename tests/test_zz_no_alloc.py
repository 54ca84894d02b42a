"""specache_attend_static, the entry point for callers that cannot allocate: its partial results live in a
static device array of the library instead of the context's scratch buffer.  Same kernels, so its output must
equal specache_attend's (checked to the 2e-3 bar of the attention outputs, and observed bit for bit), on two
calls in a row, the second on a smaller input, which finds what the first call left in the shared array."""
import numpy as np
import pytest
import torch

from paper_2503_16163_amd import binding, synth

pytestmark = pytest.mark.gpu


def _dev(bits, dtype):
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()
    return t.view(torch.float16 if dtype == synth.FP16 else torch.bfloat16)


def _one_context(B, Hq, Hkv, S, dtype, bits, g, k, seed):
    """Load S tokens, run two decode steps; on the second (prefetched pairs staged) attend through both entry
    points.  Returns (specache_attend's output, specache_attend_static's output)."""
    from tests.harness import OUT_TOL
    sc = binding.SpeCache(1, B, Hq, Hkv, bits, g, ((S + 127) // 64) * 64, k, dtype)
    try:
        kb, vb = synth.make_kv(seed, B, Hkv, S, 128, dtype)
        sc.quantize_append(0, _dev(kb, dtype), _dev(vb, dtype), S)
        side = torch.cuda.Stream()
        idx = [torch.full((B, Hkv, k), -1, dtype=torch.int32, device="cuda") for _ in range(2)]
        outs = None
        for t in range(2):
            nk, nv = synth.make_step_kv(seed, t, B, Hkv, 128, dtype)
            ks, vs = synth.make_spec_kv(seed, B, Hkv, 128, dtype, sub=t)
            q = _dev(synth.make_queries(seed, B, Hq, 128, dtype, sub=t), dtype)
            ksd, vsd = _dev(ks, dtype), _dev(vs, dtype)
            sc.quantize_append(0, _dev(nk, dtype), _dev(nv, dtype), 1)
            sc.score_topk(0, q, 2, idx[t % 2])
            sc.gather(0, idx[t % 2], (t + 1) % 2, side)
            slot = (t % 2) if t > 0 else -1
            a = torch.full((B, Hq, 2, 128), float("nan"), dtype=torch.float32, device="cuda")
            b = torch.full((B, Hq, 2, 128), float("nan"), dtype=torch.float32, device="cuda")
            sc.attend(0, q, 2, ksd, vsd, slot, a)
            sc.attend_static(0, q, 2, ksd, vsd, slot, b)
            torch.cuda.synchronize()
            outs = (a.cpu().numpy(), b.cpu().numpy())
            assert np.all(np.isfinite(outs[1]))
            denom = np.maximum(np.abs(outs[0]).max(axis=-1), 1e-6)
            err = np.abs(outs[1].astype(np.float64) - outs[0]).max(axis=-1) / denom
            assert err.max() <= OUT_TOL, f"static-scratch attend differs from attend by {err.max():.3e} at step {t}"
            assert np.array_equal(outs[0], outs[1]), "same kernels, same inputs: the outputs should be identical"
        return outs
    finally:
        torch.cuda.synchronize()
        sc.close()


def test_attend_from_static_scratch_matches_attend_twice_in_a_row():
    assert torch.cuda.is_available()
    torch.cuda.set_device(0)
    big = _one_context(2, 8, 4, 5000, synth.FP16, 2, 32, 96, seed=7100)      # 8 rows x 13 chunks x 4 query rows
    small = _one_context(1, 2, 2, 700, synth.BF16, 1, 64, 24, seed=7101)     # 2 rows x 3 chunks: reuses the head of the array
    assert big[1].shape == (2, 8, 2, 128) and small[1].shape == (1, 2, 2, 128)


def test_static_scratch_rejects_what_does_not_fit():
    """2 rows x 16 query rows x 1172 chunks x 130 floats = 19.5 MB of partial results against a 16 MiB array:
    ECAPACITY, nothing launched, and specache_attend still serves the call."""
    assert torch.cuda.is_available()
    torch.cuda.set_device(0)
    S, dtype = 300000, synth.BF16
    sc = binding.SpeCache(1, 2, 8, 1, 1, 32, 300160, 64, dtype)
    try:
        kd, vd = synth.make_kv_device(7200, 2, 1, S, 128, dtype)
        sc.quantize_append(0, kd, vd, S)
        q = synth.make_queries_device(7200, 1, 2, 8, 128, dtype)[0]
        idx = torch.full((2, 1, 64), -1, dtype=torch.int32, device="cuda")
        out = torch.empty((2, 8, 2, 128), dtype=torch.float32, device="cuda")
        sc.score_topk(0, q, 2, idx)
        with pytest.raises(binding.SpeCacheError) as ei:
            sc.attend_static(0, q, 2, None, None, -1, out)
        assert ei.value.code == binding.ECAPACITY
        sc.attend(0, q, 2, None, None, -1, out)
        torch.cuda.synchronize()
        assert np.all(np.isfinite(out.cpu().numpy()))
    finally:
        torch.cuda.synchronize()
        sc.close()

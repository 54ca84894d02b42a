"""Shared driver for the GPU-vs-oracle parity tests and the smoke check.

Runs the HIP path through the C ABI (paper_2503_16163_amd.binding) and the CPU
oracle on the same seeded synthetic inputs and compares them to the bars:
  * codes, stored (min,max) and derived (s,z): bit-exact;
  * offloaded 16-bit rows: bit-exact;
  * top-k index sets: equal, except positions whose oracle score lies within
    1e-5 * max(|tau|, max|sigma|) of the k-th score tau;
  * attention outputs: max |o - o_ref| / max(max|o_ref|, 1e-6) <= 2e-3 per
    (head, row).
"""
import numpy as np
import torch

from oracle import oracle as orc
from paper_2503_16163_amd import binding, synth

OUT_TOL = 2e-3
TIE_BAND = 1e-5
# fp32 accumulation of 128 products against the oracle's double: a few 1e-6 of the
# largest partial sum; checked loosely, the gates are the two bars above.
LOGIT_TOL = 2e-4


def to_dev(bits, dtype):
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()
    return t.view(torch.float16 if dtype == synth.FP16 else torch.bfloat16)


def check_topk(sigma, idx, k, what=""):
    """Band rule for one row.  sigma: oracle scores [Nq] (float64); idx: GPU result [k]."""
    nq = sigma.size
    keff = min(k, nq)
    sel = idx[:keff]
    assert np.all(idx[keff:] == -1), f"{what}: padding"
    assert np.all(sel >= 0) and np.all(sel < nq), f"{what}: index range"
    assert np.all(np.diff(sel) > 0), f"{what}: not strictly ascending"
    if keff == 0:
        return 0
    order = np.sort(sigma)[::-1]
    tau = order[keff - 1]
    band = TIE_BAND * max(abs(tau), np.abs(sigma).max())
    chosen = np.zeros(nq, bool)
    chosen[sel] = True
    must = sigma > tau + band
    must_not = sigma < tau - band
    assert np.all(chosen[must]), f"{what}: a position above the tie band is missing"
    assert not np.any(chosen[must_not]), f"{what}: a position below the tie band was selected"
    ref = orc.topk(sigma, k)[:keff]
    return int(keff - np.intersect1d(ref, sel).size)   # differences inside the band


def check_out(out_gpu, out_ref, what=""):
    """out_*: [G, rows, D]."""
    denom = np.maximum(np.abs(out_ref).max(axis=-1), 1e-6)
    err = np.abs(out_gpu.astype(np.float64) - out_ref).max(axis=-1) / denom
    assert np.all(np.isfinite(out_gpu)), f"{what}: non-finite output"
    assert err.max() <= OUT_TOL, f"{what}: attention output error {err.max():.3e} > {OUT_TOL}"
    return float(err.max())


class Case:
    """One configuration run on both sides.  `sample` lists the (b, hkv) pairs the oracle mirrors."""

    def __init__(self, B, Hq, Hkv, S, dtype, bits, g, k, R=64, seed=1000, n_rows=2, sample=None,
                 max_seq=None, n_outlier=4, one_bit_form=0, select_form=0, select_cache=0, async_select=0,
                 fused_append=False, one_pass=False):
        self.B, self.Hq, self.Hkv, self.S, self.dtype, self.bits, self.g, self.k, self.R = B, Hq, Hkv, S, dtype, bits, g, k, R
        self.seed, self.n_rows, self.G, self.D = seed, n_rows, Hq // Hkv, 128
        self.sm_scale = 1.0 / np.sqrt(128.0)
        self.sample = sample if sample is not None else [(b, h) for b in range(B) for h in range(Hkv)]
        cap = max_seq or ((S + 64 + 63) // 64) * 64
        self.one_bit_form, self.select_form, self.select_cache = one_bit_form, select_form, select_cache
        self.async_select = async_select
        self.fused_append = bool(fused_append) and async_select == 2   # specache_append_score[_attend] in decode_step
        self.one_pass = bool(one_pass) and async_select == 2           # specache_score_attend in decode_step
        self.pending = None
        self.staged_idx = None       # index lists of the last gather (what a mixed-cache selection scores in 16 bits)
        self.sc = binding.SpeCache(1, B, Hq, Hkv, bits, g, cap, k, dtype, residual=R, one_bit_form=one_bit_form,
                                   select_form=select_form, select_cache=select_cache, async_select=async_select)
        self.k_bits, self.v_bits = synth.make_kv(seed, B, Hkv, S, self.D, dtype, n_outlier=n_outlier)
        self.oc = {}
        self.step_k, self.step_v = [], []
        self.side = torch.cuda.Stream()
        self.idx = [torch.full((B, Hkv, k), -7, dtype=torch.int32, device="cuda") for _ in range(2)]
        self.step_no = 0
        self.stats = dict(band_diffs=0, max_out_err=0.0, max_logit_err=0.0)
        self.q_head_scale = None     # optional [Hq] factors applied to the synthetic queries of decode_step

    def close(self):
        torch.cuda.synchronize()
        self.sc.close()

    # ---- load ---------------------------------------------------------------
    def load(self, chunks=None):
        """Bulk append of the S prompt tokens (optionally split into several calls)."""
        S = self.S
        bounds = [0, S] if not chunks else [0] + list(chunks) + [S]
        for a, b in zip(bounds[:-1], bounds[1:]):
            if b > a:
                kd = to_dev(self.k_bits[:, :, a:b], self.dtype)
                vd = to_dev(self.v_bits[:, :, a:b], self.dtype)
                self.sc.quantize_append(0, kd, vd, b - a)
        torch.cuda.synchronize()
        for (b, h) in self.sample:
            c = orc.Cache(self.D, self.bits, self.g, self.R, self.dtype, self.one_bit_form)
            c.append(self.k_bits[b, h], self.v_bits[b, h])
            self.oc[(b, h)] = c

    def append_token(self, t):
        kb, vb = synth.make_step_kv(self.seed, t, self.B, self.Hkv, self.D, self.dtype)
        self._flush_pending()
        if self.fused_append:
            self.pending = (to_dev(kb, self.dtype), to_dev(vb, self.dtype))   # appended by the next decode_step
        else:
            self.sc.quantize_append(0, to_dev(kb, self.dtype), to_dev(vb, self.dtype), 1)
        for (b, h) in self.sample:
            self.oc[(b, h)].append(kb[b, h], vb[b, h])
        self.step_k.append(kb)
        self.step_v.append(vb)

    def _flush_pending(self):
        if self.pending is not None:
            self.sc.quantize_append(0, self.pending[0], self.pending[1], 1)
            self.pending = None

    # ---- checks -------------------------------------------------------------
    def check_quantized(self):
        self._flush_pending()
        e = self.sc.export_quantized(0)
        n, nq = self.sc.counts(0)
        for (b, h) in self.sample:
            c = self.oc[(b, h)]
            assert c.counts() == (n, nq), ("counts", c.counts(), (n, nq))
            o = c.export()
            assert np.array_equal(e["k_codes"][b, h], o["k_codes"]), f"K codes differ at {(b, h)}"
            assert np.array_equal(e["v_codes"][b, h], o["v_codes"]), f"V codes differ at {(b, h)}"
            assert np.array_equal(e["k_mnmx"][b, h], synth.to_bits(o["k_mnmx"], self.dtype)), "K (min,max)"
            assert np.array_equal(e["v_mnmx"][b, h], synth.to_bits(o["v_mnmx"], self.dtype)), "V (min,max)"
            assert np.array_equal(e["k_sz"][b, h].view(np.uint32), o["k_sz"].view(np.uint32)), "K (s,z)"
            assert np.array_equal(e["v_sz"][b, h].view(np.uint32), o["v_sz"].view(np.uint32)), "V (s,z)"
        return n, nq

    def check_offload(self, first=0, count=None):
        self._flush_pending()
        n, _ = self.sc.counts(0)
        count = n - first if count is None else count
        rows = self.sc.export_rows(0, first, count)
        k_all = np.concatenate([self.k_bits[:, :, first:]] + self.step_k, axis=2) if first < self.S else \
            np.concatenate(self.step_k, axis=2)[:, :, first - self.S:]
        v_all = np.concatenate([self.v_bits[:, :, first:]] + self.step_v, axis=2) if first < self.S else \
            np.concatenate(self.step_v, axis=2)[:, :, first - self.S:]
        assert np.array_equal(rows[:, :, :, 0], k_all[:, :, :count])
        assert np.array_equal(rows[:, :, :, 1], v_all[:, :, :count])

    def decode_step(self, use_spec=True, check_logits=True, do_gather=True):
        """score_topk -> gather(next slot) -> attend(current slot), each checked against the oracle."""
        t = self.step_no
        nr = self.n_rows
        q_bits = synth.make_queries(self.seed, self.B, self.Hq, self.D, self.dtype, n_rows=nr, sub=t)
        if self.q_head_scale is not None:
            scaled = synth.from_bits(q_bits, self.dtype) * np.asarray(self.q_head_scale, np.float32)[None, :, None, None]
            q_bits = synth.to_bits(scaled, self.dtype).reshape(q_bits.shape)
        ks_bits, vs_bits = synth.make_spec_kv(self.seed, self.B, self.Hkv, self.D, self.dtype, sub=t)
        q = to_dev(q_bits, self.dtype)
        ks, vs = (to_dev(ks_bits, self.dtype), to_dev(vs_bits, self.dtype)) if use_spec else (None, None)
        idx = self.idx[t % 2]
        main = torch.cuda.current_stream()
        out = torch.empty((self.B, self.Hq, nr, self.D), dtype=torch.float32, device="cuda")
        slot = (t % 2) if (t > 0 and do_gather) else -1
        if self.one_pass:            # scoring and attention in one call, then the selection and the gather
            if self.pending is not None:
                self.sc.append_score_attend(0, self.pending[0], self.pending[1], q, nr, ks, vs, slot, out, main)
                self.pending = None
            else:
                self.sc.score_attend(0, q, nr, ks, vs, slot, out, main)
            self.sc.select_gather(0, idx, (t + 1) % 2 if do_gather else -1, self.side)
        elif self.async_select == 2:   # ArgTopK on the gather's stream: the other pair of calls
            if self.pending is not None:
                self.sc.append_score(0, self.pending[0], self.pending[1], q, nr, main)
                self.pending = None
            else:
                self.sc.score(0, q, nr, main)
            self.sc.select_gather(0, idx, (t + 1) % 2 if do_gather else -1, self.side)
        else:
            self.sc.score_topk(0, q, nr, idx, main)
            if do_gather:
                self.sc.gather(0, idx, (t + 1) % 2, self.side)
        if not self.one_pass:
            self.sc.attend(0, q, nr, ks, vs, slot, out, main)
        torch.cuda.synchronize()
        idx_h = idx.cpu().numpy()
        out_h = out.cpu().numpy()
        logits_h = self.sc.debug_logits(0, nr) if check_logits else None
        prev = self.prev_idx if slot >= 0 else None
        n, nq = self.sc.counts(0)
        for (b, h) in self.sample:
            c = self.oc[(b, h)]
            qh = q_bits[b, h * self.G:(h + 1) * self.G]                      # [G, rows, D]
            staged = self.staged_idx[b, h] if (self.select_cache and self.staged_idx is not None) else None
            ref_logits, sigma = c.scores(qh, self.sm_scale, self.select_form, P=staged)
            if check_logits and nq:
                got = logits_h[b, h * self.G:(h + 1) * self.G]
                err = np.abs(got - ref_logits).max() / max(np.abs(ref_logits).max(), 1.0)
                self.stats["max_logit_err"] = max(self.stats["max_logit_err"], float(err))
                assert err <= LOGIT_TOL, f"logits differ at {(b, h)}: {err:.3e}"
            self.stats["band_diffs"] += check_topk(sigma, idx_h[b, h], self.k, what=f"top-k {(b, h)} step {t}")
            P = prev[b, h] if prev is not None else None
            ref_out = c.attend(qh, self.sm_scale, P=P, k_spec=ks_bits[b, h, 0] if use_spec else None,
                               v_spec=vs_bits[b, h, 0] if use_spec else None)
            e = check_out(out_h[b, h * self.G:(h + 1) * self.G], ref_out, what=f"attend {(b, h)} step {t}")
            self.stats["max_out_err"] = max(self.stats["max_out_err"], e)
        self.prev_idx = idx_h
        if do_gather:
            self.staged_idx = idx_h
        self.last_q_bits = q_bits
        self.step_no += 1
        return idx_h, out_h


    def nonspec_step(self):
        """Non-speculative fetching (the ablation of Section 4.4 / Table 4): select on the current token's own
        low-bit scores, fetch those pairs at once, then attend with them.  One query row, serial gather."""
        t = self.step_no
        q_bits = synth.make_queries(self.seed, self.B, self.Hq, self.D, self.dtype, n_rows=1, sub=t)
        q = to_dev(q_bits, self.dtype)
        idx = self.idx[t % 2]
        main = torch.cuda.current_stream()
        self._flush_pending()
        self.sc.score_topk(0, q, 1, idx, main)
        self.sc.gather(0, idx, 0, main)
        out = torch.empty((self.B, self.Hq, 1, self.D), dtype=torch.float32, device="cuda")
        self.sc.attend(0, q, 1, None, None, 0, out, main)
        torch.cuda.synchronize()
        idx_h, out_h = idx.cpu().numpy(), out.cpu().numpy()
        for (b, h) in self.sample:
            c = self.oc[(b, h)]
            qh = q_bits[b, h * self.G:(h + 1) * self.G]
            _, sigma = c.scores(qh, self.sm_scale, self.select_form)
            self.stats["band_diffs"] += check_topk(sigma, idx_h[b, h], self.k, what=f"non-spec top-k {(b, h)}")
            ref_out = c.attend(qh, self.sm_scale, P=idx_h[b, h])
            e = check_out(out_h[b, h * self.G:(h + 1) * self.G], ref_out, what=f"non-spec attend {(b, h)}")
            self.stats["max_out_err"] = max(self.stats["max_out_err"], e)
        self.prev_idx = idx_h
        self.step_no += 1
        return idx_h, out_h

"""GPU-vs-oracle parity in the arrangement bench.py times: the benchmark's full sizes, several layers stepped
free-running (no host synchronise between steps), ArgTopK and the gathers on the side streams that
paper_2503_16163_amd.arrangement picks for the shape, and EVERY (batch, KV head) row compared.

Every row of every layer is loaded with the same K, V and queries, so one oracle cache stands for all of them:
row (0, 0) of layer 0 is checked against the oracle step by step (codes and metadata bit for bit, index sets by
the tie-band rule, outputs to 2e-3), and every other row of every layer must equal that row: codes and index
lists bit for bit, outputs to the same 2e-3 bar.  The rows differ in their strides and addresses only, which
is what is being tested at the sizes where those are largest."""
import numpy as np
import pytest
import torch

from paper_2503_16163_amd import arrangement, binding, synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need an MI355X (run with -m gpu on the GPU box)"
    torch.cuda.set_device(0)


# name: B, Hq, Hkv, S, dtype, bits, g, k, layers stepped
SHAPES = {
    "config1": (1, 1, 1, 4096, synth.FP16, 2, 32, 64, 1),
    "config2": (1, 32, 32, 16384, synth.FP16, 2, 32, 256, 4),
    "M0_7B_32k": (1, 32, 32, 32768, synth.FP16, 2, 32, 256, 4),
    "config3": (16, 32, 32, 2048, synth.FP16, 2, 32, 128, 4),
    "config4": (4, 32, 8, 32768, synth.BF16, 2, 64, 512, 4),
    "config5": (1, 32, 8, 131072, synth.BF16, 1, 32, 1024, 4),
    "M0_1bit_g64": (1, 32, 32, 32768, synth.FP16, 1, 64, 64, 4),    # the 7B shape with 1-bit codes (Eq. 3), g = 64, k = 64
    "M0_4bit": (1, 32, 32, 32768, synth.FP16, 4, 32, 256, 4),       # the 7B shape with 4-bit codes (Eq. 2, B = 4)
    "config4_4bit_g128": (4, 32, 8, 32768, synth.BF16, 4, 128, 512, 2),
}
STEPS = 8


def _dev(bits, dtype):
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()
    return t.view(torch.float16 if dtype == synth.FP16 else torch.bfloat16)


def _same_rows(a, what):
    """a: [B, Hkv, ...]; every (b, h) entry must equal entry (0, 0) bit for bit."""
    ref = a[0, 0]
    flat = a.reshape((-1,) + ref.shape)
    bad = [i for i in range(flat.shape[0]) if not np.array_equal(flat[i], ref)]
    assert not bad, f"{what}: rows {bad[:8]} differ from row 0"


def run_free_running(name, fused_append=False, poison=False, steps=STEPS, shape=None, arrange=None, one_pass=False):
    from oracle import oracle as orc
    from tests.harness import OUT_TOL, check_out, check_topk
    B, Hq, Hkv, S, dtype, bits, g, k, layers = shape or SHAPES[name]
    G, D, R = Hq // Hkv, 128, max(64, g)
    seed = 5000 + S + k
    plan = arrangement.plan(B, Hkv, G, S, k, layers, bits)
    async_select, n_side = arrange or (plan["async_select"], plan["side_streams"])
    if arrange is None and not one_pass and not fused_append:
        # no arrangement asked for: the calls bench.py times for this shape
        one_pass, fused_append = plan["calls"] == "one-pass", plan["carry_append"]
    if (one_pass or fused_append) and arrange is None and async_select != 2:
        async_select, n_side = 2, 2     # these calls leave their keys to specache_select_gather
    if fused_append or one_pass:
        assert async_select == 2
    max_seq = ((S + steps + 63) // 64 + 1) * 64
    sc = binding.SpeCache(layers, B, Hq, Hkv, bits, g, max_seq, k, dtype, residual=R, async_select=async_select)
    try:
        kb, vb = synth.make_kv(seed, 1, 1, S, D, dtype)                      # one row's history
        kd = _dev(kb, dtype).expand(B, Hkv, S, D).contiguous()
        vd = _dev(vb, dtype).expand(B, Hkv, S, D).contiguous()
        for L in range(layers):
            sc.quantize_append(L, kd, vd, S)
        torch.cuda.synchronize()
        del kd, vd
        oc = orc.Cache(D, bits, g, R, dtype)
        oc.append(kb[0, 0], vb[0, 0])
        # the bulk-loaded cache: every row of the first and the last layer, codes and metadata bit for bit
        o = oc.export()
        for L in sorted({0, layers - 1}):
            e = sc.export_quantized(L)
            assert sc.counts(L) == oc.counts()
            for key in ("k_codes", "v_codes", "k_mnmx", "v_mnmx"):
                _same_rows(e[key], f"{name} layer {L} {key}")
            _same_rows(e["k_sz"].view(np.uint32), f"{name} layer {L} k_sz")
            _same_rows(e["v_sz"].view(np.uint32), f"{name} layer {L} v_sz")
            assert np.array_equal(e["k_codes"][0, 0], o["k_codes"]) and np.array_equal(e["v_codes"][0, 0], o["v_codes"])
            assert np.array_equal(e["k_mnmx"][0, 0], synth.to_bits(o["k_mnmx"], dtype))
            assert np.array_equal(e["v_mnmx"][0, 0], synth.to_bits(o["v_mnmx"], dtype))
            assert np.array_equal(e["k_sz"][0, 0].view(np.uint32), o["k_sz"].view(np.uint32))
            assert np.array_equal(e["v_sz"][0, 0].view(np.uint32), o["v_sz"].view(np.uint32))
            del e

        main = torch.cuda.current_stream()
        sides = [torch.cuda.Stream() for _ in range(n_side)]
        inputs = []
        for t in range(steps):
            q_bits = synth.make_queries(seed, 1, G, D, dtype, n_rows=2, sub=t)          # [1, G, 2, D]
            ks_bits, vs_bits = synth.make_spec_kv(seed, 1, 1, D, dtype, sub=t)          # [1, 1, 1, D]
            nk, nv = synth.make_step_kv(seed, t, 1, 1, D, dtype)
            q = _dev(q_bits, dtype).view(1, 1, G, 2, D).expand(B, Hkv, G, 2, D).contiguous().view(B, Hq, 2, D)
            dev = [_dev(x, dtype).expand(B, Hkv, 1, D).contiguous() for x in (ks_bits, vs_bits, nk, nv)]
            inputs.append((q_bits, ks_bits, vs_bits, nk, nv, q, dev))
        idx = [[torch.full((B, Hkv, k), -7, dtype=torch.int32, device="cuda") for _ in range(2)] for _ in range(layers)]
        idx_kept = [[torch.empty((B, Hkv, k), dtype=torch.int32, device="cuda") for _ in range(steps)] for _ in range(layers)]
        out = [[torch.empty((B, Hq, 2, D), dtype=torch.float32, device="cuda") for _ in range(steps)] for _ in range(layers)]
        torch.cuda.synchronize()

        # ---- the steps, enqueued back to back: the host looks at nothing until all of them are issued ----
        for t in range(steps):
            q_bits, ks_bits, vs_bits, nk, nv, q, (ks, vs, nkd, nvd) = inputs[t]
            slot = (t % 2) if t > 0 else -1
            for L in range(layers):
                side = sides[L % n_side]
                if one_pass and fused_append:     # the whole layer-step as one call (= append_score_attend + select_gather)
                    sc.decode_step(L, nkd, nvd, q, ks, vs, slot, out[L][t], main, idx[L][t % 2], (t + 1) % 2, side)
                elif one_pass:
                    sc.quantize_append(L, nkd, nvd, 1, main)
                    sc.score_attend(L, q, 2, ks, vs, slot, out[L][t], main)
                    sc.select_gather(L, idx[L][t % 2], (t + 1) % 2, side)
                elif async_select == 2:
                    if fused_append:
                        sc.append_score(L, nkd, nvd, q, 2, main)
                    else:
                        sc.quantize_append(L, nkd, nvd, 1, main)
                        sc.score(L, q, 2, main)
                    sc.select_gather(L, idx[L][t % 2], (t + 1) % 2, side)
                else:
                    sc.quantize_append(L, nkd, nvd, 1, main)
                    sc.score_topk(L, q, 2, idx[L][t % 2], main)
                    sc.gather(L, idx[L][t % 2], (t + 1) % 2, side)
                with torch.cuda.stream(side):        # behind the gather, which is behind the selection
                    idx_kept[L][t].copy_(idx[L][t % 2], non_blocking=True)
                if not one_pass:
                    sc.attend(L, q, 2, ks, vs, slot, out[L][t], main)
                if poison and slot >= 0:
                    # whatever reads this slot before the next gather has rewritten it now reads NaNs
                    sc.debug_poison_slot(L, slot, main)
        torch.cuda.synchronize()

        # ---- row (0, 0) of layer 0 against the oracle, everything else against that row ----
        sm = 1.0 / np.sqrt(128.0)
        stats = dict(band_diffs=0, max_out_err=0.0)
        prev = None
        for t in range(steps):
            q_bits, ks_bits, vs_bits, nk, nv = inputs[t][:5]
            oc.append(nk[0, 0], nv[0, 0])
            qh = q_bits[0]                                                   # [G, 2, D]
            _, sigma = oc.scores(qh, sm)
            got_idx = idx_kept[0][t].cpu().numpy()
            stats["band_diffs"] += check_topk(sigma, got_idx[0, 0], k, what=f"{name} step {t} top-k")
            ref = oc.attend(qh, sm, P=prev, k_spec=ks_bits[0, 0, 0], v_spec=vs_bits[0, 0, 0])
            got_out = out[0][t].cpu().numpy().reshape(B, Hkv, G, 2, D)
            stats["max_out_err"] = max(stats["max_out_err"], check_out(got_out[0, 0], ref, what=f"{name} step {t} attend"))
            _same_rows(got_idx, f"{name} step {t} index lists of layer 0")
            for L in range(layers):
                if L > 0:
                    assert np.array_equal(idx_kept[L][t].cpu().numpy(), got_idx), f"{name} step {t}: index lists of layer {L}"
                o_l = out[L][t].cpu().numpy().reshape(B, Hkv, G, 2, D)
                assert np.all(np.isfinite(o_l)), f"{name} step {t} layer {L}: non-finite output"
                denom = np.maximum(np.abs(ref).max(axis=-1), 1e-6)                    # [G, 2]
                err = np.abs(o_l.astype(np.float64) - ref[None, None]).max(axis=-1) / denom[None, None]
                worst = np.unravel_index(np.argmax(err), err.shape)
                assert err.max() <= OUT_TOL, f"{name} step {t} layer {L}: row {worst[:2]} is off by {err.max():.3e}"
            prev = got_idx[0, 0]
        assert sc.counts(0) == oc.counts()
        print(name, dict(async_select=async_select, side_streams=n_side, layers=layers, steps=steps), stats)
        return stats
    finally:
        torch.cuda.synchronize()
        sc.close()


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name", list(SHAPES))
def test_full_size_all_rows_in_the_timed_arrangement(name):
    """Every shape in the arrangement paper_2503_16163_amd.arrangement.plan picks for it, which is what bench.py times."""
    run_free_running(name)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name", ["config2", "M0_7B_32k"])
def test_full_size_all_rows_two_launches_selection_on_the_gathers_stream(name):
    """specache_score + specache_select_gather + specache_attend (bench.py --calls split) where the rule picks the
    one-pass call."""
    run_free_running(name, arrange=(2, 3))


@pytest.mark.timeout(600)
def test_full_size_fused_append_in_the_timed_arrangement():
    """bench.py --calls split --fused-append at the headline shape: the scoring launch carries the append."""
    run_free_running("M0_7B_32k", fused_append=True)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name", ["M0_7B_32k", "config3"])
def test_full_size_whole_layer_step_in_one_call(name):
    """specache_append_score_attend: append, scoring and attention of a layer-step in one call (one launch where
    no group leaves the residual), then select_gather: what bench.py times by default at these shapes."""
    run_free_running(name, one_pass=True, fused_append=True)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name", ["config1", "config2", "M0_7B_32k", "config3", "config4"])
def test_full_size_all_rows_scoring_and_attention_in_one_pass(name):
    """The same with specache_score_attend in place of specache_score + specache_attend (configs 1 to 3 and the 7B
    shape run the one-pass kernel; config 4, with four query heads per KV head, the two passes behind the one call)."""
    if name == "config1":
        run_free_running(name, one_pass=True, shape=SHAPES[name], arrange=(2, 2))
    else:
        run_free_running(name, one_pass=True)


@pytest.mark.parametrize("async_select,n_side", [(0, 2), (1, 2), (2, 2), (2, 3)])
def test_poisoned_staging_slots_show_no_read_before_gather(async_select, n_side):
    """The one race surface of the path is the pair of staging slots that a side stream fills while the main
    stream reads the other one.  After every attend the slot it read is filled with NaNs (in stream order behind
    the attend): an attend that overtakes the gather refilling its slot, or a gather that overtakes the attend
    still reading the slot (its rows would then be poisoned after they arrived), shows up as NaN outputs; stale
    rows would fail the comparison with the oracle.  Twelve steps of three layers, free-running."""
    shape = (2, 4, 4, 2300, synth.FP16, 2, 32, 72, 3)
    run_free_running("poison", poison=True, steps=12, shape=shape, arrange=(async_select, n_side))
    shape = (1, 8, 2, 1500, synth.BF16, 1, 32, 40, 3)
    run_free_running("poison-gqa", poison=True, steps=6, shape=shape, arrange=(async_select, n_side))
    if async_select == 2:
        shape = (2, 4, 4, 2300, synth.FP16, 2, 32, 72, 3)
        run_free_running("poison-one-pass", poison=True, steps=12, shape=shape, arrange=(async_select, n_side), one_pass=True)
        run_free_running("poison-one-call", poison=True, steps=40, shape=shape, arrange=(async_select, n_side), one_pass=True,
                         fused_append=True)


def test_misaligned_query_is_an_error():
    """The scoring kernels read the query rows 16 bytes at a time; a q that is not 16-byte aligned is rejected
    by the C ABI instead of being scored by some other kernel."""
    for mode in (0, 2):
        sc = binding.SpeCache(1, 1, 2, 2, 2, 32, 256, 16, synth.FP16, async_select=mode)
        try:
            k = torch.zeros((1, 2, 100, 128), dtype=torch.float16, device="cuda")
            sc.quantize_append(0, k, k, 100)
            buf = torch.zeros(2 * 2 * 128 + 8, dtype=torch.float16, device="cuda")
            q_bad = buf[1:1 + 512]
            assert q_bad.data_ptr() % 16 != 0
            idx = torch.zeros((1, 2, 16), dtype=torch.int32, device="cuda")
            with pytest.raises(binding.SpeCacheError) as ei:
                if mode == 2:
                    sc.score(0, q_bad, 2)
                else:
                    sc.score_topk(0, q_bad, 2, idx)
            assert ei.value.code == binding.EINVAL
        finally:
            sc.close()

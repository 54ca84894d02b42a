"""GPU-vs-oracle parity through the C ABI (run with -m gpu on an MI355X)."""
import numpy as np
import pytest
import torch

from paper_2503_16163_amd import binding, synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the GPU"
    binding.lib()


def _run(case, steps=3, chunks=None, use_spec=True):
    from tests import harness  # noqa: F401
    try:
        case.load(chunks=chunks)
        n, nq = case.check_quantized()
        case.check_offload()
        for t in range(steps):
            case.append_token(t)
            case.decode_step(use_spec=use_spec)
        case.check_quantized()
        case.check_offload(first=case.S, count=steps)
        return case.stats
    finally:
        case.close()


def test_config1_single_head():
    """BASELINE config 1: B=1, 1 head, S=4096, fp16, 2-bit g32, k=64."""
    from tests.harness import Case
    stats = _run(Case(1, 1, 1, 4096, synth.FP16, 2, 32, 64, seed=1001), steps=4)
    print("config1", stats)


@pytest.mark.parametrize("B,Hq,Hkv,S,dtype,bits,g,k,R", [
    (2, 3, 3, 1500, synth.FP16, 2, 32, 128, 64),     # MHA, ragged tail (1500 = 46*32 + 28)
    (1, 8, 2, 2112, synth.BF16, 2, 64, 96, 64),      # GQA 4:1, g = R = 64 (ring empties on flush)
    (1, 8, 2, 1200, synth.BF16, 1, 32, 200, 64),     # 1-bit GQA
    (2, 2, 2, 777, synth.FP16, 1, 64, 33, 128),      # 1-bit g64, R = 128, odd k
    (1, 4, 2, 900, synth.FP16, 2, 32, 64, 96),       # GQA 2:1, R = 96
    (1, 8, 1, 640, synth.BF16, 2, 32, 40, 64),       # GQA 8:1
    (1, 2, 2, 3000, synth.FP16, 2, 128, 64, 128),    # g = R = 128, MHA (integer matrix-core scoring)
    (1, 8, 2, 1500, synth.BF16, 1, 128, 50, 256),    # 1-bit g128, GQA 4:1, R = 256
    (2, 4, 2, 1000, synth.FP16, 2, 128, 32, 128),    # g128, GQA 2:1
    (1, 8, 1, 900, synth.BF16, 2, 128, 40, 256),     # g128, GQA 8:1
    (2, 3, 3, 1500, synth.FP16, 4, 32, 128, 64),     # 4-bit codes (Eq. 2, B = 4): MHA, ragged tail
    (1, 8, 2, 2112, synth.BF16, 4, 64, 96, 64),      # 4-bit, GQA 4:1, g = R = 64
    (1, 8, 1, 900, synth.BF16, 4, 128, 40, 256),     # 4-bit, g128, GQA 8:1 (16 query rows per KV head)
    (1, 4, 2, 1300, synth.FP16, 4, 32, 64, 96),      # 4-bit, GQA 2:1, R = 96
    (1, 2, 1, 700, synth.FP16, 4, 128, 32, 128),     # 4-bit, g128, GQA 2:1
])
def test_small_configs(B, Hq, Hkv, S, dtype, bits, g, k, R):
    from tests.harness import Case
    stats = _run(Case(B, Hq, Hkv, S, dtype, bits, g, k, R=R, seed=2000 + S), steps=3)
    print(stats)


@pytest.mark.parametrize("dtype,bits,g", [(synth.FP16, 2, 32), (synth.BF16, 2, 64), (synth.FP16, 1, 32), (synth.BF16, 1, 64),
                                          (synth.FP16, 2, 128), (synth.BF16, 1, 128),
                                          (synth.FP16, 4, 32), (synth.BF16, 4, 64), (synth.FP16, 4, 128)])
def test_quantiser_on_rounding_boundaries(dtype, bits, g):
    """Inputs on a grid of half quantisation steps (and their 16-bit neighbours), constant groups and groups
    with tiny ranges: the quotients of Eq. 2 / Eq. 3 land exactly on, or one rounding away from, the
    round-half-up boundaries, where codes have to stay bit-exact."""
    from tests.harness import Case
    c = Case(1, 2, 2, 1024, dtype, bits, g, 16, R=max(64, g), seed=4242)
    rng = np.random.default_rng(77)
    shape = c.k_bits.shape
    for name in ("k_bits", "v_bits"):
        m = rng.integers(0, {1: 5, 2: 7, 4: 31}[bits], size=shape)          # half steps of a unit-scale group
        e = rng.integers(-6, 5, size=(shape[0], shape[1], shape[2] // g, 1)).repeat(g, axis=2)
        if name == "v_bits":
            e = rng.integers(-6, 5, size=(shape[0], shape[1], shape[2], shape[3] // g)).repeat(g, axis=3)
        x = (m * 0.5) * np.exp2(e.astype(np.float64)) - (1.0 if bits == 1 else 0.0)
        b = synth.to_bits(x.astype(np.float32), dtype).astype(np.int32)
        b = b + rng.integers(-1, 2, size=shape) * (rng.random(shape) < 0.3)  # neighbours in the 16-bit format
        b[:, :, 2 * g:3 * g] = b[:, :, 2 * g:2 * g + 1]                       # constant key groups: s = 0
        b[:, :, 200:210, :] = b[:, :, 200:210, :1]                            # constant value groups
        b = np.where((b & 0x7FFF) >= (0x7C00 if dtype == synth.FP16 else 0x7F80), 0, b)   # no inf / nan
        setattr(c, name, b.astype(np.uint16))
    try:
        c.load()
        c.check_quantized()
        c.append_token(0)
        c.decode_step()
    finally:
        c.close()


def test_long_row_topk_in_two_launches_keeps_the_tie_rule():
    """A row longer than one workgroup's registers (> 65536 keys) is selected in two launches.  Keys repeat with
    period 32, so every group quantises alike and the scores form 32 classes of exactly equal values: the k-th
    boundary falls inside a class and ArgTopK has to keep that class's lowest positions, across the ranges."""
    from tests.harness import Case
    S, k = 70000, 3000
    c = Case(1, 1, 1, S, synth.FP16, 2, 32, k, seed=555, n_rows=2)
    c.k_bits = np.ascontiguousarray(c.k_bits[:, :, np.arange(S) % 32])
    try:
        c.load()
        c.append_token(0)
        c.decode_step()
        assert c.stats["band_diffs"] == 0, c.stats
        _, nq = c.sc.counts(0)
        assert nq > 65536
    finally:
        c.close()


@pytest.mark.parametrize("case", ["ties_top_class", "ties_second_class", "all_equal", "crowded", "gqa", "one_row_short"])
def test_topk_on_structured_scores(case):
    """ArgTopK on score patterns that stress the radix select and its tie rule: keys that repeat with period 32
    (32 classes of exactly equal scores: the boundary falls inside the top class, whose lowest positions have to
    win); period 64 with the boundary in the second class, in a row long enough for the two-launch selection;
    all keys equal; 1200 large keys crowded into 38 consecutive sub-groups of 32; four query heads per KV head
    with 1-bit codes; and one short row."""
    from tests.harness import Case
    kw = dict(B=1, Hq=1, Hkv=1, dtype=synth.FP16, bits=2, g=32, n_rows=2)
    period = None
    if case == "ties_top_class":
        S, k, period = 70000, 500, 32
    elif case == "ties_second_class":
        S, k, period = 200000, 4000, 64
    elif case == "all_equal":
        S, k, period = 70000, 500, 1
    elif case == "crowded":
        S, k = 40000, 600
    elif case == "gqa":
        S, k = 40000, 300
        kw.update(Hq=4, Hkv=1, dtype=synth.BF16, bits=1)
    else:
        S, k = 4096, 64
    c = Case(kw["B"], kw["Hq"], kw["Hkv"], S, kw["dtype"], kw["bits"], kw["g"], k, seed=560 + len(case), n_rows=2)
    if period:
        c.k_bits = np.ascontiguousarray(c.k_bits[:, :, np.arange(S) % period])
    if case == "crowded":
        u = np.where(np.random.default_rng(7).random(128) < 0.5, -8.0, 8.0).astype(np.float32)
        hot = np.stack([u if i % 2 == 0 else -u for i in range(1200)])
        c.k_bits[0, 0, 1024:1024 + 1200] = synth.to_bits(hot, kw["dtype"]).reshape(1200, 128)
    try:
        c.load()
        for t in range(2):
            c.append_token(t)
            c.decode_step(check_logits=False)
        if period:
            assert c.stats["band_diffs"] == 0, c.stats
        print(case, c.stats)
    finally:
        c.close()


@pytest.mark.parametrize("Hq,Hkv,dtype,bits,g", [(8, 2, synth.BF16, 2, 64), (8, 2, synth.FP16, 1, 32), (8, 1, synth.BF16, 2, 32)])
def test_matrix_core_value_path_keeps_fp32_accuracy(Hq, Hkv, dtype, bits, g):
    """With 8 or 16 query rows per KV head the value side of attend runs on the matrix cores with f16 operands
    (codes as subnormals, p*s split into hi + lo).  That has to stay as accurate as the fp32 vector path (errors
    of a few 1e-6): an operand split that loses its low part, or codes left in the low bits of their subnormal,
    shows as a few 1e-4, far inside the 2e-3 bar but a defect all the same."""
    from tests.harness import Case
    c = Case(1, Hq, Hkv, 3000, dtype, bits, g, 64, seed=4100 + bits * 10 + g)
    try:
        c.load()
        for t in range(2):
            c.append_token(t)
            c.decode_step()
        assert c.stats["max_out_err"] < 5e-5, c.stats
    finally:
        c.close()


@pytest.mark.parametrize("dtype,bits,g,spread", [(synth.FP16, 2, 32, 1.0), (synth.BF16, 1, 64, 1.0), (synth.FP16, 2, 32, 4096.0),
                                                  (synth.BF16, 2, 64, 4096.0)])
def test_integer_matrix_core_scoring_keeps_fp32_accuracy(dtype, bits, g, spread):
    """One query head per KV head, two rows: scoring runs on the integer matrix cores with the folded multipliers
    q*s as 32-bit fixed point relative to the largest of their (row, token group).  The logits have to stay as
    close to the oracle as an fp32 accumulation (a few 1e-7 of the largest logit); a lost byte plane, a wrong
    byte sign or a scale taken from the wrong group shows as 1e-3 or more.  spread > 1: the key channels get
    magnitudes from 1 to `spread` (a token group's multipliers then span 12 binary orders), which is where a
    fixed-point format with too few bits would lose the small channels."""
    from tests.harness import Case
    c = Case(1, 3, 3, 2500, dtype, bits, g, 64, seed=4300 + bits * 10 + g, n_outlier=4 if spread == 1.0 else 0)
    try:
        if spread > 1.0:
            scale = np.exp2(np.floor(np.linspace(0.0, np.log2(spread), 128))).astype(np.float32)
            rng = np.random.default_rng(7)
            for h in range(3):
                kf = synth.from_bits(c.k_bits[0, h], dtype) * scale[rng.permutation(128)][None, :]
                c.k_bits[0, h] = synth.to_bits(kf, dtype)
        c.load()
        for t in range(2):
            c.append_token(t)
            c.decode_step()
        assert c.stats["max_logit_err"] < 2e-6, c.stats
    finally:
        c.close()


@pytest.mark.parametrize("dtype,bits,g,one_pass", [(synth.FP16, 2, 32, False), (synth.BF16, 2, 64, True), (synth.FP16, 1, 32, True),
                                                    (synth.BF16, 1, 128, False)])
def test_integer_matrix_core_value_side_with_token_scales_far_apart(dtype, bits, g, one_pass):
    """One query head per KV head, two rows: the value side of attention runs on the integer matrix cores with p*s as
    32-bit fixed point relative to the largest value scale of a wave's 128 tokens.  Here the tokens' value
    magnitudes span 12 binary orders, so a wave mixes scales 4096 apart: a token of small scale and large weight
    is then held to 2^-18 of its own size.  The output has to stay far inside the 2e-3 bar (measured: 1e-6 to 7e-6)."""
    from tests.harness import Case
    if one_pass:
        binding.debug_kernel_choice(binding.KEEP_ONE_PASS_LOGITS)
    c = Case(1, 3, 3, 2500, dtype, bits, g, 64, R=max(64, g), seed=4500 + bits * 10 + g,
             **(dict(async_select=2, one_pass=True) if one_pass else {}))
    try:
        rng = np.random.default_rng(11)
        for h in range(3):
            scale = np.exp2(rng.integers(0, 13, size=c.v_bits.shape[2])).astype(np.float32)      # per token
            vf = synth.from_bits(c.v_bits[0, h], dtype) * scale[:, None]
            c.v_bits[0, h] = synth.to_bits(vf, dtype)
        c.load()
        for t in range(3):
            c.append_token(t)
            c.decode_step()
        print(c.stats)
        assert c.stats["max_out_err"] < 5e-5, c.stats
    finally:
        c.close()
        binding.debug_kernel_choice(0)


@pytest.mark.parametrize("bits,g,R", [(2, 32, 64), (1, 64, 128), (2, 128, 128), (4, 32, 64), (4, 128, 256)])
def test_long_decode_crosses_flushes(bits, g, R):
    """70 decode steps from a short prompt: the residual ring wraps and groups are flushed during decoding
    (every g steps), each step checked against the oracle, the whole quantised prefix and the offloaded rows
    at the end."""
    from tests.harness import Case
    c = Case(1, 4, 2, 200, synth.FP16, bits, g, 24, R=R, seed=6100 + g)
    try:
        c.load()
        n0, nq0 = c.check_quantized()
        for t in range(70):
            c.append_token(t)
            c.decode_step()
        n1, nq1 = c.check_quantized()
        assert n1 == n0 + 70 and nq1 >= nq0 + 64 - (64 % g)
        c.check_offload(first=c.S, count=70)
    finally:
        c.close()


@pytest.mark.timeout(600)
@pytest.mark.parametrize("dtype,g,R", [(synth.FP16, 32, 64), (synth.BF16, 64, 128)])
def test_one_call_layer_step_over_many_steps_and_chunk_boundaries(dtype, g, R):
    """720 decode steps through specache_append_score_attend + specache_select_gather from a 900-token prompt:
    the quantised prefix grows across two 512-token chunk boundaries (1024, 1536), the residual ring wraps many
    times, every g-th step flushes (the append then runs as a launch of its own).  Every step against the oracle."""
    from tests.harness import Case
    binding.debug_kernel_choice(binding.KEEP_ONE_PASS_LOGITS)     # for the steps whose logits are compared
    c = Case(1, 2, 2, 900, dtype, 2, g, 48, R=R, seed=6400 + g, async_select=2, one_pass=True, fused_append=True, max_seq=1664)
    try:
        c.load()
        n0, _ = c.check_quantized()
        for t in range(720):
            c.append_token(t)
            c.decode_step(check_logits=(t % 16 == 0))
        n1, nq1 = c.check_quantized()
        assert n1 == n0 + 720 and nq1 >= 1536
        c.check_offload(first=c.S, count=720)
        print(c.stats)
    finally:
        c.close()
        binding.debug_kernel_choice(0)


def test_streamed_load_equals_bulk_load():
    """Loading the prompt in uneven pieces and token by token reaches the same quantised state."""
    from tests.harness import Case
    c = Case(1, 2, 2, 333, synth.FP16, 2, 32, 16, seed=2100)
    _run(c, steps=2, chunks=[1, 2, 50, 63, 64, 65, 200, 201, 202, 203, 204, 300])


def test_pre_decoding_single_row():
    """n_rows = 1 (Appendix A "Pre-decoding"): selection on the only row, nothing prefetched."""
    from tests.harness import Case
    c = Case(1, 4, 2, 700, synth.FP16, 2, 32, 50, seed=2200, n_rows=1)
    try:
        c.load()
        c.decode_step(use_spec=False, do_gather=False)
    finally:
        c.close()


def test_non_speculative_fetching():
    """Section 4.4 / Table 4 ablation: top-k from the current token, fetched before its own attention."""
    from tests.harness import Case
    for (Hq, Hkv, bits, g) in ((2, 2, 2, 32), (8, 2, 1, 32)):
        c = Case(1, Hq, Hkv, 1000, synth.FP16, bits, g, 48, seed=2250, n_rows=1)
        try:
            c.load()
            for t in range(2):
                c.append_token(t)
                c.nonspec_step()
        finally:
            c.close()


def test_slot_reuse_orders_gather_after_attend():
    """A slot is gathered again (a) without a new selection in between and (b) after an attend that ran on a
    stream of its own: both orderings go through the library's events rather than through stream order."""
    from tests.harness import Case, check_out, to_dev
    c = Case(1, 4, 2, 1500, synth.FP16, 2, 32, 40, seed=2280)
    try:
        c.load()
        c.decode_step()                       # t = 0: gathers into slot 1
        c.decode_step()                       # t = 1: attend reads slot 1, gathers into slot 0
        t = 1
        q_bits = synth.make_queries(c.seed, 1, 4, 128, c.dtype, n_rows=2, sub=t)
        ks_bits, vs_bits = synth.make_spec_kv(c.seed, 1, 2, 128, c.dtype, sub=t)
        q, ks, vs = to_dev(q_bits, c.dtype), to_dev(ks_bits, c.dtype), to_dev(vs_bits, c.dtype)
        main, other = torch.cuda.current_stream(), torch.cuda.Stream()
        _, nq = c.sc.counts(0)
        picks = [np.arange(40, dtype=np.int32) * 3 + 1, np.arange(40, dtype=np.int32) * 7 + 2]
        assert picks[1].max() < nq
        for rnd, P in enumerate(picks):
            idx = torch.from_numpy(np.broadcast_to(P, (1, 2, 40)).copy()).cuda()
            c.sc.gather(0, idx, 1, c.side)    # slot 1 again; the last selection is older than its last attend
            out = torch.empty((1, 4, 2, 128), dtype=torch.float32, device="cuda")
            st = main if rnd == 0 else other  # second round: the reader runs on a third stream
            st.wait_stream(main)
            c.sc.attend(0, q, 2, ks, vs, 1, out, st)
            torch.cuda.synchronize()
            out_h = out.cpu().numpy()
            for (b, h) in c.sample:
                ref = c.oc[(b, h)].attend(q_bits[b, h * 2:(h + 1) * 2], c.sm_scale, P=P, k_spec=ks_bits[b, h, 0],
                                          v_spec=vs_bits[b, h, 0])
                check_out(out_h[b, h * 2:(h + 1) * 2], ref, what=f"re-gathered slot, round {rnd}, {(b, h)}")
        idx = torch.from_numpy(np.broadcast_to(picks[0], (1, 2, 40)).copy()).cuda()
        c.sc.gather(0, idx, 1, c.side)        # after the attend on `other`: waits for its recorded event
        c.decode_step()                       # t = 2 reads slot 0 and carries on as usual
    finally:
        c.close()


@pytest.mark.parametrize("Hq,Hkv,dtype,g", [(2, 2, synth.FP16, 32), (4, 2, synth.BF16, 64), (8, 1, synth.BF16, 32)])
def test_unmodified_one_bit_kivi(Hq, Hkv, dtype, g):
    """one_bit_form = SPECACHE_1BIT_KIVI: Eq. 2 with B = 1 (Section 4.4 / Table 5, "original").  Codes, stored
    extremes and derived (s, z) bit-exact, scores, selection and attention against the oracle's same form; the
    three shapes take the three scoring kernels."""
    from tests.harness import Case
    c = Case(1, Hq, Hkv, 1300, dtype, 1, g, 48, seed=2600 + g, one_bit_form=1)
    try:
        c.load()
        c.check_quantized()
        for t in range(3):
            c.decode_step()
            c.append_token(t)
        c.check_quantized()
    finally:
        c.close()
    if Hq == Hkv:
        # the same form through the call that scores and attends in one launch, the append carried
        binding.debug_kernel_choice(binding.KEEP_ONE_PASS_LOGITS)
        c = Case(1, Hq, Hkv, 1300, dtype, 1, g, 48, seed=2600 + g, one_bit_form=1, async_select=2, one_pass=True, fused_append=True)
        try:
            c.load()
            for t in range(40):
                c.append_token(t)
                c.decode_step(check_logits=(t % 8 == 0))
            c.check_quantized()
        finally:
            c.close()
            binding.debug_kernel_choice(0)
    with pytest.raises(binding.SpeCacheError):
        binding.SpeCache(1, 1, 1, 1, 1, 32, 256, 8, synth.FP16, one_bit_form=2)


@pytest.mark.parametrize("Hq,Hkv,dtype,bits,g,n_rows", [(4, 2, synth.FP16, 2, 32, 2), (8, 2, synth.BF16, 1, 32, 2), (8, 1, synth.BF16, 2, 64, 2),
                                                         (4, 1, synth.FP16, 2, 32, 1), (2, 2, synth.FP16, 2, 32, 2)])
def test_log_probability_selection(Hq, Hkv, dtype, bits, g, n_rows):
    """select_form = SPECACHE_SELECT_MAX_LOGPROB: the heads of a KV head are compared by their log-probabilities over
    the low-bit positions (the oracle's same form decides what has to be selected)."""
    from tests.harness import Case
    from oracle import oracle as orc
    c = Case(1, Hq, Hkv, 2100, dtype, bits, g, 40, seed=2700 + Hq + g, n_rows=n_rows, select_form=1)
    G = Hq // Hkv
    if G > 1:      # the first head of every KV head asks four times as loudly: the two forms then disagree
        c.q_head_scale = [4.0 if h % G == 0 else 1.0 for h in range(Hq)]
    try:
        c.load()
        for t in range(3):
            c.decode_step(use_spec=n_rows == 2, do_gather=n_rows == 2)
            c.append_token(t)
        if G > 1:  # the check above has teeth: on these inputs the max-of-logits form selects another set
            qh = c.last_q_bits[0, :G]
            _, s_logit = c.oc[(0, 0)].scores(qh, c.sm_scale, orc.SELECT_MAX_LOGIT)
            _, s_prob = c.oc[(0, 0)].scores(qh, c.sm_scale, orc.SELECT_MAX_LOGPROB)
            assert len(set(orc.topk(s_logit, 40).tolist()) & set(orc.topk(s_prob, 40).tolist())) < 30
    finally:
        c.close()
    with pytest.raises(binding.SpeCacheError):
        binding.SpeCache(1, 1, 1, 1, 2, 32, 256, 8, synth.FP16, select_form=3)


@pytest.mark.parametrize("Hq,Hkv,dtype,bits,g,form", [(2, 2, synth.FP16, 2, 32, 0), (8, 2, synth.BF16, 1, 32, 0), (4, 2, synth.FP16, 2, 64, 1)])
def test_selection_on_the_mixed_cache(Hq, Hkv, dtype, bits, g, form):
    """select_cache = SPECACHE_SELECT_MIXED: the staged positions are scored with their 16-bit keys (logits and
    selection against the oracle's mixed-cache scores), alone and together with the log-probability form."""
    from tests.harness import Case
    c = Case(1, Hq, Hkv, 1900, dtype, bits, g, 56, seed=2800 + Hq + g, select_form=form, select_cache=1)
    try:
        c.load()
        for t in range(4):
            c.decode_step()
            c.append_token(t)
        assert c.staged_idx is not None
    finally:
        c.close()
    with pytest.raises(binding.SpeCacheError):
        binding.SpeCache(1, 1, 1, 1, 2, 32, 256, 8, synth.FP16, select_cache=2)


@pytest.mark.parametrize("async_select", [0, 1, 2])
def test_layers_alternating_two_side_streams(async_select):
    """Four layers stepped in turn, their gathers alternating between two side streams (two gathers are then in
    flight at a time and the library paces them for a shared link), with ArgTopK on the caller's stream, on the
    library's own, or on the gather's (the score / select_gather pair of calls).  Two steps are enqueued back to
    back before the host looks at anything, so that the library's own ordering carries the dependencies between
    them.  Every layer holds the same cache and gets the same queries, so every layer's selection and output must
    match the one oracle cache."""
    from oracle import oracle as orc
    from tests.harness import check_out, check_topk, to_dev
    layers, Hq, S, k, dtype, seed = 4, 3, 2300, 72, synth.FP16, 2900
    sc = binding.SpeCache(layers, 1, Hq, Hq, 2, 32, 2432, k, dtype, async_select=async_select)
    try:
        kb, vb = synth.make_kv(seed, 1, Hq, S, 128, dtype)
        oc = [orc.Cache(128, 2, 32, 64, dtype) for _ in range(Hq)]
        for h in range(Hq):
            oc[h].append(kb[0, h], vb[0, h])
        main, sides = torch.cuda.current_stream(), [torch.cuda.Stream(), torch.cuda.Stream()]
        for L in range(layers):
            sc.quantize_append(L, to_dev(kb, dtype), to_dev(vb, dtype), S)
        idx = [[torch.full((1, Hq, k), -7, dtype=torch.int32, device="cuda") for _ in range(2)] for _ in range(layers)]
        out = [[torch.empty((1, Hq, 2, 128), dtype=torch.float32, device="cuda") for _ in range(2)] for _ in range(layers)]
        prev = None
        sm = 1.0 / np.sqrt(128.0)
        pending = []
        for t in range(6):
            q_bits = synth.make_queries(seed, 1, Hq, 128, dtype, n_rows=2, sub=t)
            ks_bits, vs_bits = synth.make_spec_kv(seed, 1, Hq, 128, dtype, sub=t)
            nk, nv = synth.make_step_kv(seed, t, 1, Hq, 128, dtype)
            q, ks, vs = to_dev(q_bits, dtype), to_dev(ks_bits, dtype), to_dev(vs_bits, dtype)
            nkd, nvd = to_dev(nk, dtype), to_dev(nv, dtype)
            for L in range(layers):
                sc.quantize_append(L, nkd, nvd, 1, main)
                if async_select == 2:
                    sc.score(L, q, 2, main)
                    sc.select_gather(L, idx[L][t % 2], (t + 1) % 2, sides[L % 2])
                else:
                    sc.score_topk(L, q, 2, idx[L][t % 2], main)
                    sc.gather(L, idx[L][t % 2], (t + 1) % 2, sides[L % 2])
                sc.attend(L, q, 2, ks, vs, (t % 2) if t > 0 else -1, out[L][t % 2], main)
            pending.append((t, q_bits, ks_bits, vs_bits, nk, nv, (q, ks, vs, nkd, nvd)))
            if t % 2 == 0:
                continue
            torch.cuda.synchronize()
            for (tt, q_bits, ks_bits, vs_bits, nk, nv, _) in pending:
                for h in range(Hq):
                    oc[h].append(nk[0, h], nv[0, h])
                cur = [idx[L][tt % 2].cpu().numpy() for L in range(layers)]
                for h in range(Hq):
                    qh = q_bits[0, h:h + 1]
                    _, sigma = oc[h].scores(qh, sm)
                    ref = oc[h].attend(qh, sm, P=prev[0][0, h] if prev is not None else None, k_spec=ks_bits[0, h, 0],
                                       v_spec=vs_bits[0, h, 0])
                    for L in range(layers):
                        check_topk(sigma, cur[L][0, h], k, what=f"layer {L} head {h} step {tt}")
                        check_out(out[L][tt % 2].cpu().numpy()[0, h:h + 1], ref, what=f"layer {L} head {h} step {tt}")
                for L in range(1, layers):
                    assert np.array_equal(cur[L], cur[0])
                prev = cur
            pending = []
    finally:
        torch.cuda.synchronize()
        sc.close()


@pytest.mark.parametrize("Hq,Hkv,dtype,bits,g,form,mixed", [(2, 2, synth.FP16, 2, 32, 0, 0), (8, 2, synth.BF16, 1, 32, 1, 1),
                                                             (4, 2, synth.FP16, 2, 64, 0, 1)])
def test_selection_on_a_stream_of_its_own(Hq, Hkv, dtype, bits, g, form, mixed):
    """async_select = 1: ArgTopK runs beside the attention kernels on a stream of the library.  Same results as on
    the caller's stream, through the speculative flow, the non-speculative one (gather on the main stream) and across
    flushes (the shared key array is written by the next scoring pass only after the selection has read it)."""
    from tests.harness import Case
    c = Case(1, Hq, Hkv, 1700, dtype, bits, g, 48, seed=3000 + Hq + g, select_form=form, select_cache=mixed, async_select=1)
    try:
        c.load()
        for t in range(40):
            c.append_token(t)
            if t % 8 == 0 or t > 36:
                c.decode_step()
            else:
                c.decode_step(check_logits=False)
        c.check_quantized()
    finally:
        c.close()
    c = Case(1, 2, 2, 900, synth.FP16, 2, 32, 24, seed=3050, n_rows=1, async_select=1)
    try:
        c.load()
        for t in range(3):
            c.append_token(t)
            c.nonspec_step()
    finally:
        c.close()


@pytest.mark.parametrize("Hq,Hkv,dtype,bits,g,form,mixed", [(2, 2, synth.FP16, 2, 32, 0, 0), (8, 2, synth.BF16, 1, 32, 1, 1),
                                                             (4, 2, synth.FP16, 2, 128, 0, 1)])
def test_selection_on_the_gathers_stream(Hq, Hkv, dtype, bits, g, form, mixed):
    """async_select = 2: the caller scores with specache_score and hands ArgTopK and the gather to the side stream
    in one call (specache_select_gather).  Same results as the other two arrangements across flushes; the
    non-speculative flow (gather on the main stream) still goes through specache_score_topk in such a context."""
    from tests.harness import Case
    c = Case(1, Hq, Hkv, 1700, dtype, bits, g, 48, R=max(64, g), seed=3100 + Hq + g, select_form=form, select_cache=mixed,
             async_select=2)
    try:
        c.load()
        for t in range(40):
            c.append_token(t)
            if t % 8 == 0 or t > 36:
                c.decode_step()
            else:
                c.decode_step(check_logits=False)
        c.check_quantized()
    finally:
        c.close()
    c = Case(1, 2, 2, 900, synth.FP16, 2, 32, 24, seed=3150, n_rows=1, async_select=2)
    try:
        c.load()
        for t in range(3):
            c.append_token(t)
            c.nonspec_step()
    finally:
        c.close()


@pytest.mark.parametrize("Hq,Hkv,dtype,bits,g,R", [(2, 2, synth.FP16, 2, 32, 64),      # integer matrix-core scoring kernel
                                                    (8, 2, synth.BF16, 1, 32, 64),      # 8 rows per KV head: matrix-core kernel
                                                    (4, 2, synth.FP16, 2, 64, 128),     # vector-ALU kernel
                                                    (3, 3, synth.BF16, 2, 128, 128)])
def test_append_carried_by_the_scoring_launch(Hq, Hkv, dtype, bits, g, R):
    """specache_append_score: the new token's pair reaches the host copy and the residual from inside the scoring
    launch (one extra workgroup per row) on steps that flush nothing, and through the two separate steps on the
    others.  80 decode steps cross several flushes; every step's selection and attention output (the residual
    holds the newest token) are checked against the oracle, and at the end the quantised prefix and every
    offloaded row."""
    from tests.harness import Case
    c = Case(1, Hq, Hkv, 1000, dtype, bits, g, 40, R=R, seed=3400 + Hq + g, async_select=2, fused_append=True)
    try:
        c.load()
        for t in range(80):
            c.append_token(t)
            c.decode_step(check_logits=(t % 16 == 0))
        c.check_quantized()
        c.check_offload(first=c.S, count=80)
        assert c.sc.counts(0)[0] == 1080
    finally:
        c.close()


@pytest.mark.parametrize("Hq,Hkv,S,dtype,bits,g,R,k", [
    (2, 2, 1700, synth.FP16, 2, 32, 64, 48),        # ragged tail: 1664 quantised positions = 3 chunks and a quarter
    (3, 3, 2100, synth.BF16, 2, 64, 64, 300),       # g = 64: one value group per channel set
    (2, 2, 1300, synth.FP16, 2, 128, 128, 40),      # g = 128: one value group per token
    (1, 1, 90, synth.BF16, 2, 32, 64, 16),          # 32 quantised positions: one wave of one chunk, three empty waves
    (2, 2, 5000, synth.FP16, 2, 32, 64, 700),       # index list longer than a wave walks: the workgroup-wide bitmap
    (4, 2, 1500, synth.FP16, 2, 32, 64, 32),        # two query heads per KV head: the two calls one after the other
    (2, 2, 1500, synth.BF16, 1, 32, 64, 32),        # 1-bit codes: eight channels per code byte, one word per token step
    (3, 3, 2100, synth.FP16, 1, 64, 128, 300),      # 1 bit, g = 64, workgroup-wide bitmap
    (2, 2, 1300, synth.BF16, 1, 128, 128, 40),      # 1 bit, g = 128
    (1, 1, 90, synth.FP16, 1, 32, 64, 16),          # 1 bit, one wave of one chunk
    (2, 2, 1700, synth.FP16, 4, 32, 64, 48),        # 4-bit codes: the two calls one after the other
])
@pytest.mark.parametrize("carry_append", [False, True])
def test_scoring_and_attention_in_one_pass(Hq, Hkv, S, dtype, bits, g, R, k, carry_append):
    """specache_score_attend: one launch scores a chunk's packed keys, keeps the logits on the chip and reads the
    chunk's packed values (one query head per KV head, two rows, 2-bit codes); other shapes run the two calls.
    40 decode steps across flushes; every step's selection, logits (kept on request) and output against the oracle.
    carry_append: specache_append_score_attend, the same launch also appends the step's new token (on the steps
    that flush nothing); the offloaded rows are compared at the end."""
    from tests.harness import Case
    binding.debug_kernel_choice(binding.KEEP_ONE_PASS_LOGITS)
    c = Case(1, Hq, Hkv, S, dtype, bits, g, k, R=R, seed=3600 + Hq + g + bits, async_select=2, one_pass=True,
             fused_append=carry_append)
    try:
        c.load()
        c.decode_step()                      # nothing staged yet (slot -1)
        for t in range(40):
            c.append_token(t)
            c.decode_step(check_logits=(t % 8 == 0))
        c.check_quantized()
        c.check_offload(first=c.S, count=40)
        assert c.sc.counts(0)[0] == S + 40
        print(c.stats)
    finally:
        c.close()
        binding.debug_kernel_choice(0)
    # without the request the logits are not kept, and the plain attend says so
    c = Case(1, 2, 2, 700, synth.FP16, 2, 32, 24, seed=3650, async_select=2, one_pass=True)
    try:
        c.load()
        c.decode_step(check_logits=False)
        with pytest.raises(binding.SpeCacheError) as ei:
            c.sc.debug_logits(0, 2)
        assert ei.value.code == binding.ESTATE
        q = torch.zeros((1, 2, 2, 128), dtype=torch.float16, device="cuda")
        out = torch.zeros((1, 2, 2, 128), dtype=torch.float32, device="cuda")
        with pytest.raises(binding.SpeCacheError) as ei:
            c.sc.attend(0, q, 2, None, None, -1, out)
        assert ei.value.code == binding.ESTATE
    finally:
        c.close()


@pytest.mark.parametrize("what", ["score", "attend", "both"])
def test_vector_alu_formulations_still_match(what):
    """The vector-ALU kernels that the integer-matrix-core kernels replaced for one query head per KV head and two
    rows stay reachable (A/B measurements): same parity bars."""
    from tests.harness import Case
    binding.debug_kernel_choice({"score": binding.SCORE_ON_VECTOR_ALU, "attend": binding.ATTEND_ON_VECTOR_ALU,
                                 "both": binding.SCORE_ON_VECTOR_ALU | binding.ATTEND_ON_VECTOR_ALU}[what])
    try:
        for (dtype, bits, g) in ((synth.FP16, 2, 32), (synth.BF16, 2, 64)):
            c = Case(1, 2, 2, 1700, dtype, bits, g, 48, seed=3700 + g)
            try:
                c.load()
                for t in range(3):
                    c.append_token(t)
                    c.decode_step()
            finally:
                c.close()
    finally:
        binding.debug_kernel_choice(0)


def test_repeated_selection_and_slot_refill_across_streams():
    """Call sequences a stepping loop does not produce, which the library still has to order: the same keys
    selected twice, on two side streams, into both slots; a slot refilled from another stream than its last
    gather; then the layer's next scoring pass, which overwrites those keys.  Every index list must equal the one
    a context with everything on the caller's stream produces, and attention on either slot the same output."""
    from tests.harness import to_dev
    S, k, dtype, seed, Hq = 5000, 200, synth.FP16, 3300, 2
    kb, vb = synth.make_kv(seed, 1, Hq, S, 128, dtype)
    main, sa, sb = torch.cuda.current_stream(), torch.cuda.Stream(), torch.cuda.Stream()
    res = {}
    for mode in (0, 2):
        sc = binding.SpeCache(1, 1, Hq, Hq, 2, 32, 5120, k, dtype, async_select=mode)
        try:
            sc.quantize_append(0, to_dev(kb, dtype), to_dev(vb, dtype), S)
            idx = [torch.full((1, Hq, k), -7, dtype=torch.int32, device="cuda") for _ in range(6)]
            outs = [torch.empty((1, Hq, 2, 128), dtype=torch.float32, device="cuda") for _ in range(4)]
            got = []
            for t in range(3):
                q = to_dev(synth.make_queries(seed, 1, Hq, 128, dtype, n_rows=2, sub=t), dtype)
                a, b = idx[2 * t], idx[2 * t + 1]
                if mode == 2:
                    sc.score(0, q, 2, main)
                    sc.select_gather(0, a, 0, sa)
                    sc.select_gather(0, b, 1, sb)       # same keys again, other stream, other slot
                    sc.gather(0, a, 1, sa)               # slot 1 refilled from the other stream
                else:
                    sc.score_topk(0, q, 2, a, main)
                    sc.score_topk(0, q, 2, b, main)
                    sc.gather(0, a, 0, main)
                    sc.gather(0, a, 1, main)
                sc.attend(0, q, 2, None, None, 0, outs[0], main)
                sc.attend(0, q, 2, None, None, 1, outs[1], main)
                torch.cuda.synchronize()
                got.append((a.cpu().numpy().copy(), b.cpu().numpy().copy(), outs[0].cpu().numpy().copy(), outs[1].cpu().numpy().copy()))
            res[mode] = got
        finally:
            torch.cuda.synchronize()
            sc.close()
    for (a0, b0, o00, o01), (a2, b2, o20, o21) in zip(res[0], res[2]):
        assert np.array_equal(a0, b0) and np.array_equal(a2, b2) and np.array_equal(a0, a2)
        assert np.array_equal(o00, o20) and np.array_equal(o01, o21) and np.array_equal(o00, o01)
        assert (a0 >= 0).sum() == Hq * k


def test_two_launch_selection_on_two_gather_streams():
    """async_select = 2 with rows long enough for the two-launch ArgTopK (> 65536 keys): the selections of
    consecutive layers run on different side streams and may overlap, each with candidate arrays of its own.
    Both layers hold the same cache, so both must select what the oracle does."""
    from oracle import oracle as orc
    from tests.harness import check_topk, to_dev
    S, k, dtype, seed, layers = 70000, 500, synth.FP16, 3200, 3
    sc = binding.SpeCache(layers, 1, 1, 1, 2, 32, 70144, k, dtype, async_select=2)
    try:
        kb, vb = synth.make_kv(seed, 1, 1, S, 128, dtype)
        oc = orc.Cache(128, 2, 32, 64, dtype)
        oc.append(kb[0, 0], vb[0, 0])
        main, sides = torch.cuda.current_stream(), [torch.cuda.Stream(), torch.cuda.Stream()]
        kd, vd = to_dev(kb, dtype), to_dev(vb, dtype)
        for L in range(layers):
            sc.quantize_append(L, kd, vd, S)
        assert sc.counts(0)[1] > 65536
        idx = [[torch.full((1, 1, k), -7, dtype=torch.int32, device="cuda") for _ in range(2)] for _ in range(layers)]
        out = torch.empty((1, 1, 2, 128), dtype=torch.float32, device="cuda")
        sm = 1.0 / np.sqrt(128.0)
        for t in range(3):
            q_bits = synth.make_queries(seed, 1, 1, 128, dtype, n_rows=2, sub=t)
            q = to_dev(q_bits, dtype)
            for L in range(layers):
                sc.score(L, q, 2, main)
                sc.select_gather(L, idx[L][t % 2], (t + 1) % 2, sides[L % 2])
                sc.attend(L, q, 2, None, None, (t % 2) if t > 0 else -1, out, main)
            torch.cuda.synchronize()
            _, sigma = oc.scores(q_bits[0, 0:1], sm)
            for L in range(layers):
                check_topk(sigma, idx[L][t % 2].cpu().numpy()[0, 0], k, what=f"layer {L} step {t}")
    finally:
        torch.cuda.synchronize()
        sc.close()


def test_short_cache_edges():
    """Nq = 0 (everything still in the residual), k > Nq, and a cache of one token."""
    from tests.harness import Case
    c = Case(1, 2, 1, 40, synth.BF16, 2, 32, 64, seed=2300)
    try:
        c.load()
        assert c.sc.counts(0) == (40, 0)
        idx, _ = c.decode_step()
        assert np.all(idx == -1)
        for t in range(30):          # crosses the first flush at N = 64
            c.append_token(t)
        assert c.sc.counts(0) == (70, 32)
        c.check_quantized()
        idx, _ = c.decode_step()
        assert np.array_equal(idx[0, 0, :32], np.arange(32)) and np.all(idx[0, 0, 32:] == -1)
        c.decode_step()              # uses the slot gathered with k_eff = 32 < k
    finally:
        c.close()
    c = Case(1, 1, 1, 1, synth.FP16, 1, 32, 8, seed=2301)
    try:
        c.load()
        c.decode_step()
    finally:
        c.close()


def test_all_positions_prefetched_matches_full_attention():
    """k >= Nq: every low-bit pair is replaced, so the GPU output equals textbook attention."""
    from tests.harness import Case
    from oracle import oracle as orc
    c = Case(1, 2, 2, 300, synth.FP16, 2, 32, 512, seed=2400)
    try:
        c.load()
        c.decode_step()
        _, out = c.decode_step()
        t = 1
        q_bits = synth.make_queries(c.seed, 1, 2, 128, c.dtype, sub=t)
        ks, vs = synth.make_spec_kv(c.seed, 1, 2, 128, c.dtype, sub=t)
        for h in range(2):
            ref = c.oc[(0, h)].full_attention(q_bits[0, h:h + 1], c.sm_scale, k_spec=ks[0, h, 0], v_spec=vs[0, h, 0])
            from tests.harness import check_out
            check_out(out[0, h:h + 1], ref, what="full attention")
    finally:
        c.close()


def test_error_paths():
    with pytest.raises(binding.SpeCacheError) as ei:        # rejected before anything is allocated
        binding.SpeCache(1, 1, 8, 1, 2, 32, 64 * 20000, 16, synth.FP16)
    assert ei.value.code == binding.EINVAL
    sc = binding.SpeCache(2, 1, 2, 2, 2, 32, 256, 16, synth.FP16)
    try:
        k = torch.zeros((1, 2, 300, 128), dtype=torch.float16, device="cuda")
        q = torch.zeros((1, 2, 2, 128), dtype=torch.float16, device="cuda")
        idx = torch.zeros((1, 2, 16), dtype=torch.int32, device="cuda")
        out = torch.zeros((1, 2, 2, 128), dtype=torch.float32, device="cuda")
        for fn, code in [
            (lambda: sc.quantize_append(0, k, k, 300), binding.ECAPACITY),
            (lambda: sc.quantize_append(5, k, k, 1), binding.EINVAL),
            (lambda: sc.quantize_append(0, None, k, 1), binding.EINVAL),
            (lambda: sc.score_topk(0, q, 3, idx), binding.EINVAL),
            (lambda: sc.gather(0, idx, 2), binding.EINVAL),
            (lambda: sc.attend(0, q, 2, None, None, -1, out), binding.ESTATE),   # nothing scored
            (lambda: sc.score(0, q, 2), binding.ESTATE),                         # context not created for that pair of calls
            (lambda: sc.select_gather(0, idx, 0), binding.ESTATE),
            (lambda: sc.append_score(0, k, k, q, 2), binding.ESTATE),
        ]:
            with pytest.raises(binding.SpeCacheError) as ei:
                fn()
            assert ei.value.code == code
        sc.quantize_append(0, k, k, 100)
        sc.score_topk(0, q, 2, idx)
        with pytest.raises(binding.SpeCacheError) as ei:
            sc.attend(0, q, 2, None, None, 0, out)                               # slot never gathered
        assert ei.value.code == binding.ESTATE
        with pytest.raises(binding.SpeCacheError) as ei:
            sc.attend(1, q, 2, None, None, -1, out)                              # other layer
        assert ei.value.code == binding.ESTATE
        sc.attend(0, q, 2, None, None, -1, out)
        torch.cuda.synchronize()
        assert sc.counts(0) == (100, 64) and sc.counts(1) == (0, 0)
    finally:
        sc.close()
    sc = binding.SpeCache(1, 1, 2, 2, 2, 32, 256, 16, synth.FP16, async_select=2)
    try:
        idx = torch.zeros((1, 2, 16), dtype=torch.int32, device="cuda")
        with pytest.raises(binding.SpeCacheError) as ei:
            sc.select_gather(0, idx, 0)                                          # nothing scored yet
        assert ei.value.code == binding.ESTATE
    finally:
        sc.close()
    for kwargs in [dict(bits=3), dict(bits=8), dict(group=48), dict(residual=48), dict(max_seq=100), dict(topk=0), dict(head_dim=64),
                   dict(n_q_heads=3, n_kv_heads=2)]:
        base = dict(n_layers=1, batch=1, n_q_heads=2, n_kv_heads=2, bits=2, group=32, max_seq=256, topk=16,
                    dtype=synth.FP16)
        base.update(kwargs)
        with pytest.raises(binding.SpeCacheError) as ei:
            binding.SpeCache(**base)
        assert ei.value.code == binding.EINVAL


@pytest.mark.timeout(600)
def test_very_long_row_with_the_largest_k():
    """600000 keys in one row (close to the longest the library takes) and k = 4096, the largest: ArgTopK runs as 16
    ranges of 37504 keys and a second launch over 65536 candidates, the attention as 1172 chunks of quantised tokens
    plus 33 of 16-bit pairs (limit 1280)."""
    from tests.harness import Case
    c = Case(1, 1, 1, 600000, synth.BF16, 1, 64, 4096, seed=3100)
    try:
        c.load()
        c.decode_step(check_logits=False)
        c.append_token(0)
        c.decode_step()
        assert c.sc.counts(0)[1] >= 599872
    finally:
        c.close()


# ---- the benchmark's full sizes, one layer, every call on the caller's stream with a host synchronise after
# ---- every step; the oracle mirrors a sample of distinct (batch, KV head) rows.  The arrangement bench.py times
# ---- (several layers free-running, side streams, every row compared) is tests/test_gpu_timed_arrangement.py.
FULL = {
    "config2": dict(B=1, Hq=32, Hkv=32, S=16384, dtype=synth.FP16, bits=2, g=32, k=256, sample=[(0, 0), (0, 13), (0, 31)]),
    "M0_7B_32k": dict(B=1, Hq=32, Hkv=32, S=32768, dtype=synth.FP16, bits=2, g=32, k=256, sample=[(0, 5), (0, 30)]),
    "config3": dict(B=16, Hq=32, Hkv=32, S=2048, dtype=synth.FP16, bits=2, g=32, k=128,
                    sample=[(0, 0), (7, 19), (15, 31), (3, 8)]),
    "config4": dict(B=4, Hq=32, Hkv=8, S=32768, dtype=synth.BF16, bits=2, g=64, k=512, sample=[(1, 2), (3, 7)]),
    "config5": dict(B=1, Hq=32, Hkv=8, S=131072, dtype=synth.BF16, bits=1, g=32, k=1024, sample=[(0, 6)]),
}


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name", list(FULL))
def test_full_size_sampled(name):
    from tests.harness import Case
    kw = dict(FULL[name])
    sample = kw.pop("sample")
    c = Case(kw["B"], kw["Hq"], kw["Hkv"], kw["S"], kw["dtype"], kw["bits"], kw["g"], kw["k"], seed=3000 + kw["S"],
             sample=sample)
    try:
        c.load()
        c.check_quantized()
        c.check_offload(first=kw["S"] - 70, count=70)
        for t in range(2):
            c.append_token(t)
            c.decode_step(check_logits=(t == 0))
        c.check_offload(first=kw["S"], count=2)
        print(name, c.stats)
    finally:
        c.close()


@pytest.mark.gpu
@pytest.mark.parametrize("async_select", [0, 1, 2])
def test_create_backs_out_of_every_failed_allocation(async_select):
    """specache_create with its n-th allocating call failing (device memory, the pinned host store, events, the
    library's stream), for every n: ENOMEM, no context, nothing left allocated; the create after it works."""
    import torch
    args = (2, 1, 4, 2, 2, 32, 70016, 64, synth.FP16)        # long enough for the two-launch ArgTopK's candidate arrays
    binding.SpeCache(*args, async_select=async_select).close()     # the library's code and static data are loaded
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    n = 1
    while True:
        binding.debug_fail_alloc(n)
        try:
            sc = binding.SpeCache(*args, async_select=async_select)
        except binding.SpeCacheError as e:
            assert e.code == binding.ENOMEM, (n, str(e))
            n += 1
            assert n < 200
            continue
        sc.close()            # n is past the last allocating call: the hook was consumed without effect
        break
    assert n > 40, n          # two layers: at least 18 allocating calls each
    torch.cuda.synchronize()
    assert abs(torch.cuda.mem_get_info()[0] - free0) < (64 << 20), "device memory of a failed create was not returned"
    binding.debug_fail_alloc(0)
    sc = binding.SpeCache(*args, async_select=async_select)
    sc.close()

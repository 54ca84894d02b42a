"""Benchmark of the SpeCache decode-step hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload M0|c1|c2|c3|c4|c5]

A step is one decode step of every layer of the workload: per layer
quantize_append (1 token) -> score_topk (2 query rows) -> gather (side stream,
next step's pairs) -> attend.  Inputs are synthetic and already resident in HBM
(the 16-bit copy C sits in pinned host memory, as the method prescribes).
Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# name: (B, Hq, Hkv, S, dtype, bits, g, k, layers)   dtype 0 = fp16, 1 = bf16
WORKLOADS = {
    "M0": (1, 32, 32, 32768, 0, 2, 32, 256, 32),
    "c1": (1, 1, 1, 4096, 0, 2, 32, 64, 1),
    "c2": (1, 32, 32, 16384, 0, 2, 32, 256, 32),
    "c3": (16, 32, 32, 2048, 0, 2, 32, 128, 4),
    "c4": (4, 32, 8, 32768, 1, 2, 64, 512, 4),
    "c5": (1, 32, 8, 131072, 1, 1, 32, 1024, 32),
}
DESCR = {
    "M0": "7B shape at 32k context: B=1, 32 MHA heads, D=128, S=32768, fp16, 2-bit g32, k=256, 32 layers",
    "c1": "config 1: B=1, 1 head, S=4096, fp16, 2-bit g32, k=64, 1 layer",
    "c2": "config 2: B=1, 32 MHA heads, S=16384, fp16, 2-bit g32, k=256, 32 layers",
    "c3": "config 3: B=16, 32 MHA heads, S=2048, fp16, 2-bit g32, k=128, 4 layers (512 MiB of host store each)",
    "c4": "config 4: B=4, 32/8 GQA heads, S=32768, bf16, 2-bit g64, k=512, 4 layers (512 MiB of host store each)",
    "c5": "config 5: B=1, 32/8 GQA heads, S=131072, bf16, 1-bit g32, k=1024, 32 layers",
}


def hit_rate_experiment(torch, binding, synth):
    """Selection quality of the low-bit scores, per quantiser: overlap of the selected set with the exact top-k of the
    same (speculative) query on the 16-bit keys, and the share of that query's exact attention mass the set holds.
    The exact side is a plain fp32 matmul + softmax in torch: a measuring stick, not part of the path."""
    B, H, S, D, g, seed = 1, 8, 32768, 128, 32, 1000
    rows = []
    for k in (64, 256, 1024):
        for bits, form, name in ((2, 0, "2-bit (Eq. 2)"), (1, 0, "1-bit (Eq. 3)"), (1, 1, "1-bit unmodified KIVI (Eq. 2, B = 1)")):
            sc = binding.SpeCache(1, B, H, H, bits, g, S + 64, k, synth.FP16, one_bit_form=form)
            kd, vd = synth.make_kv_device(seed, B, H, S, D, synth.FP16)
            sc.quantize_append(0, kd, vd, S)
            q = synth.make_queries_device(seed, 1, B, H, D, synth.FP16)[0]
            idx = torch.full((B, H, k), -1, dtype=torch.int32, device="cuda")
            sc.score_topk(0, q, 2, idx)
            torch.cuda.synchronize()
            nq = sc.counts(0)[1]
            exact = torch.einsum("bhd,bhsd->bhs", q[:, :, 1].float(), kd[:, :, :nq].float()) / D ** 0.5
            w = torch.softmax(exact, dim=-1)
            top = torch.topk(exact, k, dim=-1).indices
            sel = idx.long()
            hit = torch.zeros_like(exact, dtype=torch.bool).scatter_(-1, top, True).gather(-1, sel).float().mean().item()
            rows.append({"k": k, "quantiser": name, "overlap_with_exact_topk": round(hit, 4),
                         "attention_mass_selected": round(w.gather(-1, sel).sum(-1).mean().item(), 4),
                         "attention_mass_exact_topk": round(w.gather(-1, top).sum(-1).mean().item(), 4)})
            sc.close()
            del kd, vd
    print(json.dumps({"experiment": "selection from low-bit scores vs exact top-k, speculative row",
                      "data": "synthetic: K ~ N(0,1) with 4 key channels x10, q' = q + 0.1 N(0,1); 8 heads, 32768 keys, g = 32",
                      "rows": rows}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="M0", choices=sorted(WORKLOADS))
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers")
    ap.add_argument("--filler-mb", type=int, default=0,
                    help="EMULATION, not part of the method's path: after every layer's attend, stream this many MB of "
                         "stand-in weights through a plain torch reduction on the main stream (a 7B layer reads about "
                         "403 MB of fp16 weights per decode step), to see how much of the gather the rest of a model's "
                         "layer would hide")
    ap.add_argument("--topk", type=int, default=0,
                    help="override k, the number of prefetched pairs per (batch, KV head) (the k sweep of Section 4.4)")
    ap.add_argument("--group", type=int, default=0, choices=[0, 32, 64, 128],
                    help="override g, the quantisation group size (the residual becomes max(64, g))")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-gather", action="store_true", help="skip the host-link gather (attend sees nothing prefetched)")
    ap.add_argument("--serial-gather", action="store_true", help="issue the gather on the main stream (no overlap)")
    ap.add_argument("--side-streams", type=int, default=0,
                    help="side streams the gathers alternate over by layer; 0 = by the measured rule: with ArgTopK on the "
                         "gather's stream 2, or 3 where a fetched pair stands for fewer than 192 scored keys (a third "
                         "stream selects while two gathers share the link); otherwise 2 (two gathers share the link and "
                         "cover each other's launch gaps), or 1 from 384 scored keys per pair on, where the gather has "
                         "time to spare")
    ap.add_argument("--variant", default="speculative", choices=["speculative", "nonspec"],
                    help="nonspec: the non-speculative fetching of Section 4.4 (select on the current token, one query "
                         "row, gather on the main stream before attend): the whole link time is exposed")
    ap.add_argument("--compute-only-pass", action="store_true",
                    help="add two more passes of K steps that issue no gathers (attend keeps reading the pairs staged "
                         "by the last gather): wall time -> compute_us_layer, event timing -> kernel_us_no_gather")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy (3x), the known-size kernel the FETCH_SIZE/WRITE_SIZE "
                         "counters are scaled by")
    ap.add_argument("--select", default="logit", choices=["logit", "logprob"],
                    help="how the query heads of a KV head share one index set: largest logit (default) or largest "
                         "log-probability over the heads (two more small kernels per layer-step)")
    ap.add_argument("--select-cache", default="lowbit", choices=["lowbit", "mixed"],
                    help="which logits ArgTopK ranks: pure low-bit (default) or the mixed cache's (the staged positions "
                         "are scored with their 16-bit keys: one more small kernel per layer-step)")
    ap.add_argument("--select-stream", default="auto", choices=["auto", "own", "main", "gather"],
                    help="where ArgTopK runs (specache_config.async_select): on the main stream, on a stream of the "
                         "library's own beside the attention kernels, or on the gather's side stream ahead of the gather "
                         "(the specache_score / specache_select_gather pair of calls); auto = main for one layer and for the "
                         "non-speculative variant, else gather where a fetched pair stands for 96 or more scored keys "
                         "(the step is bound by compute and by the issuing thread) and own below that (bound by the link)")
    ap.add_argument("--fused-append", action="store_true",
                    help="with ArgTopK on the gather's stream: specache_append_score (the scoring launch carries the copy of "
                         "the new pair) instead of quantize_append and score as two calls.  1 to 3 us per layer faster; off "
                         "by default so that every step of the path keeps a kernel and a timing of its own")
    ap.add_argument("--one-pass", action="store_true",
                    help="with ArgTopK on the gather's stream: specache_score_attend (scoring and attention of a chunk in one "
                         "launch, the logits stay on the chip) instead of specache_score and specache_attend as two calls")
    ap.add_argument("--vector-alu", default="", choices=["", "score", "attend", "both"],
                    help="A/B measurement: run the named streaming kernel(s) in the vector-ALU formulation instead of the "
                         "integer-matrix-core one (one query head per KV head, two rows)")
    ap.add_argument("--hit-rate", action="store_true",
                    help="instead of the timing run: how well the positions selected from the low-bit scores of the "
                         "speculative row match the exact top-k on the 16-bit keys (synthetic stand-in for the "
                         "sparsity profile of Section 3.1), for 2-bit, 1-bit (Eq. 3) and unmodified 1-bit KIVI (Table 5)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2503_16163_amd import binding, synth

    assert torch.cuda.is_available(), "bench.py needs an MI355X"
    torch.cuda.set_device(0)
    if args.hit_rate:
        return hit_rate_experiment(torch, binding, synth)
    if args.vector_alu:
        binding.debug_kernel_choice({"score": binding.SCORE_ON_VECTOR_ALU, "attend": binding.ATTEND_ON_VECTOR_ALU,
                                     "both": binding.SCORE_ON_VECTOR_ALU | binding.ATTEND_ON_VECTOR_ALU}[args.vector_alu])
    B, Hq, Hkv, S, dtype, bits, g, k, layers = WORKLOADS[args.workload]
    if args.layers:
        layers = args.layers
    if args.topk:
        k = args.topk
    if args.group:
        g = args.group
    G, D, R = Hq // Hkv, 128, max(64, g)
    total_steps = args.warmup + 4 * args.steps + 2
    max_seq = ((S + total_steps + 63) // 64 + 1) * 64
    seed = 1000

    # Where ArgTopK runs (measured rule).  keys_per_pair says how much scoring work stands against one fetched
    # pair.  With much of it the step is bound by compute and by the issuing thread: ArgTopK then goes on the
    # gather's stream, which needs the fewest ordering calls between streams.  With little of it the step is
    # bound by the host link: ArgTopK on the library's own stream lets every gather start the moment its
    # selection is done.  One layer, or the non-speculative variant: everything on the main stream.
    from paper_2503_16163_amd import arrangement
    side_gathers = args.variant == "speculative" and not args.serial_gather and not args.no_gather
    auto_select, _ = arrangement.pick(G, S, k, layers, args.variant == "speculative", side_gathers)
    if args.select_stream == "auto":
        async_select = auto_select
    else:
        async_select = {"main": 0, "own": 1, "gather": 2 if side_gathers else 1}[args.select_stream]
    sc = None
    while sc is None:
        try:
            sc = binding.SpeCache(layers, B, Hq, Hkv, bits, g, max_seq, k, dtype, residual=R,
                                  select_form=1 if args.select == "logprob" else 0,
                                  select_cache=1 if args.select_cache == "mixed" else 0,
                                  async_select=async_select)
        except binding.SpeCacheError as e:
            if e.code != binding.ENOMEM or layers == 1:
                raise
            layers = max(1, layers // 2)   # the pinned host store did not fit: fewer layers
    main_s = torch.cuda.current_stream()
    n_side = args.side_streams if args.side_streams > 0 else arrangement.side_streams(async_select, G, S, k)
    side_list = [main_s] if args.serial_gather else [torch.cuda.Stream() for _ in range(n_side)]

    # ---- load the prompt: the same synthetic K/V tensor serves every layer ----------
    # This is the Quant + Offload of the prefilling procedure (Appendix A), timed per layer: the bulk
    # quantiser is HBM-bound, the copy to the pinned host store is bound by the host link.
    kd, vd = synth.make_kv_device(seed, B, Hkv, S, D, dtype)
    torch.cuda.synchronize()
    sc.timing(True)
    t0 = time.perf_counter()
    for L in range(layers):
        sc.quantize_append(L, kd, vd, S, main_s)
    torch.cuda.synchronize()
    load_wall_us = (time.perf_counter() - t0) * 1e6 / layers
    lt = sc.timing(False)
    n_flushed = sc.counts(0)[1]
    raw_bytes = B * Hkv * S * 512
    flush_us = lt["flush"][0] / lt["flush"][1] if lt["flush"][1] else None
    copy_us = lt["append_copy"][0] / lt["append_copy"][1] if lt["append_copy"][1] else None
    # bulk quantiser: reads the 16-bit pairs once, writes codes (bits/16 of that) and 32-bit (min, max) per group
    flush_bytes = B * Hkv * n_flushed * (512 + 2 * (128 * bits // 8) + 2 * 128 * 4 // g)
    prefill = {"us_per_layer": round(load_wall_us, 1), "tokens": S,
               "flush_us": round(flush_us, 1) if flush_us else None,
               "flush_gbs": round(flush_bytes / (flush_us * 1e-6) / 1e9, 1) if flush_us else None,
               "flush_frac_of_hbm_peak": round(flush_bytes / (flush_us * 1e-6) / 8e12, 3) if flush_us else None,
               "offload_us": round(copy_us, 1) if copy_us else None,
               "offload_gbs": round(raw_bytes / (copy_us * 1e-6) / 1e9, 1) if copy_us else None}
    sample = [(0, h) for h in sorted(set([0, Hkv // 3, (2 * Hkv) // 3, Hkv - 1]))]
    k_hist = {bh: [synth.bits_of(kd[bh[0], bh[1]])] for bh in sample}
    v_hist = {bh: [synth.bits_of(vd[bh[0], bh[1]])] for bh in sample}
    del kd, vd

    nq_pool = 8
    q_all = synth.make_queries_device(seed, nq_pool * layers, B, Hq, D, dtype).view(nq_pool, layers, B, Hq, 2, D)
    q1_all = q_all[:, :, :, :, :1].contiguous()   # current-token rows only (non-speculative variant)
    step_k, step_v = synth.make_kv_device(seed + 1, total_steps * B, Hkv, 1, D, dtype)
    step_k = step_k.view(total_steps, B, Hkv, 1, D).contiguous()
    step_v = step_v.view(total_steps, B, Hkv, 1, D).contiguous()
    spec_k, spec_v = synth.make_kv_device(seed + 2, B, Hkv, 1, D, dtype, n_outlier=0)
    idx = [[torch.full((B, Hkv, k), -1, dtype=torch.int32, device="cuda") for _ in range(2)] for _ in range(layers)]
    out = [torch.empty((B, Hq, 2, D), dtype=torch.float32, device="cuda") for _ in range(layers)]
    state = {"t": 0}
    filler = torch.ones(args.filler_mb * (1 << 20) // 2, dtype=torch.float16, device="cuda") if args.filler_mb else None
    filler_out = torch.empty((), dtype=torch.float16, device="cuda")

    # The step loop hands the library raw addresses and stream handles, as a serving loop would: building a
    # tensor view per call costs the issuing thread several microseconds per layer, which shows once the
    # step is short (small k).
    q_p = [[q_all[p, L].data_ptr() for L in range(layers)] for p in range(nq_pool)]
    q1_p = [[q1_all[p, L].data_ptr() for L in range(layers)] for p in range(nq_pool)]
    k_p = [step_k[t].data_ptr() for t in range(total_steps)]
    v_p = [step_v[t].data_ptr() for t in range(total_steps)]
    idx_p = [[idx[L][b].data_ptr() for b in range(2)] for L in range(layers)]
    out_p = [out[L].data_ptr() for L in range(layers)]
    spec_k_p, spec_v_p = spec_k.data_ptr(), spec_v.data_ptr()
    main_h = main_s.cuda_stream
    side_h = [s.cuda_stream for s in side_list]

    def step_nonspec():
        t = state["t"]
        for L in range(layers):
            q = q1_p[t % nq_pool][L]
            sc.quantize_append(L, k_p[t], v_p[t], 1, main_h)
            sc.score_topk(L, q, 1, idx_p[L][0], main_h)
            sc.gather(L, idx_p[L][0], 0, main_h)
            sc.attend(L, q, 1, None, None, 0, out_p[L], main_h)
        state["t"] = t + 1

    def step(gather=True):
        if args.variant == "nonspec":
            return step_nonspec()
        t = state["t"]
        do_gather = gather and not args.no_gather
        slot = (t % 2) if (t > 0 and not args.no_gather) else -1
        for L in range(layers):
            q = q_p[t % nq_pool][L]
            if async_select == 2 and args.one_pass:
                sc.quantize_append(L, k_p[t], v_p[t], 1, main_h)
                sc.score_attend(L, q, 2, spec_k_p, spec_v_p, slot, out_p[L], main_h)
                sc.select_gather(L, idx_p[L][t % 2], (t + 1) % 2 if do_gather else -1, side_h[L % len(side_h)])
                continue
            if async_select == 2:
                if not args.fused_append:
                    sc.quantize_append(L, k_p[t], v_p[t], 1, main_h)
                    sc.score(L, q, 2, main_h)
                else:
                    sc.append_score(L, k_p[t], v_p[t], q, 2, main_h)   # the scoring launch carries the append
                sc.select_gather(L, idx_p[L][t % 2], (t + 1) % 2 if do_gather else -1, side_h[L % len(side_h)])
            else:
                sc.quantize_append(L, k_p[t], v_p[t], 1, main_h)
                sc.score_topk(L, q, 2, idx_p[L][t % 2], main_h)
                if do_gather:
                    sc.gather(L, idx_p[L][t % 2], (t + 1) % 2, side_h[L % len(side_h)])
            sc.attend(L, q, 2, spec_k_p, spec_v_p, slot, out_p[L], main_h)
            if filler is not None:
                torch.sum(filler, dim=(0,), out=filler_out)
        state["t"] = t + 1

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    if args.calibrate_copy:
        src = torch.ones(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- same steps again with an event pair around every kernel phase -------------
    sc.timing(True)
    for _ in range(args.steps):
        step()
    kt = sc.timing(False)
    per_kernel_us = {n: (us / c if c else None) for n, (us, c) in kt.items()}

    # ---- optional: compute only, i.e. the same steps without issuing gathers (attend keeps
    # ---- reading the pairs staged by the last gather, so its work is unchanged) ----------------
    compute_ms, per_kernel_ng = None, None
    if args.compute_only_pass and not args.no_gather:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step(gather=False)
        torch.cuda.synchronize()
        compute_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        sc.timing(True)
        for _ in range(args.steps):
            step(gather=False)
        kt2 = sc.timing(False)
        per_kernel_ng = {n: (round(us / c, 3) if c else None) for n, (us, c) in kt2.items()}

    N, Nq = sc.counts(0)
    per_elem = (bits + 32.0 / g) / 8.0
    packed = B * Hkv * Nq * D * per_elem                       # packed K (or V) incl. metadata
    score_bytes = packed
    attend_bytes = packed + B * Hkv * ((k if not args.no_gather else 0) + (N - Nq) + 1) * 512
    layer_bytes = score_bytes + attend_bytes
    us_layer = ms_per_step * 1e3 / layers
    score_us = per_kernel_us["score"] or per_kernel_us["score_attend"]
    # which scoring kernel the library launches for this shape (two query rows per query head)
    score_name = ("score_i8_kernel" if G == 1 and args.variant != "nonspec"
                  else "score_mfma_kernel" if (G * (1 if args.variant == "nonspec" else 2)) % 8 == 0 else "score_kernel")
    roofline = {
        "bound": "hbm", "kernel": score_name,
        "achieved": score_bytes / (score_us * 1e-6) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": score_bytes / (score_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
        "traffic": None, "algorithmic_bytes": score_bytes, "avg_us": score_us,
    }
    # Second view of the same kernel: its vector instruction count (rocprofv3 --pmc SQ_INSTS_VALU,
    # profiles/valu.json; matrix-core instructions included) over its measured duration, set against the issue
    # rate of one wave64 instruction per 4 clocks per SIMD, 256 CUs x 4 SIMDs x 2.4 GHz / 4.
    roofline_alu = None
    vpath = os.path.join(ROOT, "profiles", "valu.json")
    try:
        n_valu = json.load(open(vpath)).get(args.workload, {}).get(score_name)
        if n_valu and score_us:
            peak = 256 * 4 * 2.4e9 / 4 / 1e9
            ach = n_valu / (score_us * 1e-6) / 1e9
            roofline_alu = {"bound": "alu", "kernel": score_name, "achieved": round(ach, 1), "peak": round(peak, 1),
                            "unit": "G wave64 vector instructions/s", "frac": round(ach / peak, 3),
                            "instructions_per_launch": n_valu}
    except Exception:
        roofline_alu = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            roofline["traffic"] = json.load(open(tpath)).get(args.workload, {}).get(score_name)
        except Exception:
            roofline["traffic"] = None
    attend_us = (per_kernel_us["attend"] or per_kernel_us["score_attend"]) + (per_kernel_us["attend_combine"] or 0.0)
    breakdown = {n: (round(v, 3) if v is not None else None) for n, v in per_kernel_us.items()}
    breakdown["score_topk_attend"] = round(sum(per_kernel_us[n] or 0.0 for n in ("score", "topk", "attend", "attend_combine", "score_attend")), 3)
    result = {
        "metric": "us per layer decode step (score+top-k+attend) + achieved HBM GB/s, 7B shape 32k ctx"
                  if args.workload == "M0" else "us per layer decode step (score+top-k+attend) + achieved HBM GB/s",
        "value": round(us_layer, 3), "unit": "us/layer-step", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic" if not args.filler_mb else f"synthetic; EMULATED rest of the layer: {args.filler_mb} MB streamed per layer",
        "config": {"workload": DESCR[args.workload], "layers": layers, "tokens_cached": N, "tokens_quantized": Nq,
                   "residual": R, "group": g, "gather": not args.no_gather, "variant": args.variant,
                   "value_covers": "wall time of the whole step / layers: quantize_append + score + top-k + attend on the "
                                   "main stream, gather of the next step's pairs on side streams",
                   "side_streams": len(side_list) if not args.serial_gather else 0,
                   "async_select": int(async_select),
                   "calls_per_layer": (("quantize_append, score, select_gather, attend" if not args.fused_append else
                                        "append_score, select_gather, attend") if async_select == 2 and args.variant == "speculative"
                                       else "quantize_append, score_topk, gather, attend")},
        "score_topk_attend_us": breakdown["score_topk_attend"],
        "compute_us_layer": (round(compute_ms * 1e3 / layers, 3) if compute_ms else None),
        "kernel_us_no_gather": per_kernel_ng,
        "hbm_gbs_layer": round(layer_bytes / (us_layer * 1e-6) / 1e9, 1),
        "roofline_alu": roofline_alu,
        "kernel_us": breakdown,
        "prefill_quant_offload": prefill,
        "attend_hbm_gbs": round(attend_bytes / (attend_us * 1e-6) / 1e9, 1),
        "gather_gbs": (round(B * Hkv * k * 512 / (per_kernel_us["gather"] * 1e-6) / 1e9, 2)
                       if per_kernel_us["gather"] else None),
        # with two side streams two gather kernels run at a time: the link carries one layer's pairs per layer-step
        "link_gbs_over_step": (round(B * Hkv * k * 512 / (us_layer * 1e-6) / 1e9, 2)
                               if per_kernel_us["gather"] and args.variant == "speculative" else None),
        "roofline": roofline,
    }

    if not args.no_cpu_baseline and args.variant == "speculative":
        result["cpu_baseline"] = cpu_baseline(sc, synth, sample, k_hist, v_hist, step_k, step_v, q_all, spec_k, spec_v,
                                              state["t"], layers, B, Hq, Hkv, G, D, dtype, bits, g, R, k, nq_pool)
    print(json.dumps(result))
    sc.close()


def cpu_baseline(sc, synth, sample, k_hist, v_hist, step_k, step_v, q_all, spec_k, spec_v, t_done, layers, B, Hq,
                 Hkv, G, D, dtype, bits, g, R, k, nq_pool):
    """Time the CPU oracle (as it stands, one thread) on a few (batch, KV head) rows of layer 0 for
    one decode step, extrapolate to a layer-step, and check the GPU's last step against it."""
    import numpy as np
    import torch
    from oracle import oracle as orc
    from tests.harness import check_out, check_topk

    # run one more GPU step on layer 0 alone, keeping its outputs
    t = t_done
    q = q_all[t % nq_pool, 0]
    idx = torch.full((B, Hkv, k), -1, dtype=torch.int32, device="cuda")
    out = torch.empty((B, Hq, 2, D), dtype=torch.float32, device="cuda")
    main_s = torch.cuda.current_stream()
    sc.quantize_append(0, step_k[t], step_v[t], 1, main_s)
    sc.score_topk(0, q, 2, idx, main_s)
    sc.attend(0, q, 2, spec_k, spec_v, -1, out, main_s)
    torch.cuda.synchronize()
    idx_h, out_h = idx.cpu().numpy(), out.cpu().numpy()
    q_bits = synth.bits_of(q)
    sk, sv = synth.bits_of(step_k[:t + 1]), synth.bits_of(step_v[:t + 1])
    ks_b, vs_b = synth.bits_of(spec_k), synth.bits_of(spec_v)
    sm = 1.0 / np.sqrt(128.0)
    secs, n_rows_done = 0.0, 0
    for (b, h) in sample:
        c = orc.Cache(D, bits, g, R, dtype)
        c.append(k_hist[(b, h)][0], v_hist[(b, h)][0])
        c.append(sk[:, b, h, 0], sv[:, b, h, 0])
        qh = q_bits[b, h * G:(h + 1) * G]
        t0 = time.perf_counter()
        _, sigma = c.scores(qh, sm)
        ref_idx = orc.topk(sigma, k)
        ref_out = c.attend(qh, sm, P=None, k_spec=ks_b[b, h, 0], v_spec=vs_b[b, h, 0])
        secs += time.perf_counter() - t0
        n_rows_done += 1
        check_topk(sigma, idx_h[b, h], k, what=f"bench top-k {(b, h)}")
        check_out(out_h[b, h * G:(h + 1) * G], ref_out, what=f"bench attend {(b, h)}")
        del ref_idx
        if secs > 25.0:
            break
    per_layer_us = secs / n_rows_done * (B * Hkv) * 1e6
    return {"value": round(per_layer_us, 1), "unit": "us/layer-step", "cores": 1, "kind": "oracle",
            "sample": f"score + top-k + attend of {n_rows_done} of {B * Hkv} (batch, KV head) rows of one layer at "
                      f"the benchmark's shape, scaled by {B * Hkv}/{n_rows_done}; host has {os.cpu_count()} logical CPUs",
            "parity_on_sample": "ok"}


if __name__ == "__main__":
    main()

"""Benchmark of the SpeCache decode-step hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload M0|c1|c2|c3|c4|c5]

A step is one decode step of every layer of the workload: per layer the new pair is quantised / appended and
offloaded, the low-bit keys are scored for the current and the speculative query row, ArgTopK of the
speculative row selects the pairs that a side stream fetches from pinned host memory for the next step, and
the mixed attention of Eq. 1 runs over the low-bit cache with the pairs fetched a step earlier.  Inputs are
synthetic and already resident in HBM (the 16-bit copy C sits in pinned host memory, as the method
prescribes).  Prints one JSON line.

What the line holds beside the contract's fields:
  value / ms_per_step    wall time of K free-running steps (no host synchronise inside), per layer
  median_us_layer        median over --median-steps further steps, each bracketed by events on the main stream
  compute_us_layer       the same steps without issuing gathers; gather_hidden_frac = how much of a layer's
                         gather time the step does not pay for
  host_issue_us_layer    wall time until the last call of the timed steps has returned, per layer-step (the
                         calls only enqueue; a figure near `value` means the thread waited for room in the queues)
  kernels                per kernel: mean duration (events carried by the kernel's own dispatch packet for the
                         streaming kernels), algorithmic bytes, fraction of the published peak and of the
                         peak measured in this run (hbm_stream_peak_gbs, link_peak_gbs)
  roofline               the dominant streaming kernel of the main stream
  four_call_us_layer     the same workload through the four calls the method's statement names
                         (quantize_append, score_topk, gather, attend), in a context of its own
  cpu_baseline           the CPU oracle timed on a sample of rows; parity_on_sample: the LAST free-running step
                         of the timed arrangement checked against it (selection by the tie-band rule, attention
                         output to 2e-3, with the pairs the free-running loop staged)
"""
import argparse
import json
import os
import platform
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


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return platform.processor() or "unknown"


class Run:
    """One context, its inputs and the step loop for one arrangement of the calls."""

    def __init__(self, args, torch, binding, synth, calls, total_steps):
        from paper_2503_16163_amd import arrangement
        self.args, self.torch, self.binding, self.synth, self.calls = args, torch, binding, synth, calls
        B, Hq, Hkv, S, dtype, bits, g, k, layers = WORKLOADS[args.workload]
        layers = args.layers or layers
        k = args.topk or k
        S = args.seq or S
        g = args.group or g
        bits = args.bits or bits
        self.B, self.Hq, self.Hkv, self.S, self.dtype, self.bits, self.g, self.k = B, Hq, Hkv, S, dtype, bits, g, k
        self.G, self.D, self.R = Hq // Hkv, 128, max(64, g)
        self.total_steps = total_steps
        self.spec = args.variant == "speculative"
        side_gathers = self.spec and not args.serial_gather and not args.no_gather
        # Where ArgTopK runs, how many side streams the gathers alternate over, whether the scoring launch carries
        # the append: the measured rule of paper_2503_16163_amd.arrangement (the full-size parity tests use the
        # same), unless the command line says otherwise.
        plan = arrangement.plan(B, Hkv, self.G, S, k, layers, bits, self.spec, args.select_cache == "lowbit")
        planned = plan["calls"] == calls
        if calls == "one-pass":
            async_select = 2          # specache_score_attend leaves its keys to specache_select_gather
        elif calls == "four":
            async_select = ((plan["async_select"] if planned else 1 if self.spec and layers > 1 else 0) if args.select_stream == "auto"
                            else {"main": 0, "own": 1, "gather": 1}[args.select_stream])
        elif args.select_stream == "auto":
            async_select = 2 if side_gathers or args.no_gather else 1
        else:
            async_select = {"main": 0, "own": 1, "gather": 2 if side_gathers else 1}[args.select_stream]
        self.async_select = async_select
        self.carry_append = calls == "one-pass" and (args.append == "carried" or
                                                     (args.append == "auto" and planned and plan["carry_append"]))
        self.plan_side_streams = plan["side_streams"] if planned else 2
        max_seq = ((S + total_steps + 63) // 64 + 1) * 64
        sc = None
        while sc is None:
            try:
                sc = binding.SpeCache(layers, B, Hq, Hkv, bits, g, max_seq, k, dtype, residual=self.R,
                                      select_form=1 if args.select == "logprob" else 0,
                                      select_cache=1 if args.select_cache == "mixed" else 0, async_select=async_select)
            except binding.SpeCacheError as e:
                if e.code != binding.ENOMEM or layers == 1:
                    raise
                layers = max(1, layers // 2)   # the pinned host store did not fit: fewer layers
        self.sc, self.layers = sc, layers
        self.main_s = torch.cuda.current_stream()
        n_side = args.side_streams if args.side_streams > 0 else (2 if self.carry_append else self.plan_side_streams)
        self.side_list = [self.main_s] if args.serial_gather else [torch.cuda.Stream() for _ in range(n_side)]
        self.state = {"t": 0}

    # ---- load the prompt: the same synthetic K/V tensor serves every layer ----------
    def load(self, seed=1000):
        """Quant + Offload of the prefilling procedure (Appendix A), timed per layer: the bulk quantiser is
        HBM-bound, the copy to the pinned host store is bound by the host link."""
        torch, synth, sc, args = self.torch, self.synth, self.sc, self.args
        B, Hq, Hkv, S, D, dtype, layers, k = self.B, self.Hq, self.Hkv, self.S, self.D, self.dtype, self.layers, self.k
        kd, vd = synth.make_kv_device(seed, B, Hkv, S, D, dtype)
        torch.cuda.synchronize()
        sc.timing(True)
        t0 = time.perf_counter()
        for L in range(layers):
            sc.quantize_append(L, kd, vd, S, self.main_s)
        torch.cuda.synchronize()
        load_wall_us = (time.perf_counter() - t0) * 1e6 / layers
        lt = sc.timing(False)
        n_flushed = sc.counts(0)[1]
        raw_bytes = B * Hkv * S * 512
        flush_us = lt["flush"][0] / lt["flush"][1] if lt["flush"][1] else None
        copy_us = lt["append_copy"][0] / lt["append_copy"][1] if lt["append_copy"][1] else None
        # bulk quantiser: reads the 16-bit pairs once, writes codes (bits/16 of that) and 32-bit (min, max) per group
        flush_bytes = B * Hkv * n_flushed * (512 + 2 * (128 * self.bits // 8) + 2 * 128 * 4 // self.g)
        self.prefill = {"us_per_layer": round(load_wall_us, 1), "tokens": S,
                        "flush_us": round(flush_us, 1) if flush_us else None,
                        "flush_gbs": round(flush_bytes / (flush_us * 1e-6) / 1e9, 1) if flush_us else None,
                        "flush_frac_of_hbm_peak": round(flush_bytes / (flush_us * 1e-6) / 8e12, 3) if flush_us else None,
                        "offload_us": round(copy_us, 1) if copy_us else None,
                        "offload_gbs": round(raw_bytes / (copy_us * 1e-6) / 1e9, 1) if copy_us else None}
        self.sample = [(0, h) for h in sorted(set([0, Hkv // 3, (2 * Hkv) // 3, Hkv - 1]))]
        self.k_hist = {bh: synth.bits_of(kd[bh[0], bh[1]]) for bh in self.sample}
        self.v_hist = {bh: synth.bits_of(vd[bh[0], bh[1]]) for bh in self.sample}
        del kd, vd

        self.nq_pool = 8
        total_steps = self.total_steps
        self.q_all = synth.make_queries_device(seed, self.nq_pool * layers, B, Hq, D, dtype).view(self.nq_pool, layers, B, Hq, 2, D)
        self.q1_all = self.q_all[:, :, :, :, :1].contiguous()   # current-token rows only (non-speculative variant)
        step_k, step_v = synth.make_kv_device(seed + 1, total_steps * B, Hkv, 1, D, dtype)
        self.step_k = step_k.view(total_steps, B, Hkv, 1, D).contiguous()
        self.step_v = step_v.view(total_steps, B, Hkv, 1, D).contiguous()
        self.spec_k, self.spec_v = synth.make_kv_device(seed + 2, B, Hkv, 1, D, dtype, n_outlier=0)
        self.idx = [[torch.full((B, Hkv, k), -1, dtype=torch.int32, device="cuda") for _ in range(2)] for _ in range(layers)]
        self.out = [torch.empty((B, Hq, 2, D), dtype=torch.float32, device="cuda") for _ in range(layers)]
        self.filler = torch.ones(args.filler_mb * (1 << 20) // 2, dtype=torch.float16, device="cuda") if args.filler_mb else None
        self.filler_out = torch.empty((), dtype=torch.float16, device="cuda")
        # The step loop hands the library raw addresses and stream handles, as a serving loop would: building a
        # tensor view per call costs the issuing thread several microseconds per layer, which shows once the
        # step is short (small k).
        self.q_p = [[self.q_all[p, L].data_ptr() for L in range(layers)] for p in range(self.nq_pool)]
        self.q1_p = [[self.q1_all[p, L].data_ptr() for L in range(layers)] for p in range(self.nq_pool)]
        self.k_p = [self.step_k[t].data_ptr() for t in range(total_steps)]
        self.v_p = [self.step_v[t].data_ptr() for t in range(total_steps)]
        self.idx_p = [[self.idx[L][b].data_ptr() for b in range(2)] for L in range(layers)]
        self.out_p = [self.out[L].data_ptr() for L in range(layers)]
        self.spec_k_p, self.spec_v_p = self.spec_k.data_ptr(), self.spec_v.data_ptr()
        self.main_h = self.main_s.cuda_stream
        self.side_h = [s.cuda_stream for s in self.side_list]
        torch.cuda.synchronize()

    def calls_per_layer(self):
        if not self.spec:
            return "quantize_append, score_topk, gather (main stream), attend"
        if self.calls == "one-pass":
            return "decode_step (= append_score_attend + select_gather)" if self.carry_append else "quantize_append, score_attend, select_gather"
        if self.async_select == 2:
            return "append_score, select_gather, attend" if self.args.fused_append else "quantize_append, score, select_gather, attend"
        return "quantize_append, score_topk, gather, attend"

    def step(self, gather=True):
        sc, args, layers = self.sc, self.args, self.layers
        t = self.state["t"]
        main_h, side_h, k_p, v_p = self.main_h, self.side_h, self.k_p, self.v_p
        if not self.spec:
            # non-speculative fetching (Section 4.4): select on the current token, fetch at once, then attend
            for L in range(layers):
                q = self.q1_p[t % self.nq_pool][L]
                sc.quantize_append(L, k_p[t], v_p[t], 1, main_h)
                sc.score_topk(L, q, 1, self.idx_p[L][0], main_h)
                sc.gather(L, self.idx_p[L][0], 0, main_h)
                sc.attend(L, q, 1, None, None, 0, self.out_p[L], main_h)
            self.state["t"] = t + 1
            return
        do_gather = gather and not args.no_gather
        slot = (t % 2) if (t > 0 and not args.no_gather) else -1
        n_side = len(side_h)
        for L in range(layers):
            q = self.q_p[t % self.nq_pool][L]
            ib = self.idx_p[L][t % 2]
            if self.calls == "one-pass":
                if not self.carry_append:
                    sc.quantize_append(L, k_p[t], v_p[t], 1, main_h)
                    sc.score_attend(L, q, 2, self.spec_k_p, self.spec_v_p, slot, self.out_p[L], main_h)
                    sc.select_gather(L, ib, (t + 1) % 2 if do_gather else -1, side_h[L % n_side])
                else:   # the whole layer-step as one call; its one launch on the main stream also carries the append
                    sc.decode_step(L, k_p[t], v_p[t], q, self.spec_k_p, self.spec_v_p, slot, self.out_p[L], main_h,
                                   ib, (t + 1) % 2 if do_gather else -1, side_h[L % n_side])
            else:
                if self.async_select == 2:
                    if not args.fused_append:
                        sc.quantize_append(L, k_p[t], v_p[t], 1, main_h)
                        sc.score(L, q, 2, main_h)
                    else:
                        sc.append_score(L, k_p[t], v_p[t], q, 2, main_h)   # the scoring launch carries the append
                    sc.select_gather(L, ib, (t + 1) % 2 if do_gather else -1, side_h[L % n_side])
                else:
                    sc.quantize_append(L, k_p[t], v_p[t], 1, main_h)
                    sc.score_topk(L, q, 2, ib, main_h)
                    if do_gather:
                        sc.gather(L, ib, (t + 1) % 2, side_h[L % n_side])
                sc.attend(L, q, 2, self.spec_k_p, self.spec_v_p, slot, self.out_p[L], main_h)
            if self.filler is not None:
                self.torch.sum(self.filler, dim=(0,), out=self.filler_out)
        self.state["t"] = t + 1

    def timed(self, n, gather=True):
        """Wall time of n free-running steps in ms per step."""
        self.torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            self.step(gather)
        self.issued_ms = (time.perf_counter() - t0) * 1e3 / n   # the last call has returned; the GPU may still be busy
        self.torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / n

    def event_timed(self, n, gather=True):
        """The same steps with the library's per-kernel event pairs on: mean us per launch of every kernel."""
        self.sc.timing(True)
        for _ in range(n):
            self.step(gather)
        kt = self.sc.timing(False)
        return {name: (us / c if c else None) for name, (us, c) in kt.items()}

    def median_steps(self, n):
        """n further free-running steps, an event on the main stream after each: median us per step."""
        torch = self.torch
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        torch.cuda.synchronize()
        ev[0].record(self.main_s)
        for i in range(n):
            self.step()
            ev[i + 1].record(self.main_s)
        torch.cuda.synchronize()
        d = sorted(ev[i].elapsed_time(ev[i + 1]) * 1e3 for i in range(n))
        return d[n // 2], d[n // 10], d[(9 * n) // 10]

    def close(self):
        self.torch.cuda.synchronize()
        self.sc.close()


def check_last_step_and_time_oracle(run, time_budget_s=25.0):
    """Two more free-running steps of the timed arrangement; the second is checked against the CPU oracle on a
    sample of (batch, KV head) rows of layer 0 and on one row of the last layer: ArgTopK by the tie-band rule, the
    attention output (which used the pairs that the loop staged a step earlier, P = the previous selection) to
    2e-3.  The oracle's time for score + top-k + attend of the layer-0 rows is the cpu_baseline."""
    import numpy as np
    from oracle import build as oracle_build
    from oracle import oracle as orc
    from tests.harness import check_out, check_topk
    synth, torch = run.synth, run.torch
    B, Hkv, G, D, k = run.B, run.Hkv, run.G, run.D, run.k
    run.step()
    run.step()
    torch.cuda.synchronize()
    t = run.state["t"] - 1                      # the step that is checked
    staged = not run.args.no_gather
    sk, sv = synth.bits_of(run.step_k[:t + 1]), synth.bits_of(run.step_v[:t + 1])
    ks_b, vs_b = synth.bits_of(run.spec_k), synth.bits_of(run.spec_v)
    sm = 1.0 / np.sqrt(128.0)
    secs, n_timed = 0.0, 0
    layers_checked = sorted({0, run.layers - 1})
    for L in layers_checked:
        q_bits = synth.bits_of(run.q_all[t % run.nq_pool, L])
        idx_new = run.idx[L][t % 2].cpu().numpy()
        idx_prev = run.idx[L][(t - 1) % 2].cpu().numpy()
        out_h = run.out[L].cpu().numpy()
        rows = run.sample if L == 0 else run.sample[-1:]
        for (b, h) in rows:
            c = orc.Cache(D, run.bits, run.g, run.R, run.dtype)
            c.append(run.k_hist[(b, h)], run.v_hist[(b, h)])
            c.append(sk[:, b, h, 0], sv[:, b, h, 0])
            qh = q_bits[b, h * G:(h + 1) * G]
            t0 = time.perf_counter()
            _, sigma = c.scores(qh, sm)
            orc.topk(sigma, k)
            ref_out = c.attend(qh, sm, P=idx_prev[b, h] if staged else None, k_spec=ks_b[b, h, 0], v_spec=vs_b[b, h, 0])
            if L == 0:
                secs += time.perf_counter() - t0
                n_timed += 1
            check_topk(sigma, idx_new[b, h], k, what=f"bench top-k layer {L} row {(b, h)}")
            check_out(out_h[b, h * G:(h + 1) * G], ref_out, what=f"bench attend layer {L} row {(b, h)}")
            if L == 0 and secs > time_budget_s:
                break
    per_layer_us = secs / n_timed * (B * Hkv) * 1e6
    return {"value": round(per_layer_us, 1), "unit": "us/layer-step", "cores": 1, "kind": "oracle",
            "sample": f"score + top-k + attend of {n_timed} of {B * Hkv} (batch, KV head) rows of one layer at the benchmark's "
                      f"shape, scaled by {B * Hkv}/{n_timed}",
            "cpu": cpu_model(), "logical_cpus": os.cpu_count(),
            "oracle_build": "g++ " + " ".join(oracle_build.FLAGS),
            "parity_on_sample": "ok",
            "parity_covers": f"last free-running step of the timed arrangement ({run.calls_per_layer()}), layers {layers_checked}: "
                             "ArgTopK by the tie-band rule, attention output with the staged pairs to 2e-3"}


def profile_figures(workload_key, kernel_names):
    """HBM traffic and vector-instruction counts per launch from the committed rocprofv3 --pmc summaries
    (written by paper_2503_16163_amd.profile_summary).  A figure is quoted only for a kernel whose sources still
    hash to what the file recorded for it."""
    from paper_2503_16163_amd import build as hip_build
    res = {}
    for key, fname in (("traffic", "traffic.json"), ("valu", "valu.json")):
        path = os.path.join(ROOT, "profiles", fname)
        try:
            d = json.load(open(path))
        except (OSError, ValueError):
            res[key] = ({}, "no profile file")
            continue
        w, hashes = d.get(workload_key, {}), d.get("kernel_source_hash", {}).get(workload_key, {})
        tbl, stale = {}, []
        for n in kernel_names:
            if w.get(n) is None:
                continue
            if hashes.get(n) == hip_build.kernel_source_hash(n.split("+")[0]):
                tbl[n] = w[n]
            else:
                stale.append(n)
        src = f"profiles/{fname} [{workload_key}]: rocprofv3 --pmc, per launch"
        if stale:
            src += "; not quoted, measured on other sources of the kernel: " + ", ".join(stale)
        if not w:
            src = f"profiles/{fname} holds no run of {workload_key}"
        res[key] = (tbl, src)
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="M0", choices=sorted(WORKLOADS))
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers")
    ap.add_argument("--calls", default="auto", choices=["auto", "one-pass", "split", "four"],
                    help="which calls a layer-step is made of.  one-pass: quantize_append, specache_score_attend (scoring and "
                         "attention of a chunk in one launch, the logits stay on the chip), select_gather.  split: scoring "
                         "and attention as two calls (with ArgTopK on the gather's stream: score, select_gather, attend).  "
                         "four: quantize_append, score_topk, gather, attend.  auto: what paper_2503_16163_amd.arrangement.plan "
                         "picks for the shape (one-pass where that kernel exists and the link leaves the main stream a "
                         "large part of the step; the four calls with ArgTopK on the library's stream where the link alone "
                         "bounds it; split for the shapes without a one-pass kernel)")
    ap.add_argument("--filler-mb", type=int, default=0,
                    help="EMULATION, not part of the method's path: after every layer's attend, stream this many MB of "
                         "stand-in weights through a plain torch reduction on the main stream (a 7B layer reads about "
                         "403 MB of fp16 weights per decode step), to see how much of the gather the rest of a model's "
                         "layer would hide")
    ap.add_argument("--topk", type=int, default=0,
                    help="override k, the number of prefetched pairs per (batch, KV head) (the k sweep of Section 4.4)")
    ap.add_argument("--seq", type=int, default=0,
                    help="override S, the number of cached tokens at the start (a multiple of 64)")
    ap.add_argument("--group", type=int, default=0, choices=[0, 32, 64, 128],
                    help="override g, the quantisation group size (the residual becomes max(64, g))")
    ap.add_argument("--bits", type=int, default=0, choices=[0, 1, 2, 4],
                    help="override the code width (4: Eq. 2 with B = 4, plain kernels; the paper's runs use 2 and 1)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-gather", action="store_true", help="skip the host-link gather (attend sees nothing prefetched)")
    ap.add_argument("--serial-gather", action="store_true", help="issue the gather on the main stream (no overlap)")
    ap.add_argument("--side-streams", type=int, default=0,
                    help="side streams the gathers alternate over by layer; 0 = the measured rule of paper_2503_16163_amd.arrangement")
    ap.add_argument("--variant", default="speculative", choices=["speculative", "nonspec"],
                    help="nonspec: the non-speculative fetching of Section 4.4 (select on the current token, one query "
                         "row, gather on the main stream before attend): the whole link time is exposed")
    ap.add_argument("--compute-only-pass", action="store_true", help="(the default now; kept for old command lines)")
    ap.add_argument("--no-compute-only-pass", action="store_true",
                    help="skip the two passes of K steps that issue no gathers (compute_us_layer, kernel_us_no_gather)")
    ap.add_argument("--median-steps", type=int, default=200, help="further steps timed one by one for the median (0: skip)")
    ap.add_argument("--no-peaks", action="store_true", help="skip the in-run measurement of the HBM streaming and host-link rates")
    ap.add_argument("--no-four-call", action="store_true", help="skip the extra context that times the four named calls")
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
                         "library's own beside the attention kernels, or on the gather's side stream ahead of the gather; "
                         "auto = the measured rule of paper_2503_16163_amd.arrangement")
    ap.add_argument("--fused-append", action="store_true",
                    help="with --calls split and ArgTopK on the gather's stream: specache_append_score (the scoring launch "
                         "carries the copy of the new pair) instead of quantize_append and score as two calls")
    ap.add_argument("--append", default="auto", choices=["auto", "carried", "separate"],
                    help="with --calls one-pass: specache_append_score_attend, whose one launch also carries the copy of "
                         "the new pair (carried), or quantize_append and specache_score_attend as two calls (separate); "
                         "auto = the measured rule of paper_2503_16163_amd.arrangement")
    ap.add_argument("--vector-alu", default="", choices=["", "score", "attend", "both"],
                    help="A/B measurement: run the named streaming kernel(s) in the vector-ALU formulation instead of the "
                         "integer-matrix-core one (one query head per KV head, two rows); implies --calls split")
    ap.add_argument("--hit-rate", action="store_true",
                    help="instead of the timing run: how well the positions selected from the low-bit scores of the "
                         "speculative row match the exact top-k on the 16-bit keys (synthetic stand-in for the "
                         "sparsity profile of Section 3.1), for 2-bit, 1-bit (Eq. 3) and unmodified 1-bit KIVI (Table 5)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

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
    layers = args.layers or layers
    k = args.topk or k
    S = args.seq or S
    g = args.group or g
    bits = args.bits or bits
    G, D = Hq // Hkv, 128
    spec = args.variant == "speculative"
    one_pass_kernel = G == 1 and bits in (1, 2) and spec and args.select_cache == "lowbit" and not args.vector_alu
    calls = args.calls
    if calls == "auto":
        from paper_2503_16163_amd import arrangement
        calls = arrangement.plan(B, Hkv, G, S, k, layers, bits, spec, args.select_cache == "lowbit")["calls"]
        # options that name another arrangement than the rule's
        if calls == "one-pass" and (not one_pass_kernel or args.serial_gather or args.fused_append or
                                    args.select_stream in ("main", "own")):
            calls = "split"
        if calls == "four" and args.select_stream == "gather":
            calls = "one-pass" if one_pass_kernel and not args.fused_append else "split"
        if calls == "four" and args.fused_append:
            calls = "split"
    if not spec:
        calls = "four"

    # ---- roofline denominators of this machine, measured before anything else runs ----
    peaks = {"hbm_stream_peak_gbs": None, "link_peak_gbs": None, "link_memcpy_gbs": None, "link_read_kernel_gbs": None}
    if not args.no_peaks:
        peaks["hbm_stream_peak_gbs"] = round(binding.measure_hbm_read(1 << 30, 10), 1)
        mc, rk = binding.measure_link(256 << 20, 5)
        peaks["link_memcpy_gbs"], peaks["link_read_kernel_gbs"] = round(mc, 2), round(rk, 2)
        peaks["link_peak_gbs"] = round(max(mc, rk), 2)

    do_compute_only = spec and not args.no_gather and not args.no_compute_only_pass
    total_steps = args.warmup + 2 * args.steps + (2 * args.steps if do_compute_only else 0) + args.median_steps + 8
    run = Run(args, torch, binding, synth, calls, total_steps)
    run.load()
    layers = run.layers
    for _ in range(args.warmup):
        run.step()
    ms_per_step = run.timed(args.steps)
    host_issue_us_layer = run.issued_ms * 1e3 / layers

    if args.calibrate_copy:
        src = torch.ones(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    per_kernel_us = run.event_timed(args.steps)
    median_us = run.median_steps(args.median_steps) if args.median_steps > 0 else None
    compute_ms, per_kernel_ng = None, None
    if do_compute_only:
        compute_ms = run.timed(args.steps, gather=False)
        per_kernel_ng = {n: (round(v, 3) if v is not None else None) for n, v in run.event_timed(args.steps, gather=False).items()}

    N, Nq = run.sc.counts(0)
    rows = B * Hkv
    per_elem = (bits + 32.0 / g) / 8.0
    packed = rows * Nq * D * per_elem                       # packed K (or V) incl. metadata
    pairs = rows * ((k if not args.no_gather else 0) + (N - Nq) + 1) * 512   # staged, residual and transient 16-bit pairs
    us_layer = ms_per_step * 1e3 / layers
    n_q_rows = G * (2 if spec else 1)
    score_name = ("score4_kernel" if bits == 4 else
                  "score_i8_kernel" if (G == 1 and spec and args.vector_alu not in ("score", "both"))
                  else "score_mfma_kernel" if n_q_rows % 8 == 0 else "score_kernel")
    attend_name = ("attend4_partial_kernel" if bits == 4 else
                   "attend_i8_kernel" if (G == 1 and spec and bits in (1, 2) and args.vector_alu not in ("attend", "both")) else "attend_partial_kernel")
    one_pass_name = "attend_i8_kernel<scoring pass in front>"
    stream_peak = peaks["hbm_stream_peak_gbs"]
    link_peak = peaks["link_peak_gbs"]

    def entry(kernel, what, us, nbytes, peak, measured_peak, note=None):
        if us is None:
            return None
        gbs = nbytes / (us * 1e-6) / 1e9
        e = {"kernel": kernel, "what": what, "avg_us": round(us, 3), "algorithmic_bytes": int(nbytes), "gbs": round(gbs, 1),
             "frac": round(gbs / peak, 4) if peak else None,
             "frac_of_measured_peak": round(gbs / measured_peak, 4) if measured_peak else None}
        if note:
            e["note"] = note
        return e

    kern = [
        entry(one_pass_name, "score + attend partial pass in one launch: packed K and V once, 16-bit pairs",
              per_kernel_us.get("score_attend"), 2 * packed + pairs, HBM_PEAK_GBS, stream_peak),
        entry(score_name, "fused dequantise + q.K^T, both rows: packed K once", per_kernel_us.get("score"), packed,
              HBM_PEAK_GBS, stream_peak),
        entry(attend_name, "mixed attention, partial pass: packed V once, 16-bit pairs (the fp32 logits it reads back are this "
                           "design's overhead, not counted)", per_kernel_us.get("attend"), packed + pairs, HBM_PEAK_GBS, stream_peak),
        entry("attend_combine_kernel", "merge of the chunk partials (overhead of the split over the sequence: bytes = partials read)",
              per_kernel_us.get("attend_combine"), rows * n_q_rows * ((Nq + 511) // 512 + 3) * 130 * 4, HBM_PEAK_GBS, stream_peak,
              "latency-bound: one workgroup per (row, query row)"),
        entry("topk_kernel", "ArgTopK: 4-byte selection keys of the speculative row (L2-resident)", per_kernel_us.get("topk"),
              rows * Nq * 4, HBM_PEAK_GBS, stream_peak, "latency-bound: one workgroup per row, a chain of barrier-separated steps"),
        entry("gather_kernel", "Pre-fetch(C_K): 512-byte pairs from pinned host memory", per_kernel_us.get("gather"),
              rows * k * 512, link_peak or 57.0, link_peak, "peak = the host link's rate measured in this run (57 GB/s if not measured)"),
        entry("append_copy_kernel", "Offload of the new pair to C and to the residual", per_kernel_us.get("append_copy"),
              rows * 1024, HBM_PEAK_GBS, stream_peak, "launch-bound"),
    ]
    kern = [e for e in kern if e]
    # the dominant streaming kernel of the main stream
    cands = [e for e in kern if e["kernel"] in (one_pass_name, score_name, attend_name)]
    dom = max(cands, key=lambda e: e["avg_us"])
    dom_base = dom["kernel"].split("<")[0] + ("+score" if dom["kernel"] == one_pass_name else "")
    workload_key = f"{args.workload}:k{k}:g{g}:b{bits}" + (f":S{S}" if args.seq else "")
    prof = profile_figures(workload_key, [dom_base, score_name, attend_name, "topk_kernel", "gather_kernel", "attend_combine_kernel"])
    traffic_tbl, traffic_src = prof["traffic"]
    for e in kern:   # measured HBM bytes per launch beside the algorithmic ones, where the profile covers the kernel
        base = e["kernel"].split("<")[0] + ("+score" if e["kernel"] == one_pass_name else "")
        if traffic_tbl.get(base) is not None:
            e["traffic"] = traffic_tbl[base]
    roofline = {"bound": "hbm", "kernel": dom["kernel"], "achieved": dom["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": dom["frac"], "frac_of_measured_stream_peak": dom["frac_of_measured_peak"],
                "traffic": (traffic_tbl or {}).get(dom_base), "traffic_source": traffic_src,
                "algorithmic_bytes": dom["algorithmic_bytes"], "avg_us": dom["avg_us"],
                "timing": "HIP events carried by the kernel's own dispatch packet, mean over the event-timed steps"}
    # score + top-k together against the packed keys (the target the method's statement sets is 0.70)
    score_topk = None
    if per_kernel_us.get("score") and per_kernel_us.get("topk"):
        score_topk = entry("score + ArgTopK", "packed K once; both kernels' durations added",
                           per_kernel_us["score"] + per_kernel_us["topk"], packed, HBM_PEAK_GBS, stream_peak)
    roofline_alu = None
    valu_tbl, valu_src = prof["valu"]
    if valu_tbl and valu_tbl.get(dom_base):
        n_valu = valu_tbl[dom_base]
        peak_i = 256 * 4 * 2.4e9 / 4 / 1e9
        ach = n_valu / (dom["avg_us"] * 1e-6) / 1e9
        roofline_alu = {"bound": "alu", "kernel": dom["kernel"], "achieved": round(ach, 1), "peak": round(peak_i, 1),
                        "unit": "G wave64 vector instructions/s", "frac": round(ach / peak_i, 3),
                        "instructions_per_launch": n_valu, "source": valu_src}

    breakdown = {n: (round(v, 3) if v is not None else None) for n, v in per_kernel_us.items()}
    sta = sum(per_kernel_us[n] or 0.0 for n in ("score", "topk", "attend", "attend_combine", "score_attend"))
    gather_us = per_kernel_us.get("gather")
    compute_us_layer = compute_ms * 1e3 / layers if compute_ms else None
    hidden = None
    if compute_us_layer and gather_us:
        hidden = max(0.0, min(1.0, 1.0 - max(0.0, us_layer - compute_us_layer) / gather_us))
    result = {
        "metric": "us per layer decode step (score+top-k+attend) + achieved HBM GB/s, 7B shape 32k ctx"
                  if args.workload == "M0" else "us per layer decode step (score+top-k+attend) + achieved HBM GB/s",
        "value": round(us_layer, 3), "unit": "us/layer-step", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None,
        "dtype": "f32",
        "dtype_note": "accumulation and outputs are binary32; the contractions run on the matrix cores with int8 operands (packed "
                      "codes, fixed-point multipliers, exact int32 sums) or, with 8 and 16 query rows per KV head, f16 operands",
        "data": "synthetic" if not args.filler_mb else f"synthetic; EMULATED rest of the layer: {args.filler_mb} MB streamed per layer",
        "config": {"workload": DESCR[args.workload] + (f" [code width overridden: {bits} bits]" if args.bits else "") +
                               (f" [context overridden: S = {S}]" if args.seq else ""), "layers": layers, "tokens_cached": N, "tokens_quantized": Nq,
                   "residual": run.R, "group": g, "topk": k, "gather": not args.no_gather, "variant": args.variant,
                   "value_covers": "wall time of the whole step / layers: quantize_append + score + top-k + attend, the gather of "
                                   "the next step's pairs on side streams",
                   "side_streams": len(run.side_list) if not args.serial_gather else 0,
                   "async_select": int(run.async_select), "calls_per_layer": run.calls_per_layer()},
        "median_us_layer": round(median_us[0] / layers, 3) if median_us else None,
        "p10_p90_us_layer": [round(median_us[1] / layers, 3), round(median_us[2] / layers, 3)] if median_us else None,
        "median_over_steps": args.median_steps if median_us else 0,
        "score_topk_attend_us": round(sta, 3),
        "compute_us_layer": round(compute_us_layer, 3) if compute_us_layer else None,
        "host_issue_us_layer": round(host_issue_us_layer, 3),
        "gather_hidden_frac": round(hidden, 3) if hidden is not None else None,
        "kernel_us_no_gather": per_kernel_ng,
        "hbm_gbs_layer": round((2 * packed + pairs) / (us_layer * 1e-6) / 1e9, 1),
        **peaks,
        "kernels": kern, "profile_key": workload_key,
        "score_plus_topk": score_topk,
        "roofline_alu": roofline_alu,
        "kernel_us": breakdown,
        "prefill_quant_offload": run.prefill,
        "gather_gbs": (round(rows * k * 512 / (gather_us * 1e-6) / 1e9, 2) if gather_us else None),
        # with two side streams two gather kernels run at a time: the link carries one layer's pairs per layer-step
        "link_gbs_over_step": (round(rows * k * 512 / (us_layer * 1e-6) / 1e9, 2) if gather_us and spec else None),
        "roofline": roofline,
    }

    if not args.no_cpu_baseline and spec:
        result["cpu_baseline"] = check_last_step_and_time_oracle(run)
    run.close()
    del run

    # ---- the same workload through the four calls the method's statement names, in a context of its own ----
    if spec and calls != "four" and not args.no_four_call and not args.no_gather:
        r4 = Run(args, torch, binding, synth, "four", args.warmup + args.steps + 8)
        r4.load()
        for _ in range(args.warmup):
            r4.step()
        ms4 = r4.timed(args.steps)
        result["four_call_us_layer"] = round(ms4 * 1e3 / r4.layers, 3)
        result["four_call_config"] = {"calls_per_layer": r4.calls_per_layer(), "async_select": int(r4.async_select),
                                      "side_streams": len(r4.side_list), "layers": r4.layers}
        r4.close()
    print(json.dumps(result))


if __name__ == "__main__":
    main()

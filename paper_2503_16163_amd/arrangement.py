"""How a stepping loop arranges the calls of one layer-step over streams (host logic only, no arithmetic
of the method): which calls make up the step, where ArgTopK runs (specache_config.async_select), over how
many side streams the gathers alternate by layer, and whether the launch that scores also carries the
append.  bench.py times this arrangement and the full-size parity tests check it.

The rule compares two times that follow from the shape:

  link_us  what one layer's prefetch needs on the host link: rows x k x 512 bytes at the rate
           specache_measure_link reports on these machines (57.5 GB/s);
  main_us  what the caller's stream needs for one layer with one query head per KV head and 1- or 2-bit codes,
           where scoring and attention are one launch (specache_score_attend): 22 us + 19.8 us per million
           (row, cached token) pairs, and never less than the 33 us the issuing thread needs for the
           runtime calls of a layer-step (measured without gathers: 16k tokens 33, 32k 42, 48k 52, 64k 63 us).

  link_us <= 0.9 main_us   the step is bound by compute and by the issuing thread: the fewest calls and
                           launches.  specache_append_score_attend + specache_select_gather, two side streams.
  else, link_us < 100      bound by the link, with the main stream still a large part of the step:
                           quantize_append + specache_score_attend + specache_select_gather, three side
                           streams (one selects while two gathers share the link).  The append stays a launch
                           of its own: its store to host memory, carried by the long launch, held that
                           launch's completion and the selection behind it back (32k tokens, k = 256: 80 to
                           85 us per layer against 76.5).
  else                     the link alone bounds the step: the four named calls with ArgTopK on the library's
                           own stream (async_select 1), two side streams; every gather then starts the moment
                           its selection is done instead of behind the previous gather of its stream (64k
                           tokens, k = 384: 118 us per layer against 147 to 169).

One query head per KV head without the one-launch kernel (4-bit codes, selection on the mixed cache):
the same ladder with score + select_gather + attend in place of the one-launch call.  Several query heads per
KV head: score + select_gather + attend with ArgTopK on the gather's stream and two side streams, which
measured best or level with the best at every shape tried (8B-class shape with 8k and 32k tokens and k = 256 to
1024, 131k tokens with k = 512 to 2048).  One layer, or the non-speculative variant: everything on the
caller's stream.

Evidence, us per layer at 32 rows (rule's pick against the best of five arrangements tried), shapes that are
not the benchmark's own: 8k tokens k = 32: 31.8 / 31.8; 8k k = 96: 33.5 / 33.5; 16k k = 192: 57.8 / 57.8;
16k k = 256: 75.3 / 75.3; 16k k = 384: 112.2 / 112.2; 32k k = 192: 58.7 / 58.1; 32k k = 384: 113.3 / 113.3; 48k k = 192: 64.5 to 67.5 / 64.5;
48k k = 256: 78 to 109 (unsteady from run to run) / 80.5; 48k k = 384: 113 / 113; 48k k = 512: 150 / 150;
64k k = 160: 67.3 / 67.3; 64k k = 256: 81.3 / 79.8; 64k k = 384: 118 / 118; 64k k = 512: 151 / 151."""

SELECT_ON_CALLER, SELECT_ON_OWN_STREAM, SELECT_ON_GATHER_STREAM = 0, 1, 2

LINK_GBS = 57.5


def link_us(rows, k):
    return rows * k * 512 / (LINK_GBS * 1e3)


def main_us(rows, S):
    return max(33.0, 22.0 + 19.8 * rows * S / 1e6)


def plan(B, Hkv, G, S, k, layers, bits=2, speculative=True, select_lowbit=True):
    """-> dict(calls, async_select, side_streams, carry_append).  calls: "one-pass" ([quantize_append,]
    score_attend or append_score_attend, select_gather), "split" (quantize_append, score, select_gather, attend)
    or "four" (quantize_append, score_topk, gather, attend)."""
    rows = B * Hkv
    if layers == 1 or not speculative:
        return dict(calls="four", async_select=SELECT_ON_CALLER, side_streams=1, carry_append=False)
    if G > 1:
        return dict(calls="split", async_select=SELECT_ON_GATHER_STREAM, side_streams=2, carry_append=False)
    one_pass = bits in (1, 2) and select_lowbit      # the shapes specache_score_attend has its one-launch kernel for
    if link_us(rows, k) <= 0.9 * main_us(rows, S):
        return dict(calls="one-pass" if one_pass else "split", async_select=SELECT_ON_GATHER_STREAM, side_streams=2,
                    carry_append=one_pass)
    if link_us(rows, k) < 100.0:
        return dict(calls="one-pass" if one_pass else "split", async_select=SELECT_ON_GATHER_STREAM, side_streams=3,
                    carry_append=False)
    return dict(calls="four", async_select=SELECT_ON_OWN_STREAM, side_streams=2, carry_append=False)

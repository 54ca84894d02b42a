"""How a stepping loop arranges the calls of one layer-step over streams (host logic only, no arithmetic
of the method): where ArgTopK runs (specache_config.async_select) and over how many side streams the
gathers alternate by layer.  bench.py times this arrangement and the full-size parity tests check it.

The rule is a measured one.  keys_per_pair = scored keys x query heads per KV head / k says how much
scoring work stands against one fetched pair.  With much of it the step is bound by compute and by the
issuing thread: ArgTopK goes on the gather's stream (specache_score + specache_select_gather), which
needs the fewest ordering calls between streams; three side streams below 192 keys per pair (one
selects while two gathers share the link), two from there on.  With little of it the step is bound by
the host link: ArgTopK on the library's own stream lets every gather start the moment its selection is
done; two side streams, or one from 384 keys per pair on, where the gather has time to spare.  One
layer, or the non-speculative variant: everything on the caller's stream.

Whether the launch that scores (and attends) also carries the append of the step's new pair
(specache_append_score, specache_append_score_attend) follows the same measure: from 192 keys per pair
on it saves a launch per layer-step (7B shape, k = 64: 38 to 40 us per layer against 43 to 46; k = 128: 43
against 51); below, where the link is the bound, the separate append measured faster (k = 256: 76.6 us
against 80 to 85 with the append carried, whichever number of side streams)."""

SELECT_ON_CALLER, SELECT_ON_OWN_STREAM, SELECT_ON_GATHER_STREAM = 0, 1, 2


def side_streams(async_select, G, S, k):
    keys_per_pair = G * S / k
    if async_select == SELECT_ON_GATHER_STREAM:
        return 3 if keys_per_pair < 192 else 2
    return 1 if keys_per_pair >= 384 else 2


def carry_append(G, S, k):
    return G * S / k >= 192


def pick(G, S, k, layers, speculative=True, side_gathers=True):
    """-> (async_select, number of side streams)"""
    keys_per_pair = G * S / k
    if layers == 1 or not speculative:
        async_select = SELECT_ON_CALLER
    elif side_gathers and keys_per_pair >= 96:
        async_select = SELECT_ON_GATHER_STREAM
    else:
        async_select = SELECT_ON_OWN_STREAM
    return async_select, side_streams(async_select, G, S, k)

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
layer, or the non-speculative variant: everything on the caller's stream."""

SELECT_ON_CALLER, SELECT_ON_OWN_STREAM, SELECT_ON_GATHER_STREAM = 0, 1, 2


def side_streams(async_select, G, S, k):
    keys_per_pair = G * S / k
    if async_select == SELECT_ON_GATHER_STREAM:
        return 3 if keys_per_pair < 192 else 2
    return 1 if keys_per_pair >= 384 else 2


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

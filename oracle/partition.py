"""Oracle for the partitioner (test infrastructure only; never imported by the product).

Paper Section 2.2, Algorithm 1, in the reading listed for it: the printed
listing initialises one array and returns another, appends inside the release
loop and never revisits the layer that overflowed.  What the surrounding text
describes is a greedy walk over a chain of layers:

    cuts = [0]                      # a shard opens at layer 0
    for every layer i in order:
        if the open shard plus layer i no longer fits the memory bound:
            cuts.append(i)          # cut before i
            the open shard becomes {i} alone (memory of earlier layers released)

`fits(start, end)` is the caller's memory test for the shard of layers
start..end inclusive (the paper probes the GPU; the library uses a closed-form
footprint; both are inputs here).  A single layer that does not fit is an error.
"""


def partition(n_layers, fits):
    """List of first-layer indices of the shards of a chain of n_layers layers."""
    cuts = [0]
    start = 0
    for i in range(n_layers):
        if not fits(start, i):
            if i == start:
                raise MemoryError(f"layer {i} alone exceeds the memory bound")
            cuts.append(i)
            start = i
            if not fits(i, i):
                raise MemoryError(f"layer {i} alone exceeds the memory bound")
    return cuts


def equal_shard_size(n_layers, cuts):
    """Largest divisor of n_layers not above the shortest closed shard (every shard but the last is closed)."""
    bounds = cuts + [n_layers]
    closed = [bounds[j + 1] - bounds[j] for j in range(len(cuts) - 1)]
    k = min(closed) if closed else n_layers
    while n_layers % k:
        k -= 1
    return k

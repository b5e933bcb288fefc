"""Where the big arrays lie in device memory.

Device-memory plumbing only (torch allocations): no step of the method runs here.

On MI355X the time of the fused step depends on where x, G and z lie relative to each other and
to the code rows, by up to 8 % at d = 2^30: the step streams M + 3 arrays at once, and
(presumably) arrays whose addresses differ only in certain high bits meet in the same memory
channels and banks; plain two-array copies between any two such rows run at the same rate.
Measured in one process (M = 64, same messages): x, G, z as one contiguous [3][d] block
7.2-7.6 ms per QCMD+z step depending on the block's offset (period 16 GiB); the same three rows
taken from allocations 48 GiB apart 6.7-7.0 ms, every one of the 60 ordered choices among five such
rows being faster than the block.

The address mapping is not documented, so the helpers here do not compute a placement, they
measure one: `spread_rows` allocates candidate rows far apart (temporary spacer allocations
between them, returned to the driver afterwards) and `choose_rows` times a caller-supplied probe
for choices of k rows until one is as fast as the caller asks, and returns the fastest tried.
Candidates should come from several allocations of different kinds (separate rows and a
contiguous block): in some processes every choice among the separate rows is slow and the block
is fast, in most it is the other way round.
"""
import itertools

import torch


def spread_rows(n, numel, device, dtype=torch.float32, spacer_bytes=44 << 30, reserve_bytes=48 << 30):
    """n zero-filled 1-D tensors of `numel` elements whose allocations lie about `spacer_bytes`
    apart.  The spacers shrink so that `reserve_bytes` of device memory stay free for what the
    caller allocates next; returns (rows, spacer_bytes_used)."""
    row_bytes = numel * torch.empty((), dtype=dtype).element_size()
    free, _ = torch.cuda.mem_get_info(device)
    room = free - n * row_bytes - reserve_bytes
    spacer = max(0, min(spacer_bytes, room // max(n - 1, 1)))
    spacer -= spacer % (2 << 20)
    rows, spacers = [], []
    for i in range(n):
        rows.append(torch.zeros(numel, dtype=dtype, device=device))
        if i + 1 < n and spacer:
            spacers.append(torch.empty(spacer, dtype=torch.uint8, device=device))
    del spacers
    torch.cuda.synchronize(device)
    torch.cuda.empty_cache()                 # the spacers go back to the driver
    return rows, spacer


def choose_rows(rows, k, probe_ms, good_enough_ms=None, ordered=False):
    """probe_ms(*k rows) -> milliseconds, called for choices of k of the rows (every ordered choice
    with ordered=True, else every combination in index order) until one takes at most
    `good_enough_ms` (if given) or all have been tried.  Returns (indices of the fastest choice
    tried, {choice: ms})."""
    pick = itertools.permutations if ordered else itertools.combinations
    table = {}
    for c in pick(range(len(rows)), k):
        table[c] = float(probe_ms(*[rows[i] for i in c]))
        if good_enough_ms is not None and table[c] <= good_enough_ms:
            break
    best = min(table, key=table.get)
    return best, table

"""Token samples for parity checks at sizes where the oracle cannot evaluate every token.

Each output row of the layer depends on its own token only, so a sample of tokens is a valid
check; what a uniform sample can miss is the few rows that sit at the edges of the kernels' work
units (the last rows of an expert, the short tiles behind its full row blocks, tiles whose K range
is cut into slices).  `stratified_tokens` therefore starts from those rows, as the library's own
host-side work-list introspection reports them for the routing at hand, and fills up with random
tokens."""
import numpy as np

from paper_2508_19373_amd import binding as B


def edge_rows(offs, cap_rows, ffn_shard):
    """Permuted rows at the boundaries of every tile of both grouped GEMMs, the first and last
    row of every local expert, and a row inside every tile of the down projection that runs as
    K slices (one per tile and slice)."""
    offs = np.asarray(offs, dtype=np.int32)
    rows = set()
    for e in range(offs.size - 1):
        if offs[e + 1] > offs[e]:
            rows.update((int(offs[e]), int(offs[e + 1]) - 1))
    H, I_s = ffn_shard.hidden, ffn_shard.inter_slice
    even = B.moe_debug_tile_rows(cap_rows, ffn_shard) == 160
    for ncb in ((I_s + 127) // 128, (H + 255) // 256):
        units = B.moe_debug_even_units(offs, cap_rows, ncb) if even else B.moe_debug_gemm_units(offs, cap_rows, ncb)
        for h, e, row0, row_end, nb in units[units[:, 0] > 0]:
            if nb == 0 or nb == ncb - 1:
                rows.update((int(row0), int(min(row0 + h, row_end)) - 1))
    n_sliced = 0
    if not even and B.moe_ffn_workspace_bytes(cap_rows, ffn_shard) > 0:
        _, units = B.moe_debug_down_slices(offs, cap_rows, ffn_shard, with_units=True)
        for h, e, row0, nb, z, kt0, nk, srow in units[(units[:, 0] > 0) & (units[:, 4] >= 1)]:
            end = min(row0 + h, int(offs[e + 1]))
            rows.add(int(row0 + ((7 * z + 3 * nb) % max(end - row0, 1))))
            n_sliced += 1
    return np.array(sorted(rows), dtype=np.int64), n_sliced


def stratified_tokens(T, k, offs, row_src, ffn_shard, n_random, seed=1):
    """Sorted unique token ids: the tokens that own the edge rows, plus `n_random` random ones
    (all tokens if T is no larger than that).  Returns (tokens, number of edge rows, rows in sliced tiles)."""
    if T <= n_random:
        return np.arange(T), 0, 0
    rows, n_sliced = edge_rows(offs, T * k, ffn_shard)
    edge_tokens = np.unique(np.asarray(row_src)[rows] // k) if rows.size else np.array([], dtype=np.int64)
    rng = np.random.default_rng(seed)
    rnd = rng.choice(T, size=n_random, replace=False)
    return np.unique(np.concatenate([edge_tokens, rnd])), rows.size, n_sliced

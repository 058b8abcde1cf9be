"""Algorithmic work of one Expert-module call on one shard (what the method itself must do)."""


def algorithmic_work(shape, T, counts):
    """FLOPs and minimum HBM bytes the method itself needs for one layer on this shard
    (never padded tiles, never inactive experts)."""
    H, E, I_s = shape.hidden, shape.n_experts, shape.inter_slice
    R = int(sum(counts))
    active = int(sum(1 for c in counts if c > 0))
    flops = 6.0 * R * H * I_s
    if shape.router != "zipf":
        flops += 2.0 * T * H * E
    wbytes = 3.0 * H * I_s * 2 * active
    if shape.inter_shared:
        flops += 6.0 * T * H * shape.inter_shared_slice + 2.0 * T * H
        wbytes += 3.0 * H * shape.inter_shared_slice * 2
    bytes_ = wbytes + H * E * 4 + 2.0 * T * H * 2
    return flops, bytes_, R, active

"""Operation counts of the hot path (host arithmetic only): MAC = rows * K * cols on unpadded
shapes, OP = 2 * MAC.  The per-head figures reproduce Table I of the paper."""


def head_counts(N, I, O):
    """One self-attention head with N tokens, I inputs, O outputs per head (Table I)."""
    return dict(linear_pe=I * O, linear_mac=N * I * O, layernorm_pe=2 * O, delay_pe=N * O,
                qk_pe=N * N, qk_mac=N * N * O, pv_pe=N * O, pv_mac=N * N * O)


def block_macs(D, H, N, hidden=0):
    """MACs per image of each stage of the block chain."""
    dh = D // H
    m = dict(qkv=N * D * 3 * D, qk=H * N * N * dh, pv=H * N * N * dh, proj=N * D * D)
    if hidden:
        m["fc1"] = N * D * hidden
        m["fc2"] = N * hidden * D
    return m


def block_ops(D, H, N, hidden=0):
    return 2 * sum(block_macs(D, H, N, hidden).values())


def block_algorithmic_bytes(D, H, N, hidden=0, storage_a=4, storage_w=4):
    """HBM bytes per image the method itself must move (weights excluded, listed separately):
    every inter-kernel intermediate once written and once read, packed; fp32 output once."""
    a = storage_a / 8.0
    x = N * D * a
    per_image = x + 2 * (3 * N * D * a) + 2 * x          # X read, QKV write+read, O write+read
    if hidden:
        per_image += 2 * x + 2 * (N * hidden * a)        # X2 and H write+read
    per_image += N * D * 4                               # fp32 Y
    weights = (3 * D * D + D * D + 2 * D * hidden) * storage_w / 8.0
    return dict(per_image=per_image, weights=weights)

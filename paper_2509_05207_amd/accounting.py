"""Byte and batch accounting used by the benchmark's reports.

Follows the paper's worked example of the baseline transfer footprint
(Sec. 2.3 "Baseline GraphSAGE Model": feature tensor size, per-batch transfer,
batches per epoch)."""

MIB = float(1 << 20)
GIB = float(1 << 30)


def feature_bytes(n_rows: int, feat_dim: int, bytes_per_element: int) -> int:
    return n_rows * feat_dim * bytes_per_element


def batches_per_epoch(n_train: int, batch_size: int) -> int:
    """ceil(T / B): the last, partial batch is kept."""
    return -(-n_train // batch_size)


def gather_traffic_bytes(n_rows: int, row_bytes: int) -> int:
    """Algorithmic bytes of one feature-block gather: every row read once and
    written once, one 4-byte node ID and one 8-byte routing entry per row."""
    return n_rows * (2 * row_bytes + 4 + 8)


def gather_group(n_batches: int, rows_per_epoch: int, stride_bytes: int) -> int:
    """How many consecutive batches the benchmark stages per gather launch (the prefetcher's "next Q batches" at
    once, rg_gather_batches): the whole epoch if its feature blocks together stay under 4 GiB, else eight batches,
    doubled up to 64 while a launch would stage less than 512 MiB.  A launch has to be long enough to run at the
    memory system's rate: a single small batch is launch-bound."""
    if n_batches <= 0:
        return 1
    if rows_per_epoch * stride_bytes < (4 << 30):
        return n_batches
    g = 8
    while g < 64 and g < n_batches and rows_per_epoch / n_batches * g * stride_bytes < (512 << 20):
        g *= 2
    return g


# The sampler's arithmetic per scanned row entry: ten 32-bit integer operations for the key of a neighbour ID (an XOR,
# three multiplies, three shifts, two XORs and one add folded into them as the instruction set allows) and one compare
# against the running cut.  The vector unit's peak for such operations: 256 compute units x 64 lanes x 2.4 GHz, one
# operation per lane and cycle (no fused multiply-add or packed forms apply to 32-bit integer multiplies and XORs).
SAMPLER_INT_OPS_PER_ENTRY = 11
INT32_VECTOR_PEAK_TOPS = 256 * 64 * 2.4e9 / 1e12


def sampler_int_ops(scanned_row_entries: int) -> int:
    return SAMPLER_INT_OPS_PER_ENTRY * int(scanned_row_entries)

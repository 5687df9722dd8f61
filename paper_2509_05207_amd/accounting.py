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

"""Values the paper prints (tests/golden/paper_worked_example.txt) against the
accounting helpers and the oracle's batching."""
import os

from paper_2509_05207_amd import accounting as acc


def load():
    vals = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "paper_worked_example.txt")) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if line:
                k, v = [t.strip() for t in line.split("=")]
                vals[k] = float(v) if "." in v else int(v)
    return vals


def test_feature_tensor_footprint():
    g = load()
    b = acc.feature_bytes(g["reddit_nodes"], g["reddit_feat_dim"], g["bytes_per_element"])
    assert b == g["feature_tensor_bytes"]
    assert round(b / acc.MIB, 2) == g["feature_tensor_MiB"]


def test_per_batch_transfer():
    g = load()
    b = acc.feature_bytes(g["remote_nodes_per_batch"], g["reddit_feat_dim"], g["bytes_per_element"])
    assert b == g["per_batch_bytes"]
    assert round(b / acc.MIB, 2) == g["per_batch_MiB"]


def test_batches_per_epoch_keeps_the_partial_batch(orc):
    g = load()
    assert acc.batches_per_epoch(g["train_nodes"], g["batch_size"]) == g["batches_per_epoch"]
    assert orc.num_batches(g["train_nodes"], g["batch_size"]) == g["batches_per_epoch"]
    # the printed per-epoch total is the product of the two rounded figures
    assert abs(g["batches_per_epoch"] * g["per_batch_MiB"] - g["per_epoch_MiB_as_printed"]) < 0.6
    assert round(g["per_epoch_MiB_as_printed"] / 1024, 2) == g["per_epoch_GiB"]

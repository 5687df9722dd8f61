"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, no GPU).

tests/oracle_sanitizer_driver.c calls every entry point of oracle/rapidgnn_oracle.c over the `small` workload; it is
built together with the oracle's source with -fsanitize=address,undefined and run as an ordinary executable (one
thread, then several).  It must finish without a sanitizer report, and what it writes must equal, byte for byte,
what the ordinary build of the oracle returns through ctypes for the same inputs."""
import os
import subprocess

import numpy as np
import pytest

from paper_2509_05207_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    exe = tmp_path_factory.mktemp("san") / "oracle_sanitizer_driver"
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-Wall", "-Wextra", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", os.path.join(ROOT, "tests", "oracle_sanitizer_driver.c"),
           os.path.join(ROOT, "oracle", "rapidgnn_oracle.c"), "-o", str(exe)]
    subprocess.check_call(cmd)
    return str(exe)


def expected_bytes(orc, w, cfg, K, n_threads):
    """The driver's output sequence, produced with the ordinary build of the oracle."""
    parts = []
    indptr, indices, train = w.indptr.numpy(), w.indices.numpy(), w.train.numpy()
    is_local = w.is_local.numpy()
    feats = orc.Features(is_local, w.row_of.numpy(), w.local_rows.view(-1).numpy().view(np.uint8), w.stride_bytes,
                         w.remote_rows.view(-1).numpy().view(np.uint8), w.stride_bytes, w.row_bytes)

    def dump(s, blocks):
        for hop in range(s.L + 1):
            ids, off = s.frontier(hop)
            parts.extend([off.tobytes(), ids.tobytes()])
        for hop in range(s.L):
            so, nb = s.samples(hop)
            parts.extend([so.tobytes(), nb.tobytes()])
            if blocks:
                parts.append(s.block(hop).tobytes())

    s = orc.Schedule(indptr, indices, train, cfg.batch_size, cfg.fanout, cfg.s0, cfg.worker, cfg.epoch, n_threads=n_threads)
    dump(s, True)
    freq = orc.frequency([s], w.n_nodes)
    parts.append(freq.tobytes())
    ids, slot = orc.top_hot(freq, is_local, K)
    parts.extend([np.int64(ids.size).tobytes(), ids.tobytes(), slot.tobytes()])
    parts.append(orc.cache_fill(ids, feats, table_stride=w.stride_bytes).tobytes())
    for b in range(s.n_batches):
        parts.append(orc.gather_batch(s, b, feats, out_stride=w.row_bytes).tobytes())
        for so in (slot, None):
            st = orc.batch_stats(s, b, is_local, so)
            parts.append(np.array([st["n_rows"], st["n_local"], st["n_hit"], st["n_miss"]], np.uint64).tobytes())
    nb = s.n_batches
    if nb > 1:
        dump(orc.Schedule(indptr, indices, train, cfg.batch_size, cfg.fanout, cfg.s0, cfg.worker, cfg.epoch, batch_lo=nb - 1, batch_hi=nb), False)
    dump(orc.Schedule(indptr, indices, train, cfg.batch_size, cfg.fanout, cfg.s0, cfg.worker, cfg.epoch, n_threads=n_threads,
                      sampler="positions"), False)
    return b"".join(parts)


@pytest.mark.parametrize("K_mode", ["config", "zero", "all"])
@pytest.mark.parametrize("n_threads", [1, 3])
def test_oracle_runs_clean_under_asan_and_ubsan(driver, orc, tmp_path, n_threads, K_mode):
    w = synth.make_workload("small")
    cfg = w.cfg
    K = {"config": w.K, "zero": 0, "all": w.n_nodes}[K_mode]
    w.indptr.numpy().tofile(tmp_path / "indptr.i64")
    w.indices.numpy().tofile(tmp_path / "indices.i32")
    w.train.numpy().tofile(tmp_path / "train.i32")
    w.is_local.numpy().tofile(tmp_path / "is_local.u8")
    w.row_of.numpy().tofile(tmp_path / "row_of.i32")
    w.local_rows.view(-1).numpy().view(np.uint8).tofile(tmp_path / "local.u8")
    w.remote_rows.view(-1).numpy().view(np.uint8).tofile(tmp_path / "remote.u8")
    meta = [w.n_nodes, w.indices.numel(), w.train.numel(), cfg.batch_size, len(cfg.fanout), *cfg.fanout, cfg.s0, cfg.worker, cfg.epoch, K,
            w.row_bytes, w.stride_bytes, w.extra["n_local"], w.extra["n_remote"]]
    (tmp_path / "meta.txt").write_text(" ".join(str(int(x)) for x in meta) + "\n")
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:exitcode=23", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    p = subprocess.run([driver, str(tmp_path), str(n_threads)], capture_output=True, text=True, env=env, timeout=300)
    assert p.returncode == 0, f"driver failed ({p.returncode}):\n{p.stderr[-4000:]}"
    assert "runtime error" not in p.stderr and "AddressSanitizer" not in p.stderr and "LeakSanitizer" not in p.stderr, p.stderr[-4000:]
    got = (tmp_path / "out.bin").read_bytes()
    want = expected_bytes(orc, w, cfg, K, n_threads)
    assert len(got) == len(want) and got == want

"""Pins of the trace-packing oracle (appendix A.1, eq. 4: one record per token; only tested tokens are shipped):
a hand-worked case and the library's boolean compression."""
import numpy as np

import oracle


def test_hand_worked_case():
    traj = np.array([1, 2, 0, 0, 1, 2, 2, 0], np.int8)
    h = (np.arange(8 * 3).reshape(8, 3) * 10).astype(np.uint16)
    x = np.arange(100, 108, dtype=np.int32)
    r = oracle.trace_pack(traj, h=h, x_in=x)
    assert r["n"] == 5 and r["row_index"].tolist() == [0, 1, 4, 5, 6]
    assert r["h"].tolist() == [[0, 10, 20], [30, 40, 50], [120, 130, 140], [150, 160, 170], [180, 190, 200]]
    assert r["x_in"].tolist() == [100, 101, 104, 105, 106] and r["traj"].tolist() == [1, 2, 1, 2, 2]
    assert "y_out" not in r and "topk_ids" not in r


def test_equals_library_compress_and_edge_cases():
    rng = np.random.default_rng(3)
    for rows in (0, 1, 7, 300):
        traj = rng.integers(0, 3, rows).astype(np.int8)
        ids = rng.integers(-1, 50, (rows, 6)).astype(np.int32)
        lg = rng.integers(0, 65536, (rows, 6)).astype(np.uint16)
        y = rng.integers(-1, 9, rows).astype(np.int32)
        r = oracle.trace_pack(traj, topk_ids=ids, topk_logits=lg, y_out=y)
        keep = traj != 0
        assert r["n"] == int(keep.sum())
        assert np.array_equal(r["row_index"], np.flatnonzero(keep))
        assert np.array_equal(r["topk_ids"], np.compress(keep, ids, axis=0))
        assert np.array_equal(r["topk_logits"], np.compress(keep, lg, axis=0))
        assert np.array_equal(r["y_out"], np.compress(keep, y, axis=0))
    none = oracle.trace_pack(np.zeros(5, np.int8), x_in=np.arange(5, dtype=np.int32))
    assert none["n"] == 0 and none["x_in"].shape == (0,)
    allr = oracle.trace_pack(np.full(4, 2, np.int8), x_in=np.arange(4, dtype=np.int32))
    assert allr["row_index"].tolist() == [0, 1, 2, 3]

"""Oracle of the trace-record packing (paper appendix A.1, eq. 4: the inference server ships one record
(h, l, x_in, y_out, R) per token to the training side; section 3.3: accepted and rejected tokens both carry a
training signal, untested ones none).

TEST INFRASTRUCTURE ONLY.  The definition written out: the rows whose trajectory code R is not 0 (1 = on the
accepted path, 2 = tested and rejected), in ascending row order, each with its hidden row, its kept target
logits (ids and values), its input token, the token emitted after it and its code.  Plain Python loop.
"""
from __future__ import annotations

import numpy as np


def trace_pack(traj, h=None, topk_ids=None, topk_logits=None, x_in=None, y_out=None):
    """Returns dict(n, row_index [n], and the packed copy of every array that was given)."""
    traj = np.asarray(traj)
    rows = []
    for m in range(traj.shape[0]):
        if int(traj[m]) != 0:
            rows.append(m)
    out = dict(n=len(rows), row_index=np.array(rows, dtype=np.int32))
    for name, a in (("h", h), ("topk_ids", topk_ids), ("topk_logits", topk_logits), ("x_in", x_in), ("y_out", y_out),
                    ("traj", traj)):
        if a is None:
            continue
        a = np.asarray(a)
        packed = np.empty((len(rows),) + a.shape[1:], dtype=a.dtype)
        for p, m in enumerate(rows):
            packed[p] = a[m]
        out[name] = packed
    return out

"""Pins of the drafter-loss oracle (paper section 3.3, eq. 3: acceptance term plus lambda times the
discard term, both KL(p_target || p_draft); top-k filtering on discarded tokens).  Library routines, closed
forms and a finite-difference check of the gradient - none of them the oracle's own formula re-typed."""
import numpy as np
import torch
import torch.nn.functional as F

import gen
import oracle
from oracle.loss_oracle import bf16_bits_to_f64


def _case(seed=3, rows=10, vd=300, k=40, **kw):
    return gen.loss_inputs(seed, rows, vd, top_k=k, **kw)


def test_bf16_bits_decode():
    bits = np.array([0x3F80, 0xC000, 0x0000, 0x8000, 0x7F80, 0xFF80, 0x3DCC], np.uint16)
    got = bf16_bits_to_f64(bits)
    assert got[:4].tolist() == [1.0, -2.0, 0.0, -0.0] and np.signbit(got[3])
    assert got[4] == np.inf and got[5] == -np.inf
    assert got[6] == float(torch.tensor([0x3DCC], dtype=torch.int16).view(torch.bfloat16).double()[0])


def test_full_support_equals_library_kl_div():
    """K = Vd: every id is kept, so the row KL is the library's KL between two softmaxes."""
    z, ids, bits, traj = _case(rows=6, vd=50, k=50)
    r = oracle.draft_loss(z, ids, bits, traj, 0.3)
    t = torch.zeros(6, 50, dtype=torch.float64)
    t.scatter_(1, torch.from_numpy(ids.astype(np.int64)), torch.from_numpy(bf16_bits_to_f64(bits)))
    ref = F.kl_div(F.log_softmax(torch.from_numpy(z).double(), -1), F.softmax(t, -1), reduction="none").sum(-1)
    assert np.allclose(r["row_kl"], ref.numpy(), rtol=1e-12, atol=1e-14)


def test_top1_filter_is_cross_entropy_on_the_best_target_token():
    z, ids, bits, traj = _case(rows=8)
    traj[:] = 2
    r = oracle.draft_loss(z, ids, bits, traj, 1.0, discard_top_k=1)
    ce = F.cross_entropy(torch.from_numpy(z).double(), torch.from_numpy(ids[:, 0].astype(np.int64)), reduction="none")
    assert np.allclose(r["row_kl"], ce.numpy(), rtol=1e-12)
    assert np.isclose(r["loss"], ce.mean().item(), rtol=1e-12) and r["mean_accept"] == 0.0


def test_gradient_matches_central_differences_of_the_loss():
    z, ids, bits, traj = _case(seed=5, rows=7, vd=60, k=12, pad_rows=2)
    traj[:] = [1, 2, 0, 2, 1, 1, 2]
    lam, kd = 0.7, 5
    r = oracle.draft_loss(z, ids, bits, traj, lam, discard_top_k=kd)
    rng = np.random.default_rng(0)
    z64 = z.astype(np.float64)
    coords = [(m, int(ids[m, j])) for m in range(7) for j in (0, 3, 7) if ids[m, j] >= 0]
    coords += [(int(rng.integers(7)), int(rng.integers(60))) for _ in range(25)]
    h = 1e-5
    for m, v in coords:
        zp, zm = z64.copy(), z64.copy()
        zp[m, v] += h
        zm[m, v] -= h
        lp = oracle.draft_loss(zp, ids, bits, traj, lam, discard_top_k=kd, want_grad=False)["loss"]
        lm = oracle.draft_loss(zm, ids, bits, traj, lam, discard_top_k=kd, want_grad=False)["loss"]
        assert abs((lp - lm) / (2 * h) - r["grad"][m, v]) < 1e-8, (m, v)
    assert np.abs(r["grad"][2]).max() == 0.0                      # an unused row has no gradient
    assert np.allclose(r["grad"].sum(axis=1), 0.0, atol=1e-15)    # both distributions sum to one


def test_drafter_equal_to_target_gives_zero():
    z, ids, bits, traj = _case(rows=4, vd=80, k=20)
    traj[:] = 1
    z[:] = -1e30
    for m in range(4):
        z[m, ids[m]] = bf16_bits_to_f64(bits[m]).astype(np.float32)
    r = oracle.draft_loss(z, ids, bits, traj, 0.5)
    assert np.abs(r["row_kl"]).max() < 1e-12 and np.abs(r["grad"]).max() < 1e-12


def test_class_means_lambda_and_unused_rows():
    z, ids, bits, traj = _case(seed=9, rows=12)
    traj[:] = [1, 1, 2, 0, 2, 2, 1, 0, 0, 2, 1, 2]
    a = oracle.draft_loss(z, ids, bits, traj, 0.25, discard_top_k=9)
    kl = a["row_kl"]
    assert np.isclose(a["mean_accept"], kl[traj == 1].mean()) and np.isclose(a["mean_discard"], kl[traj == 2].mean())
    assert np.isclose(a["loss"], a["mean_accept"] + 0.25 * a["mean_discard"])
    # the batch twice over: same loss, half the gradient per row
    b = oracle.draft_loss(np.tile(z, (2, 1)), np.tile(ids, (2, 1)), np.tile(bits, (2, 1)), np.tile(traj, 2), 0.25,
                          discard_top_k=9)
    assert np.isclose(b["loss"], a["loss"], rtol=1e-13) and np.allclose(b["grad"][:12], a["grad"] / 2, rtol=1e-13)
    # changing unused rows changes nothing; without discarded rows the second term vanishes
    z2 = z.copy()
    z2[traj == 0] += 3.0
    assert oracle.draft_loss(z2, ids, bits, traj, 0.25, discard_top_k=9)["loss"] == a["loss"]
    t3 = np.where(traj == 2, 0, traj)
    c = oracle.draft_loss(z, ids, bits, t3, 0.25)
    assert c["mean_discard"] == 0.0 and np.isclose(c["loss"], a["mean_accept"])
    # the filter applies to discarded rows only
    d = oracle.draft_loss(z, ids, bits, traj, 0.25, discard_top_k=None)
    assert np.array_equal(d["row_kl"][traj == 1], kl[traj == 1]) and not np.allclose(d["row_kl"][traj == 2], kl[traj == 2])


def test_padding_and_minus_infinity_carry_no_mass():
    z, ids, bits, traj = _case(seed=11, rows=5, vd=90, k=30, pad_rows=5)
    traj[:] = 1
    full = oracle.draft_loss(z, ids, bits, traj, 0.5)
    for m in range(5):
        fin = (ids[m] >= 0) & (bf16_bits_to_f64(bits[m]) > -np.inf)
        n = int(fin.sum())
        assert 0 < n < 30 or n == 30
        one = oracle.draft_loss(z[m:m + 1], ids[m:m + 1, :n], bits[m:m + 1, :n], traj[m:m + 1], 0.5)
        assert np.isclose(one["row_kl"][0], full["row_kl"][m], rtol=1e-13)


def test_generator_rows_are_ordered_and_distinct():
    z, ids, bits, traj = gen.loss_inputs(2, 20, 1000, top_k=128, pad_rows=4)
    v = bf16_bits_to_f64(bits)
    for m in range(20):
        fin = v[m][np.isfinite(v[m])]
        assert (np.diff(fin) <= 0).all()
    for m in range(20):
        real = ids[m][ids[m] >= 0]
        assert len(np.unique(real)) == len(real) and real.max() < 1000
    assert set(np.unique(traj)) <= {0, 1, 2} and z.dtype == np.float32

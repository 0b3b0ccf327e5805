"""Pins of the 8-bit floating-point LM-head oracle (oracle_logits_fp8): the E4M3 decoding against
hand-computed values and a library conversion, the projection against a library float64 product of
library-decoded operands, and a unit-row weight that catches a transposed operand.  Paper: the
frontier targets are served in FP8 (sections 1, 4.3); the format and scaling are this build's reading."""
import numpy as np
import torch

import gen
import oracle


def test_e4m3_decoding_hand_values_and_library():
    hand = {0x00: 0.0, 0x38: 1.0, 0x40: 2.0, 0x3C: 1.5, 0x7E: 448.0, 0x01: 2.0 ** -9, 0x07: 7 * 2.0 ** -9,
            0x08: 2.0 ** -6, 0xC0: -2.0, 0xB8: -1.0, 0x77: 240.0}
    codes = np.array(sorted(hand), np.uint8)
    got = oracle.decode_e4m3(codes)
    assert got.tolist() == [hand[int(c)] for c in codes]
    allc = np.arange(256, dtype=np.uint8)
    mine = oracle.decode_e4m3(allc)
    lib = torch.from_numpy(allc).view(torch.float8_e4m3fn).float().numpy().astype(np.float64)
    nan = np.isnan(lib)
    assert nan.sum() == 2 and np.array_equal(np.isnan(mine), nan)
    assert np.array_equal(mine[~nan], lib[~nan])
    assert np.signbit(mine[0x80]) and mine[0x80] == 0.0


def test_fp8_logits_equal_library_product_of_library_decoded_operands():
    rng = np.random.default_rng(4)
    hid, hs = gen.quantize_e4m3_rows(rng.standard_normal((3, 5, 40)).astype(np.float32))
    W, ws = gen.quantize_e4m3_rows((rng.standard_normal((23, 40)) * 0.02).astype(np.float32))
    got = oracle.logits_fp8(hidden=hid, hidden_scale=hs, lm_head=W, lm_head_scale=ws)
    hd = torch.from_numpy(hid).view(torch.float8_e4m3fn).double().numpy() * hs.astype(np.float64)[..., None]
    wd = torch.from_numpy(W).view(torch.float8_e4m3fn).double().numpy() * ws.astype(np.float64)[:, None]
    ref = hd @ wd.T
    assert got.shape == (3, 5, 23)
    assert np.allclose(got, ref, rtol=1e-13, atol=1e-15)
    # the quantised operands stay close to what they were drawn from
    assert np.abs(gen.e4m3_rows_to_f32(hid, hs)).max() <= np.abs(hd).max() + 1e-6


def test_fp8_unit_rows_select_single_products():
    H, V = 16, 16
    hid = np.arange(2 * H, dtype=np.uint8).reshape(2, H) + 0x30      # codes 0x30.. : distinct positive values
    W = np.zeros((V, H), np.uint8)
    W[np.arange(V), (np.arange(V) * 5) % H] = 0x38                   # 1.0 at column 5v mod 16
    hs = np.array([0.5, 2.0], np.float32)
    ws = np.linspace(1.0, 2.5, V).astype(np.float32)
    got = oracle.logits_fp8(hidden=hid, hidden_scale=hs, lm_head=W, lm_head_scale=ws)
    dec = oracle.decode_e4m3(hid)
    for m in range(2):
        for v in range(V):
            assert got[m, v] == float(hs[m]) * dec[m, (v * 5) % H] * float(ws[v])


def test_fp8_workload_runs_through_the_acceptance_oracle():
    w = gen.llama_chain(41, batch=4, len_lo=20, len_hi=40, vocab=600, hidden_size=128, head_fp8=True, draft_noise=0.5)
    assert w.hidden.dtype == np.uint8 and w.lm_head.dtype == np.uint8 and w.head_dtype == "fp8"
    a = oracle.accept_workload(w, want_logits=True)
    # per-row scaling keeps the dequantised logits at the magnitude of the float32 recipe (N(0,1) x N(0, 0.02))
    assert 0.05 < a.logits.std() < 0.5
    assert a.accept_len.max() >= 1

"""Pins for the numeric oracle (rescale, INT8 quantisation, pruning, bf16 dequantisation, GEMV)."""
import numpy as np
import pytest
import torch

import oracle.quant as oq
import synth


def small_w(rows=64, cols=96, seed=1):
    return synth.gen_weight(rows, cols, seed)


def test_channel_scale_special_exponents():
    a = synth.gen_act_absmax(512, 3)
    assert (oq.channel_scale(a, 0.0) == 1.0).all()
    assert (oq.channel_scale(a, 1.0) == a).all()
    s = oq.channel_scale(a, 0.5).astype(np.float64)
    assert np.allclose(s * s, a.astype(np.float64), rtol=2e-7)  # Eq. 2 with alpha = 1/2


def test_rescale_is_along_input_channels_and_preserves_product():
    """Eq. 1: (X / s)(s W) = X W.  A rescale along the wrong axis fails this."""
    w = small_w(48, 80, 2)
    a = synth.gen_act_absmax(80, 2)
    s = oq.channel_scale(a, 0.5)
    x = np.random.default_rng(0).standard_normal(80)
    w2 = oq.rescale(w, s)
    assert w2.shape == w.shape
    y0 = w.astype(np.float64) @ x
    y1 = w2.astype(np.float64) @ (x / s.astype(np.float64))
    assert np.allclose(y0, y1, rtol=1e-5, atol=1e-7)
    assert np.array_equal(w2[:, 7], w[:, 7] * s[7])


def test_quantise_range_absmax_and_error_bound():
    w = small_w(128, 256, 3)
    q, scale = oq.quantise_rows(w)
    assert q.dtype == np.int8 and scale.dtype == np.float32 and scale.shape == (128,)
    assert q.min() >= -127 and q.max() <= 127
    assert (np.abs(q.astype(int)).max(axis=1) == 127).all()  # the row's absmax element maps to +-127
    err = np.abs(q.astype(np.float64) * scale[:, None].astype(np.float64) - w.astype(np.float64))
    assert (err <= 0.5000001 * scale[:, None]).all()  # nearest level
    assert np.array_equal(np.sign(q), np.sign(np.where(q == 0, 0, w)))


def test_round_half_to_even_and_true_division():
    # row absmax 127 -> scale exactly 1, so q = rint(w): halves go to the even neighbour
    w = np.array([[127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.49, -126.5]], dtype=np.float32)
    q, scale = oq.quantise_rows(w)
    assert scale[0] == 1.0
    assert q[0].tolist() == [127, 0, 2, 2, 0, -2, -2, 3, -126]


def test_power_of_two_row_gain_leaves_codes_unchanged():
    """Per-row absmax absorbs a whole-row gain: the x8 outlier rows change the scale, not the bytes."""
    w = small_w(32, 128, 4)
    q0, s0 = oq.quantise_rows(w)
    w8 = w.copy()
    w8[5] *= np.float32(8)
    q1, s1 = oq.quantise_rows(w8)
    assert np.array_equal(q0, q1)
    assert s1[5] == s0[5] * 8 and np.array_equal(np.delete(s0, 5), np.delete(s1, 5))


def test_zero_row():
    w = small_w(4, 32, 5)
    w[2] = 0
    q, s = oq.quantise_rows(w)
    assert s[2] == 1.0 and not q[2].any()


def test_quantise_tensor_one_scale_for_all_rows():
    w = small_w(64, 256, 12)
    q, scale = oq.quantise_tensor(w)
    assert scale.dtype == np.float32 and scale == np.float32(np.abs(w).max() / np.float32(127.0))
    i, j = np.unravel_index(np.argmax(np.abs(w)), w.shape)
    assert abs(int(q[i, j])) == 127  # the largest magnitude takes the end of the range
    assert (np.abs(w - q.astype(np.float32) * scale) <= scale * 0.5000001).all()
    # a power-of-two gain on the whole tensor changes the scale, not the codes
    q4, scale4 = oq.quantise_tensor(w * np.float32(4.0))
    assert np.array_equal(q4, q) and scale4 == scale * 4
    # rows of equal largest magnitude: per-tensor and per-row quantisation coincide
    w2 = w / np.abs(w).max(axis=1, keepdims=True)
    qt, st = oq.quantise_tensor(w2)
    qr, sr = oq.quantise_rows(w2)
    assert np.array_equal(qt, qr) and (sr == st).all()
    # an all-zero tensor
    qz, sz = oq.quantise_tensor(np.zeros((3, 5), np.float32))
    assert sz == 1 and not qz.any()


def test_prune_removes_plus_minus_one_only():
    q = np.arange(-127, 128, dtype=np.int16).astype(np.int8).reshape(1, -1)
    p = oq.prune(q)
    assert np.array_equal(p[q.astype(int) ** 2 > 1], q[q.astype(int) ** 2 > 1])
    assert not p[np.abs(q.astype(int)) <= 1].any()
    hist = np.bincount(p.view(np.uint8).ravel(), minlength=256)
    assert hist[0x01] == 0 and hist[0xFF] == 0 and hist[0] == 3


def test_prune_by_score_reaches_sparsity_and_reduces_to_magnitude():
    w = small_w(128, 256, 6)
    q, _ = oq.quantise_rows(w)
    a = synth.gen_act_absmax(256, 6)
    p = oq.prune_by_score(q, a, 0.2)
    frac = float((p == 0).mean())
    assert int(0.2 * q.size) / q.size <= frac < 0.23
    assert np.array_equal(p[p != 0], q[p != 0])
    ones = np.ones(256, dtype=np.float32)
    pm = oq.prune_by_score(q, ones, 0.2)  # equal channel norms: plain magnitude pruning
    thr = np.abs(q.astype(int))[pm == 0].max()
    assert (np.abs(q.astype(int))[pm != 0] > thr).all()


def test_bf16_round_matches_torch():
    r = np.random.default_rng(7)
    x = np.concatenate([r.standard_normal(4096).astype(np.float32) * 3,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.0e-39, 65280.0], dtype=np.float32)])
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oq.bf16_round(x), want)
    assert np.array_equal(oq.bf16_to_f64(want), torch.from_numpy(x).to(torch.bfloat16).double().numpy())


def test_dequant_bf16_is_one_product_one_rounding():
    w = small_w(16, 64, 8)
    q, s = oq.quantise_rows(w)
    got = oq.dequant_bf16(q, s)
    assert got.shape == q.shape and got.dtype == np.uint16
    for i in (0, 7, 15):  # element by element in Python floats (exact products of 8-bit x 24-bit)
        for j in (0, 13, 63):
            prod = np.float32(float(q[i, j]) * float(s[i]))
            assert got[i, j] == oq.bf16_round(np.array([prod], dtype=np.float32))[0]
    back = oq.bf16_to_f64(got)
    ref = q.astype(np.float64) * s[:, None]
    assert (np.abs(back - ref) <= np.abs(ref) * 2.0 ** -8).all()


def test_gemv_ref_closed_forms_and_loops():
    x_bits = synth.gen_activation_bf16(40, 9)
    x = oq.bf16_to_f64(x_bits)
    q = np.ones((3, 40), dtype=np.int8)
    q[1] = -2
    q[2, ::2] = 0
    s = np.array([0.5, 0.25, 2.0], dtype=np.float32)
    y = oq.gemv_ref(q, s, x_bits)
    assert np.allclose(y, [0.5 * x.sum(), -0.5 * x.sum(), 2.0 * x[1::2].sum()], rtol=1e-14)
    r = np.random.default_rng(1)
    q = r.integers(-127, 128, size=(5, 40)).astype(np.int8)
    y = oq.gemv_ref(q, s[[0, 1, 2, 0, 1]], x_bits)
    for i in range(5):
        acc = 0.0
        for j in range(40):
            acc += float(q[i, j]) * float(x[j])
        assert abs(y[i] - acc * float(s[[0, 1, 2, 0, 1]][i])) <= 1e-12 * max(1.0, abs(y[i]))


def test_generator_is_deterministic_and_shaped():
    w1 = synth.gen_weight(64, 128, synth.matrix_seed(0, 0))
    w2 = synth.gen_weight(64, 128, synth.matrix_seed(0, 0))
    assert np.array_equal(w1, w2) and w1.dtype == np.float32
    assert not np.array_equal(w1, synth.gen_weight(64, 128, synth.matrix_seed(0, 1)))
    big = synth.gen_weight(400, 64, 5)
    rowstd = big.std(axis=1)
    assert int((rowstd > 0.08).sum()) == 4  # 1 % of 400 rows carry the x8 gain
    a = synth.gen_act_absmax(4096, 1)
    assert a.min() > 0 and 0.8 < np.median(a) < 1.25
    assert [m.rows * m.cols for m in synth.LLAMA7B_LAYER] == [4096 * 4096] * 4 + [11008 * 4096] * 3
    assert sum(m.rows * m.cols for m in synth.LLAMA7B_LAYER) == 202375168
    assert sum(m.rows * m.cols for m in synth.LLAMA13B_LAYER) == 317194240


# ---------------------------------------------------------------- W8A8 product (Eq. 4)

def test_quantise_vector_closed_forms():
    x = np.array([0.0, 1.0, -2.0, 0.5, 2.0], dtype=np.float32)
    xq, s = oq.quantise_vector(x)
    assert s == np.float32(2.0) / np.float32(127.0)
    assert xq.tolist() == [0, 64, -127, 32, 127]  # 63.5 rounds to the even 64, 31.75 to 32
    xq, s = oq.quantise_vector(np.zeros(7, dtype=np.float32))
    assert s == 1.0 and not xq.any()
    r = np.random.default_rng(3)
    x = r.standard_normal(1000).astype(np.float32)
    xq, s = oq.quantise_vector(x)
    assert np.abs(xq).max() == 127 and np.abs(xq.astype(np.float64) * float(s) - x).max() <= float(s) * 0.5 * (1 + 1e-6)


def test_w8a8_sum_is_exact_and_matches_python_integers():
    r = np.random.default_rng(4)
    q = r.integers(-127, 128, (9, 48), dtype=np.int64).astype(np.int8)
    xq = r.integers(-127, 128, 48, dtype=np.int64).astype(np.int8)
    want = [sum(int(a) * int(b) for a, b in zip(row, xq)) for row in q]
    assert oq.gemv_w8a8_acc(q, xq).tolist() == want
    # the largest sum the library allows (16384 columns of 127 * 127) is far inside 32 bits
    big = oq.gemv_w8a8_acc(np.full((1, 16384), 127, np.int8), np.full(16384, -127, np.int8))
    assert big.tolist() == [-16384 * 127 * 127] and abs(int(big[0])) < 2 ** 31


def test_w8a8_result_against_real_arithmetic_and_special_cases():
    r = np.random.default_rng(5)
    q = r.integers(-127, 128, (40, 512), dtype=np.int64).astype(np.int8)
    scale = ((r.random(40) + 0.5) * 0.01).astype(np.float32)
    x = r.standard_normal(512).astype(np.float32)
    xq, sx = oq.quantise_vector(x)
    y = oq.gemv_w8a8(q, scale, xq, sx)
    real = oq.gemv_w8a8_acc(q, xq).astype(np.float64) * scale.astype(np.float64) * float(sx)
    assert y.dtype == np.float32
    assert (np.abs(y - real) <= np.abs(real) * 2.0 ** -22).all()  # an int-to-float rounding and two products
    # sums below 2^24 convert exactly, a power-of-two scale multiplies exactly: the result is the integer sum, scaled
    y2 = oq.gemv_w8a8(q[:, :64], np.full(40, 0.25, np.float32), xq[:64], np.float32(0.5))
    assert np.array_equal(y2.astype(np.float64), oq.gemv_w8a8_acc(q[:, :64], xq[:64]) * 0.125)
    # dequantise-then-multiply in fp64 is the same product up to the quantisation of x
    deq = (q.astype(np.float64) * scale.astype(np.float64)[:, None]) @ x.astype(np.float64)
    bound = np.abs(q.astype(np.float64) * scale.astype(np.float64)[:, None]).sum(axis=1) * float(sx) * 0.5
    assert (np.abs(y - deq) <= bound * (1 + 1e-6) + 1e-6).all()


def test_generator_and_quantiser_reproduce_the_recorded_digests():
    """The seeded draws (their order and dtype) and the oracle's rescale / quantise / prune arithmetic, end to end:
    the digests in tests/golden/quantised_hashes.txt were written by the script beside them from synth/ and
    oracle/quant.py alone; the library's quantiser is compared with the oracle's elsewhere."""
    import hashlib
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "quantised_hashes.txt")
    rows_seen = 0
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        rows, cols, layer, m, rescale, hq, hs = line.split()
        seed = synth.matrix_seed(int(layer), int(m))
        w = synth.gen_weight(int(rows), int(cols), seed)
        if int(rescale):
            w = oq.rescale(w, oq.channel_scale(synth.gen_act_absmax(int(cols), seed), 0.5))
        q, scale = oq.quantise_rows(w)
        q = oq.prune(q)
        assert hashlib.sha256(q.tobytes()).hexdigest() == hq, line
        assert hashlib.sha256(scale.tobytes()).hexdigest() == hs, line
        rows_seen += 1
    assert rows_seen == 4

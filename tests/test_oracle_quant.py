"""Pins for the oracle's integer quantisation of the compressed cache (Sec. 4.3):
hand-computed codes, exact recovery of on-grid inputs, the round-trip error bound,
flat groups, clamping, invariance of attention to the key zero point, and closeness
of 8-bit attention to the unquantised result."""
import numpy as np

from oracle import skv_oracle as O
from paper_2601_21686_amd import synth


def test_groups_are_runs_of_64_channels():
    assert O.group_slices(32) == [slice(0, 32)]
    assert O.group_slices(64) == [slice(0, 64)]
    assert O.group_slices(96) == [slice(0, 64), slice(64, 96)]
    assert O.group_slices(128) == [slice(0, 64), slice(64, 128)]


def test_static_codes_by_hand():
    # scale 0.5, zero -1: x -> (x + 1) / 0.5, half-way cases go to the even code, out of range clamps
    y = np.array([[-1.0, -0.75, -0.5, 0.0, 0.25, 0.75, 126.5, 200.0, -3.0, 0.126]])
    want = np.array([[0, 0, 1, 2, 2, 4, 255, 255, 0, 2]], np.uint8)
    #            (x+1)/.5 = 0, 0.5->0, 1, 2, 2.5->2, 3.5->4, 255, clamp, clamp, 2.252->2
    got = O.quantize_static(y, np.array([0.5], np.float32), np.array([-1.0], np.float32))
    assert np.array_equal(got, want)
    back = O.dequantize(got, np.array([0.5]), np.array([-1.0]))
    assert np.array_equal(back, want * 0.5 - 1.0)


def test_static_on_grid_inputs_are_recovered_exactly_per_group():
    rng = np.random.default_rng(0)
    r = 96
    scale = np.array([2.0 ** -5, 2.0 ** -3], np.float32)
    zero = np.array([-3.0, 1.5], np.float32)
    codes = rng.integers(0, 256, size=(40, r)).astype(np.uint8)
    y = O.dequantize(codes, scale, zero)
    assert np.array_equal(y[:, :64], codes[:, :64] * 2.0 ** -5 - 3.0)        # group 0 uses pair 0
    assert np.array_equal(y[:, 64:], codes[:, 64:] * 2.0 ** -3 + 1.5)        # group 1 uses pair 1
    assert np.array_equal(O.quantize_static(y, scale, zero), codes)


def test_static_round_trip_error_is_half_a_step_inside_the_range():
    rng = np.random.default_rng(1)
    y = rng.uniform(-2.0, 3.0, size=(200, 128))
    scale, zero = O.calibrate_static_range(y)
    assert scale.shape == (2,) and np.allclose(zero, [y[:, :64].min(), y[:, 64:].min()], rtol=1e-6)
    codes = O.quantize_static(y, scale, zero)
    assert codes.min() == 0 and codes.max() == 255
    back = O.dequantize(codes, scale, zero)
    step = np.repeat(scale.astype(np.float64), 64)[None]
    assert np.all(np.abs(back - y) <= step / 2 * (1 + 1e-4) + 1e-6)
    # beyond the calibrated range values clamp to the ends
    far = np.full((1, 128), 100.0)
    assert np.all(O.quantize_static(far, scale, zero) == 255)
    assert np.all(O.quantize_static(-far, scale, zero) == 0)


def test_dynamic_quantisation_by_hand_and_flat_groups():
    # group 0: values 0 .. 255/64 on a grid of 1/64: scale = 2^-6 exactly, zero = 0, codes = 64 * value
    k = np.arange(64) * 4 % 256
    row = np.concatenate([k / 64.0, np.full(32, 0.3)])[None]                # group 1 is flat
    row[0, 5] = 255 / 64.0
    row[0, 6] = 0.0
    codes, sb, zb = O.quantize_dynamic(row)
    assert O.bf16_bits_to_f64(sb)[0, 0] == 2.0 ** -6 and O.bf16_bits_to_f64(zb)[0, 0] == 0.0
    assert np.array_equal(codes[0, :64], (row[0, :64] * 64).astype(np.uint8))
    # flat group: scale falls back to 1, zero = bf16(0.3), all codes 0, and the value comes back as bf16(0.3)
    assert O.bf16_bits_to_f64(sb)[0, 1] == 1.0
    assert np.all(codes[0, 64:] == 0)
    back = O.dequantize(codes, O.bf16_bits_to_f64(sb), O.bf16_bits_to_f64(zb))
    assert np.array_equal(back[0, :64], row[0, :64])
    assert np.all(back[0, 64:] == O.round_to_bf16(0.3))


def test_dynamic_round_trip_error_bound_and_monotone_codes():
    rng = np.random.default_rng(2)
    y = rng.standard_normal((300, 128)) * np.exp(rng.uniform(-3, 3, (300, 1)))
    codes, sb, zb = O.quantize_dynamic(y)
    s = O.bf16_bits_to_f64(sb)
    z = O.bf16_bits_to_f64(zb)
    back = O.dequantize(codes, s, z)
    y32 = y                                    # the definition works on the float64 rows themselves
    for gi, g in enumerate(O.group_slices(128)):
        lo, hi = y32[:, g].min(1), y32[:, g].max(1)
        # zero is bf16(lo), scale is bf16((hi-lo)/255): both within 2^-8 relative of the exact values
        assert np.all(np.abs(z[:, gi] - lo) <= np.abs(lo) * 2.0 ** -8)
        assert np.all(np.abs(s[:, gi] - (hi - lo) / 255) <= (hi - lo) / 255 * 2.0 ** -8 * 1.01)
        # inside [z, z + 255 s] the error is half a step; outside, the overshoot adds to it
        over = np.maximum(0, y32[:, g] - (z[:, gi] + 255 * s[:, gi])[:, None]) + np.maximum(0, z[:, gi][:, None] - y32[:, g])
        assert np.all(np.abs(back[:, g] - y32[:, g]) <= s[:, gi][:, None] / 2 * (1 + 1e-4) + over + 1e-12)
        # codes are monotone in the value
        order = np.argsort(y32[:, g], axis=1)
        sorted_codes = np.take_along_axis(codes[:, g].astype(int), order, axis=1)
        assert np.all(np.diff(sorted_codes, axis=1) >= 0)
        assert np.all(codes[:, g].min(1) <= 1) and np.all(codes[:, g].max(1) >= 250)   # the range is used


def _quant_pair(rng, B, HQ, HKV, rk, rv, n):
    d = 128
    Pk64, Pk = synth.orthonormal_bases(1, HKV, d, rk)
    Pv64, Pv = synth.orthonormal_bases(2, HKV, d, rv)
    pk = O.bf16_bits_to_f64(synth.torch_bf16_to_bits(Pk))
    pv = O.bf16_bits_to_f64(synth.torch_bf16_to_bits(Pv))
    sk = synth.channel_scales(3, HKV, d)
    K = O.bf16_bits_to_f64(synth.torch_bf16_to_bits(synth.kv_activations(4, B, n, HKV, d, sk)))
    V = O.bf16_bits_to_f64(synth.torch_bf16_to_bits(synth.kv_activations(5, B, n, HKV, d, sk)))
    ngk = len(O.group_slices(rk))
    ks, kz = np.empty((HKV, ngk), np.float32), np.empty((HKV, ngk), np.float32)
    for h in range(HKV):
        ks[h], kz[h] = O.calibrate_static_range(np.concatenate([O.compress(K[b, :, h], pk[h]) for b in range(B)]))
    Lq = O.new_quant_layer(B, HQ, HKV, d, pk, pv, ks, kz, n)
    O.quant_project_append(Lq, K, V, 0)
    Lb = O.new_layer(B, HQ, HKV, d, pk, pv, n, store="bf16")
    O.project_append(Lb, K, V, 0)
    q = O.bf16_bits_to_f64(synth.torch_bf16_to_bits(synth.queries(6, B, HQ, d)))
    return Lq, Lb, q


def test_attention_does_not_depend_on_the_key_zero_point():
    # a shift of a group's zero point adds the same constant to every score of a query: softmax removes it
    rng = np.random.default_rng(3)
    Lq, _, q = _quant_pair(rng, 1, 4, 2, 96, 64, 200)
    a = O.quant_decode_attention(Lq, q, 200)
    Lq.k_zero = Lq.k_zero + np.array([[0.7, -1.3], [2.0, 0.25]], np.float32)
    b = O.quant_decode_attention(Lq, q, 200)
    assert np.allclose(a, b, rtol=1e-10, atol=1e-12)
    # the scale, in contrast, matters
    Lq.k_scale = Lq.k_scale * np.float32(1.5)
    assert not np.allclose(a, O.quant_decode_attention(Lq, q, 200), rtol=1e-3)


def test_eight_bit_cache_stays_close_to_the_unquantised_cache():
    rng = np.random.default_rng(4)
    Lq, Lb, q = _quant_pair(rng, 2, 8, 2, 64, 64, 600)
    a = O.quant_decode_attention(Lq, q, 600)
    b = O.decode_attention(Lb, q, 600)
    err = np.max(np.abs(a - b), axis=-1) / np.max(np.abs(b), axis=-1)
    assert err.max() < 3e-2            # "essentially unchanged" at 8 bits (Sec. 4.3)
    assert err.max() > 1e-6            # but it is a different cache


def test_quant_append_places_rows_and_leaves_the_rest():
    # Selection bases (P = columns of the identity) make the projection a copy of chosen channels, so every
    # code and range below is worked out by hand.  Keys: scale 0.5, zero -2 -> code = rne((x + 2) / 0.5).
    B, HKV, d, r, cap, T, cur = 2, 2, 128, 32, 10, 3, 4
    pick = [(7 * c + 3) % d for c in range(r)]                       # channel c of a row = input channel pick[c]
    P = np.zeros((HKV, d, r))
    for h in range(HKV):
        P[h, pick, np.arange(r)] = 1.0
    L = O.new_quant_layer(B, HKV, HKV, d, P, P, np.full((HKV, 1), 0.5), np.full((HKV, 1), -2.0), cap)
    L.k_codes[:] = 77
    L.v_codes[:] = 78
    L.v_scale_bits[:] = 0x1234
    L.v_zero_bits[:] = 0x4321
    hand_in = [-2.0, -1.75, -1.5, -0.75, 0.0, 0.124, 10.0, 125.5, 125.75, 300.0, -9.0, 1.25]
    hand_code = [0, 0, 1, 2, 4, 4, 24, 255, 255, 255, 0, 6]
    #  (x+2)/.5:  0, .5->0, 1, 2.5->2, 4, 4.248->4, 24, 255, 255.5->clamp, clamp, clamp at 0, 6.5->6
    K = np.zeros((B, T, HKV, d))
    V = np.zeros((B, T, HKV, d))
    want_k = np.zeros((B, HKV, T, r), np.uint8)
    want_v = np.zeros((B, HKV, T, r), np.uint8)
    want_s = np.zeros((B, HKV, T), np.float64)
    want_z = np.zeros((B, HKV, T), np.float64)
    for b in range(B):
        for t in range(T):
            for h in range(HKV):
                rot = 5 * b + 3 * t + h
                for c in range(r):
                    K[b, t, h, pick[c]] = hand_in[(c + rot) % len(hand_in)]
                    want_k[b, h, t, c] = hand_code[(c + rot) % len(hand_in)]
                # values: a row spanning [z, z + 255 s] with s a power of two and entries on the grid z + n s,
                # plus entries a quarter step above a level (round down) and three quarters above (round up)
                s_, z_ = 2.0 ** -(1 + (rot % 3)), float(rot % 4) - 1.5
                n_ = [(37 * c + rot) % 256 for c in range(r)]
                n_[0], n_[1] = 0, 255
                frac = [0.0, 0.25, 0.75, 0.0][rot % 4]
                for c in range(r):
                    off = frac if 2 <= c < r - 1 and n_[c] < 255 else 0.0
                    V[b, t, h, pick[c]] = z_ + (n_[c] + off) * s_
                    want_v[b, h, t, c] = n_[c] + (1 if off > 0.5 else 0)
                want_s[b, h, t], want_z[b, h, t] = s_, z_
    K[:, :, :, [p_ for p_ in range(d) if p_ not in pick]] = 999.0            # channels the basis does not select
    O.quant_project_append(L, K, V, cur)
    rest = np.ones(cap, bool)
    rest[cur:cur + T] = False
    assert np.all(L.k_codes[:, :, rest] == 77) and np.all(L.v_codes[:, :, rest] == 78)
    assert np.all(L.v_scale_bits[:, :, rest] == 0x1234) and np.all(L.v_zero_bits[:, :, rest] == 0x4321)
    assert np.array_equal(L.k_codes[:, :, cur:cur + T], want_k)
    assert np.array_equal(L.v_codes[:, :, cur:cur + T], want_v)
    assert np.array_equal(O.bf16_bits_to_f64(L.v_scale_bits[:, :, cur:cur + T, 0]), want_s)
    assert np.array_equal(O.bf16_bits_to_f64(L.v_zero_bits[:, :, cur:cur + T, 0]), want_z)


def test_codes_are_decided_in_float64():
    # Inputs a hair on either side of a rounding boundary that float32 cannot tell apart: the definition is
    # evaluated in float64, so they receive different codes.
    eps = 2.0 ** -40
    y = np.array([[1.5 - eps, 1.5 + eps, 2.5 - eps, 2.5 + eps, 0.0, 255.0]])
    got = O.quantize_static(y, np.array([1.0], np.float32), np.array([0.0], np.float32))
    assert got.tolist() == [[1, 2, 2, 3, 0, 255]]
    cd, sb, zb = O.quantize_dynamic(y)
    assert O.bf16_bits_to_f64(sb)[0, 0] == 1.0 and O.bf16_bits_to_f64(zb)[0, 0] == 0.0
    assert cd.tolist() == [[1, 2, 2, 3, 0, 255]]


def test_four_bit_codes_by_hand_and_round_trip():
    # 16 levels: scale 0.5, zero -1 -> codes 0..15, half-way cases to the even code, clamping at 15
    y = np.array([[-1.0, -0.75, -0.5, 0.25, 6.5, 6.4, 7.0, -2.0]])
    want = np.array([[0, 0, 1, 2, 15, 15, 15, 0]], np.uint8)
    #            (x+1)/.5 =  0, 0.5->0, 1, 2.5->2, 15, 14.8->15, 16->clamp, clamp
    got = O.quantize_static(y, np.array([0.5], np.float32), np.array([-1.0], np.float32), bits=4)
    assert np.array_equal(got, want)
    rng = np.random.default_rng(3)
    # on-grid inputs come back exactly; the calibrated range spans codes 0..15; error at most half a step
    codes = rng.integers(0, 16, size=(30, 128)).astype(np.uint8)
    scale, zero = np.array([0.25, 2.0 ** -4], np.float32), np.array([-2.0, 0.5], np.float32)
    assert np.array_equal(O.quantize_static(O.dequantize(codes, scale, zero), scale, zero, bits=4), codes)
    x = rng.uniform(-1.0, 2.0, size=(100, 64))
    sc, zr = O.calibrate_static_range(x, bits=4)
    c = O.quantize_static(x, sc, zr, bits=4)
    assert c.min() == 0 and c.max() == 15
    assert np.all(np.abs(O.dequantize(c, sc, zr) - x) <= sc[0] / 2 * (1 + 1e-4) + 1e-6)
    # per-row ranges: scale = bf16((max - min) / 15)
    row = np.concatenate([np.arange(64) % 16 * 0.125, np.full(64, 3.0)])[None]
    cd, sb, zb = O.quantize_dynamic(row, bits=4)
    assert O.bf16_bits_to_f64(sb)[0, 0] == 0.125 and O.bf16_bits_to_f64(zb)[0, 0] == 0.0
    assert np.array_equal(cd[0, :64], np.arange(64) % 16)
    assert O.bf16_bits_to_f64(sb)[0, 1] == 1.0 and np.all(cd[0, 64:] == 0)          # flat group

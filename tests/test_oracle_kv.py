"""Pins for the oracle's gather and key re-rotation: copies are byte copies of
the pool rows and touch nothing else; the rotation is checked against closed
forms, the group law of rotations, numpy's complex exponential and torch's
float -> bf16 rounding."""
import math

import numpy as np
import pytest
import torch

import oracle as O

THETA = 500000.0


def bf16_bits(x):
    """float32 array -> bf16 bit patterns with torch's own rounding (library routine)."""
    t = torch.from_numpy(np.asarray(x, np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def bits_to_f64(b):
    return (np.asarray(b, np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


# ---------------------------------------------------------------- bf16 <-> double


def test_bf16_decode_known_values():
    assert O.bf16_to_double(0x3F80) == 1.0 and O.bf16_to_double(0x4000) == 2.0
    assert O.bf16_to_double(0xC0A0) == -5.0 and O.bf16_to_double(0x3F81) == 1.0 + 2.0**-7
    assert O.bf16_to_double(0x0001) == 2.0**-133 and O.bf16_to_double(0x0080) == 2.0**-126


def test_bf16_round_ties_to_even_and_range():
    assert O.double_to_bf16(1.0 + 2.0**-8) == 0x3F80  # tie -> even mantissa (down)
    assert O.double_to_bf16(1.0 + 3 * 2.0**-8) == 0x3F82  # tie -> even mantissa (up)
    assert O.double_to_bf16(1.0 + 2.0**-8 + 2.0**-40) == 0x3F81  # just above the tie
    assert O.double_to_bf16(-(1.0 + 2.0**-8 - 2.0**-40)) == 0xBF80
    assert O.double_to_bf16(0.0) == 0 and O.double_to_bf16(-0.0) == 0x8000
    assert O.double_to_bf16(2.0**-133 * 0.5) == 0  # tie between 0 and the smallest subnormal -> 0
    assert O.double_to_bf16(2.0**-133 * 1.5) == 2
    assert O.double_to_bf16(3.4e38) == 0x7F80 and O.double_to_bf16(float("inf")) == 0x7F80
    assert O.double_to_bf16(bits_to_f64([0x7F7F])[0]) == 0x7F7F  # largest finite stays


def test_bf16_roundtrip_all_patterns_and_torch_rounding():
    allb = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = bits_to_f64(allb)
    for b, v in zip(allb[::7], vals[::7]):
        if math.isnan(v):
            continue
        assert O.double_to_bf16(float(v)) == b
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(4000), rng.standard_normal(500) * 1e-30,
                        rng.standard_normal(500) * 1e30]).astype(np.float32)
    want = bf16_bits(x)
    got = np.array([O.double_to_bf16(float(v)) for v in x], np.uint16)
    assert np.array_equal(got, want)


# ---------------------------------------------------------------- rotation, double precision


@pytest.mark.parametrize("style", [0, 1])
def test_rotation_matches_complex_exponential(style):
    rng = np.random.default_rng(1)
    D = 128
    x = rng.standard_normal(D)
    for delta in [1, -1, 17, -512, 512, 4097, -100000]:
        y = O.rope_head_f64(x, delta, THETA, style)
        j = np.arange(D // 2)
        ang = delta * THETA ** (-2.0 * j / D)
        if style == 0:
            z = (x[: D // 2] + 1j * x[D // 2 :]) * np.exp(1j * ang)
            want = np.concatenate([z.real, z.imag])
        else:
            z = (x[0::2] + 1j * x[1::2]) * np.exp(1j * ang)
            want = np.empty(D)
            want[0::2], want[1::2] = z.real, z.imag
        assert np.abs(y - want).max() < 1e-11 * max(1.0, abs(delta) / 512)


def test_rotation_first_pair_turns_by_delta_radians():
    x = np.zeros(128)
    x[0], x[64] = 1.0, 0.0  # pair j = 0 has frequency theta^0 = 1
    y = O.rope_head_f64(x, 3.0, THETA, 0)
    assert abs(y[0] - math.cos(3.0)) < 1e-15 and abs(y[64] - math.sin(3.0)) < 1e-15
    # the slowest pair (j = 63) turns by delta * theta^(-126/128)
    x = np.zeros(128)
    x[63] = 1.0
    y = O.rope_head_f64(x, 100.0, THETA, 0)
    a = 100.0 * math.exp(-126.0 / 128.0 * math.log(THETA))
    assert abs(y[63] - math.cos(a)) < 1e-14 and abs(y[127] - math.sin(a)) < 1e-14


@pytest.mark.parametrize("style", [0, 1])
def test_rotation_group_law_and_norm(style):
    rng = np.random.default_rng(2)
    for D in (64, 128):
        k = rng.standard_normal(D)
        for p, d in [(5, 7), (300, -300), (512, 512), (-13, 1000)]:
            a = O.rope_head_f64(O.rope_head_f64(k, p, THETA, style), d, THETA, style)
            b = O.rope_head_f64(k, p + d, THETA, style)
            assert np.abs(a - b).max() < 1e-12  # rot(rot(k, p), d) = rot(k, p + d)
        y = O.rope_head_f64(k, 123, THETA, style)
        if style == 0:
            n0, n1 = k[: D // 2] ** 2 + k[D // 2 :] ** 2, y[: D // 2] ** 2 + y[D // 2 :] ** 2
        else:
            n0, n1 = k[0::2] ** 2 + k[1::2] ** 2, y[0::2] ** 2 + y[1::2] ** 2
        assert np.abs(n0 - n1).max() < 1e-13  # every pair keeps its length
        assert np.array_equal(O.rope_head_f64(k, 0, THETA, style), k)


def test_styles_are_the_same_rotation_on_permuted_elements():
    rng = np.random.default_rng(3)
    D = 128
    x = rng.standard_normal(D)
    perm = np.empty(D, int)  # interleaved position of half-split element
    perm[: D // 2], perm[D // 2 :] = np.arange(0, D, 2), np.arange(1, D, 2)
    xi = np.empty(D)
    xi[perm] = x
    y0 = O.rope_head_f64(x, 77, THETA, 0)
    y1 = O.rope_head_f64(xi, 77, THETA, 1)
    assert np.array_equal(y1[perm], y0)


# ---------------------------------------------------------------- rotation on bf16 rows


def test_bf16_rotation_is_one_rounding_of_the_double_result():
    rng = np.random.default_rng(4)
    D = 128
    xb = bf16_bits(rng.standard_normal(D))
    for delta in [1, -37, 512]:
        yb = O.rope_head(xb, delta, THETA, 0)
        y = O.rope_head_f64(bits_to_f64(xb), delta, THETA, 0)
        assert np.array_equal(yb, np.array([O.double_to_bf16(float(v)) for v in y], np.uint16))
        # undoing the shift comes back within 2 bf16 steps of the input
        zb = O.rope_head(yb, -delta, THETA, 0)
        err = np.abs(bits_to_f64(zb) - bits_to_f64(xb))
        step = np.maximum(np.abs(bits_to_f64(xb)), 2.0**-126) * 2.0**-7
        r = np.hypot(bits_to_f64(xb)[:64], bits_to_f64(xb)[64:])
        assert (err <= 2 * np.maximum(step, np.concatenate([r, r]) * 2.0**-8)).all()
    assert np.array_equal(O.rope_head(xb, 0, THETA, 0), xb)


# ---------------------------------------------------------------- gather


def _layouts(L, H, D, n_pool, n_tok, pool_token_major):
    rb = H * D * 2
    pool_l = O.Layout(L, H, D, L * 2 * rb, 2 * rb, rb) if pool_token_major else O.Layout(L, H, D, rb, 2 * n_pool * rb,
                                                                                         n_pool * rb)
    dst_l = O.Layout(L, H, D, rb, 2 * n_tok * rb, n_tok * rb)
    return pool_l, dst_l


@pytest.mark.parametrize("token_major", [True, False])
def test_gather_copies_exactly_the_span_rows(token_major):
    rng = np.random.default_rng(5)
    L, H, D, S, N = 3, 2, 8, 50, 40
    re = H * D
    pool = rng.integers(0, 65536, (S, L, 2, re) if token_major else (L, 2, S, re)).astype(np.uint16)
    row = (lambda s, l, kv: pool[s, l, kv]) if token_major else (lambda s, l, kv: pool[l, kv, s])
    dst = np.full((L, 2, N, re), 0xAAAA, np.uint16)
    pool_l, dst_l = _layouts(L, H, D, S, N, token_major)
    src, dpos, ln = [10, 3, 44], [0, 7, 30], [4, 1, 6]
    O.gather_kv(pool, pool_l, dst, dst_l, src, dpos, ln)
    covered = np.zeros(N, bool)
    for s, d, n in zip(src, dpos, ln):
        for k in range(n):
            covered[d + k] = True
            for l in range(L):
                for kv in range(2):
                    assert np.array_equal(dst[l, kv, d + k], row(s + k, l, kv))
    assert (dst[:, :, ~covered] == 0xAAAA).all()  # unmatched positions are left for the engine
    # no spans: nothing happens
    dst2 = np.full((L, 2, N, re), 0xAAAA, np.uint16)
    O.gather_kv(pool, pool_l, dst2, dst_l, [], [], [])
    assert (dst2 == 0xAAAA).all()


def test_gather_with_rotation_touches_only_keys_of_shifted_spans():
    rng = np.random.default_rng(6)
    L, H, D, S, N = 2, 2, 64, 20, 12
    pool = bf16_bits(rng.standard_normal((S, L, 2, H * D))).reshape(S, L, 2, H * D)
    dst = np.full((L, 2, N, H * D), 0xAAAA, np.uint16)
    pool_l, dst_l = _layouts(L, H, D, S, N, True)
    src, dpos, ln, delta = [5, 9], [1, 6], [3, 2], [0, -19]
    O.gather_kv(pool, pool_l, dst, dst_l, src, dpos, ln, delta, O.Rope(THETA, 0))
    for k in range(3):  # delta = 0: plain copy, K and V
        assert np.array_equal(dst[:, :, 1 + k], pool[5 + k])
    for k in range(2):
        assert np.array_equal(dst[:, 1, 6 + k], pool[9 + k, :, 1])  # V copied
        for l in range(L):
            for h in range(H):
                want = O.rope_head(pool[9 + k, l, 0, h * D : (h + 1) * D], -19, THETA, 0)
                assert np.array_equal(dst[l, 0, 6 + k, h * D : (h + 1) * D], want)
    # without rope parameters the deltas are ignored
    dst2 = np.full((L, 2, N, H * D), 0xAAAA, np.uint16)
    O.gather_kv(pool, pool_l, dst2, dst_l, src, dpos, ln, delta, None)
    assert np.array_equal(dst2[:, :, 6], pool[9])


def test_rotation_against_80_digit_arithmetic():
    """cpo_rope_head (double precision, libm) against cos/sin summed in 80-digit decimals, up to the largest deltas
    an int32 holds: equal bf16 values up to |delta| ~ 2^21, at most one step apart beyond (there the product
    delta * frequency is itself rounded to about 2^-22 rad in double precision)."""
    from tests.exact_rope import exact_rotation

    def ordinal(bits):
        b = bits.astype(np.int32)
        return np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)

    rng = np.random.default_rng(8)
    for dl, tol in ((1, 0), (-3, 0), (511, 0), (-512, 0), (40000, 0), (-2097151, 0), ((1 << 28) + 12345, 1), (2**31 - 1, 1),
                    (-(2**31), 1)):
        x = (rng.standard_normal(128).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
        got = O.rope_head(x, dl, 500000.0, 0)
        want = exact_rotation(x, dl, 500000.0, 128)
        assert np.abs(ordinal(got) - ordinal(want)).max() <= tol, dl

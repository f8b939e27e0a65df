"""Pins of the oracle's E4M3 quantisation (8-bit storage of the K/V cache): the format's value table, exhaustive
round trips, nearest-value brute force with ties to even, saturation, scale closed forms, an independent library
cast, and the rollout that carries codes."""
import numpy as np
import pytest

from oracle import pafu_oracle as orc


def _all_finite_codes():
    c = np.arange(256, dtype=np.uint8)
    return c[(c & 0x7F) != 0x7F]


def test_value_table_of_the_format():
    # hand-computed from the definition: sign, exponent bias 7, 3 mantissa bits, subnormals below 2^-6
    table = {0x00: 0.0, 0x01: 2.0 ** -9, 0x07: 7 * 2.0 ** -9, 0x08: 2.0 ** -6, 0x38: 1.0, 0x39: 1.125, 0x3C: 1.5,
             0x40: 2.0, 0x7E: 448.0, 0x77: 240.0, 0xB8: -1.0, 0xFE: -448.0, 0x0F: 1.875 * 2.0 ** -6, 0x30: 0.5}
    for code, value in table.items():
        assert orc.dequantise_e4m3(np.array([code], np.uint8))[0] == value, hex(code)
        assert orc.quantise_e4m3(np.array([value]))[0] == code, hex(code)
    assert np.isnan(orc.dequantise_e4m3(np.array([0x7F, 0xFF], np.uint8))).all()
    assert orc.quantise_e4m3(np.array([np.nan]))[0] & 0x7F == 0x7F
    assert orc.quantise_e4m3(np.array([-0.0]))[0] == 0x80          # the sign of zero is kept


def test_every_code_survives_a_round_trip_and_the_grid_is_monotone():
    codes = _all_finite_codes()
    vals = orc.dequantise_e4m3(codes)
    back = orc.quantise_e4m3(vals)
    assert np.array_equal(back, codes)
    pos = vals[codes < 0x80]
    assert np.all(np.diff(pos) > 0) and pos[0] == 0.0 and pos[-1] == 448.0
    assert len(pos) == 127


def test_rounds_to_the_nearest_value_ties_to_the_even_mantissa():
    codes = _all_finite_codes()
    codes = codes[codes < 0x80]
    grid = orc.dequantise_e4m3(codes)
    rng = np.random.default_rng(3)
    x = np.concatenate([rng.uniform(0, 460, 4000), rng.uniform(0, 0.05, 4000), np.abs(rng.standard_normal(4000)),
                        (grid[:-1] + grid[1:]) / 2.0])           # includes every midpoint (exact in float64)
    got = orc.quantise_e4m3(x)
    for xi, gi in zip(x, got):
        d = np.abs(grid - min(xi, 448.0))
        best = np.flatnonzero(d == d.min())
        want = best[0] if len(best) == 1 else [b for b in best if codes[b] % 2 == 0][0]
        assert gi == codes[want], (xi, gi, codes[want])
    # two midpoints spelled out: between 1.0 (mantissa 0) and 1.125 -> 1.0; between 1.125 and 1.25 (mantissa 2) -> 1.25
    assert orc.quantise_e4m3(np.array([1.0625, 1.1875])).tolist() == [0x38, 0x3A]
    # midpoint between the largest subnormal and the smallest normal goes to the normal (even: mantissa 0)
    assert orc.quantise_e4m3(np.array([7.5 * 2.0 ** -9]))[0] == 0x08


def test_saturation_symmetry_and_scale():
    assert orc.quantise_e4m3(np.array([449.0, 1e9, np.inf])).tolist() == [0x7E] * 3
    assert orc.quantise_e4m3(np.array([-1e9, -np.inf])).tolist() == [0xFE] * 2
    x = np.random.default_rng(1).standard_normal(2000) * 3
    assert np.array_equal(orc.quantise_e4m3(-x), orc.quantise_e4m3(x) ^ 0x80)
    for e in (-7, -3, 0, 2):
        assert np.array_equal(orc.quantise_e4m3(x, e), orc.quantise_e4m3(x / 2.0 ** e))
        codes = orc.quantise_e4m3(x, e)
        assert np.array_equal(orc.dequantise_e4m3(codes, e), orc.dequantise_e4m3(codes) * 2.0 ** e)
        # relative error of a normal value is at most half a mantissa step: 2^-4
        back = orc.dequantise_e4m3(codes, e)
        big = (np.abs(x) >= 2.0 ** (e - 6)) & (np.abs(x) <= 448.0 * 2.0 ** e)     # normal and not saturated
        assert np.all(np.abs(back[big] - x[big]) <= np.abs(x[big]) * 2.0 ** -4 + 1e-300)


def test_agrees_with_an_independent_library_cast_inside_the_range():
    torch = pytest.importorskip("torch")
    if not hasattr(torch, "float8_e4m3fn"):
        pytest.skip("this torch has no float8_e4m3fn")
    x = np.random.default_rng(5).standard_normal(20000).astype(np.float32) * 20.0
    x = x[np.abs(x) < 440.0]
    lib = torch.from_numpy(x).to(torch.float8_e4m3fn)
    assert np.array_equal(lib.view(torch.uint8).numpy(), orc.quantise_e4m3(x))
    assert np.array_equal(lib.to(torch.float32).numpy().astype(np.float64), orc.dequantise_e4m3(orc.quantise_e4m3(x)))


def test_rollout_with_a_code_cache_equals_the_plain_rollout_on_dequantised_tensors():
    rng = np.random.default_rng(9)
    N, D, Lc, F, M, k, ek, ev = 2, 16, 12, 8, 4, 20, -5, -6
    W1, W2 = rng.standard_normal((M, F)) * 0.3, rng.standard_normal((1, M)) * 0.3
    st8 = orc.RolloutState(N, D, np.uint8)
    st = orc.RolloutState(N, D, np.float64)
    for t in range(4):
        X = rng.standard_normal((Lc, F))
        Q, K, V = (rng.standard_normal((Lc, N, D)) for _ in range(3))
        out8 = orc.rollout_step_fp8(st8, X, W1, None, W2, None, Q, K, V, k, Lc, ek, ev)
        Kd = orc.dequantise_e4m3(orc.quantise_e4m3(K, ek), ek)
        Vd = orc.dequantise_e4m3(orc.quantise_e4m3(V, ev), ev)
        out = orc.rollout_step(st, X, W1, None, W2, None, Q, Kd, Vd, k, Lc)
        assert np.array_equal(out8["ids"], out["ids"])
        assert np.allclose(out8["O"], out["O"], rtol=1e-12, atol=1e-14)
        assert st8.K.dtype == np.uint8 and st8.n == st.n
        assert np.array_equal(orc.dequantise_e4m3(st8.K, ek), st.K) and np.array_equal(orc.dequantise_e4m3(st8.V, ev), st.V)
    assert st8.n == k + Lc
    # the quantisation error of the attention output stays at the format's level (about 2^-4 / sqrt(keys) relative)
    assert np.abs(Kd - K).max() <= np.abs(K).max() * 2.0 ** -4

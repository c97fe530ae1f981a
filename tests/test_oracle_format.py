"""Pins for the oracle's E2M1 format, rounding rule and packing (App. A)."""
import numpy as np
import pytest

from oracle import fp4_oracle as o

F32 = np.float32
GRID15 = [-6, -4, -3, -2, -1.5, -1, -0.5, 0, 0.5, 1, 1.5, 2, 3, 4, 6]


def test_decode_matches_printed_table(golden):
    rows = golden("e2m1_table.txt")
    assert len(rows) == 16
    seen = set()
    for bits, val in rows:
        code = int(bits, 2)
        seen.add(code)
        assert float(o.e2m1_decode(np.array([code], np.uint8))[0]) == float(val)
    assert seen == set(range(16))
    # 15 distinct values, max 6 (Sec. 2: MAX_fp4 = 6.0)
    vals = o.e2m1_decode(np.arange(16, dtype=np.uint8))
    assert len(set(vals.tolist())) == 15 and vals.max() == 6.0 == float(o.FP4_MAX)


def test_code_layout_is_sign_exp_mantissa():
    # value = (-1)^s * (e == 0 ? m/2 : (1 + m/2) * 2^(e-1)), the E2M1 definition (bias 1)
    for code in range(16):
        s, e, m = code >> 3, (code >> 1) & 3, code & 1
        v = (m * 0.5) if e == 0 else (1 + 0.5 * m) * 2.0 ** (e - 1)
        v = -v if s else v
        assert float(o.e2m1_decode(np.array([code], np.uint8))[0]) == v


def test_chain_at_every_printed_threshold(golden):
    rows = golden("q_listing_thresholds.txt")
    bounds = [float(r[0]) for r in rows]
    values = [float(r[1]) for r in rows]
    for i, b in enumerate(bounds[:-1]):
        b32 = F32(b)
        below = np.nextafter(b32, F32(-np.inf))
        above = np.nextafter(b32, F32(np.inf))
        got = o.q_e2m1_value(np.array([below, b32, above], F32))
        assert got[0] == values[i]            # strictly below the bound
        assert got[1] == values[i + 1]        # on the bound: not '<', falls through
        assert got[2] == values[i + 1]
    # ties go towards +inf for either sign
    t = o.q_e2m1_value(np.array([0.25, -0.25, 2.5, -2.5, 5, -5, 0.75, -0.75], F32))
    assert t.tolist() == [0.5, 0.0, 3.0, -2.0, 6.0, -4.0, 1.0, -0.5]


def _nearest_ties_up(v):
    """Independent definition: nearest of the 15 grid values, the larger one on a tie."""
    best = None
    for g in GRID15:
        d = abs(float(v) - g)
        if best is None or d < best[0] or (d == best[0] and g > best[1]):
            best = (d, g)
    return best[1]


def test_q_is_nearest_neighbour_bruteforce():
    rng = np.random.default_rng(1)
    v = np.concatenate([rng.uniform(-7, 7, 4000), rng.normal(0, 1, 2000),
                        np.arange(-28, 29) * 0.25]).astype(F32)
    got = o.q_e2m1_value(v)
    want = np.array([_nearest_ties_up(x) for x in v], F32)
    assert np.array_equal(got, want)


def test_q_idempotent_monotone_saturating():
    g = np.array(GRID15, F32)
    assert np.array_equal(o.q_e2m1_value(g), g)
    v = np.sort(np.random.default_rng(2).uniform(-8, 8, 10000).astype(F32))
    q = o.q_e2m1_value(v)
    assert np.all(np.diff(q) >= 0)
    assert np.all(np.abs(q[np.abs(v) <= 6] - v[np.abs(v) <= 6]) <= 1.0)
    sp = o.q_e2m1_value(np.array([6.5, 1e30, np.inf, -6.5, -1e30, -np.inf, np.nan], F32))
    assert sp.tolist() == [6, 6, 6, -6, -6, -6, 6]


def test_codes_agree_with_values_and_never_emit_negative_zero():
    v = np.random.default_rng(3).uniform(-7, 7, 20000).astype(F32)
    v = np.concatenate([v, np.array([-0.0, 0.0, -0.1, -0.25, -0.2499], F32)])
    codes = o.q_e2m1(v)
    assert np.array_equal(o.e2m1_decode(codes), o.q_e2m1_value(v))
    assert not np.any(codes == 8)
    assert codes.max() <= 15


def test_pack_nibble_order_and_roundtrip():
    codes = np.array([[1, 2, 3, 15], [7, 0, 9, 4]], np.uint8)
    packed = o.pack_codes(codes)
    assert packed.tolist() == [[0x21, 0xF3], [0x07, 0x49]]
    assert np.array_equal(o.unpack_codes(packed), codes)
    r = np.random.default_rng(4).integers(0, 16, (5, 64)).astype(np.uint8)
    assert np.array_equal(o.unpack_codes(o.pack_codes(r)), r)


def test_bf16_rounding_matches_library_cast():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(5)
    y = rng.normal(size=50000) * np.exp(rng.normal(size=50000) * 8)
    y = np.concatenate([y, [1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, -1 - 2.0 ** -8, 0.0, 2.0 ** -133 * 1.5]])
    want = torch.from_numpy(y).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(o.round_to_dtype(y, "bf16"), want)
    assert np.array_equal(o.round_to_dtype(y, "f32"), y.astype(F32))

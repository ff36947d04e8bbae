"""Pins for the oracle's quantiser, packing and fp16 conversion (CPU only).

Everything here is checked against something other than the oracle itself: values worked by
hand from Sec. 2.1 Eq. 2-3 (tests/golden), the paper's printed memory table, numpy's own
float16 converter, and invariants that the arithmetic fixes.
"""
import numpy as np
import pytest

import oracle


def _parse_cases(path):
    cases, cur = [], None
    for line in path.read_text().splitlines():
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *rest = line.split()
        if key == "case":
            cur = {"name": rest[0]}
            cases.append(cur)
        else:
            cur[key] = [float(t) for t in rest]
    return cases


def _unpack(codes):
    """Independent nibble split: even element = low nibble (Eq. 5)."""
    codes = np.asarray(codes, np.uint8)
    out = np.empty(codes.shape[:-1] + (codes.shape[-1] * 2,), np.uint8)
    out[..., 0::2] = codes & 0xF
    out[..., 1::2] = codes >> 4
    return out


def test_closed_form_groups(golden_dir):
    cases = _parse_cases(golden_dir / "quant_closed_forms.txt")
    assert len(cases) >= 8 and {int(c.get("g", [32])[0]) for c in cases} == {32, 64, 128}
    for c in cases:
        g = int(c.get("g", [32])[0])
        x = np.array(c["x"], np.float16)
        assert len(c["x"]) == g == len(c["q"]), c["name"]
        assert np.array_equal(x.astype(np.float64), np.array(c["x"])), c["name"]
        codes, s, z = oracle.quantize(x[None, :], group=g)
        assert s.shape == (1, 1) and codes.shape == (1, g // 2), c["name"]
        assert float(s[0, 0]) == c["s"][0], c["name"]
        assert float(z[0, 0]) == c["z"][0], c["name"]
        assert _unpack(codes)[0].tolist() == [int(v) for v in c["q"]], c["name"]
        # Eq. 3 with the hand-derived triple: x^ = (q - z) s
        xhat = (np.array(c["q"]) - c["z"][0]) * c["s"][0]
        assert np.array_equal(oracle.dequantize(codes, s, z)[0], xhat), c["name"]
        if c["name"] not in ("ties", "halves_64", "quarters_128"):   # on-grid inputs reconstruct exactly
            assert np.array_equal(xhat, np.array(c["x"])), c["name"]
        if g == 32:
            # the same values repeated fill a group of 64 or 128 with the same min and max: same s and z, codes repeated
            for big in (64, 128):
                xb = np.tile(x, big // 32)[None, :]
                cb, sb, zb = oracle.quantize(xb, group=big)
                assert float(sb[0, 0]) == c["s"][0] and float(zb[0, 0]) == c["z"][0], (c["name"], big)
                assert _unpack(cb)[0].tolist() == [int(v) for v in c["q"]] * (big // 32), (c["name"], big)


GROUPS = [32, 64, 128]


@pytest.mark.parametrize("g", GROUPS)
@pytest.mark.parametrize("e", [-10, -3, 0, 2, 5])
@pytest.mark.parametrize("m", [-1024, -37, -8, 0, 5, 600, 1009])
def test_power_of_two_ramps(e, m, g):
    # x = (m + k) 2^e with k covering 0..15  =>  s = 2^e, z = -m, q = k   (Eq. 2-3, exact arithmetic)
    rng = np.random.default_rng(100 * (e + 20) + (m + 2000) + g)
    k = np.concatenate([np.arange(16), rng.integers(0, 16, g - 16)])
    rng.shuffle(k)
    x64 = (m + k) * 2.0 ** e
    x = x64.astype(np.float16)
    assert np.array_equal(x.astype(np.float64), x64)
    codes, s, z = oracle.quantize(x[None], group=g)
    assert float(s[0, 0]) == 2.0 ** e and float(z[0, 0]) == -m
    assert np.array_equal(_unpack(codes)[0], k)


def test_constant_group_and_signed_zero():
    for val in [0.0, -0.0, 3.25, -117.0, 6.1e-5, 65504.0]:
        x = np.full((1, 32), val, np.float16)
        codes, s, z = oracle.quantize(x)
        assert s.view(np.uint16)[0, 0] == 0x3C00            # scale 1.0
        assert not np.any(codes)
        assert z.view(np.uint16)[0, 0] != 0x8000            # never -0
        assert np.array_equal(oracle.dequantize(codes, s, z)[0], x[0].astype(np.float64))


def test_underflowing_range_uses_unit_scale():
    # range/15 below half the smallest fp16 subnormal -> stored scale would be 0 -> rule: 1.0
    x = np.zeros((1, 32), np.float16)
    x[0, 5] = np.float16(2.0 ** -24)                        # range 2^-24, /15 rounds to 0 in fp16
    codes, s, z = oracle.quantize(x)
    assert s.view(np.uint16)[0, 0] == 0x3C00
    assert np.all(_unpack(codes) == 0)


def test_zero_point_saturates():
    x = np.full((1, 32), -60000.0, np.float16)
    x[0, 0] = np.float16(-60000.0 + 32.0)                   # tiny range, huge |min|/range
    codes, s, z = oracle.quantize(x)
    assert np.isfinite(z.astype(np.float64)).all()
    assert abs(float(z[0, 0])) <= 65504.0


def _roundtrip_inputs():
    rng = np.random.default_rng(12345)
    a = rng.standard_normal((4096, 128)).astype(np.float16)
    b = (rng.standard_normal((1024, 256)) * 0.1).astype(np.float16)
    c = rng.standard_normal((1024, 128))
    c[:, [3, 40, 77, 101]] *= 8.0                            # outlier channels
    return [a, b, c.astype(np.float16)]


@pytest.mark.parametrize("g", GROUPS)
def test_roundtrip_error_at_most_half_a_step(g):
    # |x^ - x| <= s/2 per element (plus fp32 rounding of x/s+z) whenever nothing clamps, i.e. |z| <= 1024
    for x in _roundtrip_inputs():
        codes, s, z = oracle.quantize(x, group=g)
        assert np.all(np.abs(z.astype(np.float64)) <= 1024)
        xh = oracle.dequantize(codes, s, z)
        step = np.repeat(s.astype(np.float64), g, axis=-1)
        err = np.abs(xh - x.astype(np.float64))
        assert np.all(err <= step * (0.5 + 1e-3))
        # the step really is the group's range / 15 up to fp16 rounding
        xg = x.astype(np.float64).reshape(x.shape[0], -1, g)
        rng_ = xg.max(-1) - xg.min(-1)
        assert np.allclose(s.astype(np.float64), rng_ / 15, rtol=2 ** -11 * 1.01, atol=0)


@pytest.mark.parametrize("g", GROUPS)
def test_min_maps_to_0_and_max_to_15(g):
    for x in _roundtrip_inputs():
        codes, s, z = oracle.quantize(x, group=g)
        q = _unpack(codes).reshape(x.shape[0], -1, g)
        xg = x.reshape(x.shape[0], -1, g)
        assert np.all(np.take_along_axis(q, xg.argmin(-1)[..., None], -1) == 0)
        assert np.all(np.take_along_axis(q, xg.argmax(-1)[..., None], -1) == 15)
        assert set(np.unique(q)) == set(range(16))


def test_a_larger_group_never_has_a_finer_step():
    """A group of 64 (128) is the union of two (four) groups of 32: its range, hence its stored scale, is at least
    the largest of theirs (fp16 rounding is monotone), and equal where one part already spans the whole range."""
    for x in _roundtrip_inputs():
        s32 = oracle.quantize(x, group=32)[1].astype(np.float64)
        for g in (64, 128):
            sg = oracle.quantize(x, group=g)[1].astype(np.float64)
            parts = s32.reshape(x.shape[0], -1, g // 32)
            assert np.all(sg >= parts.max(-1))
            xg = x.astype(np.float64).reshape(x.shape[0], -1, g)
            x32 = x.astype(np.float64).reshape(x.shape[0], -1, g // 32, 32)
            spans_all = (x32.max(-1) - x32.min(-1)).max(-1) == xg.max(-1) - xg.min(-1)
            assert np.all(sg[spans_all] == parts.max(-1)[spans_all])


@pytest.mark.parametrize("g", GROUPS)
def test_codes_match_independent_numpy_evaluation(g):
    """Eq. 2-3 evaluated with numpy float32 ops and numpy's own fp16 rounding."""
    for x in _roundtrip_inputs():
        xf = x.astype(np.float32).reshape(x.shape[0], -1, g)
        mn, mx = xf.min(-1), xf.max(-1)
        s16 = ((mx - mn) / np.float32(15)).astype(np.float16)
        sf = s16.astype(np.float32)
        assert np.all(sf > 0)
        z16 = ((np.float32(0) - mn) / sf).astype(np.float16)
        v = xf / sf[..., None] + z16.astype(np.float32)[..., None]
        q = np.clip(np.rint(v), 0, 15).astype(np.uint8).reshape(x.shape)
        codes, s, z = oracle.quantize(x, group=g)
        assert np.array_equal(s.view(np.uint16), s16.view(np.uint16))
        assert np.array_equal(z.view(np.uint16), z16.view(np.uint16))
        assert np.array_equal(_unpack(codes), q)


def test_nibble_order_matches_eq5_masks():
    # Eq. 5: packed stream viewed as uint16; element j of a 4-tuple is (w & (0xF << 4j)) >> 4j
    x = np.tile(np.arange(16, dtype=np.float16), 2)[None, :]            # codes == values
    perm = np.random.default_rng(3).permutation(32)
    x = np.concatenate([x, x[:, perm]], 0)
    codes, s, z = oracle.quantize(x)
    w = codes.view("<u2")                                                # [2, 8]
    for j in range(4):
        got = (w & (0xF << (4 * j))) >> (4 * j)
        assert np.array_equal(got, x[:, j::4].astype(np.uint16))


def test_pack_unpack_all_byte_values(golden_dir):
    txt = (golden_dir / "packed_bytes.txt").read_text().splitlines()
    rec = {l.split()[0]: l.split()[1:] for l in txt if l and not l.startswith("#")}
    codes = np.array([int(b, 16) for b in rec["bytes"]], np.uint8)[None]
    s = np.array([[float(rec["s"][0])]], np.float16)
    z = np.array([[float(rec["z"][0])]], np.float16)
    assert oracle.dequantize(codes, s, z)[0].tolist() == [float(v) for v in rec["xhat"]]
    # every byte value: dequantise with s=1, z=0 gives (low nibble, high nibble)
    allb = np.arange(256, dtype=np.uint8).reshape(16, 16)
    one = np.ones((16, 1), np.float16)
    xh = oracle.dequantize(allb, one, one * 0)
    assert np.array_equal(xh[:, 0::2], (allb & 0xF).astype(np.float64))
    assert np.array_equal(xh[:, 1::2], (allb >> 4).astype(np.float64))


def test_format_size_and_paper_memory_table(golden_dir):
    rows = [l.split() for l in (golden_dir / "memory_table.txt").read_text().splitlines()
            if l and not l.startswith("#")]
    gib = 2.0 ** 30
    for r in rows:
        if r[0] == "compression":
            ratio = oracle.kv_bytes_fp16(80, 8, 131072, 128) / oracle.kv_bytes_int4(80, 8, 131072, 128)
            assert round(ratio, 1) == float(r[1])
            continue
        S, fp16_gb, int4_gb = int(r[0]), float(r[1]), float(r[2])
        assert round(oracle.kv_bytes_fp16(80, 8, S, 128) / gib, 1) == fp16_gb
        assert round(oracle.kv_bytes_int4(80, 8, S, 128) / gib + 1e-9, 1) == int4_gb
    assert oracle.kv_bytes_fp16(80, 8, 131072, 128) == 40 * 2 ** 30          # Eq. 1
    # 5.0 bits per element including fp16 scale and zero-point per group of 32
    assert oracle.kv_bytes_int4(1, 1, 1, 128) * 8 / (2 * 128) == 5.0
    codes, s, z = oracle.quantize(np.zeros((7, 256), np.float16))
    assert (codes.nbytes + s.nbytes + z.nbytes) * 8 / (7 * 256) == 5.0
    # groups of g elements: 4 bits of code + 32 bits of fp16 scale and zero-point per g elements (Sec. 2.1)
    for g, bits in ((32, 5.0), (64, 4.5), (128, 4.25)):
        assert oracle.kv_bytes_int4(1, 1, 1, 128, group=g) * 8 / (2 * 128) == bits
        codes, s, z = oracle.quantize(np.zeros((7, 256), np.float16), group=g)
        assert (codes.nbytes + s.nbytes + z.nbytes) * 8 / (7 * 256) == bits
        assert oracle.kv_bytes_int4(80, 8, 131072, 128, group=g) == 2 * 80 * 8 * 131072 * 128 * bits / 8   # Eq. 1's form


def test_fp16_to_fp32_exhaustive_against_numpy():
    L = oracle.lib()
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float32)
    got = np.array([L.orc_half_to_float(int(b)) for b in bits], np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), ref[~nan].view(np.uint32))
    back = np.array([L.orc_float_to_half(float(v)) for v in ref[~nan]], np.uint16)
    assert np.array_equal(back, bits[~nan])


def test_fp32_to_fp16_rne_against_numpy():
    L = oracle.lib()
    rng = np.random.default_rng(99)
    pats = [rng.integers(0, 2 ** 32, 150000, dtype=np.uint64).astype(np.uint32)]
    # every halfway point and its two fp32 neighbours, subnormal range and overflow edge included
    h = np.arange(0, 0x7C00, dtype=np.uint16).view(np.float16).astype(np.float64)
    mid = ((h[:-1] + h[1:]) / 2).astype(np.float32)
    for arr in (mid, np.nextafter(mid, np.float32(np.inf)), np.nextafter(mid, np.float32(-np.inf))):
        pats += [arr.view(np.uint32), (-arr).view(np.uint32)]
    edge = np.array([65504, 65519.99, 65520, 65536, 1e9, 2.0 ** -25, np.nextafter(np.float32(2.0 ** -25), np.float32(1)),
                     2.0 ** -24, 2.0 ** -14, 0.0, -0.0], np.float32)
    pats.append(edge.view(np.uint32))
    f = np.concatenate(pats).view(np.float32)
    f = f[np.isfinite(f)]
    with np.errstate(over="ignore"):
        ref = f.astype(np.float16).view(np.uint16)
    got = np.array([L.orc_float_to_half(float(v)) for v in f], np.uint16)
    assert np.array_equal(got, ref)


def test_dense_fp16_dequant_is_single_rounding():
    rng = np.random.default_rng(5)
    x = (rng.standard_normal((512, 128)) * 3).astype(np.float16)
    codes, s, z = oracle.quantize(x)
    exact = oracle.dequantize(codes, s, z)
    with np.errstate(over="ignore"):
        ref = exact.astype(np.float16)            # numpy rounds fp64 -> fp16 once
    assert np.array_equal(oracle.dequantize_f16(codes, s, z).view(np.uint16), ref.view(np.uint16))

"""Pins for the CPU oracle: every function of oracle/oqm_oracle.c is checked against
something other than itself - numbers the paper prints (tests/golden/), closed forms,
invariants, library routines (torch / numpy) and brute force.  CPU only."""
import json
import os

import numpy as np
import pytest
import torch

HERE = os.path.dirname(os.path.abspath(__file__))


def _rng(seed):
    return np.random.default_rng(seed)


# --------------------------------------------------------------------------- paper numbers
@pytest.fixture(scope="module")
def golden():
    with open(os.path.join(HERE, "golden", "paper_closed_forms.json")) as f:
        return json.load(f)


def test_kv_cache_footprint_matches_paper(oracle, golden):
    g = golden["kv_cache_one_hour"]
    b = oracle.kv_cache_bytes(g["L"], g["N"], g["H_kv"], g["d_h"], g["elem_bytes"], g["frames"])
    assert b == g["product_bytes"]                       # the footnote's product, exactly
    assert round(b / 2 ** 30, 1) == g["printed_GB"]      # "about 18.8 GB"


def test_compression_ratio_matches_paper(oracle, golden):
    g = golden["compression_ratio"]
    r = oracle.compression_ratio(g["N"], g["G"], g["bits"])
    assert r == pytest.approx(4 * g["N"] / g["G"], rel=1e-15)   # Eq. 10: 4N/G
    assert round(r, 1) == g["printed"]
    one_hour = golden["kv_cache_one_hour"]["product_bytes"] / 2 ** 30 / r
    assert round(one_hour, 1) == golden["compressed_one_hour_GB"]["printed"]


def test_ablation_ratio_column(oracle, golden):
    for row in golden["ablation_ratio_percent"]["rows"]:
        pct = 100.0 / oracle.compression_ratio(196, row["tokens"], row["bits"])
        assert round(pct + 1e-9, 1) == row["printed"], row


def test_k_from_budget(oracle, golden):
    g = golden["retrieval_budget"]
    assert g["frames"] * g["tokens_per_frame"] == g["budget_tokens"]
    # 196-token groups: the budget is exactly 64 groups once enough is stored
    assert oracle.k_from_budget(g["budget_tokens"], 196, 1000 * 196) == 64
    # paper's G = 50: ceil(12544 / 50) = 251
    assert oracle.k_from_budget(g["budget_tokens"], g["G"], 10 ** 9) == 251
    # fewer groups stored than the budget allows: T / G wins
    assert oracle.k_from_budget(g["budget_tokens"], g["G"], 7 * 50) == 7
    assert oracle.k_from_budget(1, 50, 500) == 1


def test_bits_per_element(oracle):
    assert oracle.bits_per_element(4, oracle.QAXIS_HEAD_DIM, 64, 196) == 5.0
    assert oracle.bits_per_element(4, oracle.QAXIS_HEAD_DIM, 32, 196) == 6.0
    assert oracle.bits_per_element(4, oracle.QAXIS_TOKENS, 64, 50) == pytest.approx(4 + 64 / 50)


# --------------------------------------------------------------------------- dtype conversion
def test_bf16_roundtrip_against_torch(oracle):
    x = torch.randn(20000, generator=torch.Generator().manual_seed(3)) * 37.0
    x = torch.cat([x, torch.tensor([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38,
                                    1e-40, -1e-40, 65504.0, 2.0 ** -126])])
    ref = x.to(torch.bfloat16)
    got = oracle.from_f32(x.numpy(), oracle.BF16)
    assert np.array_equal(got, ref.view(torch.int16).numpy().view(np.uint16))
    back = oracle.to_f32(got, oracle.BF16)
    assert np.array_equal(back, ref.float().numpy())


def test_f16_against_numpy(oracle):
    # every finite binary16 pattern widens exactly
    bits = np.arange(0, 1 << 16, dtype=np.uint16)
    finite = (bits & 0x7c00) != 0x7c00
    wide = oracle.to_f32(bits[finite], oracle.F16)
    assert np.array_equal(wide, bits[finite].view(np.float16).astype(np.float32))
    # narrowing: random values, halves between representable values, subnormals, overflow
    r = _rng(5)
    x = np.concatenate([
        r.standard_normal(50000).astype(np.float32) * 100,
        r.standard_normal(50000).astype(np.float32) * 1e-5,
        r.standard_normal(20000).astype(np.float32) * 1e-7,
        np.array([65504, 65519.99, 65520, 65536, 1e6, 2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0001,
                  3 * 2.0 ** -25, 0.0, -0.0, 1 + 2.0 ** -11, 1 + 3 * 2.0 ** -11, 6.1e-5],
                 np.float32)])
    x = np.concatenate([x, -x])
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16).view(np.uint16)
    assert np.array_equal(oracle.from_f32(x, oracle.F16), ref)


# --------------------------------------------------------------------------- quantizer
def _torch_quant_headdim(x, gs, levels=15):
    """Library-routine statement of Eq. 9 along head_dim, float32 torch CPU ops."""
    G, d = x.shape
    t = torch.from_numpy(x).view(G, d // gs, gs)
    mn = t.amin(-1, keepdim=True) + 0.0
    mx = t.amax(-1, keepdim=True)
    s = (mx - mn) / float(levels)
    ok = s >= torch.finfo(torch.float32).tiny
    s = torch.where(ok, s, torch.zeros_like(s))
    inv = torch.where(ok, 1.0 / torch.where(ok, s, torch.ones_like(s)), torch.zeros_like(s))
    # float32 difference, then the exact product (float64 holds it exactly), rounded once
    c = torch.clamp(torch.round((t - mn).double() * inv.double()), 0, levels).to(torch.uint8)
    return c.view(G, d).numpy(), s.view(G, d // gs).numpy(), mn.view(G, d // gs).numpy()


@pytest.mark.parametrize("G,d,gs,bits", [(16, 64, 32, 4), (7, 128, 64, 4), (50, 128, 32, 4),
                                         (5, 24, 8, 4), (3, 16, 16, 2), (9, 128, 64, 2)])
def test_quantize_tile_equals_torch_expression(oracle, G, d, gs, bits):
    r = _rng(G * 1000 + d + gs)
    x = (r.standard_normal((G, d)) * r.uniform(0.1, 30)).astype(np.float32)
    x[0, :gs] = 1.25                # a flat quant-group
    x[-1, 0] = -0.0
    codes, packed, scale, zero = oracle.quantize_tile(x, gs, oracle.QAXIS_HEAD_DIM, bits)
    tc, ts, tz = _torch_quant_headdim(x, gs, (1 << bits) - 1)
    assert np.array_equal(codes, tc)
    assert np.array_equal(scale.view(np.uint32), ts.view(np.uint32))
    assert np.array_equal(zero.view(np.uint32), tz.view(np.uint32))


@pytest.mark.parametrize("G,d,gs,bits,qaxis", [(16, 64, 32, 4, 0), (9, 128, 64, 2, 0), (50, 64, 64, 4, 1),
                                               (7, 32, 8, 2, 1)])
def test_bf16_metadata_variant(oracle, G, d, gs, bits, qaxis):
    """scale / zero kept in bfloat16: both are rounded (torch's own bfloat16 rounding) before
    the codes are taken, the codes are taken against the rounded pair and clamped, and the
    reconstruction stays within half a (rounded) step plus what the rounding of m and s moves."""
    r = _rng(G * 31 + d + bits)
    x = (r.standard_normal((G, d)) * r.uniform(0.1, 30) + r.uniform(-5, 5)).astype(np.float32)
    if qaxis == 0:
        x[0, :gs] = 1.25                                             # a flat quant-group
    levels = (1 << bits) - 1
    codes, packed, scale, zero = oracle.quantize_tile(x, gs, qaxis, bits, oracle.BF16)
    # library-routine statement
    t = torch.from_numpy(x)
    t = t.view(G, d // gs, gs) if qaxis == 0 else t.t().contiguous().view(d, 1, G)
    mn = t.amin(-1, keepdim=True) + 0.0
    mx = t.amax(-1, keepdim=True)
    s = (mx - mn) / float(levels)
    s = torch.where(s >= torch.finfo(torch.float32).tiny, s, torch.zeros_like(s))
    s = s.to(torch.bfloat16).float()
    m = mn.to(torch.bfloat16).float()
    ok = s >= torch.finfo(torch.float32).tiny
    inv = torch.where(ok, 1.0 / torch.where(ok, s, torch.ones_like(s)), torch.zeros_like(s))
    c = torch.clamp(torch.round((t - m).double() * inv.double()), 0, levels).to(torch.uint8)
    if qaxis == 0:
        c, s_, m_ = c.view(G, d).numpy(), s.view(G, d // gs).numpy(), m.view(G, d // gs).numpy()
        step = np.repeat(s_, gs, axis=1)
        zpt = np.repeat(m_, gs, axis=1)
    else:
        c, s_, m_ = c.view(d, G).t().contiguous().numpy(), s.view(d).numpy(), m.view(d).numpy()
        step = np.broadcast_to(s_, (G, d))
        zpt = np.broadcast_to(m_, (G, d))
    assert np.array_equal(codes, c)
    assert np.array_equal(scale.view(np.uint32), s_.view(np.uint32))
    assert np.array_equal(zero.view(np.uint32), m_.view(np.uint32))
    # representable in 16 bits
    assert np.all(scale.view(np.uint32) & 0xFFFF == 0) and np.all(zero.view(np.uint32) & 0xFFFF == 0)
    # the rounding moved scale and zero by at most half a bfloat16 ulp
    _, _, s32, m32 = oracle.quantize_tile(x, gs, qaxis, bits, oracle.F32)
    assert np.all(np.abs(scale - s32) <= np.abs(s32) * 2.0 ** -8) and np.all(np.abs(zero - m32) <= np.abs(m32) * 2.0 ** -8)
    # reconstruction: half a step, plus the shift of the zero point, plus the top code's stretch
    xh = oracle.dequant_tile(packed, scale, zero, G, d, gs, qaxis, bits)
    bound = 0.5 * step * (1 + 1e-5) + 2.0 ** -8 * (np.abs(zpt) + levels * step) + 1e-6
    assert np.all(np.abs(xh - x) <= bound)
    assert codes.max() <= levels


def test_quantize_invariants(oracle):
    r = _rng(11)
    G, d, gs = 33, 128, 64
    x = (r.standard_t(3, (G, d)) * 2).astype(np.float32)
    codes, packed, scale, zero = oracle.quantize_tile(x, gs)
    assert codes.min() >= 0 and codes.max() <= 15
    xg = x.reshape(G, d // gs, gs)
    cg = codes.reshape(G, d // gs, gs)
    # zero point is the group's minimum, exactly; 15*scale is max-min within an ulp or two
    assert np.array_equal(zero, xg.min(-1))
    rng_ = xg.max(-1) - xg.min(-1)
    assert np.all(np.abs(scale * np.float32(15) - rng_) <= 2 * np.spacing(rng_))
    # the minimum gets code 0 and the maximum code 15
    assert np.all(np.take_along_axis(cg, xg.argmin(-1)[..., None], -1) == 0)
    assert np.all(np.take_along_axis(cg, xg.argmax(-1)[..., None], -1) == 15)
    # monotone inside a quant-group
    order = np.argsort(xg, -1, kind="stable")
    assert np.all(np.diff(np.take_along_axis(cg.astype(np.int32), order, -1), axis=-1) >= 0)
    # reconstruction error at most half a step (plus float32 rounding of the affine map)
    xh = oracle.dequant_tile(packed, scale, zero, G, d, gs)
    s_e = np.repeat(scale, gs, axis=1)
    m_e = np.repeat(zero, gs, axis=1)
    bound = 0.5 * s_e * (1 + 1e-5) + 2.0 ** -22 * (np.abs(m_e) + 15 * s_e)
    assert np.all(np.abs(x - xh) <= bound)


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("qaxis,bits,meta", [(0, 4, 0), (0, 2, 0), (1, 4, 0), (1, 2, 0), (0, 4, 1), (1, 2, 1)])
def test_quantizer_properties_on_random_tiles(oracle, seed, qaxis, bits, meta):
    """Every variant, random shapes and value recipes: codes in range, monotone inside a
    quant-group, extremes at the ends (float32 metadata), reconstruction within the bound."""
    r = _rng(1000 * seed + 7 * qaxis + bits + 100 * meta)
    G = int(r.choice([1, 2, 7, 16, 50, 61]))
    d = int(r.choice([8, 32, 64, 128]))
    gs = int(r.choice([g for g in (8, 16, 32, 64, 128) if d % g == 0]))
    kind = int(r.integers(0, 3))
    x = r.standard_normal((G, d)) if kind == 0 else r.standard_t(3, (G, d)) * 3 if kind == 1 else \
        r.standard_normal((G, d)) * np.exp(r.uniform(-8, 8, (1, d)))
    x = (x + r.uniform(-4, 4)).astype(np.float32)
    levels = (1 << bits) - 1
    codes, packed, scale, zero = oracle.quantize_tile(x, gs, qaxis, bits, meta)
    assert codes.max() <= levels
    if qaxis == 0:
        xg, cg = x.reshape(G, d // gs, gs), codes.reshape(G, d // gs, gs)
        step, zpt = np.repeat(scale, gs, axis=1), np.repeat(zero, gs, axis=1)
    else:
        xg, cg = x.T, codes.T                                      # [d][G]: a group per channel
        step, zpt = np.broadcast_to(scale, (G, d)), np.broadcast_to(zero, (G, d))
    order = np.argsort(xg, -1, kind="stable")
    assert np.all(np.diff(np.take_along_axis(cg.astype(np.int32), order, -1), axis=-1) >= 0)
    live = (xg.max(-1) - xg.min(-1)) / levels >= np.finfo(np.float32).tiny
    if meta == 0:
        assert np.array_equal(zero.reshape(xg.shape[:-1]), xg.min(-1) + np.float32(0))
        assert np.all(np.take_along_axis(cg, xg.argmin(-1)[..., None], -1) == 0)
        assert np.all(np.take_along_axis(cg, xg.argmax(-1)[..., None], -1)[live] == levels)
    xh = oracle.dequant_tile(packed, scale, zero, G, d, gs, qaxis, bits)
    slack = 2.0 ** -8 if meta else 2.0 ** -22
    assert np.all(np.abs(x - xh) <= 0.5 * step * (1 + 1e-5) + slack * (np.abs(zpt) + levels * step) + 1e-30)


def test_grid_points_round_trip_exactly(oracle):
    # inputs m + c*s with dyadic s reproduce c and dequantize exactly
    G, d, gs = 4, 64, 32
    r = _rng(2)
    c = r.integers(0, 16, (G, d)).astype(np.uint8)
    c.reshape(G, d // gs, gs)[:, :, 0] = 0
    c.reshape(G, d // gs, gs)[:, :, 1] = 15
    m, s = np.float32(-2.0), np.float32(0.25)
    x = (m + c.astype(np.float32) * s).astype(np.float32)
    codes, packed, scale, zero = oracle.quantize_tile(x, gs)
    assert np.array_equal(codes, c)
    assert np.all(scale == s) and np.all(zero == m)
    assert np.array_equal(oracle.dequant_tile(packed, scale, zero, G, d, gs), x)


def test_hand_worked_example(oracle):
    """16 values -2, -1.75, ..., 1.75: min -2, max 1.75, s = 3.75/15 = 0.25, codes 0..15.
    Packing: even channel in the low nibble -> bytes 0x10 0x32 0x54 0x76 0x98 0xBA 0xDC 0xFE."""
    x = (np.arange(16, dtype=np.float32) * 0.25 - 2.0).reshape(1, 16)
    codes, packed, scale, zero = oracle.quantize_tile(x, 16)
    assert codes.tolist() == [list(range(16))]
    assert scale.item() == 0.25 and zero.item() == -2.0
    assert packed.tolist() == [[0x10, 0x32, 0x54, 0x76, 0x98, 0xBA, 0xDC, 0xFE]]
    # 2 bits: values 0, 1, 2, 3, 3, 2, 1, 0 -> s = 1, codes as given; 4 codes per byte,
    # first channel in the lowest two bits: 0b11100100 = 0xE4, 0b00011011 = 0x1B
    x2 = np.array([[0, 1, 2, 3, 3, 2, 1, 0]], np.float32)
    codes, packed, scale, zero = oracle.quantize_tile(x2, 8, oracle.QAXIS_HEAD_DIM, 2)
    assert codes.tolist() == [[0, 1, 2, 3, 3, 2, 1, 0]]
    assert packed.tolist() == [[0xE4, 0x1B]] and scale.item() == 1.0 and zero.item() == 0.0
    # rounding is half-to-even: with m=0, s=1 the inputs 0.5, 1.5, 2.5 give 0, 2, 2
    x3 = np.array([[0, 15, 0.5, 1.5, 2.5, 3.5, 14.5, 7.49]], np.float32)
    codes, _, scale, zero = oracle.quantize_tile(x3, 8)
    assert scale.item() == 1.0 and codes.tolist() == [[0, 15, 0, 2, 2, 4, 14, 7]]


def test_flat_and_tiny_range_groups(oracle):
    x = np.full((2, 32), 3.5, np.float32)
    x[1] = np.float32(1e-30)
    x[1, 3] = np.float32(1e-30) + np.float32(1e-38)      # range far below 15*FLT_MIN
    codes, packed, scale, zero = oracle.quantize_tile(x, 32)
    assert not codes.any() and not packed.any()
    assert np.all(scale == 0)
    assert zero[0, 0] == np.float32(3.5)
    xh = oracle.dequant_tile(packed, scale, zero, 2, 32, 32)
    assert np.all(xh[0] == np.float32(3.5)) and np.all(xh[1] == x[1].min())
    # negative zero never reaches the stored zero point
    xz = np.zeros((1, 32), np.float32)
    xz[0, ::2] = -0.0
    xz[0, 5] = 1.0
    _, _, _, zero = oracle.quantize_tile(xz, 32)
    assert zero.view(np.uint32).item() == 0


def test_rounding_reading_is_pinned_on_half_way_cases(oracle):
    """code = rne(d * inv) with d = float32(x - m), inv = float32(1 / s) and the product NOT
    rounded before the rounding to an integer.  The (max, x) pairs below were found by search
    next to half-way points; the expected code is worked out here in numpy, and it differs
    from what x / s would give (first list) and from what a float32-rounded product would
    give (second list)."""
    vs_division = [(20.71695327758789, 15.882997512817383), (38.04331588745117, 21.557878494262695),
                   (12.817342758178711, 3.845202922821045), (21.379276275634766, 14.965494155883789),
                   (18.413166046142578, 1.8413165807724), (38.81205368041992, 3.8812053203582764)]
    vs_f32_product = [(12.476195335388184, 12.060322761535645), (1.5885850191116333, 0.1588584929704666),
                      (20.680110931396484, 10.340054512023926), (20.71695327758789, 15.882997512817383)]
    n_div = n_prod = 0
    for mx, xv in vs_division + vs_f32_product:
        mx, xv = np.float32(mx), np.float32(xv)
        s = np.float32(mx / np.float32(15))
        inv = np.float32(np.float32(1) / s)
        want = int(np.rint(np.float64(xv) * np.float64(inv)))          # exact product, one rounding
        n_div += want != int(np.rint(np.float32(xv / s)))
        n_prod += want != int(np.rint(np.float32(xv * inv)))
        x = np.zeros((1, 8), np.float32)
        x[0, 1], x[0, 2] = mx, xv
        codes, _, scale, zero = oracle.quantize_tile(x, 8)
        assert scale.item() == s and zero.item() == 0
        assert codes[0, 2] == want and codes[0, 1] == 15 and codes[0, 0] == 0
    assert n_div >= len(vs_division) and n_prod >= len(vs_f32_product)


def test_subnormal_step_is_treated_as_flat(oracle):
    # range 1e-37 -> step 6.7e-39 is below FLT_MIN: stored scale 0, all codes 0
    x = np.zeros((1, 16), np.float32)
    x[0, 3] = np.float32(1e-37)
    codes, packed, scale, zero = oracle.quantize_tile(x, 16)
    assert scale.item() == 0 and zero.item() == 0 and not codes.any()
    # just above the threshold the group is quantized normally
    x[0, 3] = np.float32(15 * 1.2e-38)
    codes, _, scale, _ = oracle.quantize_tile(x, 16)
    assert scale.item() >= np.finfo(np.float32).tiny and codes[0, 3] == 15


def test_pack_unpack_is_lossless(oracle):
    r = _rng(9)
    for bits in (4, 2):
        G, d, gs = 6, 64, 32
        x = r.standard_normal((G, d)).astype(np.float32)
        codes, packed, scale, zero = oracle.quantize_tile(x, gs, oracle.QAXIS_HEAD_DIM, bits)
        per = 8 // bits
        un = np.stack([(packed >> (bits * u)) & ((1 << bits) - 1) for u in range(per)], -1)
        assert np.array_equal(un.reshape(G, d), codes)
        # code 0 dequantizes to the zero point exactly
        xh = oracle.dequant_tile(packed, scale, zero, G, d, gs, oracle.QAXIS_HEAD_DIM, bits)
        m_e = np.repeat(zero, gs, axis=1)
        assert np.array_equal(xh[codes == 0], m_e[codes == 0])
        # Eq. 11, code * s + m rounded once: exact in float64 for these magnitudes
        ref = codes.astype(np.float64) * np.repeat(scale, gs, axis=1).astype(np.float64) + m_e
        assert np.array_equal(xh, ref.astype(np.float32))


def test_token_axis_is_the_same_quantizer_transposed(oracle):
    """Paper Eq. 9 (per channel over the G tokens) must equal the head_dim-axis quantizer
    applied to the transposed tile with one quant-group per row."""
    r = _rng(21)
    G, d = 50, 128
    x = (r.standard_normal((G, d)) * 3).astype(np.float32)
    ct, pt, st, zt = oracle.quantize_tile(x, 64, oracle.QAXIS_TOKENS)
    ch, _, sh, zh = oracle.quantize_tile(np.ascontiguousarray(x.T), G, oracle.QAXIS_HEAD_DIM)
    assert st.shape == (d,) and np.array_equal(st, sh[:, 0]) and np.array_equal(zt, zh[:, 0])
    assert np.array_equal(ct, ch.T)
    assert np.array_equal(zt, x.min(0))
    # packing still runs along the channel axis
    assert np.array_equal(pt, ct[:, 0::2] | (ct[:, 1::2] << 4))
    xh = oracle.dequant_tile(pt, st, zt, G, d, 64, oracle.QAXIS_TOKENS)
    assert np.array_equal(xh, (ct.astype(np.float64) * st[None, :].astype(np.float64) + zt[None, :]).astype(np.float32))
    assert np.all(np.abs(xh - x) <= 0.5 * st[None, :] * (1 + 1e-5) + 2.0 ** -22 * (np.abs(zt) + 15 * st))


def test_summary_key_is_the_mean_over_tokens(oracle):
    r = _rng(4)
    x = (r.standard_normal((196, 128)) * 5).astype(np.float32)
    key = oracle.summary_key(x)
    # double-precision mean, rounded once to float32 (summation order may differ in the
    # last double bit, which can move the float32 result by at most one ulp, very rarely)
    ref = x.astype(np.float64).mean(0)
    assert np.all(np.abs(key.astype(np.float64) - ref) <= 0.5000001 * np.spacing(np.abs(ref).astype(np.float32)))
    const = np.full((7, 16), -2.75, np.float32)
    assert np.all(oracle.summary_key(const) == np.float32(-2.75))
    # a single large token must not be lost (mean, not max / last)
    one = np.zeros((4, 8), np.float32)
    one[2, 3] = 8.0
    assert oracle.summary_key(one)[3] == 2.0 and oracle.summary_key(one).sum() == 2.0


# --------------------------------------------------------------------------- store / append
def _small_cfg(oracle, **kw):
    base = dict(n_layers=2, n_kv_heads=2, n_q_heads=6, head_dim=32, group_tokens=5, qgroup=16,
                capacity_groups=9, in_dtype=oracle.F32, out_dtype=oracle.F32,
                sim=oracle.SIM_COSINE)
    base.update(kw)
    return oracle.make_config(**base)


def test_append_places_tiles_and_keys(oracle):
    cfg = _small_cfg(oracle)
    st = oracle.new_store(cfg)
    r = _rng(8)
    F = 3
    k = r.standard_normal((F, 2, 2, 5, 32)).astype(np.float32)
    v = r.standard_normal((F, 2, 2, 5, 32)).astype(np.float32)
    assert oracle.quantize_append(st, k[:1], v[:1]) == 0
    assert oracle.quantize_append(st, k[1:], v[1:]) == 1
    assert st.n_groups == 3
    for f in range(F):
        for l in range(2):
            for h in range(2):
                for kv, src in ((0, k), (1, v)):
                    packed, scale, zero = oracle.tile_view(st, l, kv, f, h)
                    _, p2, s2, z2 = oracle.quantize_tile(src[f, l, h], 16)
                    assert np.array_equal(packed, p2)
                    assert np.array_equal(scale, s2.ravel()) and np.array_equal(zero, z2.ravel())
                assert np.array_equal(st.keys[l, f, h], oracle.summary_key(k[f, l, h]))
    # slots beyond n_groups stay untouched
    assert not st.keys[:, 3:].any()
    # capacity is enforced, history is never evicted
    big = r.standard_normal((7, 2, 2, 5, 32)).astype(np.float32)
    with pytest.raises(ValueError):
        oracle.quantize_append(st, big, big)
    assert st.n_groups == 3


def test_append_strides_layers_and_separate_summary_source(oracle):
    cfg = _small_cfg(oracle, in_dtype=oracle.BF16)
    st = oracle.new_store(cfg)
    g = torch.Generator().manual_seed(5)
    # token-major source buffer [F][G][L][H][d] (as a model's K projection would hand over)
    buf_k = torch.randn(2, 5, 2, 2, 32, generator=g).to(torch.bfloat16)
    buf_v = torch.randn(2, 5, 2, 2, 32, generator=g).to(torch.bfloat16)
    pre = torch.randn(2, 5, 2, 2, 32, generator=g).to(torch.bfloat16)
    bits = lambda t: t.view(torch.int16).numpy().view(np.uint16)
    strides = (5 * 2 * 2 * 32, 2 * 32, 32, 2 * 2 * 32)      # frame, layer, head, token
    # only layer 1 is appended, from a pointer already offset to that layer
    off = 1 * strides[1]
    oracle.quantize_append(st, bits(buf_k).ravel()[off:], bits(buf_v).ravel()[off:],
                           bits(pre).ravel()[off:], layer0=1, strides=strides, n_frames=2,
                           n_layers=1)
    for f in range(2):
        for h in range(2):
            x = buf_k[f, :, 1, h, :].float().numpy()
            packed, scale, zero = oracle.tile_view(st, 1, 0, f, h)
            _, p2, s2, z2 = oracle.quantize_tile(x, 16)
            assert np.array_equal(packed, p2) and np.array_equal(scale, s2.ravel())
            # the summary comes from the separate (pre-rotary) keys, not from K
            assert np.array_equal(st.keys[1, f, h], oracle.summary_key(pre[f, :, 1, h, :].float().numpy()))
    assert not st.keys[0].any() and not oracle.tile_view(st, 0, 0, 0, 0)[0].any()


# --------------------------------------------------------------------------- scoring
def _fold_query(q, H_k):
    """[L][H_q][T_q][d] -> mean over each block of r consecutive query heads, then tokens."""
    L, Hq, Tq, d = q.shape
    qt = q.double().view(L, H_k, Hq // H_k, Tq, d).mean(2)        # [L][H_k][T_q][d]
    return qt, qt.mean(2)                                         # q~, q-bar [L][H_k][d]


@pytest.mark.parametrize("sim", ["cosine", "dot"])
def test_score_equals_torch_fp64(oracle, sim):
    cfg = _small_cfg(oracle, sim=oracle.SIM_COSINE if sim == "cosine" else oracle.SIM_DOT)
    st = oracle.new_store(cfg)
    g = torch.Generator().manual_seed(12)
    k = torch.randn(9, 2, 2, 5, 32, generator=g)
    oracle.quantize_append(st, k.numpy(), k.numpy().copy())
    q = torch.randn(2, 6, 3, 32, generator=g)
    scores, tok = oracle.score_groups(st, q.numpy(), oracle.F32, want_token_scores=True)
    keys = torch.from_numpy(st.keys).double()                     # [L][T][H_k][d]
    qt, qb = _fold_query(q, 2)
    for l in range(2):
        kk = keys[l].reshape(9, -1)
        if sim == "cosine":
            ref = torch.nn.functional.cosine_similarity(qb[l].reshape(1, -1), kk, dim=1)
        else:
            ref = kk @ qb[l].reshape(-1)
        assert np.allclose(scores[l], ref.numpy(), rtol=1e-6, atol=1e-7)
        assert np.array_equal(scores[l], ref.float().numpy()) or \
            np.max(np.abs(scores[l] - ref.float().numpy())) <= np.spacing(np.float32(np.abs(ref).max()))
        # per-token scores: GQA-folded token j against key t, flattened over heads
        ref_tok = torch.einsum("hjc,thc->jt", qt[l], keys[l])
        assert np.allclose(tok[l], ref_tok.numpy(), rtol=1e-6, atol=1e-6)
        # their mean over tokens is the numerator of the score (dot is linear)
        num = tok[l].astype(np.float64).mean(0)
        if sim == "dot":
            assert np.allclose(num, scores[l], rtol=1e-5, atol=1e-6)
    if sim == "cosine":
        assert np.all(np.abs(scores) <= 1 + 1e-6)


def test_score_gqa_blocks_are_consecutive_heads(oracle):
    # only query head 4 (block 1 of r=3) is non-zero -> only KV head 1 contributes
    cfg = _small_cfg(oracle, sim=oracle.SIM_DOT)
    st = oracle.new_store(cfg)
    k = np.zeros((1, 2, 2, 5, 32), np.float32)
    k[0, :, 0] = 1.0
    k[0, :, 1] = 2.0
    oracle.quantize_append(st, k, k)
    q = np.zeros((2, 6, 1, 32), np.float32)
    q[:, 4] = 3.0
    s = oracle.score_groups(st, q, oracle.F32)
    # q-bar[h=1] = 3/3 = 1 on every channel; key[h=1] = 2  ->  32 * 1 * 2
    assert np.all(s == 64.0)
    q[:] = 0
    q[:, 1] = 3.0                                                  # block 0 -> KV head 0
    assert np.all(oracle.score_groups(st, q, oracle.F32) == 32.0)


def test_planted_query_retrieves_its_group(oracle):
    cfg = _small_cfg(oracle, n_q_heads=2)
    st = oracle.new_store(cfg)
    r = _rng(31)
    k = r.standard_normal((9, 2, 2, 5, 32)).astype(np.float32)
    oracle.quantize_append(st, k, k)
    j = 6
    # r = 1: the GQA mean is the identity; one query token equal to the stored key
    q = st.keys[:, j].reshape(2, 2, 1, 32).copy()
    s = oracle.score_groups(st, q, oracle.F32)
    assert np.allclose(s[:, j], 1.0, atol=1e-6)
    assert np.all(s.argmax(1) == j)
    idx, k_eff = oracle.topk(s, 1)
    assert k_eff == 1 and np.all(idx[:, 0] == j)
    # zero query: norms are clamped, score is 0, nothing is NaN
    s0 = oracle.score_groups(st, np.zeros_like(q), oracle.F32)
    assert np.all(s0 == 0)


# --------------------------------------------------------------------------- top-k
def _brute_topk(row, k):
    order = np.argsort(-(row + np.float32(0.0)), kind="stable")    # full sort, lowest index first on ties
    return order[:min(k, row.size)]


def test_topk_equals_full_sort(oracle):
    r = _rng(77)
    for T, k in [(1, 1), (5, 2), (32, 4), (33, 33), (64, 100), (200, 17)]:
        s = r.standard_normal((3, T)).astype(np.float32)
        s[1] = np.round(s[1] * 2) / 2                              # many exact ties
        s[2, ::3] = 0.0
        s[2, 1::3] = -0.0                                          # -0 ties with +0
        idx, k_eff = oracle.topk(s, k)
        assert k_eff == min(k, T)
        idd, _ = oracle.topk(s, k, oracle.ORDER_SCORE_DESC)
        for row in range(3):
            want = _brute_topk(s[row], k)
            assert idd[row, :k_eff].tolist() == want.tolist()
            assert idx[row, :k_eff].tolist() == sorted(want.tolist())
            assert np.all(idx[row, k_eff:] == -1)                  # untouched tail


def test_topk_degenerate_cases(oracle):
    s = np.full((2, 10), 0.5, np.float32)
    idx, k_eff = oracle.topk(s, 4)
    assert idx.tolist() == [[0, 1, 2, 3]] * 2                      # all equal -> lowest indices
    idx, k_eff = oracle.topk(s, 10)
    assert idx.tolist() == [list(range(10))] * 2
    # a row stride larger than the number of groups: the padding is never selected
    pad = np.full((2, 16), 9.0, np.float32)
    pad[:, :10] = np.arange(10, dtype=np.float32)
    idx, k_eff = oracle.topk(pad, 3, n_groups=10)
    assert idx.tolist() == [[7, 8, 9]] * 2
    # increasing scores: the LAST k groups win, output ascending
    idx, _ = oracle.topk(np.arange(12, dtype=np.float32).reshape(1, 12), 5)
    assert idx.tolist() == [[7, 8, 9, 10, 11]]
    with pytest.raises(ValueError):
        oracle.topk(s, 0)


# --------------------------------------------------------------------------- gather
@pytest.mark.parametrize("out_dtype", ["f32", "bf16", "f16"])
def test_gather_rows_are_the_named_groups(oracle, out_dtype):
    od = {"f32": oracle.F32, "bf16": oracle.BF16, "f16": oracle.F16}[out_dtype]
    cfg = _small_cfg(oracle, out_dtype=od)
    st = oracle.new_store(cfg)
    r = _rng(55)
    k = r.standard_normal((9, 2, 2, 5, 32)).astype(np.float32)
    v = r.standard_normal((9, 2, 2, 5, 32)).astype(np.float32)
    oracle.quantize_append(st, k, v)
    idx = np.array([[1, 4, 8, -1], [0, 2, 7, -1]], np.int32)       # k = 4, k_eff = 3
    fill = 0x7FC0 if od != oracle.F32 else np.float32(123.0)
    ko, vo = oracle.dequant_gather(st, idx, 3, fill=fill)
    G = 5
    assert ko.shape == (2, 2, 4 * G, 32)
    for l in range(2):
        for rnk in range(3):
            for h in range(2):
                for kv, out in ((0, ko), (1, vo)):
                    packed, scale, zero = oracle.tile_view(st, l, kv, idx[l, rnk], h)
                    x = oracle.dequant_tile(packed, scale, zero, G, 32, 16)
                    want = oracle.from_f32(x, od)
                    assert np.array_equal(out[l, h, rnk * G:(rnk + 1) * G], want)
    # active buffer bound: rows beyond k_eff*G are not written
    assert np.all(ko[:, :, 3 * G:] == fill) and np.all(vo[:, :, 3 * G:] == fill)
    # torch's own rounding agrees with the narrowing used for the output
    if od == oracle.BF16:
        packed, scale, zero = oracle.tile_view(st, 0, 0, 1, 0)
        x = oracle.dequant_tile(packed, scale, zero, G, 32, 16)
        ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        assert np.array_equal(ko[0, 0, :G], ref)
    # reconstruction stays within half a quantization step of the original
    if od == oracle.F32:
        err = np.abs(ko[0, 0, :G] - k[1, 0, 0])
        _, scale, _ = oracle.tile_view(st, 0, 0, 1, 0)
        assert err.max() <= 0.5 * scale.max() * (1 + 1e-4) + 1e-6


@pytest.mark.parametrize("qaxis", [0, 1])
def test_two_bit_store_and_gather(oracle, qaxis):
    """The 2-bit variant through append and gather: four codes per byte, three steps between
    min and max, reconstruction within half a step, Table 4's ratio for the code payload."""
    cfg = _small_cfg(oracle, bits=2, qaxis=qaxis)
    st = oracle.new_store(cfg)
    r = _rng(77)
    k = r.standard_normal((4, 2, 2, 5, 32)).astype(np.float32)
    oracle.quantize_append(st, k, 2 * k)
    assert st.codes.size == 2 * 2 * 9 * 2 * 5 * 32 // 4          # L * (K,V) * T_cap * H * G * d / 4
    idx = np.array([[3, 0], [1, 2]], np.int32)
    ko, vo = oracle.dequant_gather(st, idx, 2)
    for l in range(2):
        for rnk in range(2):
            for h in range(2):
                x = k[idx[l, rnk], l, h]
                codes, packed, scale, zero = oracle.quantize_tile(x, 16, qaxis, 2)
                assert codes.max() <= 3 and np.array_equal(oracle.tile_view(st, l, 0, idx[l, rnk], h)[0].ravel(),
                                                           packed.ravel())
                step = np.repeat(scale, 16, axis=1) if qaxis == 0 else np.broadcast_to(scale, x.shape)
                got = ko[l, h, rnk * 5:(rnk + 1) * 5]
                assert np.all(np.abs(got - x) <= 0.5 * step * (1 + 1e-5) + 1e-6)
                assert np.allclose(vo[l, h, rnk * 5:(rnk + 1) * 5], 2 * got, rtol=1e-6, atol=1e-6)
    assert oracle.lib().tomref_compression_ratio(196, 50, 2) == pytest.approx(196 * 16 / (50 * 2))


def test_gather_rejects_bad_index(oracle):
    cfg = _small_cfg(oracle)
    st = oracle.new_store(cfg)
    k = np.ones((2, 2, 2, 5, 32), np.float32)
    oracle.quantize_append(st, k, k)
    with pytest.raises(ValueError):
        oracle.dequant_gather(st, np.array([[0, 5], [0, 1]], np.int32), 2)   # 5 >= n_groups


def test_assemble_places_system_prefix_then_groups(oracle):
    """Dual-structure memory: the active buffer of every (layer, head) is the 16-bit system
    rows, bit for bit, followed by exactly what the plain gather produces."""
    cfg = _small_cfg(oracle, out_dtype=oracle.BF16)
    st = oracle.new_store(cfg)
    r = _rng(56)
    k = r.standard_normal((6, 2, 2, 5, 32)).astype(np.float32)
    oracle.quantize_append(st, k, -k)
    idx = np.array([[0, 3, 5, -1], [1, 2, 4, -1]], np.int32)
    G, P = 5, 3
    plain_k, plain_v = oracle.dequant_gather(st, idx, 3, fill=0x7FC0)
    sys_k = r.integers(0, 2 ** 16, (2, 2, P, 32)).astype(np.uint16)
    sys_v = r.integers(0, 2 ** 16, (2, 2, P, 32)).astype(np.uint16)
    ko, vo = oracle.assemble_active(st, idx, 3, P, sys_k, sys_v, fill=0x7FC0)
    assert ko.shape == (2, 2, P + 4 * G, 32)
    assert np.array_equal(ko[:, :, :P], sys_k) and np.array_equal(vo[:, :, :P], sys_v)
    assert np.array_equal(ko[:, :, P:], plain_k) and np.array_equal(vo[:, :, P:], plain_v)
    # no system tensors: the prefix rows are left as they were
    ko, vo = oracle.assemble_active(st, idx, 3, P, None, None, fill=0x1234)
    assert np.all(ko[:, :, :P] == 0x1234) and np.array_equal(ko[:, :, P:P + 3 * G], plain_k[:, :, :3 * G])
    # prefix of zero rows is the plain gather
    ko, vo = oracle.assemble_active(st, idx, 3, 0, None, None, fill=0x7FC0)
    assert np.array_equal(ko, plain_k) and np.array_equal(vo, plain_v)


# --------------------------------------------------------------------------- whole path, C1
def test_tiny_stream_end_to_end_brute_force(oracle):
    """The smallest benchmark configuration, every step re-derived with numpy/torch."""
    import synth_kv
    w = synth_kv.WORKLOADS["C1"]
    cfg = oracle.make_config(w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim, w.group_tokens,
                             w.qgroup, w.n_frames, in_dtype=oracle.F32, out_dtype=oracle.F32,
                             sim=oracle.SIM_DOT)
    st = oracle.new_store(cfg)
    k, v = synth_kv.kv_frames(w, 0, w.n_frames)
    oracle.quantize_append(st, k.numpy(), v.numpy())
    q = synth_kv.query(w)
    s = oracle.score_groups(st, q.numpy(), oracle.F32)
    mean_key = k.double().mean(3)                                  # [T][L][H][d]
    ref = torch.einsum("tlhc,lhc->lt", mean_key, q.double()[:, :, 0])
    assert np.allclose(s, ref.numpy(), rtol=1e-6, atol=1e-6)
    idx, k_eff = oracle.topk(s, w.top_k)
    assert k_eff == 4
    assert idx[0].tolist() == sorted(np.argsort(-s[0], kind="stable")[:4].tolist())
    ko, vo = oracle.dequant_gather(st, idx, k_eff)
    assert ko.shape == (1, 2, 4 * 16, 64)                          # the active buffer bound k*G
    for rnk, t in enumerate(idx[0]):
        for h in range(2):
            for src, out in ((k, ko), (v, vo)):
                x = src[t, 0, h].numpy()
                c, s_, m_ = _torch_quant_headdim(x, 32)
                xh = (c.astype(np.float64) * np.repeat(s_, 32, 1) + np.repeat(m_, 32, 1)).astype(np.float32)
                assert np.array_equal(out[0, h, rnk * 16:(rnk + 1) * 16], xh)
                assert np.all(np.abs(xh - x) <= 0.5 * np.repeat(s_, 32, 1) * (1 + 1e-5) + 1e-6)

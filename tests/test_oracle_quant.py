"""Pins for the oracle's decision arithmetic: scaling, FindInterval, V_init, RTN, hardening,
packing (paper Sec. 3.1, Table 2 steps 2-5 and 25-26, Eq. 4, Eq. 7)."""
import numpy as np
import pytest

from oracle import faar_oracle as fo
from workloads import synth

NODES = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]      # retyped from the paper, not imported


def _cases():
    c1 = synth.config1(0)
    yield "config1_fp32", c1.W, False
    yield "student_t_bf16", synth.student_t_weight(96, 320, 3), True
    yield "adversarial_bf16", synth.adversarial_weight(1, True), True
    yield "adversarial_fp32", synth.adversarial_weight(2, False), False


CASES = list(_cases())
IDS = [c[0] for c in CASES]


def _unpacked(q):
    return fo.unpack_nibbles(q["codes"])


@pytest.mark.parametrize("name,W,isbf", CASES, ids=IDS)
def test_interval_brackets_normalised_magnitude(name, W, isbf):
    sg = fo.tensor_scale(W)
    sb = fo.block_scale_bytes(W, sg)
    wt = fo.normalised_magnitude(W, sb, sg).astype(np.float64)
    k = fo.find_interval(wt.astype(np.float32))
    lo = np.array(NODES)[k]
    hi = np.array(NODES)[k + 1]
    assert k.min() >= 0 and k.max() <= 6
    sat = wt > 6.0
    assert np.all(lo <= wt)
    assert np.all((wt < hi) | sat | (wt == 6.0))        # on-node values open the interval above
    assert np.all(k[sat] == 6)
    assert wt.max() < 6.0 * 1.07                        # scale rounding is at most half an E4M3 step (1/16)


@pytest.mark.parametrize("name,W,isbf", CASES, ids=IDS)
def test_hardening_v_init_reproduces_rtn_bit_for_bit(name, W, isbf):
    q = fo.quant_rtn(W, isbf)
    iv = fo.init_v(W, q["s_global"], q["scales"])
    hp = fo.harden_pack(W, isbf, q["s_global"], q["scales"], iv["V"])
    assert np.array_equal(hp["codes"], q["codes"])
    assert np.array_equal(hp["W_final"].view(np.uint32), q["W_dq"].view(np.uint32))
    assert hp["flip_count"] == 0
    assert iv["V"].min() >= 0.0 and iv["V"].max() <= 1.0


@pytest.mark.parametrize("name,W,isbf", CASES, ids=IDS)
def test_rtn_is_the_nearest_node_by_brute_force(name, W, isbf):
    """Independent of FindInterval: the chosen magnitude minimises |w~ - node| over all 8 nodes,
    exact ties going to the larger node."""
    q = fo.quant_rtn(W, isbf)
    wt = fo.normalised_magnitude(W, q["scales"], q["s_global"]).astype(np.float64)
    d = np.abs(wt[..., None] - np.array(NODES)[None, None, :])
    best = d.shape[2] - 1 - np.argmin(d[..., ::-1], axis=2)     # last index of the minimum
    mag = _unpacked(q) & 7
    nz = W != 0
    assert np.array_equal(mag[nz], best[nz])
    assert np.all(mag[~nz] == 0)
    assert np.array_equal(_unpacked(q) >> 3, np.signbit(W).astype(np.uint8))


@pytest.mark.parametrize("name,W,isbf", CASES, ids=IDS)
def test_interpolation_identity(name, W, isbf):
    """Eq. 2 with h replaced by the identity, evaluated at V_init, gives back w (unsaturated)."""
    sg = fo.tensor_scale(W)
    sb = fo.block_scale_bytes(W, sg)
    iv = fo.init_v(W, sg, sb)
    sign, lo, hi, s = fo.interval_terms(W, sg, sb)
    wt = fo.normalised_magnitude(W, sb, sg)
    rec = sign * (lo + iv["V"].astype(np.float64) * (hi - lo)) * s
    ok = (wt <= 6.0) & (s > 0)
    err = np.abs(rec - W.astype(np.float64))[ok]
    assert np.all(err <= 2.0 ** -22 * np.abs(W[ok]) + 1e-44)
    # saturated elements reconstruct to exactly 6 s
    sat = wt > 6.0
    assert np.allclose(rec[sat], (sign * 6.0 * s)[sat], rtol=0, atol=0)


@pytest.mark.parametrize("name,W,isbf", CASES, ids=IDS)
def test_final_weights_lie_on_the_scaled_grid(name, W, isbf):
    rng = np.random.default_rng(0)
    sg = fo.tensor_scale(W)
    sb = fo.block_scale_bytes(W, sg)
    V = synth.rounding_variables(W.shape[0], W.shape[1], 4)
    hp = fo.harden_pack(W, False, sg, sb, V)
    codes = fo.unpack_nibbles(hp["codes"])
    s_g = np.repeat(fo.e4m3_decode(sb), 16, axis=1)
    expect = fo.e2m1_decode(codes) * s_g * float(sg)             # float64 product of the three factors
    assert np.allclose(hp["W_final"], expect, rtol=2.0 ** -23, atol=1e-45)
    # the hardened value is one of the two neighbours picked by v >= 0.5
    wt = fo.normalised_magnitude(W, sb, sg)
    k = fo.find_interval(wt)
    want_mag = np.where(W == 0, 0, k + (V >= 0.5))
    assert np.array_equal(codes & 7, want_mag)
    # decision bitmask layout
    bits = np.unpackbits(hp["decisions"], bitorder="little").reshape(W.shape)
    assert np.array_equal(bits, (V >= 0.5).astype(np.uint8))


def test_lower_and_upper_rounding_bracket_the_weight():
    W = synth.student_t_weight(64, 256, 9)
    sg = fo.tensor_scale(W)
    sb = fo.block_scale_bytes(W, sg)
    lo = fo.harden_pack(W, False, sg, sb, np.zeros_like(W))["W_final"]
    hi = fo.harden_pack(W, False, sg, sb, np.ones_like(W))["W_final"]
    wt = fo.normalised_magnitude(W, sb, sg)
    ok = wt <= 6.0
    tol = 2.0 ** -22 * np.abs(W)
    assert np.all((np.abs(lo) <= np.abs(W) + tol)[ok])
    assert np.all((np.abs(hi) >= np.abs(W) - tol)[ok])
    assert np.all(np.sign(lo) * np.sign(W) >= 0) and np.all(np.sign(hi) * np.sign(W) >= 0)


@pytest.mark.parametrize("name,W,isbf", CASES, ids=IDS)
def test_scale_structure(name, W, isbf):
    """The block holding the tensor amax gets the largest E4M3 scale (448) and its amax element
    the largest node; zero blocks get scale 0 and code 0; scale bytes never exceed 0x7E."""
    q = fo.quant_rtn(W, isbf)
    O, K = W.shape
    amax = np.abs(W).max()
    r, c = np.unravel_index(np.argmax(np.abs(W)), W.shape)
    assert q["scales"][r, c // 16] == 0x7E
    assert (_unpacked(q)[r, c] & 7) == 7
    assert q["scales"].max() <= 0x7E
    assert np.float32(q["s_global"]) == np.float32(amax) / np.float32(6 * 448)
    blocks = np.abs(W).reshape(O, K // 16, 16).max(axis=2)
    zero = blocks == 0
    assert np.all(q["scales"][zero] == 0)
    # a non-zero block's decoded scale is within half an E4M3 step of amax_b / 6 (or underflowed/saturated)
    ideal = blocks.astype(np.float64) / 6.0 / float(q["s_global"])
    got = fo.e4m3_decode(q["scales"])
    mid = (ideal >= 2.0 ** -6) & (ideal <= 448)
    assert np.all(np.abs(got - ideal)[mid] <= ideal[mid] / 16.0 * (1 + 1e-6))
    sub = ideal < 2.0 ** -6
    assert np.all(np.abs(got - ideal)[sub] <= 2.0 ** -10 * (1 + 1e-6))


def test_all_zero_tensor():
    W = np.zeros((4, 32), dtype=np.float32)
    W[1, 3] = -0.0
    q = fo.quant_rtn(W, True)
    assert q["s_global"] == 1.0 and not q["scales"].any()
    codes = _unpacked(q)
    assert codes[1, 3] == 8 and np.count_nonzero(codes) == 1
    assert not fo.init_v(W, q["s_global"], q["scales"])["V"].any()


def test_adversarial_blocks_by_hand():
    W = synth.adversarial_weight(1, True)
    q = fo.quant_rtn(W, True)
    codes = _unpacked(q)
    assert q["s_global"] == np.float32(2.0 ** -7)
    # row 2: amax element -> code 7, its tiny neighbours -> 0 (1e-3 / (21/6) << 0.25)
    assert codes[2, 0] == 7 and not codes[2, 1:16].any() and q["scales"][2, 0] == 0x7E
    # row 3: |w| = 1e-30: ideal scale far below 2^-10 -> byte 0 -> w~ defined as 0 -> code 0
    assert q["scales"][3, 0] == 0 and not codes[3, 0:32].any()
    # row 1: raw nodes/midpoints with block amax 6 -> scale 128 * 2^-7 = 1 (byte 0x70), w~ = |w|
    assert q["scales"][1, 0] == 0x70 and q["scales"][1, 1] == 0x70
    assert list(codes[1, :16]) == [7, 7, 6, 6, 5, 5, 4, 4, 3, 3, 2, 2, 1, 1, 0, 8 | 1]
    assert list(codes[1, 16:32]) == [15, 15, 14, 14, 13, 13, 12, 12, 11, 11, 10, 10, 9, 9, 8, 1]
    # row 4: block amax = 6 * s_global -> scale byte of 1.0 (0x38); weights are node multiples and
    # exact midpoints of s_global: midpoints go UP (v_init = 0.5 -> upper)
    assert q["scales"][4, 0] == 0x38
    wt = fo.normalised_magnitude(W, q["scales"], q["s_global"])[4, :16]
    want = {6: 7, 5: 7, 4: 6, 3.5: 6, 3: 5, 2.5: 5, 2: 4, 1.75: 4, 1.5: 3, 1.25: 3, 1: 2, 0.75: 2, 0.5: 1, 0.25: 1, 0: 0}
    for j in range(16):
        assert codes[4, j] == want[float(wt[j])], (j, wt[j])
    # row 5: negative zeros keep their sign bit, magnitude 0
    assert np.all(codes[5, :16] == 8)
    # row 7: constant block, one negative element: all code 7 / 15
    assert np.all((codes[7, :16] & 7) == 7) and codes[7, 3] == 15


def test_packing_order():
    codes = np.arange(32, dtype=np.uint8).reshape(2, 16) % 16
    p = fo.pack_nibbles(codes)
    assert p.shape == (2, 8)
    assert p[0, 0] == (codes[0, 0] | (codes[0, 1] << 4))
    assert np.array_equal(fo.unpack_nibbles(p), codes)


def test_flip_count_counts_changed_nibbles():
    W = synth.student_t_weight(32, 64, 2)
    q = fo.quant_rtn(W, True)
    V = fo.init_v(W, q["s_global"], q["scales"])["V"].copy()
    V[0, :10] = np.where(V[0, :10] >= 0.5, 0.0, 1.0)           # flip ten decisions
    hp = fo.harden_pack(W, True, q["s_global"], q["scales"], V)
    changed = np.count_nonzero(fo.unpack_nibbles(hp["codes"]) != fo.unpack_nibbles(q["codes"]))
    assert hp["flip_count"] == changed
    assert 1 <= changed <= 10


def test_philox_known_answers_and_stochastic_rounding_statistics():
    """The generator against the known-answer vectors published with it (Random123 kat_vectors, philox4x32 10
    rounds), and the candidate sampler against what its definition implies."""
    kat = [((0, 0, 0, 0), (0, 0), (0x6627e8d5, 0xe169c58d, 0xbc57ac4c, 0x9b00dbd8)),
           ((0xffffffff,) * 4, (0xffffffff,) * 2, (0x408f276d, 0x41c83b0e, 0xa20bc7c6, 0x6d5451fd)),
           ((0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344), (0xa4093822, 0x299f31d0),
            (0xd16cfe09, 0x94fdcceb, 0x5001e420, 0x24126ea1))]
    for ctr, key, want in kat:
        got = fo.philox4x32_10(np.array(ctr, dtype=np.uint32), np.array(key, dtype=np.uint32))
        assert tuple(int(x) for x in got) == want
    v = np.linspace(0.0, 1.0, 11, dtype=np.float32)[None, :].repeat(20000, axis=0)
    s = fo.stochastic_v(v, seed=5, sample=3)
    assert set(np.unique(s)) <= {0.0, 1.0}
    assert not s[:, 0].any() and s[:, -1].all()                       # v = 0 never goes up, v = 1 always
    assert np.abs(s.mean(axis=0) - v[0]).max() < 0.015                # unbiased: P(up) = v  (sigma <= 0.0036)
    assert not np.array_equal(s, fo.stochastic_v(v, seed=5, sample=4))
    assert np.array_equal(s, fo.stochastic_v(v, seed=5, sample=3))

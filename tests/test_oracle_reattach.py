"""Pins for the oracle's re-attachment (paper Alg. 1 steps 8-10; Sec. 7.2 "k_r rotation";
Sec. 7.3 precision; App. C gather-rotate-scatter).

The oracle rotates pair by pair with libm sin/cos.  It is pinned here to the
group law R(a)R(b) = R(a+b) (Alg. 1 step 9), to the complex-exponential form
of the same rotation, to the quarter-turn special case, to norm preservation,
to the bf16 precision the paper reports for this rotation (4.7e-3 rel-L2,
non-accumulating), to exhaustive checks of the fp64 -> bf16 rounding, and to
the byte-for-byte reuse of c_KV.
"""
import os

import numpy as np
import pytest
import torch

from oracle import irm_oracle as orc
from paper_2605_05696_amd import workloads as wl

INV = wl.inv_freq_plain()


def bf16_bits(x):
    """fp32/fp64 numpy -> bf16 bit patterns via torch's conversion (inputs only)."""
    return torch.from_numpy(np.asarray(x, np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


# ----------------------------------------------------------------- rounding --

def test_bf16_widening_is_exact_for_all_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    want = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64).numpy()
    got = orc.bf16_to_f64(bits)
    both_nan = np.isnan(want) & np.isnan(got)
    assert np.all((got == want) | both_nan)
    assert np.array_equal(np.signbit(got[~both_nan]), np.signbit(want[~both_nan]))


def test_rounding_every_representable_value_is_a_fixed_point():
    bits = np.arange(65536, dtype=np.uint16)
    vals = orc.bf16_to_f64(bits)
    finite = np.isfinite(vals)
    back = orc.f64_to_bf16(vals[finite])
    assert np.array_equal(back, bits[finite])            # includes +-0 and subnormals


def test_rounding_between_all_adjacent_pairs_is_nearest_ties_to_even():
    # positive finite bf16 values are ordered like their bit patterns
    bits = np.arange(0x0000, 0x7F80, dtype=np.uint16)     # 0 .. largest finite
    v = orc.bf16_to_f64(bits)
    lo, hi, lo_bits, hi_bits = v[:-1], v[1:], bits[:-1], bits[1:]
    mid = (lo + hi) / 2.0                                 # exact in fp64
    even = np.where(lo_bits % 2 == 0, lo_bits, hi_bits)
    assert np.array_equal(orc.f64_to_bf16(mid), even)
    assert np.array_equal(orc.f64_to_bf16(np.nextafter(mid, -np.inf)), lo_bits)
    assert np.array_equal(orc.f64_to_bf16(np.nextafter(mid, np.inf)), hi_bits)
    # mirrored for negative values
    assert np.array_equal(orc.f64_to_bf16(-mid), even | np.uint16(0x8000))
    assert np.array_equal(orc.f64_to_bf16(np.nextafter(-mid, np.inf)), lo_bits | np.uint16(0x8000))


def test_rounding_edges():
    big = float(orc.bf16_to_f64(np.array([0x7F7F], np.uint16))[0])     # largest finite
    half_ulp = 2.0 ** (127 - 8)
    f = lambda x: int(orc.f64_to_bf16(np.array([x]))[0])
    assert f(big + 0.999 * half_ulp) == 0x7F7F
    assert f(big + half_ulp) == 0x7F80                                 # tie goes to the even side: inf
    assert f(-1e300) == 0xFF80 and f(np.inf) == 0x7F80
    assert f(2.0 ** -134) == 0x0000 and f(np.nextafter(2.0 ** -134, 1.0)) == 0x0001
    assert f(-1e-320) == 0x8000
    assert f(float("nan")) & 0x7FFF > 0x7F80
    # a value whose fp32 rounding would land on a bf16 tie: single rounding must not
    x = 1.0 + 2.0 ** -8 + 2.0 ** -30
    assert f(x) == 0x3F81
    assert f(1.0 + 2.0 ** -8) == 0x3F80


# ----------------------------------------------------------------- rotation --

def test_delta_zero_is_the_identity():
    rng = np.random.default_rng(0)
    row = bf16_bits(rng.standard_normal(576))
    assert np.array_equal(orc.reattach_row(row, 0, INV), row)
    k = rng.standard_normal(64)
    assert np.array_equal(orc.rotate_kr_f64(k, 0, INV), k)


@pytest.mark.parametrize("inv", [INV, wl.inv_freq_yarn()])
def test_group_law_and_inverse(inv):
    rng = np.random.default_rng(1)
    for a, b in [(1, 1), (17, -5), (-2048, 2047), (100000, -99999), (40, 60), (12345, 54321)]:
        k = rng.standard_normal(64)
        two_steps = orc.rotate_kr_f64(orc.rotate_kr_f64(k, a, inv), b, inv)
        one_step = orc.rotate_kr_f64(k, a + b, inv)
        assert np.max(np.abs(two_steps - one_step)) < 1e-10
        back = orc.rotate_kr_f64(orc.rotate_kr_f64(k, a, inv), -a, inv)
        assert np.max(np.abs(back - k)) < 1e-10


def test_rotating_a_key_made_at_p_by_delta_gives_the_key_made_at_p_plus_delta():
    """The key at position p is R(p) applied to the un-rotated key; written here in
    complex form, pair (i, i+32) <-> z_i = k_i + 1j*k_{i+32}, z_i * exp(1j p w_i)."""
    rng = np.random.default_rng(2)
    w = INV.astype(np.float64)
    for p, delta in [(0, 77), (500, -468), (4000, 2048), (31, 100000), (90000, -90000)]:
        k = rng.standard_normal(64)
        z = k[:32] + 1j * k[32:]
        at_p = z * np.exp(1j * p * w)
        at_q = z * np.exp(1j * (p + delta) * w)
        got = orc.rotate_kr_f64(np.concatenate([at_p.real, at_p.imag]), delta, INV)
        assert np.max(np.abs(got - np.concatenate([at_q.real, at_q.imag]))) < 1e-10


def test_quarter_turn_is_rotate_half():
    rng = np.random.default_rng(3)
    k = rng.standard_normal(64)
    delta = 8
    inv = np.full(32, (np.pi / 2) / delta, np.float32)
    got = orc.rotate_kr_f64(k, delta, inv)
    err = abs(delta * float(inv[0]) - np.pi / 2)           # fp32 cannot hold pi/16 exactly
    assert err < 1e-6
    assert np.max(np.abs(got[:32] - (-k[32:]))) < 2e-6 * np.max(np.abs(k))
    assert np.max(np.abs(got[32:] - k[:32])) < 2e-6 * np.max(np.abs(k))
    # exact quarter turn through the half turn instead: delta*w = pi => out = -in
    got = orc.rotate_kr_f64(k, 2 * delta, inv)
    assert np.max(np.abs(got + k)) < 4e-6 * np.max(np.abs(k))


def test_only_the_rotating_pairs_move_and_direction_is_counter_clockwise():
    k = np.zeros(64)
    k[3] = 1.0                                             # unit vector on the "a" side of pair 3
    inv = np.zeros(32, np.float32)
    inv[3] = np.float32(0.001)
    out = orc.rotate_kr_f64(k, 100, inv)                   # angle 0.1 rad
    want = np.zeros(64)
    want[3], want[35] = np.cos(100 * float(inv[3])), np.sin(100 * float(inv[3]))
    assert np.max(np.abs(out - want)) < 1e-15
    assert out[35] > 0                                     # positive delta turns a towards +b
    out = orc.rotate_kr_f64(k, -100, inv)
    assert out[35] < 0


def test_pair_norms_are_preserved():
    rng = np.random.default_rng(4)
    for inv in (INV, wl.inv_freq_yarn()):
        k = rng.standard_normal(64)
        out = orc.rotate_kr_f64(k, -73211, inv)
        assert np.max(np.abs(np.hypot(out[:32], out[32:]) - np.hypot(k[:32], k[32:]))) < 1e-12


def test_angle_precision_against_exact_reduction():
    """phi = delta * (exact value of the fp32 frequency).  Reduce it mod 2*pi with
    python's exact rationals and a 60-digit pi, then compare."""
    from fractions import Fraction
    pi60 = Fraction("3.14159265358979323846264338327950288419716939937510582097494")
    k = np.zeros(64)
    k[1] = 1.0
    for delta in (100000, -99991, 131071):
        w = Fraction(float(INV[1]))                         # exact value of the fp32 number
        phi = w * delta
        turns = phi / (2 * pi60)
        frac = turns - (turns.numerator // turns.denominator)
        small = float(frac * 2 * pi60)                      # in [0, 2pi), error ~1e-16
        out = orc.rotate_kr_f64(k, delta, INV)
        assert abs(out[1] - np.cos(small)) < 1e-11 and abs(out[33] - np.sin(small)) < 1e-11


def test_bf16_precision_matches_the_reported_bound_and_does_not_accumulate():
    """Sec. 7.3: the rotation error is 4.7e-3 rel-L2 in bf16 and does not accumulate.
    bf16(R(delta) * bf16(R(p) k)) against the exact R(p+delta) k must sit at a few
    1e-3 -- two bf16 roundings, each about 2^-9/sqrt(3)*... relative -- below the
    paper's figure, and flat in |delta|."""
    rng = np.random.default_rng(5)
    w = INV.astype(np.float64)

    def rel_l2(p, delta, n=300):
        num = den = 0.0
        for _ in range(n):
            k = rng.standard_normal(64)
            z = k[:32] + 1j * k[32:]
            at_p = z * np.exp(1j * p * w)
            exact = z * np.exp(1j * (p + delta) * w)
            exact = np.concatenate([exact.real, exact.imag])
            row = np.zeros(576, np.uint16)
            row[512:] = orc.f64_to_bf16(np.concatenate([at_p.real, at_p.imag]))   # cached base, bf16
            out = orc.bf16_to_f64(orc.reattach_row(row, delta, INV)[512:])
            num += np.sum((out - exact) ** 2)
            den += np.sum(exact ** 2)
        return np.sqrt(num / den)

    errs = [rel_l2(1000, d) for d in (1, 64, 2048, 16384, 100000, -100000)]
    assert all(1.0e-3 < e < 4.7e-3 for e in errs), errs
    assert max(errs) / min(errs) < 1.25                      # flat in |delta|
    # a pure bf16 rounding of N(0,1) data has rel-L2 ~ 1.65e-3; two roundings ~ sqrt(2) of that
    assert abs(np.mean(errs) / 1.65e-3 - np.sqrt(2)) < 0.25


def test_yarn_frequencies_match_the_hand_derived_anchors():
    inv = wl.inv_freq_yarn()
    path = os.path.join(os.path.dirname(__file__), "golden", "yarn_inv_freq.txt")
    n = 0
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        i, v = line.split()
        assert abs(float(inv[int(i)]) / float(v) - 1.0) < 2e-6, (i, inv[int(i)], v)
        n += 1
    assert n == 9
    plain = wl.inv_freq_plain()
    assert np.array_equal(inv[:11], plain[:11])
    assert abs(float(plain[16]) - 0.01) < 1e-9 and plain[0] == 1.0


# ------------------------------------------------------------ whole gather --

def test_gather_rotate_scatter_rows_layers_slots():
    rng = np.random.default_rng(6)
    L, src_rows, dst_rows = 3, 50, 40
    src = bf16_bits(rng.standard_normal((L, src_rows, 576)))
    dst = np.full((L, dst_rows, 576), wl.SENTINEL_BF16, np.uint16)
    dst_slots = rng.permutation(dst_rows).astype(np.int32)
    hits = orc.Hits(src_row=np.array([5, 30], np.uint32), dst_tok=np.array([2, 20], np.uint32),
                    len=np.array([7, 11], np.uint32), delta=np.array([-300, 41], np.int32))
    orc.reattach(src, dst, dst_slots, hits, INV)
    touched = np.zeros(dst_rows, bool)
    for h in range(2):
        for j in range(int(hits.len[h])):
            srow, drow = int(hits.src_row[h]) + j, int(dst_slots[int(hits.dst_tok[h]) + j])
            touched[drow] = True
            for l in range(L):
                # c_KV reused verbatim (Sec. 1: the bulk of the row is position-free)
                assert np.array_equal(dst[l, drow, :512], src[l, srow, :512])
                # k_r: complex form, rounded by torch (fp64 -> fp32 -> bf16 may double-round,
                # so allow one bf16 step against it)
                k = orc.bf16_to_f64(src[l, srow, 512:])
                z = (k[:32] + 1j * k[32:]) * np.exp(1j * int(hits.delta[h]) * INV.astype(np.float64))
                want = np.concatenate([z.real, z.imag])
                got = orc.bf16_to_f64(dst[l, drow, 512:])
                assert np.all(np.abs(got - want) <= np.abs(want) * 2.0 ** -8 + 1e-30)
    assert np.all(dst[:, ~touched, :] == wl.SENTINEL_BF16)      # other rows untouched
    assert touched.sum() == 18


def test_out_of_range_indices_are_refused():
    src = np.zeros((1, 4, 576), np.uint16)
    dst = np.zeros((1, 4, 576), np.uint16)
    slots = np.arange(4, dtype=np.int32)
    bad = orc.Hits(np.array([2], np.uint32), np.array([0], np.uint32), np.array([3], np.uint32),
                   np.array([0], np.int32))
    with pytest.raises(IndexError):
        orc.reattach(src, dst, slots, bad, INV)


# ------------------------------------------------------------- split pool --

def test_split_pool_variant_references_ckv_and_materialises_only_kr():
    """App. C "Split TokenToKVPool": c_KV is shared by reference, only the 64-dim k_r is
    written per request.  The k_r written must be the k_r slice the full materialisation
    writes, and the index must name the source row whose c_KV that materialisation copies."""
    rng = np.random.default_rng(8)
    L, src_rows, dst_rows = 2, 60, 45
    src = bf16_bits(rng.standard_normal((L, src_rows, 576)))
    slots = rng.permutation(dst_rows).astype(np.int32)
    hits = orc.Hits(src_row=np.array([3, 40], np.uint32), dst_tok=np.array([1, 25], np.uint32),
                    len=np.array([9, 13], np.uint32), delta=np.array([777, -12], np.int32))
    full = np.full((L, dst_rows, 576), wl.SENTINEL_BF16, np.uint16)
    orc.reattach(src, full, slots, hits, INV)
    kr = np.full((L, dst_rows, 64), wl.SENTINEL_BF16, np.uint16)
    idx = np.full(dst_rows, -1, np.int32)
    orc.reattach_kr(src, kr, idx, slots, hits, INV)
    assert np.array_equal(kr, full[:, :, 512:])                       # same rotated keys, same untouched rows
    touched = idx >= 0
    assert touched.sum() == 22
    for l in range(L):
        assert np.array_equal(src[l, idx[touched], :512], full[l, touched, :512])   # the referenced c_KV
    assert np.all(full[:, ~touched, :512] == wl.SENTINEL_BF16)


# ------------------------------------------------- interleaved pair layout --

def to_half_split(x):
    """interleaved layout (pair i = elements 2i, 2i+1) -> half-split (i, i+32)"""
    return np.concatenate([x[..., 0::2], x[..., 1::2]], axis=-1)


def to_interleaved(x):
    out = np.empty_like(x)
    out[..., 0::2], out[..., 1::2] = x[..., :32], x[..., 32:]
    return out


@pytest.mark.parametrize("inv", [INV, wl.inv_freq_yarn()], ids=["plain", "yarn"])
def test_interleaved_layout_is_the_half_split_rotation_under_the_pair_permutation(inv):
    rng = np.random.default_rng(21)
    for delta in (0, 1, -7, 4097, -99999):
        k = rng.standard_normal(64)
        got = orc.rotate_kr_f64(k, delta, inv, pair_mode=1)
        want = to_interleaved(orc.rotate_kr_f64(to_half_split(k), delta, inv, pair_mode=0))
        assert np.array_equal(got, want)                   # same operations on the same numbers
        z = (k[0::2] + 1j * k[1::2]) * np.exp(1j * delta * inv.astype(np.float64))
        assert np.max(np.abs(got[0::2] - z.real)) < 1e-12 and np.max(np.abs(got[1::2] - z.imag)) < 1e-12


def test_interleaved_single_pair_moves_its_neighbour_not_its_far_partner():
    k = np.zeros(64)
    k[6] = 1.0                                             # "a" of pair 3 in the interleaved layout
    inv = np.zeros(32, np.float32)
    inv[3] = np.float32(0.001)
    out = orc.rotate_kr_f64(k, 100, inv, pair_mode=1)
    want = np.zeros(64)
    want[6], want[7] = np.cos(100 * float(inv[3])), np.sin(100 * float(inv[3]))
    assert np.max(np.abs(out - want)) < 1e-15 and out[7] > 0 and out[38] == 0.0


def test_interleaved_rows_through_the_gather_rotate_scatter():
    rng = np.random.default_rng(22)
    L, src_rows, dst_rows = 2, 40, 50
    src = bf16_bits(rng.standard_normal((L, src_rows, 576)))
    slots = rng.permutation(dst_rows).astype(np.int32)[:30]
    hits = orc.Hits(np.array([3, 20], np.uint32), np.array([0, 12], np.uint32), np.array([12, 18], np.uint32),
                    np.array([-513, 77], np.int32))
    got = np.full((L, dst_rows, 576), 0x7FC1, np.uint16)
    orc.reattach(src, got, slots, hits, INV, pair_mode=1)
    # the same through the half-split path on permuted k_r columns
    src_hs = src.copy()
    src_hs[..., 512:] = to_half_split(src[..., 512:])
    want = np.full((L, dst_rows, 576), 0x7FC1, np.uint16)
    orc.reattach(src_hs, want, slots, hits, INV, pair_mode=0)
    touched = np.zeros(dst_rows, bool)
    touched[slots] = True
    want[:, touched, 512:] = to_interleaved(want[:, touched, 512:])
    assert np.array_equal(got, want)
    kr = np.full((L, dst_rows, 64), 0x7FC1, np.uint16)
    idx = np.full(dst_rows, -1, np.int32)
    orc.reattach_kr(src, kr, idx, slots, hits, INV, pair_mode=1)
    assert np.array_equal(kr[:, touched], got[:, touched, 512:]) and np.all(kr[:, ~touched] == 0x7FC1)


# ------------------------------------------------- no-materialise variant --

@pytest.mark.parametrize("pair_mode", [0, 1])
def test_reference_variant_rotated_at_load_time_equals_the_materialised_rows(pair_mode):
    """What a load path would do with the references and the per-hit (cos, sin) table, done
    here by numpy in complex arithmetic, must give the rows the materialising oracle writes."""
    rng = np.random.default_rng(31)
    L, src_rows, dst_rows = 2, 300, 260
    src = bf16_bits(rng.standard_normal((L, src_rows, 576)))
    slots = rng.permutation(dst_rows).astype(np.int32)[:200]
    hits = orc.Hits(np.array([5, 100, 210], np.uint32), np.array([0, 60, 130], np.uint32),
                    np.array([60, 70, 50], np.uint32), np.array([-99999, 0, 4097], np.int32))
    inv = wl.inv_freq_yarn()
    want = np.full((L, dst_rows, 576), 0x7FC1, np.uint16)
    orc.reattach(src, want, slots, hits, inv, pair_mode)
    row_index = np.full(dst_rows, -1, np.int32)
    hit_index = np.full(dst_rows, -1, np.int32)
    trig = orc.reattach_ref(src_rows, row_index, hit_index, slots, hits, inv)
    touched = row_index >= 0
    assert touched.sum() == 180 and np.array_equal(touched, hit_index >= 0)
    assert np.all(want[:, ~touched] == 0x7FC1)
    assert np.array_equal(trig[1], np.tile([1.0, 0.0], (32, 1)))          # delta = 0: the exact identity
    assert np.max(np.abs(trig[..., 0] ** 2 + trig[..., 1] ** 2 - 1.0)) < 1e-15
    for slot in np.nonzero(touched)[0]:
        rows = src[:, row_index[slot]]                                     # [L][576], read "at load time"
        assert np.array_equal(rows[:, :512], want[:, slot, :512])          # c_KV by reference: the same bits
        k = orc.bf16_to_f64(rows[:, 512:])
        a, b = (k[:, 0::2], k[:, 1::2]) if pair_mode else (k[:, :32], k[:, 32:])
        z = (a + 1j * b) * (trig[hit_index[slot], :, 0] + 1j * trig[hit_index[slot], :, 1])
        out = np.empty_like(k)
        if pair_mode:
            out[:, 0::2], out[:, 1::2] = z.real, z.imag
        else:
            out[:, :32], out[:, 32:] = z.real, z.imag
        got = orc.f64_to_bf16(out)
        step = np.abs(got.astype(np.int32) - want[:, slot, 512:].astype(np.int32))
        assert step.max() <= 1                                             # complex product vs the oracle's a c - b s
        assert (step == 0).mean() > 0.99


# ----------------------------------------------------------------- fp8 rows --

def fp8_rows(rng, shape_lr, kr_bits):
    """[L][rows][328] u16: 512 arbitrary bytes (e4m3 codes, every pattern allowed), four fp32 scales,
    then the given 64 bf16 k_r elements."""
    L, rows = shape_lr
    out = np.empty((L, rows, 328), np.uint16)
    out[:, :, :256] = rng.integers(0, 65536, (L, rows, 256), dtype=np.uint16)
    scales = rng.uniform(1e-3, 4.0, (L, rows, 4)).astype(np.float32)
    out[:, :, 256:264] = scales.view(np.uint16).reshape(L, rows, 8)
    out[:, :, 264:] = kr_bits
    return out


@pytest.mark.parametrize("pair_mode", [0, 1], ids=["half-split", "interleaved"])
def test_fp8_rows_copy_the_quantised_part_and_rotate_kr_as_in_bf16_rows(pair_mode):
    """Rows whose c_KV is quantised (512 e4m3 bytes and four fp32 block scales, k_r left in bf16):
    the 528 position-free bytes come through bit for bit, the k_r that follows them is the k_r a
    bf16 row with the same key gets, and nothing else is written."""
    rng = np.random.default_rng(21)
    L, src_rows, dst_rows = 2, 40, 33
    wide = bf16_bits(rng.standard_normal((L, src_rows, 576)))
    src = fp8_rows(rng, (L, src_rows), wide[:, :, 512:])
    slots = rng.permutation(dst_rows).astype(np.int32)
    hits = orc.Hits(src_row=np.array([4, 22], np.uint32), dst_tok=np.array([0, 17], np.uint32),
                    len=np.array([6, 10], np.uint32), delta=np.array([1234, -77], np.int32))
    dst = np.full((L, dst_rows, 328), wl.SENTINEL_BF16, np.uint16)
    orc.reattach(src, dst, slots, hits, INV, pair_mode)
    ref = np.full((L, dst_rows, 576), wl.SENTINEL_BF16, np.uint16)
    orc.reattach(wide, ref, slots, hits, INV, pair_mode)
    assert np.array_equal(dst[:, :, 264:], ref[:, :, 512:])            # same keys, same untouched rows
    touched = np.zeros(dst_rows, bool)
    for h in range(2):
        for j in range(int(hits.len[h])):
            srow, drow = int(hits.src_row[h]) + j, int(slots[int(hits.dst_tok[h]) + j])
            touched[drow] = True
            assert np.array_equal(dst[:, drow, :264], src[:, srow, :264])
            # the key sits right behind the 528 bytes: complex form of the rotation, one bf16 step allowed
            k = orc.bf16_to_f64(src[0, srow, 264:])
            a, b = (k[0::2], k[1::2]) if pair_mode else (k[:32], k[32:])
            z = (a + 1j * b) * np.exp(1j * int(hits.delta[h]) * INV.astype(np.float64))
            got = orc.bf16_to_f64(dst[0, drow, 264:])
            ga, gb = (got[0::2], got[1::2]) if pair_mode else (got[:32], got[32:])
            assert np.all(np.abs(ga - z.real) <= np.abs(z.real) * 2.0 ** -8 + 1e-30)
            assert np.all(np.abs(gb - z.imag) <= np.abs(z.imag) * 2.0 ** -8 + 1e-30)
    assert touched.sum() == 16 and np.all(dst[:, ~touched] == wl.SENTINEL_BF16)
    # one row alone, and the identity
    one = orc.reattach_row(src[1, 9], 0, INV, pair_mode)
    assert one.shape == (328,) and np.array_equal(one, src[1, 9])
    # split pool over fp8 rows: the same keys, references to the same rows
    kr = np.full((L, dst_rows, 64), wl.SENTINEL_BF16, np.uint16)
    idx = np.full(dst_rows, -1, np.int32)
    orc.reattach_kr(src, kr, idx, slots, hits, INV, pair_mode)
    assert np.array_equal(kr, dst[:, :, 264:]) and np.array_equal(idx >= 0, touched)
    assert np.array_equal(src[:, idx[touched], :264], dst[:, touched, :264])


def test_rows_of_any_other_width_are_refused():
    with pytest.raises(AssertionError):
        orc.reattach_row(np.zeros(320, np.uint16), 1, INV)

"""The checks that pin the CPU oracle to things other than itself.

Each ``pin_*`` function takes a loaded oracle library handle (``lib=None`` is
the real one) and raises AssertionError if that library breaks what the paper
and the arithmetic fix.  ``test_oracle_pins.py`` runs them on the real oracle;
``test_oracle_mutants.py`` runs them on deliberately wrong builds of the
oracle's source and expects them to fail.

Expected values come from: closed forms; exact rational arithmetic rounded by
the IEEE definition (``exact_fp``); the error bound of the method; a library
bf16 cast (torch); the error figures printed with Fig. 7 of the paper.
"""
from __future__ import annotations

import os
from fractions import Fraction

import numpy as np
import torch

from exact_fp import bf16_bits_to_f32, frac, rne_int, round_to_f32
from oracle import equarx_oracle as o

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
TINY = 127.0 * 2.0 ** -126          # smallest absmax that still gets a non-zero scale


def _rng(seed):
    return np.random.default_rng(seed)


def _bf16(v: np.ndarray) -> np.ndarray:
    """fp32 -> raw bf16 bits through torch's cast (a library routine, not the oracle's)."""
    t = torch.from_numpy(np.ascontiguousarray(v, np.float32)).to(torch.bfloat16)
    return t.view(torch.uint16).numpy().copy()


# --------------------------------------------------------------------------- quantizer

def pin_zero_block(lib=None):
    """All-zero block: scale 0 and codes 0 (also -0, and blocks whose absmax is below the threshold)."""
    for B in (32, 256):
        v = np.zeros(3 * B, np.float32)
        v[B:2 * B] = -0.0
        v[2 * B:] = np.float32(2.0 ** -126)            # normal, but absmax/127 would be subnormal
        c, s = o.quantize_f32(v, B, lib=lib)
        assert not c.any() and not s.any()
        c, s = o.quantize_bf16(_bf16(v), B, lib=lib)
        assert not c.any() and not s.any()
    # exactly at the threshold the block is quantized normally
    v = np.array([TINY, -TINY, TINY / 2, 0.0], np.float32)
    c, s = o.quantize_f32(v, 4, lib=lib)
    assert s[0] == np.float32(2.0 ** -126)
    assert c.tolist() == [127, -127, 64, 0]            # 63.5 is a tie: to even


def pin_absmax_to_127_all_bf16(lib=None):
    """+-absmax maps to +-127 and scale = RN(absmax/127), for every finite bf16 absmax above the threshold."""
    pats = np.arange(1, 0x7F80, dtype=np.uint16)        # all positive finite bf16
    vals = bf16_bits_to_f32(pats)
    pats = pats[vals >= np.float32(TINY)]
    vals = vals[vals >= np.float32(TINY)]
    B = 4
    x = np.zeros((pats.size, B), np.uint16)
    x[:, 0] = pats
    x[:, 1] = pats | 0x8000                             # -a
    x[:, 3] = pats
    c, s = o.quantize_bf16(x, B, lib=lib)
    c = c.reshape(-1, B)
    assert (c[:, 0] == 127).all() and (c[:, 1] == -127).all() and (c[:, 2] == 0).all() and (c[:, 3] == 127).all()
    # the scale is the correctly rounded quotient; check every 37th value exactly, all of them loosely
    for k in range(0, vals.size, 37):
        want = round_to_f32(frac(vals[k]) / 127)
        assert s[k] == want, (k, vals[k], s[k], want)
    np.testing.assert_allclose(s.astype(np.float64), vals.astype(np.float64) / 127.0, rtol=2.0 ** -23)


def pin_round_trip_half_scale(lib=None):
    """|v - code*scale| <= scale/2 (plus fp32 rounding slack) for every element; codes stay in [-127,127]."""
    rng = _rng(11)
    for B, n in ((32, 4096), (64, 4096 + 64), (128, 8192), (256, 8192 + 100), (512, 4096), (7, 700)):
        for kind in range(3):
            if kind == 0:
                v = rng.standard_normal(n)
            elif kind == 1:
                v = rng.standard_normal(n) * np.exp(3 * rng.standard_normal(n))
            else:
                v = rng.standard_t(3, n) * 1e-20
            v = v.astype(np.float32)
            c, s = o.quantize_f32(v, B, lib=lib)
            assert c.min() >= -127 and c.max() <= 127
            se = np.repeat(s.astype(np.float64), B)[:n]
            err = np.abs(v.astype(np.float64) - c.astype(np.float64) * se)
            assert (err <= se * (0.5 + 2.0 ** -15)).all()
            # the block's largest element sits on +-127
            for b in range(0, o.num_blocks(n, B), 5):
                blk = slice(b * B, min(n, (b + 1) * B))
                j = np.argmax(np.abs(v[blk]))
                assert abs(int(c[blk][j])) == 127


def pin_special_blocks(lib=None):
    """Closed-form cases: repeated value, exact multiples, power-of-two scaling, negation, ties, permutation."""
    B = 256
    # (i) one repeated value
    for a in (3.0, 0.37, 1e-12, 6e30):
        v = np.full(B, a, np.float32)
        v[1::2] *= -1
        c, s = o.quantize_f32(v, B, lib=lib)
        assert (c[0::2] == 127).all() and (c[1::2] == -127).all()
        assert s[0] == round_to_f32(frac(np.float32(a)) / 127)
    # (ii) values k * 2^e with absmax 127 * 2^e: scale = 2^e, codes = k, no rounding anywhere
    k = np.arange(-127, 128)
    for e in (-40, -3, 0, 5, 60):
        v = (k * 2.0 ** e).astype(np.float32)
        c, s = o.quantize_f32(v, v.size, lib=lib)
        assert s[0] == np.float32(2.0 ** e)
        assert (c == k).all()
    # (iii) scaling a tensor by 2^k scales the scales and leaves the codes
    rng = _rng(5)
    v = rng.standard_normal(4 * B).astype(np.float32)
    c0, s0 = o.quantize_f32(v, B, lib=lib)
    for p in (-30, -1, 7, 40):
        c1, s1 = o.quantize_f32(v * np.float32(2.0 ** p), B, lib=lib)
        assert (c1 == c0).all() and (s1 == s0 * np.float32(2.0 ** p)).all()
    # (iv) negation negates the codes (ties-to-even is symmetric)
    c1, s1 = o.quantize_f32(-v, B, lib=lib)
    assert (c1 == -c0).all() and (s1 == s0).all()
    # (v) ties go to the even code: absmax 127 gives scale 1, inv 1
    t = np.array([127, 0.5, 1.5, 2.5, 3.5, -0.5, -1.5, -2.5, 126.5, -126.5, 0.49999997, 0.50000006], np.float32)
    c, s = o.quantize_f32(t, t.size, lib=lib)
    assert s[0] == 1.0
    assert c.tolist() == [127, 0, 2, 2, 4, 0, -2, -2, 126, -126, 0, 1]
    # (vi) permuting a block permutes its codes; blocks do not see each other
    perm = rng.permutation(B)
    vp = v.copy()
    vp[:B] = v[:B][perm]
    c2, s2 = o.quantize_f32(vp, B, lib=lib)
    assert (c2[:B] == c0[:B][perm]).all() and (c2[B:] == c0[B:]).all() and (s2 == s0).all()
    # (vii) a ragged tail is a shorter block of its own
    c3, s3 = o.quantize_f32(v[: 3 * B + 17], B, lib=lib)
    ct, st = o.quantize_f32(v[3 * B: 3 * B + 17], 17, lib=lib)
    assert (c3[: 3 * B] == c0[: 3 * B]).all() and (c3[3 * B:] == ct).all() and s3[3] == st[0]
    # (viii) without the absolute value a block of negatives would lose its range
    vneg = -np.abs(v[:B]) - 1
    c4, s4 = o.quantize_f32(vneg, B, lib=lib)
    assert c4.min() == -127 and s4[0] == round_to_f32(frac(np.abs(vneg).max()) / 127)


def _expected_block(vals):
    """Q_B of one block by the IEEE definition, in exact arithmetic."""
    a = max(abs(frac(v)) for v in vals)
    if a < Fraction(127) * Fraction(2) ** -126:
        return [0] * len(vals), np.float32(0)
    scale = round_to_f32(a / 127)
    inv = round_to_f32(127 / a)
    codes = []
    for v in vals:
        r = round_to_f32(frac(v) * frac(inv))
        codes.append(max(-127, min(127, rne_int(frac(r)))))
    return codes, scale


def pin_quantizer_exact_small(lib=None):
    """Codes and scales on small inputs equal the exactly rounded definition, bit for bit."""
    rng = _rng(21)
    B = 8
    # bf16-valued inputs land on rounding ties often, which is where a wrong formula shows
    v = rng.standard_normal(40 * B).astype(np.float32)
    u = _bf16(v)
    vb = bf16_bits_to_f32(u)
    c, s = o.quantize_bf16(u, B, lib=lib)
    for b in range(40):
        codes, scale = _expected_block(vb[b * B:(b + 1) * B])
        assert c[b * B:(b + 1) * B].tolist() == codes
        assert s[b] == scale
    w = (rng.standard_normal(40 * B) * np.exp(4 * rng.standard_normal(40 * B))).astype(np.float32)
    c, s = o.quantize_f32(w, B, lib=lib)
    for b in range(40):
        codes, scale = _expected_block(w[b * B:(b + 1) * B])
        assert c[b * B:(b + 1) * B].tolist() == codes
        assert s[b] == scale
    # pairs (absmax, v) on which multiplying by fl(127/absmax) and dividing by fl(absmax/127) round to
    # different codes: numpy only SELECTS them; what is expected comes from the exact arithmetic above
    a = np.abs(bf16_bits_to_f32(_bf16(rng.standard_normal(400_000).astype(np.float32)))) + np.float32(2.0)
    a = bf16_bits_to_f32(_bf16(a))
    v = bf16_bits_to_f32(_bf16((rng.uniform(-1, 1, a.size) * a).astype(np.float32)))
    by_mul = np.rint(v * (np.float32(127.0) / a))
    by_div = np.rint(v / (a / np.float32(127.0)))
    pick = np.flatnonzero(by_mul != by_div)[:60]
    assert pick.size >= 20
    blocks = np.stack([a[pick], v[pick]], axis=1).astype(np.float32)
    c, s = o.quantize_f32(blocks, 2, lib=lib)
    for k in range(pick.size):
        codes, scale = _expected_block(blocks[k])
        assert c[2 * k: 2 * k + 2].tolist() == codes and s[k] == scale


# --------------------------------------------------------------------------- dequantize, bf16

def pin_dequantize(lib=None):
    """Dq is code*scale of the element's own block; the bf16 output is its correctly rounded narrowing."""
    rng = _rng(31)
    B, nb = 32, 9
    n = B * nb - 5
    c = rng.integers(-127, 128, n).astype(np.int8)
    s = np.exp(rng.standard_normal(nb) * 5).astype(np.float32)
    d = o.dequantize_f32(c, s, B, lib=lib)
    want = np.array([round_to_f32(Fraction(int(c[j])) * frac(s[j // B])) for j in range(n)], np.float32)
    assert (d.view(np.uint32) == want.view(np.uint32)).all()
    out = o.dequantize_bf16(c, s, B, lib=lib)
    assert (out == _bf16(want)).all()


def pin_bf16_narrowing(lib=None):
    """fp32 -> bf16 agrees with torch's cast on random values, ties, subnormals, the overflow edge, +-0, inf."""
    rng = _rng(41)
    bits = rng.integers(0, 2 ** 32, 200_000, dtype=np.uint64).astype(np.uint32)
    bits = bits[(bits & 0x7F800000) != 0x7F800000]                      # finite
    ties = (rng.integers(0, 2 ** 16, 5000, dtype=np.uint64).astype(np.uint32) << 16) | 0x8000
    ties = ties[(ties & 0x7F800000) != 0x7F800000]
    near = np.concatenate([ties - 1, ties + 1])
    special = np.array([0x00000000, 0x80000000, 0x7F7FFFFF, 0xFF7FFFFF, 0x7F7F8000, 0x7F7F7FFF, 0x7F800000,
                        0xFF800000, 0x00000001, 0x00008000, 0x00018000, 0x007FFFFF], np.uint32)
    allb = np.concatenate([bits, ties, near, special])
    v = allb.view(np.float32)
    lib_ = lib or o._L()
    out = np.empty(v.size, np.uint16)
    lib_.equarx_oracle_f32_to_bf16(v.ctypes.data_as(o._c_f32p), v.size, out.ctypes.data_as(o._c_u16p))
    assert (out == _bf16(v)).all()
    # widening is the bit pattern shifted up
    u = np.arange(0, 2 ** 16, dtype=np.uint16)
    u = u[(u & 0x7F80) != 0x7F80]
    wide = np.empty(u.size, np.float32)
    lib_.equarx_oracle_bf16_to_f32(u.ctypes.data_as(o._c_u16p), u.size, wide.ctypes.data_as(o._c_f32p))
    assert (wide.view(np.uint32) == (u.astype(np.uint32) << 16)).all()


# --------------------------------------------------------------------------- one hop

def pin_hop_exact_small(lib=None):
    """The hop's partial sum is q*s + x rounded ONCE (exact rational check), then Q_B of it."""
    rng = _rng(51)
    B, nb = 8, 30
    n = B * nb
    cin = rng.integers(-127, 128, n).astype(np.int8)
    sin = (np.abs(rng.standard_normal(nb)) / 40 + 1e-3).astype(np.float32)
    x = _bf16(rng.standard_normal(n).astype(np.float32))
    xf = bf16_bits_to_f32(x)
    # a case where rounding the product first and the sum second gives another answer:
    # 3*(1+2^-23) - 3 is exactly 3*2^-23, but the product alone rounds (on a tie) to 3+2^-21
    cin[:B] = 0
    cin[0] = 3
    sin[0] = np.float32(1.0 + 2.0 ** -23)
    x[:B] = 0
    x[0] = _bf16(np.array([-3.0], np.float32))[0]
    xf = bf16_bits_to_f32(x)
    c, s = o.hop(cin, sin, x, B, lib=lib)
    assert s[0] == round_to_f32(Fraction(3) * Fraction(2) ** -23 / 127) and c[0] == 127
    for b in range(nb):
        t = [round_to_f32(Fraction(int(cin[j])) * frac(sin[b]) + frac(xf[j])) for j in range(b * B, (b + 1) * B)]
        codes, scale = _expected_block(t)
        assert s[b] == scale, b
        assert c[b * B:(b + 1) * B].tolist() == codes, b


def pin_hop_special(lib=None):
    """Adding to an all-zero wire is plain Q_B(x); adding a zero shard to a wire leaves the wire as it is."""
    rng = _rng(61)
    for B in (32, 256):
        n = 6 * B + 11
        nb = o.num_blocks(n, B)
        x = _bf16((rng.standard_normal(n) * np.exp(rng.standard_normal(n))).astype(np.float32))
        c0, s0 = o.quantize_bf16(x, B, lib=lib)
        c1, s1 = o.hop(np.zeros(n, np.int8), np.zeros(nb, np.float32), x, B, lib=lib)
        assert (c1 == c0).all() and (s1 == s0).all()
        # a wire with arbitrary scales and zero codes is also a zero
        c1, s1 = o.hop(np.zeros(n, np.int8), np.full(nb, 3.25, np.float32), x, B, lib=lib)
        assert (c1 == c0).all() and (s1 == s0).all()
        # requantizing what is already on the grid changes nothing (Q(Dq(Q(v))) = Q(v))
        c2, s2 = o.hop(c0, s0, np.zeros(n, np.uint16), B, lib=lib)
        assert (c2 == c0).all() and (s2 == s0).all()
        # the wire's sign and the local shard's sign both matter
        neg = x ^ np.uint16(0x8000)
        c3, s3 = o.hop(c0, s0, neg, B, lib=lib)      # Dq(Q(x)) - x: a residual bounded by scale/2
        res = np.abs(o.dequantize_f32(c3, s3, B, lib=lib).astype(np.float64))
        assert (res <= np.repeat(s0.astype(np.float64), B)[:n] * (0.5 + 2.0 ** -10)).all()


# --------------------------------------------------------------------------- whole chain

def _chain_inputs(seed, P, n, heavy=False):
    rng = _rng(seed)
    parts = []
    for _ in range(P):
        v = rng.standard_normal(n)
        if heavy:
            v = v * np.exp(rng.standard_normal(n))
        parts.append(_bf16(v.astype(np.float32)))
    return parts


def pin_chain_error_bound(lib=None):
    """|out - exact sum| <= sum over hops of scale_i/2 (<= P*max scale/2), plus fp32/bf16 rounding slack."""
    for seed, P, n, B, heavy in ((1, 4, 4096, 256, False), (2, 8, 2048 + 96, 64, True), (3, 16, 1024, 128, False),
                                 (4, 2, 999, 32, True), (5, 8, 4096, 512, False)):
        parts = _chain_inputs(seed, P, n, heavy)
        out, wc, ws = o.reduce_chain(parts, B, keep_wire=True, lib=lib)
        ref = np.zeros(n, np.float64)
        for p in parts:
            ref += bf16_bits_to_f32(p).astype(np.float64)
        se = np.repeat(ws.astype(np.float64), B, axis=1)[:, :n]
        dq = wc[-1].astype(np.float64) * se[-1]
        bound = se.sum(axis=0) * 0.5 * (1 + 2.0 ** -14) + P * 2.0 ** -23 * (np.abs(ref) + se.max(axis=0) * 127)
        assert (np.abs(dq - ref) <= bound).all()
        assert (bound <= P * se.max(axis=0) * 0.5 * (1 + 2.0 ** -10) + 1e-30).all()
        # the bf16 output is the last wire content, dequantized and narrowed by a library cast
        assert (out == _bf16((wc[-1].astype(np.float32) * np.repeat(ws[-1], B)[:n]).astype(np.float32))).all()
        # and it is not trivially loose: the quantization noise is really there
        assert np.abs(dq - ref).max() > 0.05 * bound.max() / P


def pin_chain_degenerate(lib=None):
    """P=1 is Dq(Q(x)); zero partials after the first leave the result unchanged; order of partials matters."""
    rng = _rng(71)
    B, n = 128, 5 * 128 + 40
    x = _bf16(rng.standard_normal(n).astype(np.float32))
    z = np.zeros(n, np.uint16)
    c, s = o.quantize_bf16(x, B, lib=lib)
    one = o.reduce_chain([x], B, lib=lib)
    assert (one == _bf16(c.astype(np.float32) * np.repeat(s, B)[:n])).all()
    for P in (2, 5, 16):
        assert (o.reduce_chain([x] + [z] * (P - 1), B, lib=lib) == one).all()
    # zeros first: the chain starts from an all-zero wire, then takes x unquantized, quantizes once
    assert (o.reduce_chain([z, z, x], B, lib=lib) == one).all()
    # x + (-x) through the chain leaves only the first quantization's residual, quantized again
    neg = x ^ np.uint16(0x8000)
    out, wc, ws = o.reduce_chain([x, neg], B, keep_wire=True, lib=lib)
    resid = bf16_bits_to_f32(out).astype(np.float64)
    assert (np.abs(resid) <= np.repeat(ws[0].astype(np.float64), B)[:n] * 0.51).all()
    # each partial enters exactly once: y + 0 + x equals the two-partial chain [y, x] hop for hop
    y = _bf16(rng.standard_normal(n).astype(np.float32))
    out2, wc2, ws2 = o.reduce_chain([y, z, x], B, keep_wire=True, lib=lib)
    out3, wc3, ws3 = o.reduce_chain([y, x], B, keep_wire=True, lib=lib)
    assert (out2 == out3).all() and (wc2[0] == wc2[1]).all() and (wc2[2] == wc3[1]).all()
    # the wire kept by the chain is what hop-by-hop application produces
    parts = _chain_inputs(9, 5, n)
    out, wc, ws = o.reduce_chain(parts, B, keep_wire=True, lib=lib)
    cc, ss = o.quantize_bf16(parts[0], B, lib=lib)
    assert (wc[0] == cc).all() and (ws[0] == ss).all()
    for i in range(1, 5):
        cc, ss = o.hop(cc, ss, parts[i], B, lib=lib)
        assert (wc[i] == cc).all() and (ws[i] == ss).all()


def pin_exact_sums(lib=None):
    """The unquantized reference sums agree with numpy's (fp64 exact; fp32 in array order)."""
    rng = _rng(81)          # magnitudes spread over 2^+-12 so that every fp32 addition really rounds
    parts = [_bf16((rng.standard_normal(3000) * 2.0 ** rng.integers(-12, 13, 3000)).astype(np.float32))
             for _ in range(6)]
    ref = np.zeros(3000, np.float64)
    acc = bf16_bits_to_f32(parts[0]).copy()
    for i, p in enumerate(parts):
        ref += bf16_bits_to_f32(p).astype(np.float64)
        if i:
            acc = (acc + bf16_bits_to_f32(p)).astype(np.float32)
    assert (o.exact_sum_f64(parts, lib=lib) == ref).all()
    assert (o.sum_f32(parts, lib=lib).view(np.uint32) == acc.view(np.uint32)).all()


# --------------------------------------------------------------------------- the paper's own numbers

def read_golden(name):
    vals = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                k, v = line.split()
                vals[k] = float(v)
    return vals


def pin_fig7_error(lib=None):
    """Fig. 7 setting (8 devices, block 64, N(0,1)): MSE of the fully quantized full-loop chain and of the
    all-gather-only flavour land on the paper's printed values (0.0014 and 0.0003) within a factor 1.5 --
    the paper's block geometry and torus chain differ from the contiguous, fixed-order reading here."""
    g = read_golden("fig7_error.txt")
    P, B = int(g["devices"]), int(g["block"])
    n = 256 * 4096                                      # a 256-row slice of the (4096, 4096) tensor
    parts = _chain_inputs(2024, P, n)
    ref = np.zeros(n, np.float64)
    for p in parts:
        ref += bf16_bits_to_f32(p).astype(np.float64)
    base = bf16_bits_to_f32(_bf16(ref.astype(np.float32))).astype(np.float64)    # the bf16 AllReduce result
    out = bf16_bits_to_f32(o.reduce_chain(parts, B, lib=lib)).astype(np.float64)
    mse_full = float(np.mean((out - base) ** 2))
    assert g["full_loop_rs_ag"] / 1.5 <= mse_full <= g["full_loop_rs_ag"] * 1.5, mse_full
    # all-gather only: the reduce-scatter result (fp32 sum) is quantized once and dequantized
    acc = bf16_bits_to_f32(parts[0]).copy()
    for p in parts[1:]:
        acc = (acc + bf16_bits_to_f32(p)).astype(np.float32)
    c, s = o.quantize_f32(acc, B, lib=lib)
    ag = bf16_bits_to_f32(o.dequantize_bf16(c, s, B, lib=lib)).astype(np.float64)
    mse_ag = float(np.mean((ag - base) ** 2))
    assert g["full_loop_ag_only"] / 1.5 <= mse_ag <= g["full_loop_ag_only"] * 1.5, mse_ag
    assert mse_ag < mse_full
    # textbook model of a uniform quantizer: noise variance = step^2 / 12 (plus the bf16 cast of the output)
    step2 = float(np.mean(np.repeat(s.astype(np.float64), B) ** 2)) / 12.0
    mse_q = float(np.mean((c.astype(np.float64) * np.repeat(s.astype(np.float64), B) - acc) ** 2))
    assert 0.93 * step2 <= mse_q <= 1.03 * step2, (mse_q, step2)
    return mse_full, mse_ag


ALL_PINS = [pin_zero_block, pin_absmax_to_127_all_bf16, pin_round_trip_half_scale, pin_special_blocks,
            pin_quantizer_exact_small, pin_dequantize, pin_bf16_narrowing, pin_hop_exact_small, pin_hop_special,
            pin_chain_error_bound, pin_chain_degenerate, pin_exact_sums, pin_fig7_error]


# --------------------------------------------------------------------------- variants of the chain

def _fma_exact(q, s, x):
    """fl32(q*s + x) for fp32 arrays q, s, x, by exact rational arithmetic (small inputs only)."""
    return np.array([round_to_f32(frac(a) * frac(b) + frac(c)) for a, b, c in zip(q, s, x)], np.float32)


def _dq(c, s, B):
    return c.astype(np.float32), np.repeat(s, B)[: c.size]


def pin_stage_knobs(lib=None):
    """The stage knob (Sec. 3.4): both = the pinned chain; none = an fp32 running sum cast by a library;
    all-gather only = one Q/Dq of that sum; reduce-scatter only = the chain without its last quantization."""
    for seed, P, n, B in ((1, 4, 3 * 256 + 100, 256), (2, 8, 640, 64), (3, 1, 300, 32), (4, 2, 512, 128)):
        parts = _chain_inputs(100 + seed, P, n, heavy=bool(seed & 1))
        assert (o.reduce_stages(parts, B, True, True, lib=lib) == o.reduce_chain(parts, B)).all()
        acc = bf16_bits_to_f32(parts[0]).copy()
        for p in parts[1:]:
            acc = (acc + bf16_bits_to_f32(p)).astype(np.float32)
        assert (o.reduce_stages(parts, B, False, False, lib=lib) == _bf16(acc)).all()
        c, s = o.quantize_f32(acc, B)
        assert (o.reduce_stages(parts, B, False, True, lib=lib) == o.dequantize_bf16(c, s, B)).all()
        # reduce-scatter only: the wire before the last hop comes from the pinned chain; the owner's sum is
        # fl32(q*s + x_last), checked exactly on a prefix
        got = o.reduce_stages(parts, B, True, False, lib=lib)
        if P == 1:
            assert (got == parts[0]).all()
        else:
            _, wc, ws = o.reduce_chain(parts[:-1], B, keep_wire=True)
            q, sc = _dq(wc[-1], ws[-1], B)
            m = min(n, 200)
            t = _fma_exact(q[:m], sc[:m], bf16_bits_to_f32(parts[-1])[:m])
            assert (got[:m] == _bf16(t)).all()
            # and over the whole tensor in fp64 (exact product, one rounding: at most an fp32 ulp off)
            t64 = q.astype(np.float64) * sc.astype(np.float64) + bf16_bits_to_f32(parts[-1]).astype(np.float64)
            back = bf16_bits_to_f32(got).astype(np.float64)
            assert (np.abs(back - t64) <= np.abs(t64) * 2.0 ** -8 + 1e-30).all()


def pin_semi_loop(lib=None):
    """Semi-loop (Sec. 3.3): the paper's 4-device example written out with pinned primitives; P=1, P=2;
    error bound; and lower error than the full loop."""
    B, n = 64, 256
    parts = _chain_inputs(7, 4, n)
    x = [bf16_bits_to_f32(p) for p in parts]
    # device 3 -> device 0 ; device 2 -> device 1 -> device 0 ; device 0 adds what arrives first, first
    c3, s3 = o.quantize_bf16(parts[3], B)
    own = _fma_exact(*_dq(c3, s3, B), x[0])
    c2, s2 = o.quantize_bf16(parts[2], B)
    t1 = _fma_exact(*_dq(c2, s2, B), x[1])
    c1, s1 = o.quantize_f32(t1, B)
    own = _fma_exact(*_dq(c1, s1, B), own)
    assert (o.reduce_semi_loop(parts, B, quantize_ag=False, lib=lib) == _bf16(own)).all()
    ca, sa = o.quantize_f32(own, B)
    assert (o.reduce_semi_loop(parts, B, quantize_ag=True, lib=lib) == o.dequantize_bf16(ca, sa, B)).all()
    # one device: nothing is sent; two devices: device 1 sends its quantized shard to the owner
    assert (o.reduce_semi_loop(parts[:1], B, False, lib=lib) == parts[0]).all()
    assert (o.reduce_semi_loop(parts[:1], B, True, lib=lib) == o.reduce_chain(parts[:1], B)).all()
    assert (o.reduce_semi_loop(parts[:2], B, True, lib=lib) == o.reduce_chain([parts[1], parts[0]], B)).all()
    # five devices (odd): chains 2 -> 1 -> owner and 3 -> 4 -> owner, the latter added first
    parts5 = _chain_inputs(8, 5, n)
    x5 = [bf16_bits_to_f32(p) for p in parts5]
    c, s = o.quantize_bf16(parts5[3], B)
    t = _fma_exact(*_dq(c, s, B), x5[4])
    c, s = o.quantize_f32(t, B)
    own = _fma_exact(*_dq(c, s, B), x5[0])
    c, s = o.quantize_bf16(parts5[2], B)
    t = _fma_exact(*_dq(c, s, B), x5[1])
    c, s = o.quantize_f32(t, B)
    own = _fma_exact(*_dq(c, s, B), own)
    assert (o.reduce_semi_loop(parts5, B, False, lib=lib) == _bf16(own)).all()
    # seven devices: counter-clockwise 4 -> 5 -> 6 -> owner, clockwise 3 -> 2 -> 1 -> owner
    parts7 = _chain_inputs(10, 7, n)
    x7 = [bf16_bits_to_f32(p) for p in parts7]

    def sent_by(order):
        c, s = o.quantize_bf16(parts7[order[0]], B)
        for i in order[1:]:
            c, s = o.quantize_f32(_fma_exact(*_dq(c, s, B), x7[i]), B)
        return c, s

    own = _fma_exact(*_dq(*sent_by([4, 5, 6]), B), x7[0])
    own = _fma_exact(*_dq(*sent_by([3, 2, 1]), B), own)
    assert (o.reduce_semi_loop(parts7, B, False, lib=lib) == _bf16(own)).all()
    # every partial enters exactly once: exact sum within the accumulated half-steps
    P, n2 = 8, 4096
    parts8 = _chain_inputs(9, P, n2)
    ref = sum(bf16_bits_to_f32(p).astype(np.float64) for p in parts8)
    semi = bf16_bits_to_f32(o.reduce_semi_loop(parts8, B, True, lib=lib)).astype(np.float64)
    assert np.abs(semi - ref).max() < 0.2 and np.abs(semi - ref).max() > 1e-3


def pin_fig7_semi_loop(lib=None):
    """Fig. 7: semi-loop with both stages quantized has MSE 0.001 (8 devices, block 64, N(0,1)), below the
    full loop's 0.0014."""
    g = read_golden("fig7_error.txt")
    P, B = int(g["devices"]), int(g["block"])
    n = 256 * 4096
    parts = _chain_inputs(2024, P, n)
    ref = np.zeros(n, np.float64)
    for p in parts:
        ref += bf16_bits_to_f32(p).astype(np.float64)
    base = bf16_bits_to_f32(_bf16(ref.astype(np.float32))).astype(np.float64)
    semi = bf16_bits_to_f32(o.reduce_semi_loop(parts, B, True, lib=lib)).astype(np.float64)
    mse_semi = float(np.mean((semi - base) ** 2))
    assert g["semi_loop_rs_ag"] / 1.5 <= mse_semi <= g["semi_loop_rs_ag"] * 1.5, mse_semi
    full = bf16_bits_to_f32(o.reduce_chain(parts, B)).astype(np.float64)
    assert mse_semi < float(np.mean((full - base) ** 2))
    return mse_semi


def pin_flat(lib=None):
    """Flat one-shot reduce: one remote = a pinned hop + dequantize; accumulation order and single rounding
    checked exactly on a small case; zero remotes = Q/Dq of the local shard."""
    rng = _rng(91)
    for B, n in ((32, 32 * 7 + 5), (256, 1024)):
        nb = o.num_blocks(n, B)
        local = _bf16(rng.standard_normal(n).astype(np.float32))
        rem = [_bf16(rng.standard_normal(n).astype(np.float32)) for _ in range(3)]
        qs = [o.quantize_bf16(r, B) for r in rem]
        out, co, so = o.reduce_flat(local, [], [], B, lib=lib)
        c0, s0 = o.quantize_bf16(local, B)
        assert (co == c0).all() and (so == s0).all() and (out == o.dequantize_bf16(c0, s0, B)).all()
        out, co, so = o.reduce_flat(local, [qs[0][0]], [qs[0][1]], B, lib=lib)
        ch, sh = o.hop(qs[0][0], qs[0][1], local, B)
        assert (co == ch).all() and (so == sh).all() and (out == o.dequantize_bf16(ch, sh, B)).all()
        acc = bf16_bits_to_f32(local)
        m = min(n, 160)
        acc = acc[:m]
        for c, s in qs:
            q, sc = _dq(c, s, B)
            acc = _fma_exact(q[:m], sc[:m], acc)
        out, co, so = o.reduce_flat(local, [c for c, _ in qs], [s for _, s in qs], B, lib=lib)
        full_blocks = (m // B) * B
        ce, se = o.quantize_f32(acc[:full_blocks], B)
        assert (co[:full_blocks] == ce).all() and (so[: full_blocks // B] == se).all()
        assert (out[:full_blocks] == o.dequantize_bf16(ce, se, B)).all()
        # two quantizations per value instead of P: the error stays within (sum of remote scales + own)/2
        ref = bf16_bits_to_f32(local).astype(np.float64) + sum(bf16_bits_to_f32(r).astype(np.float64) for r in rem)
        bound = (sum(np.repeat(s.astype(np.float64), B)[:n] for _, s in qs) + np.repeat(so.astype(np.float64), B)[:n]) * 0.5
        err = np.abs(bf16_bits_to_f32(out).astype(np.float64) - ref)
        assert (err <= bound * (1 + 2.0 ** -10) + np.abs(ref) * 2.0 ** -8).all()


def pin_ring_order(lib=None):
    """Ring layout: shard k is reduced in the order k+1, k+2, ..., k; with identical partials the order cannot
    matter; with different ones each shard equals the chain run in its own rotated order."""
    B, P = 32, 4
    n = 32 * 10 + 7
    rng = _rng(95)
    same = _bf16(rng.standard_normal(n).astype(np.float32))
    assert (o.reduce_ring([same] * P, B, lib=lib) == o.reduce_chain([same] * P, B)).all()
    assert o.ring_order(4, 0) == [1, 2, 3, 0] and o.ring_order(4, 3) == [0, 1, 2, 3] and o.ring_order(1, 0) == [0]
    bounds = o.shard_bounds(n, B, P)
    assert bounds[0][0] == 0 and bounds[-1][1] == n and all(a[1] == b[0] for a, b in zip(bounds, bounds[1:]))
    assert all(lo % B == 0 for lo, _ in bounds)
    parts = _chain_inputs(96, P, n)
    got = o.reduce_ring(parts, B, lib=lib)
    lo, hi = bounds[3]
    assert (got[lo:hi] == o.reduce_chain([p[lo:hi] for p in parts], B)).all()      # shard 3: natural order
    lo, hi = bounds[1]
    assert (got[lo:hi] == o.reduce_chain([parts[d][lo:hi] for d in (2, 3, 0, 1)], B)).all()


def pin_strided_geometry(lib=None):
    """Sec. 3.2's own geometry: the paper's worked example (a shard of a (512,512) tensor on 4 devices is 64
    chunks of 8x128, gets 1024 scales, block size 64), which element shares a scale with which, and scale and
    codes of single positions computed directly from the definition."""
    g = read_golden("sec32_block_example.txt")
    shard = int(g["tensor_rows"] * g["tensor_cols"] / g["shards"])
    chunk = int(g["chunk_rows"] * g["chunk_cols"])
    chunks = shard // chunk
    assert chunk == o.CHUNK and chunks == g["chunks_per_shard"] == g["block_size"]
    rng = _rng(33)
    x = _bf16(rng.standard_normal(shard).astype(np.float32))
    c, s = o.quantize_bf16_strided(x, chunks, lib=lib)
    assert s.size == g["scales_per_shard"] and c.size == shard
    xf = bf16_bits_to_f32(x)
    # scale j is decided by the 64 entries at position j of every chunk, and by nothing else
    for j in (0, 1, 127, 128, 600, 1023):
        members = xf[j::chunk]
        assert members.size == g["block_size"]
        codes, scale = _expected_block(members)
        assert s[j] == scale and c[j::chunk].tolist() == codes
    big = x.copy()
    big[5 * chunk + 77] = _bf16(np.array([1000.0], np.float32))[0]
    c2, s2 = o.quantize_bf16_strided(big, chunks, lib=lib)
    changed = np.flatnonzero(s2 != s)
    assert changed.tolist() == [77]
    assert (np.flatnonzero(c2 != c) % chunk == 77).all() and c2[5 * chunk + 77] == 127
    # m minishards: block 64/m, 1024 scales each (two minishards of 32 chunks here)
    cm, sm = o.quantize_bf16_strided(x, chunks // 2, lib=lib)
    assert sm.size == 2048
    codes, scale = _expected_block(xf[32 * chunk + 9::chunk])
    assert sm[1024 + 9] == scale and cm[32 * chunk + 9::chunk].tolist() == codes
    # dequantize, hop and chain follow the same element -> scale map
    d = o.dequantize_bf16_strided(c, s, chunks, lib=lib)
    want = _bf16((c.astype(np.float32) * np.tile(s, chunks)).astype(np.float32))
    assert (d == want).all()
    y = _bf16(rng.standard_normal(shard).astype(np.float32))
    ch, sh = o.hop_strided(c, s, y, chunks, lib=lib)
    j = 300
    t = _fma_exact(c[j::chunk].astype(np.float32), np.full(chunks, s[j], np.float32), bf16_bits_to_f32(y)[j::chunk])
    codes, scale = _expected_block(t)
    assert sh[j] == scale and ch[j::chunk].tolist() == codes
    out, wc, ws = o.reduce_chain_strided([x, y], chunks, keep_wire=True, lib=lib)
    assert (wc[0] == c).all() and (ws[0] == s).all() and (wc[1] == ch).all() and (ws[1] == sh).all()
    assert (out == o.dequantize_bf16_strided(ch, sh, chunks, lib=lib)).all()
    # the two transpositions are inverse permutations
    idx = np.arange(shard)
    assert (o.from_block_major(o.to_block_major(idx, chunks), chunks) == idx).all()
    assert o.to_block_major(idx, chunks)[:3].tolist() == [0, 1024, 2048]


ALL_PINS += [pin_stage_knobs, pin_semi_loop, pin_fig7_semi_loop, pin_flat, pin_ring_order, pin_strided_geometry]


def pin_ring_variants(lib=None):
    """Ring layout combined with the semi-loop and with the stage knobs (Sec. 3, 3.3, 3.4).  Shard k ends on
    device k.  Semi-loop: device k owns shard k and the devices k+1, k+2, k+3 sit around it, so the paper's
    4-device example (device 3 sends to the owner; device 2 sends to device 1, which sends to the owner) is
    written out once per shard with the device numbers rotated by hand.  Stage knobs: every shard equals the
    pinned full-loop flavour run on the partials in that shard's own order, the orders spelled out."""
    B, P = 64, 4
    n = 64 * 7 + 20                                     # 8 blocks, 2 per shard, the last one ragged
    parts = _chain_inputs(97, P, n)
    x = [bf16_bits_to_f32(p) for p in parts]
    bounds = [(0, 128), (128, 256), (256, 384), (384, n)]
    around = {0: (1, 2, 3), 1: (2, 3, 0), 2: (3, 0, 1), 3: (0, 1, 2)}       # owner -> the devices after it on the ring
    semi_plain = o.reduce_ring(parts, B, semi=True, quantize_ag=False, lib=lib)
    semi_ag = o.reduce_ring(parts, B, semi=True, quantize_ag=True, lib=lib)
    for k, (lo, hi) in enumerate(bounds):
        d1, d2, d3 = around[k]
        # the device before the owner sends its shard straight to it; it arrives first and is added first
        c, s = o.quantize_bf16(parts[d3][lo:hi], B)
        own = _fma_exact(*_dq(c, s, B), x[k][lo:hi])
        # the device opposite the owner sends to the device after the owner, which adds its own and forwards
        c, s = o.quantize_bf16(parts[d2][lo:hi], B)
        t = _fma_exact(*_dq(c, s, B), x[d1][lo:hi])
        c, s = o.quantize_f32(t, B)
        own = _fma_exact(*_dq(c, s, B), own)
        assert (semi_plain[lo:hi] == _bf16(own)).all(), k
        c, s = o.quantize_f32(own, B)
        assert (semi_ag[lo:hi] == o.dequantize_bf16(c, s, B)).all(), k
    # the knobs reach every shard: each equals the pinned flavour on that shard's rotated inputs
    chain_of = {0: (1, 2, 3, 0), 1: (2, 3, 0, 1), 2: (3, 0, 1, 2), 3: (0, 1, 2, 3)}     # full loop: k+1, ..., k
    both = o.reduce_ring(parts, B, lib=lib)
    for rs, ag in ((True, False), (False, True)):
        got = o.reduce_ring(parts, B, quantize_rs=rs, quantize_ag=ag, lib=lib)
        assert (got != both).any()
        for k, (lo, hi) in enumerate(bounds):
            want = o.reduce_stages([parts[d][lo:hi] for d in chain_of[k]], B, rs, ag)
            assert (got[lo:hi] == want).all(), (rs, ag, k)
    # reduce-scatter only, checked without reduce_stages on one shard: the wire that reaches device 2 is the
    # pinned chain over devices 3, 0, 1; device 2 adds its own shard with one rounding and narrows
    lo, hi = bounds[2]
    _, wc, ws = o.reduce_chain([parts[d][lo:hi] for d in (3, 0, 1)], B, keep_wire=True)
    t = _fma_exact(*_dq(wc[-1], ws[-1], B), x[2][lo:hi])
    assert (o.reduce_ring(parts, B, quantize_ag=False, lib=lib)[lo:hi] == _bf16(t)).all()
    # an odd ring and one that is longer than the tensor has blocks (empty shards at the end)
    P5, n5 = 5, 32 * 3
    parts5 = _chain_inputs(98, P5, n5)
    got = o.reduce_ring(parts5, 32, semi=True, lib=lib)
    for k, order in enumerate(((0, 1, 2, 3, 4), (1, 2, 3, 4, 0), (2, 3, 4, 0, 1))):
        lo, hi = 32 * k, 32 * (k + 1)
        assert (got[lo:hi] == o.reduce_semi_loop([parts5[d][lo:hi] for d in order], 32, True)).all(), k


ALL_PINS += [pin_ring_variants]


def pin_strided_variants(lib=None):
    """The flavours of Sec. 3.3 / 3.4 in the paper's own block geometry (Sec. 3.2): the elements at one position of
    every chunk of a minishard form one block, so gathering them with a plain stride and running the pinned
    contiguous flavour on that single block must give the strided result at exactly those elements -- for every
    knob setting and the semi-loop, at positions in different minishards.  And the paper's Fig. 7 error figures
    hold in its own geometry too (i.i.d. values: the statistics do not depend on which elements share a scale)."""
    chunks, P = 32, 5
    n = 2 * o.CHUNK * chunks
    parts = _chain_inputs(131, P, n, heavy=True)
    got = {
        (True, True): o.reduce_stages_strided(parts, chunks, True, True, lib=lib),
        (True, False): o.reduce_stages_strided(parts, chunks, True, False, lib=lib),
        (False, True): o.reduce_stages_strided(parts, chunks, False, True, lib=lib),
        (False, False): o.reduce_stages_strided(parts, chunks, False, False, lib=lib),
    }
    semi = {ag: o.reduce_semi_loop_strided(parts, chunks, ag, lib=lib) for ag in (True, False)}
    assert (got[(True, True)] == o.reduce_chain_strided(parts, chunks)).all()
    assert len({g.tobytes() for g in got.values()} | {g.tobytes() for g in semi.values()}) == 6      # all different
    for m, j in ((0, 0), (0, 517), (0, 1023), (1, 1), (1, 640)):
        idx = m * o.CHUNK * chunks + np.arange(chunks) * o.CHUNK + j
        block = [p[idx] for p in parts]
        for (rs, ag), g in got.items():
            assert (g[idx] == o.reduce_stages(block, chunks, rs, ag)).all(), (m, j, rs, ag)
        for ag, g in semi.items():
            assert (g[idx] == o.reduce_semi_loop(block, chunks, ag)).all(), (m, j, ag)
    # Fig. 7 in the paper's own geometry: 8 devices, block 64 = 64 chunks, N(0,1)
    gold = read_golden("fig7_error.txt")
    P8, B = int(gold["devices"]), int(gold["block"])
    n8 = 4 * o.CHUNK * B
    parts8 = _chain_inputs(2025, P8, n8)
    ref = np.zeros(n8, np.float64)
    for p in parts8:
        ref += bf16_bits_to_f32(p).astype(np.float64)
    base = bf16_bits_to_f32(_bf16(ref.astype(np.float32))).astype(np.float64)
    mse = lambda out: float(np.mean((bf16_bits_to_f32(out).astype(np.float64) - base) ** 2))
    full = mse(o.reduce_stages_strided(parts8, B, True, True, lib=lib))
    semi8 = mse(o.reduce_semi_loop_strided(parts8, B, True, lib=lib))
    ag_only = mse(o.reduce_stages_strided(parts8, B, False, True, lib=lib))
    assert gold["full_loop_rs_ag"] / 1.5 <= full <= gold["full_loop_rs_ag"] * 1.5, full
    assert gold["semi_loop_rs_ag"] / 1.5 <= semi8 <= gold["semi_loop_rs_ag"] * 1.5, semi8
    assert gold["full_loop_ag_only"] / 1.5 <= ag_only <= gold["full_loop_ag_only"] * 1.5, ag_only
    assert ag_only < semi8 < full


ALL_PINS += [pin_strided_variants]


def pin_ring_strided(lib=None):
    """Ring layout with strided blocks (Sec. 3 with Sec. 3.2): shards are whole minishards and shard k ends on
    device k.  Three devices, four minishards, so two per shard and an empty third shard; the minishard ranges and
    every shard's device order are spelled out by hand and fed to the pinned strided flavours.  Identical
    partials make the order irrelevant.  One position of one shard is also taken through the pinned CONTIGUOUS
    chain on a plain strided gather in that shard's order, so neither the shard rule nor the order rests on a
    strided function."""
    chunks, P = 32, 3
    ms = o.CHUNK * chunks
    n = 4 * ms
    parts = _chain_inputs(141, P, n, heavy=True)
    shards = [(0, 2 * ms, (1, 2, 0), (0, 1, 2)), (2 * ms, 4 * ms, (2, 0, 1), (1, 2, 0))]     # lo, hi, full-loop order, owner first
    plain = o.reduce_stages_strided(parts, chunks, lib=lib)
    seen = set()
    for rs, ag in ((True, True), (True, False), (False, True)):
        got = o.reduce_ring_strided(parts, chunks, quantize_rs=rs, quantize_ag=ag, lib=lib)
        seen.add(got.tobytes())
        for lo, hi, chain, _ in shards:
            want = o.reduce_stages_strided([parts[d][lo:hi] for d in chain], chunks, rs, ag)
            assert (got[lo:hi] == want).all(), (rs, ag, lo)
    for ag in (True, False):
        got = o.reduce_ring_strided(parts, chunks, semi=True, quantize_ag=ag, lib=lib)
        seen.add(got.tobytes())
        for lo, hi, _, around in shards:
            want = o.reduce_semi_loop_strided([parts[d][lo:hi] for d in around], chunks, ag)
            assert (got[lo:hi] == want).all(), (ag, lo)
    assert len(seen) == 5 and plain.tobytes() not in seen              # the rotation matters for every flavour
    # one strided block of shard 1 (minishard 3, position 700) through the contiguous chain in the order 2, 0, 1
    idx = 3 * ms + np.arange(chunks) * o.CHUNK + 700
    got = o.reduce_ring_strided(parts, chunks, lib=lib)
    assert (got[idx] == o.reduce_chain([parts[d][idx] for d in (2, 0, 1)], chunks)).all()
    same = [parts[0]] * P
    assert (o.reduce_ring_strided(same, chunks, lib=lib) == o.reduce_stages_strided(same, chunks)).all()
    # a ring longer than the tensor has minishards: shards 0 and 1 hold one each, the rest are empty
    P5 = 5
    parts5 = _chain_inputs(142, P5, 2 * ms)
    got = o.reduce_ring_strided(parts5, chunks, semi=True, lib=lib)
    for k, around in enumerate(((0, 1, 2, 3, 4), (1, 2, 3, 4, 0))):
        lo, hi = k * ms, (k + 1) * ms
        assert (got[lo:hi] == o.reduce_semi_loop_strided([parts5[d][lo:hi] for d in around], chunks, True)).all(), k


ALL_PINS += [pin_ring_strided]

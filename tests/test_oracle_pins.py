"""Pins of the CPU oracle to things outside it (no GPU needed).

Each test fixes the oracle to a value or property that the paper or plain
mathematics dictates: hand-derived values of Eq. 2, the scale/2 error bound,
lossless grids, textbook softmax attention from a library routine (window-only
and lossless caches), permutation invariance of Eq. 1, closed forms, and the
average-bit figures the paper prints.
"""
import os

import numpy as np
import pytest
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
D = 128


# ----------------------------------------------------------------- fp16 ----

def test_half_to_float_all_bit_patterns(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float32)
    got = np.array([oracle.half_to_float(int(b)) for b in bits], np.float32)
    fin = np.isfinite(want)
    assert np.array_equal(got[fin].view(np.uint32), want[fin].view(np.uint32))
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(np.isinf(got), np.isinf(want))


def test_float_to_half_rounds_to_nearest_even(oracle):
    rng = np.random.default_rng(5)
    xs = np.concatenate([
        rng.standard_normal(20000).astype(np.float32) * 10.0 ** rng.uniform(-9, 5, 20000).astype(np.float32),
        # exact ties between neighbouring fp16 values, normal and subnormal
        np.array([1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 2.0 ** -25, 3 * 2.0 ** -25, 65519.9, 65520.0,
                  2.0 ** -14 - 2.0 ** -25, 0.0, -0.0, 1e-9], np.float32)])
    with np.errstate(over="ignore"):
        want = xs.astype(np.float16).view(np.uint16)
    got = np.array([oracle.float_to_half(float(x)) for x in xs], np.uint16)
    assert np.array_equal(got, want)


# -------------------------------------------------------- Eq. 2 encoder ----

def test_encoder_hand_derived_values(oracle):
    # Eq. 2 by hand, N = 2: x = [-1, 0, 1, 2], alpha = 1 -> h = 3/3 = 1, alpha*min = -1.
    c, h, z = oracle.encode_group(np.array([-1, 0, 1, 2], np.float32), 1.0, 4)
    assert list(c) == [0, 1, 2, 3] and h == 1.0 and z == -1.0
    # alpha = 0.5 -> range [-0.5, 1], h = 0.5, (x + 0.5)/0.5 = [-1, 1, 3, 5] -> clamp to [0, 1, 3, 3].
    c, h, z = oracle.encode_group(np.array([-1, 0, 1, 2], np.float32), 0.5, 4)
    assert list(c) == [0, 1, 3, 3] and h == 0.5 and z == -0.5
    # ties: h = 1, zero = 0, (x - z)/h = x ; 0.5 -> 0, 1.5 -> 2, 2.5 -> 2 (ties to even)
    c, h, z = oracle.encode_group(np.array([0, 0.5, 1.5, 2.5, 3], np.float32), 1.0, 4)
    assert list(c) == [0, 0, 2, 2, 3] and h == 1.0 and z == 0.0
    # three levels ("1.5-bit" reading): top code 2, h = (2 - 0)/2 = 1
    c, h, z = oracle.encode_group(np.array([0, 0.5, 1, 1.5, 2], np.float32), 1.0, 3)
    assert list(c) == [0, 0, 1, 2, 2] and h == 1.0 and z == 0.0
    # N = 4: sixteen levels, h = (15 - 0)/15 = 1; 7.5 and 8.5 both tie to 8; alpha = 0.5 clamps the top half
    c, h, z = oracle.encode_group(np.array([0, 7.5, 8.5, 11, 15], np.float32), 1.0, 16)
    assert list(c) == [0, 8, 8, 11, 15] and h == 1.0 and z == 0.0
    c, h, z = oracle.encode_group(np.array([0, 1.25, 6, 15, 30], np.float32), 0.5, 16)
    assert h == 1.0 and z == 0.0 and list(c) == [0, 1, 6, 15, 15]
    # N = 3: eight levels, h = (7 - 0)/7 = 1; 2.5 ties down to 2, 3.5 up to 4
    c, h, z = oracle.encode_group(np.array([0, 2.5, 3.5, 6.4, 7], np.float32), 1.0, 8)
    assert list(c) == [0, 2, 4, 6, 7] and h == 1.0 and z == 0.0
    # both ends are scaled by alpha (Eq. 2 and Algorithm 1 agree): all-positive group
    c, h, z = oracle.encode_group(np.array([4, 8, 16], np.float32), 0.5, 4)
    assert z == 2.0 and h == (8.0 - 2.0) / 3 and list(c) == [1, 3, 3]


def test_encoder_divides_by_multiplying_with_the_rounded_reciprocal(oracle):
    """Reading of Eq. 2's division (X - z)/h: t = (x - z) * fl(1/h), one fp32 reciprocal per group and one
    fp32 multiply per value -- not an fp32 division per value.  The two differ on rare ties; groups worked
    out by hand where they do:
      2-bit, alpha = 1, group {0, 37.5, 45}: z = 0, h = 45/3 = 15.  Exact quotient of 37.5: 2.5, a tie, which
        a division would round to the even code 2.  fl(1/15) = 0x3D888889 = 0.0666666701436..., above 1/15 by
        5.2e-8 relative; 37.5 * fl(1/15) = 2.50000013..., more than half an ulp (1.19e-7) above 2.5, so the fp32
        product is 2.5 + 2^-22 and rounds to code 3.
      4-bit, alpha = 1, group {0, 45.5, 105}: h = 105/15 = 7; exact quotient 6.5 (division: code 6);
        fl(1/7) = 0x3E124925 is 4.5e-8 relative above 1/7, the product 6.50000029... rounds to 6.5 + 2^-21: code 7."""
    f32 = np.float32
    inv15 = f32(1) / f32(15)
    assert inv15.view(np.uint32) == 0x3D888889 and float(f32(37.5) * inv15) == 2.5 + 2.0 ** -22
    assert float(f32(37.5) / f32(15)) == 2.5                       # what a per-value division would see
    c, h, z = oracle.encode_group(np.array([0, 37.5, 45], np.float32), 1.0, 4)
    assert h == 15.0 and z == 0.0 and list(c) == [0, 3, 3]
    inv7 = f32(1) / f32(7)
    assert inv7.view(np.uint32) == 0x3E124925 and float(f32(45.5) * inv7) == 6.5 + 2.0 ** -21
    c, h, z = oracle.encode_group(np.array([0, 45.5, 105], np.float32), 1.0, 16)
    assert h == 7.0 and z == 0.0 and list(c) == [0, 7, 15]
    # the same groups scaled by a power of two (exact in every step): same codes
    c, h, z = oracle.encode_group(np.array([0, 37.5, 45], np.float32) / 64, 1.0, 4)
    assert h == 15.0 / 64 and list(c) == [0, 3, 3]


@pytest.mark.parametrize("levels", [4, 3, 16, 8])
def test_encoder_error_bound_and_clipping(oracle, levels):
    rng = np.random.default_rng(11 + levels)
    top = levels - 1
    for trial in range(200):
        n = int(rng.choice([4, 32, 64, 128]))
        x = (rng.standard_normal(n) * 10.0 ** rng.uniform(-2, 1.5)).astype(np.float16).astype(np.float32)
        alpha = float(np.float32(rng.choice([1.0, 0.95, 0.8, 0.5])))
        c, h, z = oracle.encode_group(x, alpha, levels)
        lo, hi = np.float64(z), np.float64(z) + top * np.float64(h)
        deq = c.astype(np.float64) * np.float64(h) + np.float64(z)
        assert c.min() >= 0 and c.max() <= top
        inside = (x >= lo) & (x <= hi)
        assert np.all(np.abs(x[inside] - deq[inside]) <= 0.5 * h * (1 + 1e-5) + 1e-30)
        assert np.all(c[x < lo] == 0) and np.all(c[x > hi + 1e-6 * abs(hi)] == top)
        # zero and scale are exactly what Eq. 2 prescribes, evaluated in fp32
        a32 = np.float32(alpha)
        assert z == a32 * x.min()
        assert h == np.float32(np.float32(a32 * x.max()) - np.float32(a32 * x.min())) / np.float32(top)


@pytest.mark.parametrize("levels", [4, 3, 16, 8])
def test_encoder_picks_the_nearest_level(oracle, levels):
    """Brute force: among all codes the chosen one is nearest to x (exact arithmetic)."""
    rng = np.random.default_rng(23 + levels)
    for trial in range(100):
        x = rng.standard_normal(16).astype(np.float16).astype(np.float32)
        c, h, z = oracle.encode_group(x, 0.9, levels)
        grid = np.float64(z) + np.arange(levels)[None, :] * np.float64(h)
        dist = np.abs(x.astype(np.float64)[:, None] - grid)
        best = dist.min(axis=1)
        chosen = dist[np.arange(16), c]
        assert np.all(chosen <= best + 1e-6 * h)


@pytest.mark.parametrize("levels", [4, 3, 16, 8])
def test_encoder_lossless_on_a_grid_and_power_of_two_scaling(oracle, levels):
    rng = np.random.default_rng(31 + levels)
    top = levels - 1
    for trial in range(50):
        step = 2.0 ** int(rng.integers(-6, 4))
        base = step * int(rng.integers(-40, 40))
        k = rng.integers(0, levels, 32)
        k[0], k[1] = 0, top
        x = (base + step * k).astype(np.float32)
        c, h, z = oracle.encode_group(x, 1.0, levels)
        assert h == step and z == base and np.array_equal(c, k)
        c2, h2, z2 = oracle.encode_group(x * 8.0, 1.0, levels)
        assert np.array_equal(c2, c) and h2 == 8 * h and z2 == 8 * z
    # lossy data too: multiplying by a power of two scales scale and zero exactly, codes unchanged
    x = rng.standard_normal(128).astype(np.float16).astype(np.float32)
    c, h, z = oracle.encode_group(x, 0.95, levels)
    c2, h2, z2 = oracle.encode_group(x * 0.25, 0.95, levels)
    assert np.array_equal(c, c2) and h2 == np.float32(0.25) * h and z2 == np.float32(0.25) * z


def test_encoder_degenerate_groups(oracle):
    c, h, z = oracle.encode_group(np.full(8, 3.0, np.float32), 0.5, 4)
    assert h == 0.0 and z == 1.5 and not c.any()          # decodes to alpha*min, the formula's own value
    c, h, z = oracle.encode_group(np.array([-0.0, 0.0, -0.0], np.float32), 1.0, 4)
    assert h == 0.0 and np.float32(z).view(np.uint32) == 0  # one bit pattern for a zero minimum
    c, h, z = oracle.encode_group(np.array([-0.0, 1.0], np.float32), 1.0, 3)
    assert np.float32(z).view(np.uint32) == 0 and h == 0.5 and list(c) == [0, 2]


# ----------------------------------------------------- paper's avg bits ----

def test_average_bits_match_the_paper(oracle):
    rows = 0
    for line in open(os.path.join(HERE, "golden", "avg_bits.txt")):
        line = line.split("#")[0].split()
        if not line:
            continue
        cb, mb, g, want = float(line[0]), int(line[1]), int(line[2]), float(line[3])
        assert oracle.avg_bits(cb, mb, g) == pytest.approx(want, abs=1e-12)
        rows += 1
    assert rows == 8


# -------------------------------------------------------------- formats ----

def test_k_row_layout_is_position_p_at_bit_2p(oracle):
    for p in range(D):
        row = np.zeros(32, np.uint8)
        oracle.lib().skvq_ref_k_put(row.ctypes.data, 4, p, 3)
        assert int.from_bytes(row.tobytes(), "little") == 3 << (2 * p)
        assert oracle.lib().skvq_ref_k_get(row.ctypes.data, 4, p) == 3
    rng = np.random.default_rng(3)
    row = rng.integers(0, 256, 32, dtype=np.uint8)
    big = int.from_bytes(row.tobytes(), "little")
    assert [oracle.lib().skvq_ref_k_get(row.ctypes.data, 4, p) for p in range(D)] == \
           [(big >> (2 * p)) & 3 for p in range(D)]


def test_k_row_4bit_layout_is_position_p_at_bit_4p(oracle):
    for p in range(D):
        row = np.zeros(64, np.uint8)
        oracle.lib().skvq_ref_k_put(row.ctypes.data, 16, p, 15)
        assert int.from_bytes(row.tobytes(), "little") == 15 << (4 * p)
        oracle.lib().skvq_ref_k_put(row.ctypes.data, 16, p, 9)      # overwrite, not OR
        assert int.from_bytes(row.tobytes(), "little") == 9 << (4 * p)
        assert oracle.lib().skvq_ref_k_get(row.ctypes.data, 16, p) == 9
    rng = np.random.default_rng(5)
    row = rng.integers(0, 256, 64, dtype=np.uint8)
    big = int.from_bytes(row.tobytes(), "little")
    assert [oracle.lib().skvq_ref_k_get(row.ctypes.data, 16, p) for p in range(D)] == \
           [(big >> (4 * p)) & 15 for p in range(D)]


KSIG = [[0, 2, 1, 3, 4, 6, 8, 5], [7, 9, 10, 12, 11, 13, 15, 14]]      # the format statement's tables
VTAU = [[0, 2, 4, 12], [1, 3, 5, 13], [6, 8, 10, 14], [7, 9, 11, 15]]


def test_k_row_3bit_layout_is_a_2bit_row_plus_a_top_bit_plane(oracle):
    seen = 0
    for p in range(D):
        row = np.zeros(48, np.uint8)
        oracle.lib().skvq_ref_k_put(row.ctypes.data, 8, p, 7)
        big = int.from_bytes(row.tobytes(), "little")
        top = 256 + 32 * (p // 32) + 16 * ((p % 16) // 8) + KSIG[(p % 32) // 16][p % 8]
        assert big == (3 << (2 * p)) | (1 << top) and not (big & seen)
        seen |= big
        oracle.lib().skvq_ref_k_put(row.ctypes.data, 8, p, 4)       # overwrite: only the top bit stays
        assert int.from_bytes(row.tobytes(), "little") == 1 << top
        assert oracle.lib().skvq_ref_k_get(row.ctypes.data, 8, p) == 4
    assert seen == (1 << 384) - 1
    rng = np.random.default_rng(7)
    codes = rng.integers(0, 8, D)
    row = np.zeros(48, np.uint8)
    for p in range(D):
        oracle.lib().skvq_ref_k_put(row.ctypes.data, 8, p, int(codes[p]))
    assert [oracle.lib().skvq_ref_k_get(row.ctypes.data, 8, p) for p in range(D)] == list(codes)
    # the first 32 bytes are the 2-bit row of the low two bits
    two = np.zeros(32, np.uint8)
    for p in range(D):
        oracle.lib().skvq_ref_k_put(two.ctypes.data, 4, p, int(codes[p]) & 3)
    assert np.array_equal(row[:32], two)


def test_v_block_3bit_layout_is_a_2bit_unit_plus_a_top_bit_plane(oracle):
    seen = 0
    for s_ in range(32):
        for p in range(D):
            blk = np.zeros(1536, np.uint8)
            oracle.lib().skvq_ref_v_put(blk.ctypes.data, 8, s_, p, 7)
            big = int.from_bytes(blk.tobytes(), "little")
            u, n, i = 16 * (s_ // 8) + p % 16, p // 16, s_ % 8
            low = 32 * (n // 2) + 16 * (i % 2) + 8 * (n % 2) + 2 * (i // 2)
            top = 128 + 32 * (n // 4) + 16 * (i % 2) + VTAU[n % 4][i // 2]
            assert big == ((3 << low) | (1 << top)) << (192 * u) and not (big & seen)
            seen |= big
            assert oracle.lib().skvq_ref_v_get(blk.ctypes.data, 8, s_, p) == 7
    assert seen == (1 << (1536 * 8)) - 1
    rng = np.random.default_rng(8)
    codes = rng.integers(0, 8, (32, D))
    blk = np.zeros(1536, np.uint8)
    for s_ in range(32):
        for p in range(D):
            oracle.lib().skvq_ref_v_put(blk.ctypes.data, 8, s_, p, int(codes[s_, p]))
    got = [[oracle.lib().skvq_ref_v_get(blk.ctypes.data, 8, s_, p) for p in range(D)] for s_ in range(32)]
    assert np.array_equal(np.array(got), codes)


def test_v_block_4bit_layout_is_a_bijection_with_token_neighbours(oracle):
    seen = 0
    for s in range(32):
        for p in range(D):
            blk = np.zeros(2048, np.uint8)
            oracle.lib().skvq_ref_v_put(blk.ctypes.data, 16, s, p, 15)
            big = int.from_bytes(blk.tobytes(), "little")
            assert bin(big).count("1") == 4 and not (big & seen)
            seen |= big
            # unit u = 16*(s/8) + p%16 of 32 bytes, one dword per n = p/16; tokens 2m and 2m+1
            # sit 16 bits apart in it
            u, n, i = 16 * (s // 8) + p % 16, p // 16, s % 8
            assert big == 15 << (256 * u + 32 * n + 16 * (i % 2) + 4 * (i // 2))
            assert oracle.lib().skvq_ref_v_get(blk.ctypes.data, 16, s, p) == 15
    assert seen == (1 << 16384) - 1
    rng = np.random.default_rng(6)
    codes = rng.integers(0, 16, (32, D))
    blk = np.zeros(2048, np.uint8)
    for s in range(32):
        for p in range(D):
            oracle.lib().skvq_ref_v_put(blk.ctypes.data, 16, s, p, int(codes[s, p]))
    got = [[oracle.lib().skvq_ref_v_get(blk.ctypes.data, 16, s, p) for p in range(D)] for s in range(32)]
    assert np.array_equal(np.array(got), codes)


def test_v_block_2bit_layout_is_a_bijection_with_token_neighbours(oracle):
    seen = 0
    for s in range(32):
        for p in range(D):
            blk = np.zeros(1024, np.uint8)
            oracle.lib().skvq_ref_v_put(blk.ctypes.data, 4, s, p, 3)
            big = int.from_bytes(blk.tobytes(), "little")
            assert bin(big).count("1") == 2 and not (big & seen)
            seen |= big
            # unit u = 16*(s/8) + p%16 of 16 bytes; tokens 2m and 2m+1 sit 16 bits apart in one dword
            u, n, i = 16 * (s // 8) + p % 16, p // 16, s % 8
            assert big == 3 << (128 * u + 32 * (n // 2) + 16 * (i % 2) + 8 * (n % 2) + 2 * (i // 2))
    assert seen == (1 << 8192) - 1


def test_v_block_ternary_fields_are_base3_numbers(oracle):
    rng = np.random.default_rng(4)
    codes = rng.integers(0, 3, (32, D))
    blk = np.full(832, 0, np.uint8)
    for s in range(32):
        for p in range(D):
            oracle.lib().skvq_ref_v_put(blk.ctypes.data, 3, s, p, int(codes[s, p]))
    for u in range(64):
        unit = int.from_bytes(blk[13 * u:13 * u + 13].tobytes(), "little")
        kb, j = u // 16, u % 16
        for n in range(8):
            f = (unit >> (13 * n)) & 0x1FFF
            assert f < 3 ** 8
            assert f == sum(int(codes[8 * kb + i, 16 * n + j]) * 3 ** i for i in range(8))
    got = [[oracle.lib().skvq_ref_v_get(blk.ctypes.data, 3, s, p) for p in range(D)] for s in range(32)]
    assert np.array_equal(np.array(got), codes)
    # overwriting one code leaves every other code alone
    oracle.lib().skvq_ref_v_put(blk.ctypes.data, 3, 5, 77, (int(codes[5, 77]) + 1) % 3)
    got2 = np.array([[oracle.lib().skvq_ref_v_get(blk.ctypes.data, 3, s, p) for p in range(D)] for s in range(32)])
    assert (got2 != codes).sum() == 1


def test_bytes_per_token_match_the_byte_model(oracle):
    perm = np.tile(np.arange(D, dtype=np.int32), (8, 1))
    clip = np.ones((8, 1), np.float32)
    c = oracle.OracleCache(1, 32, 8, 128, 1.5, 128, 4096, perm, perm, clip, clip)
    per_token = sum(c.sizes[:4]) / (8 * 4096)
    assert per_token == 32 + 26 + 8 + 8       # 2-bit K row, 13 bits per 8 values for V, fp32 scale+zero each
    assert c.sizes[4] == 8 * 128 * 128 * 2
    c2 = oracle.OracleCache(1, 32, 8, 32, 2.0, 128, 4096, perm, perm, np.ones((8, 4), np.float32),
                            np.ones((8, 4), np.float32))
    assert sum(c2.sizes[:4]) / (8 * 4096) == 32 + 32 + 32 + 32
    # 4-bit keys and values, group 64, FP8 (scale, zero): Table 1's 4.25 average bits
    two = np.ones((8, 2), np.float32)
    c3 = oracle.OracleCache(1, 32, 8, 64, 4.0, 128, 4096, perm, perm, two, two, k_bits=4.0, meta="e4m3")
    assert sum(c3.sizes[:4]) / (8 * 4096) == 64 + 64 + 4 + 4
    assert sum(c3.sizes[:4]) * 8 / (8 * 4096 * 2 * D) == 4.25
    # 3-bit, same setting: Table 1's 3.25
    c4 = oracle.OracleCache(1, 32, 8, 64, 3.0, 128, 4096, perm, perm, two, two, k_bits=3.0, meta="e4m3")
    assert sum(c4.sizes[:4]) / (8 * 4096) == 48 + 48 + 4 + 4
    assert sum(c4.sizes[:4]) * 8 / (8 * 4096 * 2 * D) == 3.25


# ------------------------------------------------------------ attention ----

def sdpa64(q, k, v, sm_scale):
    """Textbook softmax attention from the library, fp64, GQA by repeating kv heads.
    q [B][Hq][D], k/v [B][Hk][T][D] -> [B][Hq][D]."""
    qt = torch.from_numpy(q.astype(np.float64))[:, :, None, :]
    rep = q.shape[1] // k.shape[1]
    kt = torch.from_numpy(k.astype(np.float64)).repeat_interleave(rep, dim=1)
    vt = torch.from_numpy(v.astype(np.float64)).repeat_interleave(rep, dim=1)
    o = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, scale=float(sm_scale))
    return o[:, :, 0, :].numpy()


def random_perms(rng, hk):
    return np.stack([rng.permutation(D) for _ in range(hk)]).astype(np.int32)


def grid_data(rng, shape_bht, G, levels, perm):
    """fp16 tensor [B][Hk][T][D] whose every (token, head, group of the REORDERED axis)
    lies on its own `levels`-point grid with a power-of-two step, both end points present."""
    B, Hk, T = shape_bht
    x = np.zeros((B, Hk, T, D), np.float32)
    for b in range(B):
        for h in range(Hk):
            for t in range(T):
                for g in range(D // G):
                    step = 2.0 ** int(rng.integers(-5, 2))
                    base = step * int(rng.integers(-20, 20))
                    k = rng.integers(0, levels, G)
                    k[rng.integers(0, G // 2)] = 0
                    k[G // 2 + rng.integers(0, G // 2)] = levels - 1
                    x[b, h, t, perm[h, g * G:(g + 1) * G]] = base + step * k
    return x.astype(np.float16)


def test_window_only_cache_is_textbook_attention(oracle):
    rng = np.random.default_rng(100)
    B, Hq, Hk, W = 2, 8, 2, 16
    for T in (1, 7, 16):
        k = rng.standard_normal((B, Hk, T, D)).astype(np.float16)
        v = rng.standard_normal((B, Hk, T, D)).astype(np.float16)
        q = rng.standard_normal((B, Hq, D)).astype(np.float16)
        c = oracle.OracleCache(B, Hq, Hk, 128, 1.5, W, 64, random_perms(rng, Hk), random_perms(rng, Hk),
                               np.full((Hk, 1), 0.9, np.float32), np.full((Hk, 1), 0.9, np.float32))
        assert c.prefill(k, v) == 0 and c.n_quant == 0
        out, out16 = c.decode(q, want_f16=True)
        ref = sdpa64(q, k, v, 1 / np.sqrt(D))
        assert np.abs(out - ref).max() < 2e-6
        assert np.array_equal(out16, out.astype(np.float16))
        # the ring holds the tokens bit for bit, token a in slot a % W
        for a in range(T):
            assert np.array_equal(c.k_win[:, :, a % W].view(np.float16), k[:, :, a])
            assert np.array_equal(c.v_win[:, :, a % W].view(np.float16), v[:, :, a])


@pytest.mark.parametrize("k_bits,v_bits,G", [(2.0, 2.0, 128), (2.0, 1.5, 128), (2.0, 1.5, 32), (2.0, 2.0, 64),
                                             (4.0, 4.0, 128), (4.0, 4.0, 32), (4.0, 2.0, 64), (2.0, 4.0, 128),
                                             (3.0, 3.0, 128), (3.0, 3.0, 32)])
def test_lossless_cache_equals_textbook_attention(oracle, k_bits, v_bits, G):
    """Data that Eq. 2 represents exactly (alpha = 1) makes the quantized path exact, so the whole
    chain reorder -> encode -> pack -> unpack -> dequantize -> Eq. 1 must reproduce the library's
    attention on the ORIGINAL tensors, for any permutation (Eq. 1's invariance)."""
    rng = np.random.default_rng(200 + G)
    B, Hq, Hk, W, T = 1, 4, 2, 8, 77
    pk, pv = random_perms(rng, Hk), random_perms(rng, Hk)
    k = grid_data(rng, (B, Hk, T), G, oracle.levels_of(k_bits), pk)
    v = grid_data(rng, (B, Hk, T), G, oracle.levels_of(v_bits), pv)
    q = rng.standard_normal((B, Hq, D)).astype(np.float16)
    ones = np.ones((Hk, D // G), np.float32)
    c = oracle.OracleCache(B, Hq, Hk, G, v_bits, W, 96, pk, pv, ones, ones, sm_scale=0.05, k_bits=k_bits)
    assert c.prefill(k, v) == 0 and c.n_quant == T - W
    out = c.decode(q)
    ref = sdpa64(q, k, v, 0.05)
    assert np.abs(out - ref).max() < 1e-5 * max(1.0, np.abs(ref).max())


def test_permutation_invariance_when_group_is_the_whole_head(oracle):
    """With G = D a permutation only moves codes around (same min/max, same codes), so by
    Eq. 1 the attention output cannot depend on P_k or P_v, lossy data included."""
    rng = np.random.default_rng(300)
    B, Hq, Hk, W, T = 1, 4, 2, 8, 60
    k = rng.standard_normal((B, Hk, T, D)).astype(np.float16)
    v = rng.standard_normal((B, Hk, T, D)).astype(np.float16)
    q = rng.standard_normal((B, Hq, D)).astype(np.float16)
    clip = np.full((Hk, 1), 0.95, np.float32)
    outs = []
    for trial in range(3):
        c = oracle.OracleCache(B, Hq, Hk, 128, 1.5, W, 64, random_perms(rng, Hk), random_perms(rng, Hk),
                               clip, clip)
        c.prefill(k, v)
        outs.append(c.decode(q))
    assert np.abs(outs[0] - outs[1]).max() < 1e-6 and np.abs(outs[0] - outs[2]).max() < 1e-6


def numpy_dequantize(c, T):
    """Independent unpack + dequantize of an OracleCache's packed rows, straight from the
    format statement, vectorised; returns K', V' float64 [B][Hk][nq][D] in ORIGINAL channel order."""
    B, Hk = c.k_codes.shape[:2]
    nq = max(T - c.window, 0)
    G = c.cfg.group_size
    kq = np.zeros((B, Hk, nq, D))
    vq = np.zeros((B, Hk, nq, D))
    p = np.arange(D)
    bounds = getattr(c, "group_bounds", None)       # None or [Hk][D/G + 1]
    gof = np.stack([p // G if bounds is None else np.searchsorted(np.asarray(bounds[h]), p, side="right") - 1
                    for h in range(Hk)])             # [Hk][D]: group of position p of head h
    if c.cfg.k_levels == 16:
        kc = (c.k_codes[:, :, :nq, p // 2] >> (4 * (p % 2))) & 15
    elif c.cfg.k_levels == 8:
        top = np.array([256 + 32 * (x // 32) + 16 * ((x % 16) // 8) + KSIG[(x % 32) // 16][x % 8] for x in range(D)])
        kc = ((c.k_codes[:, :, :nq, p // 4] >> (2 * (p % 4))) & 3) + 4 * ((c.k_codes[:, :, :nq, top // 8] >> (top % 8)) & 1)
    else:
        kc = (c.k_codes[:, :, :nq, p // 4] >> (2 * (p % 4))) & 3
    def per_position(meta, x):      # [B][Hk][nq][D]: the group's value for every position
        return np.stack([meta[:, h, :nq][:, :, gof[h], x] for h in range(Hk)], axis=1).astype(np.float64)
    ks, kz = per_position(c.k_meta, 0), per_position(c.k_meta, 1)
    kd = kc * ks + kz
    vs, vz = per_position(c.v_meta, 0), per_position(c.v_meta, 1)
    vc = np.zeros((B, Hk, nq, D), np.int64)
    for b in range(B):
        for h in range(Hk):
            for t in range(nq):
                blk = c.v_codes[b, h, t // 32]
                s = t % 32
                for pp in range(D):
                    u, n, i = 16 * (s // 8) + pp % 16, pp // 16, s % 8
                    if c.cfg.v_levels == 3:
                        unit = int.from_bytes(blk[13 * u:13 * u + 13].tobytes(), "little")
                        vc[b, h, t, pp] = ((unit >> (13 * n)) & 0x1FFF) // 3 ** i % 3
                    elif c.cfg.v_levels == 8:
                        unit = int.from_bytes(blk[24 * u:24 * u + 24].tobytes(), "little")
                        low = (unit >> (32 * (n // 2) + 16 * (i % 2) + 8 * (n % 2) + 2 * (i // 2))) & 3
                        top = (unit >> (128 + 32 * (n // 4) + 16 * (i % 2) + VTAU[n % 4][i // 2])) & 1
                        vc[b, h, t, pp] = low + 4 * top
                    elif c.cfg.v_levels == 16:
                        word = int.from_bytes(blk[32 * u + 4 * n:32 * u + 4 * n + 4].tobytes(), "little")
                        vc[b, h, t, pp] = (word >> (16 * (i % 2) + 4 * (i // 2))) & 15
                    else:
                        unit = int.from_bytes(blk[16 * u:16 * u + 16].tobytes(), "little")
                        vc[b, h, t, pp] = (unit >> (32 * (n // 2) + 16 * (i % 2) + 8 * (n % 2) + 2 * (i // 2))) & 3
    vd = vc * vs + vz
    for h in range(Hk):
        kq[:, h][..., c.perm_k[h]] = kd[:, h]      # position p holds channel perm[p]
        vq[:, h][..., c.perm_v[h]] = vd[:, h]
    return kq, vq


@pytest.mark.parametrize("k_bits,v_bits,G", [(2.0, 1.5, 128), (2.0, 2.0, 32), (2.0, 1.5, 64), (4.0, 4.0, 128),
                                             (4.0, 4.0, 32), (4.0, 2.0, 64), (3.0, 3.0, 128), (3.0, 3.0, 64)])
def test_lossy_cache_equals_dequantize_then_textbook_attention(oracle, k_bits, v_bits, G):
    rng = np.random.default_rng(400 + G)
    B, Hq, Hk, W, T = 2, 4, 2, 8, 45
    k = (rng.standard_normal((B, Hk, T, D)) * 10 ** rng.uniform(-1, 1, (1, Hk, 1, D))).astype(np.float16)
    v = (rng.standard_normal((B, Hk, T, D)) * 10 ** rng.uniform(-1, 1, (1, Hk, 1, D))).astype(np.float16)
    q = rng.standard_normal((B, Hq, D)).astype(np.float16)
    pk, pv = random_perms(rng, Hk), random_perms(rng, Hk)
    ck = rng.uniform(0.8, 1.0, (Hk, D // G)).astype(np.float32)
    cv = rng.uniform(0.8, 1.0, (Hk, D // G)).astype(np.float32)
    c = oracle.OracleCache(B, Hq, Hk, G, v_bits, W, 64, pk, pv, ck, cv, k_bits=k_bits)
    c.prefill(k, v)
    out = c.decode(q)
    kq, vq = numpy_dequantize(c, T)
    kfull = np.concatenate([kq, k[:, :, T - W:].astype(np.float64)], axis=2)
    vfull = np.concatenate([vq, v[:, :, T - W:].astype(np.float64)], axis=2)
    ref = sdpa64(q, kfull, vfull, 1 / np.sqrt(D))
    assert np.abs(out - ref).max() < 1e-5 * max(1.0, np.abs(ref).max())
    # the decoded keys really are within scale/2 (or clipped) of the originals
    err = np.abs(kq - k[:, :, :T - W].astype(np.float64))
    assert err.max() < np.abs(k.astype(np.float64)).max()
    # uniform weights (softmax scale 0): output is the plain mean of the decoded values
    c0 = oracle.OracleCache(B, Hq, Hk, G, v_bits, W, 64, pk, pv, ck, cv, sm_scale=0.0, k_bits=k_bits)
    c0.prefill(k, v)
    out0 = c0.decode(q)
    mean = vfull.mean(axis=2).repeat(Hq // Hk, axis=1)
    assert np.abs(out0 - mean).max() < 1e-5 * max(1.0, np.abs(mean).max())
    # convex combination: every output channel lies between min and max of the decoded values
    lo = vfull.min(axis=2).repeat(Hq // Hk, axis=1)
    hi = vfull.max(axis=2).repeat(Hq // Hk, axis=1)
    assert np.all(out >= lo - 1e-4) and np.all(out <= hi + 1e-4)


def test_prefill_then_appends_equals_one_longer_prefill(oracle):
    rng = np.random.default_rng(500)
    B, Hq, Hk, W, T0, n = 2, 4, 2, 8, 37, 44
    k = rng.standard_normal((B, Hk, T0 + n, D)).astype(np.float16)
    v = rng.standard_normal((B, Hk, T0 + n, D)).astype(np.float16)
    pk, pv = random_perms(rng, Hk), random_perms(rng, Hk)
    clip = np.full((Hk, 2), 0.95, np.float32)
    for v_bits in (1.5, 2.0):
        a = oracle.OracleCache(B, Hq, Hk, 64, v_bits, W, 96, pk, pv, clip, clip, fill=0xAB)
        b = oracle.OracleCache(B, Hq, Hk, 64, v_bits, W, 96, pk, pv, clip, clip, fill=0xAB)
        assert a.prefill(k[:, :, :T0], v[:, :, :T0]) == 0
        for s in range(n):
            assert a.append(k[:, :, T0 + s], v[:, :, T0 + s]) == 0
        assert b.prefill(k, v) == 0
        assert a.n_tokens == b.n_tokens == T0 + n
        for x, y in zip(a.arrays(), b.arrays()):
            assert np.array_equal(x, y)
    # appends from an empty cache too (the window fills first, nothing is quantized until it is full)
    e = oracle.OracleCache(B, Hq, Hk, 64, 1.5, W, 96, pk, pv, clip, clip, fill=0xAB)
    for s in range(W):
        e.append(k[:, :, s], v[:, :, s])
    assert e.n_quant == 0 and np.all(e.k_codes == 0xAB)
    e.append(k[:, :, W], v[:, :, W])
    assert e.n_quant == 1


def test_capacity_and_empty_cache_errors(oracle):
    perm = np.tile(np.arange(D, dtype=np.int32), (1, 1))
    clip = np.ones((1, 1), np.float32)
    c = oracle.OracleCache(1, 1, 1, 128, 2.0, 4, 2, perm, perm, clip, clip)
    x = np.zeros((1, 1, 7, D), np.float16)
    assert c.prefill(x, x) == -3                      # 7 - 4 = 3 rows > capacity 2
    assert c.prefill(x[:, :, :6], x[:, :, :6]) == 0
    assert c.append(x[:, :, 0], x[:, :, 0]) == -3
    with pytest.raises(RuntimeError):
        oracle.OracleCache(1, 1, 1, 128, 2.0, 4, 2, perm, perm, clip, clip).decode(np.zeros((1, 1, D), np.float16))


# ------------------------------------------------ attention sinks (filter rule) ----
# Section 3.2 ("filter rules") and the Algorithm 1 body: tokens a filter selects stay in full
# precision when they slide out of the window; the rule used in the paper's experiments keeps the
# first few tokens (the attention sinks).

def test_sink_tokens_are_kept_bit_for_bit_and_only_shift_the_packed_rows(oracle):
    """With S sinks the packed rows are exactly what a cache without sinks stores for the
    sequence with its first S tokens removed, and sink row a is token a bit for bit."""
    rng = np.random.default_rng(600)
    B, Hq, Hk, W, T, S = 2, 4, 2, 8, 61, 5
    k = (rng.standard_normal((B, Hk, T, D)) * 3).astype(np.float16)
    v = (rng.standard_normal((B, Hk, T, D)) * 3).astype(np.float16)
    pk, pv = random_perms(rng, Hk), random_perms(rng, Hk)
    clip = np.full((Hk, 2), 0.9, np.float32)
    for v_bits in (1.5, 2.0):
        a = oracle.OracleCache(B, Hq, Hk, 64, v_bits, W, 64, pk, pv, clip, clip, n_sink=S)
        b = oracle.OracleCache(B, Hq, Hk, 64, v_bits, W, 64, pk, pv, clip, clip)
        assert a.prefill(k, v) == 0 and b.prefill(k[:, :, S:], v[:, :, S:]) == 0
        assert a.n_quant == b.n_quant == T - W - S
        for x, y in zip(a.arrays()[:4], b.arrays()[:4]):
            assert np.array_equal(x, y)
        for t in range(S):
            assert np.array_equal(a.k_win[:, :, W + t].view(np.float16), k[:, :, t])
            assert np.array_equal(a.v_win[:, :, W + t].view(np.float16), v[:, :, t])
        for t in range(T - W, T):
            assert np.array_equal(a.k_win[:, :, t % W].view(np.float16), k[:, :, t])


def test_sinks_that_cover_everything_old_give_textbook_attention(oracle):
    """If every token older than the window is a sink nothing is quantized: exact attention."""
    rng = np.random.default_rng(601)
    B, Hq, Hk, W = 1, 4, 2, 8
    for T, S in ((20, 12), (20, 40), (9, 1), (5, 3)):
        k = rng.standard_normal((B, Hk, T, D)).astype(np.float16)
        v = rng.standard_normal((B, Hk, T, D)).astype(np.float16)
        q = rng.standard_normal((B, Hq, D)).astype(np.float16)
        c = oracle.OracleCache(B, Hq, Hk, 128, 1.5, W, 4, random_perms(rng, Hk), random_perms(rng, Hk),
                               np.full((Hk, 1), 0.9, np.float32), np.full((Hk, 1), 0.9, np.float32), n_sink=S)
        assert c.prefill(k, v) == 0 and c.n_quant == 0
        assert np.abs(c.decode(q) - sdpa64(q, k, v, 1 / np.sqrt(D))).max() < 2e-6


@pytest.mark.parametrize("v_bits,G,S", [(1.5, 128, 5), (2.0, 32, 3), (1.5, 64, 1)])
def test_lossy_cache_with_sinks_equals_dequantize_then_textbook_attention(oracle, v_bits, G, S):
    """Token order of the mixed cache: sinks (exact), packed rows (decoded independently from the
    format statement), window (exact)."""
    rng = np.random.default_rng(610 + G)
    B, Hq, Hk, W, T = 2, 4, 2, 8, 45
    k = (rng.standard_normal((B, Hk, T, D)) * 10 ** rng.uniform(-1, 1, (1, Hk, 1, D))).astype(np.float16)
    v = (rng.standard_normal((B, Hk, T, D)) * 10 ** rng.uniform(-1, 1, (1, Hk, 1, D))).astype(np.float16)
    q = rng.standard_normal((B, Hq, D)).astype(np.float16)
    pk, pv = random_perms(rng, Hk), random_perms(rng, Hk)
    ck = rng.uniform(0.8, 1.0, (Hk, D // G)).astype(np.float32)
    cv = rng.uniform(0.8, 1.0, (Hk, D // G)).astype(np.float32)
    c = oracle.OracleCache(B, Hq, Hk, G, v_bits, W, 64, pk, pv, ck, cv, n_sink=S)
    c.prefill(k, v)
    kq, vq = numpy_dequantize(c, T - S)     # T - S - W packed rows
    f64 = np.float64
    kfull = np.concatenate([k[:, :, :S].astype(f64), kq, k[:, :, T - W:].astype(f64)], axis=2)
    vfull = np.concatenate([v[:, :, :S].astype(f64), vq, v[:, :, T - W:].astype(f64)], axis=2)
    assert kfull.shape[2] == T
    ref = sdpa64(q, kfull, vfull, 1 / np.sqrt(D))
    assert np.abs(c.decode(q) - ref).max() < 1e-5 * max(1.0, np.abs(ref).max())
    # keeping the sinks exact can only bring the cache closer to the fp16 one on those tokens:
    # a query that attends (almost) only to token 0 gets (almost) exactly v[0] back
    c2 = oracle.OracleCache(B, Hq, Hk, G, v_bits, W, 64, pk, pv, ck, cv, n_sink=S, sm_scale=40.0)
    c2.prefill(k, v)
    q0 = np.repeat(k[:, :, 0], Hq // Hk, axis=1)
    out = c2.decode(q0)
    want = np.repeat(v[:, :, 0].astype(f64), Hq // Hk, axis=1)
    assert np.abs(out - want).max() < 1e-3 * np.abs(want).max()


# ---- general filter rules: any mask over the tokens that leave the window (Algorithm 1, "for filter in F") ----

def test_filter_mask_of_the_first_tokens_is_the_sink_rule(oracle):
    """keep[a] = (a < S) through the general entry points: buffers and outputs identical to the sink rule's,
    at prefill and over appends."""
    rng = np.random.default_rng(630)
    B, Hq, Hk, W, T, S = 2, 4, 2, 8, 40, 3
    k = (rng.standard_normal((B, Hk, T + 20, D)) * 3).astype(np.float16)
    v = (rng.standard_normal((B, Hk, T + 20, D)) * 3).astype(np.float16)
    q = rng.standard_normal((B, Hq, D)).astype(np.float16)
    pk, pv = random_perms(rng, Hk), random_perms(rng, Hk)
    clip = np.full((Hk, 2), 0.9, np.float32)
    a = oracle.OracleCache(B, Hq, Hk, 64, 1.5, W, 64, pk, pv, clip, clip, n_sink=S)
    b = oracle.OracleCache(B, Hq, Hk, 64, 1.5, W, 64, pk, pv, clip, clip, n_sink=S)
    assert a.prefill(k[:, :, :T], v[:, :, :T]) == 0
    assert b.prefill(k[:, :, :T], v[:, :, :T], keep=np.arange(T - W) < S) == 0
    for t in range(T, T + 20):
        kn, vn = np.ascontiguousarray(k[:, :, t]), np.ascontiguousarray(v[:, :, t])
        assert a.append(kn, vn) == 0 and b.append(kn, vn, keep=False) == 0
    assert a.n_quant == b.n_quant
    for x, y in zip(a.arrays(), b.arrays()):
        assert np.array_equal(x, y)
    assert np.array_equal(a.decode(q), b.decode(q))


def test_append_without_a_decision_follows_the_sink_rule(oracle):
    """A cache driven by masks, then appended to without a decision (keep=None): the token that leaves is
    kept exactly when its number is below S (the attention-sink rule; a row is then always free, since at
    most that many older tokens can have been kept).  Expected buffers are built from the statement of the
    rule: kept token j-th in order sits in fp16 row W + j bit for bit, the others are the packed rows of a
    cache without kept rows over the same tokens in order."""
    rng = np.random.default_rng(640)
    B, Hq, Hk, W, S = 1, 2, 2, 4, 3
    n = 12
    k = (rng.standard_normal((B, Hk, n, D)) * 3).astype(np.float16)
    v = (rng.standard_normal((B, Hk, n, D)) * 3).astype(np.float16)
    pk, pv = random_perms(rng, Hk), random_perms(rng, Hk)
    clip = np.full((Hk, 1), 0.9, np.float32)

    def tok(t):
        return np.ascontiguousarray(k[:, :, t]), np.ascontiguousarray(v[:, :, t])

    # (a) the mask kept token 0 at prefill; tokens 1 and 2 leave undecided -> kept (1, 2 < S); token 3 -> packed
    a = oracle.OracleCache(B, Hq, Hk, 128, 2.0, W, 16, pk, pv, clip, clip, n_sink=S)
    assert a.prefill(k[:, :, :W + 1], v[:, :, :W + 1], keep=np.array([True])) == 0
    for t in range(W + 1, W + 4):
        assert a.append(*tok(t)) == 0
    assert a.n_quant == 1
    for j in range(3):
        assert np.array_equal(a.k_win[:, :, W + j].view(np.float16), k[:, :, j])
        assert np.array_equal(a.v_win[:, :, W + j].view(np.float16), v[:, :, j])
    ref = oracle.OracleCache(B, Hq, Hk, 128, 2.0, W, 16, pk, pv, clip, clip)
    assert ref.prefill(k[:, :, 3:W + 4], v[:, :, 3:W + 4]) == 0 and ref.n_quant == 1
    for x, y in zip(a.arrays()[:4], ref.arrays()[:4]):
        assert np.array_equal(x, y)
    # (b) the mask kept nothing of tokens 0, 1 (rows free): undecided token 2 < S is kept, in the first free row
    b = oracle.OracleCache(B, Hq, Hk, 128, 2.0, W, 16, pk, pv, clip, clip, n_sink=S)
    assert b.prefill(k[:, :, :W + 2], v[:, :, :W + 2], keep=np.array([False, False])) == 0
    assert b.append(*tok(W + 2)) == 0 and b.n_quant == 2
    assert np.array_equal(b.k_win[:, :, W].view(np.float16), k[:, :, 2])
    assert b.append(*tok(W + 3)) == 0 and b.n_quant == 3          # token 3 >= S: packed although rows are free
    # (c) no row free (S = 1, taken by the mask): undecided token 1 >= S is packed
    c = oracle.OracleCache(B, Hq, Hk, 128, 2.0, W, 16, pk, pv, clip, clip, n_sink=1)
    assert c.prefill(k[:, :, :W + 1], v[:, :, :W + 1], keep=np.array([True])) == 0
    assert c.append(*tok(W + 1)) == 0 and c.n_quant == 1
    ref = oracle.OracleCache(B, Hq, Hk, 128, 2.0, W, 16, pk, pv, clip, clip)
    assert ref.prefill(k[:, :, 1:W + 2], v[:, :, 1:W + 2]) == 0
    for x, y in zip(c.arrays()[:4], ref.arrays()[:4]):
        assert np.array_equal(x, y)


def test_filter_mask_packed_rows_are_the_unkept_tokens_in_order(oracle):
    """A random mask: the packed region equals what a cache without kept rows stores for the sequence with the
    kept tokens taken out; kept row j is the j-th kept token bit for bit; more kept tokens than rows is refused."""
    rng = np.random.default_rng(631)
    B, Hq, Hk, W, T, S = 1, 2, 2, 8, 70, 9
    k = (rng.standard_normal((B, Hk, T, D)) * 3).astype(np.float16)
    v = (rng.standard_normal((B, Hk, T, D)) * 3).astype(np.float16)
    pk, pv = random_perms(rng, Hk), random_perms(rng, Hk)
    clip = np.full((Hk, 1), 0.9, np.float32)
    keep = np.zeros(T - W, bool)
    keep[[0, 1, 17, 18, 40, 61]] = True
    for v_bits, k_bits in ((1.5, 2.0), (4.0, 4.0)):
        a = oracle.OracleCache(B, Hq, Hk, 128, v_bits, W, 64, pk, pv, clip, clip, n_sink=S, k_bits=k_bits)
        b = oracle.OracleCache(B, Hq, Hk, 128, v_bits, W, 64, pk, pv, clip, clip, k_bits=k_bits)
        rest = np.concatenate([np.flatnonzero(~keep), np.arange(T - W, T)])
        assert a.prefill(k, v, keep=keep) == 0 and b.prefill(k[:, :, rest], v[:, :, rest]) == 0
        assert a.n_quant == b.n_quant == T - W - 6
        for x, y in zip(a.arrays()[:4], b.arrays()[:4]):
            assert np.array_equal(x, y)
        for j, t in enumerate(np.flatnonzero(keep)):
            assert np.array_equal(a.k_win[:, :, W + j].view(np.float16), k[:, :, t])
            assert np.array_equal(a.v_win[:, :, W + j].view(np.float16), v[:, :, t])
    too_many = np.zeros(T - W, bool)
    too_many[:S + 1] = True
    assert a.prefill(k, v, keep=too_many) == -3


@pytest.mark.parametrize("v_bits,G", [(1.5, 128), (2.0, 32)])
def test_filter_mask_attention_equals_dequantize_then_textbook_attention(oracle, v_bits, G):
    """Kept tokens exact, the others decoded independently from the format statement, the window exact; also
    through appends with per-step decisions, and for several query tokens."""
    rng = np.random.default_rng(632 + G)
    B, Hq, Hk, W, T0, n_app, S = 2, 4, 2, 8, 30, 25, 12
    T = T0 + n_app
    k = (rng.standard_normal((B, Hk, T, D)) * 10 ** rng.uniform(-1, 1, (1, Hk, 1, D))).astype(np.float16)
    v = (rng.standard_normal((B, Hk, T, D)) * 10 ** rng.uniform(-1, 1, (1, Hk, 1, D))).astype(np.float16)
    q = rng.standard_normal((B, Hq, D)).astype(np.float16)
    pk, pv = random_perms(rng, Hk), random_perms(rng, Hk)
    ck = rng.uniform(0.8, 1.0, (Hk, D // G)).astype(np.float32)
    cv = rng.uniform(0.8, 1.0, (Hk, D // G)).astype(np.float32)
    keep = rng.random(T - W) < 0.2
    keep[T0 - W] = True              # the first token that an append moves out is kept
    assert keep.sum() <= S
    c = oracle.OracleCache(B, Hq, Hk, G, v_bits, W, 64, pk, pv, ck, cv, n_sink=S)
    assert c.prefill(k[:, :, :T0], v[:, :, :T0], keep=keep[:T0 - W]) == 0
    for t in range(T0, T):
        assert c.append(np.ascontiguousarray(k[:, :, t]), np.ascontiguousarray(v[:, :, t]), keep=keep[t - W]) == 0
    # the same cache state from one prefill with the whole mask
    d = oracle.OracleCache(B, Hq, Hk, G, v_bits, W, 64, pk, pv, ck, cv, n_sink=S)
    assert d.prefill(k, v, keep=keep) == 0
    for x, y in zip(c.arrays(), d.arrays()):
        assert np.array_equal(x, y)
    n_packed = int((~keep).sum())
    assert c.n_quant == n_packed
    kq, vq = numpy_dequantize(c, n_packed + W)
    f64 = np.float64
    kept_ids = np.flatnonzero(keep)
    kfull = np.concatenate([k[:, :, kept_ids].astype(f64), kq, k[:, :, T - W:].astype(f64)], axis=2)
    vfull = np.concatenate([v[:, :, kept_ids].astype(f64), vq, v[:, :, T - W:].astype(f64)], axis=2)
    assert kfull.shape[2] == T
    ref = sdpa64(q, kfull, vfull, 1 / np.sqrt(D))
    assert np.abs(c.decode(q) - ref).max() < 1e-5 * max(1.0, np.abs(ref).max())
    # two query tokens: the last one is the single-token call, the first one does not see the newest token
    q2 = np.stack([rng.standard_normal((B, Hq, D)).astype(np.float16), q], axis=1)
    out2 = c.decode_multi(q2)
    assert np.abs(out2[:, 1] - c.decode(q)).max() < 1e-6
    ref0 = sdpa64(q2[:, 0], kfull[:, :, :T - 1], vfull[:, :, :T - 1], 1 / np.sqrt(D))
    assert np.abs(out2[:, 0] - ref0).max() < 1e-5 * max(1.0, np.abs(ref0).max())


def test_filter_mask_that_keeps_everything_gives_textbook_attention(oracle):
    rng = np.random.default_rng(634)
    B, Hq, Hk, W, T = 1, 4, 2, 8, 24
    k = rng.standard_normal((B, Hk, T, D)).astype(np.float16)
    v = rng.standard_normal((B, Hk, T, D)).astype(np.float16)
    q = rng.standard_normal((B, Hq, D)).astype(np.float16)
    c = oracle.OracleCache(B, Hq, Hk, 128, 1.5, W, 4, random_perms(rng, Hk), random_perms(rng, Hk),
                           np.full((Hk, 1), 0.9, np.float32), np.full((Hk, 1), 0.9, np.float32), n_sink=T - W)
    assert c.prefill(k, v, keep=np.ones(T - W, bool)) == 0 and c.n_quant == 0
    assert np.abs(c.decode(q) - sdpa64(q, k, v, 1 / np.sqrt(D))).max() < 2e-6
    # the kept rows are full: the next token to leave can only be packed
    x = np.zeros((B, Hk, D), np.float16)
    assert c.append(x, x, keep=True) == -3 and c.append(x, x, keep=False) == 0 and c.n_quant == 1


def test_prefill_then_appends_equals_one_longer_prefill_with_sinks(oracle):
    """Appends walk tokens through all three places: ring -> sink rows (the first S) -> packed."""
    rng = np.random.default_rng(620)
    B, Hq, Hk, W, S = 2, 4, 2, 8, 5
    k = rng.standard_normal((B, Hk, 60, D)).astype(np.float16)
    v = rng.standard_normal((B, Hk, 60, D)).astype(np.float16)
    pk, pv = random_perms(rng, Hk), random_perms(rng, Hk)
    clip = np.full((Hk, 2), 0.95, np.float32)
    for T0 in (0, 3, 8, 11, 13, 30):
        a = oracle.OracleCache(B, Hq, Hk, 64, 1.5, W, 64, pk, pv, clip, clip, fill=0xAB, n_sink=S)
        b = oracle.OracleCache(B, Hq, Hk, 64, 1.5, W, 64, pk, pv, clip, clip, fill=0xAB, n_sink=S)
        if T0:
            assert a.prefill(k[:, :, :T0], v[:, :, :T0]) == 0
        for s in range(T0, 60):
            assert a.append(k[:, :, s], v[:, :, s]) == 0
        assert b.prefill(k, v) == 0
        assert a.n_tokens == b.n_tokens == 60 and a.n_quant == 60 - W - S
        for x, y in zip(a.arrays(), b.arrays()):
            assert np.array_equal(x, y)
    # capacity counts packed rows only
    c = oracle.OracleCache(B, Hq, Hk, 64, 1.5, W, 2, pk, pv, clip, clip, n_sink=S)
    assert c.prefill(k[:, :, :W + S + 3], v[:, :, :W + S + 3]) == -3
    assert c.prefill(k[:, :, :W + S + 2], v[:, :, :W + S + 2]) == 0
    assert c.append(k[:, :, 0], v[:, :, 0]) == -3


# --------------------------------------- compact (scale, zero): fp16 and FP8 E4M3 ----
# Section 4.1 stores scale and zero in FP8 (E4M3); Table 2 / the breakdown paragraph of Section
# 4.3 count 2 + 16*2/32 bits with fp16 metadata and 2 + 8*2/32 with FP8.

def e4m3_value(b: int) -> float:
    """The format's definition, written out independently of the oracle."""
    s, e, m = b >> 7, (b >> 3) & 15, b & 7
    if e == 15 and m == 7:
        return float("nan")
    v = m / 8 * 2.0 ** -6 if e == 0 else (1 + m / 8) * 2.0 ** (e - 7)
    return -v if s else v


def test_e4m3_decoding_all_bit_patterns(oracle):
    want = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float32).numpy()  # library
    for b in range(256):
        got = oracle.e4m3_to_float(b)
        if b & 0x7f == 0x7f:
            assert np.isnan(got) and np.isnan(want[b])
        else:
            assert got == e4m3_value(b) == want[b], b
    assert oracle.e4m3_to_float(0x7e) == 448.0 and oracle.e4m3_to_float(0x01) == 2.0 ** -9


def test_e4m3_narrowing_is_nearest_even_and_saturates(oracle):
    rng = np.random.default_rng(700)
    finite = [(e4m3_value(b), b) for b in range(256) if b & 0x7f != 0x7f]
    xs = np.concatenate([rng.standard_normal(3000) * 10 ** rng.uniform(-4, 2.6, 3000),
                         [0.0, -0.0, 2.0 ** -10, 3 * 2.0 ** -10, 2.0 ** -9, 432.0, 447.9, 448.0, 0.0029296875],
                         [(finite[i][0] + finite[i + 1][0]) / 2 for i in range(0, 120, 7)]]).astype(np.float32)
    xs = xs[np.abs(xs) <= 448]
    lib = torch.from_numpy(xs).to(torch.float8_e4m3fn).view(torch.uint8).numpy()       # library routine
    for x, lb in zip(xs, lib):
        got = oracle.float_to_e4m3(float(x))
        # brute force: nearest finite value, ties to the even mantissa
        best = min(finite, key=lambda vb: (abs(vb[0] - float(x)), vb[1] & 1))
        assert oracle.e4m3_to_float(got) == best[0], (x, got, best)
        assert got & 0x7f == lb & 0x7f, (x, got, lb)          # (the sign of a rounded-to-zero value aside)
    for x, want in ((449.0, 0x7e), (1e9, 0x7e), (-500.0, 0xfe), (464.0, 0x7e)):
        assert oracle.float_to_e4m3(x) == want
    # reading back what was stored changes nothing
    for meta in ("f16", "e4m3"):
        for x in xs[:200]:
            r = oracle.round_meta(float(x), meta)
            assert oracle.round_meta(r, meta) == r
    assert oracle.round_meta(0.1, "f32") == float(np.float32(0.1))
    assert oracle.round_meta(0.1, "f16") == float(np.float16(0.1))


@pytest.mark.parametrize("meta", ["f16", "e4m3"])
@pytest.mark.parametrize("levels", [4, 3, 16, 8])
def test_encoder_with_compact_meta_uses_the_stored_values(oracle, meta, levels):
    """scale and zero come back exactly representable in the storage format, and every code is
    the nearest level of the grid THOSE values span (so decoding, which only sees them, is
    as close as it can be)."""
    rng = np.random.default_rng(710 + levels)
    top = levels - 1
    for trial in range(200):
        n = int(rng.choice([4, 32, 128]))
        x = (rng.standard_normal(n) * 10 ** rng.uniform(-2, 1.5)).astype(np.float16).astype(np.float32)
        alpha = float(rng.uniform(0.7, 1.0))
        c, h, z = oracle.encode_group(x, alpha, levels, meta)
        assert oracle.round_meta(h, meta) == h and oracle.round_meta(z, meta) == z
        # they are the rounded values of the fp32 formula's
        c32, h32, z32 = oracle.encode_group(x, alpha, levels, "f32")
        assert h == oracle.round_meta(h32, meta) and z == oracle.round_meta(z32, meta)
        if h == 0:
            assert not c.any()
            continue
        t = (x.astype(np.float64) - float(z)) / float(h)
        grid = np.arange(levels)
        for ti, ci in zip(t, c):
            d = np.abs(grid - ti)
            assert d[ci] <= d.min() + 1e-5 * max(1.0, abs(ti)), (ti, ci)
        inside = (t >= 0) & (t <= top)
        deq = c * np.float64(h) + np.float64(z)
        assert np.all(np.abs(deq - x)[inside] <= float(h) / 2 * (1 + 1e-5))


def test_fp32_meta_is_unchanged_by_the_format_argument(oracle):
    rng = np.random.default_rng(720)
    for _ in range(50):
        x = (rng.standard_normal(64) * 3).astype(np.float16).astype(np.float32)
        a = oracle.encode_group(x, 0.9, 4)
        b = oracle.encode_group(x, 0.9, 4, "f32")
        assert np.array_equal(a[0], b[0]) and a[1] == b[1] and a[2] == b[2]


def meta_as_float64(arr, meta):
    if meta == "e4m3":
        table = np.array([e4m3_value(b) for b in range(256)])
        return table[arr]
    return arr.astype(np.float64)


@pytest.mark.parametrize("meta,v_bits,G", [("f16", 1.5, 128), ("e4m3", 1.5, 128), ("e4m3", 2.0, 32), ("f16", 2.0, 64)])
def test_lossy_cache_with_compact_meta_equals_dequantize_then_textbook_attention(oracle, meta, v_bits, G):
    rng = np.random.default_rng(730 + G)
    B, Hq, Hk, W, T, S = 2, 4, 2, 8, 45, 2
    k = (rng.standard_normal((B, Hk, T, D)) * 10 ** rng.uniform(-1, 1, (1, Hk, 1, D))).astype(np.float16)
    v = (rng.standard_normal((B, Hk, T, D)) * 10 ** rng.uniform(-1, 1, (1, Hk, 1, D))).astype(np.float16)
    q = rng.standard_normal((B, Hq, D)).astype(np.float16)
    pk, pv = random_perms(rng, Hk), random_perms(rng, Hk)
    ck = rng.uniform(0.8, 1.0, (Hk, D // G)).astype(np.float32)
    cv = rng.uniform(0.8, 1.0, (Hk, D // G)).astype(np.float32)
    c = oracle.OracleCache(B, Hq, Hk, G, v_bits, W, 64, pk, pv, ck, cv, n_sink=S, meta=meta)
    assert c.prefill(k, v) == 0
    # independent dequantization: the stored meta decoded from the format statement
    class View:
        pass
    vw = View()
    vw.k_codes, vw.v_codes, vw.window, vw.cfg, vw.perm_k, vw.perm_v = c.k_codes, c.v_codes, c.window, c.cfg, c.perm_k, c.perm_v
    vw.k_meta, vw.v_meta = meta_as_float64(c.k_meta, meta), meta_as_float64(c.v_meta, meta)
    kq, vq = numpy_dequantize(vw, T - S)
    f64 = np.float64
    kfull = np.concatenate([k[:, :, :S].astype(f64), kq, k[:, :, T - W:].astype(f64)], axis=2)
    vfull = np.concatenate([v[:, :, :S].astype(f64), vq, v[:, :, T - W:].astype(f64)], axis=2)
    ref = sdpa64(q, kfull, vfull, 1 / np.sqrt(D))
    assert np.abs(c.decode(q) - ref).max() < 1e-5 * max(1.0, np.abs(ref).max())
    # the stored bytes per packed token-head: Section 4.3's accounting with 16- / 8-bit metadata
    es = {"f16": 2, "e4m3": 1}[meta]
    assert c.k_meta.nbytes == B * Hk * 64 * (D // G) * 2 * es
    assert (32 * 8 + (D // G) * 2 * es * 8) / D == oracle.avg_bits(2, 8 * es, G)
    # appends agree with the longer prefill in these formats too
    a = oracle.OracleCache(B, Hq, Hk, G, v_bits, W, 64, pk, pv, ck, cv, n_sink=S, meta=meta, fill=0xAB)
    b = oracle.OracleCache(B, Hq, Hk, G, v_bits, W, 64, pk, pv, ck, cv, n_sink=S, meta=meta, fill=0xAB)
    a.prefill(k[:, :, :20], v[:, :, :20])
    for s in range(20, T):
        a.append(k[:, :, s], v[:, :, s])
    b.prefill(k, v)
    for x, y in zip(a.arrays(), b.arrays()):
        assert np.array_equal(x, y)


# ---- unequal groups (Section 4.1: clustering the channels gives groups of unequal size) ----

UNEQUAL_BOUNDS = [(32, [0, 16, 32, 80, 128]), (64, [0, 48, 128]), (32, [0, 7, 8, 100, 128]), (64, [0, 127, 128])]


def grid_data_bounds(rng, shape_bht, bounds, levels, perm):
    """Like grid_data, with one grid per (token, kv head, unequal group)."""
    B, Hk, T = shape_bht
    x = np.zeros((B, Hk, T, D), np.float32)
    for b in range(B):
        for h in range(Hk):
            for t in range(T):
                for lo, hi in zip(bounds[:-1], bounds[1:]):
                    step = 2.0 ** int(rng.integers(-5, 2))
                    base = step * int(rng.integers(-20, 20))
                    k = rng.integers(0, levels, hi - lo)
                    if hi - lo >= 2:
                        k[0], k[-1] = 0, levels - 1
                    x[b, h, t, perm[h, lo:hi]] = base + step * k
    return x.astype(np.float16)


@pytest.mark.parametrize("G,bounds", UNEQUAL_BOUNDS)
def test_unequal_groups_scale_and_zero_come_from_exactly_their_positions(oracle, G, bounds):
    """(scale, zero) of group g are Eq. 2 over the reordered positions [b_g, b_{g+1}) and nothing
    else; the codes of a group use its own pair."""
    rng = np.random.default_rng(800 + len(bounds) + bounds[1])
    B, Hq, Hk, W, T = 1, 2, 2, 4, 30
    ng = D // G
    k = (rng.standard_normal((B, Hk, T, D)) * 10 ** rng.uniform(-1, 1, (1, Hk, 1, D))).astype(np.float16)
    v = (rng.standard_normal((B, Hk, T, D)) * 10 ** rng.uniform(-1, 1, (1, Hk, 1, D))).astype(np.float16)
    pk, pv = random_perms(rng, Hk), random_perms(rng, Hk)
    ck = rng.uniform(0.8, 1.0, (Hk, ng)).astype(np.float32)
    cv = rng.uniform(0.8, 1.0, (Hk, ng)).astype(np.float32)
    c = oracle.OracleCache(B, Hq, Hk, G, 2.0, W, 32, pk, pv, ck, cv, group_bounds=bounds)
    assert c.prefill(k, v) == 0
    f32 = np.float32
    for h in range(Hk):
        for t in range(T - W):
            for x, perm, clip, meta, code in ((k, pk, ck, c.k_meta, c.k_code), (v, pv, cv, c.v_meta, c.v_code)):
                xp = x[0, h, t, perm[h]].astype(f32)
                for g, (lo, hi) in enumerate(zip(bounds[:-1], bounds[1:])):
                    mn, mx = xp[lo:hi].min(), xp[lo:hi].max()
                    zero = f32(clip[h, g] * mn)
                    scale = f32(f32(f32(clip[h, g] * mx) - zero) / f32(3))
                    assert meta[0, h, t, g, 0] == scale and meta[0, h, t, g, 1] == zero
                    want, _, _ = oracle.encode_group(xp[lo:hi], float(clip[h, g]), 4)
                    assert [code(0, h, t, p) for p in range(lo, hi)] == list(want)


@pytest.mark.parametrize("G,bounds", UNEQUAL_BOUNDS)
@pytest.mark.parametrize("k_bits,v_bits", [(2.0, 1.5), (4.0, 4.0)])
def test_unequal_groups_lossless_and_lossy_caches(oracle, G, bounds, k_bits, v_bits):
    rng = np.random.default_rng(900 + bounds[1])
    B, Hq, Hk, W, T = 1, 4, 2, 8, 50
    ng = D // G
    pk, pv = random_perms(rng, Hk), random_perms(rng, Hk)
    q = rng.standard_normal((B, Hq, D)).astype(np.float16)
    ones = np.ones((Hk, ng), np.float32)
    # lossless: every unequal group on its own exact grid -> the library's attention on the originals
    k = grid_data_bounds(rng, (B, Hk, T), bounds, oracle.levels_of(k_bits), pk)
    v = grid_data_bounds(rng, (B, Hk, T), bounds, oracle.levels_of(v_bits), pv)
    c = oracle.OracleCache(B, Hq, Hk, G, v_bits, W, 64, pk, pv, ones, ones, sm_scale=0.05, k_bits=k_bits,
                           group_bounds=bounds)
    assert c.prefill(k, v) == 0
    ref = sdpa64(q, k, v, 0.05)
    assert np.abs(c.decode(q) - ref).max() < 1e-5 * max(1.0, np.abs(ref).max())
    # lossy: independent unpack + dequantize with the same boundaries, then the library's attention
    k = (rng.standard_normal((B, Hk, T, D)) * 10 ** rng.uniform(-1, 1, (1, Hk, 1, D))).astype(np.float16)
    v = (rng.standard_normal((B, Hk, T, D)) * 10 ** rng.uniform(-1, 1, (1, Hk, 1, D))).astype(np.float16)
    ck = rng.uniform(0.8, 1.0, (Hk, ng)).astype(np.float32)
    c = oracle.OracleCache(B, Hq, Hk, G, v_bits, W, 64, pk, pv, ck, ck, k_bits=k_bits, group_bounds=bounds)
    assert c.prefill(k[:, :, :20], v[:, :, :20]) == 0
    for s in range(20, T):
        assert c.append(k[:, :, s], v[:, :, s]) == 0
    kq, vq = numpy_dequantize(c, T)
    kfull = np.concatenate([kq, k[:, :, T - W:].astype(np.float64)], axis=2)
    vfull = np.concatenate([vq, v[:, :, T - W:].astype(np.float64)], axis=2)
    ref = sdpa64(q, kfull, vfull, 1 / np.sqrt(D))
    assert np.abs(c.decode(q) - ref).max() < 1e-5 * max(1.0, np.abs(ref).max())


def test_uniform_boundaries_are_the_uniform_groups_and_bad_boundaries_are_refused(oracle):
    rng = np.random.default_rng(950)
    B, Hq, Hk, W, T, G = 1, 2, 2, 4, 40, 32
    k = rng.standard_normal((B, Hk, T, D)).astype(np.float16)
    v = rng.standard_normal((B, Hk, T, D)).astype(np.float16)
    pk, pv = random_perms(rng, Hk), random_perms(rng, Hk)
    clip = np.full((Hk, D // G), 0.9, np.float32)
    a = oracle.OracleCache(B, Hq, Hk, G, 1.5, W, 64, pk, pv, clip, clip)
    b = oracle.OracleCache(B, Hq, Hk, G, 1.5, W, 64, pk, pv, clip, clip, group_bounds=[0, 32, 64, 96, 128])
    assert a.prefill(k, v) == 0 and b.prefill(k, v) == 0
    for x, y in zip(a.arrays(), b.arrays()):
        assert np.array_equal(x, y)
    for bad in ([0, 32, 32, 96, 128], [1, 32, 64, 96, 128], [0, 32, 64, 96, 127], [0, 64, 32, 96, 128]):
        c = oracle.OracleCache(B, Hq, Hk, G, 1.5, W, 64, pk, pv, clip, clip, group_bounds=bad)
        assert c.prefill(k, v) == -1


# ---- prefill attention (Section 3.2, phase 1: the prompt's own attention, full precision) ----

def test_prefill_attention_is_the_librarys_causal_attention(oracle):
    rng = np.random.default_rng(1200)
    for B, Hq, Hk, T in ((1, 4, 2, 37), (2, 6, 2, 130), (1, 3, 3, 1)):
        q = rng.standard_normal((B, Hq, T, D)).astype(np.float16)
        k = (rng.standard_normal((B, Hk, T, D)) * 2).astype(np.float16)
        v = (rng.standard_normal((B, Hk, T, D)) * 3).astype(np.float16)
        perm = np.tile(np.arange(D, dtype=np.int32), (Hk, 1))
        one = np.ones((Hk, 1), np.float32)
        c = oracle.OracleCache(B, Hq, Hk, 128, 1.5, 8, 8, perm, perm, one, one, sm_scale=0.11)
        out = c.prefill_attention(q, k, v)
        rep = Hq // Hk
        qt = torch.from_numpy(q.astype(np.float64))
        kt = torch.from_numpy(k.astype(np.float64)).repeat_interleave(rep, dim=1)
        vt = torch.from_numpy(v.astype(np.float64)).repeat_interleave(rep, dim=1)
        ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, is_causal=True, scale=0.11).numpy()
        assert np.abs(out - ref).max() < 1e-5
        # row 0 sees only token 0
        assert np.abs(out[:, :, 0] - v.astype(np.float64).repeat(rep, axis=1)[:, :, 0]).max() < 1e-6


def test_prefill_attention_with_uniform_weights_is_the_running_mean(oracle):
    rng = np.random.default_rng(1201)
    B, Hq, Hk, T = 1, 2, 1, 50
    q = rng.standard_normal((B, Hq, T, D)).astype(np.float16)
    k = rng.standard_normal((B, Hk, T, D)).astype(np.float16)
    v = rng.standard_normal((B, Hk, T, D)).astype(np.float16)
    perm = np.tile(np.arange(D, dtype=np.int32), (Hk, 1))
    one = np.ones((Hk, 1), np.float32)
    c = oracle.OracleCache(B, Hq, Hk, 128, 1.5, 8, 8, perm, perm, one, one, sm_scale=0.0)
    out = c.prefill_attention(q, k, v)
    mean = np.cumsum(v.astype(np.float64), axis=2) / np.arange(1, T + 1)[None, None, :, None]
    assert np.abs(out - mean.repeat(Hq // Hk, axis=1)).max() < 1e-6


def test_prefill_attention_rows_are_the_librarys_rows(oracle):
    """The chosen-rows entry (for prompts too long to compute whole) against the library's causal
    attention and against the whole-prompt entry; an index out of range is refused."""
    rng = np.random.default_rng(1202)
    B, Hq, Hk, T = 2, 6, 2, 130
    q = rng.standard_normal((B, Hq, T, D)).astype(np.float16)
    k = (rng.standard_normal((B, Hk, T, D)) * 2).astype(np.float16)
    v = (rng.standard_normal((B, Hk, T, D)) * 3).astype(np.float16)
    perm = np.tile(np.arange(D, dtype=np.int32), (Hk, 1))
    one = np.ones((Hk, 1), np.float32)
    c = oracle.OracleCache(B, Hq, Hk, 128, 1.5, 8, 8, perm, perm, one, one, sm_scale=0.11)
    rows = [(0, 0, 0), (1, 5, 129), (0, 3, 64), (1, 2, 63), (0, 4, 1), (1, 0, 100)]
    out = c.prefill_attention_rows(q, k, v, rows)
    rep = Hq // Hk
    qt = torch.from_numpy(q.astype(np.float64))
    kt = torch.from_numpy(k.astype(np.float64)).repeat_interleave(rep, dim=1)
    vt = torch.from_numpy(v.astype(np.float64)).repeat_interleave(rep, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, is_causal=True, scale=0.11).numpy()
    whole = c.prefill_attention(q, k, v)
    for i, (b, h, t) in enumerate(rows):
        assert np.abs(out[i] - ref[b, h, t]).max() < 1e-5
        assert np.array_equal(out[i], whole[b, h, t])
    for bad in ((2, 0, 0), (0, 6, 0), (0, 0, 130), (0, -1, 0)):
        with pytest.raises(RuntimeError):
            c.prefill_attention_rows(q, k, v, [bad])


# ---- clip calibration (Eq. 3; Algorithm 1 Prologue, get_group_clipping) ----

def calib_setup(oracle, rng, G, lossless=False, T=48, W=8, Hq=4, Hk=2, n_q=3, v_bits=2.0):
    B = 1
    pk, pv = random_perms(rng, Hk), random_perms(rng, Hk)
    if lossless:
        k = grid_data(rng, (B, Hk, T), G, 4, pk)
        v = grid_data(rng, (B, Hk, T), G, oracle.levels_of(v_bits), pv)
    else:
        # heavy-tailed channels: a few outliers per group make clipping pay
        k = (rng.standard_t(2.5, (B, Hk, T, D)) * 0.5).astype(np.float16)
        v = (rng.standard_t(2.5, (B, Hk, T, D)) * 0.5).astype(np.float16)
    q = rng.standard_normal((n_q, B, Hq, D)).astype(np.float16)
    o_ref = np.stack([sdpa64(q[i], k, v, 1 / np.sqrt(D)) for i in range(n_q)]).astype(np.float32)
    ones = np.ones((Hk, D // G), np.float32)

    def make(ck=ones, cv=ones):
        return oracle.OracleCache(B, Hq, Hk, G, v_bits, W, T, pk, pv, ck, cv)

    def loss_of(ck, cv):
        """Per-kv-head summed squared error of a fresh cache with these clips (numpy arithmetic)."""
        c = make(ck, cv)
        assert c.prefill(k, v) == 0
        out = np.stack([c.decode(q[i]) for i in range(n_q)]).astype(np.float64)
        d2 = (out - o_ref.astype(np.float64)) ** 2
        return d2.reshape(n_q, B, Hk, Hq // Hk, D).sum(axis=(0, 1, 3, 4))
    return make, loss_of, k, v, q, o_ref


def test_clip_calibration_follows_coordinate_descent_on_the_output_error(oracle):
    rng = np.random.default_rng(1300)
    G = 64
    make, loss_of, k, v, q, o_ref = calib_setup(oracle, rng, G)
    alphas = np.array([1.0, 0.9, 0.8, 0.65], np.float32)
    ck, cv, loss = make().calibrate_clip(k, v, q, o_ref, alphas)
    # the same search, driven from here with independent evaluations
    Hk, ng = ck.shape
    wk, wv = np.ones((Hk, ng), np.float32), np.ones((Hk, ng), np.float32)
    for clip in (wk, wv):
        for g in range(ng):
            errs = []
            for a in alphas:
                clip[:, g] = a
                errs.append(loss_of(wk, wv))
            clip[:, g] = alphas[np.argmin(np.array(errs), axis=0)]     # first minimum per head
    assert np.array_equal(ck, wk) and np.array_equal(cv, wv)
    final = loss_of(ck, cv)
    assert np.allclose(loss, final, rtol=1e-9)
    # never worse than where it started, and clipping does pay on heavy-tailed data
    start = loss_of(np.ones_like(ck), np.ones_like(cv))
    assert np.all(final <= start) and np.any(ck < 1.0) and np.any(cv < 1.0) and np.all(final < start)


def test_clip_calibration_keeps_alpha_one_when_the_data_is_exactly_representable(oracle):
    rng = np.random.default_rng(1301)
    make, loss_of, k, v, q, o_ref = calib_setup(oracle, rng, 128, lossless=True)
    ck, cv, loss = make().calibrate_clip(k, v, q, o_ref, np.array([0.8, 1.0, 0.9], np.float32))
    assert np.all(ck == 1.0) and np.all(cv == 1.0) and np.all(loss < 1e-9)
    # a one-point grid returns that point
    ck, cv, _ = make().calibrate_clip(k, v, q, o_ref, np.array([0.75], np.float32))
    assert np.all(ck == 0.75) and np.all(cv == 0.75)


def test_unequal_groups_may_differ_between_kv_heads(oracle):
    """Clustering each kv head's channels gives each head its own group sizes."""
    rng = np.random.default_rng(960)
    B, Hq, Hk, W, T, G = 1, 4, 2, 8, 40, 32
    bounds = np.array([[0, 16, 32, 80, 128], [0, 5, 64, 127, 128]], np.int32)
    pk, pv = random_perms(rng, Hk), random_perms(rng, Hk)
    k = (rng.standard_normal((B, Hk, T, D)) * 10 ** rng.uniform(-1, 1, (1, Hk, 1, D))).astype(np.float16)
    v = (rng.standard_normal((B, Hk, T, D)) * 10 ** rng.uniform(-1, 1, (1, Hk, 1, D))).astype(np.float16)
    q = rng.standard_normal((B, Hq, D)).astype(np.float16)
    clip = rng.uniform(0.8, 1.0, (Hk, D // G)).astype(np.float32)
    c = oracle.OracleCache(B, Hq, Hk, G, 2.0, W, 64, pk, pv, clip, clip, group_bounds=bounds)
    assert c.prefill(k, v) == 0
    f32 = np.float32
    for h in range(Hk):
        xp = k[0, h, 3, pk[h]].astype(f32)
        for g in range(D // G):
            lo, hi = bounds[h, g], bounds[h, g + 1]
            zero = f32(clip[h, g] * xp[lo:hi].min())
            assert c.k_meta[0, h, 3, g, 1] == zero
            assert c.k_meta[0, h, 3, g, 0] == f32(f32(f32(clip[h, g] * xp[lo:hi].max()) - zero) / f32(3))
    kq, vq = numpy_dequantize(c, T)
    kfull = np.concatenate([kq, k[:, :, T - W:].astype(np.float64)], axis=2)
    vfull = np.concatenate([vq, v[:, :, T - W:].astype(np.float64)], axis=2)
    ref = sdpa64(q, kfull, vfull, 1 / np.sqrt(D))
    assert np.abs(c.decode(q) - ref).max() < 1e-5 * max(1.0, np.abs(ref).max())
    # each head's own head-0 bounds alone give the same head-0 rows
    c0 = oracle.OracleCache(B, Hq, Hk, G, 2.0, W, 64, pk, pv, clip, clip, group_bounds=bounds[0])
    assert c0.prefill(k, v) == 0
    assert np.array_equal(c0.k_codes[:, 0], c.k_codes[:, 0]) and not np.array_equal(c0.k_codes[:, 1], c.k_codes[:, 1])


# ---- channel reorder (Section 3.1; Algorithm 1 Prologue, get_permutation_matrix) ----

def test_channel_stats_are_min_and_max_over_all_tokens(oracle):
    rng = np.random.default_rng(1400)
    x = (rng.standard_normal((3, 2, 41, D)) * 10 ** rng.uniform(-1, 1, (1, 2, 1, D))).astype(np.float16)
    st = oracle.channel_stats(x)
    assert np.array_equal(st[..., 0], x.min(axis=(0, 2)).astype(np.float32))
    assert np.array_equal(st[..., 1], x.max(axis=(0, 2)).astype(np.float32))


def test_reorder_recovers_planted_channel_families(oracle):
    """Four families of channels with well separated ranges and unequal sizes: the clusters are
    the families, listed by range; the permutation lists each family's channels together."""
    rng = np.random.default_rng(1401)
    sizes, scales = [16, 48, 24, 40], [8.0, 0.05, 1.0, 0.3]
    stats = np.zeros((2, D, 2), np.float32)
    fam = np.zeros((2, D), int)
    for h in range(2):
        fam[h] = rng.permutation(np.repeat(np.arange(4), sizes))
        for ch in range(D):
            sc = scales[fam[h, ch]] * rng.uniform(0.9, 1.1)
            stats[h, ch] = (-sc * rng.uniform(0.8, 1.0), sc * rng.uniform(0.8, 1.0))
    perm, bounds = oracle.calibrate_reorder(stats, 32)
    by_range = np.argsort(scales)                                  # families from narrow to wide
    assert np.array_equal(bounds, np.tile(np.concatenate([[0], np.cumsum(np.array(sizes)[by_range])]), (2, 1)))
    for h in range(2):
        assert sorted(perm[h]) == list(range(D))
        for j, f in enumerate(by_range):
            assert set(perm[h, bounds[h, j]:bounds[h, j + 1]]) == set(np.flatnonzero(fam[h] == f))
            r = stats[h, perm[h, bounds[h, j]:bounds[h, j + 1]], 1] - stats[h, perm[h, bounds[h, j]:bounds[h, j + 1]], 0]
            assert np.all(np.diff(r) >= 0)                         # inside a cluster: by range
    # multiples of 16: every boundary moves to the nearest one, every group keeps 16 positions
    perm16, bounds16 = oracle.calibrate_reorder(stats, 32, granularity=16)
    assert np.array_equal(perm16, perm)
    assert np.all(bounds16 % 16 == 0) and np.all(np.diff(bounds16, axis=1) >= 16)
    assert np.all(np.abs(bounds16 - bounds) <= 8)


def test_reorder_is_lloyds_kmeans_from_the_stated_start(oracle):
    """Against the library's KMeans (Lloyd, same initial centroids, no restarts) on data without
    obvious clusters: the same partition of the channels."""
    from sklearn.cluster import KMeans
    rng = np.random.default_rng(1402)
    for G in (32, 64):
        ng = D // G
        sc = 10 ** rng.uniform(-1.5, 1.0, D)
        stats = np.stack([-sc * rng.uniform(0.3, 1.0, D), sc * rng.uniform(0.3, 1.0, D)], axis=1).astype(np.float32)[None]
        perm, bounds = oracle.calibrate_reorder(stats, G)
        assert np.all(np.diff(bounds[0]) >= 1)
        f = stats[0].astype(np.float64)
        order = np.lexsort((np.arange(D), f[:, 1] - f[:, 0]))
        init = np.stack([f[order[j * G:(j + 1) * G]].mean(axis=0) for j in range(ng)])
        km = KMeans(n_clusters=ng, init=init, n_init=1, algorithm="lloyd", max_iter=100, tol=0.0).fit(f)
        theirs = {frozenset(np.flatnonzero(km.labels_ == j)) for j in range(ng)}
        ours = {frozenset(perm[0, bounds[0, j]:bounds[0, j + 1]]) for j in range(ng)}
        assert ours == theirs


def test_reorder_lowers_the_quantization_error_on_outlier_channels(oracle):
    rng = np.random.default_rng(1403)
    B, Hk, T, G = 1, 2, 64, 32
    scale = np.where(rng.random((1, Hk, 1, D)) < 0.1, 12.0, 1.0) * 10 ** rng.uniform(-0.3, 0.3, (1, Hk, 1, D))
    k = (rng.standard_normal((B, Hk, T, D)) * scale).astype(np.float16)
    perm, bounds = oracle.calibrate_reorder(oracle.channel_stats(k), G, granularity=16)
    ident = np.tile(np.arange(D, dtype=np.int32), (Hk, 1))
    ones = np.ones((Hk, D // G), np.float32)

    def key_error(pm, gb):
        c = oracle.OracleCache(B, Hk, Hk, G, 2.0, 1, T, pm, pm, ones, ones, group_bounds=gb)
        assert c.prefill(k, k) == 0
        c.perm_v = pm
        kq, _ = numpy_dequantize(c, T)
        return ((kq - k[:, :, :T - 1].astype(np.float64)) ** 2).sum()
    assert key_error(perm, bounds) < 0.5 * key_error(ident, None)


# ---- several query tokens at once (Algorithm 1 with l > 1 on a non-empty cache) ----

def test_multi_token_decode_is_causal_attention_over_the_stored_cache(oracle):
    rng = np.random.default_rng(1500)
    B, Hq, Hk, W, G = 2, 4, 2, 8, 64
    pk, pv = random_perms(rng, Hk), random_perms(rng, Hk)
    clip = rng.uniform(0.8, 1.0, (Hk, D // G)).astype(np.float32)
    for T, n_new in ((45, 3), (45, 8), (6, 4), (8, 1)):
        k = (rng.standard_normal((B, Hk, T, D)) * 10 ** rng.uniform(-1, 1, (1, Hk, 1, D))).astype(np.float16)
        v = (rng.standard_normal((B, Hk, T, D)) * 10 ** rng.uniform(-1, 1, (1, Hk, 1, D))).astype(np.float16)
        q = rng.standard_normal((B, n_new, Hq, D)).astype(np.float16)
        c = oracle.OracleCache(B, Hq, Hk, G, 2.0, W, 64, pk, pv, clip, clip)
        assert c.prefill(k, v) == 0
        out = c.decode_multi(q)
        # the last query token is the single-token decode
        assert np.array_equal(out[:, -1], c.decode(np.ascontiguousarray(q[:, -1])))
        # every query token: the library's attention over the dequantized cache cut at its own position
        nq = max(T - W, 0)
        kq, vq = numpy_dequantize(c, T)
        kfull = np.concatenate([kq, k[:, :, nq:].astype(np.float64)], axis=2)
        vfull = np.concatenate([vq, v[:, :, nq:].astype(np.float64)], axis=2)
        for j in range(n_new):
            Tv = T - n_new + j + 1
            ref = sdpa64(np.ascontiguousarray(q[:, j]), kfull[:, :, :Tv], vfull[:, :, :Tv], 1 / np.sqrt(D))
            assert np.abs(out[:, j] - ref).max() < 1e-5 * max(1.0, np.abs(ref).max())
        if T <= W:      # nothing packed: the last rows of the prompt's own causal attention
            qfull = np.zeros((B, Hq, T, D), np.float16)
            qfull[:, :, T - n_new:] = q.transpose(0, 2, 1, 3)
            pa = c.prefill_attention(qfull, k, v)
            assert np.abs(out - pa[:, :, T - n_new:].transpose(0, 2, 1, 3)).max() < 1e-5
    with pytest.raises(RuntimeError):       # more new tokens than the window holds
        c.decode_multi(rng.standard_normal((B, 9, Hq, D)).astype(np.float16))

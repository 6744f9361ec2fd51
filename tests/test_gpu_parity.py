"""GPU parity: the HIP library against the CPU oracle on the same seeded inputs, through the
C ABI.  Codes, (scale, zero) and ring contents must match bit for bit; attention outputs
within 2e-3 max-abs (fp32 outputs)."""
import dataclasses

import numpy as np
import pytest
import torch

from paper_2405_06219_amd import synth

pytestmark = pytest.mark.gpu

D = 128


@pytest.fixture(scope="module")
def P():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import parity_util
    return parity_util


def small(name, **kw):
    base = dict(name=name, batch=1, n_q_heads=4, n_kv_heads=4, context=700, v_bits=1.5, group_size=128,
                window=128, seed=77)
    base.update(kw)
    return synth.Workload(**base)


QUANT_CASES = [
    small("mha_t15_g128"),
    small("mha_v2_g128", v_bits=2.0, channel_profile="outlier4", perm_stat="absmax"),
    small("gqa_t15_g64", n_q_heads=8, n_kv_heads=2, group_size=64, batch=2, context=391),
    small("gqa_v2_g32", n_q_heads=8, n_kv_heads=2, group_size=32, v_bits=2.0, context=333, window=16),
    small("short_window_only", context=100),
    small("one_quantized_token", context=129),
    small("w1", window=1, context=70),
    # 4-bit codes (Table 1's 4-bit setting), alone and mixed with the narrower formats
    small("k4v4_g128", k_bits=4.0, v_bits=4.0),
    small("k4v4_gqa_g64", k_bits=4.0, v_bits=4.0, n_q_heads=8, n_kv_heads=2, group_size=64, batch=2, context=391),
    small("k4v4_g32_w16", k_bits=4.0, v_bits=4.0, n_q_heads=8, n_kv_heads=2, group_size=32, context=333, window=16),
    small("k4v2_outlier", k_bits=4.0, v_bits=2.0, channel_profile="outlier4", perm_stat="absmax"),
    small("k4_t15_g64", k_bits=4.0, v_bits=1.5, group_size=64, context=300),
    small("k2v4_g32", k_bits=2.0, v_bits=4.0, group_size=32, context=450),
    # 3-bit codes (Table 1's 3-bit setting)
    small("k3v3_g128", k_bits=3.0, v_bits=3.0),
    small("k3v3_gqa_g64_b2", k_bits=3.0, v_bits=3.0, n_q_heads=8, n_kv_heads=2, group_size=64, batch=2, context=391),
    small("k3v3_g32_w16_outlier", k_bits=3.0, v_bits=3.0, n_q_heads=8, n_kv_heads=2, group_size=32, context=333, window=16,
          channel_profile="outlier4", perm_stat="absmax"),
]


@pytest.mark.parametrize("w", QUANT_CASES, ids=lambda w: w.name)
def test_prefill_codes_and_meta_bit_exact(P, w):
    print("case", w, flush=True)
    pair, k, v, q = P.make_pair(w, extra_tokens=40)
    pair.prefill(k, v)
    pair.assert_buffers_equal()


@pytest.mark.parametrize("w", [QUANT_CASES[0], QUANT_CASES[2], QUANT_CASES[3], small("from_empty", context=0, window=8),
                               QUANT_CASES[8], QUANT_CASES[9], QUANT_CASES[10], QUANT_CASES[12],
                               small("k4v4_from_empty", k_bits=4.0, v_bits=4.0, context=0, window=8),
                               QUANT_CASES[13], QUANT_CASES[14], QUANT_CASES[15],
                               small("k3v3_from_empty", k_bits=3.0, v_bits=3.0, context=0, window=8)],
                         ids=lambda w: w.name)
def test_append_evicts_bit_exact_and_equals_longer_prefill(P, w):
    print("case", w, flush=True)
    n = 75
    pair, k, v, q = P.make_pair(w, extra_tokens=n)
    if w.context:
        pair.prefill(k, v)
    for s in range(n):
        kn, vn = synth.make_new_token(w, s)
        pair.append(kn, vn)
        if s in (0, 1, 7, 8, 31, 32, 33, n - 1):
            pair.assert_buffers_equal()


def test_encoder_special_values_bit_exact(P):
    """Constant groups, signed zeros, tiny and large magnitudes, exact ties."""
    w = small("special", n_q_heads=2, n_kv_heads=2, context=8 + 64, window=8, group_size=32, v_bits=1.5)
    rng = np.random.default_rng(9)
    T = w.context
    k = rng.standard_normal((1, 2, T, D)).astype(np.float16)
    v = rng.standard_normal((1, 2, T, D)).astype(np.float16)
    k[0, 0, 0] = 3.0                       # constant -> scale 0
    v[0, 0, 0] = -2.5
    k[0, 0, 1, ::2], k[0, 0, 1, 1::2] = -0.0, 0.0
    v[0, 0, 1] = -0.0
    k[0, 0, 2] = (rng.integers(0, 4, D) * 0.5).astype(np.float16)      # exact grid and ties
    v[0, 0, 2] = (rng.integers(0, 5, D) * 0.25).astype(np.float16)
    k[0, 1, 3] = (rng.standard_normal(D) * 6e-6).astype(np.float16)    # fp16 subnormals
    v[0, 1, 3] = (rng.standard_normal(D) * 2e4).astype(np.float16)     # near the top of fp16
    k[0, 1, 4, :64] = 0.0
    v[0, 1, 5] = np.float16(65504.0) * np.sign(rng.standard_normal(D)).astype(np.float16)
    pk = np.stack([rng.permutation(D) for _ in range(2)]).astype(np.int32)
    pv = np.stack([rng.permutation(D) for _ in range(2)]).astype(np.int32)
    ck = rng.uniform(0.5, 1.0, (2, 4)).astype(np.float32)
    cv = rng.uniform(0.5, 1.0, (2, 4)).astype(np.float32)
    pair = P.Pair(w, 96, pk, pv, ck, cv)
    pair.prefill(k, v)
    pair.assert_buffers_equal()


@pytest.mark.parametrize("bits,vals", [(2.0, (0.0, 37.5, 45.0, 15.0, 30.0)), (4.0, (0.0, 45.5, 105.0, 87.5, 101.5, 7.0))])
def test_encoder_reciprocal_ties_bit_exact(P, bits, vals):
    """Groups whose step h has an inexact reciprocal and whose values sit exactly on a tie of (x - z)/h:
    (x - z) * fl(1/h) lands on the other side (codes worked out in the oracle's pin of this reading)."""
    w = small("recip_ties", n_q_heads=2, n_kv_heads=2, context=8 + 40, window=8, group_size=32, v_bits=bits, k_bits=bits)
    rng = np.random.default_rng(19)
    T = w.context
    k = np.zeros((1, 2, T, D), np.float16)
    v = np.zeros((1, 2, T, D), np.float16)
    for t in range(T):
        for h in range(2):
            scale = np.float16(2.0 ** int(rng.integers(-6, 3)))     # power-of-two scalings keep the ties
            k[0, h, t] = rng.choice(np.array(vals, np.float16), D) * scale
            v[0, h, t] = rng.choice(np.array(vals, np.float16), D) * scale
    ident = np.tile(np.arange(D, dtype=np.int32), (2, 1))
    ones = np.ones((2, 4), np.float32)
    pair = P.Pair(w, 64, ident, ident, ones, ones)
    pair.prefill(k, v)
    pair.assert_buffers_equal()


DECODE_CASES = [
    small("mha_t15", context=1500),
    small("mha_v2_outlier", v_bits=2.0, channel_profile="outlier4", perm_stat="absmax", context=2048),
    small("gqa4_t15", n_q_heads=16, n_kv_heads=4, context=1333, batch=2),
    small("gqa4_v2", n_q_heads=8, n_kv_heads=2, context=999, v_bits=2.0),
    small("gqa2_t15", n_q_heads=8, n_kv_heads=4, context=2100),
    small("gqa2_v2_w512", n_q_heads=4, n_kv_heads=2, v_bits=2.0, window=512, context=3000),
    small("mha_t15_w33", window=33, context=5000, batch=3),
    small("gqa2_g64", n_q_heads=4, n_kv_heads=2, group_size=64, context=611),
    small("gqa4_g32_t15", n_q_heads=8, n_kv_heads=2, group_size=32, context=5000),
    small("gqa4_g64_v2", n_q_heads=16, n_kv_heads=4, group_size=64, v_bits=2.0, context=3000),
    small("mha_g64_t15_b2", group_size=64, context=9000, batch=2),
    small("gqa2_g32_v2", n_q_heads=4, n_kv_heads=2, group_size=32, v_bits=2.0, context=2500, window=40),
    small("gqa8_g32_v2", n_q_heads=8, n_kv_heads=1, group_size=32, v_bits=2.0, context=450, window=16),
    small("gqa8_t15", n_q_heads=16, n_kv_heads=2, context=2300, batch=2),
    small("gqa3_t15", n_q_heads=6, n_kv_heads=2, context=1900),
    small("gqa5_v2_g64", n_q_heads=5, n_kv_heads=1, group_size=64, v_bits=2.0, context=1500),
    small("gqa6_t15", n_q_heads=12, n_kv_heads=2, context=1000),
    small("gqa7_t15_g32", n_q_heads=7, n_kv_heads=1, group_size=32, context=800),
    small("mha_g32_t15", group_size=32, context=300),
    # 4-bit codes
    small("k4v4_mha", k_bits=4.0, v_bits=4.0, context=1500),
    small("k4v4_gqa4_b2", k_bits=4.0, v_bits=4.0, n_q_heads=16, n_kv_heads=4, context=1333, batch=2),
    small("k4v4_gqa2_g64", k_bits=4.0, v_bits=4.0, n_q_heads=8, n_kv_heads=4, group_size=64, context=2100),
    small("k4v4_gqa8_g32", k_bits=4.0, v_bits=4.0, n_q_heads=8, n_kv_heads=1, group_size=32, context=3000, window=16),
    small("k4v4_gqa5_outlier", k_bits=4.0, v_bits=4.0, n_q_heads=5, n_kv_heads=1, context=5000,
          channel_profile="outlier4", perm_stat="absmax"),
    small("k4v2_gqa4", k_bits=4.0, v_bits=2.0, n_q_heads=8, n_kv_heads=2, context=999),
    small("k4_t15_g32", k_bits=4.0, v_bits=1.5, n_q_heads=4, n_kv_heads=2, group_size=32, context=2500, window=40),
    small("k2v4_g64_b3", k_bits=2.0, v_bits=4.0, group_size=64, context=5000, window=33, batch=3),
    small("k4v4_one_packed_row", k_bits=4.0, v_bits=4.0, context=129),
    # 3-bit codes
    small("k3v3_mha", k_bits=3.0, v_bits=3.0, context=1500),
    small("k3v3_gqa4_b2", k_bits=3.0, v_bits=3.0, n_q_heads=16, n_kv_heads=4, context=1333, batch=2),
    small("k3v3_gqa2_g64", k_bits=3.0, v_bits=3.0, n_q_heads=8, n_kv_heads=4, group_size=64, context=2100),
    small("k3v3_gqa8_g32", k_bits=3.0, v_bits=3.0, n_q_heads=8, n_kv_heads=1, group_size=32, context=3000, window=16),
    small("k3v3_gqa6_outlier", k_bits=3.0, v_bits=3.0, n_q_heads=6, n_kv_heads=1, context=5000,
          channel_profile="outlier4", perm_stat="absmax"),
    small("k3v3_one_packed_row", k_bits=3.0, v_bits=3.0, context=129),
    small("window_only", context=77),
    small("exactly_window", context=128),
    small("one_packed_row", context=129),
    small("single_token", context=1),
]


@pytest.mark.parametrize("w", DECODE_CASES, ids=lambda w: w.name)
def test_decode_attention_matches_oracle(P, w):
    print("case", w, flush=True)
    pair, k, v, q = P.make_pair(w)
    pair.prefill(k, v)
    (out, out16), (ref, ref16) = pair.decode_both(q, want_f16=True)
    err = np.abs(out - ref).max()
    P.log(f"decode {w.name}: max abs err {err:.3e} (ref max {np.abs(ref).max():.3f})")
    assert err <= P.TOL
    assert np.abs(out16.astype(np.float32) - out).max() <= 2.0 ** -11 * np.abs(out).max() + 1e-7


def test_decode_is_independent_of_the_split_count(P):
    w = small("splits", n_q_heads=8, n_kv_heads=2, context=128 + 64 * 37 + 5)
    pair, k, v, q = P.make_pair(w)
    pair.prefill(k, v)
    ref = pair.ref.decode(q)
    qd = torch.from_numpy(q).cuda()
    outs = []
    for s in (1, 2, 3, 7, 37, 38, 128):
        pair.gpu.skvq_set_num_splits(s)
        o = pair.gpu.skvq_decode_attention(qd).cpu().numpy()
        P.log(f"splits {s}: max abs err {np.abs(o - ref).max():.3e}")
        assert np.abs(o - ref).max() <= P.TOL, s
        outs.append(o)
    assert max(np.abs(o - outs[0]).max() for o in outs) <= 5e-4


MERGE_CASES = [
    (small("merge_gqa4_hk8", n_q_heads=32, n_kv_heads=8, context=9000), (1, 8, 24, 128)),
    (small("merge_mha_hk8_b2_v2", n_q_heads=8, n_kv_heads=8, context=2500, batch=2, v_bits=2.0), (1, 32)),
    (small("merge_gqa6_two_passes", n_q_heads=24, n_kv_heads=4, context=3000, group_size=64), (1, 40)),
    (small("merge_k4v4_hk16", n_q_heads=32, n_kv_heads=16, context=1200, k_bits=4.0, v_bits=4.0), (1, 16)),
]


@pytest.mark.parametrize("w,splits", MERGE_CASES, ids=[c[0].name for c in MERGE_CASES])
def test_one_chunk_writes_the_output_itself_and_many_chunks_are_merged(P, w, splits):
    """A kv head read as one chunk (no merge launch: the chunk's workgroup writes the output) and as many
    chunks (merge launch, up to 128 partials): outputs against the oracle and against each other, the
    fp16 copy too, also with the fp16 workspace poisoned in between; then the one-call step."""
    print("case", w, splits, flush=True)
    pair, k, v, q = P.make_pair(w, extra_tokens=8)
    pair.prefill(k, v)
    qd = torch.from_numpy(q).cuda()
    ref = pair.ref.decode(q)
    outs = []
    for n in splits:
        pair.gpu.skvq_set_num_splits(n)
        pair.gpu.buffers["workspace"].fill_(0xFF)       # NaN patterns: nothing may be read before it is written
        o16 = torch.zeros(q.shape, dtype=torch.float16, device="cuda")
        out = pair.gpu.skvq_decode_attention(qd, out_f16=o16)
        torch.cuda.synchronize()
        outs.append(out.cpu().numpy())
        assert np.abs(outs[-1] - ref).max() <= P.TOL, n
        assert np.array_equal(o16.cpu().numpy(), outs[-1].astype(np.float16))
        assert np.abs(outs[-1] - outs[0]).max() <= 1e-5 * max(1.0, np.abs(ref).max())
    for n in (1, splits[-1]):
        pair.gpu.skvq_set_num_splits(n)
        for s_ in range(2):
            out, ref2 = pair.append_decode_both(*synth.make_new_token(w, s_ if n == 1 else 2 + s_), q)
            assert np.abs(out - ref2).max() <= P.TOL
    pair.assert_buffers_equal()


@pytest.mark.parametrize("G,meta", [(32, "f32"), (64, "e4m3")])
def test_decode_with_small_groups_is_independent_of_the_split_count(P, G, meta):
    w = small("splits_g", n_q_heads=8, n_kv_heads=2, group_size=G, context=128 + 64 * 41 + 17)
    pair, k, v, q = P.make_pair(w, meta=meta, n_sink=2)
    pair.prefill(k, v)
    ref = pair.ref.decode(q)
    qd = torch.from_numpy(q).cuda()
    for s in (1, 2, 5, 41, 128):
        pair.gpu.skvq_set_num_splits(s)
        o = pair.gpu.skvq_decode_attention(qd).cpu().numpy()
        P.log(f"G {G} splits {s}: max abs err {np.abs(o - ref).max():.3e}")
        assert np.abs(o - ref).max() <= P.TOL, s


def test_decode_after_appends_and_peaked_softmax(P):
    """Appends move tokens from the ring into the packed region; a large softmax scale makes
    one token dominate (the worst case for rounding of the weights)."""
    w = small("peaked", n_q_heads=8, n_kv_heads=2, context=900)
    pair, k, v, q = P.make_pair(w, extra_tokens=50, sm_scale=0.6)
    pair.prefill(k, v)
    for s in range(50):
        pair.append(*synth.make_new_token(w, s))
    pair.assert_buffers_equal()
    out, ref = pair.decode_both(q)
    P.log(f"peaked: max abs err {np.abs(out - ref).max():.3e} (ref max {np.abs(ref).max():.3f})")
    assert np.abs(out - ref).max() <= P.TOL


# ---- one decode step as one call: the new token is appended inside the attention launch ----
STEP_CASES = [
    # (workload, cache options, forced chunks per kv head: from four on the step is one launch)
    (small("step_mha_t15", context=700), {}, 4),
    (small("step_from_empty", context=0, window=16), {}, 0),            # ring fills, then the first evictions: two launches
    (small("step_gqa4_v2_g64", n_q_heads=8, n_kv_heads=2, group_size=64, v_bits=2.0, context=391, batch=2), {}, 4),
    (small("step_gqa2_k4v4_g32_w16", k_bits=4.0, v_bits=4.0, n_q_heads=4, n_kv_heads=2, group_size=32, context=333, window=16), {}, 5),
    (small("step_gqa3_k3v3", k_bits=3.0, v_bits=3.0, n_q_heads=6, n_kv_heads=2, context=450), {"meta": "f16"}, 6),
    (small("step_k4_t15_e4m3", k_bits=4.0, v_bits=1.5, group_size=64, context=300), {"meta": "e4m3"}, 4),
    (small("step_k2v4", k_bits=2.0, v_bits=4.0, n_q_heads=2, n_kv_heads=1, context=200), {}, 0),
    (small("step_sinks", n_q_heads=8, n_kv_heads=2, context=120), {"n_sink": 5}, 4),  # sink rows first (two launches), then packed rows
    (small("step_gqa8_two_launches", n_q_heads=8, n_kv_heads=1, context=450, window=16), {}, 4),
    (small("step_uneq_g32", n_q_heads=8, n_kv_heads=2, group_size=32, context=600),
     {"group_bounds": [0, 16, 32, 80, 128]}, 4),
    (small("step_long_b2", group_size=64, context=9000, batch=2), {}, 7),
    (small("step_long_w33", window=33, context=5000, batch=3), {}, 2),   # two chunks: two launches
    (small("step_long_short_last_chunk", n_q_heads=8, n_kv_heads=2, context=13000), {}, 4),  # the last chunk is the shorter one
    (small("step_long_k4v4_g64", k_bits=4.0, v_bits=4.0, n_q_heads=4, n_kv_heads=2, context=14000, group_size=64), {"meta": "f16"}, 4),
    (small("step_long_k3v3_g32", k_bits=3.0, v_bits=3.0, n_q_heads=6, n_kv_heads=2, context=13500, group_size=32), {"meta": "e4m3"}, 4),
    (small("step_long_k2v4_uneq", k_bits=2.0, v_bits=4.0, n_q_heads=4, n_kv_heads=1, context=13000, group_size=32),
     {"group_bounds": [0, 16, 32, 80, 128]}, 4),
    (small("step_long_sinks_b2", k_bits=4.0, v_bits=1.5, n_q_heads=2, n_kv_heads=2, context=16000, batch=2), {"n_sink": 5}, 5),
]


@pytest.mark.parametrize("w,kw,splits", STEP_CASES, ids=[c[0].name for c in STEP_CASES])
def test_append_and_attention_in_one_call(P, w, kw, splits):
    """skvq_append_decode_attention step by step against the oracle's append followed by its
    decode: outputs within 2e-3 at every step, every packed byte, (scale, zero) and ring row
    bit-exact along the way (V block and tile boundaries included)."""
    print("case", w, kw, splits, flush=True)
    n = 70
    pair, k, v, q = P.make_pair(w, extra_tokens=n, **kw)
    if w.context:
        pair.prefill(k, v)
    if splits:
        pair.gpu.skvq_set_num_splits(splits)
    rng = np.random.default_rng(77)
    worst = 0.0
    for s in range(n):
        kn, vn = synth.make_new_token(w, s)
        qs = (q * rng.uniform(0.5, 1.5)).astype(np.float16)
        out, ref = pair.append_decode_both(kn, vn, qs)
        worst = max(worst, float(np.abs(out - ref).max()))
        assert np.abs(out - ref).max() <= P.TOL, s
        if s in (0, 1, 7, 8, 15, 16, 31, 32, 33, 63, 64, n - 1):
            pair.assert_buffers_equal()
    P.log(f"one-call step {w.name}: max abs err over {n} steps {worst:.3e}")


def test_one_call_step_equals_the_two_calls(P):
    """The same steps through skvq_quantize_append + skvq_decode_attention on a second cache: the
    packed buffers end up identical bit for bit and the outputs equal to rounding."""
    w = small("step_vs_two", n_q_heads=8, n_kv_heads=2, context=2100)
    pair, k, v, q = P.make_pair(w, extra_tokens=40)
    other, _, _, _ = P.make_pair(w, extra_tokens=40)
    pair.gpu.skvq_set_num_splits(4)   # one launch per step
    other.gpu.skvq_set_num_splits(4)
    pair.prefill(k, v)
    other.gpu.skvq_prefill_quantize(torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda())
    qd = torch.from_numpy(q).cuda()
    for s in range(40):
        kn, vn = (torch.from_numpy(x).cuda() for x in synth.make_new_token(w, s))
        a = pair.gpu.skvq_append_decode_attention(kn, vn, qd)
        other.gpu.skvq_quantize_append(kn, vn)
        b = other.gpu.skvq_decode_attention(qd)
        torch.cuda.synchronize()
        assert float((a - b).abs().max()) <= 2e-5, s
    for x, y in zip(pair.gpu.host_arrays(), other.gpu.host_arrays()):
        assert np.array_equal(x.view(np.uint8), y.view(np.uint8))


def test_runtime_errors(P):
    w = small("errors", context=300)
    pair, k, v, q = P.make_pair(w, extra_tokens=2)
    B = P.B
    qd = torch.from_numpy(q).cuda()
    with pytest.raises(B.SkvqError) as e:
        pair.gpu.skvq_decode_attention(qd)           # empty cache
    assert e.value.status == B.SKVQ_ERR_STATE
    kd, vd = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
    big_k = torch.zeros((1, 4, 300 + 10, D), dtype=torch.float16, device="cuda")
    with pytest.raises(B.SkvqError) as e:
        pair.gpu.skvq_prefill_quantize(big_k, big_k)  # 310 - 128 rows > capacity 174
    assert e.value.status == B.SKVQ_ERR_CAPACITY
    pair.gpu.skvq_prefill_quantize(kd, vd)
    x = torch.zeros((1, 4, D), dtype=torch.float16, device="cuda")
    pair.gpu.skvq_quantize_append(x, x)
    pair.gpu.skvq_quantize_append(x, x)
    with pytest.raises(B.SkvqError) as e:
        pair.gpu.skvq_quantize_append(x, x)
    assert e.value.status == B.SKVQ_ERR_CAPACITY
    assert pair.gpu.skvq_get_state() == (302, 174, 128)
    torch.cuda.synchronize()
    # an empty prompt empties the cache; the first tokens then arrive one by one
    assert B.lib().skvq_prefill_quantize(pair.gpu._h, None, None, 0, None) == B.SKVQ_OK
    assert pair.gpu.skvq_get_state() == (0, 0, 0)
    with pytest.raises(B.SkvqError) as e:
        pair.gpu.skvq_decode_attention(qd)
    assert e.value.status == B.SKVQ_ERR_STATE
    pair.gpu.skvq_append_decode_attention(x, x, qd)
    assert pair.gpu.skvq_get_state() == (1, 0, 1)
    torch.cuda.synchronize()


def test_set_state_adopts_buffers_and_refuses_a_rewind(P):
    """skvq_set_state: a second cache whose buffers are copies of a filled cache's, told the token
    count, continues exactly like the first (appends, sink rows and attention against the oracle);
    a count below the current one is refused (SKVQ_ERR_STATE) and changes nothing."""
    B = P.B
    w = small("adopt", n_q_heads=8, n_kv_heads=2, context=300, window=16, v_bits=1.5)
    S = 3
    pair, k, v, q = P.make_pair(w, extra_tokens=40, n_sink=S)
    pair.prefill(k, v)
    for s in range(5):
        pair.append(*synth.make_new_token(w, s))
    torch.cuda.synchronize()
    other = B.SkvqCache(w.batch, w.n_q_heads, w.n_kv_heads, w.group_size, w.v_bits, w.window,
                        pair.gpu.cfg.max_quant_tokens, pair.gpu._keep[0], pair.gpu._keep[1], pair.gpu._keep[2],
                        pair.gpu._keep[3], n_sink=S, k_bits=w.k_bits, fill=0x5C)
    for name in B.BUFFER_NAMES[:6]:
        other.buffers[name].copy_(pair.gpu.buffers[name])
    n_now = pair.gpu.skvq_get_state()[0]
    with pytest.raises(B.SkvqError) as e:
        other.skvq_set_state(10 ** 9)                    # cannot fit
    assert e.value.status == B.SKVQ_ERR_CAPACITY and other.skvq_get_state() == (0, 0, 0)
    other.skvq_set_state(n_now)
    assert other.skvq_get_state() == pair.gpu.skvq_get_state()
    with pytest.raises(B.SkvqError) as e:
        other.skvq_set_state(n_now - 1)                  # no rewind
    assert e.value.status == B.SKVQ_ERR_STATE and other.skvq_get_state() == pair.gpu.skvq_get_state()
    other.skvq_set_state(n_now)                          # the same count again is fine
    pair.gpu = other                                     # from here on the adopted cache is the one compared
    for s in range(5, 40):
        pair.append(*synth.make_new_token(w, s))
    pair.assert_buffers_equal()
    out, ref = pair.decode_both(q)
    assert np.abs(out - ref).max() <= P.TOL
    out, ref = pair.append_decode_both(*synth.make_new_token(w, 40), q)
    assert np.abs(out - ref).max() <= P.TOL
    pair.assert_buffers_equal()


def test_full_size_c3_in_the_benchmarked_launch_configuration(P):
    """Mistral-7B-shaped layer at 131072 tokens (the benchmark's workload, library-chosen split
    count): every packed byte, every (scale, zero) and the ring bit-exact against the oracle's
    own prefill of the same seeded inputs, after appends too; attention outputs within 2e-3."""
    w = synth.WORKLOADS["c3_mistral7b_128k"]
    P.log(f"full size: generating {w.name}")
    pair, k, v, q = P.make_pair(w, extra_tokens=4)
    P.log("full size: prefill (oracle + gpu)")
    pair.prefill(k, v)
    del k, v
    for s in range(3):
        pair.append(*synth.make_new_token(w, s))
    pair.assert_buffers_equal()
    P.log("full size: decode (oracle + gpu)")
    out, ref = pair.decode_both(q)
    err = np.abs(out - ref).max()
    P.log(f"full size c3: max abs err {err:.3e} (ref max {np.abs(ref).max():.3f})")
    assert err <= P.TOL
    P.log("full size: one-call step (oracle + gpu)")
    out, ref = pair.append_decode_both(*synth.make_new_token(w, 3), q)
    err = np.abs(out - ref).max()
    P.log(f"full size c3, append + attention in one call: max abs err {err:.3e}")
    assert err <= P.TOL
    pair.assert_buffers_equal()


@pytest.mark.parametrize("name,n_heads,bits", [("c1_mha4_2k", 8, None), ("c2_llama7b_32k", 3, None),
                                               ("c5_batch16_32k", 4, None), ("c4_llama7b_1m", 2, None),
                                               ("c3_mistral7b_128k", 3, (4.0, 4.0)),
                                               ("c3_mistral7b_128k", 2, (3.0, 3.0))])
def test_full_size_sampled_heads(P, name, n_heads, bits):
    """The batch-16 and the 1M-token workloads (and the 128k one with 4-bit keys and values) at
    full size, library-chosen split count: the
    whole layer is prefilled, appended to and attended on the GPU; for seeded sampled
    (sequence, kv head) pairs the oracle builds that head's cache from the same inputs and
    must agree bit for bit on every packed byte, (scale, zero) and ring entry of the head and
    within 2e-3 on the outputs of its query heads."""
    from oracle import skvq_oracle as O
    from paper_2405_06219_amd import binding as B

    w = synth.WORKLOADS[name]
    if bits:
        w = dataclasses.replace(w, k_bits=bits[0], v_bits=bits[1])
        name = f"{name}_k{bits[0]:g}v{bits[1]:g}"
    dev = torch.device("cuda:0")
    P.log(f"{name}: generating on the device")
    k, v, pk, pv = synth.make_kv_device(w, dev)
    ck, cv = synth.make_clip(w)
    n_app = 3
    tcap = w.context - w.window + n_app + 1
    gpu = B.SkvqCache(w.batch, w.n_q_heads, w.n_kv_heads, w.group_size, w.v_bits, w.window, tcap, pk, pv, ck, cv,
                      fill=0xAB, device=dev, k_bits=w.k_bits)
    gpu.skvq_prefill_quantize(k, v)
    news = [synth.make_new_token(w, s) for s in range(n_app)]
    for kn, vn in news:
        gpu.skvq_quantize_append(torch.from_numpy(kn).to(dev), torch.from_numpy(vn).to(dev))
    q = synth.make_query(w)
    out = gpu.skvq_decode_attention(torch.from_numpy(q).to(dev))
    torch.cuda.synchronize()
    out = out.cpu().numpy()
    P.log(f"{name}: gpu done ({gpu.skvq_get_state()})")

    R = w.n_q_heads // w.n_kv_heads
    ng = D // w.group_size
    vb = {1.5: 832, 2.0: 1024, 3.0: 1536, 4.0: 2048}[w.v_bits]
    views = {"k_codes": gpu.buffers["k_codes"].view(w.batch, w.n_kv_heads, tcap, {2.0: 32, 3.0: 48, 4.0: 64}[w.k_bits]),
             "v_codes": gpu.buffers["v_codes"].view(w.batch, w.n_kv_heads, (tcap + 31) // 32, vb),
             "k_meta": gpu.buffers["k_meta"].view(torch.float32).view(w.batch, w.n_kv_heads, tcap, ng, 2),
             "v_meta": gpu.buffers["v_meta"].view(torch.float32).view(w.batch, w.n_kv_heads, tcap, ng, 2),
             "k_win": gpu.buffers["k_win"].view(torch.int16).view(w.batch, w.n_kv_heads, w.window, D),
             "v_win": gpu.buffers["v_win"].view(torch.int16).view(w.batch, w.n_kv_heads, w.window, D)}
    rng = np.random.default_rng(w.seed)
    picks = {(int(rng.integers(w.batch)), int(rng.integers(w.n_kv_heads))) for _ in range(n_heads)}
    picks.add((w.batch - 1, w.n_kv_heads - 1))
    worst = 0.0
    for b, hk in sorted(picks):
        ref = O.OracleCache(1, R, 1, w.group_size, w.v_bits, w.window, tcap, pk[hk:hk + 1], pv[hk:hk + 1],
                            ck[hk:hk + 1], cv[hk:hk + 1], fill=0xAB, k_bits=w.k_bits)
        assert ref.prefill(k[b:b + 1, hk:hk + 1].cpu().numpy(), v[b:b + 1, hk:hk + 1].cpu().numpy()) == 0
        for kn, vn in news:
            assert ref.append(np.ascontiguousarray(kn[b:b + 1, hk:hk + 1]), np.ascontiguousarray(vn[b:b + 1, hk:hk + 1])) == 0
        for nm, r in zip(["k_codes", "v_codes", "k_meta", "v_meta", "k_win", "v_win"], ref.arrays()):
            g = views[nm][b, hk].cpu().numpy()
            r = r[0, 0]
            if nm.endswith("meta"):
                g, r = g.view(np.uint32), r.view(np.uint32)
            elif nm.endswith("win"):
                g = g.view(np.uint16)
            if not np.array_equal(g, r):
                bad = np.argwhere(g != r)
                raise AssertionError(f"{name} head ({b},{hk}) {nm}: {len(bad)} mismatches, first at {bad[0].tolist()}")
        o_ref = ref.decode(np.ascontiguousarray(q[b:b + 1, hk * R:(hk + 1) * R]))
        err = np.abs(out[b, hk * R:(hk + 1) * R] - o_ref[0]).max()
        worst = max(worst, float(err))
        P.log(f"{name} head ({b},{hk}): buffers bit-exact, max abs err {err:.3e} (ref max {np.abs(o_ref).max():.3f})")
    del k, v
    assert worst <= P.TOL


# ---- attention sinks (the filter rule of Section 3.2 / Algorithm 1): the first S tokens stay fp16 ----

SINK_CASES = [
    (small("sink5_gqa4_t15", n_q_heads=16, n_kv_heads=4, context=1333, batch=2), 5),
    (small("sink5_mha_v2", v_bits=2.0, context=900), 5),
    (small("sink3_gqa2_g64", n_q_heads=4, n_kv_heads=2, group_size=64, context=611), 3),
    (small("sink1_w16_g32", n_q_heads=8, n_kv_heads=1, group_size=32, v_bits=2.0, context=450, window=16), 1),
    (small("sink_larger_than_old_part", context=140), 40),
    (small("sink_window_only", context=77), 5),
    (small("sink130_gqa4", n_q_heads=8, n_kv_heads=2, context=700), 130),
]


@pytest.mark.parametrize("w,S", SINK_CASES, ids=lambda x: x.name if hasattr(x, "name") else str(x))
def test_sinks_prefill_bit_exact_and_decode_matches_oracle(P, w, S):
    print("case", w, S, flush=True)
    pair, k, v, q = P.make_pair(w, extra_tokens=8, n_sink=S)
    pair.prefill(k, v)
    pair.assert_buffers_equal()
    assert pair.gpu.skvq_get_state()[1] == max(w.context - w.window - S, 0)
    out, ref = pair.decode_both(q)
    err = np.abs(out - ref).max()
    P.log(f"decode {w.name} S={S}: max abs err {err:.3e} (ref max {np.abs(ref).max():.3f})")
    assert err <= P.TOL


@pytest.mark.parametrize("T0", [0, 5, 130, 133, 200])
def test_sinks_appends_walk_ring_then_sink_rows_then_packed_rows(P, T0):
    """Appends from T0 tokens on: tokens leave the window into the sink rows (the first five) and
    into packed rows (the others); buffers stay bit-exact and attention matches at every stage."""
    S, n = 5, 150
    w = small("sink_append", n_q_heads=8, n_kv_heads=2, context=T0)
    pair, k, v, q = P.make_pair(w, extra_tokens=n + 128, n_sink=S)
    if T0:
        pair.prefill(k, v)
    for s in range(n):
        pair.append(*synth.make_new_token(w, s))
        if s in (0, 1, 2, 3, 4, 5, 6, 127, 128, 129, 132, 133, 134, n - 1):
            pair.assert_buffers_equal()
            out, ref = pair.decode_both(q)
            assert np.abs(out - ref).max() <= P.TOL, s
    # capacity counts packed rows only
    tight = P.Pair(w, 3, *synth.make_permutations(w, *synth.make_kv(w, n_tokens=64)), *synth.make_clip(w), n_sink=S)
    x = torch.zeros((1, 2, D), dtype=torch.float16, device="cuda")
    for _ in range(128 + S + 3):
        tight.gpu.skvq_quantize_append(x, x)
    with pytest.raises(P.B.SkvqError) as e:
        tight.gpu.skvq_quantize_append(x, x)
    assert e.value.status == P.B.SKVQ_ERR_CAPACITY
    torch.cuda.synchronize()


# ---- compact (scale, zero): fp16 and FP8 E4M3 storage (Section 4.1; Section 4.3's bit accounting) ----

META_CASES = [
    (small("e4m3_gqa4_t15", n_q_heads=16, n_kv_heads=4, context=1333, batch=2), "e4m3", 5),
    (small("f16_gqa4_t15", n_q_heads=16, n_kv_heads=4, context=1333, batch=2), "f16", 0),
    (small("e4m3_mha_v2_outlier", v_bits=2.0, channel_profile="outlier4", perm_stat="absmax", context=2048), "e4m3", 0),
    (small("f16_gqa2_v2", n_q_heads=4, n_kv_heads=2, v_bits=2.0, context=999), "f16", 3),
    (small("e4m3_gqa2_g64", n_q_heads=4, n_kv_heads=2, group_size=64, context=611), "e4m3", 0),
    (small("f16_gqa8_g32_v2", n_q_heads=8, n_kv_heads=1, group_size=32, v_bits=2.0, context=450, window=16), "f16", 1),
    (small("e4m3_mha_g32_t15", group_size=32, context=300), "e4m3", 0),
]


# ---- general filter rules: the caller decides which tokens stay fp16 when they leave the window ----
FILTER_CASES = [
    (small("filter_gqa4_t15", n_q_heads=8, n_kv_heads=2, context=700), {}, 9, 0.01),
    (small("filter_k4v4_g32_b2", k_bits=4.0, v_bits=4.0, group_size=32, context=391, batch=2), {"meta": "f16"}, 16, 0.03),
    (small("filter_k3v3_w16", k_bits=3.0, v_bits=3.0, n_q_heads=4, n_kv_heads=1, context=333, window=16), {}, 7, 0.015),
    (small("filter_v2_uneq", v_bits=2.0, n_q_heads=4, n_kv_heads=2, group_size=64, context=600),
     {"group_bounds": [0, 48, 128], "meta": "e4m3"}, 12, 0.01),
    (small("filter_long", n_q_heads=8, n_kv_heads=2, context=5000), {}, 40, 0.005),
    (small("filter_from_empty", context=0, window=16), {}, 6, 0.0),
]


@pytest.mark.parametrize("w,kw,S,frac", FILTER_CASES, ids=[c[0].name for c in FILTER_CASES])
def test_filter_mask_prefill_appends_and_attention(P, w, kw, S, frac):
    """A seeded mask over the prompt's old tokens, then appends with a decision per step (kept while rows are
    free): every packed byte, (scale, zero), ring and kept row bit-exact, attention within 2e-3 along the way;
    a kept token beyond the rows is refused and leaves the cache unchanged."""
    print("case", w, kw, S, frac, flush=True)
    n = 60
    pair, k, v, q = P.make_pair(w, extra_tokens=n, n_sink=S, **kw)
    rng = np.random.default_rng(99)
    if w.context:
        keep = rng.random(max(w.context - w.window, 0)) < frac
        keep[:2] = True
        while keep.sum() > S - 3:
            keep[np.flatnonzero(keep)[-1]] = False
        pair.prefill_filtered(k, v, keep)
        pair.assert_buffers_equal()
        out, ref = pair.decode_both(q)
        assert np.abs(out - ref).max() <= P.TOL
    used = int(pair.gpu.skvq_get_state()[0] - pair.gpu.skvq_get_state()[1] - pair.gpu.skvq_get_state()[2])
    for s in range(n):
        leaving = pair.ref.n_tokens >= w.window
        want = bool(s % 7 == 3) and used < S
        pair.append_filtered(*synth.make_new_token(w, s), want)
        used += int(want and leaving)
        if s in (0, 3, 4, 10, 17, 31, 32, 33, n - 1):
            pair.assert_buffers_equal()
            out, ref = pair.decode_both(q)
            assert np.abs(out - ref).max() <= P.TOL, s
    # fill the kept rows, then one more kept token must be refused
    s = n
    while used < S:
        leaving = pair.ref.n_tokens >= w.window
        pair.append_filtered(*synth.make_new_token(w, s), True)
        used += int(leaving)
        s += 1
    state = pair.gpu.skvq_get_state()
    kn, vn = (torch.from_numpy(x).cuda() for x in synth.make_new_token(w, s))
    with pytest.raises(P.B.SkvqError) as e:
        pair.gpu.skvq_quantize_append_filtered(kn, vn, True)
    assert e.value.status == P.B.SKVQ_ERR_CAPACITY and pair.gpu.skvq_get_state() == state
    # the sink rule's entry points go on from here (no row is free: the token is packed), and so does the one-call step
    pair.append(*synth.make_new_token(w, s))
    out, ref = pair.append_decode_both(*synth.make_new_token(w, s + 1), q)
    assert np.abs(out - ref).max() <= P.TOL
    pair.assert_buffers_equal()


@pytest.mark.parametrize("w,meta,S", META_CASES, ids=lambda x: x.name if hasattr(x, "name") else str(x))
def test_compact_meta_prefill_appends_bit_exact_and_decode_matches_oracle(P, w, meta, S):
    print("case", w, meta, S, flush=True)
    n = 40
    pair, k, v, q = P.make_pair(w, extra_tokens=n, n_sink=S, meta=meta)
    pair.prefill(k, v)
    pair.assert_buffers_equal()
    out, ref = pair.decode_both(q)
    err = np.abs(out - ref).max()
    P.log(f"decode {w.name} meta={meta}: max abs err {err:.3e} (ref max {np.abs(ref).max():.3f})")
    assert err <= P.TOL
    for s in range(n):
        pair.append(*synth.make_new_token(w, s))
    pair.assert_buffers_equal()
    out, ref = pair.decode_both(q)
    assert np.abs(out - ref).max() <= P.TOL


@pytest.mark.parametrize("meta", ["f16", "e4m3"])
def test_compact_meta_special_values_bit_exact(P, meta):
    """Ranges that saturate FP8 (scale or zero beyond 448), that underflow it (scale below
    2^-10 -> 0, codes all 0), ties of the meta rounding, constant and zero groups."""
    rng = np.random.default_rng(5)
    w = small("meta_special", n_q_heads=2, n_kv_heads=2, group_size=32, context=128 + 96)
    T = w.context
    k = (rng.standard_normal((1, 2, T, D)) * 3).astype(np.float16)
    v = (rng.standard_normal((1, 2, T, D)) * 3).astype(np.float16)
    k[0, 0, 0, :] = 0.0
    k[0, 0, 1, :] = 1000.0                      # constant, zero point beyond 448
    k[0, 0, 2, :] = np.linspace(-3000, 3000, D)  # scale beyond 448
    k[0, 0, 3, :] = np.linspace(0, 2e-4, D)      # scale below the smallest FP8 value
    k[0, 0, 4, :] = np.linspace(-6e-5, 6e-5, D)  # fp16 subnormal inputs
    k[0, 1, 5, :32] = np.array([0, 27] * 16)     # scale 27/3 = 9 -> FP8 tie between 9 and 10? (9 is exact)
    k[0, 1, 6, :32] = np.array([0, 25.5] * 16)   # scale 8.5: FP8 tie (8 and 9): to even
    k[0, 1, 7, :] = 65504.0
    k[0, 1, 8, :] = np.where(np.arange(D) % 2, 65504.0, -65504.0)
    v[0, :, :16] = k[0, :, :16]
    pk = np.stack([rng.permutation(D) for _ in range(2)]).astype(np.int32)
    pv = np.stack([rng.permutation(D) for _ in range(2)]).astype(np.int32)
    ck = rng.uniform(0.5, 1.0, (2, 4)).astype(np.float32)
    cv = np.ones((2, 4), np.float32)
    pair = P.Pair(w, 96, pk, pv, ck, cv, meta=meta)
    pair.prefill(k, v)
    pair.assert_buffers_equal()


# ---- unequal groups (Section 4.1): boundaries at multiples of 16 reordered positions ----
UNEQUAL_CASES = [
    (small("uneq_g32_t15", n_q_heads=8, n_kv_heads=2, group_size=32, context=2200), [0, 16, 32, 80, 128], "f32", 0),
    (small("uneq_g32_v2_mha_b2", group_size=32, v_bits=2.0, context=900, batch=2), [0, 48, 64, 112, 128], "f32", 0),
    (small("uneq_g32_k4v4_gqa4", k_bits=4.0, v_bits=4.0, n_q_heads=4, n_kv_heads=1, group_size=32, context=1500),
     [0, 16, 32, 48, 128], "f16", 5),
    (small("uneq_g64_t15_gqa2", n_q_heads=4, n_kv_heads=2, group_size=64, context=3100, window=33), [0, 48, 128], "e4m3", 0),
    (small("uneq_g64_k4v2_gqa8", k_bits=4.0, v_bits=2.0, n_q_heads=8, n_kv_heads=1, group_size=64, context=700),
     [0, 112, 128], "f32", 1),
    (small("uneq_g64_k2v4_gqa3", k_bits=2.0, v_bits=4.0, n_q_heads=6, n_kv_heads=2, group_size=64, context=450, window=16),
     [0, 16, 128], "f32", 0),
    (small("uneq_g32_written_uniform", group_size=32, context=600), [0, 32, 64, 96, 128], "f32", 0),
    (small("uneq_g32_per_head_t15", n_q_heads=8, n_kv_heads=4, group_size=32, context=1300),
     [[0, 16, 32, 80, 128], [0, 32, 64, 96, 128], [0, 64, 96, 112, 128], [0, 16, 32, 48, 128]],
     "f16", 0),
    (small("uneq_g64_per_head_k4v4", k_bits=4.0, v_bits=4.0, n_q_heads=4, n_kv_heads=2, group_size=64, context=800, batch=2),
     [[0, 16, 128], [0, 112, 128]], "f32", 5),
    (small("uneq_g32_k3v3_gqa2", k_bits=3.0, v_bits=3.0, n_q_heads=4, n_kv_heads=2, group_size=32, context=1100),
     [0, 64, 80, 96, 128], "e4m3", 5),
]


@pytest.mark.parametrize("w,bounds,meta,S", UNEQUAL_CASES, ids=lambda x: x.name if hasattr(x, "name") else None)
def test_unequal_groups_prefill_appends_and_decode(P, w, bounds, meta, S):
    """Prefill, a run of appends across V block and sub-block boundaries, then attention: codes,
    (scale, zero) and ring bit-exact; outputs within 2e-3."""
    print("case", w, bounds, meta, S, flush=True)
    n = 41
    pair, k, v, q = P.make_pair(w, extra_tokens=n, n_sink=S, meta=meta, group_bounds=bounds)
    pair.prefill(k, v)
    pair.assert_buffers_equal()
    for s in range(n):
        pair.append(*synth.make_new_token(w, s))
        if s in (0, 7, 8, 31, 32, n - 1):
            pair.assert_buffers_equal()
    out, ref = pair.decode_both(q)
    err = np.abs(out - ref).max()
    P.log(f"unequal groups {w.name} {bounds}: max abs err {err:.3e} (ref max {np.abs(ref).max():.3f})")
    assert err <= P.TOL
    # the split count must not matter
    for splits in (1, 7):
        pair.gpu.skvq_set_num_splits(splits)
        out2, _ = pair.decode_both(q)
        assert np.abs(out2 - ref).max() <= P.TOL


# ---- prefill attention (Section 3.2, phase 1): the prompt's causal attention, full precision ----
PREFILL_ATTN_CASES = [(1, 4, 4, 300), (2, 8, 2, 777), (1, 3, 1, 1000), (1, 2, 2, 1), (1, 2, 1, 64), (1, 8, 1, 128),
                      (3, 2, 2, 129), (1, 5, 5, 2049)]


@pytest.mark.parametrize("B,Hq,Hk,T", PREFILL_ATTN_CASES)
def test_prefill_attention_matches_oracle(P, B, Hq, Hk, T):
    """fp32 outputs against the fp64 oracle, within the 2e-3 of every attention output (the weights
    enter the value product as a high and a low fp16 part); K and V with the channel spread of the
    baseline workloads (scales 0.1 .. 10)."""
    from oracle import skvq_oracle as O
    from paper_2405_06219_amd import binding as Bd
    print("case", B, Hq, Hk, T, flush=True)
    rng = np.random.default_rng(3000 + T)
    q = rng.standard_normal((B, Hq, T, D)).astype(np.float16)
    k = (rng.standard_normal((B, Hk, T, D)) * 10 ** rng.uniform(-1.0, 1.0, (1, Hk, 1, D))).astype(np.float16)
    v = (rng.standard_normal((B, Hk, T, D)) * 10 ** rng.uniform(-1.0, 1.0, (1, Hk, 1, D))).astype(np.float16)
    perm = np.tile(np.arange(D, dtype=np.int32), (Hk, 1))
    one = np.ones((Hk, 1), np.float32)
    ref = O.OracleCache(B, Hq, Hk, 128, 1.5, 8, 8, perm, perm, one, one).prefill_attention(q, k, v)
    gpu = Bd.SkvqCache(B, Hq, Hk, 128, 1.5, 8, 8, perm, perm, one, one)
    dev = "cuda:0"
    o16 = torch.empty((B, Hq, T, D), dtype=torch.float16, device=dev)
    out = gpu.skvq_prefill_attention(torch.from_numpy(q).to(dev), torch.from_numpy(k).to(dev),
                                     torch.from_numpy(v).to(dev), out_f16=o16)
    torch.cuda.synchronize()
    out = out.cpu().numpy()
    err = np.abs(out - ref).max()
    bound = P.TOL
    P.log(f"prefill attention B{B} Hq{Hq} Hk{Hk} T{T}: max abs err {err:.3e} (bound {bound:.3e}, ref max {np.abs(ref).max():.3f})")
    assert err <= bound
    assert np.array_equal(o16.cpu().numpy(), out.astype(np.float16))


@pytest.mark.parametrize("B,Hq,Hk,T", [(1, 32, 8, 32768), (2, 8, 2, 16384 + 77)])
def test_prefill_attention_long_prompt_sampled_rows(P, B, Hq, Hk, T):
    """Prompts of the size that is timed (32 q / 8 kv heads, 32k tokens: 128 workgroups per head,
    up to 512 tiles each) and a ragged one: rows chosen at tile and workgroup edges plus random
    ones, each computed by the oracle one by one; every output must be finite."""
    from oracle import skvq_oracle as O
    from paper_2405_06219_amd import binding as Bd
    print("case", B, Hq, Hk, T, flush=True)
    rng = np.random.default_rng(3100 + T)
    q = rng.standard_normal((B, Hq, T, D), dtype=np.float32).astype(np.float16)
    k = (rng.standard_normal((B, Hk, T, D), dtype=np.float32) * 10 ** rng.uniform(-1.0, 1.0, (1, Hk, 1, D))).astype(np.float16)
    v = (rng.standard_normal((B, Hk, T, D), dtype=np.float32) * 10 ** rng.uniform(-1.0, 1.0, (1, Hk, 1, D))).astype(np.float16)
    perm = np.tile(np.arange(D, dtype=np.int32), (Hk, 1))
    one = np.ones((Hk, 1), np.float32)
    ts = [0, 1, 31, 32, 63, 64, 65, 127, 255, 256, 257, 511, 512, 8191, 8192, T // 2 - 1, T // 2, T - 257, T - 256,
          T - 65, T - 64, T - 33, T - 32, T - 2, T - 1]
    rows = [(int(rng.integers(B)), int(rng.integers(Hq)), t) for t in ts]
    rows += [(int(rng.integers(B)), int(rng.integers(Hq)), int(rng.integers(T))) for _ in range(40)]
    rows += [(B - 1, Hq - 1, T - 1), (0, 0, 0), (B - 1, 0, T - 1), (0, Hq - 1, 255)]
    ref = O.OracleCache(B, Hq, Hk, 128, 1.5, 8, 8, perm, perm, one, one).prefill_attention_rows(q, k, v, rows)
    gpu = Bd.SkvqCache(B, Hq, Hk, 128, 1.5, 8, 8, perm, perm, one, one)
    dev = "cuda:0"
    out = gpu.skvq_prefill_attention(torch.from_numpy(q).to(dev), torch.from_numpy(k).to(dev), torch.from_numpy(v).to(dev))
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all())
    idx = np.asarray(rows)
    got = out[idx[:, 0], idx[:, 1], idx[:, 2]].cpu().numpy()
    err = np.abs(got - ref).max()
    bound = P.TOL
    P.log(f"prefill attention (sampled rows) B{B} Hq{Hq} Hk{Hk} T{T}: {len(rows)} rows, max abs err {err:.3e} (bound {bound:.3e})")
    assert err <= bound


def test_prefill_phase_in_one_call(P):
    """skvq_prefill_attention_quantize: the prompt's attention against the oracle's, the cache against the
    oracle's prefill, then a decode step; a prompt that does not fit is refused with the cache untouched."""
    from oracle import skvq_oracle as O
    w = small("prefill_one_call", n_q_heads=8, n_kv_heads=2, context=777, group_size=64)
    pair, k, v, q = P.make_pair(w, extra_tokens=4, n_sink=3)
    rng = np.random.default_rng(5)
    qp = rng.standard_normal((w.batch, w.n_q_heads, w.context, D)).astype(np.float16)
    ref_attn = pair.ref.prefill_attention(qp, k, v)
    assert pair.ref.prefill(k, v) == 0
    dev = "cuda:0"
    out = pair.gpu.skvq_prefill_attention_quantize(torch.from_numpy(qp).to(dev), torch.from_numpy(k).to(dev),
                                                   torch.from_numpy(v).to(dev))
    torch.cuda.synchronize()
    assert np.abs(out.cpu().numpy() - ref_attn).max() <= P.TOL
    pair.assert_buffers_equal()
    o, r = pair.append_decode_both(*synth.make_new_token(w, 0), q)
    assert np.abs(o - r).max() <= P.TOL
    state = pair.gpu.skvq_get_state()
    big = torch.zeros((w.batch, w.n_kv_heads, w.context + 50, D), dtype=torch.float16, device=dev)
    bigq = torch.zeros((w.batch, w.n_q_heads, w.context + 50, D), dtype=torch.float16, device=dev)
    with pytest.raises(P.B.SkvqError) as e:
        pair.gpu.skvq_prefill_attention_quantize(bigq, big, big)
    assert e.value.status == P.B.SKVQ_ERR_CAPACITY and pair.gpu.skvq_get_state() == state


# ---- the read-only kernel that bench.py prices the decode call against ----

@pytest.mark.gpu
def test_read_yardstick_reads_and_leaves_memory_alone(P):
    """The kernel runs over whole buffers and ragged ones (a tail shorter than the grid's stride),
    changes neither the source nor the sink, and refuses a length that is no multiple of 16."""
    from paper_2405_06219_amd import binding as Bd
    dev = "cuda:0"
    for n_bytes in (16, 4096, 1 << 20, (1 << 20) + 16 * 37, 78065664):
        src = torch.arange(n_bytes // 4, dtype=torch.int32, device=dev)
        want = src.clone()
        sink = torch.full((1,), 0x5A5A5A5A, dtype=torch.int32, device=dev)
        Bd.skvq_read_yardstick(src, sink)
        torch.cuda.synchronize()
        assert torch.equal(src, want) and int(sink.item()) == 0x5A5A5A5A, n_bytes
    with pytest.raises(Bd.SkvqError):
        Bd.skvq_read_yardstick(torch.zeros(5, dtype=torch.int32, device=dev), sink)


@pytest.mark.gpu
def test_read_write_yardstick_writes_the_xor_of_what_it_reads(P):
    """4 KB piece g of the destination is the XOR of the source's pieces g * ratio .. g * ratio + ratio - 1,
    for every ratio the kernel takes; the source stays as it was and nothing is written past the end."""
    from paper_2405_06219_amd import binding as Bd
    dev = "cuda:0"
    gen = torch.Generator(device=dev)
    gen.manual_seed(11)
    for ratio, pieces in ((1, 3), (2, 1), (7, 5), (7, 2500), (8, 129)):
        src = torch.randint(-2**31, 2**31 - 1, (pieces * ratio, 1024), generator=gen, dtype=torch.int32, device=dev)
        keep = src.clone()
        dst = torch.full((pieces + 1, 1024), 0x5A5A5A5A, dtype=torch.int32, device=dev)
        Bd.skvq_read_write_yardstick(src, dst[:pieces], ratio)
        torch.cuda.synchronize()
        want = src.view(pieces, ratio, 1024)[:, 0].clone()
        for j in range(1, ratio):
            want ^= src.view(pieces, ratio, 1024)[:, j]
        assert torch.equal(dst[:pieces], want), (ratio, pieces)
        assert torch.equal(src, keep) and bool((dst[pieces] == 0x5A5A5A5A).all()), (ratio, pieces)
    with pytest.raises(Bd.SkvqError):
        Bd.skvq_read_write_yardstick(src, dst[:1, :1000], 7)
    with pytest.raises(Bd.SkvqError):
        Bd.skvq_read_write_yardstick(src[:3], dst[:1], 7)


# ---- clip calibration (Eq. 3; Algorithm 1 Prologue, get_group_clipping) ----

@pytest.mark.parametrize("G,v_bits,k_bits,Hq,Hk,B", [(64, 2.0, 2.0, 4, 2, 1), (128, 1.5, 2.0, 8, 2, 2), (32, 4.0, 4.0, 3, 3, 1)])
def test_clip_calibration_matches_oracle_search(P, G, v_bits, k_bits, Hq, Hk, B):
    """The same calibration tokens, queries, full-precision outputs and grid on both sides.  The
    chosen scales must be the oracle's; where a near-tie makes them differ, the oracle's own
    evaluation of the library's choice must be within 0.1 % of the oracle's result.  The scales
    that the library then uses must encode bit-exactly like the oracle with the same scales."""
    from oracle import skvq_oracle as O
    from paper_2405_06219_amd import binding as Bd
    rng = np.random.default_rng(4000 + G)
    T, W, n_q = 300, 16, 4
    dev = "cuda:0"
    pk = np.stack([rng.permutation(D) for _ in range(Hk)]).astype(np.int32)
    pv = np.stack([rng.permutation(D) for _ in range(Hk)]).astype(np.int32)
    k = (rng.standard_t(2.5, (B, Hk, T, D)) * 0.5).astype(np.float16)
    v = (rng.standard_t(2.5, (B, Hk, T, D)) * 0.5).astype(np.float16)
    q = rng.standard_normal((n_q, B, Hq, D)).astype(np.float16)
    kt = torch.from_numpy(k.astype(np.float64)).repeat_interleave(Hq // Hk, dim=1)
    vt = torch.from_numpy(v.astype(np.float64)).repeat_interleave(Hq // Hk, dim=1)
    o_ref = np.stack([torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q[i].astype(np.float64))[:, :, None, :], kt, vt)[:, :, 0].numpy() for i in range(n_q)]).astype(np.float32)
    ones = np.ones((Hk, D // G), np.float32)
    alphas = np.array([1.0, 0.95, 0.9, 0.8, 0.7], np.float32)

    ref = O.OracleCache(B, Hq, Hk, G, v_bits, W, T, pk, pv, ones, ones, k_bits=k_bits, fill=0xAB)
    rk, rv, rloss = ref.calibrate_clip(k, v, q, o_ref, alphas)
    gpu = Bd.SkvqCache(B, Hq, Hk, G, v_bits, W, T, pk, pv, ones, ones, k_bits=k_bits, fill=0xAB, device=dev)
    kd, vd = torch.from_numpy(k).to(dev), torch.from_numpy(v).to(dev)
    gk, gv, gloss = gpu.skvq_calibrate_clip(kd, vd, torch.from_numpy(q).to(dev), torch.from_numpy(o_ref).to(dev), alphas)
    P.log(f"clip calibration G{G}: oracle K {rk.tolist()} V {rv.tolist()} loss {rloss.tolist()}")
    P.log(f"clip calibration G{G}: gpu    K {gk.tolist()} V {gv.tolist()} loss {gloss.tolist()}")

    def oracle_loss(ck, cv):
        c = O.OracleCache(B, Hq, Hk, G, v_bits, W, T, pk, pv, ck, cv, k_bits=k_bits)
        assert c.prefill(k, v) == 0
        out = np.stack([c.decode(q[i]) for i in range(n_q)]).astype(np.float64)
        return ((out - o_ref) ** 2).reshape(n_q, B, Hk, Hq // Hk, D).sum(axis=(0, 1, 3, 4))

    same_choice = np.array_equal(gk, rk) and np.array_equal(gv, rv)
    P.log(f"clip calibration G{G}: the library's scales {'are' if same_choice else 'are NOT'} the oracle's "
          f"({int(np.sum(gk != rk) + np.sum(gv != rv))} of {gk.size + gv.size} differ)")
    if not same_choice:
        assert np.all(oracle_loss(gk, gv) <= rloss * 1.001)
    assert np.allclose(gloss, oracle_loss(gk, gv), rtol=2e-3)
    assert np.any(gk < 1.0) or np.any(gv < 1.0)           # heavy-tailed data: clipping pays
    # the library now encodes with the scales it chose
    want = O.OracleCache(B, Hq, Hk, G, v_bits, W, T, pk, pv, gk, gv, k_bits=k_bits, fill=0xAB)
    assert want.prefill(k, v) == 0
    gpu.skvq_prefill_quantize(kd, vd)
    for name, g, r in zip(["k_codes", "v_codes", "k_meta", "v_meta"], gpu.host_arrays(), want.arrays()):
        assert np.array_equal(g.view(np.uint8), r.view(np.uint8)), name
    # skvq_set_clip: back to other scales, bit-exact again
    other = rng.uniform(0.6, 1.0, (Hk, D // G)).astype(np.float32)
    gpu.skvq_set_clip(other, ones)
    want = O.OracleCache(B, Hq, Hk, G, v_bits, W, T, pk, pv, other, ones, k_bits=k_bits, fill=0xAB)
    assert want.prefill(k, v) == 0
    gpu.skvq_prefill_quantize(kd, vd)
    for name, g, r in zip(["k_codes", "v_codes", "k_meta", "v_meta"], gpu.host_arrays(), want.arrays()):
        assert np.array_equal(g.view(np.uint8), r.view(np.uint8)), name
    with pytest.raises(Bd.SkvqError):
        gpu.skvq_set_clip(other * 0.0, ones)


# ---- channel reorder calibration (Section 3.1; Algorithm 1 Prologue, get_permutation_matrix) ----

@pytest.mark.parametrize("B,Hk,T,G", [(1, 2, 300, 32), (3, 4, 1000, 64), (1, 1, 1, 128), (2, 8, 4099, 32)])
def test_channel_stats_and_reorder_feed_a_cache_that_matches_the_oracle(P, B, Hk, T, G):
    """Channel statistics from the GPU equal numpy's; the reorder built on them equals the
    oracle's; a cache configured with that permutation and those group boundaries is bit-exact
    with the oracle's and attends within 2e-3."""
    from oracle import skvq_oracle as O
    from paper_2405_06219_amd import binding as Bd
    rng = np.random.default_rng(5000 + T)
    scale = np.where(rng.random((1, Hk, 1, D)) < 0.1, 12.0, 1.0) * 10 ** rng.uniform(-0.5, 0.5, (1, Hk, 1, D))
    k = (rng.standard_normal((B, Hk, T, D)) * scale).astype(np.float16)
    v = (rng.standard_normal((B, Hk, T, D)) * scale[..., ::-1]).astype(np.float16)
    dev = "cuda:0"
    kd, vd = torch.from_numpy(k).to(dev), torch.from_numpy(v).to(dev)
    sk, sv = Bd.skvq_calibrate_channel_stats(kd), Bd.skvq_calibrate_channel_stats(vd)
    assert np.array_equal(sk[..., 0], k.min(axis=(0, 2)).astype(np.float32))
    assert np.array_equal(sk[..., 1], k.max(axis=(0, 2)).astype(np.float32))
    assert np.array_equal(sv, O.channel_stats(v))
    pk, bounds = Bd.skvq_calibrate_reorder(sk, G, 16, 100)
    rpk, rbounds = O.calibrate_reorder(sk, G, 16, 100)
    assert np.array_equal(pk, rpk) and np.array_equal(bounds, rbounds)
    pv, _ = Bd.skvq_calibrate_reorder(sv, G, 16, 100)      # values: their own order, the keys' boundaries
    if T < 40:
        return
    W, Hq = 16, 2 * Hk
    clip = np.full((Hk, D // G), 0.95, np.float32)
    gb = bounds if G < 128 else None
    ref = O.OracleCache(B, Hq, Hk, G, 1.5, W, T, pk, pv, clip, clip, fill=0xAB, group_bounds=gb)
    gpu = Bd.SkvqCache(B, Hq, Hk, G, 1.5, W, T, pk, pv, clip, clip, fill=0xAB, device=dev, group_bounds=gb)
    assert ref.prefill(k, v) == 0
    gpu.skvq_prefill_quantize(kd, vd)
    for name, g, r in zip(["k_codes", "v_codes", "k_meta", "v_meta"], gpu.host_arrays(), ref.arrays()):
        assert np.array_equal(g.view(np.uint8), r.view(np.uint8)), name
    q = rng.standard_normal((B, Hq, D)).astype(np.float16)
    out = gpu.skvq_decode_attention(torch.from_numpy(q).to(dev)).cpu().numpy()
    err = np.abs(out - ref.decode(q)).max()
    P.log(f"reorder calibration B{B} Hk{Hk} T{T} G{G}: bounds {bounds.tolist()} max abs err {err:.3e}")
    assert err <= P.TOL


# ---- several query tokens at once (Algorithm 1 with l > 1 on a non-empty cache) ----
MULTI_CASES = [
    (small("multi_mha_t15", context=1500), 3, 0, "f32"),
    (small("multi_gqa4_v2", n_q_heads=8, n_kv_heads=2, v_bits=2.0, context=999, batch=2), 4, 5, "f32"),
    (small("multi_gqa8_g32_k4v4", k_bits=4.0, v_bits=4.0, n_q_heads=8, n_kv_heads=1, group_size=32, context=700, window=16), 7, 0, "e4m3"),
    (small("multi_gqa3_k3v3_g64", k_bits=3.0, v_bits=3.0, n_q_heads=6, n_kv_heads=2, group_size=64, context=450), 2, 1, "f16"),
    (small("multi_window_only", context=40), 16, 0, "f32"),
    (small("multi_whole_window", window=8, context=300), 8, 0, "f32"),
    (small("multi_most_tokens_gqa8", n_q_heads=8, n_kv_heads=1, context=600), 64, 0, "f32"),   # the most query tokens a call takes
]


@pytest.mark.parametrize("w,n_new,S,meta", MULTI_CASES, ids=lambda x: x.name if hasattr(x, "name") else None)
def test_multi_token_decode_matches_oracle(P, w, n_new, S, meta):
    """The last n_new cached tokens' queries in one call: every row within 2e-3 of the oracle,
    the last row equal to the single-token call, and the split count must not matter."""
    print("case", w, n_new, S, meta, flush=True)
    pair, k, v, q1 = P.make_pair(w, extra_tokens=n_new + 1, n_sink=S, meta=meta, max_new_tokens=n_new)
    pair.prefill(k, v)
    for s in range(n_new):
        pair.append(*synth.make_new_token(w, s))
    rng = np.random.default_rng(w.seed + n_new)
    q = rng.standard_normal((w.batch, n_new, w.n_q_heads, D)).astype(np.float16)
    ref = pair.ref.decode_multi(q)
    qd = torch.from_numpy(q).to(pair.device)
    for splits in (0, 1, 5):
        pair.gpu.skvq_set_num_splits(splits)
        o16 = torch.empty(q.shape, dtype=torch.float16, device=pair.device)
        out = pair.gpu.skvq_decode_attention_multi(qd, out_f16=o16).cpu().numpy()
        err = np.abs(out - ref).max()
        P.log(f"multi-token decode {w.name} n_new={n_new} splits={splits}: max abs err {err:.3e}")
        assert err <= P.TOL
        assert np.array_equal(o16.cpu().numpy(), out.astype(np.float16))
    pair.gpu.skvq_set_num_splits(0)
    single = pair.gpu.skvq_decode_attention(qd[:, -1].contiguous()).cpu().numpy()
    assert np.abs(single - out[:, -1]).max() <= 2e-4     # other row grouping, other summation order
    from paper_2405_06219_amd import binding as Bd
    with pytest.raises(Bd.SkvqError):        # more query tokens than the workspace was sized for
        pair.gpu.skvq_decode_attention_multi(torch.zeros((w.batch, n_new + 1, w.n_q_heads, D), dtype=torch.float16,
                                                         device=pair.device))


def test_random_configurations(P):
    """Seeded random walk over the configuration space the ABI accepts: batch, kv heads, query
    heads per kv head (1..8), group size, V format, (scale, zero) format, window, sinks, context,
    appended tokens and a forced split count; the sink rule or a seeded mask of the caller's, and
    every appended token through one of the three append paths.  Buffers bit-exact, outputs
    within 2e-3."""
    rng = np.random.default_rng(20240506)
    for case in range(80):
        hk = int(rng.integers(1, 4))
        r = int(rng.integers(1, 9))
        w = small(f"rand{case}", batch=int(rng.integers(1, 4)), n_kv_heads=hk, n_q_heads=hk * r,
                  group_size=int(rng.choice([32, 64, 128])), v_bits=float(rng.choice([1.5, 2.0, 4.0])),
                  k_bits=float(rng.choice([2.0, 4.0])),
                  window=int(rng.choice([1, 3, 16, 33, 128, 200])), context=int(rng.integers(0, 2600)),
                  seed=500 + case)
        if rng.integers(4) == 0:     # the 3-bit setting: keys and values together
            w = dataclasses.replace(w, k_bits=3.0, v_bits=3.0)
        S = int(rng.choice([0, 0, 1, 5, 9]))
        meta = str(rng.choice(["f32", "f16", "e4m3"]))
        n_app = int(rng.integers(0, 40))
        splits = int(rng.choice([0, 0, 1, 2, 3, 9, 40, 128]))
        bounds = None
        if w.group_size < 128 and rng.integers(2):     # unequal groups: random multiples of 16
            ng = D // w.group_size
            cuts = np.sort(rng.choice(np.arange(1, 8), ng - 1, replace=False)) * 16
            bounds = [0, *[int(x) for x in cuts], D]
        P.log(f"random case {case}: {w} S={S} meta={meta} appends={n_app} splits={splits} bounds={bounds}")
        pair, k, v, q = P.make_pair(w, extra_tokens=n_app + 1, n_sink=S, meta=meta, group_bounds=bounds)
        # the caller's own filter rules in every other case with rows for kept tokens; each step through
        # one of the three append paths (sink rule, caller's decision, append + attention in one call)
        rng2 = np.random.default_rng(7000 + case)
        own_rules = S > 0 and case % 2 == 1
        if w.context:
            if own_rules:
                keep = rng2.random(max(w.context - w.window, 0)) < 0.002
                keep[np.flatnonzero(keep)[S:]] = False
                pair.prefill_filtered(k, v, keep)
            else:
                pair.prefill(k, v)
        pair.gpu.skvq_set_num_splits(splits)
        for s in range(n_app):
            kn, vn = synth.make_new_token(w, s)
            how = int(rng2.integers(3))
            if how == 0:
                pair.append(kn, vn)
            elif how == 1:
                st = pair.gpu.skvq_get_state()
                free = S - (st[0] - st[1] - st[2])
                pair.append_filtered(kn, vn, bool(own_rules and free > 0 and rng2.integers(3) == 0))
            else:
                o, r = pair.append_decode_both(kn, vn, q)
                assert np.abs(o - r).max() <= P.TOL, (case, s)
        pair.assert_buffers_equal()
        if pair.ref.n_tokens == 0:
            continue
        out, ref = pair.decode_both(q)
        err = np.abs(out - ref).max()
        P.log(f"random case {case}: max abs err {err:.3e} (ref max {np.abs(ref).max():.3f})")
        assert err <= P.TOL, case

"""Pins for the fp64 CPU oracle (oracle/fd_oracle.c): CPU only.

The paper prints no worked numeric example for Flash Decode (Section 4.2 and
Algorithm 4 give structure only), so the oracle is pinned to what mathematics
fixes: closed forms, invariants, an fp64 library softmax-attention, and a
pure-Python brute force that shares nothing with the C code.
"""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2511_02168_amd.inputs import f32_to_bf16_bits, bf16_bits_to_f32
from paper_2511_02168_amd import inputs as fi

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bf(x):
    return f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def rand_bits(rng, shape, scale=1.0):
    return bf(rng.standard_normal(shape).astype(np.float32) * scale)


def f64(bits):
    return bf16_bits_to_f32(bits).astype(np.float64)


def golden_constants():
    vals = {}
    with open(os.path.join(GOLDEN, "closed_form_constants.txt")) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if line:
                key, val = line.split("=")
                vals[key.strip()] = float(val)
    return vals


# ---------------------------------------------------------------- closed forms

def test_single_key_returns_v_exactly():
    rng = np.random.default_rng(1)
    B, Hq, Hkv, D, S_max = 2, 4, 2, 128, 5
    q, k, v = rand_bits(rng, (B, Hq, D)), rand_bits(rng, (B, Hkv, S_max, D)), rand_bits(rng, (B, Hkv, S_max, D))
    out, lse = oracle.decode(q, k, v, np.ones(B, np.int32))
    G = Hq // Hkv
    for b in range(B):
        for h in range(Hq):
            assert np.array_equal(out[b, h], f64(v[b, h // G, 0]))     # weight is exactly 1
            s = float(np.dot(f64(q[b, h]), f64(k[b, h // G, 0]))) / math.sqrt(D)
            assert lse[b, h] == pytest.approx(s, rel=1e-14, abs=1e-14)


def test_identical_keys_give_mean_of_v():
    rng = np.random.default_rng(2)
    D, S = 128, 37
    q = rand_bits(rng, (1, 1, D))
    k = np.tile(rand_bits(rng, (1, 1, 1, D)), (1, 1, S, 1))
    v = rand_bits(rng, (1, 1, S, D))
    out, lse = oracle.decode(q, k, v, np.array([S], np.int32))
    s = float(np.dot(f64(q[0, 0]), f64(k[0, 0, 0]))) / math.sqrt(D)
    np.testing.assert_allclose(out[0, 0], f64(v[0, 0]).mean(axis=0), rtol=1e-13, atol=1e-14)
    assert lse[0, 0] == pytest.approx(s + math.log(S), rel=1e-14)


def test_zero_keys_uniform_weights():
    rng = np.random.default_rng(3)
    D, S = 128, 64
    q = rand_bits(rng, (1, 2, D))
    k = np.zeros((1, 1, S, D), np.uint16)
    v = rand_bits(rng, (1, 1, S, D))
    out, lse = oracle.decode(q, k, v, np.array([S], np.int32))
    for h in range(2):
        np.testing.assert_allclose(out[0, h], f64(v[0, 0]).mean(axis=0), rtol=1e-13, atol=1e-14)
        assert lse[0, h] == pytest.approx(math.log(64.0), rel=1e-15)


def test_two_keys_logistic_weights_against_printed_constants():
    """Two keys: weights are sigma(s1-s2), 1-sigma; lse = s2 + ln(1+e^(s1-s2)).

    Scores are built to be exact (s1 = 1 or sqrt(2), s2 = 0) and the expected
    numbers are the tabulated constants in tests/golden/closed_form_constants.txt.
    """
    c = golden_constants()
    # D = 4: scale = 1/2, q = 2 e0, k1 = e0 -> s1 = 1, k2 = 0 -> s2 = 0
    q = bf([[[2, 0, 0, 0]]])
    k = bf([[[[1, 0, 0, 0], [0, 0, 0, 0]]]])
    v = bf([[[[1, -2, 4, 0.5], [-1, 2, 0, 8]]]])
    out, lse = oracle.decode(q, k, v, np.array([2], np.int32))
    w1 = c["sigmoid_1"]
    expect = w1 * np.array([1, -2, 4, 0.5]) + (1 - w1) * np.array([-1, 2, 0, 8])
    np.testing.assert_allclose(out[0, 0], expect, rtol=1e-14)
    assert lse[0, 0] == pytest.approx(c["softplus_1"], rel=1e-14)
    # D = 128, default scale 1/sqrt(128): q = ones, k1 = 16 ones -> s1 = 16/sqrt(128) = sqrt(2)
    q = bf(np.ones((1, 1, 128)))
    k1 = np.zeros(128)
    k1[5:21] = 1
    k = bf(np.stack([k1, np.zeros(128)])[None, None])
    v = bf(np.stack([np.full(128, 3.0), np.full(128, -1.0)])[None, None])
    out, lse = oracle.decode(q, k, v, np.array([2], np.int32))
    w1 = c["sigmoid_sqrt2"]
    np.testing.assert_allclose(out[0, 0], np.full(128, 3 * w1 - (1 - w1)), rtol=1e-14)
    assert lse[0, 0] == pytest.approx(c["softplus_sqrt2"], rel=1e-14)


def test_explicit_scale_argument_is_used():
    c = golden_constants()
    q = bf([[[1, 0, 0, 0]]])
    k = bf([[[[1, 0, 0, 0], [0, 0, 0, 0]]]])
    v = bf([[[[1, 0, 0, 0], [0, 1, 0, 0]]]])
    out, lse = oracle.decode(q, k, v, np.array([2], np.int32), scale=1.0)
    assert out[0, 0, 0] == pytest.approx(c["sigmoid_1"], rel=1e-14)
    assert lse[0, 0] == pytest.approx(c["softplus_1"], rel=1e-14)
    out, lse = oracle.decode(q, k, v, np.array([2], np.int32), scale=2.0)
    assert out[0, 0, 0] == pytest.approx(c["sigmoid_2"], rel=1e-14)


def test_dominant_key_selects_its_value_row():
    rng = np.random.default_rng(4)
    D, S = 128, 50
    q = bf(np.full((1, 1, D), 2.0))
    kk = rng.integers(-1, 2, size=(S, D)).astype(np.float32) * 0.25     # scores within +-5.7
    kk[17] = 4.0                                                       # score 2*4*128/sqrt(128) = 90.5
    k = bf(kk[None, None])
    v = rand_bits(rng, (1, 1, S, D))
    out, lse = oracle.decode(q, k, v, np.array([S], np.int32))
    np.testing.assert_allclose(out[0, 0], f64(v[0, 0, 17]), rtol=0, atol=1e-30)
    assert lse[0, 0] == pytest.approx(2 * 4 * 128 / math.sqrt(128), rel=1e-14)


def test_gqa_head_mapping_consecutive_heads_share_a_kv_head():
    rng = np.random.default_rng(5)
    B, Hq, Hkv, D = 1, 12, 3, 128
    q = rand_bits(rng, (B, Hq, D))
    k = rand_bits(rng, (B, Hkv, 1, D))
    v = rand_bits(rng, (B, Hkv, 1, D))
    out, _ = oracle.decode(q, k, v, np.ones(B, np.int32))
    for h in range(Hq):
        assert np.array_equal(out[0, h], f64(v[0, h // 4, 0]))


def test_seq_lens_bound_the_keys_and_empty_sequence():
    rng = np.random.default_rng(6)
    B, Hq, Hkv, D, S_max = 3, 2, 1, 128, 40
    q, k, v = rand_bits(rng, (B, Hq, D)), rand_bits(rng, (B, Hkv, S_max, D)), rand_bits(rng, (B, Hkv, S_max, D))
    sl = np.array([40, 13, 0], np.int32)
    kn, vn = k.copy(), v.copy()
    for b in range(B):
        kn[b, :, sl[b]:] = 0x7FC0          # NaN beyond the end must never be read
        vn[b, :, sl[b]:] = 0x7FC0
    out, lse = oracle.decode(q, kn, vn, sl)
    assert np.isfinite(out).all() and np.isfinite(lse[:2]).all()
    ref, ref_lse = oracle.decode(q[1:2], k[1:2, :, :13].copy(), v[1:2, :, :13].copy(), np.array([13], np.int32))
    assert np.array_equal(out[1], ref[0]) and np.array_equal(lse[1], ref_lse[0])
    assert np.all(out[2] == 0.0) and np.all(np.isneginf(lse[2]))


# ------------------------------------------------------------------ invariants

def _random_case(seed, B=2, Hq=4, Hkv=2, D=128, S=97, kscale=1.0):
    rng = np.random.default_rng(seed)
    return (rand_bits(rng, (B, Hq, D)), rand_bits(rng, (B, Hkv, S, D), kscale),
            rand_bits(rng, (B, Hkv, S, D)), np.full(B, S, np.int32))


@pytest.mark.parametrize("seed", [10, 11, 12])
def test_merge_of_any_partition_equals_unsplit(seed):
    q, k, v, sl = _random_case(seed, kscale=2.0)
    out, lse = oracle.decode(q, k, v, sl)
    rng = np.random.default_rng(seed + 100)
    S = int(sl[0])
    for n_parts in (1, 2, 5, 16, S, S + 7):
        cuts = np.sort(rng.integers(0, S + 1, size=n_parts - 1)) if n_parts > 1 else np.array([], int)
        bounds = np.concatenate([[0], cuts, [S]]).astype(int)            # may contain empty parts
        for b in range(q.shape[0]):
            for h in range(q.shape[1]):
                parts = [oracle.partial(q, k, v, b, h, int(bounds[i]), int(bounds[i + 1]))
                         for i in range(len(bounds) - 1)]
                po = np.stack([p[0] for p in parts])
                pl = np.array([p[1] for p in parts])
                o, L = oracle.merge(po, pl)
                np.testing.assert_allclose(o, out[b, h], rtol=1e-12, atol=1e-13)
                assert L == pytest.approx(lse[b, h], rel=1e-13)


def test_merge_is_order_independent_and_skips_empty_parts():
    rng = np.random.default_rng(20)
    po = rng.standard_normal((6, 128))
    pl = rng.standard_normal(6) * 5
    o, L = oracle.merge(po, pl)
    perm = rng.permutation(6)
    o2, L2 = oracle.merge(po[perm], pl[perm])
    np.testing.assert_allclose(o2, o, rtol=1e-13, atol=1e-15)
    assert L2 == pytest.approx(L, rel=1e-14)
    # empty parts (lse = -inf) carry any garbage, even NaN, and must not matter
    po3 = np.concatenate([po, np.full((2, 128), np.nan)])
    pl3 = np.concatenate([pl, [-np.inf, -np.inf]])
    o3, L3 = oracle.merge(po3, pl3)
    assert np.array_equal(o3, o) and L3 == L
    # library cross-check of L
    assert L == pytest.approx(float(torch.logsumexp(torch.tensor(pl), 0)), rel=1e-14)
    o4, L4 = oracle.merge(np.zeros((3, 8)), np.full(3, -np.inf))
    assert np.all(o4 == 0) and L4 == -np.inf


def test_merge_two_parts_closed_form():
    c = golden_constants()
    o, L = oracle.merge(np.array([[1.0, 0.0], [0.0, 1.0]]), np.array([1.0, 0.0]))
    assert o[0] == pytest.approx(c["sigmoid_1"], rel=1e-15)
    assert o[1] == pytest.approx(1 - c["sigmoid_1"], rel=1e-13)
    assert L == pytest.approx(c["softplus_1"], rel=1e-15)


def test_key_permutation_changes_nothing():
    q, k, v, sl = _random_case(30)
    out, lse = oracle.decode(q, k, v, sl)
    perm = np.random.default_rng(31).permutation(k.shape[2])
    out2, lse2 = oracle.decode(q, k[:, :, perm].copy(), v[:, :, perm].copy(), sl)
    np.testing.assert_allclose(out2, out, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(lse2, lse, rtol=1e-14)


def test_shift_of_all_keys_moves_lse_only():
    """K + u for every key: every score rises by scale*<q,u>; out is unchanged.

    All numbers are small dyadic rationals, so K + u is exact in bf16 and
    <q,u> is exact in fp64: nothing is re-rounded.
    """
    rng = np.random.default_rng(40)
    D, S = 128, 33
    q32 = rng.choice([-2.0, -1.0, -0.5, 0.5, 1.0, 2.0], size=(1, 2, D)).astype(np.float32)
    k32 = rng.integers(-8, 9, size=(1, 1, S, D)).astype(np.float32) / 8.0
    u32 = rng.integers(-8, 9, size=D).astype(np.float32) / 8.0
    v = rand_bits(rng, (1, 1, S, D))
    sl = np.array([S], np.int32)
    out, lse = oracle.decode(bf(q32), bf(k32), v, sl)
    assert np.array_equal(bf16_bits_to_f32(bf(k32 + u32)), k32 + u32)     # exactness of the shift
    out2, lse2 = oracle.decode(bf(q32), bf(k32 + u32), v, sl)
    for h in range(2):
        shift = float(np.dot(q32[0, h].astype(np.float64), u32.astype(np.float64))) / math.sqrt(D)
        np.testing.assert_allclose(out2[0, h], out[0, h], rtol=1e-11, atol=1e-13)
        assert lse2[0, h] == pytest.approx(lse[0, h] + shift, rel=1e-13, abs=1e-13)
    # a shift orthogonal to q changes nothing at all
    w32 = np.zeros(D, np.float32)
    w32[0], w32[1] = q32[0, 0, 1], -q32[0, 0, 0]
    out3, lse3 = oracle.decode(bf(q32[:, :1]), bf(k32 + w32), v, sl)
    np.testing.assert_allclose(out3[0, 0], out[0, 0], rtol=1e-12, atol=1e-14)
    assert lse3[0, 0] == pytest.approx(lse[0, 0], rel=1e-14)


def test_output_in_convex_hull_of_values():
    q, k, v, sl = _random_case(50, kscale=3.0)
    out, _ = oracle.decode(q, k, v, sl)
    vv = f64(v)
    G = q.shape[1] // k.shape[1]
    for b in range(q.shape[0]):
        for h in range(q.shape[1]):
            lo, hi = vv[b, h // G].min(axis=0), vv[b, h // G].max(axis=0)
            assert np.all(out[b, h] >= lo - 1e-12) and np.all(out[b, h] <= hi + 1e-12)


# ------------------------------------------------- library and brute-force pins

@pytest.mark.parametrize("B,Hq,Hkv,S,kscale", [(2, 8, 2, 257, 1.0), (1, 8, 8, 1024, 1.0),
                                                 (3, 8, 1, 100, 4.0), (1, 6, 2, 31, 0.5)])
def test_against_fp64_library_attention(B, Hq, Hkv, S, kscale):
    D = 128
    q, k, v, sl = _random_case(60 + S, B, Hq, Hkv, D, S, kscale)
    out, lse = oracle.decode(q, k, v, sl)
    G = Hq // Hkv
    tq = torch.from_numpy(f64(q)).unsqueeze(2)                                   # [B,Hq,1,D]
    tk = torch.from_numpy(f64(k)).repeat_interleave(G, dim=1)                     # [B,Hq,S,D]
    tv = torch.from_numpy(f64(v)).repeat_interleave(G, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).squeeze(2).numpy()
    np.testing.assert_allclose(out, ref, rtol=1e-11, atol=1e-13)
    scores = torch.einsum("bhd,bhsd->bhs", tq.squeeze(2), tk) / math.sqrt(D)
    np.testing.assert_allclose(lse, torch.logsumexp(scores, dim=-1).numpy(), rtol=1e-13)


def test_ragged_against_library_logsumexp():
    rng = np.random.default_rng(70)
    B, Hq, Hkv, D, S_max = 4, 4, 2, 128, 64
    q, k, v = rand_bits(rng, (B, Hq, D)), rand_bits(rng, (B, Hkv, S_max, D)), rand_bits(rng, (B, Hkv, S_max, D))
    sl = np.array([1, 64, 17, 32], np.int32)
    out, lse = oracle.decode(q, k, v, sl)
    for b in range(B):
        for h in range(Hq):
            kk = torch.from_numpy(f64(k[b, h // 2, :sl[b]]))
            s = kk @ torch.from_numpy(f64(q[b, h])) / math.sqrt(D)
            w = torch.softmax(s, 0)
            np.testing.assert_allclose(out[b, h], (w[:, None] * torch.from_numpy(f64(v[b, h // 2, :sl[b]]))).sum(0).numpy(),
                                       rtol=1e-12, atol=1e-14)
            assert lse[b, h] == pytest.approx(float(torch.logsumexp(s, 0)), rel=1e-13)


def _brute_force(qv, kv, vv, S, G, scale):
    """Straight sums with math.exp, no max subtraction (tiny scores only)."""
    Hq, D = len(qv), len(qv[0])
    outs, lses = [], []
    for h in range(Hq):
        kvh = h // G
        e = []
        for j in range(S):
            dot = 0.0
            for d in range(D):
                dot += qv[h][d] * kv[kvh][j][d]
            e.append(math.exp(scale * dot))
        z = sum(e)
        outs.append([sum(e[j] * vv[kvh][j][d] for j in range(S)) / z for d in range(D)])
        lses.append(math.log(z))
    return outs, lses


@pytest.mark.parametrize("S,D,Hq,Hkv", [(1, 1, 1, 1), (2, 2, 2, 1), (3, 4, 2, 2), (4, 3, 4, 2), (4, 4, 2, 1)])
def test_brute_force_tiny_shapes(S, D, Hq, Hkv):
    rng = np.random.default_rng(80 + S * 10 + D)
    q = rand_bits(rng, (1, Hq, D))
    k = rand_bits(rng, (1, Hkv, S, D))
    v = rand_bits(rng, (1, Hkv, S, D))
    out, lse = oracle.decode(q, k, v, np.array([S], np.int32))
    bo, bl = _brute_force(f64(q)[0].tolist(), f64(k)[0].tolist(), f64(v)[0].tolist(), S, Hq // Hkv,
                          1.0 / math.sqrt(D))
    np.testing.assert_allclose(out[0], np.array(bo), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(lse[0], np.array(bl), rtol=1e-13, atol=1e-15)


def test_partial_over_full_range_is_decode():
    q, k, v, sl = _random_case(90)
    out, lse = oracle.decode(q, k, v, sl)
    o, L = oracle.partial(q, k, v, 1, 3, 0, int(sl[1]))
    assert np.array_equal(o, out[1, 3]) and L == lse[1, 3]
    o, L = oracle.partial(q, k, v, 0, 0, 5, 5)
    assert np.all(o == 0) and L == -np.inf


def test_bad_arguments_are_rejected():
    q, k, v, sl = _random_case(91)
    with pytest.raises((ValueError, TypeError)):
        oracle.decode(q.astype(np.float32), k, v, sl)
    with pytest.raises(ValueError):
        oracle.decode(q, k, v[:, :, :5], sl)
    with pytest.raises(ValueError):
        oracle.decode(q, k, v, sl + 1000)
    with pytest.raises(ValueError):
        oracle.decode(q[:, :3], k, v, sl)            # Hq % Hkv != 0


def test_bf16_helpers_round_to_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -0.0, 3.0e38, 1e-40], np.float32)
    b = f32_to_bf16_bits(x)
    # 1 + 2^-8 is a tie -> rounds to even (1.0); 1 + 3*2^-8 is a tie -> rounds up to 1 + 2^-6
    assert b[0] == 0x3F80 and b[1] == 0x3F80 and b[2] == 0x3F82 and b[3] == 0x8000
    t = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(b, t)
    rng = np.random.default_rng(0)
    y = rng.standard_normal(10000).astype(np.float32)
    assert np.array_equal(f32_to_bf16_bits(y), torch.from_numpy(y).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))


# ---- paged KV cache: the oracle's gather against things fixed from outside it --------------

def _tiny_paged(seed, B=2, Hq=4, Hkv=2, D=8, page_size=4, lens=(7, 10)):
    rng = np.random.default_rng(seed)
    max_pages = -(-max(lens) // page_size)
    S = max_pages * page_size
    q = fi.f32_to_bf16_bits(rng.standard_normal((B, Hq, D)).astype(np.float32))
    k = fi.f32_to_bf16_bits(rng.standard_normal((B, Hkv, S, D)).astype(np.float32))
    v = fi.f32_to_bf16_bits(rng.standard_normal((B, Hkv, S, D)).astype(np.float32))
    return q, k, v, np.array(lens, dtype=np.int32), page_size, max_pages


def _to_pages(k, v, page_size, order):
    """Cuts [B,Hkv,S,D] into pages and stores page (b, p) at pool slot order[b * max_pages + p]."""
    B, Hkv, S, D = k.shape
    max_pages = S // page_size
    kp = np.zeros((B * max_pages, Hkv, page_size, D), dtype=np.uint16)
    vp = np.zeros_like(kp)
    bt = np.zeros((B, max_pages), dtype=np.int32)
    for b in range(B):
        for p in range(max_pages):
            slot = order[b * max_pages + p]
            bt[b, p] = slot
            kp[slot] = k[b, :, p * page_size:(p + 1) * page_size]
            vp[slot] = v[b, :, p * page_size:(p + 1) * page_size]
    return kp, vp, bt


def test_paged_with_identity_table_is_the_contiguous_result():
    q, k, v, sl, ps, mp = _tiny_paged(11)
    kp, vp, bt = _to_pages(k, v, ps, list(range(k.shape[0] * mp)))
    o_ref, l_ref = oracle.decode(q, k, v, sl)
    o, l = oracle.decode_paged(q, kp, vp, bt, sl)
    assert np.array_equal(o, o_ref) and np.array_equal(l, l_ref)


def test_paged_result_does_not_depend_on_where_pages_live():
    q, k, v, sl, ps, mp = _tiny_paged(12, lens=(9, 16))
    n = k.shape[0] * mp
    o_ref, l_ref = oracle.decode(q, k, v, sl)
    for seed in (1, 2, 3):
        order = np.random.default_rng(seed).permutation(n).tolist()
        kp, vp, bt = _to_pages(k, v, ps, order)
        o, l = oracle.decode_paged(q, kp, vp, bt, sl)
        assert np.array_equal(o, o_ref) and np.array_equal(l, l_ref)


def test_paged_against_pure_python_indexing():
    """Brute force with the page arithmetic written inline: score_j uses row j % ps of page bt[b][j // ps]."""
    q, k, v, sl, ps, mp = _tiny_paged(13, B=1, Hq=2, Hkv=1, D=4, page_size=2, lens=(5,))
    order = [2, 0, 1]
    kp, vp, bt = _to_pages(k, v, ps, order)
    o, l = oracle.decode_paged(q, kp, vp, bt, sl)
    qf, kf, vf = (fi.bf16_bits_to_f32(x).astype(np.float64) for x in (q, kp, vp))
    for h in range(2):
        scores = []
        for j in range(5):
            row = kf[bt[0, j // ps], 0, j % ps]
            scores.append(sum(qf[0, h, d] * row[d] for d in range(4)) / math.sqrt(4))
        m = max(scores)
        w = [math.exp(s - m) for s in scores]
        tot = sum(w)
        for d in range(4):
            ref = sum(w[j] * vf[bt[0, j // ps], 0, j % ps, d] for j in range(5)) / tot
            assert abs(o[0, h, d] - ref) < 1e-12
        assert abs(l[0, h] - (m + math.log(tot))) < 1e-12


def test_paged_ignores_table_entries_past_the_sequence_and_rejects_bad_ones():
    q, k, v, sl, ps, mp = _tiny_paged(14, lens=(3, 6))
    kp, vp, bt = _to_pages(k, v, ps, list(range(k.shape[0] * mp)))
    o_ref, l_ref = oracle.decode_paged(q, kp, vp, bt, sl)
    bt2 = bt.copy()
    bt2[0, 1:] = 10 ** 6          # sequence 0 has 3 keys = 1 page: later entries are never read
    o, l = oracle.decode_paged(q, kp, vp, bt2, sl)
    assert np.array_equal(o, o_ref) and np.array_equal(l, l_ref)
    bt2[1, 0] = kp.shape[0]       # a page that sequence 1 does use
    with pytest.raises(ValueError):
        oracle.decode_paged(q, kp, vp, bt2, sl)


def test_make_paged_round_trips_through_the_oracle():
    """The input generator's scatter and the oracle's gather are written independently
    (torch slices there, row-by-row numpy copies here): together they must be the identity."""
    import torch
    wl = fi.Workload("paged_rt", 77, B=3, Hq=4, Hkv=2, S_max=50, n_splits=0, ragged=True)
    inp = fi.make_inputs(wl, "cpu")
    o_ref, l_ref = oracle.decode(fi.bits(inp.q), fi.bits(inp.k), fi.bits(inp.v), inp.seq_lens.numpy())
    for ps in (16, 32):
        pg = fi.make_paged(inp, ps, seed=5)
        assert pg.k_pages.shape[2] == ps and torch.isnan(pg.k_pages[-1].float()).all()
        o, l = oracle.decode_paged(fi.bits(pg.q), fi.bits(pg.k_pages), fi.bits(pg.v_pages),
                                   pg.block_table.numpy(), pg.seq_lens.numpy())
        assert np.array_equal(o, o_ref) and np.array_equal(l, l_ref)


# ---- fp16 inputs: the oracle's half -> double widening against numpy's and fixed patterns ----

def test_fp16_widening_matches_numpy_for_every_bit_pattern():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.element(int(b), "fp16") for b in bits])
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(ref[~nan]))          # -0.0 stays -0.0


def test_fp16_and_bf16_fixed_patterns():
    for bits, val in ((0x3C00, 1.0), (0xC000, -2.0), (0x7BFF, 65504.0), (0x0001, 2.0 ** -24), (0x0400, 2.0 ** -14),
                      (0x3555, 0.333251953125)):
        assert oracle.element(bits, "fp16") == val
    for bits, val in ((0x3F80, 1.0), (0xC000, -2.0), (0x3EAB, 0.333984375)):
        assert oracle.element(bits, "bf16") == val


def test_fp16_decode_equals_fp64_reference_on_the_widened_values():
    """The fp16 path against torch's fp64 attention on the exactly widened inputs (library pin)."""
    rng = np.random.default_rng(21)
    B, Hq, Hkv, S, D = 2, 4, 2, 37, 16
    q = rng.standard_normal((B, Hq, D)).astype(np.float16)
    k = rng.standard_normal((B, Hkv, S, D)).astype(np.float16)
    v = rng.standard_normal((B, Hkv, S, D)).astype(np.float16)
    sl = np.array([S, 20], dtype=np.int32)
    o, l = oracle.decode(q.view(np.uint16), k.view(np.uint16), v.view(np.uint16), sl, fmt="fp16")
    for b in range(B):
        n = int(sl[b])
        qt = torch.from_numpy(q[b].astype(np.float64))                      # [Hq, D]
        kt = torch.from_numpy(k[b, :, :n].astype(np.float64)).repeat_interleave(Hq // Hkv, 0)
        vt = torch.from_numpy(v[b, :, :n].astype(np.float64)).repeat_interleave(Hq // Hkv, 0)
        s = torch.einsum("hd,hjd->hj", qt, kt) / math.sqrt(D)
        ref = torch.einsum("hj,hjd->hd", torch.softmax(s, -1), vt).numpy()
        assert np.allclose(o[b], ref, rtol=1e-12, atol=1e-13)
        assert np.allclose(l[b], torch.logsumexp(s, -1).numpy(), rtol=1e-12, atol=1e-13)


# ---- FP8 (E4M3) KV cache ------------------------------------------------------------------

def test_fp8_e4m3_widening_matches_torch_and_fixed_patterns():
    for bits, val in ((0x38, 1.0), (0x7E, 448.0), (0x01, 2.0 ** -9), (0x08, 2.0 ** -6), (0xC0, -2.0), (0x3C, 1.5), (0x00, 0.0)):
        assert oracle.element_fp8(bits) == val
    assert math.isnan(oracle.element_fp8(0x7F)) and math.isnan(oracle.element_fp8(0xFF))
    allb = torch.arange(256, dtype=torch.int32).to(torch.uint8)
    ref = allb.view(torch.float8_e4m3fn).to(torch.float64).numpy()          # torch's own decoder
    got = np.array([oracle.element_fp8(b) for b in range(256)])
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan) and np.array_equal(got[~nan], ref[~nan])


def test_fp8kv_decode_equals_bf16_decode_on_fp8_representable_values():
    """Every E4M3 value is a bf16 value: feeding the bf16 oracle the same numbers must give the same result
    (scales 1), and the scales act as plain factors on the scores and on the output."""
    rng = np.random.default_rng(31)
    B, Hq, Hkv, S, D = 2, 4, 2, 29, 16
    kb = rng.integers(0, 256, (B, Hkv, S, D)).astype(np.uint8)
    vb = rng.integers(0, 256, (B, Hkv, S, D)).astype(np.uint8)
    kb[(kb & 0x7F) == 0x7F] = 0x38                                           # no NaN patterns
    vb[(vb & 0x7F) == 0x7F] = 0x38
    kb = np.where((kb & 0x78) > 0x48, (kb & 0x87) | 0x30, kb).astype(np.uint8)   # keep |K| small: no overflowing scores
    q = f32_to_bf16_bits(rng.standard_normal((B, Hq, D)).astype(np.float32))
    sl = np.array([S, 11], dtype=np.int32)
    dec = np.vectorize(oracle.element_fp8)
    k16 = f32_to_bf16_bits(dec(kb).astype(np.float32))
    v16 = f32_to_bf16_bits(dec(vb).astype(np.float32))
    assert np.array_equal(bf16_bits_to_f32(k16).astype(np.float64), dec(kb))          # exactly representable
    o_ref, l_ref = oracle.decode(q, k16, v16, sl)
    o, l = oracle.decode_fp8kv(q, kb, vb, sl)
    assert np.allclose(o, o_ref, rtol=1e-13, atol=1e-15) and np.allclose(l, l_ref, rtol=1e-13, atol=1e-13)
    o2, l2 = oracle.decode_fp8kv(q, kb, vb, sl, k_scale=0.5, v_scale=3.0)
    o3, l3 = oracle.decode(q, k16, v16, sl, scale=0.5 / math.sqrt(D))
    assert np.allclose(o2, 3.0 * o3, rtol=1e-13, atol=1e-15) and np.allclose(l2, l3, rtol=1e-13, atol=1e-13)


def test_fp8kv_paged_is_the_contiguous_result_wherever_pages_live():
    rng = np.random.default_rng(41)
    B, Hq, Hkv, D, ps = 2, 4, 2, 8, 4
    lens = np.array([7, 10], dtype=np.int32)
    S = 12
    kb = rng.integers(0, 0x58, (B, Hkv, S, D)).astype(np.uint8)
    vb = rng.integers(0, 0x78, (B, Hkv, S, D)).astype(np.uint8)
    q = f32_to_bf16_bits(rng.standard_normal((B, Hq, D)).astype(np.float32))
    o_ref, l_ref = oracle.decode_fp8kv(q, kb, vb, lens, k_scale=0.25, v_scale=2.0)
    for seed in (0, 1):
        order = np.random.default_rng(seed).permutation(B * (S // ps)).tolist()
        kp, vp, bt = _to_pages(kb.astype(np.uint16), vb.astype(np.uint16), ps, order)
        o, l = oracle.decode_fp8kv_paged(q, kp.astype(np.uint8), vp.astype(np.uint8), bt, lens, k_scale=0.25, v_scale=2.0)
        assert np.array_equal(o, o_ref) and np.array_equal(l, l_ref)

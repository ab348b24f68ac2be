"""Pins the float64 attention oracle to things other than itself: a pure-Python
brute force, a library attention routine, closed forms that read out the mask,
and exhaustive checks of the bf16 conversions.  No GPU."""
import os

import numpy as np
import pytest
import torch

from oracle import attention, brute
from paper_2603_14371_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_bits(rng, shape, sigma=1.0):
    return synth.f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32) * np.float32(sigma))


def _case(rng, kind, m, n_own, n_prefix, heads, d):
    return (kind, _rand_bits(rng, (m, heads, d)), _rand_bits(rng, (n_prefix, d)),
            _rand_bits(rng, (n_prefix, d)), _rand_bits(rng, (n_own, d)), _rand_bits(rng, (n_own, d)))


# ---- conversions ---------------------------------------------------------
def test_widen_bf16_matches_library_for_every_bit_pattern():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ours = attention.widen_bf16(bits)
    lib = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    nan = np.isnan(lib)
    assert np.array_equal(np.isnan(ours), nan)
    assert np.array_equal(ours[~nan], lib[~nan])
    assert all(brute.bf16_to_float(int(b)) == ours[b] for b in range(0, 65536, 257) if not nan[b])


def test_generator_rounding_is_rne_like_the_library():
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.standard_normal(200000).astype(np.float32) * 3,
                        np.float32([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38])])
    ours = synth.f32_to_bf16_bits(x)
    lib = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, lib)


# ---- brute force on tiny inputs (I0) ---------------------------------------
@pytest.mark.parametrize("seed", range(6))
def test_numpy_oracle_equals_pure_python_loops(seed):
    rng = np.random.default_rng(100 + seed)
    kind = seed % 2
    heads, d = int(rng.integers(1, 4)), int(rng.choice([4, 8, 16]))
    n_prefix = int(rng.integers(0, 9))
    m = int(rng.integers(1, 4))
    n_own = m + (int(rng.integers(0, 4)) if kind == attention.DECODE else 0)
    args = _case(rng, kind, m, n_own, n_prefix, heads, d)
    o, lse = attention.attend_item(*args, scale=0.37)
    ob, lb = brute.attend_item_loops(args[0], *[a.tolist() for a in args[1:]], scale=0.37)
    np.testing.assert_allclose(o, np.array(ob), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse, np.array(lb), rtol=1e-12, atol=1e-13)


def test_tiny_config_against_loops():
    """Config 0 geometry at reduced head_dim so the pure-Python loops stay fast."""
    rng = np.random.default_rng(7)
    for kind, m, n_own in ((attention.ACTION, 10, 10), (attention.DECODE, 1, 5)):
        args = _case(rng, kind, m, n_own, 64, 8, 16)
        o, lse = attention.attend_item(*args, scale=0.25)
        ob, lb = brute.attend_item_loops(args[0], *[a.tolist() for a in args[1:]], scale=0.25)
        np.testing.assert_allclose(o, np.array(ob), rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(lse, np.array(lb), rtol=1e-12, atol=1e-13)


# ---- library routine (I2) --------------------------------------------------
@pytest.mark.parametrize("kind,m,n_own,n_prefix", [
    (attention.DECODE, 1, 5, 64), (attention.DECODE, 3, 7, 33), (attention.DECODE, 4, 4, 0),
    (attention.ACTION, 10, 10, 64), (attention.ACTION, 5, 5, 0), (attention.DECODE, 1, 1, 70)])
def test_against_torch_sdpa_with_explicit_mask(kind, m, n_own, n_prefix):
    """A decode item is rows P+p of causal attention over [prefix; own]; an action item is
    un-masked attention of the chunk over [prefix; chunk]."""
    rng = np.random.default_rng(11)
    heads, d = 8, 64
    args = _case(rng, kind, m, n_own, n_prefix, heads, d)
    scale = 1.0 / np.sqrt(d)
    o, _ = attention.attend_item(*args, scale=scale)
    w = lambda b: torch.from_numpy(b.view(np.int16)).view(torch.bfloat16).to(torch.float64)
    q = w(args[1]).permute(1, 0, 2)[None]                       # [1, H, m, d]
    k = torch.cat([w(args[2]), w(args[4])])[None, None].expand(1, heads, -1, -1)
    v = torch.cat([w(args[3]), w(args[5])])[None, None].expand(1, heads, -1, -1)
    n_all = n_prefix + n_own
    mask = torch.ones(m, n_all, dtype=torch.bool)
    if kind == attention.DECODE:
        full = torch.tril(torch.ones(n_all, n_all, dtype=torch.bool))
        mask = full[n_all - m:]
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=mask, scale=scale)
    np.testing.assert_allclose(o, ref[0].permute(1, 0, 2).numpy(), rtol=1e-10, atol=1e-12)


# ---- closed forms (I7) ----------------------------------------------------
def _golden_visible():
    rows = {}
    for line in open(os.path.join(GOLDEN, "visible_sets_tiny.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, p, o, f, t = line.split()
        rows[name] = (int(p), int(o), int(f), int(t))
    return rows


def test_zero_keys_read_out_the_visible_set_counts():
    """K = 0 makes softmax uniform over the visible set, so one-hot class values make O the
    class fractions: the mask is read out exactly (64/69, 5/69; 64/74, 10/74)."""
    gold = _golden_visible()
    d = 8
    one_hot = lambda cls, n: synth.f32_to_bf16_bits(np.tile(np.eye(d, dtype=np.float32)[cls], (n, 1)))
    zeros = lambda n: np.zeros((n, d), np.uint16)
    rng = np.random.default_rng(3)
    # decode: 4 prior own + the new one visible; there are no future own tokens for one query
    q = _rand_bits(rng, (1, 8, d))
    o, lse = attention.attend_item(attention.DECODE, q, zeros(64), one_hot(0, 64), zeros(5),
                                   one_hot(1, 5), 0.5)
    p, own, foreign, total = gold["decode"]
    np.testing.assert_allclose(o[0, :, 0], p / total, rtol=1e-13)
    np.testing.assert_allclose(o[0, :, 1], own / total, rtol=1e-13)
    assert np.all(o[0, :, 2:] == 0) and foreign == 0
    np.testing.assert_allclose(lse, np.log(total), rtol=1e-13)
    # action: whole chunk visible to every chunk query
    q = _rand_bits(rng, (10, 8, d))
    o, lse = attention.attend_item(attention.ACTION, q, zeros(64), one_hot(0, 64), zeros(10),
                                   one_hot(1, 10), 0.5)
    p, own, foreign, total = gold["action"]
    np.testing.assert_allclose(o[:, :, 0], p / total, rtol=1e-13)
    np.testing.assert_allclose(o[:, :, 1], own / total, rtol=1e-13)
    np.testing.assert_allclose(lse, np.log(total), rtol=1e-13)


def test_multi_token_decode_is_causal_over_own_tokens():
    """With m new decode queries, query r sees own tokens 0..(n-m+r): own V = one-hot(position)
    and K = 0 reads out exactly which own tokens each query saw."""
    d, n_own, m, n_prefix = 16, 7, 3, 4
    v_own = synth.f32_to_bf16_bits(np.eye(d, dtype=np.float32)[:n_own])
    zeros = lambda n: np.zeros((n, d), np.uint16)
    q = np.zeros((m, 2, d), np.uint16)
    o, _ = attention.attend_item(attention.DECODE, q, zeros(n_prefix), zeros(n_prefix),
                                 zeros(n_own), v_own, 1.0)
    for r in range(m):
        seen = n_own - m + r + 1
        expect = np.zeros(d)
        expect[:seen] = 1.0 / (n_prefix + seen)
        np.testing.assert_allclose(o[r, 0], expect, rtol=1e-13)


def test_constant_values_come_back_exactly_and_dominant_key_selects_its_value():
    rng = np.random.default_rng(4)
    d = 32
    args = list(_case(rng, attention.DECODE, 2, 6, 9, 4, d))
    const = _rand_bits(rng, (1, d))
    args[3] = np.repeat(const, 9, axis=0)
    args[5] = np.repeat(const, 6, axis=0)
    o, _ = attention.attend_item(*args, scale=0.2)
    np.testing.assert_allclose(o, np.broadcast_to(attention.widen_bf16(const)[0], o.shape),
                               rtol=1e-14)
    # one prefix key aligned with q and huge: softmax collapses onto it
    args = list(_case(rng, attention.ACTION, 1, 1, 5, 1, d))
    qf = attention.widen_bf16(args[1])[0, 0]
    args[2][3] = synth.f32_to_bf16_bits((qf * 64).astype(np.float32))
    o, _ = attention.attend_item(*args, scale=1.0)
    np.testing.assert_allclose(o[0, 0], attention.widen_bf16(args[3])[3], rtol=1e-9, atol=1e-12)


def test_scale_is_applied_to_logits_not_to_values():
    """scale -> 0 must give the mean of visible V (not zero output)."""
    rng = np.random.default_rng(9)
    args = _case(rng, attention.ACTION, 2, 2, 3, 2, 8)
    o, lse = attention.attend_item(*args, scale=0.0)
    vis = np.concatenate([attention.widen_bf16(args[3]), attention.widen_bf16(args[5])])
    np.testing.assert_allclose(o, np.broadcast_to(vis.mean(axis=0), o.shape), rtol=1e-13)
    np.testing.assert_allclose(lse, np.log(5.0), rtol=1e-13)


# ---- split/merge identity (I9) -----------------------------------------------
def test_merge_of_disjoint_key_sets_equals_attention_over_union():
    rng = np.random.default_rng(21)
    d, heads = 16, 3
    q = attention.widen_bf16(_rand_bits(rng, (heads, d)))
    k = attention.widen_bf16(_rand_bits(rng, (37, d), 3.0))
    v = attention.widen_bf16(_rand_bits(rng, (37, d)))
    whole = attention.softmax_attend(q, k, v, 0.4)
    cuts = [0, 5, 6, 20, 37]
    parts = [attention.softmax_attend(q, k[a:b], v[a:b], 0.4) for a, b in zip(cuts, cuts[1:])]
    o, lse = attention.merge_partials(parts)
    np.testing.assert_allclose(o, whole[0], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(lse, whole[1], rtol=1e-13)

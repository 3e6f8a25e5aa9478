"""Pins of the oracle's E4M3 decoding and of decode attention over E4M3 pools.

The decoder is written from the format's definition; it is pinned to the values the OCP
8-bit floating point specification tabulates for E4M3 (largest normal S.1111.110 = 448,
smallest normal S.0001.000 = 2^-6, largest subnormal S.0000.111 = 0.875 * 2^-6, smallest
subnormal S.0000.001 = 2^-9, NaN S.1111.111, no infinities), to torch's independent
conversion of all 256 codes, and to structural facts of a binary floating-point format.
The attention over such pools is pinned to a dense fp64 softmax written with numpy on the
explicitly dequantised values, and to the bfloat16 oracle on the same values (every E4M3
value is a bfloat16 value).
"""
import math

import numpy as np
import torch

import oracle
from oracle.fp8 import E4M3_TABLE, decode_e4m3, e4m3_value
from workload import (CONFIGS, make_tree, make_values_fp8_host, random_tree, to_bf16_bits,
                      bf16_bits_to_f32)


def test_e4m3_values_tabulated_by_the_specification():
    assert e4m3_value(0x00) == 0.0 and math.copysign(1.0, e4m3_value(0x00)) == 1.0
    assert e4m3_value(0x80) == 0.0 and math.copysign(1.0, e4m3_value(0x80)) == -1.0
    assert e4m3_value(0x7E) == 448.0 and e4m3_value(0xFE) == -448.0
    assert e4m3_value(0x08) == 2.0 ** -6
    assert e4m3_value(0x07) == 0.875 * 2.0 ** -6
    assert e4m3_value(0x01) == 2.0 ** -9
    assert math.isnan(e4m3_value(0x7F)) and math.isnan(e4m3_value(0xFF))
    assert e4m3_value(0x38) == 1.0 and e4m3_value(0x3C) == 1.5 and e4m3_value(0x40) == 2.0
    assert e4m3_value(0xB8) == -1.0
    assert np.isfinite(E4M3_TABLE).sum() == 254            # no infinities, two NaNs


def test_e4m3_table_against_torch_conversion():
    t = torch.arange(256, dtype=torch.int16).to(torch.uint8).view(torch.float8_e4m3fn)
    ref = t.to(torch.float32).numpy().astype(np.float64)
    nan = np.isnan(ref)
    assert nan.sum() == 2 and np.array_equal(nan, np.isnan(E4M3_TABLE))
    assert np.array_equal(ref[~nan], E4M3_TABLE[~nan])
    assert np.array_equal(np.signbit(ref[~nan]), np.signbit(E4M3_TABLE[~nan]))
    codes = np.arange(256, dtype=np.uint8).reshape(4, 8, 8)
    d = decode_e4m3(codes)
    assert d.dtype == np.float32 and d.shape == codes.shape
    assert np.array_equal(d.ravel()[~nan], ref[~nan].astype(np.float32))


def test_e4m3_structure():
    pos = E4M3_TABLE[:0x7F]
    assert np.all(np.diff(pos) > 0)                          # codes order like magnitudes
    assert np.array_equal(E4M3_TABLE[0x80:0xFF], -pos)       # sign bit only flips the sign
    # spacing doubles with every exponent step; subnormals continue the first binade
    steps = np.diff(pos)
    assert np.all(steps[:15] == 2.0 ** -9)
    for e in range(1, 15):
        assert np.all(steps[8 * e:8 * e + 7] == 2.0 ** (e - 7 - 3))
    # every value is a bfloat16 value (8 significant bits suffice for 4)
    f = E4M3_TABLE[np.isfinite(E4M3_TABLE)].astype(np.float32)
    assert np.array_equal(bf16_bits_to_f32(to_bf16_bits(f)), f)


def _dense_reference(tree, kc, vc, ks, vs, q_bits, hkv, hq, d, sm_scale):
    """Softmax attention over each leaf's chain on explicitly dequantised pools, numpy fp64."""
    K = E4M3_TABLE[kc] * np.broadcast_to(np.asarray(ks, np.float64), (hkv,))[None, :, None]
    V = E4M3_TABLE[vc] * np.broadcast_to(np.asarray(vs, np.float64), (hkv,))[None, :, None]
    Q = bf16_bits_to_f32(q_bits).astype(np.float64)
    g = hq // hkv
    L = tree.n_leaves
    out = np.zeros((L, hq, d))
    lse = np.full((L, hq), -np.inf)
    for l in range(L):
        rows = oracle.visible_rows(tree.parent, tree.tok_offset, tree.n_tokens, tree.leaf_node[l])
        if rows.size == 0:
            continue
        for j in range(hq):
            s = sm_scale * (K[rows, j // g, :] @ Q[l, j])
            m = s.max()
            w = np.exp(s - m)
            lse[l, j] = m + np.log(w.sum())
            out[l, j] = (w / w.sum()) @ V[rows, j // g, :]
    return out, lse


def test_fp8kv_attention_against_dense_softmax_on_dequantised_pools():
    cfg = CONFIGS["c2_w16"]
    for seed, (ks, vs) in enumerate([(1.0, 1.0), (0.0123, 0.0217), (0.5, 3.0)]):
        tree = random_tree(40 + seed, 30, 9, 24)
        kc, vc, q = make_values_fp8_host(cfg, tree, ks, vs, seed=77 + seed)
        assert kc.dtype == np.uint8 and kc.shape == (tree.pool_tokens, 8, 128)
        assert len(np.unique(kc)) > 100 and not np.isin(kc, [0x7F, 0xFF]).any()
        sm = 1.0 / math.sqrt(128)
        out, lse = oracle.tree_decode_attn_fp8kv(tree.parent, tree.tok_offset, tree.n_tokens,
                                                 tree.leaf_node, kc, vc, ks, vs, q, 8, 32, 128)
        ro, rl = _dense_reference(tree, kc, vc, ks, vs, q, 8, 32, 128, sm)
        assert np.allclose(out, ro, rtol=1e-10, atol=1e-12)
        fin = np.isfinite(rl)
        assert np.array_equal(fin, np.isfinite(lse)) and np.allclose(lse[fin], rl[fin], rtol=1e-12)
        # an explicit sm_scale is honoured, and rows= picks the same results
        out2, lse2 = oracle.tree_decode_attn_fp8kv(tree.parent, tree.tok_offset, tree.n_tokens,
                                                   tree.leaf_node, kc, vc, ks, vs, q, 8, 32, 128,
                                                   sm_scale=0.11, rows=([3, 5], [7, 31]))
        ro2, rl2 = _dense_reference(tree, kc, vc, ks, vs, q, 8, 32, 128, 0.11)
        assert np.allclose(out2, ro2[[3, 5], [7, 31]], rtol=1e-10, atol=1e-12)


def test_fp8kv_attention_equals_bf16_attention_on_the_same_values():
    cfg = CONFIGS["c2_w16"]
    tree = make_tree(cfg)
    kc, vc, q = make_values_fp8_host(cfg, tree, 1.0, 1.0)
    kb = to_bf16_bits(decode_e4m3(kc))
    vb = to_bf16_bits(decode_e4m3(vc))
    rows = (np.arange(16, dtype=np.int32), (np.arange(16, dtype=np.int32) * 5) % 32)
    a = oracle.tree_decode_attn_fp8kv(tree.parent, tree.tok_offset, tree.n_tokens, tree.leaf_node,
                                      kc, vc, 1.0, 1.0, q, 8, 32, 128, rows=rows)
    b = oracle.tree_decode_attn(tree.parent, tree.tok_offset, tree.n_tokens, tree.leaf_node,
                                kb, vb, q, 8, 32, 128, rows=rows)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    # the scales act as the definition says: on the scores and on the output
    c = oracle.tree_decode_attn_fp8kv(tree.parent, tree.tok_offset, tree.n_tokens, tree.leaf_node,
                                      kc, vc, 0.25, 3.0, q, 8, 32, 128, rows=rows)
    d = oracle.tree_decode_attn(tree.parent, tree.tok_offset, tree.n_tokens, tree.leaf_node,
                                kb, vb, q, 8, 32, 128, sm_scale=0.25 / math.sqrt(128), rows=rows)
    assert np.allclose(c[0], 3.0 * d[0], rtol=1e-13) and np.allclose(c[1], d[1], rtol=1e-13)


def test_quantiser_of_the_input_generator_rounds_to_nearest_code():
    """The generator's codes are nearest-value codes of x / scale (checked by brute force
    over the table), so the synthetic pools are what a quantising cache would hold."""
    from workload import quantize_e4m3
    r = np.random.default_rng(3)
    x = np.concatenate([r.standard_normal(4000).astype(np.float32) * 40,
                        r.standard_normal(2000).astype(np.float32) * 0.01,
                        np.array([0.0, 447.9, 460.0, -1e4, 2.0 ** -10, 1e-8], np.float32)])
    sc = 0.37
    codes = quantize_e4m3(torch.from_numpy(x), sc).numpy()
    val = E4M3_TABLE[codes]
    fin = E4M3_TABLE[np.isfinite(E4M3_TABLE)]
    y = np.clip(x.astype(np.float32) / np.float32(sc), -448, 448).astype(np.float64)
    best = np.abs(y[:, None] - fin[None, :]).min(axis=1)
    assert np.all(np.isfinite(val))
    assert np.all(np.abs(val - y) <= best * (1 + 1e-12) + 0.0)


def test_fp8kv_prefill_against_dense_masked_softmax_and_the_bf16_oracle():
    """Step prefill over E4M3 pools: every query token against a dense fp64 softmax over the
    rows it sees (ancestors in full, own node up to itself) on explicitly dequantised pools;
    with unit scales, bitwise the bf16 prefill oracle on the same values."""
    from workload import make_prefill_queries_host
    cfg = CONFIGS["c2_w16"]
    hkv, hq, d = 2, 4, 128
    tree = random_tree(77, 14, 5, 9)
    ks, vs = 0.31, 1.7
    kc, vc, _ = make_values_fp8_host(cfg, tree, ks, vs, seed=5)
    kc, vc = np.ascontiguousarray(kc[:, :hkv]), np.ascontiguousarray(vc[:, :hkv])
    nrows = int(tree.n_tokens[tree.leaf_node].sum())
    q = to_bf16_bits(np.random.default_rng(9).standard_normal((nrows, hq, d)).astype(np.float32))
    out, lse = oracle.tree_prefill_attn_fp8kv(tree.parent, tree.tok_offset, tree.n_tokens,
                                              tree.leaf_node, kc, vc, ks, vs, q, hkv, hq, d)
    K = E4M3_TABLE[kc] * ks
    V = E4M3_TABLE[vc] * vs
    Q = bf16_bits_to_f32(q).astype(np.float64)
    sm = 1.0 / math.sqrt(d)
    r = 0
    for l in range(tree.n_leaves):
        node = tree.leaf_node[l]
        for i in range(tree.n_tokens[node]):
            rows = oracle.visible_rows(tree.parent, tree.tok_offset, tree.n_tokens, node, i + 1)
            for j in range(hq):
                s = sm * (K[rows, j // (hq // hkv), :] @ Q[r, j])
                w = np.exp(s - s.max())
                assert abs(lse[r, j] - (s.max() + np.log(w.sum()))) < 1e-12
                assert np.allclose(out[r, j], (w / w.sum()) @ V[rows, j // (hq // hkv), :],
                                   rtol=1e-10, atol=1e-12)
            r += 1
    assert r == nrows
    a = oracle.tree_prefill_attn_fp8kv(tree.parent, tree.tok_offset, tree.n_tokens, tree.leaf_node,
                                       kc, vc, 1.0, 1.0, q, hkv, hq, d)
    b = oracle.tree_prefill_attn(tree.parent, tree.tok_offset, tree.n_tokens, tree.leaf_node,
                                 to_bf16_bits(decode_e4m3(kc)), to_bf16_bits(decode_e4m3(vc)), q,
                                 hkv, hq, d)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_fp8kv_attention_with_one_scale_per_kv_head():
    """One scale per kv head and pool: decode attention (all rows and picked rows) against
    the dense fp64 softmax on explicitly dequantised pools."""
    cfg = CONFIGS["c2_w16"]
    r = np.random.default_rng(21)
    ks = r.uniform(0.01, 2.0, size=8)
    vs = r.uniform(0.01, 3.0, size=8)
    tree = random_tree(61, 30, 9, 24)
    kc, vc, q = make_values_fp8_host(cfg, tree, 1.0, 1.0, seed=3)
    out, lse = oracle.tree_decode_attn_fp8kv(tree.parent, tree.tok_offset, tree.n_tokens,
                                             tree.leaf_node, kc, vc, ks, vs, q, 8, 32, 128)
    ro, rl = _dense_reference(tree, kc, vc, ks, vs, q, 8, 32, 128, 1.0 / math.sqrt(128))
    assert np.allclose(out, ro, rtol=1e-10, atol=1e-12)
    fin = np.isfinite(rl)
    assert np.array_equal(fin, np.isfinite(lse)) and np.allclose(lse[fin], rl[fin], rtol=1e-12)
    sel = (np.array([0, 8, 3, 3, 5], np.int32), np.array([31, 0, 12, 13, 4], np.int32))
    o2, l2 = oracle.tree_decode_attn_fp8kv(tree.parent, tree.tok_offset, tree.n_tokens,
                                           tree.leaf_node, kc, vc, ks, vs, q, 8, 32, 128, rows=sel)
    assert np.array_equal(o2, out[sel[0], sel[1]]) and np.array_equal(l2, lse[sel[0], sel[1]])
    # a scalar is the same scale on every head
    a = oracle.tree_decode_attn_fp8kv(tree.parent, tree.tok_offset, tree.n_tokens, tree.leaf_node,
                                      kc, vc, 0.3, 0.7, q, 8, 32, 128)
    b = oracle.tree_decode_attn_fp8kv(tree.parent, tree.tok_offset, tree.n_tokens, tree.leaf_node,
                                      kc, vc, np.full(8, 0.3), np.full(8, 0.7), q, 8, 32, 128)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])

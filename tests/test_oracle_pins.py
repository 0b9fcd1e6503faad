"""Pins for the CPU oracle: brute force, a library routine, closed forms and invariants.

None of these re-uses the oracle's own formula: the brute force is nested Python loops over an
independently materialised branch, the library check is torch's fp64 scaled_dot_product_attention,
and the rest are hand-derived values or properties.
"""

import math
import os

import numpy as np
import pytest
import torch

import spex_workloads as sw
from oracle.adapters import OracleSink, queries_fp64
from oracle.tree_attention import (OracleTree, decode_bf16, decode_e4m3, lse_merge,
                                   partial_attention)
from helpers import RecordingSink

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "closed_form_cases.txt")


def run_oracle(wl):
    sink = OracleSink.for_workload(wl)
    sw.replay(wl, sink)
    q = queries_fp64(sw.gen_queries(wl))
    return sink.tree, q, sink.tree.attention(wl.leaves, wl.q_lens, q, wl.sm_scale)


def small_workloads():
    return [
        sw.random_trace(11, kv_dtype="f32", q_dtype="f32", value_scale=1.0, n_ops=25, max_tokens=9),
        sw.random_trace(12, kv_dtype="bf16", q_dtype="bf16", n_ops=25, max_tokens=9, max_q_len=3),
        sw.random_trace(13, heads=(6, 3, 8), kv_dtype="fp8_e4m3", q_dtype="bf16", n_ops=25,
                        max_tokens=20, max_q_len=2),
    ]


# ------------------------------------------------------------------------- brute force
@pytest.mark.parametrize("wl", small_workloads(), ids=lambda w: w.name + "_" + w.kv_dtype)
def test_brute_force_loops(wl):
    _, _, (out, lse) = run_oracle(wl)
    rec = RecordingSink(wl)
    sw.replay(wl, rec)
    q = sw.gen_queries(wl).to(torch.float64)
    G = wl.num_q_heads // wl.num_kv_heads
    row = 0
    for leaf, ql in zip(wl.leaves, wl.q_lens):
        K, V = rec.branch(leaf)
        K, V = K.tolist(), V.tolist()
        T = len(K)
        for i in range(ql):
            visible = T - ql + i + 1
            for h in range(wl.num_q_heads):
                g = h // G
                qv = q[row, h].tolist()
                scores = []
                for t in range(visible):
                    dot = 0.0
                    for d in range(wl.head_dim):
                        dot += qv[d] * K[t][g][d]
                    scores.append(dot * wl.sm_scale)
                z = sum(math.exp(s) for s in scores)
                for d in range(wl.head_dim):
                    acc = 0.0
                    for t in range(visible):
                        acc += math.exp(scores[t]) / z * V[t][g][d]
                    assert abs(acc - out[row, h, d]) < 1e-12
                assert abs(math.log(z) - lse[row, h]) < 1e-12
            row += 1
    assert row == out.shape[0]


# ------------------------------------------------------------------------- library routine
def reduced_configs():
    return [
        sw.tiny_tree(),
        sw.bfs_tot(n_queries=2, prompt=40, step=24),
        sw.mcts_skewed(n_queries=3, prompt=(20, 60), step=(5, 40), max_leaves=12),
        sw.spec_at_scale(n_queries=2, prompt=70, step=20, branches=6),
        sw.tot_with_drafts(n_queries=2, prompt=50, step=16),
    ]


@pytest.mark.parametrize("wl", reduced_configs(), ids=lambda w: w.name)
def test_against_torch_sdpa_fp64(wl):
    _, _, (out, lse) = run_oracle(wl)
    rec = RecordingSink(wl)
    sw.replay(wl, rec)
    q = sw.gen_queries(wl).to(torch.float64)
    G = wl.num_q_heads // wl.num_kv_heads
    row = 0
    for leaf, ql in zip(wl.leaves, wl.q_lens):
        K, V = rec.branch(leaf)                                   # [T, Hkv, D]
        T = K.shape[0]
        Kh = K.permute(1, 0, 2).repeat_interleave(G, dim=0)       # [Hq, T, D]
        Vh = V.permute(1, 0, 2).repeat_interleave(G, dim=0)
        qh = q[row:row + ql].permute(1, 0, 2)                     # [Hq, ql, D]
        mask = torch.arange(T)[None, :] <= (T - ql + torch.arange(ql))[:, None]
        ref = torch.nn.functional.scaled_dot_product_attention(
            qh[None], Kh[None], Vh[None], attn_mask=mask[None, None], scale=wl.sm_scale)[0]
        got = torch.from_numpy(out[row:row + ql]).permute(1, 0, 2)
        assert torch.max(torch.abs(ref - got)).item() < 1e-12
        s = torch.einsum("hqd,htd->hqt", qh, Kh) * wl.sm_scale
        s = s.masked_fill(~mask[None], float("-inf"))
        ref_lse = torch.logsumexp(s, dim=-1)                      # [Hq, ql]
        got_lse = torch.from_numpy(lse[row:row + ql]).T
        assert torch.max(torch.abs(ref_lse - got_lse)).item() < 1e-12
        row += ql


def test_tiny_tree_matches_config_1():
    wl = sw.tiny_tree()
    tree, q, (out, lse) = run_oracle(wl)
    assert out.shape == (4, 8, 64) and lse.shape == (4, 8)
    assert [tree.path_tokens(u) for u in wl.leaves] == [320] * 4
    assert wl.unique_kv_tokens() == 512 and wl.flat_kv_tokens() == 1280
    assert abs(wl.sm_scale - 0.125) < 1e-15


# ------------------------------------------------------------------------- closed forms
def golden_cases():
    cases = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, root, keys, vals, qlen, outs, zs = [c.strip() for c in line.split("|")]
            cases.append((name, int(root), [float(x) for x in keys.split()],
                          [float(x) for x in vals.split()], int(qlen),
                          [float(x) for x in outs.split()], [float(x) for x in zs.split()]))
    return cases


@pytest.mark.parametrize("case", golden_cases(), ids=lambda c: c[0])
def test_golden_closed_forms(case):
    _, root, keys, vals, qlen, outs, zs = case
    tree = OracleTree(1, 1, 1, "f32")
    k = np.log(np.array(keys)).reshape(-1, 1, 1)
    v = np.array(vals).reshape(-1, 1, 1)
    (r,) = tree.fork(-1, 1)
    tree.append(r, k[:root], v[:root])
    (c,) = tree.fork(r, 1)
    tree.append(c, k[root:], v[root:])
    q = np.ones((qlen, 1, 1))
    out, lse = tree.attention([c], [qlen], q, 1.0)
    assert np.allclose(out[:, 0, 0], outs, rtol=0, atol=1e-12)
    assert np.allclose(np.exp(lse[:, 0]), zs, rtol=1e-13, atol=0)


def _chain_tree(K, V, cuts, Hq=None):
    """Tree that is a single chain cut into nodes at `cuts`; returns (tree, leaf)."""
    Hkv, D = K.shape[1], K.shape[2]
    tree = OracleTree(Hq or Hkv, Hkv, D, "f32")
    node = -1
    edges = [0] + list(cuts) + [K.shape[0]]
    for a, b in zip(edges[:-1], edges[1:]):
        (node,) = tree.fork(node, 1)
        tree.append(node, K[a:b], V[a:b])
    return tree, node


def test_special_cases():
    rng = np.random.default_rng(0)
    T, Hkv, G, D = 37, 2, 3, 5
    V = rng.normal(size=(T, Hkv, D))
    q = rng.normal(size=(1, Hkv * G, D))
    # all keys equal -> uniform weights -> mean of V
    K = np.tile(rng.normal(size=(1, Hkv, D)), (T, 1, 1))
    tree, leaf = _chain_tree(K, V, [10, 11], Hq=Hkv * G)
    out, lse = tree.attention([leaf], None, q, 0.3)
    for h in range(Hkv * G):
        assert np.allclose(out[0, h], V[:, h // G].mean(0), atol=1e-13)
    # q = 0 -> uniform weights, lse = ln T
    K = rng.normal(size=(T, Hkv, D))
    tree, leaf = _chain_tree(K, V, [20], Hq=Hkv * G)
    out, lse = tree.attention([leaf], None, np.zeros_like(q), 0.3)
    assert np.allclose(out[0, 4], V[:, 1].mean(0), atol=1e-13)
    assert np.allclose(lse, math.log(T), atol=1e-13)
    # T = 1 -> V[0]
    tree, leaf = _chain_tree(K[:1], V[:1], [], Hq=Hkv * G)
    out, _ = tree.attention([leaf], None, q, 0.3)
    assert np.allclose(out[0, 0], V[0, 0], atol=1e-15) and np.allclose(out[0, 5], V[0, 1], atol=1e-15)
    # V constant -> that constant, whatever the weights
    tree, leaf = _chain_tree(K, np.full_like(V, 2.5), [3, 30], Hq=Hkv * G)
    out, _ = tree.attention([leaf], None, q, 0.3)
    assert np.allclose(out, 2.5, atol=1e-13)
    # one key far above the rest -> its value row
    K2 = K.copy()
    K2[17, 0] = q[0, 0] * 1e3
    tree, leaf = _chain_tree(K2, V, [5], Hq=Hkv * G)
    out, _ = tree.attention([leaf], None, q, 1.0)
    assert np.allclose(out[0, 0], V[17, 0], atol=1e-9)


def test_gqa_head_mapping_uses_consecutive_blocks():
    # K of kv head 1 is huge at token 0, of kv head 0 at token 1: query heads 0..G-1 must pick
    # token 1, heads G..2G-1 token 0.
    G, D = 4, 3
    K = np.zeros((2, 2, D))
    K[1, 0, :] = 100.0
    K[0, 1, :] = 100.0
    V = np.zeros((2, 2, D))
    V[0, :, :] = 1.0
    V[1, :, :] = 2.0
    tree, leaf = _chain_tree(K, V, [1], Hq=2 * G)
    out, _ = tree.attention([leaf], None, np.ones((1, 2 * G, D)), 1.0)
    assert np.allclose(out[0, :G], 2.0) and np.allclose(out[0, G:], 1.0)


# ------------------------------------------------------------------------- invariants
@pytest.mark.parametrize("wl", small_workloads() + reduced_configs()[1:3], ids=lambda w: w.name)
def test_weights_sum_to_one_and_lse(wl):
    tree, q, _ = run_oracle(wl)
    out, lse, weights = tree.attention(wl.leaves, wl.q_lens, q, wl.sm_scale, return_weights=True)
    G = wl.num_q_heads // wl.num_kv_heads
    row = 0
    for leaf, ql in zip(wl.leaves, wl.q_lens):
        K, _ = tree.materialise(leaf)
        for i in range(ql):
            w = weights[row]
            assert w.shape[1] == K.shape[0] - ql + 1 + i
            assert np.all(w >= 0)
            assert np.max(np.abs(w.sum(axis=1) - 1.0)) < 1e-14
            for h in range(0, wl.num_q_heads, max(1, wl.num_q_heads // 3)):
                s = wl.sm_scale * (K[:w.shape[1], h // G] @ q[row, h])
                assert abs(math.log(np.sum(np.exp(s))) - lse[row, h]) < 1e-12
            row += 1


def test_identical_token_paths_give_identical_outputs():
    wl = sw.Workload("twins", 8, 2, 16, 16, "bf16", "bf16", 0.5, 77)
    b = sw.trees._Builder(wl)
    (root,) = b.fork(-1, 1)
    b.append(root, 21)
    a1, a2 = b.fork(root, 2)
    b.append(a1, 13, key=1234)
    b.append(a2, 13, key=1234)                 # same logical tokens as a1
    (c1,) = b.fork(a1, 1)
    (c2,) = b.fork(a2, 1)
    b.append(c1, 7, key=99)
    b.append(c2, 7, key=99)
    b.request(c1, 2, key=5)
    b.request(c2, 2, key=5)
    _, _, (out, lse) = run_oracle(wl)
    assert np.array_equal(out[:2], out[2:]) and np.array_equal(lse[:2], lse[2:])


def test_split_of_a_step_into_nodes_does_not_matter():
    rng = np.random.default_rng(3)
    K = rng.normal(size=(50, 2, 8))
    V = rng.normal(size=(50, 2, 8))
    q = rng.normal(size=(3, 4, 8))
    t1, l1 = _chain_tree(K, V, [], Hq=4)
    t2, l2 = _chain_tree(K, V, [1, 17, 18, 40], Hq=4)
    o1, s1 = t1.attention([l1], [3], q, 0.4)
    o2, s2 = t2.attention([l2], [3], q, 0.4)
    assert np.array_equal(o1, o2) and np.array_equal(s1, s2)


def test_causal_drafts_equal_truncated_single_queries():
    rng = np.random.default_rng(4)
    T, ql = 41, 6
    K = rng.normal(size=(T, 2, 8))
    V = rng.normal(size=(T, 2, 8))
    q = rng.normal(size=(ql, 4, 8))
    tree, leaf = _chain_tree(K, V, [30], Hq=4)
    out, lse = tree.attention([leaf], [ql], q, 0.35)
    for i in range(ql):
        keep = T - ql + 1 + i
        t_i, l_i = _chain_tree(K[:keep], V[:keep], [min(30, keep - 1)] if keep > 1 else [], Hq=4)
        o, s = t_i.attention([l_i], [1], q[i:i + 1], 0.35)
        assert np.allclose(o[0], out[i], atol=1e-14) and np.allclose(s[0], lse[i], atol=1e-14)


def test_lse_merge_over_random_partitions():
    rng = np.random.default_rng(5)
    for trial in range(20):
        T, D = int(rng.integers(1, 60)), 6
        K = rng.normal(size=(T, 1, D)) * 3
        V = rng.normal(size=(T, 1, D))
        q = rng.normal(size=(1, 1, D))
        tree, leaf = _chain_tree(K, V, [])
        out, lse = tree.attention([leaf], None, q, 0.7)
        ncut = int(rng.integers(0, 5))
        cuts = sorted(rng.integers(0, T + 1, size=ncut).tolist())      # empty pieces allowed
        edges = [0] + cuts + [T]
        parts = [partial_attention(q[0, 0], K[a:b, 0], V[a:b, 0], 0.7)
                 for a, b in zip(edges[:-1], edges[1:])]
        o, l = lse_merge(parts)
        assert np.allclose(o, out[0, 0], atol=1e-13) and abs(l - lse[0, 0]) < 1e-13
        # merge is order independent, and merging one piece is the identity
        o2, l2 = lse_merge(parts[::-1])
        assert np.allclose(o2, o, atol=1e-13) and abs(l2 - l) < 1e-13
    m, l, o = partial_attention(q[0, 0], K[:, 0], V[:, 0], 0.7)
    o1, l1 = lse_merge([(m, l, o)])
    assert np.allclose(o1, o / l, atol=1e-15) and abs(l1 - (m + math.log(l))) < 1e-15


# ------------------------------------------------------------------------- bit decoders
def test_bf16_and_e4m3_decoders_match_torch():
    bits = np.arange(0, 65536, dtype=np.uint16)
    ref = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64).numpy()
    got = decode_bf16(bits)
    finite = np.isfinite(ref)
    assert np.array_equal(got[finite], ref[finite]) and np.array_equal(np.isnan(got), np.isnan(ref))
    codes = np.arange(256, dtype=np.uint8)
    ref8 = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    got8 = decode_e4m3(codes)
    ok = ~np.isnan(ref8)
    assert np.array_equal(got8[ok], ref8[ok]) and np.array_equal(np.isnan(got8), np.isnan(ref8))
    assert got8[0x7E] == 448.0 and got8[0x08] == 2.0 ** -6 and got8[0x01] == 2.0 ** -9


def test_pruned_and_interior_nodes():
    tree = OracleTree(1, 1, 2, "f32")
    (r,) = tree.fork(-1, 1)
    tree.append(r, np.ones((3, 1, 2)), np.ones((3, 1, 2)))
    a, b = tree.fork(r, 2)
    tree.append(a, np.ones((2, 1, 2)), np.ones((2, 1, 2)))
    with pytest.raises(ValueError):
        tree.append(r, np.ones((1, 1, 2)), np.ones((1, 1, 2)))       # r has children
    tree.prune(a)
    with pytest.raises(KeyError):
        tree.attention([a], None, np.ones((1, 1, 2)), 1.0)
    tree.prune(b)
    tree.append(r, np.ones((1, 1, 2)), np.ones((1, 1, 2)))           # childless again
    assert tree.path_tokens(r) == 4
    with pytest.raises(ValueError):
        tree.attention([r], [5], np.ones((5, 1, 2)), 1.0)            # q_len > T


# ------------------------------------------------------------------------- draft token trees
def _random_draft_tree(rng, n):
    """Parents of a seeded token tree (draft 0 is the root) and each draft's ancestor-or-self mask."""
    parent = [-1] + [int(rng.integers(0, j)) for j in range(1, n)]
    masks = []
    for j in range(n):
        m, u = 0, j
        while u >= 0:
            m |= 1 << u
            u = parent[u]
        masks.append(m)
    return parent, masks


def test_draft_masks_brute_force_and_library():
    """Nested loops over an explicit visibility table, and torch's fp64 attention with a boolean
    mask, on a branch whose last q_len tokens form a draft token tree."""
    rng = np.random.default_rng(21)
    T, ql, Hkv, G, D = 29, 7, 2, 3, 8
    K = rng.normal(size=(T, Hkv, D))
    V = rng.normal(size=(T, Hkv, D))
    q = rng.normal(size=(ql, Hkv * G, D))
    _, masks = _random_draft_tree(rng, ql)
    tree, leaf = _chain_tree(K, V, [9, 20], Hq=Hkv * G)
    out, lse = tree.attention([leaf], [ql], q, 0.31, draft_masks=masks)
    base = T - ql
    for i in range(ql):
        for h in range(Hkv * G):
            g = h // G
            num, den, seen = np.zeros(D), 0.0, 0
            for t in range(T):
                if t >= base and not (masks[i] >> (t - base)) & 1:
                    continue
                w = math.exp(0.31 * sum(q[i, h, d] * K[t, g, d] for d in range(D)))
                den += w
                seen += 1
                for d in range(D):
                    num[d] += w * V[t, g, d]
            assert seen == base + bin(masks[i]).count("1")
            assert np.allclose(out[i, h], num / den, atol=1e-12) and abs(lse[i, h] - math.log(den)) < 1e-12
    allowed = torch.ones((ql, T), dtype=torch.bool)
    for i in range(ql):
        for j in range(ql):
            allowed[i, base + j] = bool((masks[i] >> j) & 1)
    qt = torch.from_numpy(q).permute(1, 0, 2)[None]                                  # [1, Hq, ql, D]
    kt = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(G, 0)[None]
    vt = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(G, 0)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, attn_mask=allowed, scale=0.31)
    assert np.allclose(ref[0].permute(1, 0, 2).numpy(), out, atol=1e-12)


def test_draft_masks_equal_a_branch_holding_only_the_ancestors():
    """Query i of a draft tree must give what a plain single query gives on a branch that holds
    the prefix followed by i's ancestors and i itself, in order."""
    rng = np.random.default_rng(22)
    T, ql, Hkv, D = 33, 9, 2, 6
    K = rng.normal(size=(T, Hkv, D))
    V = rng.normal(size=(T, Hkv, D))
    q = rng.normal(size=(ql, 4, D))
    _, masks = _random_draft_tree(rng, ql)
    tree, leaf = _chain_tree(K, V, [5, 26], Hq=4)
    out, lse = tree.attention([leaf], [ql], q, 0.4, draft_masks=masks)
    base = T - ql
    for i in range(ql):
        keep = list(range(base)) + [base + j for j in range(ql) if (masks[i] >> j) & 1]
        t_i, l_i = _chain_tree(K[keep], V[keep], [3], Hq=4)
        o, s = t_i.attention([l_i], [1], q[i:i + 1], 0.4)
        assert np.allclose(o[0], out[i], atol=1e-13) and np.allclose(s[0], lse[i], atol=1e-13)


def test_chain_masks_equal_the_causal_default_and_hand_values():
    rng = np.random.default_rng(23)
    T, ql = 20, 5
    K = rng.normal(size=(T, 1, 4))
    V = rng.normal(size=(T, 1, 4))
    q = rng.normal(size=(ql, 2, 4))
    tree, leaf = _chain_tree(K, V, [7])
    tree.Hq = 2
    a = tree.attention([leaf], [ql], q, 0.5)
    b = tree.attention([leaf], [ql], q, 0.5, draft_masks=[(2 << i) - 1 for i in range(ql)])
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    # hand case: keys ln 1, ln 2, ln 3, ln 6, values 6 12 18 36, q = 1, head_dim 1; the last
    # three tokens are drafts 0 <- 1 and 0 <- 2 (two children of draft 0)
    Kh = np.log(np.array([1.0, 2.0, 3.0, 6.0])).reshape(4, 1, 1)
    Vh = np.array([6.0, 12.0, 18.0, 36.0]).reshape(4, 1, 1)
    th, lh = _chain_tree(Kh, Vh, [1])
    o, s = th.attention([lh], [3], np.ones((3, 1, 1)), 1.0, draft_masks=[0b001, 0b011, 0b101])
    # weights 1 2 3 6: query 0 sees {1,2} -> (6 + 24) / 3; query 1 sees {1,2,3} -> (6 + 24 + 54) / 6;
    # query 2 sees {1,2,6} -> (6 + 24 + 216) / 9
    assert np.allclose(o[:, 0, 0], [10.0, 14.0, 246.0 / 9.0], atol=1e-13)
    assert np.allclose(np.exp(s[:, 0]), [3.0, 6.0, 9.0], atol=1e-12)
    with pytest.raises(ValueError):
        th.attention([lh], [3], np.ones((3, 1, 1)), 1.0, draft_masks=[0b001, 0b011, 0b1101])


# ------------------------------------------------------------------ e4m3 encoder / quantising append
def test_e4m3_encoder_round_trips_ties_and_saturation():
    from oracle.tree_attention import decode_e4m3, encode_e4m3
    codes = np.array([c for c in range(256) if c & 0x7F != 0x7F], dtype=np.uint8)
    vals = decode_e4m3(codes)
    assert np.array_equal(encode_e4m3(vals), codes)                       # -0.0 -> 0x80 included
    grid = decode_e4m3(np.arange(0x7F, dtype=np.uint8))
    assert np.all(np.diff(grid) > 0) and grid[0] == 0 and grid[8] == 2.0 ** -6 and grid[-1] == 448
    mid = (grid[:-1] + grid[1:]) / 2                                      # exact in fp64 and in fp32
    assert np.array_equal(mid.astype(np.float32).astype(np.float64), mid)
    want_even = np.where(np.arange(0x7E) % 2 == 0, np.arange(0x7E), np.arange(1, 0x7F))
    assert np.array_equal(encode_e4m3(mid), want_even)
    assert np.array_equal(encode_e4m3(-mid), want_even | 0x80)
    below = np.nextafter(mid.astype(np.float32), np.float32(0))
    above = np.nextafter(mid.astype(np.float32), np.float32(1e9))
    assert np.array_equal(encode_e4m3(below), np.arange(0x7E))
    assert np.array_equal(encode_e4m3(above), np.arange(1, 0x7F))
    big = np.array([448.0, 449.0, 464.0, 480.0, 1e6, np.inf, -500.0, -np.inf])
    assert encode_e4m3(big).tolist() == [0x7E] * 6 + [0xFE] * 2
    assert encode_e4m3(np.array([np.nan]))[0] & 0x7F == 0x7F
    tiny = np.array([2.0 ** -10, 2.0 ** -10 * 1.0001, 2.0 ** -9 * 1.5, 1e-30, 0.0])
    assert encode_e4m3(tiny).tolist() == [0, 1, 2, 0, 0]                  # 2^-10 ties to the even code 0


def test_e4m3_encoder_matches_torch_cast_and_exact_rationals():
    from fractions import Fraction
    from oracle.tree_attention import decode_e4m3, encode_e4m3
    rng = np.random.default_rng(31)
    y = np.concatenate([rng.normal(size=20000) * s for s in (1e-3, 0.05, 1.0, 30.0, 150.0)]).astype(np.float32)
    y = y[np.abs(y) <= 448]
    want = torch.from_numpy(y).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(encode_e4m3(y), want)
    grid = [Fraction(float(g)) for g in decode_e4m3(np.arange(0x7F, dtype=np.uint8))]
    for v in y[:400]:
        a = abs(Fraction(float(v)))
        best = min(range(0x7F), key=lambda c: (abs(grid[c] - a), c % 2))  # nearest, then the even code
        assert encode_e4m3(np.array([v]))[0] == best | (0x80 if v < 0 else 0)


def test_quantising_append_uses_the_scale_of_the_block_a_token_falls_in():
    from oracle.tree_attention import OracleTree, decode_e4m3

    def bf16_bits(x):
        return (np.asarray(x, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)

    t = OracleTree(2, 1, 4, "fp8_e4m3", scale_block=4)
    (r,) = t.fork(-1, 1)
    # block 0, scale 2^-3: values scale * grid point are encoded exactly; block never requantised
    k0 = np.array([[[0.25, -0.5, 2.0 ** -3 * 448, 2.0 ** -3 * 2.0 ** -9]]])
    t.append_quantised(r, bf16_bits(k0), bf16_bits(k0), np.array([[2.0 ** -3]]), np.array([[2.0 ** -3]]))
    assert t.last_codes[0].ravel().tolist() == [0x40, 0xC8, 0x7E, 0x01]   # 2, -4, 448, 2^-9 in units of the scale
    # second token of the same block: 100 > 448 * 2^-3 saturates, no new scale is taken
    k1 = np.array([[[100.0, -100.0, 3.0, 0.0]]])
    t.append_quantised(r, bf16_bits(k1), bf16_bits(k1))
    assert t.last_codes[0].ravel().tolist() == [0x7E, 0xFE, 0x5C, 0x00]   # 3 / 2^-3 = 24 = 1.5 * 2^4: exponent field 11, mantissa 100
    # tokens 2..4 of the path: the third starts block 1 and takes the scale passed with it
    k2 = np.array([[[1.0, 1.0, 1.0, 1.0]]] * 3)
    t.append_quantised(r, bf16_bits(k2), bf16_bits(k2), np.array([[2.0 ** -1]]), np.array([[1.0]]))
    assert t.last_codes[0][:, 0, 0].tolist() == [0x50, 0x50, 0x40]        # 8, 8 | 2
    assert t.last_codes[1][:, 0, 0].tolist() == [0x50, 0x50, 0x38]        # V scale of block 1 is 1
    K, V = t.materialise(r)
    assert np.array_equal(K[:, 0, 0], [0.25, 56.0, 1.0, 1.0, 1.0]) and V[4, 0, 0] == 1.0
    # any scale: the stored value is within half a grid step of x (fp32 rounding of x / scale aside)
    rng = np.random.default_rng(5)
    t2 = OracleTree(2, 1, 64, "fp8_e4m3", scale_block=16)
    (r2,) = t2.fork(-1, 1)
    x = bf16_bits(rng.normal(size=(1, 1, 64)))
    xv = (x.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    s = np.float32(np.abs(xv).max() / 448 * 1.37)
    t2.append_quantised(r2, x, x, np.array([[s]]), np.array([[s]]))
    got = decode_e4m3(t2.last_codes[0]) * float(s)
    step = np.maximum(2.0 ** (np.floor(np.log2(np.maximum(np.abs(xv) / float(s), 2.0 ** -6))) - 3), 2.0 ** -9) * float(s)
    assert np.all(np.abs(got - xv) <= step / 2 * (1 + 1e-6))


def test_quantising_append_derives_block_scales_from_the_tokens_it_places():
    from oracle.tree_attention import OracleTree, decode_e4m3

    def bf16_bits(x):
        return (np.asarray(x, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)

    t = OracleTree(2, 1, 2, "fp8_e4m3", scale_block=4)
    (r,) = t.fork(-1, 1)
    # six tokens: block 0 gets four (K amax 7 -> scale 7 / 448 = 2^-6), block 1 two (K amax 3.5 -> 2^-7)
    k = np.array([[[1.0, -7.0]], [[0.5, 0.25]], [[3.5, 0.0]], [[-1.75, 7.0]], [[3.5, 1.0]], [[-0.875, 0.4375]]])
    v = k * 2
    t.append_quantised(r, bf16_bits(k), bf16_bits(v), derive_scales=True)
    assert t.last_scales[0].ravel().tolist() == [2.0 ** -6, 2.0 ** -7]
    assert t.last_scales[1].ravel().tolist() == [2.0 ** -5, 2.0 ** -6]
    assert t.last_codes[0][1].ravel().tolist() == [0x60, 0x58]            # 0.5 * 64 = 32, 0.25 * 64 = 16
    assert t.last_codes[0][0, 0, 1] == 0xFE and t.last_codes[0][3, 0, 1] == 0x7E    # -7 and 7 sit at the end of the grid
    assert np.array_equal(t.last_codes[0], t.last_codes[1])               # V = 2 K, scales doubled too
    K, _ = t.materialise(r)
    assert np.array_equal(K, k)                                            # every value is on its block's grid
    # two more tokens continue block 1 (scale 2^-7, never requantised): 10 saturates at 448 * 2^-7 = 3.5
    k2 = np.array([[[10.0, 0.4375]], [[-10.0, 1.0]]])
    t.append_quantised(r, bf16_bits(k2), bf16_bits(k2), derive_scales=True)
    assert t.last_scales == [None, None]
    assert t.last_codes[0][:, 0, 0].tolist() == [0x7E, 0xFE]
    K, _ = t.materialise(r)
    assert K[6, 0, 0] == 3.5 and K[7, 0, 0] == -3.5 and K[6, 0, 1] == 0.4375
    # an all-zero block takes the floor scale and stays zero
    z = np.zeros((4, 1, 2))
    t.append_quantised(r, bf16_bits(z), bf16_bits(z), derive_scales=True)
    assert t.last_scales[0].ravel().tolist() == [2.0 ** -40] and not t.last_codes[0].any()


def test_quantising_append_agrees_with_the_generators_quantiser():
    """Two independent implementations of one recipe (the workload generator's, in torch integer
    arithmetic, and the oracle's table search) give the same codes and scales."""
    import spex_workloads as sw
    from oracle.tree_attention import OracleTree
    rng = np.random.default_rng(9)
    t = OracleTree(4, 2, 64, "fp8_e4m3", scale_block=16)
    (r,) = t.fork(-1, 1)
    filled, prev = 0, None
    for n in (5, 30, 1, 16, 43):
        x = torch.from_numpy(rng.normal(size=(n, 2, 64)).astype(np.float32) * 0.7).to(torch.bfloat16)
        bits = x.view(torch.int16).numpy().view(np.uint16)
        pk = None if prev is None else prev[0]
        pv = None if prev is None else prev[1]
        kc, ks = sw.quantise_pages(x.float(), filled, 16, pk)
        vc, vs = sw.quantise_pages(-x.float(), filled, 16, pv)
        t.append_quantised(r, bits, (x.neg()).view(torch.int16).numpy().view(np.uint16), derive_scales=True)
        assert np.array_equal(t.last_codes[0], kc.numpy()) and np.array_equal(t.last_codes[1], vc.numpy())
        if ks.shape[0]:
            assert np.array_equal(t.last_scales[0], ks.numpy()) and np.array_equal(t.last_scales[1], vs.numpy())
            prev = (ks[-1], vs[-1])
        filled += n
        if filled % 16 == 0:
            prev = None

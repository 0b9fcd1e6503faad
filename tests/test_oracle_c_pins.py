"""Pins for the C form of the attention oracle (oracle/attention_ref.c).

The C routine is held by the same kind of evidence as the numpy oracle, none of which re-uses its
loops: hand-derived closed forms (tests/golden/closed_form_cases.txt), nested Python loops over an
independently materialised branch, torch's fp64 scaled_dot_product_attention (with a boolean mask
for draft token trees), special cases with known answers, and independence of the thread count.
Agreement with the numpy oracle on random trees is checked last.
"""

import math

import numpy as np
import pytest
import torch

import spex_workloads as sw
from oracle import attention_c
from oracle.adapters import OracleSink, queries_fp64
from oracle.tree_attention import OracleTree
from helpers import RecordingSink
from test_oracle_pins import (_chain_tree, _random_draft_tree, golden_cases, reduced_configs,
                              small_workloads)


def run_c(wl, threads=0):
    sink = OracleSink.for_workload(wl)
    sw.replay(wl, sink)
    q = queries_fp64(sw.gen_queries(wl))
    out, lse, info = attention_c.attention(sink.tree, wl.leaves, wl.q_lens, q, wl.sm_scale,
                                           draft_masks=wl.draft_masks, threads=threads)
    return sink.tree, q, out, lse, info


@pytest.mark.parametrize("case", golden_cases(), ids=lambda c: c[0])
def test_c_golden_closed_forms(case):
    _, root, keys, vals, qlen, outs, zs = case
    tree = OracleTree(1, 1, 1, "f32")
    k = np.log(np.array(keys)).reshape(-1, 1, 1)
    v = np.array(vals).reshape(-1, 1, 1)
    (r,) = tree.fork(-1, 1)
    tree.append(r, k[:root], v[:root])
    (c,) = tree.fork(r, 1)
    tree.append(c, k[root:], v[root:])
    out, lse, _ = attention_c.attention(tree, [c], [qlen], np.ones((qlen, 1, 1)), 1.0)
    assert np.allclose(out[:, 0, 0], outs, rtol=0, atol=1e-12)
    assert np.allclose(np.exp(lse[:, 0]), zs, rtol=1e-13, atol=0)


@pytest.mark.parametrize("wl", small_workloads(), ids=lambda w: w.name + "_" + w.kv_dtype)
def test_c_brute_force_loops(wl):
    _, _, out, lse, _ = run_c(wl)
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
                scores = [wl.sm_scale * sum(qv[d] * K[t][g][d] for d in range(wl.head_dim))
                          for t in range(visible)]
                z = sum(math.exp(s) for s in scores)
                for d in range(wl.head_dim):
                    acc = sum(math.exp(scores[t]) / z * V[t][g][d] for t in range(visible))
                    assert abs(acc - out[row, h, d]) < 1e-12
                assert abs(math.log(z) - lse[row, h]) < 1e-12
            row += 1
    assert row == out.shape[0]


@pytest.mark.parametrize("wl", reduced_configs(), ids=lambda w: w.name)
def test_c_against_torch_sdpa_fp64(wl):
    _, _, out, lse, _ = run_c(wl)
    rec = RecordingSink(wl)
    sw.replay(wl, rec)
    q = sw.gen_queries(wl).to(torch.float64)
    G = wl.num_q_heads // wl.num_kv_heads
    row = 0
    for leaf, ql in zip(wl.leaves, wl.q_lens):
        K, V = rec.branch(leaf)
        T = K.shape[0]
        Kh = K.permute(1, 0, 2).repeat_interleave(G, dim=0)
        Vh = V.permute(1, 0, 2).repeat_interleave(G, dim=0)
        qh = q[row:row + ql].permute(1, 0, 2)
        mask = torch.arange(T)[None, :] <= (T - ql + torch.arange(ql))[:, None]
        ref = torch.nn.functional.scaled_dot_product_attention(
            qh[None], Kh[None], Vh[None], attn_mask=mask[None, None], scale=wl.sm_scale)[0]
        got = torch.from_numpy(out[row:row + ql]).permute(1, 0, 2)
        assert torch.max(torch.abs(ref - got)).item() < 1e-12
        s = torch.einsum("hqd,htd->hqt", qh, Kh) * wl.sm_scale
        ref_lse = torch.logsumexp(s.masked_fill(~mask[None], float("-inf")), dim=-1)
        assert torch.max(torch.abs(ref_lse - torch.from_numpy(lse[row:row + ql]).T)).item() < 1e-12
        row += ql


def test_c_special_cases_and_head_mapping():
    rng = np.random.default_rng(0)
    T, Hkv, G, D = 37, 2, 3, 5
    V = rng.normal(size=(T, Hkv, D))
    q = rng.normal(size=(1, Hkv * G, D))
    K = np.tile(rng.normal(size=(1, Hkv, D)), (T, 1, 1))          # equal keys -> mean of V
    tree, leaf = _chain_tree(K, V, [10, 11], Hq=Hkv * G)
    out, lse, _ = attention_c.attention(tree, [leaf], None, q, 0.3)
    for h in range(Hkv * G):
        assert np.allclose(out[0, h], V[:, h // G].mean(0), atol=1e-13)
    K = rng.normal(size=(T, Hkv, D))
    tree, leaf = _chain_tree(K, V, [20], Hq=Hkv * G)              # q = 0 -> uniform, lse = ln T
    out, lse, _ = attention_c.attention(tree, [leaf], None, np.zeros_like(q), 0.3)
    assert np.allclose(out[0, 4], V[:, 1].mean(0), atol=1e-13) and np.allclose(lse, math.log(T), atol=1e-13)
    tree, leaf = _chain_tree(K[:1], V[:1], [], Hq=Hkv * G)        # T = 1 -> V[0]
    out, _, _ = attention_c.attention(tree, [leaf], None, q, 0.3)
    assert np.allclose(out[0, 0], V[0, 0], atol=1e-15) and np.allclose(out[0, 5], V[0, 1], atol=1e-15)
    tree, leaf = _chain_tree(K, np.full_like(V, 2.5), [3, 30], Hq=Hkv * G)
    out, _, _ = attention_c.attention(tree, [leaf], None, q, 0.3)
    assert np.allclose(out, 2.5, atol=1e-13)
    K2 = K.copy()                                                  # one dominant key -> its value row
    K2[17, 0] = q[0, 0] * 1e3
    tree, leaf = _chain_tree(K2, V, [5], Hq=Hkv * G)
    out, _, _ = attention_c.attention(tree, [leaf], None, q, 1.0)
    assert np.allclose(out[0, 0], V[17, 0], atol=1e-9)
    # kv head of query head h is h // G (consecutive blocks)
    G2, D2 = 4, 3
    K3 = np.zeros((2, 2, D2))
    K3[1, 0, :] = 100.0
    K3[0, 1, :] = 100.0
    V3 = np.zeros((2, 2, D2))
    V3[0], V3[1] = 1.0, 2.0
    tree, leaf = _chain_tree(K3, V3, [1], Hq=2 * G2)
    out, _, _ = attention_c.attention(tree, [leaf], None, np.ones((1, 2 * G2, D2)), 1.0)
    assert np.allclose(out[0, :G2], 2.0) and np.allclose(out[0, G2:], 1.0)


def test_c_draft_masks_brute_force_library_and_hand_values():
    rng = np.random.default_rng(21)
    T, ql, Hkv, G, D = 29, 7, 2, 3, 8
    K = rng.normal(size=(T, Hkv, D))
    V = rng.normal(size=(T, Hkv, D))
    q = rng.normal(size=(ql, Hkv * G, D))
    _, masks = _random_draft_tree(rng, ql)
    tree, leaf = _chain_tree(K, V, [9, 20], Hq=Hkv * G)
    out, lse, _ = attention_c.attention(tree, [leaf], [ql], q, 0.31, draft_masks=masks)
    base = T - ql
    for i in range(ql):
        for h in range(Hkv * G):
            g = h // G
            num, den = np.zeros(D), 0.0
            for t in range(T):
                if t >= base and not (masks[i] >> (t - base)) & 1:
                    continue
                w = math.exp(0.31 * sum(q[i, h, d] * K[t, g, d] for d in range(D)))
                den += w
                num += w * V[t, g]
            assert np.allclose(out[i, h], num / den, atol=1e-12) and abs(lse[i, h] - math.log(den)) < 1e-12
    allowed = torch.ones((ql, T), dtype=torch.bool)
    for i in range(ql):
        for j in range(ql):
            allowed[i, base + j] = bool((masks[i] >> j) & 1)
    qt = torch.from_numpy(q).permute(1, 0, 2)[None]
    kt = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(G, 0)[None]
    vt = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(G, 0)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, attn_mask=allowed, scale=0.31)
    assert np.allclose(ref[0].permute(1, 0, 2).numpy(), out, atol=1e-12)
    # hand case (weights 1 2 3 6, drafts 0 <- 1 and 0 <- 2): 30/3, 84/6, 246/9
    Kh = np.log(np.array([1.0, 2.0, 3.0, 6.0])).reshape(4, 1, 1)
    Vh = np.array([6.0, 12.0, 18.0, 36.0]).reshape(4, 1, 1)
    th, lh = _chain_tree(Kh, Vh, [1])
    o, s, _ = attention_c.attention(th, [lh], [3], np.ones((3, 1, 1)), 1.0, draft_masks=[0b001, 0b011, 0b101])
    assert np.allclose(o[:, 0, 0], [10.0, 14.0, 246.0 / 9.0], atol=1e-13)
    assert np.allclose(np.exp(s[:, 0]), [3.0, 6.0, 9.0], atol=1e-12)
    with pytest.raises(ValueError):
        attention_c.attention(th, [lh], [3], np.ones((3, 1, 1)), 1.0, draft_masks=[0b001, 0b011, 0b1101])
    with pytest.raises(ValueError):
        attention_c.attention(th, [lh], [5], np.ones((5, 1, 1)), 1.0)            # q_len > T
    with pytest.raises(ValueError):
        attention_c.attention(th, [lh], [4], np.ones((4, 1, 1)), 1.0, draft_masks=[0, 1, 3, 7])  # query 0 sees nothing


def test_c_result_does_not_depend_on_the_thread_count_and_agrees_with_the_numpy_oracle():
    for wl in reduced_configs()[1:] + small_workloads():
        tree, q, out1, lse1, info1 = run_c(wl, threads=1)
        _, _, out4, lse4, info4 = run_c(wl, threads=4)
        assert info1["threads"] == 1 and info4["threads"] == 4
        assert np.array_equal(out1, out4) and np.array_equal(lse1, lse4)
        ref, ref_lse = tree.attention(wl.leaves, wl.q_lens, q, wl.sm_scale, draft_masks=wl.draft_masks)
        assert np.max(np.abs(out1 - ref)) < 1e-12 and np.max(np.abs(lse1 - ref_lse)) < 1e-12

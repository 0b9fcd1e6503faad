"""The synthetic input generators: determinism, fp8 encoding, and the shapes of the five trees."""

import numpy as np
import torch

import spex_workloads as sw
from spex_workloads.rng import normal_values


def test_values_depend_on_logical_position_only():
    a = normal_values(7, 1, 42, torch.arange(10, 20), 2, 8, 0.5)
    b = normal_values(7, 1, 42, torch.arange(0, 30), 2, 8, 0.5)
    assert torch.equal(a, b[10:20])
    c = normal_values(7, 2, 42, torch.arange(10, 20), 2, 8, 0.5)
    d = normal_values(8, 1, 42, torch.arange(10, 20), 2, 8, 0.5)
    e = normal_values(7, 1, 43, torch.arange(10, 20), 2, 8, 0.5)
    assert not torch.equal(a, c) and not torch.equal(a, d) and not torch.equal(a, e)


def test_values_look_standard_normal():
    x = normal_values(1, 1, 5, torch.arange(4096), 4, 64, 1.0).double().flatten()
    assert abs(x.mean().item()) < 5e-3
    assert abs(x.std().item() - 1.0) < 5e-3
    assert abs(((x ** 4).mean() / x.var() ** 2).item() - 3.0) < 0.05      # kurtosis
    lag = (x[:-1] * x[1:]).mean().item()
    assert abs(lag) < 5e-3


def test_e4m3_encoder_matches_torch_conversion():
    g = torch.Generator().manual_seed(0)
    x = torch.cat([torch.randn(20000, generator=g) * s for s in (1e-3, 0.02, 1.0, 50.0, 300.0)])
    x = torch.cat([x, torch.tensor([0.0, -0.0, 448.0, -448.0, 1e4, -1e4, 2.0 ** -9, 2.0 ** -10,
                                    1.5 * 2.0 ** -9, 2.5 * 2.0 ** -9, 0.0078125 - 1e-6, 464.0])])
    got = sw.encode_e4m3(x)
    ref = x.clamp(-448, 448).to(torch.float8_e4m3fn).view(torch.uint8)
    assert torch.equal(got, ref)
    # every code decodes back to itself
    codes = torch.tensor([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=torch.uint8)
    assert torch.equal(sw.encode_e4m3(codes.view(torch.float8_e4m3fn).float()), codes)


def test_quantise_pages_scales_and_continuation():
    x = normal_values(3, 1, 9, torch.arange(40), 2, 8, 0.5)
    codes, scales = sw.quantise_pages(x, 0, 16, None)
    assert codes.shape == (40, 2, 8) and scales.shape == (3, 2)
    for p in range(3):
        blk = x[p * 16:(p + 1) * 16]
        assert torch.equal(scales[p], blk.abs().amax(dim=(0, 2)) / 448.0)
    deq = codes.view(torch.float8_e4m3fn).float() * scales.repeat_interleave(16, 0)[:40, :, None]
    assert (deq - x).abs().max().item() <= (x.abs().max() / 16).item()
    # continuing a partial page keeps that page's scale and adds scales only for new pages
    c2, s2 = sw.quantise_pages(x[:30], 8, 16, scales[0])
    assert s2.shape == (2, 2)
    assert torch.equal(c2[:8], sw.encode_e4m3(x[:8] * (1.0 / scales[0]).reshape(1, 2, 1)))


def test_config_shapes():
    w1 = sw.tiny_tree()
    assert (w1.num_q_heads, w1.num_kv_heads, w1.head_dim, w1.page_size) == (8, 2, 64, 16)
    assert len(w1.leaves) == 4 and w1.unique_kv_tokens() == 512

    w2 = sw.bfs_tot()
    assert len(w2.leaves) == 32 * 16 and all(q == 1 for q in w2.q_lens)
    tokens, parent, alive = w2.node_tokens()
    assert all(w2.path_tokens(u) == 512 + 5 * 128 for u in w2.leaves[:40])
    uniq = w2.unique_kv_tokens()
    assert 32 * 3456 <= uniq <= 32 * 4608
    assert w2.flat_kv_tokens() == 32 * 16 * 1152
    assert sum(1 for op in w2.ops if op.kind == "prune") > 32 * 4
    # every node that is still alive lies on a requested path (losers and dead ancestors pruned)
    on_path = set()
    for u in w2.leaves:
        while u != -1:
            on_path.add(u)
            u = parent[u]
    assert on_path == {u for u in range(len(alive)) if alive[u]}

    w3 = sw.mcts_skewed()
    per_tree = np.zeros(64, dtype=int)
    tokens, parent, alive = w3.node_tokens()
    roots = sorted(u for u in range(len(parent)) if parent[u] == -1)
    for u in w3.leaves:
        r = u
        depth = 0
        while parent[r] != -1:
            r = parent[r]
            depth += 1
        assert depth <= 10
        per_tree[roots.index(r)] += 1
    assert per_tree.min() >= 1 and per_tree.max() <= 64 and per_tree.max() >= 32
    assert np.median(per_tree) < per_tree.mean()                       # heavy tail
    assert all(256 <= tokens[r] <= 1024 for r in roots)
    assert all(32 <= tokens[u] <= 256 for u in range(len(tokens)) if parent[u] != -1)

    w4 = sw.spec_at_scale()
    assert len(w4.leaves) == 256 * 32
    assert 256 * (2048 + 32 * 256) <= w4.unique_kv_tokens() <= 256 * (2048 + 35 * 256)
    assert w4.peak_pages() == 256 * (2048 + 3 * 256 + 32 * 256) // 16 == 176128
    lens = sorted({w4.path_tokens(u) for u in w4.leaves[:64]})
    assert set(lens) <= {2048 + 256 * d for d in (1, 2, 3, 4)}

    w5 = sw.tot_with_drafts()
    assert len(w5.leaves) == 512 and sum(w5.q_lens) == 3072
    assert w5.peak_pages() == 64 * 184
    assert w5.path_tokens(w5.leaves[0]) == 1024 + 3 * 128 + 6
    assert w5.kv_dtype == "fp8_e4m3" and w5.q_dtype == "bf16"


def test_replay_is_deterministic_and_batching_invariant():
    from helpers import RecordingSink
    wl = sw.random_trace(21, n_ops=30, max_tokens=30)
    a, b = RecordingSink(wl), RecordingSink(wl)
    sw.replay(wl, a, batch_tokens=1)
    sw.replay(wl, b, batch_tokens=10 ** 6)
    for u in wl.leaves:
        ka, va = a.branch(u)
        kb, vb = b.branch(u)
        assert torch.equal(ka, kb) and torch.equal(va, vb)
    q1, q2 = sw.gen_queries(wl), sw.gen_queries(wl)
    assert torch.equal(q1, q2) and q1.dtype == torch.bfloat16


def test_the_shaped_inputs_do_move_the_softmax_reference():
    """The premise of the peaked-softmax GPU tests, checked on the inputs themselves (host
    arithmetic on the seeded values, no kernel): along a 'rising' path the largest score seen so
    far grows by more than 8 / log2(e) -- the distance at which the tree-walk kernel moves its
    reference -- at least five times; with i.i.d. values it does so once."""
    import numpy as np
    from oracle.adapters import OracleSink, queries_fp64
    from peaked_cases import make_workload, shaped
    for kind, least, most in (("rising", 5, 10 ** 6), (None, 1, 1)):
        wl = shaped("bfs_bf16", kind) if kind else make_workload("bfs_bf16")
        sink = OracleSink.for_workload(wl)
        sw.replay(wl, sink)
        q = queries_fp64(sw.gen_queries(wl))
        K, _ = sink.tree.materialise(wl.leaves[0])
        s = wl.sm_scale * (K[:, 0, :] @ q[0, 0]) * 1.4426950408889634
        moves, ref = 0, -1e30
        for b in range(0, len(s), 32):
            mx = s[b:b + 32].max()
            if mx > ref + 8.0:
                ref, moves = mx, moves + 1
        assert least <= moves <= most, (kind, moves)
    # a spike dominates: the weight of every other token is below e^-40
    wl = shaped("bfs_bf16", "spike_root")
    sink = OracleSink.for_workload(wl)
    sw.replay(wl, sink)
    q = queries_fp64(sw.gen_queries(wl))
    K, _ = sink.tree.materialise(wl.leaves[0])
    s = np.sort(wl.sm_scale * (K[:, 0, :] @ q[0, 0]))
    assert s[-1] - s[-2] > 40.0

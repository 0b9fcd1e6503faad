"""The entry point that allocates nothing (spex_tree_decode_attention_static) against
spex_tree_decode_attention: same kernels, so the outputs must be equal bit for bit.

Two calls in a row through the C ABI, the second with a smaller input (fewer branches of a smaller
tree): the per-GPU static array keeps the first call's lists and partial states, and the second
call must not read any of them.  Both kernel sets: the tree-walk kernel reads its lists from the
array, the shared-prefix / suffix / merge kernels also keep their partial softmax states there.
A request beyond the array's size is refused before anything is launched."""

import numpy as np
import pytest
import torch

import spex_workloads as sw
from gpu_common import build_gpu_tree

pytestmark = pytest.mark.gpu


def both_entry_points(tree, wl, leaves, q_lens, q):
    nq = q.shape[0]
    ref_o, ref_l = tree.decode_attention(leaves, q_lens, q, wl.sm_scale)
    torch.cuda.synchronize()
    out = torch.full((nq, wl.num_q_heads, wl.head_dim), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((nq, wl.num_q_heads), float("nan"), dtype=torch.float32, device="cuda")
    tree.decode_attention(leaves, q_lens, q, wl.sm_scale, out, lse, static_scratch=True)
    torch.cuda.synchronize()
    return (out.cpu().numpy(), lse.cpu().numpy()), (ref_o.cpu().numpy(), ref_l.cpu().numpy())


@pytest.mark.parametrize("mode", [3, 2, 0])
@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8_e4m3"])
def test_static_entry_point_equals_the_allocating_one_on_two_calls_in_a_row(kv_dtype, mode):
    big = sw.bfs_tot(n_queries=6, prompt=200, step=50, heads=(16, 4, 128), kv_dtype=kv_dtype)
    small = sw.mcts_skewed(n_queries=2, prompt=(40, 90), step=(10, 40), max_leaves=6, heads=(16, 4, 128),
                           kv_dtype=kv_dtype)
    t_big = build_gpu_tree(big, kernel_mode=mode)
    t_small = build_gpu_tree(small, kernel_mode=mode)
    q_big = sw.gen_queries(big, device="cuda")
    q_small = sw.gen_queries(small, device="cuda")
    for tree, wl, q in ((t_big, big, q_big), (t_small, small, q_small), (t_big, big, q_big)):
        got, ref = both_entry_points(tree, wl, wl.leaves, wl.q_lens, q)
        assert np.all(np.isfinite(got[0])) and np.all(np.isfinite(got[1])), wl.name
        assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1]), wl.name
    # the same handle, a subset of its branches (a smaller request right after the larger one)
    half = len(big.leaves) // 3
    got, ref = both_entry_points(t_big, big, big.leaves[:half], big.q_lens[:half], q_big[:half].contiguous())
    assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])
    t_big.close()
    t_small.close()


def test_static_entry_point_follows_appends_and_matches_the_oracle():
    """Decode iterations through the static entry point only: tokens appended between calls
    (cached host plan patched or redone), every result checked against the oracle."""
    from oracle import attention_c
    from oracle.adapters import OracleSink, queries_fp64
    from gpu_common import TOL, error_report
    wl = sw.bfs_tot(n_queries=3, prompt=100, step=30, heads=(16, 4, 128))
    tree = build_gpu_tree(wl, extra_pages=4 * len(wl.leaves), kernel_mode=0)
    sink = OracleSink.for_workload(wl)
    sw.replay(wl, sink, device="cuda")
    q = sw.gen_queries(wl, device="cuda")
    qd = queries_fp64(q)
    out = torch.empty((q.shape[0], wl.num_q_heads, wl.head_dim), dtype=torch.float32, device="cuda")
    lse = torch.empty((q.shape[0], wl.num_q_heads), dtype=torch.float32, device="cuda")
    for step in range(5):
        tree.decode_attention(wl.leaves, wl.q_lens, q, wl.sm_scale, out, lse, static_scratch=True)
        ref_o, ref_l, _ = attention_c.attention(sink.tree, wl.leaves, wl.q_lens, qd, wl.sm_scale)
        rep = error_report(out.cpu().numpy().astype(np.float64), ref_o)
        assert rep["max_abs"] <= TOL["bf16"][0] and rep["rel_l2"] <= TOL["bf16"][1], (step, rep)
        assert np.max(np.abs(lse.cpu().numpy() - ref_l)) <= TOL["bf16"][0]
        k = sw.normal_values(51, 1, 10 + step, torch.arange(len(wl.leaves)), 4, 128, 0.5, "cuda").to(torch.bfloat16)
        v = sw.normal_values(51, 2, 10 + step, torch.arange(len(wl.leaves)), 4, 128, 0.5, "cuda").to(torch.bfloat16)
        tree.append_tokens(wl.leaves, k, v)
        for i, u in enumerate(wl.leaves):
            sink.append(u, k[i:i + 1], v[i:i + 1])
    tree.close()


def test_static_entry_point_refuses_what_does_not_fit():
    """Partial softmax states beyond the 48 MiB the array sets aside: SPEX_ERR_CAPACITY, nothing
    launched (the output keeps its fill value), and the allocating entry point still serves it."""
    import paper_2605_10195_amd as spex
    wl = sw.bfs_tot(n_queries=48, prompt=64, step=32)             # 768 branches x 32 heads, six pieces per row
    tree = build_gpu_tree(wl, kernel_mode=2)
    q = sw.gen_queries(wl, device="cuda")
    out = torch.full((q.shape[0], wl.num_q_heads, wl.head_dim), 7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(spex.SpexError) as e:
        tree.decode_attention(wl.leaves, wl.q_lens, q, wl.sm_scale, out, None, want_lse=False, static_scratch=True)
    assert e.value.name == "CAPACITY"
    torch.cuda.synchronize()
    assert torch.all(out == 7.0)
    ref_o, _ = tree.decode_attention(wl.leaves, wl.q_lens, q, wl.sm_scale)
    torch.cuda.synchronize()
    assert torch.all(torch.isfinite(ref_o))
    tree.close()

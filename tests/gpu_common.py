"""Shared code of the GPU parity tests: run a workload through the C ABI and through the oracle."""

import numpy as np
import torch

import spex_workloads as sw
from oracle.adapters import OracleSink, queries_fp64

# Tolerances.  bf16 / fp8 inputs with fp32 accumulation: the target stated for this build
# (max abs error <= 2e-3, relative L2 <= 1e-3 over the output tensor).  fp32 inputs: 1e-5 both
# (fp32 dot products over head_dim <= 128 and sums over a few hundred weights).
TOL = {"bf16": (2e-3, 1e-3), "fp8_e4m3": (2e-3, 1e-3), "f32": (1e-5, 1e-5)}


def build_gpu_tree(wl, free_order=None, extra_pages=0, pool_fill=None, **kw):
    import paper_2605_10195_amd as spex
    n_pages = wl.peak_pages() + extra_pages
    tree = spex.SpexTree(wl.num_q_heads, wl.num_kv_heads, wl.head_dim, wl.page_size, wl.q_dtype,
                         wl.kv_dtype, num_pages=n_pages, device="cuda", free_order=free_order,
                         pool_fill=pool_fill, **kw)
    sw.replay(wl, tree, device="cuda")
    return tree


def run_gpu(wl, tree=None, **kw):
    own = tree is None
    if own:
        tree = build_gpu_tree(wl, **kw)
    q = sw.gen_queries(wl, device="cuda")
    out, lse = tree.decode_attention(wl.leaves, wl.q_lens, q, wl.sm_scale, draft_masks=wl.draft_masks)
    torch.cuda.synchronize()
    res = out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64)
    if own:
        tree.close()
    return res


def run_oracle(wl, leaves=None, q_lens=None, q_rows=None, draft_masks=None):
    """Oracle output for all requested nodes, or for a subset (then only the nodes on those
    paths hold values; draft_masks are then the subset's)."""
    sink = OracleSink.for_workload(wl)
    only = None
    if leaves is not None:
        _, parent, _ = wl.node_tokens()
        only = set()
        for u in leaves:
            while u != -1 and u not in only:
                only.add(u)
                u = parent[u]
    sw.replay(wl, sink, device="cpu", only_nodes=only)
    q = queries_fp64(sw.gen_queries(wl, device="cpu"))
    if leaves is None:
        return sink.tree.attention(wl.leaves, wl.q_lens, q, wl.sm_scale, draft_masks=wl.draft_masks)
    return sink.tree.attention(leaves, q_lens, q[q_rows], wl.sm_scale, draft_masks=draft_masks)


def assert_close(got, ref, kv_dtype, what=""):
    max_abs_tol, rel_tol = TOL[kv_dtype]
    got_o, got_l = got
    ref_o, ref_l = ref
    assert np.all(np.isfinite(got_o)) and np.all(np.isfinite(got_l)), what
    max_abs = np.max(np.abs(got_o - ref_o))
    rel = np.linalg.norm(got_o - ref_o) / np.linalg.norm(ref_o)
    lse_err = np.max(np.abs(got_l - ref_l))
    assert max_abs <= max_abs_tol, f"{what}: max abs {max_abs:.3e} > {max_abs_tol}"
    assert rel <= rel_tol, f"{what}: rel L2 {rel:.3e} > {rel_tol}"
    assert lse_err <= max_abs_tol, f"{what}: lse {lse_err:.3e}"
    return max_abs, rel

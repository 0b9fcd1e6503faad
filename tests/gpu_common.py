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


def run_oracle_c(wl, leaves=None, q_lens=None, q_rows=None, draft_masks=None, device="cpu", threads=0):
    """As run_oracle, through the C form of the oracle (oracle/attention_ref.c), which spreads the
    requested nodes over threads.  device: where the seeded input generator runs (its values are
    bit-identical on CPU and GPU); the oracle itself always computes on the host."""
    from oracle import attention_c
    sink = OracleSink.for_workload(wl)
    only = None
    if leaves is not None:
        _, parent, _ = wl.node_tokens()
        only = set()
        for u in leaves:
            while u != -1 and u not in only:
                only.add(u)
                u = parent[u]
    sw.replay(wl, sink, device=device, only_nodes=only)
    qt = sw.gen_queries(wl, device=device)
    if leaves is None:
        leaves, q_lens, draft_masks = wl.leaves, wl.q_lens, wl.draft_masks
    else:
        qt = qt[torch.as_tensor(np.asarray(q_rows), device=qt.device)]
    q = queries_fp64(qt)
    out, lse, _ = attention_c.attention(sink.tree, leaves, q_lens, q, wl.sm_scale, draft_masks=draft_masks,
                                        threads=threads)
    return out, lse


def assert_v_round_trip(got_v, want_v, what=""):
    """V read back with gather_kv against what was appended.  In an MFMA-tiled bf16 pool V is held
    in IEEE half precision (converted toward zero when it is appended): every bf16 of magnitude in
    [2^-17, 65504], and zero, comes back bit for bit; a smaller one comes back as the multiple of
    2^-24 below it.  Other pools (fp32, fp8 codes, row-major bf16) return V bit for bit."""
    got_v, want_v = got_v.cpu(), want_v.cpu()
    if want_v.dtype != torch.bfloat16:
        assert torch.equal(got_v.view(want_v.dtype), want_v), what
        return
    g, w = got_v.view(torch.bfloat16).float(), want_v.float()
    small = (w.abs() < 2.0 ** -17) & (w != 0)
    assert torch.equal(g[~small], w[~small]), what
    assert torch.all((g[small] - w[small]).abs() < 2.0 ** -24) and torch.all(g[small].abs() <= w[small].abs()), what


def error_report(got_o, ref_o):
    """max abs error, relative L2 over the whole tensor, and the worst relative L2 of a single
    query row (one query token and head)."""
    d = got_o - ref_o
    max_abs = float(np.max(np.abs(d))) if d.size else 0.0
    rel = float(np.linalg.norm(d) / max(np.linalg.norm(ref_o), 1e-300))
    rows_d = np.linalg.norm(d.reshape(-1, d.shape[-1]), axis=1)
    rows_r = np.linalg.norm(ref_o.reshape(-1, d.shape[-1]), axis=1)
    worst = float(np.max(rows_d / np.maximum(rows_r, 1e-300))) if d.size else 0.0
    return dict(max_abs=max_abs, rel_l2=rel, worst_row_rel_l2=worst)


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

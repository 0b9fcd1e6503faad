"""GPU parity on inputs whose softmax is far from uniform, and on the edges of the value range.

With i.i.d. values the scores of a row differ by a fraction of a unit, the running reference of
the online softmax settles in the first block and the rescaling of the accumulators never runs
again.  Here the scores are shaped (spex_workloads.ValueProfile): they rise or fall along the path,
so that the reference moves many times; one key dominates everything else, placed in a block
shared by the whole workgroup, in a node shared by some wavefronts, in the last (partial) page of a
private suffix, or in a block that a later append patched into the plan; all scores are far below
zero; sm_scale is 8 times larger or smaller.  Both kernel sets (shared-prefix + suffix + merge,
tree-walk with 4 and 8 wavefronts and 1 / 2 / 4 row tiles), bf16 and fp8 pools, against the
oracle at the unchanged tolerance.  V magnitudes of 10^3, 4 * 10^4 and 2^-20, values beyond the
half-precision range, pages with scale 0.
"""

import functools

import numpy as np
import pytest
import torch

import spex_workloads as sw
from gpu_common import TOL, build_gpu_tree, error_report, run_oracle_c
from peaked_cases import make_workload, shaped

pytestmark = pytest.mark.gpu


@functools.lru_cache(maxsize=None)
def reference(shape, kind):
    return run_oracle_c(shaped(shape, kind), device="cuda")


def check(wl, got, ref, what, value_range=1.0):
    out, lse = got
    assert np.all(np.isfinite(out)) and np.all(np.isfinite(lse)), what
    tol_abs, tol_rel = TOL[wl.kv_dtype]
    rep = error_report(out, ref[0])
    lse_err = float(np.max(np.abs(lse - ref[1])))
    print(f"{what}: {rep} lse_max_abs={lse_err:.2e}")
    assert rep["max_abs"] <= tol_abs * value_range, (what, rep)
    assert rep["rel_l2"] <= tol_rel, (what, rep)
    assert lse_err <= tol_abs, (what, lse_err)
    return rep


def run(wl, mode, row_tiles, waves, **kw):
    tree = build_gpu_tree(wl, kernel_mode=mode, walk_row_tiles=row_tiles, walk_waves=waves, **kw)
    q = sw.gen_queries(wl, device="cuda")
    out, lse = tree.decode_attention(wl.leaves, wl.q_lens, q, wl.sm_scale, draft_masks=wl.draft_masks)
    torch.cuda.synchronize()
    info = tree.last_launch_info()
    tree.close()
    assert (info["walk_row_tiles"] > 0) == (mode == 3)
    return out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64)


SHAPES = ["bfs_bf16", "spec_bf16", "mcts_bf16", "drafts_fp8"]
KINDS = ["rising", "falling", "negative", "spike_root", "spike_mid", "spike_last", "rising_spike",
         "scale_x8", "scale_div8"]
LAUNCHES = [(2, 0, 0), (3, 0, 0), (3, 2, 8), (3, 2, 2)]


@pytest.mark.parametrize("launch", LAUNCHES, ids=lambda l: "mode%d_t%d_w%d" % l)
@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("shape", SHAPES)
def test_peaked_softmax_matches_oracle(shape, kind, launch):
    wl = shaped(shape, kind)
    got = run(wl, *launch)
    check(wl, got, reference(shape, kind), f"{shape} {kind} {launch}")


@pytest.mark.parametrize("launch", [(3, 1, 4), (3, 2, 4), (3, 4, 4), (3, 1, 8), (3, 4, 8), (3, 1, 2)],
                         ids=lambda l: "mode%d_t%d_w%d" % l)
@pytest.mark.parametrize("kind", ["rising", "spike_last", "rising_spike"])
@pytest.mark.parametrize("shape", SHAPES)
def test_peaked_softmax_every_tree_walk_shape(shape, kind, launch):
    wl = shaped(shape, kind)
    if wl.num_q_heads // wl.num_kv_heads > 16 * launch[1]:
        pytest.skip("one query token's rows do not fit a wavefront of this many row tiles")
    got = run(wl, *launch)
    check(wl, got, reference(shape, kind), f"{shape} {kind} {launch}")


# ------------------------------------------------------------------ a dominant key in a patched block
@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8_e4m3"])
def test_dominant_key_in_a_block_patched_into_the_plan(kv_dtype):
    """Steps of 64 tokens fill four pages, so the next decode token starts a page that opens a new
    block in its wavefront's room (a patch of the cached tree-walk lists, applied by the append
    launch).  That token's key dominates the row; four tokens later another one does."""
    from oracle.adapters import OracleSink, queries_fp64
    from oracle import attention_c
    wl = sw.bfs_tot(n_queries=2, prompt=128, step=64, heads=(16, 4, 128), kv_dtype=kv_dtype)
    wl.profile = sw.ValueProfile(q0=4.0)
    leaves = wl.leaves
    tree = build_gpu_tree(wl, extra_pages=4 * len(leaves), kernel_mode=3)
    sink = OracleSink.for_workload(wl)
    sw.replay(wl, sink, device="cuda")
    q = sw.gen_queries(wl, device="cuda")
    qd = queries_fp64(q)
    tree.decode_attention(leaves, wl.q_lens, q, wl.sm_scale)           # makes and uploads the plan
    H, D = wl.num_kv_heads, wl.head_dim
    states = []
    for step in range(6):
        k = sw.normal_values(31, 1, 700 + step, torch.arange(len(leaves)), H, D, 0.5, "cuda")
        v = sw.normal_values(31, 2, 700 + step, torch.arange(len(leaves)), H, D, 0.5, "cuda")
        if step in (0, 4):
            k[::2, :, 0] += 150.0 if step == 0 else 300.0                # every other branch
        k, v = k.to(torch.bfloat16).contiguous(), v.to(torch.bfloat16).contiguous()
        if kv_dtype == "fp8_e4m3":
            ks = torch.full((len(leaves), H), 1.0, dtype=torch.float32, device="cuda")
            vs = torch.full((len(leaves), H), 2.0 ** -6, dtype=torch.float32, device="cuda")
            new_page = [tree.node_info(u)["n_tokens"] % 16 == 0 for u in leaves]
            tree.append_tokens(leaves, k, v, ks, vs, quantize=True)
            for i, u in enumerate(leaves):
                sink.append_quantised(u, k[i:i + 1], v[i:i + 1], ks[i:i + 1] if new_page[i] else None,
                                      vs[i:i + 1] if new_page[i] else None)
        else:
            tree.append_tokens(leaves, k, v)
            for i, u in enumerate(leaves):
                sink.append(u, k[i:i + 1], v[i:i + 1])
        out, lse = tree.decode_attention(leaves, wl.q_lens, q, wl.sm_scale)
        states.append(tree.last_launch_info()["plan_rebuilt"])
        ref_o, ref_l, _ = attention_c.attention(sink.tree, leaves, wl.q_lens, qd, wl.sm_scale)
        got = (out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64))
        check(wl, got, (ref_o, ref_l), f"patched block, step {step}")
    assert states == [2] * 6, states          # every iteration ran on a patched plan
    tree.close()


# ------------------------------------------------------------------ value range of V
@pytest.mark.parametrize("launch", LAUNCHES, ids=lambda l: "mode%d_t%d_w%d" % l)
@pytest.mark.parametrize("shape", ["bfs_bf16", "drafts_fp8"])
@pytest.mark.parametrize("log2_mult", [11, 14, -20])
def test_v_magnitudes_inside_the_half_precision_range(shape, log2_mult, launch):
    """|V| up to 2.45 * 2^11 = 5 * 10^3, 2.45 * 2^14 = 4 * 10^4 and 2.45 * 2^-20.  The absolute
    bound scales with the value range (it is stated for values of magnitude 0.5 * N(0,1)); the
    relative bound is unchanged, except below 2^-14 where half precision is subnormal and the
    header promises an absolute error below 2^-24 (bf16 pools) or 2^-23 (fp8 pools) per element instead."""
    wl = make_workload(shape)
    mult = 2.0 ** log2_mult
    wl.profile = sw.ValueProfile(v_mult=mult)
    got = run(wl, *launch)
    ref = run_oracle_c(wl, device="cuda")
    assert np.all(np.isfinite(got[0]))
    rep = error_report(got[0], ref[0])
    print(f"{shape} V x 2^{log2_mult} {launch}: {rep}")
    tol_abs, tol_rel = TOL[wl.kv_dtype]
    if log2_mult >= 0:
        assert rep["max_abs"] <= tol_abs * mult and rep["rel_l2"] <= tol_rel, rep
    else:   # bf16: stored toward zero in half precision; fp8: code * scale formed in two half-precision steps
        assert rep["max_abs"] <= (2.0 ** -24 if wl.kv_dtype == "bf16" else 2.0 ** -23), rep
    assert np.max(np.abs(got[1] - ref[1])) <= tol_abs


@pytest.mark.parametrize("launch", [(3, 0, 0), (3, 2, 8)], ids=lambda l: "mode%d_t%d_w%d" % l)
def test_v_beyond_the_half_precision_range_saturates(launch):
    """bf16 V of magnitude up to 3 * 10^5: an MFMA-tiled bf16 pool holds V in half precision, and the
    append stores a magnitude above 65504 as 65504 (never as infinity), so every kernel on that
    pool -- the generic one included -- matches the oracle on the clipped values, not on the
    unclipped ones."""
    from oracle.adapters import OracleSink, queries_fp64
    from oracle import attention_c
    wl = make_workload("bfs_bf16")
    mult = 2.0 ** 17
    wl.profile = sw.ValueProfile(v_mult=mult)
    got = run(wl, *launch)
    assert np.all(np.isfinite(got[0]))
    sink = OracleSink.for_workload(wl)
    sw.replay(wl, sink, device="cuda")
    q = queries_fp64(sw.gen_queries(wl, device="cuda"))
    exact = attention_c.attention(sink.tree, wl.leaves, wl.q_lens, q, wl.sm_scale)
    clipped = 0
    for pieces in sink.tree.V:
        for i, a in enumerate(pieces):
            clipped += int((np.abs(a) > 65504.0).sum())
            pieces[i] = np.clip(a, -65504.0, 65504.0)
    assert clipped > 1000
    ref = attention_c.attention(sink.tree, wl.leaves, wl.q_lens, q, wl.sm_scale)
    rep = error_report(got[0], ref[0])
    print(f"saturating V {launch}: {rep}")
    assert rep["max_abs"] <= 2e-3 * mult and rep["rel_l2"] <= 1e-3, rep
    got1 = run(wl, 1, 0, 0)
    rep1 = error_report(got1[0], ref[0])
    assert rep1["max_abs"] <= 2e-3 * mult and rep1["rel_l2"] <= 1e-3, rep1
    assert error_report(got1[0], exact[0])["rel_l2"] > 1e-2      # the clipping is visible


def test_gather_returns_v_as_the_pool_holds_it():
    """Round trip of chosen bf16 V values through an MFMA-tiled pool (half precision, toward zero)
    and through a row-major one (bf16 as given)."""
    import paper_2605_10195_amd as spex
    vals = torch.tensor([0.0, 1.0, -2.5, 65280.0, 65536.0, -3.0e5, 2.0 ** -14, 2.0 ** -17, -1.5 * 2.0 ** -17,
                         (1 + 2.0 ** -7) * 2.0 ** -18, 1.5 * 2.0 ** -24, 2.0 ** -25, -2.0 ** -30, 448.0], dtype=torch.float32)
    want = torch.tensor([0.0, 1.0, -2.5, 65280.0, 65504.0, -65504.0, 2.0 ** -14, 2.0 ** -17, -1.5 * 2.0 ** -17,
                         2.0 ** -18, 2.0 ** -24, 0.0, -0.0, 448.0], dtype=torch.float32)
    for D, tiled in ((128, True), (96, False)):
        tree = spex.SpexTree(4, 2, D, 16, "bf16", "bf16", num_pages=8, device="cuda")
        (r,) = tree.fork(-1, 1)
        n = 20
        v = vals.repeat((n * 2 * D + len(vals) - 1) // len(vals))[:n * 2 * D].reshape(n, 2, D).to(torch.bfloat16).cuda()
        k = v.flip(0).contiguous()
        tree.append(r, k, v.contiguous())
        gk, gv, _, _ = tree.gather_kv(r, 0, n)
        assert torch.equal(gk, k)
        exp = want if tiled else vals
        exp = exp.repeat((n * 2 * D + len(vals) - 1) // len(vals))[:n * 2 * D].reshape(n, 2, D).to(torch.bfloat16)
        if tiled:  # 65504 is not a bf16: what comes back is the bf16 below it
            exp = torch.where(exp.float().abs() > 65504.0, torch.sign(exp.float()) * 65280.0, exp.float()).to(torch.bfloat16)
        assert torch.equal(gv.cpu().view(torch.int16), exp.view(torch.int16)), (D, gv.cpu().float().flatten()[:14], exp.float().flatten()[:14])
        tree.close()


@pytest.mark.parametrize("launch", LAUNCHES, ids=lambda l: "mode%d_t%d_w%d" % l)
def test_fp8_pages_with_scale_zero_and_large_v_scale(launch):
    """A page of zeros may carry scale 0 (amax / 448 of an all-zero page): its scores are 0, masked
    slots of a partial page stay masked (no -inf * 0), and the result is finite.  A V scale of 100
    (values up to 44 800) is inside the stated range."""
    import paper_2605_10195_amd as spex
    from oracle.tree_attention import OracleTree
    from oracle.adapters import raw_array, queries_fp64
    from oracle import attention_c
    Hq, Hkv, D = 8, 2, 128
    rng = np.random.default_rng(5)
    tree = spex.SpexTree(Hq, Hkv, D, 16, "bf16", "fp8_e4m3", num_pages=64, device="cuda",
                         kernel_mode=launch[0], walk_row_tiles=launch[1], walk_waves=launch[2])
    oracle = OracleTree(Hq, Hkv, D, "fp8_e4m3", scale_block=16)
    (r,) = tree.fork(-1, 1)
    oracle.fork(-1, 1)

    def codes(n, zero=False):
        c = rng.integers(0, 0x7F, size=(n, Hkv, D), dtype=np.uint8) | (rng.integers(0, 2, size=(n, Hkv, D), dtype=np.uint8) << 7)
        return np.zeros_like(c) if zero else c

    def append(node, k, v, ks, vs):
        tree.append(node, torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda(),
                    torch.from_numpy(ks).cuda(), torch.from_numpy(vs).cuda())
        oracle.append(node, k, v, ks, vs)

    # root: 3 pages; the middle one is all zeros with K scale 0
    ks = np.array([[0.01, 0.02], [0.0, 0.0], [0.015, 0.01]], dtype=np.float32)
    vs = np.array([[0.01, 100.0], [0.02, 0.0], [100.0, 0.01]], dtype=np.float32)
    k = codes(40)
    k[16:32] = 0
    append(r, k, codes(40), ks, vs)
    kids = tree.fork(r, 3)
    oracle.fork(r, 3)
    for j, c in enumerate(kids):
        n = 5 + 16 * j                     # partial last pages; the last page of child 1 is zeros with scale 0
        kk = codes(n)
        npg = (n + 15) // 16
        ksc = np.full((npg, Hkv), 0.02, dtype=np.float32)
        if j == 1:
            kk[16:] = 0
            ksc[1] = 0.0
        append(c, kk, codes(n), ksc, np.full((npg, Hkv), 0.01, dtype=np.float32))
    q = torch.from_numpy(rng.standard_normal((3, Hq, D)).astype(np.float32)).to(torch.bfloat16).cuda()
    out, lse = tree.decode_attention(kids, None, q, 0.09)
    torch.cuda.synchronize()
    tree.close()
    ref_o, ref_l, _ = attention_c.attention(oracle, kids, None, queries_fp64(q), 0.09)
    got = out.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got)) and np.all(np.isfinite(lse.cpu().numpy()))
    rep = error_report(got, ref_o)
    print(f"zero scales {launch}: {rep}")
    assert rep["max_abs"] <= 2e-3 * 44800 / 2.45 and rep["rel_l2"] <= 1e-3, rep
    assert np.max(np.abs(lse.cpu().numpy() - ref_l)) <= 2e-3


def test_duplicate_request_then_append_across_a_page_boundary():
    """The same node requested twice, a plan made, then decode tokens that start a page: the plan
    cannot be patched for a node that two requests share, so the library must plan afresh (it
    once kept a half-patched plan)."""
    from oracle.adapters import OracleSink, queries_fp64
    from oracle import attention_c
    wl = sw.bfs_tot(n_queries=1, prompt=64, step=47, heads=(8, 2, 128), width=4, keep=2, depth=2)
    u, w = wl.leaves[0], wl.leaves[1]
    leaves, q_lens = [u, u, w], [1, 1, 1]
    tree = build_gpu_tree(wl, extra_pages=16, kernel_mode=3)
    sink = OracleSink.for_workload(wl)
    sw.replay(wl, sink)
    q = sw.gen_queries(wl, device="cuda")[:3].contiguous()
    qd = queries_fp64(q)
    tree.decode_attention(leaves, q_lens, q, wl.sm_scale)
    for step in range(4):                           # 47 -> 48 fills the page, 49 starts the next one
        k = sw.normal_values(41, 1, 50 + step, torch.arange(2), 2, 128, 0.5, "cuda").to(torch.bfloat16)
        v = sw.normal_values(41, 2, 50 + step, torch.arange(2), 2, 128, 0.5, "cuda").to(torch.bfloat16)
        tree.append_tokens([u, w], k, v)
        for i, node in enumerate([u, w]):
            sink.append(node, k[i:i + 1], v[i:i + 1])
        out, lse = tree.decode_attention(leaves, q_lens, q, wl.sm_scale)
        ref_o, ref_l, _ = attention_c.attention(sink.tree, leaves, q_lens, qd, wl.sm_scale)
        got = (out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64))
        check(wl, got, (ref_o, ref_l), f"duplicate request, step {step}")
    tree.close()

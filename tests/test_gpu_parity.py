"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle, element by element."""

import numpy as np
import pytest
import torch

import spex_workloads as sw
from gpu_common import assert_close, assert_v_round_trip, build_gpu_tree, run_gpu, run_oracle

pytestmark = pytest.mark.gpu


def test_generators_agree_between_cpu_and_gpu():
    for tag, scale in ((1, 0.5), (2, 1.0)):
        a = sw.normal_values(9, tag, 1234567, torch.arange(300), 4, 128, scale, "cpu")
        b = sw.normal_values(9, tag, 1234567, torch.arange(300), 4, 128, scale, "cuda").cpu()
        assert torch.equal(a, b)
    x = sw.normal_values(9, 1, 5, torch.arange(100), 4, 128, 0.5, "cpu")
    ca, sa = sw.quantise_pages(x, 0, 16, None)
    cb, sb = sw.quantise_pages(x.cuda(), 0, 16, None)
    assert torch.equal(ca, cb.cpu()) and torch.equal(sa, sb.cpu())
    assert torch.equal(x.to(torch.bfloat16), x.cuda().to(torch.bfloat16).cpu())


@pytest.mark.parametrize("kv_dtype,heads", [("f32", (4, 2, 64)), ("f32", (2, 1, 40)),
                                            ("bf16", (8, 2, 64)), ("bf16", (4, 4, 128)),
                                            ("bf16", (2, 2, 96)), ("fp8_e4m3", (10, 2, 128)),
                                            ("fp8_e4m3", (4, 2, 64))])
def test_append_then_gather_is_bit_exact(kv_dtype, heads):
    """K always; V up to the half-precision storage of MFMA-tiled bf16 pools (see assert_v_round_trip)."""
    wl = sw.random_trace(31, heads=heads, kv_dtype=kv_dtype,
                         q_dtype="f32" if kv_dtype == "f32" else "bf16", n_ops=40, max_tokens=45)
    rng = np.random.default_rng(1)
    order = rng.permutation(wl.peak_pages() + 3).tolist()
    tree = build_gpu_tree(wl, free_order=order, extra_pages=3, pool_fill=0xFF)

    class Rec:
        def __init__(self):
            self.k, self.v, self.ks, self.vs, self.n = {}, {}, {}, {}, []

        def fork(self, parent, n):
            ids = list(range(len(self.n), len(self.n) + n))
            self.n += [0] * n
            return ids

        def prune(self, node):
            pass

        def append(self, node, k, v, ks, vs, n_tokens=None):
            self.k.setdefault(node, []).append(k)
            self.v.setdefault(node, []).append(v)
            if ks is not None:
                self.ks.setdefault(node, []).append(ks)
                self.vs.setdefault(node, []).append(vs)

    rec = Rec()
    sw.replay(wl, rec, device="cpu")
    _, _, alive = wl.node_tokens()
    checked = 0
    for u, pieces in rec.k.items():
        if not alive[u]:
            continue
        k_ref, v_ref = torch.cat(pieces, 0), torch.cat(rec.v[u], 0)
        n = k_ref.shape[0]
        k, v, ks, vs = tree.gather_kv(u, 0, n)
        assert torch.equal(k.cpu(), k_ref)
        assert_v_round_trip(v, v_ref, f"node {u}")
        if n > 3:
            k2, v2, _, _ = tree.gather_kv(u, 2, n - 3)
            assert torch.equal(k2.cpu(), k_ref[2:n - 1])
            assert_v_round_trip(v2, v_ref[2:n - 1], f"node {u}, from token 2")
        if kv_dtype == "fp8_e4m3":
            ks_ref = torch.cat(rec.ks[u], 0).repeat_interleave(16, 0)[:n]
            vs_ref = torch.cat(rec.vs[u], 0).repeat_interleave(16, 0)[:n]
            assert torch.equal(ks.cpu(), ks_ref) and torch.equal(vs.cpu(), vs_ref)
        checked += 1
    assert checked > 5
    tree.close()


def test_config_1_tiny_tree_fp32():
    wl = sw.tiny_tree()
    assert_close(run_gpu(wl), run_oracle(wl), "f32", "tiny_tree")


RANDOM_CASES = [
    dict(seed=41, heads=(8, 2, 64), kv_dtype="bf16", max_q_len=1),
    dict(seed=42, heads=(8, 2, 128), kv_dtype="bf16", max_q_len=4),
    dict(seed=43, heads=(28, 4, 128), kv_dtype="bf16", max_q_len=3),
    dict(seed=44, heads=(16, 2, 64), kv_dtype="bf16", max_q_len=6),
    dict(seed=45, heads=(10, 2, 128), kv_dtype="fp8_e4m3", max_q_len=6),
    dict(seed=46, heads=(8, 8, 64), kv_dtype="fp8_e4m3", max_q_len=2),
    dict(seed=47, heads=(4, 2, 64), kv_dtype="f32", max_q_len=3),
    dict(seed=48, heads=(6, 3, 40), kv_dtype="bf16", max_q_len=2),      # no MFMA kernel: generic
    dict(seed=49, heads=(4, 1, 128), kv_dtype="bf16", max_q_len=9),     # 36 rows: cut into pieces
    dict(seed=50, heads=(16, 2, 64), kv_dtype="bf16", max_q_len=20),    # up to 160 rows per request
    dict(seed=53, heads=(40, 2, 128), kv_dtype="fp8_e4m3", max_q_len=5),  # G = 20: two row tiles at least
]


@pytest.mark.parametrize("case", RANDOM_CASES, ids=lambda c: f"{c['kv_dtype']}-{c['heads']}-q{c['max_q_len']}")
@pytest.mark.parametrize("chunks", [(0, 0), (1, 1), (3, 2)])
def test_random_trees_match_oracle(case, chunks):
    wl = sw.random_trace(case["seed"], heads=case["heads"], kv_dtype=case["kv_dtype"],
                         q_dtype="f32" if case["kv_dtype"] == "f32" else "bf16",
                         n_ops=70, max_tokens=90, max_q_len=case["max_q_len"])
    ref = run_oracle(wl)
    got = run_gpu(wl, prefix_chunk_pages=chunks[0], suffix_chunk_pages=chunks[1], kernel_mode=2)
    assert_close(got, ref, case["kv_dtype"], wl.name)


def walk_applies(wl, row_tiles=0):
    # wider requests are cut into pieces of query tokens; one query token must fit a wavefront
    G = wl.num_q_heads // wl.num_kv_heads
    mfma = wl.kv_dtype != "f32" and wl.head_dim in (64, 128)
    return mfma and G <= (16 * row_tiles if row_tiles else 64)


@pytest.mark.parametrize("case", RANDOM_CASES, ids=lambda c: f"{c['kv_dtype']}-{c['heads']}-q{c['max_q_len']}")
@pytest.mark.parametrize("row_tiles,waves", [(0, 0), (1, 4), (2, 4), (4, 4), (1, 8), (2, 8), (4, 8), (1, 2), (2, 2)])
def test_random_trees_tree_walk_kernel(case, row_tiles, waves):
    import paper_2605_10195_amd as spex
    wl = sw.random_trace(case["seed"], heads=case["heads"], kv_dtype=case["kv_dtype"],
                         q_dtype="f32" if case["kv_dtype"] == "f32" else "bf16",
                         n_ops=70, max_tokens=90, max_q_len=case["max_q_len"])
    if not walk_applies(wl, row_tiles):
        with pytest.raises(spex.SpexError) as e:
            run_gpu(wl, kernel_mode=3, walk_row_tiles=row_tiles, walk_waves=waves)
        assert e.value.name == "UNSUPPORTED"
        return
    tree = build_gpu_tree(wl, kernel_mode=3, walk_row_tiles=row_tiles, walk_waves=waves)
    got = run_gpu(wl, tree=tree)
    info = tree.last_launch_info()
    tree.close()
    assert info["walk_row_tiles"] == (row_tiles or info["walk_row_tiles"]) and info["walk_row_tiles"] > 0
    assert info["walk_waves"] == (waves or info["walk_waves"]) and info["walk_waves"] in (2, 4, 8)
    assert_close(got, run_oracle(wl), case["kv_dtype"], wl.name)


@pytest.mark.parametrize("waves", [0, 2])
@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8_e4m3"])
def test_tree_walk_kernel_with_more_blocks_than_its_lds_copy_holds(kv_dtype, waves):
    # 9 000-token prompt + 1 100-token steps: > 256 two-page blocks per row block, so the kernel
    # reads its block records through the scalar path instead of from LDS
    wl = sw.bfs_tot(n_queries=1, prompt=9000, step=1100, width=4, keep=2, depth=2, heads=(8, 2, 128),
                    kv_dtype=kv_dtype)
    tree = build_gpu_tree(wl, kernel_mode=3, walk_waves=waves)
    got = run_gpu(wl, tree=tree)
    dump = tree.walk_dump(wl.leaves, wl.q_lens)
    tree.close()
    rbs = np.array(dump["row_blocks"]).reshape(-1, 3 + 3 * dump["waves"])
    assert (rbs[:, 2] + rbs[:, 3:3 + dump["waves"]].sum(1)).max() > 256
    assert_close(got, run_oracle(wl), kv_dtype, wl.name)


def test_automatic_mode_picks_the_tree_walk_kernel_for_short_paths():
    wl = sw.random_trace(42, heads=(8, 2, 128), kv_dtype="bf16", n_ops=70, max_tokens=90, max_q_len=4)
    tree = build_gpu_tree(wl)
    got = run_gpu(wl, tree=tree)
    assert tree.last_launch_info()["walk_row_tiles"] > 0
    tree.set_tuning(0, 0, 2, 0, 0)
    split = run_gpu(wl, tree=tree)
    assert tree.last_launch_info()["walk_row_tiles"] == 0
    tree.close()
    ref = run_oracle(wl)
    assert_close(got, ref, "bf16", "walk")
    assert_close(split, ref, "bf16", "split")


@pytest.mark.parametrize("case", RANDOM_CASES[:6], ids=lambda c: f"{c['kv_dtype']}-{c['heads']}")
def test_generic_kernels_match_oracle_and_mfma(case):
    wl = sw.random_trace(case["seed"] + 100, heads=case["heads"], kv_dtype=case["kv_dtype"],
                         n_ops=60, max_tokens=70, max_q_len=case["max_q_len"])
    ref = run_oracle(wl)
    slow = run_gpu(wl, kernel_mode=1)
    assert_close(slow, ref, case["kv_dtype"], "generic")
    for mode in (2, 3):
        fast = run_gpu(wl, kernel_mode=mode)
        assert_close(fast, ref, case["kv_dtype"], f"mfma mode {mode}")
        assert np.max(np.abs(slow[0] - fast[0])) < 1e-3


REDUCED = [
    sw.bfs_tot(n_queries=3, prompt=200, step=72),
    sw.mcts_skewed(n_queries=5, prompt=(100, 300), step=(10, 90), max_leaves=24),
    sw.spec_at_scale(n_queries=3, prompt=300, step=100, branches=12),
    sw.tot_with_drafts(n_queries=3, prompt=250, step=56),
    sw.bfs_tot(n_queries=2, prompt=64, step=32, kv_dtype="fp8_e4m3", heads=(16, 2, 64)),
    sw.step_prefill(n_queries=2, prompt=90, step=44, width=8, keep=2, depth=3),           # q_len = 44: 176 rows per branch
    sw.step_prefill(n_queries=1, prompt=50, step=70, width=4, keep=2, depth=2, kv_dtype="fp8_e4m3",
                    heads=(10, 2, 128)),                                                   # 350 rows, G = 5
]


@pytest.mark.parametrize("wl", REDUCED, ids=lambda w: w.name + "_" + w.kv_dtype)
@pytest.mark.parametrize("mode,waves", [(2, 0), (3, 4), (3, 8), (3, 2)])
def test_reduced_config_shapes_match_oracle(wl, mode, waves):
    assert_close(run_gpu(wl, kernel_mode=mode, walk_waves=waves), run_oracle(wl), wl.kv_dtype,
                 f"{wl.name} mode {mode} waves {waves}")


def test_nan_poisoned_pool_and_ragged_pages():
    # 0xFF bytes are NaN in bf16 and in e4m3: unused slots of partial pages must never contribute.
    for kv in ("bf16", "fp8_e4m3"):
        wl = sw.random_trace(51, heads=(8, 2, 128), kv_dtype=kv, n_ops=60, max_tokens=37, max_q_len=3)
        ref = run_oracle(wl)
        for mode, waves in ((2, 0), (3, 4), (3, 8)):
            got = run_gpu(wl, pool_fill=0xFF, extra_pages=7, kernel_mode=mode, walk_waves=waves)
            assert_close(got, ref, kv, f"poisoned {kv} mode {mode} waves {waves}")


def test_page_placement_does_not_change_the_result():
    wl = sw.random_trace(52, heads=(8, 2, 128), kv_dtype="bf16", n_ops=60, max_tokens=80, max_q_len=2)
    n = wl.peak_pages() + 11
    for mode in (2, 3):
        base = run_gpu(wl, kernel_mode=mode)
        for s in range(3):
            order = np.random.default_rng(s).permutation(n).tolist()
            other = run_gpu(wl, free_order=order, extra_pages=11, kernel_mode=mode)
            assert np.array_equal(base[0], other[0]) and np.array_equal(base[1], other[1])


def test_identical_token_paths_give_identical_outputs():
    wl = sw.Workload("twins", 8, 2, 128, 16, "bf16", "bf16", 0.5, 78)
    b = sw.trees._Builder(wl)
    (root,) = b.fork(-1, 1)
    b.append(root, 100)
    a1, a2 = b.fork(root, 2)
    b.append(a1, 45, key=1234)
    b.append(a2, 45, key=1234)
    (c1,) = b.fork(a1, 1)
    (c2,) = b.fork(a2, 1)
    b.append(c1, 30, key=99)
    b.append(c2, 30, key=99)
    b.request(c1, 3, key=5)
    b.request(c2, 3, key=5)
    for mode in (2, 3):
        out, lse = run_gpu(wl, kernel_mode=mode)
        assert np.array_equal(out[:3], out[3:]) and np.array_equal(lse[:3], lse[3:])
        assert_close((out, lse), run_oracle(wl), "bf16", "twins")


def test_duplicate_interior_and_empty_requests():
    wl = sw.Workload("odd_requests", 8, 2, 64, 16, "bf16", "bf16", 0.5, 79)
    b = sw.trees._Builder(wl)
    (root,) = b.fork(-1, 1)
    b.append(root, 37)
    a, e = b.fork(root, 2)
    b.append(a, 5)
    b.request(a, 1)
    b.request(a, 7)          # same node again; 7 queries reach 2 tokens into the shared root
    b.request(root, 2)       # interior node
    b.request(e, 1)          # empty child: sees exactly the root
    for mode in (2, 3):
        assert_close(run_gpu(wl, kernel_mode=mode), run_oracle(wl), "bf16", f"{wl.name} mode {mode}")


@pytest.mark.parametrize("mode", [2, 3])
def test_decode_loop_patches_or_replans_after_every_append(mode):
    wl = sw.bfs_tot(n_queries=2, prompt=48, step=20)
    tree = build_gpu_tree(wl, extra_pages=64, kernel_mode=mode)
    states = set()
    from oracle.adapters import OracleSink, queries_fp64
    sink = OracleSink.for_workload(wl)
    sw.replay(wl, sink)
    q = sw.gen_queries(wl, device="cuda")
    qd = queries_fp64(q)
    for step in range(20):                                   # crosses a page boundary
        k = sw.normal_values(5, 1, 777 + step, torch.arange(len(wl.leaves)), 8, 128, 0.5, "cuda")
        v = sw.normal_values(5, 2, 777 + step, torch.arange(len(wl.leaves)), 8, 128, 0.5, "cuda")
        k, v = k.to(torch.bfloat16), v.to(torch.bfloat16)
        for i, leaf in enumerate(wl.leaves):
            tree.append_step(leaf, k[i:i + 1].contiguous(), v[i:i + 1].contiguous())
            sink.append(leaf, k[i:i + 1], v[i:i + 1])
        # the first call plans afresh; later ones only when an append has started a page
        new_page = step == 0 or tree.node_info(wl.leaves[0])["n_tokens"] % 16 == 1
        out, lse = tree.decode_attention(wl.leaves, None, q, wl.sm_scale)
        state = tree.last_launch_info()["plan_rebuilt"]          # 1 planned afresh, 2 patched
        states.add(state)
        out2, _ = tree.decode_attention(wl.leaves, None, q, wl.sm_scale)
        # split lists cannot take a started page; tree-walk lists take it as a patch (page b of
        # the last block, or a block in the wavefront's room) unless it is the first plan
        want_state = 1 if (new_page and (mode == 2 or step == 0)) else 2
        assert state == want_state and tree.last_launch_info()["plan_rebuilt"] == 0
        if step % 3 == 2 or new_page:
            ref = sink.tree.attention(wl.leaves, None, qd, wl.sm_scale)
            got = (out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64))
            assert_close(got, ref, "bf16", f"decode step {step}")
            assert torch.equal(out, out2)
    assert states == {1, 2}
    tree.close()


def test_device_errors_are_reported_not_raised_from_kernels():
    import paper_2605_10195_amd as spex
    t = spex.SpexTree(8, 2, 64, 16, "bf16", "bf16", num_pages=4, device="cuda")
    (r,) = t.fork(-1, 1)
    q = torch.zeros((1, 8, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(spex.SpexError) as e:
        t.decode_attention([r], None, q, 0.125)              # no tokens yet
    assert e.value.name == "EMPTY_PATH"
    k = torch.zeros((70, 2, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(spex.SpexError) as e:
        t.append_step(r, k, k)                                # 5 pages > 4
    assert e.value.name == "OOM_PAGES"
    t.append_step(r, k[:64].contiguous(), k[:64].contiguous())
    out, lse = t.decode_attention([r], None, q, 0.125)
    torch.cuda.synchronize()
    assert torch.all(out == 0) and abs(lse[0, 0].item() - np.log(64)) < 1e-5
    t.close()


# ------------------------------------------------------------------ wide groups / pool layouts
WIDE = [
    # 40 branches x G=8 -> 320 stacked rows at the root: three 128-row spans of the cooperative kernel
    sw.spec_at_scale(n_queries=2, prompt=150, step=40, branches=40, heads=(32, 4, 128)),
    # 24 branches x 6 drafts x G=5 -> 720 rows, fp8, causal drafts reach into partial pages
    sw.tot_with_drafts(n_queries=1, prompt=90, step=24, depth=3, drafts=6, heads=(20, 4, 128)),
    sw.spec_at_scale(n_queries=2, prompt=100, step=30, branches=20, heads=(16, 2, 64), kv_dtype="fp8_e4m3"),
    sw.bfs_tot(n_queries=2, prompt=100, step=40, width=64, keep=16, depth=3, heads=(16, 4, 64)),
]


@pytest.mark.parametrize("wl", WIDE, ids=lambda w: f"{w.name}_{w.kv_dtype}_{w.num_q_heads}")
@pytest.mark.parametrize("mode", [2, 1, 3, 38])
def test_wide_groups_match_oracle(wl, mode):
    ref = run_oracle(wl)
    waves, mode = (8, 3) if mode == 38 else (0, mode)          # 38: tree-walk with 8 wavefronts
    for chunks in ((0, 0), (3, 2)) if mode != 3 else ((0, 0),):
        got = run_gpu(wl, prefix_chunk_pages=chunks[0], suffix_chunk_pages=chunks[1], kernel_mode=mode,
                      walk_waves=waves)
        assert_close(got, ref, wl.kv_dtype, f"{wl.name} mode {mode} chunks {chunks}")


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8_e4m3", "f32"])
def test_interleaved_kv_pool(kv_dtype):
    wl = sw.random_trace(61, heads=(8, 2, 128) if kv_dtype != "f32" else (4, 2, 64), kv_dtype=kv_dtype,
                         q_dtype="f32" if kv_dtype == "f32" else "bf16", n_ops=60, max_tokens=70,
                         max_q_len=3)
    ref = run_oracle(wl)
    order = np.random.default_rng(3).permutation(wl.peak_pages() + 5).tolist()
    got = run_gpu(wl, interleave_kv=True, free_order=order, extra_pages=5, pool_fill=0xFF)
    assert_close(got, ref, kv_dtype, "interleaved " + kv_dtype)
    sep = run_gpu(wl, free_order=order, extra_pages=5)
    assert np.array_equal(got[0], sep[0])


def test_softmax_scale_must_be_positive():
    import paper_2605_10195_amd as spex
    t = spex.SpexTree(8, 2, 64, 16, "bf16", "bf16", num_pages=4, device="cuda")
    (r,) = t.fork(-1, 1)
    k = torch.zeros((5, 2, 64), dtype=torch.bfloat16, device="cuda")
    t.append_step(r, k, k)
    q = torch.zeros((1, 8, 64), dtype=torch.bfloat16, device="cuda")
    for bad in (0.0, -1.0, float("nan"), float("inf")):
        with pytest.raises(spex.SpexError) as e:
            t.decode_attention([r], None, q, bad)
        assert e.value.name == "INVALID_ARG"
    t.close()


# ------------------------------------------------------------------ started pages as patches
@pytest.mark.parametrize("kv_dtype,heads,shape", [("bf16", (28, 4, 128), (0, 0)), ("fp8_e4m3", (8, 2, 128), (0, 0)),
                                                  ("bf16", (8, 8, 64), (0, 0)), ("bf16", (8, 2, 128), (2, 8)),
                                                  ("bf16", (8, 2, 64), (2, 4))])
def test_decode_loop_starts_pages_by_patches(kv_dtype, heads, shape):
    """Branches of different lengths: in almost every iteration some branch starts a page.  With the
    tree-walk lists those pages are patched in (free half of the last block, else the room behind
    the wavefront's private blocks) until some wavefront's room is used up; the attention must
    match the oracle after every kind of step, and the patched device lists must give what a
    fresh plan gives."""
    from oracle.adapters import OracleSink, queries_fp64
    wl = sw.mcts_skewed(n_queries=3, prompt=(30, 90), step=(5, 40), max_leaves=10, heads=heads, kv_dtype=kv_dtype)
    nodes = sorted(set(wl.leaves))
    tree = build_gpu_tree(wl, extra_pages=8 * len(nodes) + 8, kernel_mode=3, walk_row_tiles=shape[0],
                          walk_waves=shape[1])
    sink = OracleSink.for_workload(wl)
    sw.replay(wl, sink)
    q = sw.gen_queries(wl, device="cuda")
    qd = queries_fp64(q)
    H, D = heads[1], heads[2]
    childless = [u for u in nodes if tree.node_info(u)["n_live_children"] == 0]
    assert len(childless) >= 6
    page_patches = fresh = 0
    for step in range(76):
        x_k = sw.normal_values(8, 1, 300 + step, torch.arange(len(childless)), H, D, 0.5, "cuda").to(torch.bfloat16)
        x_v = sw.normal_values(8, 2, 300 + step, torch.arange(len(childless)), H, D, 0.5, "cuda").to(torch.bfloat16)
        started = sum(tree.append_new_pages(u, 1) for u in childless)
        if kv_dtype == "fp8_e4m3":
            s = torch.full((len(childless), H), 2.0 ** -6, dtype=torch.float32, device="cuda")
            tree.append_tokens(childless, x_k.contiguous(), x_v.contiguous(), s, s, quantize=True)
            for i, u in enumerate(childless):
                new = tree.node_info(u)["n_tokens"] % 16 == 1
                sink.append_quantised(u, x_k[i:i + 1].cpu(), x_v[i:i + 1].cpu(), s[i:i + 1].cpu() if new else None,
                                      s[i:i + 1].cpu() if new else None)
        else:
            tree.append_tokens(childless, x_k.contiguous(), x_v.contiguous())
            for i, u in enumerate(childless):
                sink.append(u, x_k[i:i + 1].cpu(), x_v[i:i + 1].cpu())
        out, lse = tree.decode_attention(wl.leaves, wl.q_lens, q, wl.sm_scale)
        state = tree.last_launch_info()["plan_rebuilt"]
        assert state in (1, 2)
        page_patches += state == 2 and started > 0
        fresh += state == 1
        if started or step % 6 == 0:
            ref = sink.tree.attention(wl.leaves, wl.q_lens, qd, wl.sm_scale)
            got = (out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64))
            assert_close(got, ref, kv_dtype, f"{kv_dtype} step {step} state {state} started {started}")
    assert page_patches >= 20 and fresh >= 2          # room ran out at least once after the first plan
    tree.close()


def test_step_appends_that_start_several_pages_are_patched():
    """Whole steps (runs of 5-45 tokens) appended to some branches between attention calls: the
    tree-walk lists on the device take the started pages as one batch of patches in which no
    index appears twice."""
    from oracle.adapters import OracleSink, queries_fp64
    wl = sw.mcts_skewed(n_queries=3, prompt=(30, 90), step=(5, 40), max_leaves=10, heads=(8, 2, 128))
    nodes = sorted(set(wl.leaves))
    tree = build_gpu_tree(wl, extra_pages=24 * len(nodes) + 8, kernel_mode=3)
    sink = OracleSink.for_workload(wl)
    sw.replay(wl, sink)
    q = sw.gen_queries(wl, device="cuda")
    qd = queries_fp64(q)
    childless = [u for u in nodes if tree.node_info(u)["n_live_children"] == 0]
    rng = np.random.default_rng(21)
    tree.decode_attention(wl.leaves, wl.q_lens, q, wl.sm_scale)
    patched = fresh = 0
    for step in range(14):
        for i, u in enumerate(childless):
            if rng.random() < 0.6:
                n = int(rng.integers(5, 46))
                k = sw.normal_values(9, 1, 1000 * step + i, torch.arange(n), 2, 128, 0.5, "cuda").to(torch.bfloat16)
                v = sw.normal_values(9, 2, 1000 * step + i, torch.arange(n), 2, 128, 0.5, "cuda").to(torch.bfloat16)
                tree.append_step(u, k.contiguous(), v.contiguous())
                sink.append(u, k, v)
        out, lse = tree.decode_attention(wl.leaves, wl.q_lens, q, wl.sm_scale)
        state = tree.last_launch_info()["plan_rebuilt"]
        patched += state == 2
        fresh += state == 1
        ref = sink.tree.attention(wl.leaves, wl.q_lens, qd, wl.sm_scale)
        got = (out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64))
        assert_close(got, ref, "bf16", f"step {step} state {state}")
    assert patched >= 3 and fresh >= 1
    tree.close()


def test_patches_left_waiting_are_merged_with_later_ones():
    """Requests with 40 queries each: one appended token moves 41 list entries per branch, more
    than an append launch takes along, so they wait for the next attention call.  A second append
    before that call adds newer values for the same entries; the device must end up with the
    newest of each."""
    from oracle.adapters import OracleSink, queries_fp64
    wl = sw.step_prefill(n_queries=2, prompt=64, step=40, heads=(8, 2, 128))
    tree = build_gpu_tree(wl, extra_pages=4 * len(wl.leaves) + 4, kernel_mode=3)
    sink = OracleSink.for_workload(wl)
    sw.replay(wl, sink)
    q = sw.gen_queries(wl, device="cuda")
    qd = queries_fp64(q)
    tree.decode_attention(wl.leaves, wl.q_lens, q, wl.sm_scale)
    L = len(wl.leaves)
    for rnd in range(3):
        for rep in range(2):                                  # two appends, no attention in between
            k = sw.normal_values(7, 1, 50 + 2 * rnd + rep, torch.arange(L), 2, 128, 0.5, "cuda").to(torch.bfloat16)
            v = sw.normal_values(7, 2, 50 + 2 * rnd + rep, torch.arange(L), 2, 128, 0.5, "cuda").to(torch.bfloat16)
            tree.append_tokens(wl.leaves, k.contiguous(), v.contiguous())
            for i, u in enumerate(wl.leaves):
                sink.append(u, k[i:i + 1], v[i:i + 1])
        out, lse = tree.decode_attention(wl.leaves, wl.q_lens, q, wl.sm_scale)
        assert tree.last_launch_info()["plan_rebuilt"] == 2
        ref = sink.tree.attention(wl.leaves, wl.q_lens, qd, wl.sm_scale)
        got = (out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64))
        assert_close(got, ref, "bf16", f"round {rnd}")
    tree.close()


# ------------------------------------------------------------------ capture in a HIP graph
@pytest.mark.parametrize("mode", [2, 3])
def test_attention_with_a_cached_plan_can_be_captured_in_a_graph(mode):
    """A call that repeats the previous request on an unchanged tree only launches kernels (no
    planning, upload, allocation or event), so a caller may record it in a HIP graph -- e.g. one
    call per model layer.  Every replay, with eager work and synchronisation in between and new
    query values in the same buffer, must give what the eager call gives."""
    wl = sw.bfs_tot(n_queries=3, prompt=72, step=24)
    tree = build_gpu_tree(wl, kernel_mode=mode)
    q = sw.gen_queries(wl, device="cuda")
    out = torch.empty((q.shape[0], wl.num_q_heads, wl.head_dim), dtype=torch.float32, device="cuda")
    lse = torch.empty((q.shape[0], wl.num_q_heads), dtype=torch.float32, device="cuda")
    tree.decode_attention(wl.leaves, wl.q_lens, q, wl.sm_scale, out, lse)      # plans, uploads, allocates
    tree.decode_attention(wl.leaves, wl.q_lens, q, wl.sm_scale, out, lse)
    assert tree.last_launch_info()["plan_rebuilt"] == 0
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            tree.decode_attention(wl.leaves, wl.q_lens, q, wl.sm_scale, out, lse)
    torch.cuda.synchronize()
    for rep in range(4):
        q.copy_((q.float() * (0.5 + 0.25 * rep)).to(q.dtype))                  # new queries, same buffer
        eager_out, eager_lse = tree.decode_attention(wl.leaves, wl.q_lens, q, wl.sm_scale)
        out.fill_(7.0)
        lse.fill_(7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager_out) and torch.equal(lse, eager_lse), rep
    del graph
    tree.close()


# ------------------------------------------------------------------ decode loop, one launch per append
@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8_e4m3", "f32"])
def test_decode_loop_with_append_tokens(kv_dtype):
    """Every iteration appends one token to every leaf with one call, then attends.  Checked
    against the oracle (same tokens appended to its own tree) and against gather_kv bit for bit."""
    from oracle.adapters import OracleSink, queries_fp64
    heads = (8, 2, 128) if kv_dtype != "f32" else (4, 2, 64)
    wl = sw.bfs_tot(n_queries=2, prompt=40, step=13, heads=heads, kv_dtype=kv_dtype,
                    q_dtype="f32" if kv_dtype == "f32" else "bf16")
    tree = build_gpu_tree(wl, extra_pages=2 * len(wl.leaves) + 4, pool_fill=0xFF)
    sink = OracleSink.for_workload(wl)
    sw.replay(wl, sink)
    q = sw.gen_queries(wl, device="cuda")
    qd = queries_fp64(q)
    H, D = heads[1], heads[2]
    L = len(wl.leaves)
    grown = {u: [] for u in wl.leaves}
    states = set()
    for step in range(22):
        x_k = sw.normal_values(6, 1, 900 + step, torch.arange(L), H, D, 0.5, "cuda")
        x_v = sw.normal_values(6, 2, 900 + step, torch.arange(L), H, D, 0.5, "cuda")
        ks = vs = None
        if kv_dtype == "fp8_e4m3":
            # a token that starts a page brings its own scale; others use the page's scale
            k = torch.empty((L, H, D), dtype=torch.uint8, device="cuda")
            v = torch.empty_like(k)
            ks = torch.ones((L, H), dtype=torch.float32, device="cuda")
            vs = torch.ones((L, H), dtype=torch.float32, device="cuda")
            for i, u in enumerate(wl.leaves):
                n_old = tree.node_info(u)["n_tokens"]
                prev = None
                if n_old % 16:
                    _, _, pk, pv = tree.gather_kv(u, n_old - 1, 1)
                    prev = (pk[0], pv[0])
                ck, sk = sw.quantise_pages(x_k[i:i + 1], n_old % 16, 16, None if prev is None else prev[0])
                cv, sv = sw.quantise_pages(x_v[i:i + 1], n_old % 16, 16, None if prev is None else prev[1])
                k[i], v[i] = ck[0], cv[0]
                if sk.shape[0]:
                    ks[i], vs[i] = sk[0], sv[0]
                sink.append(u, ck.cpu(), cv.cpu(), sk.cpu() if sk.shape[0] else None,
                            sv.cpu() if sv.shape[0] else None)
                grown[u].append((ck.cpu(), cv.cpu()))
            k, v = k.view(torch.float8_e4m3fn), v.view(torch.float8_e4m3fn)
        else:
            dt = torch.bfloat16 if kv_dtype == "bf16" else torch.float32
            k, v = x_k.to(dt).contiguous(), x_v.to(dt).contiguous()
            for i, u in enumerate(wl.leaves):
                sink.append(u, k[i:i + 1].cpu(), v[i:i + 1].cpu())
                grown[u].append((k[i:i + 1].cpu(), v[i:i + 1].cpu()))
        tree.append_tokens(wl.leaves, k, v, ks, vs)
        out, lse = tree.decode_attention(wl.leaves, None, q, wl.sm_scale)
        states.add(tree.last_launch_info()["plan_rebuilt"])
        if step % 4 == 3 or step < 2:
            ref = sink.tree.attention(wl.leaves, None, qd, wl.sm_scale)
            got = (out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64))
            assert_close(got, ref, kv_dtype, f"{kv_dtype} decode step {step}")
    assert states == {1, 2}
    for u in wl.leaves[:6]:                                    # what was appended is what is stored
        n = tree.node_info(u)["n_tokens"]
        gk, gv, _, _ = tree.gather_kv(u, n - 22, 22)
        want_k = torch.cat([a for a, _ in grown[u]], 0)
        want_v = torch.cat([b for _, b in grown[u]], 0)
        assert torch.equal(gk.cpu().view(want_k.dtype), want_k)
        assert_v_round_trip(gv.view(want_v.dtype), want_v, f"node {u}")
    tree.close()


# ------------------------------------------------------------------ draft token trees (Sec. 6.5)
TOKEN_TREE_CASES = [
    dict(seed=71, heads=(8, 2, 64), kv_dtype="bf16", max_q_len=16),      # up to 64 rows per request
    dict(seed=72, heads=(4, 4, 128), kv_dtype="bf16", max_q_len=32),     # the widest mask
    dict(seed=73, heads=(28, 4, 128), kv_dtype="bf16", max_q_len=8),
    dict(seed=74, heads=(10, 2, 128), kv_dtype="fp8_e4m3", max_q_len=12),
    dict(seed=75, heads=(8, 8, 64), kv_dtype="fp8_e4m3", max_q_len=16),
    dict(seed=76, heads=(4, 2, 64), kv_dtype="f32", max_q_len=8),        # generic kernels only
    dict(seed=77, heads=(6, 3, 40), kv_dtype="bf16", max_q_len=8),       # no MFMA kernel: generic
]


def token_tree_workload(case, arbitrary=False):
    wl = sw.random_trace(case["seed"], heads=case["heads"], kv_dtype=case["kv_dtype"],
                         q_dtype="f32" if case["kv_dtype"] == "f32" else "bf16",
                         n_ops=60, max_tokens=90, max_q_len=case["max_q_len"])
    wl = sw.with_draft_trees(wl)
    if arbitrary:
        # any bit pattern is a valid request as long as every query sees something: also queries
        # that see no draft at all (not even themselves) or a later draft
        rng = np.random.default_rng(case["seed"])
        masks, o = [], 0
        for leaf, ql in zip(wl.leaves, wl.q_lens):
            prefix = wl.path_tokens(leaf) - ql
            for j in range(ql):
                m = int(rng.integers(0, 1 << ql)) if rng.random() < 0.8 else 0
                masks.append(m if (m or prefix) else 1 << j)
            o += ql
        wl.draft_masks = masks
    return wl


@pytest.mark.parametrize("case", TOKEN_TREE_CASES, ids=lambda c: f"{c['kv_dtype']}-{c['heads']}-q{c['max_q_len']}")
@pytest.mark.parametrize("mode,row_tiles", [(0, 0), (1, 0), (2, 0), (3, 0), (3, 2), (3, 4)])
@pytest.mark.parametrize("arbitrary", [False, True], ids=["ancestors", "any_bits"])
def test_draft_token_trees_match_oracle(case, mode, row_tiles, arbitrary):
    import paper_2605_10195_amd as spex
    wl = token_tree_workload(case, arbitrary)
    assert max(wl.q_lens) > 4
    if mode == 3 and not walk_applies(wl, row_tiles):
        with pytest.raises(spex.SpexError) as e:
            run_gpu(wl, kernel_mode=3, walk_row_tiles=row_tiles)
        assert e.value.name == "UNSUPPORTED"
        return
    tree = build_gpu_tree(wl, kernel_mode=mode, walk_row_tiles=row_tiles)
    got = run_gpu(wl, tree=tree)
    info = tree.last_launch_info()
    tree.close()
    if mode == 3:
        assert info["walk_row_tiles"] > 0 and info["walk_waves"] == 4
    elif mode in (1, 2):
        assert info["walk_row_tiles"] == 0          # mode 0: the library's choice, as without masks
    assert_close(got, run_oracle(wl), case["kv_dtype"], wl.name)


@pytest.mark.parametrize("case", TOKEN_TREE_CASES[:5], ids=lambda c: f"{c['kv_dtype']}-{c['heads']}")
def test_chain_masks_give_the_bits_of_the_call_without_masks(case):
    wl = token_tree_workload(case)
    chain = [(2 << j) - 1 for ql in wl.q_lens for j in range(ql)]
    q = sw.gen_queries(wl, device="cuda")
    for mode in (3, 1):
        tree = build_gpu_tree(wl, kernel_mode=mode)
        a, la = tree.decode_attention(wl.leaves, wl.q_lens, q, wl.sm_scale)
        b, lb = tree.decode_attention(wl.leaves, wl.q_lens, q, wl.sm_scale, draft_masks=chain)
        assert tree.last_launch_info()["plan_rebuilt"] == 1       # the masks are part of the request
        torch.cuda.synchronize()
        assert torch.equal(a, b) and torch.equal(la, lb)
        tree.close()


def test_draft_masks_in_every_kernel_set():
    """Masks in the shared-prefix / suffix / merge kernels (kernel_mode 2) and in the tree-walk kernel
    with 8 wavefronts; only the kernel that splits the path (walk_waves 2) refuses them."""
    import paper_2605_10195_amd as spex
    wl = token_tree_workload(TOKEN_TREE_CASES[0])
    q = sw.gen_queries(wl, device="cuda")
    ref = run_oracle(wl)
    for kw in (dict(kernel_mode=2), dict(kernel_mode=2, prefix_chunk_pages=1, suffix_chunk_pages=1),
               dict(kernel_mode=3, walk_waves=8), dict(kernel_mode=0, walk_waves=8)):
        tree = build_gpu_tree(wl, **kw)
        got = run_gpu(wl, tree=tree)
        assert (tree.last_launch_info()["walk_row_tiles"] > 0) == (kw["kernel_mode"] == 3)
        tree.close()
        assert_close(got, ref, "bf16", f"{wl.name} {kw}")
    tree = build_gpu_tree(wl, kernel_mode=3, walk_waves=2)
    with pytest.raises(spex.SpexError) as e:
        tree.decode_attention(wl.leaves, wl.q_lens, q, wl.sm_scale, draft_masks=wl.draft_masks)
    assert e.value.name == "UNSUPPORTED"
    tree.close()


TOKEN_TREE_SHAPES = [
    sw.tot_with_drafts(n_queries=3, prompt=250, step=56, token_trees=True),                       # 6 drafts, G = 5
    sw.tot_with_drafts(n_queries=2, prompt=130, step=40, drafts=16, heads=(16, 4, 128), token_trees=True),
    sw.tot_with_drafts(n_queries=2, prompt=200, step=30, drafts=8, heads=(32, 4, 128), kv_dtype="bf16",
                       token_trees=True),
    sw.tot_with_drafts(n_queries=2, prompt=90, step=24, drafts=4, heads=(16, 2, 64), kv_dtype="bf16",
                       token_trees=True),
]


@pytest.mark.parametrize("wl", TOKEN_TREE_SHAPES, ids=lambda w: f"{w.name}_{w.kv_dtype}_{w.num_q_heads}_{w.q_lens[0]}")
@pytest.mark.parametrize("mode", [0, 1, 2, 3])
def test_token_tree_sizes_of_the_paper_match_oracle(wl, mode):
    # Sec. 6.5 verifies token trees of 16, 8 and 4 drafts per branch
    tree = build_gpu_tree(wl, kernel_mode=mode)
    got = run_gpu(wl, tree=tree)
    if mode != 0:
        assert (tree.last_launch_info()["walk_row_tiles"] > 0) == (mode == 3)
    tree.close()
    assert_close(got, run_oracle(wl), wl.kv_dtype, wl.name)


def test_decode_loop_with_draft_masks_patches_lengths():
    """Tokens appended in place shift the window of drafts; the cached lists (with their masks) are
    patched and every call matches the oracle on the grown tree."""
    wl = sw.bfs_tot(n_queries=2, prompt=48, step=20)
    wl.q_lens = [5] * len(wl.leaves)
    wl = sw.with_draft_trees(wl)
    tree = build_gpu_tree(wl, extra_pages=64, kernel_mode=3)
    from oracle.adapters import OracleSink, queries_fp64
    sink = OracleSink.for_workload(wl)
    sw.replay(wl, sink)
    q = sw.gen_queries(wl, device="cuda")
    qd = queries_fp64(q)
    states = set()
    for step in range(12):
        k = sw.normal_values(6, 1, 900 + step, torch.arange(len(wl.leaves)), 8, 128, 0.5, "cuda").to(torch.bfloat16)
        v = sw.normal_values(6, 2, 900 + step, torch.arange(len(wl.leaves)), 8, 128, 0.5, "cuda").to(torch.bfloat16)
        tree.append_tokens(wl.leaves, k, v)
        for i, leaf in enumerate(wl.leaves):
            sink.append(leaf, k[i:i + 1], v[i:i + 1])
        out, lse = tree.decode_attention(wl.leaves, wl.q_lens, q, wl.sm_scale, draft_masks=wl.draft_masks)
        states.add(tree.last_launch_info()["plan_rebuilt"])
        ref = sink.tree.attention(wl.leaves, wl.q_lens, qd, wl.sm_scale, draft_masks=wl.draft_masks)
        got = (out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64))
        assert_close(got, ref, "bf16", f"masked decode step {step}")
    assert states == {1, 2}
    tree.close()


# ------------------------------------------------------------------ cache quantised on append
@pytest.mark.parametrize("heads", [(10, 2, 128), (8, 8, 64), (4, 2, 96)])
def test_quantising_append_gives_the_oracle_codes_and_attention(heads):
    """spex_tree_append_tokens_quantize: bf16 tokens in, e4m3 codes in the pool.  The codes read
    back are the oracle's byte for byte (also where values saturate), then attention matches."""
    from oracle.adapters import OracleSink, queries_fp64
    wl = sw.random_trace(91, heads=heads, kv_dtype="fp8_e4m3", n_ops=40, max_tokens=50, max_q_len=2)
    _, _, alive = wl.node_tokens()
    leaves = sorted(set(u for u in wl.leaves))
    tree = build_gpu_tree(wl, extra_pages=4 * len(leaves) + 8)
    sink = OracleSink.for_workload(wl)
    sw.replay(wl, sink)
    grow = [u for u in leaves if tree.node_info(u)["n_live_children"] == 0]
    H, D = wl.num_kv_heads, wl.head_dim
    rng = np.random.default_rng(3)
    start = {u: tree.node_info(u)["n_tokens"] for u in grow}
    want_k = {u: [] for u in grow}
    want_v = {u: [] for u in grow}
    for step in range(37):                                     # crosses two page boundaries per node
        boost = 40.0 if step % 5 == 4 else 1.0                 # every fifth token overflows its page's scale
        k = (sw.normal_values(8, 1, 300 + step, torch.arange(len(grow)), H, D, 0.5, "cuda") * boost).to(torch.bfloat16)
        v = (sw.normal_values(8, 2, 300 + step, torch.arange(len(grow)), H, D, 0.5, "cuda") * boost).to(torch.bfloat16)
        if step == 7:
            k[0, 0, :4] = torch.tensor([0.0, -0.0, 3e-9, -3e-9], dtype=torch.bfloat16)
        ks = torch.from_numpy(rng.uniform(0.004, 0.02, size=(len(grow), H)).astype(np.float32)).cuda()
        vs = torch.from_numpy(rng.uniform(0.004, 0.02, size=(len(grow), H)).astype(np.float32)).cuda()
        new_page = [tree.node_info(u)["n_tokens"] % 16 == 0 for u in grow]
        tree.append_tokens(grow, k, v, ks, vs, quantize=True)
        for i, u in enumerate(grow):
            sink.append_quantised(u, k[i:i + 1], v[i:i + 1], ks[i:i + 1] if new_page[i] else None,
                                  vs[i:i + 1] if new_page[i] else None)
            want_k[u].append(sink.tree.last_codes[0])
            want_v[u].append(sink.tree.last_codes[1])
    saturated = 0
    for u in grow:
        kc, vc, _, _ = tree.gather_kv(u, start[u], 37)
        wk, wv = np.concatenate(want_k[u]), np.concatenate(want_v[u])
        assert np.array_equal(kc.cpu().view(torch.uint8).numpy(), wk), u
        assert np.array_equal(vc.cpu().view(torch.uint8).numpy(), wv), u
        saturated += int(((wk & 0x7F) == 0x7E).sum())
    assert saturated > 100
    q = sw.gen_queries(wl, device="cuda")
    out, lse = tree.decode_attention(wl.leaves, wl.q_lens, q, wl.sm_scale)
    ref = sink.tree.attention(wl.leaves, wl.q_lens, queries_fp64(q), wl.sm_scale)
    got = (out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64))
    # values up to 448 * 0.02 in V: the absolute bound scales with the value range (x 4)
    assert np.max(np.abs(got[0] - ref[0])) <= 8e-3 and np.max(np.abs(got[1] - ref[1])) <= 2e-3
    assert np.linalg.norm(got[0] - ref[0]) / np.linalg.norm(ref[0]) <= 1e-3
    tree.close()


def test_quantising_append_special_values_and_errors():
    import paper_2605_10195_amd as spex
    from oracle.tree_attention import decode_e4m3, encode_e4m3
    t = spex.SpexTree(8, 2, 64, 16, "bf16", "fp8_e4m3", num_pages=4, device="cuda")
    (r,) = t.fork(-1, 1)
    grid = decode_e4m3(np.arange(0x7F, dtype=np.uint8))
    mids = ((grid[:-1] + grid[1:]) / 2)[:126]                  # two heads x 64 dims hold 128 values
    vals = np.concatenate([mids[:62], [np.inf, -np.inf], mids[62:124], [1e30, -1e-30]]).astype(np.float32)
    x = torch.from_numpy(vals).to(torch.bfloat16).reshape(1, 2, 64).cuda()      # mid-points of small codes are exact in bf16
    one = torch.ones((1, 2), dtype=torch.float32, device="cuda")
    t.append_tokens([r], x, x.neg().contiguous(), one, one, quantize=True)
    kc, vc, ks, _ = t.gather_kv(r, 0, 1)
    xf = x.float().cpu().numpy().ravel()
    assert np.array_equal(kc.cpu().view(torch.uint8).numpy().ravel(), encode_e4m3(xf))
    assert np.array_equal(vc.cpu().view(torch.uint8).numpy().ravel(), encode_e4m3(-xf))
    assert torch.all(ks == 1)
    nan = torch.full((1, 2, 64), float("nan"), dtype=torch.bfloat16, device="cuda")
    t.append_tokens([r], nan, nan, None, None, quantize=True)                    # continues the page: no scales needed
    kc, _, _, _ = t.gather_kv(r, 1, 1)
    assert np.all(kc.cpu().view(torch.uint8).numpy() & 0x7F == 0x7F)
    t.close()
    b = spex.SpexTree(8, 2, 64, 16, "bf16", "bf16", num_pages=4, device="cuda")
    (r,) = b.fork(-1, 1)
    with pytest.raises(spex.SpexError) as e:
        b.append_tokens([r], x, x, one, one, quantize=True)
    assert e.value.name == "UNSUPPORTED" and b.node_info(r)["n_tokens"] == 0
    b.close()


# ------------------------------------------------------------------ a search that grows while it is served
@pytest.mark.parametrize("kv_dtype,heads", [("bf16", (8, 2, 128)), ("fp8_e4m3", (16, 4, 128)), ("bf16", (8, 8, 64))])
def test_dynamic_search_attention_matches_oracle_while_the_tree_changes(kv_dtype, heads):
    """REBASE widths, speculative children, prunes and early termination (the C-ABI scheduling
    primitives) reshape the tree every few iterations; the attention of sampled iterations is
    compared with the oracle driven by its own primitives through the same seeded search."""
    import paper_2605_10195_amd as spex
    from paper_2605_10195_amd import binding as B
    from oracle import scheduling as sch
    from oracle.adapters import OracleDynamicSink
    from spex_workloads.dynamic import DynamicConfig, DynamicShape, DynamicValues, LibrarySink, RebaseSpexDriver

    class LibSched:
        rebase_widths = staticmethod(B.spex_sched_rebase_widths)
        allocate_budget = staticmethod(B.spex_sched_allocate_budget)
        early_termination = staticmethod(B.spex_sched_early_termination)

    class OracleSched:
        rebase_widths = staticmethod(sch.rebase_widths)
        allocate_budget = staticmethod(sch.allocate_budget)
        early_termination = staticmethod(sch.early_termination)

    cfg = DynamicConfig(n_queries=4, prompt=(40, 150), budget=6, max_depth=4, step=(4, 30), k_total=10, seed=31)
    shape = DynamicShape(heads[0], heads[1], heads[2], 16, kv_dtype)
    every = 7
    ora = OracleDynamicSink(shape, DynamicValues(shape, cfg.seed, "cpu"), attend_every=every)
    ref_driver = RebaseSpexDriver(cfg, ora, OracleSched)
    ref_stats = ref_driver.run(400)
    tree = spex.SpexTree(heads[0], heads[1], heads[2], 16, "bf16", kv_dtype, num_pages=4000, device="cuda",
                         pool_fill=0xFF)

    class Checked(LibrarySink):
        checked = 0

        def attend(self, nodes, iteration):
            super().attend(nodes, iteration)
            if iteration in ora.results:
                ref_nodes, ref_out, ref_lse = ora.results[iteration]
                assert ref_nodes == list(nodes)
                _, _, out, lse = self.last
                got = (out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64))
                assert_close(got, (ref_out, ref_lse), kv_dtype, f"iteration {iteration}")
                Checked.checked += 1

    sink = Checked(tree, shape, DynamicValues(shape, cfg.seed, "cuda"), B.spex_tree_path_kv_bytes)
    driver = RebaseSpexDriver(cfg, sink, LibSched)
    stats = driver.run(400)
    assert stats == ref_stats and driver.decisions == ref_driver.decisions
    assert Checked.checked >= 5 and stats["spec_children"] > 0 and stats["prunes"] > 5
    assert sink.plan_states[1] > 0 and sink.plan_states[2] > 0       # fresh plans and patched plans both occurred
    assert tree.stats()[:2] == (0, 0)
    tree.close()


def test_draft_masks_edge_cases():
    """No prefix at all (T == q_len), drafts that straddle two nodes of which the first is shared,
    a single query with an empty mask, and an empty request list."""
    import paper_2605_10195_amd as spex
    wl = sw.Workload("mask_edges", 8, 2, 128, 16, "bf16", "bf16", 0.5, 81)
    b = sw.trees._Builder(wl)
    (r1,) = b.fork(-1, 1)
    b.append(r1, 5)
    b.request(r1, 5)                               # the whole path is drafts
    (r2,) = b.fork(-1, 1)
    b.append(r2, 19)
    c1, c2 = b.fork(r2, 2)
    b.append(c1, 4)
    b.append(c2, 2)
    b.request(c1, 7)                               # 3 drafts in the shared root (partial page), 4 in the child
    b.request(c2, 1)                               # mask 0: sees the 20 tokens before its own
    b.request(c2, 2)                               # the same node again, two drafts
    wl.draft_masks = [0b00001, 0b00011, 0b00101, 0b01001, 0b10101,
                      0b0000001, 0b0000011, 0b0000101, 0b0001011, 0b0010011, 0b0100101, 0b1001011,
                      0,
                      0b01, 0b10]
    ref = run_oracle(wl)
    for mode in (0, 1, 3):
        assert_close(run_gpu(wl, kernel_mode=mode), ref, "bf16", f"mask edges mode {mode}")
    tree = build_gpu_tree(wl)
    q = sw.gen_queries(wl, device="cuda")
    out, lse = tree.decode_attention([], [], q[:0].contiguous(), wl.sm_scale, draft_masks=[])
    assert out.shape[0] == 0
    with pytest.raises(spex.SpexError) as e:       # the first query of r1 would see nothing
        tree.decode_attention([r1], [5], q[:5].contiguous(), wl.sm_scale, draft_masks=[0, 1, 1, 1, 1])
    assert e.value.name == "EMPTY_PATH"
    tree.append_tokens([], None, None, quantize=False)      # nothing to do
    tree.close()


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8_e4m3"])
def test_causal_drafts_equal_single_queries_on_truncated_trees(kv_dtype):
    """Draft i of a q_len = 6 request sees exactly what a single query sees on the same tree cut
    off after draft i: both through the library, on two different trees."""
    def tree_with(n_drafts, q_len):
        wl = sw.Workload("drafts", 8, 2, 128, 16, "bf16", kv_dtype, 0.5, 83)
        b = sw.trees._Builder(wl)
        (root,) = b.fork(-1, 1)
        b.append(root, 70)
        a, c = b.fork(root, 2)
        b.append(a, 21, key=1)
        b.append(c, 33, key=2)
        b.append(a, n_drafts, key=3)            # the drafts start a token run of their own
        b.append(c, n_drafts, key=4)
        b.request(a, q_len, key=5)
        b.request(c, q_len, key=6)
        return wl
    full = tree_with(6, 6)
    out6, lse6 = run_gpu(full, kernel_mode=0)
    q6 = sw.gen_queries(full, device="cuda")
    for i in range(6):
        wl = tree_with(i + 1, 1)
        tree = build_gpu_tree(wl)
        q = torch.stack([q6[i], q6[6 + i]]).contiguous()        # the same query vectors
        out, lse = tree.decode_attention(wl.leaves, wl.q_lens, q, wl.sm_scale)
        torch.cuda.synchronize()
        got = out.cpu().numpy().astype(np.float64)
        want = np.stack([out6[i], out6[6 + i]])
        assert np.max(np.abs(got - want)) <= 2e-3, i
        assert np.max(np.abs(lse.cpu().numpy() - np.stack([lse6[i], lse6[6 + i]]))) <= 2e-3, i
        tree.close()
    assert_close((out6, lse6), run_oracle(full), kv_dtype, "six causal drafts")


def test_flat_copies_of_every_branch_agree_with_the_shared_tree():
    """Every requested branch stored privately (one root per branch holding a copy of its path's
    tokens) gives what the prefix-sharing tree gives."""
    shared = sw.bfs_tot(n_queries=2, prompt=70, step=27, width=8, keep=2, depth=3, heads=(8, 2, 128))
    tokens, parent, _ = shared.node_tokens()
    key_of = {}
    for op in shared.ops:
        if op.kind == "append":
            assert op.tok0 == 0                     # one append per node in this generator
            key_of[op.node] = op.key
    flat = sw.Workload("flat", 8, 2, 128, 16, "bf16", "bf16", 0.5, shared.seed)
    b = sw.trees._Builder(flat)
    for leaf, ql, qk in zip(shared.leaves, shared.q_lens, shared.q_keys):
        path = []
        u = leaf
        while u != -1:
            path.append(u)
            u = parent[u]
        (r,) = b.fork(-1, 1)
        for u in reversed(path):                    # the same token streams, laid end to end
            flat.ops.append(sw.TreeOp("append", r, tokens[u], key_of[u], 0))
            b.tokens[r] += tokens[u]
        b.request(r, ql, key=qk)
    assert flat.unique_kv_tokens() == shared.flat_kv_tokens() > 2 * shared.unique_kv_tokens()
    ref = run_oracle(shared)
    got_shared = run_gpu(shared)
    got_flat = run_gpu(flat)
    assert_close(got_shared, ref, "bf16", "shared")
    assert_close(got_flat, ref, "bf16", "flat")
    assert np.max(np.abs(got_shared[0] - got_flat[0])) <= 2e-3
    assert_close(run_oracle(flat), ref, "bf16", "oracle flat vs shared")     # 1e-12 in fact


@pytest.mark.parametrize("kv_dtype,heads", [("bf16", (8, 2, 128)), ("fp8_e4m3", (16, 4, 128))])
def test_mcts_search_attention_matches_oracle_while_the_tree_changes(kv_dtype, heads):
    """Depth-first search: UCB descents and Alg. 1 speculative expansions (C-ABI primitives) grow
    deep trees; sampled iterations are compared with the oracle driven by its own primitives."""
    import paper_2605_10195_amd as spex
    from paper_2605_10195_amd import binding as B
    from oracle import scheduling as sch
    from oracle.adapters import OracleDynamicSink
    from spex_workloads.dynamic import DynamicShape, DynamicValues, LibrarySink, MctsConfig, MctsSpexDriver

    class LibSched:
        allocate_budget = staticmethod(B.spex_sched_allocate_budget)
        early_termination = staticmethod(B.spex_sched_early_termination)
        ucb_select = staticmethod(B.spex_sched_ucb_select)
        dfs_speculate = staticmethod(B.spex_sched_dfs_speculate)
        make_tree = staticmethod(B.SearchTree)

    class OracleSched:
        allocate_budget = staticmethod(sch.allocate_budget)
        early_termination = staticmethod(sch.early_termination)
        ucb_select = staticmethod(sch.ucb_select)
        dfs_speculate = staticmethod(sch.dfs_speculate)
        make_tree = staticmethod(sch.SearchTree)

    cfg = MctsConfig(n_queries=3, prompt=(40, 150), branch=3, rollouts=14, c=0.6, step=(4, 30), k_total=8,
                     k_per_query=3, seed=37)
    shape = DynamicShape(heads[0], heads[1], heads[2], 16, kv_dtype)
    ora = OracleDynamicSink(shape, DynamicValues(shape, cfg.seed, "cpu"), attend_every=9)
    ref_driver = MctsSpexDriver(cfg, ora, OracleSched)
    ref_stats = ref_driver.run(600)
    tree = spex.SpexTree(heads[0], heads[1], heads[2], 16, "bf16", kv_dtype, num_pages=6000, device="cuda",
                         pool_fill=0xFF)
    checked = []

    class Checked(LibrarySink):
        def attend(self, nodes, iteration):
            super().attend(nodes, iteration)
            if iteration in ora.results:
                ref_nodes, ref_out, ref_lse = ora.results[iteration]
                assert ref_nodes == list(nodes)
                _, _, out, lse = self.last
                got = (out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64))
                assert_close(got, (ref_out, ref_lse), kv_dtype, f"iteration {iteration}")
                checked.append(iteration)

    sink = Checked(tree, shape, DynamicValues(shape, cfg.seed, "cuda"), B.spex_tree_path_kv_bytes)
    driver = MctsSpexDriver(cfg, sink, LibSched)
    stats = driver.run(600)
    assert stats == ref_stats and driver.decisions == ref_driver.decisions
    assert len(checked) >= 5 and stats["spec_expansions"] > 0 and stats["spec_hits"] > 0
    assert tree.stats()[:2] == (0, 0)
    tree.close()


@pytest.mark.parametrize("heads", [(10, 2, 128), (8, 8, 64), (4, 2, 96)])
def test_quantising_step_append_gives_the_oracle_codes_scales_and_attention(heads):
    """spex_tree_append_step_quantize: runs of bf16 tokens in, page scales and e4m3 codes made by
    the scatter kernel.  Codes and scales read back equal the oracle's bit for bit, for appends
    that start pages, continue partial ones, and span many pages in several launches."""
    import paper_2605_10195_amd as spex
    from oracle.adapters import OracleSink, queries_fp64
    Hq, Hkv, D = heads
    tree = spex.SpexTree(Hq, Hkv, D, 16, "bf16", "fp8_e4m3", num_pages=400, device="cuda", pool_fill=0xFF)
    sink = OracleSink(Hq, Hkv, D, "fp8_e4m3", 16)
    rng = np.random.default_rng(4)
    (r,) = tree.fork(-1, 1)
    sink.fork(-1, 1)
    want_k, want_v, want_ks = [], [], []
    lengths = [5, 30, 1, 16, 43, 11, 2200, 7]            # 2200 tokens: 138 pages, several scatter launches
    for i, n in enumerate(lengths):
        scale = [0.3, 2.0, 0.01, 1.0, 0.5, 40.0, 1.0, 1e-3][i]
        x = sw.normal_values(9, 1, 1000 + i, torch.arange(n), Hkv, D, 1.0, "cuda") * scale
        y = sw.normal_values(9, 2, 1000 + i, torch.arange(n), Hkv, D, 1.0, "cuda") * scale
        k, v = x.to(torch.bfloat16).contiguous(), y.to(torch.bfloat16).contiguous()
        tree.append_step(r, k, v, quantize=True)
        sink.append_quantised(0, k, v, derive_scales=True)
        want_k.append(sink.tree.last_codes[0])
        want_v.append(sink.tree.last_codes[1])
    total = sum(lengths)
    kc, vc, ks, vs = tree.gather_kv(r, 0, total)
    assert np.array_equal(kc.cpu().view(torch.uint8).numpy(), np.concatenate(want_k))
    assert np.array_equal(vc.cpu().view(torch.uint8).numpy(), np.concatenate(want_v))
    ref_ks = np.stack(sink.tree._scales[0][0]).astype(np.float32)            # [pages, Hkv]
    ref_vs = np.stack(sink.tree._scales[0][1]).astype(np.float32)
    assert np.array_equal(ks.cpu().numpy(), np.repeat(ref_ks, 16, axis=0)[:total])
    assert np.array_equal(vs.cpu().numpy(), np.repeat(ref_vs, 16, axis=0)[:total])
    # children forked below see it; decode tokens continue with the quantising token append
    a, b = tree.fork(r, 2)
    sink.fork(0, 2)
    for u in (a, b):
        x = (sw.normal_values(9, 1, 2000 + u, torch.arange(21), Hkv, D, 0.5, "cuda")).to(torch.bfloat16)
        tree.append_step(u, x.contiguous(), x.neg().contiguous(), quantize=True)
        sink.append_quantised(u, x, x.neg(), derive_scales=True)
    q = sw.normal_values(9, 3, 77, torch.arange(5), Hq, D, 0.5, "cuda").to(torch.bfloat16).contiguous()
    out, lse = tree.decode_attention([a, b], [2, 3], q, D ** -0.5)
    ref = sink.tree.attention([a, b], [2, 3], queries_fp64(q), D ** -0.5)
    got = (out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64))
    # the absolute bound is stated for |V| <= 2.45 (P is rounded to 11 bits): scale it with this test's values
    vmax = max(np.abs(sink.tree.materialise(u)[1]).max() for u in (a, b))
    assert np.max(np.abs(got[0] - ref[0])) <= 2e-3 * vmax / 2.45 and np.max(np.abs(got[1] - ref[1])) <= 2e-3
    assert np.linalg.norm(got[0] - ref[0]) / np.linalg.norm(ref[0]) <= 1e-3
    tree.close()
    bf = spex.SpexTree(8, 2, 64, 16, "bf16", "bf16", num_pages=4, device="cuda")
    (r,) = bf.fork(-1, 1)
    x = torch.zeros((3, 2, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(spex.SpexError) as e:
        bf.append_step(r, x, x, quantize=True)
    assert e.value.name == "UNSUPPORTED" and bf.node_info(r)["n_tokens"] == 0
    bf.close()


@pytest.mark.parametrize("shape", ["bfs", "drafts_fp8"])
def test_both_phase_orders_give_the_same_rows(shape):
    """Half of the tree-walk workgroups take their private blocks before the shared ones, by their
    place in the launch (places 16 .. 31 of every 32, flipped in every other round of 256).  A
    tree requested alone sits at places below 16 (shared blocks first); requested together with
    the others, some trees sit at places 16 and up.  Both must match the oracle, and each other up
    to the rounding of a different summation order -- bit for bit where the order is the same."""
    wl = sw.bfs_tot(n_queries=4, prompt=200, step=72) if shape == "bfs" else sw.tot_with_drafts(n_queries=4, prompt=250, step=56)
    tree = build_gpu_tree(wl, kernel_mode=3)
    q = sw.gen_queries(wl, device="cuda")
    out_a, lse_a = tree.decode_attention(wl.leaves, wl.q_lens, q, wl.sm_scale)
    assert tree.last_launch_info()["prefix_items"] >= 32          # places 16.. exist: both orders run
    ref = run_oracle(wl)
    assert_close((out_a.cpu().numpy().astype(np.float64), lse_a.cpu().numpy().astype(np.float64)), ref, wl.kv_dtype, "together")
    ref_tree = roots_of_requests(wl)
    lens = torch.tensor(wl.q_lens)
    starts = (torch.cumsum(lens, 0) - lens).tolist()
    same = different = 0
    for root in sorted(set(ref_tree)):
        idx = [i for i in range(len(wl.leaves)) if ref_tree[i] == root]
        rows = torch.cat([torch.arange(starts[i], starts[i] + wl.q_lens[i]) for i in idx]).cuda()
        out_b, lse_b = tree.decode_attention([wl.leaves[i] for i in idx], [wl.q_lens[i] for i in idx],
                                             q[rows].contiguous(), wl.sm_scale)
        assert tree.last_launch_info()["prefix_items"] <= 16
        assert float((out_a[rows] - out_b).abs().max()) < 1e-4 and float((lse_a[rows] - lse_b).abs().max()) < 1e-4
        if torch.equal(out_a[rows], out_b):
            same += 1
        else:
            different += 1
    tree.close()
    assert same >= 1 and different >= 1, (same, different)


def roots_of_requests(wl):
    """Root of every requested node of a workload (from its trace: node -> parent)."""
    _, parent, _ = wl.node_tokens()
    roots = []
    for u in wl.leaves:
        while parent[u] != -1:
            u = parent[u]
        roots.append(u)
    return roots

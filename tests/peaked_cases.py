"""Reduced workloads whose values are shaped so that the softmax is far from uniform (inputs only)."""

import spex_workloads as sw


def make_workload(shape):
    if shape == "bfs_bf16":
        return sw.bfs_tot(n_queries=3, prompt=300, step=70)                       # T = 650, G = 4
    if shape == "spec_bf16":
        return sw.spec_at_scale(n_queries=2, prompt=400, step=90, branches=20)    # 160 rows per kv head: two row blocks
    if shape == "mcts_bf16":
        return sw.mcts_skewed(n_queries=4, prompt=(100, 300), step=(20, 90), max_leaves=12)   # G = 7
    if shape == "drafts_fp8":
        return sw.tot_with_drafts(n_queries=3, prompt=200, step=48)               # q_len 6, G = 5, fp8
    raise KeyError(shape)


def shaped(shape, kind):
    """The workload `shape` with its values shaped as `kind` says."""
    wl = make_workload(shape)
    tokens, parent, _ = wl.node_tokens()
    P = sw.ValueProfile
    if kind == "rising":            # +0.088 nats per token: the reference moves about every 90 tokens
        wl.profile = P(q0=4.0, k_ramp=0.25)
    elif kind == "falling":         # the first block holds the maximum, later weights underflow
        wl.profile = P(q0=4.0, k_ramp=-0.25)
    elif kind == "negative":        # every score near -280
        wl.profile = P(q0=4.0, k_bias=-800.0)
    elif kind == "spike_root":      # one key 53 nats above the rest, in a block every row shares
        roots = [u for u in range(len(tokens)) if parent[u] == -1]
        wl.profile = P(q0=4.0, spikes={r: [(min(100, tokens[r] - 1), 150.0)] for r in roots})
    elif kind == "spike_mid":       # ... in the parent of every requested node
        mids = {parent[u] for u in wl.leaves if parent[u] != -1}
        wl.profile = P(q0=4.0, spikes={m: [(tokens[m] // 2, 150.0)] for m in mids if tokens[m] > 0})
    elif kind == "spike_last":      # ... in the last token a row sees before its own drafts
        wl.profile = P(q0=4.0, spikes={u: [(max(tokens[u] - ql, 0), 150.0)] for u, ql in zip(wl.leaves, wl.q_lens)})
    elif kind == "rising_spike":
        wl.profile = P(q0=4.0, k_ramp=0.25,
                       spikes={u: [(max(tokens[u] - ql, 0), -300.0)] for u, ql in zip(wl.leaves, wl.q_lens)})
    elif kind == "scale_x8":
        wl.sm_scale *= 8.0
    elif kind == "scale_div8":
        wl.sm_scale /= 8.0
    else:
        raise KeyError(kind)
    return wl

"""tt_tree_gdn_plan (host C++): run the chunk program on symbolic states (the state after token t is
called t) and check that every chunk enters with the state of its first token's predecessor."""
import numpy as np
import pytest

import paper_2511_00413_amd as T
import workloads as W
from oracle import meta as M


def _simulate(parent, seg):
    m = M.dfs_meta(parent, seg)
    plan = T.tree_gdn_plan(parent, seg)
    assert plan.n_chunks == sum(-(-int(s) // T.GDN_CHUNK) for s in seg)
    state = -1                       # symbolic: index of the token whose state is held on chip; -1 = zero
    slots = {}
    covered = []
    for c in range(plan.n_chunks):
        t0, n, src, dst = (int(x[c]) for x in (plan.chunk_tok0, plan.chunk_len, plan.chunk_src, plan.chunk_dst))
        assert 1 <= n <= T.GDN_CHUNK
        if src == -1:
            state = -1
        elif src >= 0:
            assert src in slots, "a slot is read before it was written"
            state = slots[src]
        assert state == m["tok_pred"][t0], f"chunk {c} enters with the wrong state"
        toks = list(range(t0, t0 + n))
        assert len(set(m["tok_node"][toks])) == 1, "a chunk crosses a node boundary"
        for t in toks[1:]:
            assert m["tok_pred"][t] == t - 1
        covered += toks
        state = toks[-1]
        if dst >= 0:
            assert 0 <= dst < plan.n_slots
            slots[dst] = state
    assert covered == list(range(m["n_tokens"]))
    _check_schedule(plan, m)
    return plan


def _check_schedule(plan, m):
    """tt_tree_gdn_schedule: segments = maximal runs that stay on chip, grouped into dependency levels.  Structure
    first, then the chunk program is run again level by level with the segments of a level taken in REVERSE order
    (any order inside a level must do): every chunk must still enter with its first token's predecessor state."""
    src, dst = plan.chunk_src, plan.chunk_dst
    c0, c1, lo = plan.seg_chunk0, plan.seg_chunk1, plan.level_off
    assert len(c0) == len(c1) == plan.n_segments and lo[0] == 0 and lo[-1] == plan.n_segments
    assert sorted((int(a), int(b)) for a, b in zip(c0, c1)) == [
        (a, b) for a, b in zip(sorted(int(x) for x in c0), sorted(int(x) for x in c1))]      # ranges pair up in order
    covered = sorted(c for a, b in zip(c0, c1) for c in range(a, b))
    assert covered == list(range(plan.n_chunks)), "segments must cover every chunk once"
    for a, b in zip(c0, c1):
        assert b > a and src[a] != -2 and all(src[c] == -2 for c in range(a + 1, b))
    level_of_seg = np.zeros(plan.n_segments, dtype=int)
    for l in range(plan.n_levels):
        assert lo[l + 1] > lo[l]
        level_of_seg[lo[l]:lo[l + 1]] = l
        order = [(-(int(c1[s_]) - int(c0[s_])), int(c0[s_])) for s_ in range(lo[l], lo[l + 1])]
        assert order == sorted(order), "inside a level: longest segment first, ties in chunk order"
    seg_of_chunk = {c: s for s, (a, b) in enumerate(zip(c0, c1)) for c in range(a, b)}
    saver = {int(dst[c]): c for c in range(plan.n_chunks) if dst[c] >= 0}
    for s_, a in enumerate(c0):
        if src[a] == -1:
            assert level_of_seg[s_] == 0
        else:
            assert level_of_seg[s_] == level_of_seg[seg_of_chunk[saver[int(src[a])]]] + 1
    # consumers of every slot, in chunk order
    for k in range(plan.n_slots):
        cons = list(plan.slot_cons[plan.slot_cons_off[k]:plan.slot_cons_off[k + 1]])
        want = [s_ for s_, a in sorted(enumerate(c0), key=lambda x: x[1]) if src[a] == k]
        assert cons == want, (k, cons, want)
    assert plan.slot_cons_off[-1] == len(plan.slot_cons) == sum(1 for a in c0 if src[a] >= 0)
    # level-by-level execution, reversed inside a level
    slots = {}
    for l in range(plan.n_levels):
        written = {}
        for s_ in reversed(range(lo[l], lo[l + 1])):
            state = None
            for c in range(c0[s_], c1[s_]):
                t0, n = int(plan.chunk_tok0[c]), int(plan.chunk_len[c])
                if src[c] == -1:
                    state = -1
                elif src[c] >= 0:
                    assert int(src[c]) in slots, "a slot is read in the level that writes it, or earlier"
                    state = slots[int(src[c])]
                assert state == m["tok_pred"][t0]
                state = t0 + n - 1
                if dst[c] >= 0:
                    written[int(dst[c])] = state
        slots.update(written)              # visible to later levels only


@pytest.mark.parametrize("seed", range(25))
def test_random_trees(seed):
    t = W.random_tree(860 + seed, n_nodes=2 + 3 * seed, lo=1, hi=200, n_roots=1 + seed % 3, p_zero=0.2)
    _simulate(list(t.parent), list(t.seg_len))


def test_shapes():
    plan = _simulate([-1, 0, 1], [64, 65, 1])                 # a chain: nothing is saved, everything continues
    assert plan.n_slots == 0 and plan.chunk_src.tolist() == [-1, -2, -2, -2] and plan.chunk_len.tolist() == [64, 64, 1, 1]
    plan = _simulate([-1, 0, 0, 0], [10, 5, 0, 7])           # two token-bearing children + an empty one
    assert plan.n_slots == 1 and plan.chunk_src.tolist() == [-1, 0, 0] and plan.chunk_dst.tolist() == [0, -1, -1]
    assert plan.n_segments == 3 and plan.level_off.tolist() == [0, 1, 3]     # both branches in one level
    plan = _simulate([-1, 0, 1, 1], [10, 0, 3, 4])           # children hang below a zero-length node
    assert plan.chunk_src.tolist() == [-1, 0, 0]
    plan = _simulate([-1, 0, 0], [10, 5, 0])                 # one token-bearing child: it continues on chip
    assert plan.n_slots == 0 and plan.chunk_src.tolist() == [-1, -2]
    for cfg in (2, 3, 4):
        t = W.tree_config(cfg)
        _simulate(list(t.parent), list(t.seg_len))
    assert T.tree_gdn_plan([], []).n_chunks == 0


def test_capture_nodes():
    """chunk_cap marks the chunk that ends with a capture node's last token (a zero-length node stands for its
    nearest token-bearing ancestor)."""
    parent, seg = [-1, 0, 0, 1, 1, 4], [70, 30, 40, 0, 64, 5]
    m = M.dfs_meta(parent, seg)
    rank = {int(i): rk for rk, i in enumerate(m["dfs_order"])}
    plan = T.tree_gdn_plan(parent, seg, capture_nodes=[4, 0, 3])        # node 3 is empty -> its parent, node 1
    assert plan.n_capture == 3
    ends = {k: int(plan.chunk_tok0[c] + plan.chunk_len[c] - 1) for c, k in enumerate(plan.chunk_cap) if k >= 0}
    assert ends == {0: m["node_end"][rank[4]] - 1, 1: m["node_end"][rank[0]] - 1, 2: m["node_end"][rank[1]] - 1}
    assert (plan.chunk_cap >= 0).sum() == 3
    with pytest.raises(T.TreeTrainError) as e:
        T.tree_gdn_plan(parent, seg, capture_nodes=[1, 3])                # both end in node 1's last chunk
    assert e.value.status == -2
    with pytest.raises(T.TreeTrainError) as e:
        T.tree_gdn_plan([-1, 0], [0, 5], capture_nodes=[0])               # nothing on or above it
    assert e.value.status == -2
    assert np.all(T.tree_gdn_plan(parent, seg).chunk_cap == -1)

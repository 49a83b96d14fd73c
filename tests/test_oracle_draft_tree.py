"""Pins for the oracle's tree drafting (CPU only).  The row forward is the one draft_step
uses (pinned in test_oracle_lmhead_draft.py against library routines); here the tree
bookkeeping is pinned: a path-shaped tree is the chain of draft steps, every root path of
a tree is independent of the other branches and of the node numbering, children carry
their parent's ranked tokens, the ranking is the library's stable sort."""
import numpy as np
import pytest

from oracle import specexit_oracle as O
from workloads import gen


def small(B=2, seed=0):
    shape = gen.scaled(gen.config(0), D=64, Hq=4, Hkv=2, d=16, I=96, V=211, B=B, ctx=(5, 12), k=5, n_q=10)
    w = gen.draft_weights(shape, seed, std=0.3)
    w.update(gen.perturbed_norm_vectors(shape, seed))
    L = gen.context_lengths(shape, seed)
    kv = gen.kv_cache(shape, L, 16, seed)
    tok0 = gen.token_ids(shape, B, seed)
    g0 = gen.hidden_rows(shape, B, seed)
    dims = O.DraftDims(shape.D, shape.Hq, shape.Hkv, shape.d, shape.V, shape.rms_eps, shape.rope_theta)
    return shape, dims, w, L, kv, tok0, g0


def run_tree(dims, w, kv, tok0, g0, L, parent, rank):
    kc, vc = kv.k.astype(np.float64), kv.v.astype(np.float64)
    out = O.draft_tree(dims, w, kc, vc, tok0, g0, L, parent, rank)
    return out, kc, vc


def test_ranking_is_the_stable_descending_sort():
    r = np.random.default_rng(0)
    z = r.integers(0, 6, size=40).astype(np.float64)          # many ties
    ref = np.argsort(-z, kind="stable")
    for b in (1, 2, 5, 40):
        np.testing.assert_array_equal(O.top_b_lowest(z, b), ref[:b])
    assert O.top_b_lowest(z, 1)[0] == O.argmax_lowest(z)
    big = r.standard_normal(10000)
    np.testing.assert_array_equal(O.top_b_lowest(big, 4), np.argsort(-big, kind="stable")[:4])


def test_depths():
    assert O.tree_depths([-1, 0, 0, 1, 3, 2]).tolist() == [0, 1, 1, 2, 3, 2]


def test_a_path_shaped_tree_is_the_chain_of_draft_steps():
    shape, dims, w, L, kv, tok0, g0 = small()
    n = 5
    parent = np.arange(-1, n - 1)
    out, kc, vc = run_tree(dims, w, kv, tok0, g0, L, parent, np.zeros(n, int))
    kc2, vc2 = kv.k.astype(np.float64), kv.v.astype(np.float64)
    tok, g = tok0, g0
    for j in range(n - 1):                                   # nodes 0..n-2 have a child
        st = O.draft_step(dims, w, kc2, vc2, tok, g, L + j)
        np.testing.assert_array_equal(out["block_tok"][:, j + 1], st["next_tok"])
        np.testing.assert_allclose(out["hidden_out"][:, j], st["hidden_out"], rtol=0, atol=1e-12)
        np.testing.assert_allclose(out["sig"][:, j], st["sig"], rtol=1e-12, atol=1e-12)
        tok, g = st["next_tok"], st["hidden_out"]
    assert np.isnan(out["hidden_out"][:, n - 1]).all()       # the leaf is not run
    np.testing.assert_allclose(kc, kc2, rtol=0, atol=1e-12)
    np.testing.assert_allclose(vc, vc2, rtol=0, atol=1e-12)


def test_children_hold_the_parents_ranked_tokens_and_sigs_follow_eqs():
    shape, dims, w, L, kv, tok0, g0 = small(seed=1)
    parent = np.array([-1, 0, 0, 0, 1, 1, 2, 4])
    rank = np.array([0, 0, 1, 2, 0, 1, 0, 0])
    out, _, _ = run_tree(dims, w, kv, tok0, g0, L, parent, rank)
    assert out["expanded"].tolist() == [True, True, True, False, True, False, False, False]
    for b in range(shape.B):
        for c in range(1, 8):
            order = np.argsort(-out["logits"][b, parent[c]], kind="stable")
            assert out["block_tok"][b, c] == order[rank[c]]
    e = out["expanded"]
    np.testing.assert_allclose(out["sig"][:, e, 0], 1 / (1 + np.exp(-out["sig_raw"][:, e, 0])), rtol=1e-12)
    np.testing.assert_allclose(out["sig"][:, e, 2], np.maximum(0, np.expm1(out["sig_raw"][:, e, 2])), rtol=1e-12)


@pytest.mark.parametrize("seed", [0, 1])
def test_every_root_path_is_independent_of_the_other_branches(seed):
    """Node c of the tree equals the last node of the path-shaped tree made of c's ancestors
    alone (same ranks): siblings' cache entries are invisible, the rotary position is the
    depth and not the node number, the hidden state comes from the parent."""
    shape, dims, w, L, kv, tok0, g0 = small(seed=seed)
    tree_shape = gen.scaled(shape, B=1, tree=True, n_q=10, k=4)
    parent = gen.random_tree_parents(tree_shape, seed)[0]
    rank = np.zeros(10, int)
    for p in range(10):
        for i, c in enumerate([c for c in range(1, 10) if parent[c] == p]):
            rank[c] = i
    out, _, _ = run_tree(dims, w, kv, tok0, g0, L, parent, rank)
    assert out["expanded"].sum() >= 3
    for c in range(1, 10):
        path = []
        a = c
        while a >= 0:
            path.append(a)
            a = parent[a]
        path = path[::-1]                                    # root .. c
        pp = np.arange(-1, len(path) - 1)
        pr = np.array([rank[a] for a in path])
        ext = np.concatenate([pp, [len(path) - 1]])          # one more node so that c is expanded
        sub, _, _ = run_tree(dims, w, kv, tok0, g0, L, ext, np.concatenate([pr, [0]]))
        np.testing.assert_array_equal(sub["block_tok"][:, :len(path)], out["block_tok"][:, path])
        if out["expanded"][c]:
            np.testing.assert_allclose(sub["hidden_out"][:, len(path) - 1], out["hidden_out"][:, c], rtol=0, atol=1e-11)
            np.testing.assert_allclose(sub["logits"][:, len(path) - 1], out["logits"][:, c], rtol=0, atol=1e-11)


def test_the_tree_block_in_the_cache_is_what_ancestor_masked_attention_reads():
    """Cross-check with the pinned verification attention: for an expanded node, attention
    of any query over the draft cache under the node's ancestor mask must not depend on the
    entries of non-ancestors; overwrite those with junk and the node's subtree is unchanged."""
    shape, dims, w, L, kv, tok0, g0 = small(seed=2)
    parent = np.array([-1, 0, 0, 1, 1, 2, 3])
    rank = np.array([0, 0, 1, 0, 1, 0, 0])
    out, kc, vc = run_tree(dims, w, kv, tok0, g0, L, parent, rank)
    # a second run over a cache whose tree-block entries start as junk: nothing may leak in
    kv2 = gen.kv_cache(shape, L, 16, 2)
    for b in range(shape.B):
        kv2.k[b, :, L[b]:] = 1e3
        kv2.v[b, :, L[b]:] = -1e3
    out2, _, _ = run_tree(dims, w, kv2, tok0, g0, L, parent, rank)
    np.testing.assert_array_equal(out2["block_tok"], out["block_tok"])
    e = out["expanded"]
    np.testing.assert_allclose(out2["hidden_out"][:, e], out["hidden_out"][:, e], rtol=0, atol=1e-11)


def test_hidden_states_are_handed_on_in_the_storage_type():
    shape, dims, w, L, kv, tok0, g0 = small(seed=3)
    parent = np.array([-1, 0, 1])
    rank = np.zeros(3, int)
    calls = []

    def store(a):
        calls.append(a.shape)
        return gen.round_to_bf16(np.asarray(a, np.float32))
    kc, vc = kv.k.astype(np.float64), kv.v.astype(np.float64)
    out = O.draft_tree(dims, w, kc, vc, tok0, g0, L, parent, rank, store=store)
    kc2, vc2 = kv.k.astype(np.float64), kv.v.astype(np.float64)
    s0 = O.draft_step(dims, w, kc2, vc2, tok0, g0, L, store=store)
    s1 = O.draft_step(dims, w, kc2, vc2, s0["next_tok"], store(s0["hidden_out"]), L + 1, store=store)
    np.testing.assert_allclose(out["hidden_out"][:, 1], s1["hidden_out"], rtol=0, atol=1e-12)
    assert (dims.D,) in calls

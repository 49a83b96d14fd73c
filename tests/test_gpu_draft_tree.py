"""GPU parity: tree drafting (specexit_draft_tree_level + specexit_tree_gather, level by level)
against the oracle's draft_tree: tokens of the whole block bit-exact (the top_b + 1 best
logits of every expanded node are forced more than 0.05 apart), hidden states, signals,
candidate logits and the cache entries written within the storage type's tolerance."""
import numpy as np
import pytest

from oracle import specexit_oracle as O
from workloads import gen

from harness import TOL, GpuDraft, force_tree_gap, rel_err

pytestmark = pytest.mark.gpu


def setup(shape, seed, paged=False, std=0.05):
    w = gen.draft_weights(shape, seed, std=std)
    w.update(gen.perturbed_norm_vectors(shape, seed))
    # token embeddings as large as the hidden states, so that sibling nodes (same parent state,
    # different token) do not end up with nearly the same output
    w["embed"] = gen.store(shape, w["embed"] * np.float32(1.0 / std))
    L = gen.context_lengths(shape, seed)
    kv = gen.kv_cache(shape, L, shape.n_q, seed, paged=paged)
    tok0 = gen.token_ids(shape, shape.B, seed)
    g0 = gen.hidden_rows(shape, shape.B, seed)
    return w, kv, tok0, g0, L


def check_tree(shape, w, kv, tok0, g0, L, parent, rank, top_b, label):
    print(f"draft tree {label}: dtype={shape.dtype} B={shape.B} n={len(parent)} D={shape.D} V={shape.V} "
          f"paged={kv.paged} parent={list(parent)}", flush=True)
    w, ref, kc, vc = force_tree_gap(shape, w, kv, tok0, g0, L, parent, rank, top_b)
    gd = GpuDraft(shape, w, kv)
    got = gd.tree(tok0, g0, L, parent, rank, top_b)
    tol = TOL[shape.dtype]
    np.testing.assert_array_equal(got["block_tok"], ref["block_tok"])
    gk, gv = gd.cache()
    for c in np.flatnonzero(ref["expanded"]):
        assert rel_err(got["hidden_out"][c], ref["hidden_out"][:, c]) < tol, f"hidden_out node {c}"
        assert rel_err(got["sig_raw"][c], ref["sig_raw"][:, c]) < tol
        assert rel_err(got["sig"][c][:, :2], ref["sig"][:, c, :2]) < tol
        assert rel_err(got["sig"][c][:, 2], ref["sig"][:, c, 2]) < tol
        for b in range(shape.B):
            order = O.top_b_lowest(ref["logits"][b, c], top_b)
            np.testing.assert_array_equal(got["cand_tok"][c][b], order)
            assert rel_err(got["cand_logit"][c][b], ref["logits"][b, c][order]) < tol
            p = int(L[b]) + int(c)
            if kv.paged:
                pg, sl = kv.page_table[b, p // kv.page_size], p % kv.page_size
                assert rel_err(gk[pg, :, sl], kc[pg, :, sl]) < tol and rel_err(gv[pg, :, sl], vc[pg, :, sl]) < tol
            else:
                assert rel_err(gk[b, :, p], kc[b, :, p]) < tol and rel_err(gv[b, :, p], vc[b, :, p]) < tol
    return ref, got


def test_tiny_fp32_tree():
    shape = gen.scaled(gen.config(0), B=2, tree=True, n_q=12, k=4, V=1024)
    parent, rank = gen.level_ordered_tree(shape, 0)
    w, kv, tok0, g0, L = setup(shape, 0)
    check_tree(shape, w, kv, tok0, g0, L, parent, rank, 3, "config 0")


@pytest.mark.parametrize("B,paged,seed", [(1, False, 1), (3, True, 2), (5, False, 3)])
def test_small_bf16_trees(B, paged, seed):
    shape = gen.scaled(gen.config(3), D=256, Hq=4, Hkv=2, d=128, I=512, V=3000, B=B, ctx=(0, 300), n_q=16, k=5)
    parent, rank = gen.level_ordered_tree(shape, seed)
    w, kv, tok0, g0, L = setup(shape, seed, paged=paged)
    L[0] = 0
    kv = gen.kv_cache(shape, L, shape.n_q, seed, paged=paged)
    check_tree(shape, w, kv, tok0, g0, L, parent, rank, 3, "small bf16")


def test_a_path_shaped_tree_matches_the_chain_entry_point():
    """W = 1, top_b = 1: the level call must reproduce specexit_draft_step step by step."""
    shape = gen.scaled(gen.config(1), D=256, Hq=4, Hkv=2, d=128, I=512, V=2000, B=2, ctx=(40, 200), n_q=5, k=4)
    parent, rank = np.arange(-1, 4, dtype=np.int32), np.zeros(5, np.int32)
    w, kv, tok0, g0, L = setup(shape, 4)
    ref, got = check_tree(shape, w, kv, tok0, g0, L, parent, rank, 1, "path")
    gd = GpuDraft(shape, force_tree_gap(shape, w, kv, tok0, g0, L, parent, rank, 1)[0], kv)
    tok, g = tok0, g0
    for j in range(4):
        st = gd.step(tok, g, L + j)
        np.testing.assert_array_equal(st["next_tok"], got["block_tok"][:, j + 1])
        np.testing.assert_array_equal(st["hidden_out"], got["hidden_out"][j])
        np.testing.assert_array_equal(st["sig"], got["sig"][j])
        tok, g = st["next_tok"], st["hidden_out"]


@pytest.mark.timeout(900)
def test_full_size_config_3_tree():
    # 16-node tree, depth 5, <= 3 children, 8192-token cache; one sequence keeps the oracle's
    # passes (8 full forwards each, in float64) to about a minute
    shape = gen.scaled(gen.config(3), B=1)
    parent, rank = gen.level_ordered_tree(shape, 0)
    w = gen.draft_weights(shape, 0)
    w["embed"] = gen.store(shape, w["embed"] * np.float32(32.0))     # see setup()
    L = gen.context_lengths(shape, 0)
    kv = gen.kv_cache(shape, L, shape.n_q, 0)
    tok0 = gen.token_ids(shape, shape.B, 0)
    g0 = gen.hidden_rows(shape, shape.B, 0)
    check_tree(shape, w, kv, tok0, g0, L, parent, rank, 3, "config 3 full size")


def test_rejected_arguments():
    shape = gen.scaled(gen.config(1), D=256, Hq=4, Hkv=2, d=128, I=512, V=2000, B=2, ctx=(10, 20), n_q=5, k=4)
    w, kv, tok0, g0, L = setup(shape, 5)
    gd = GpuDraft(shape, w, kv)
    lib = gd.lib
    assert lib.specexit_draft_tree_level_workspace_bytes(gd.desc, gd.view, 2, 40, 1) == 0      # 80 rows
    assert lib.specexit_draft_tree_level_workspace_bytes(gd.desc, gd.view, 2, 2, 5) == 0       # top_b too large
    assert lib.specexit_draft_tree_level_workspace_bytes(gd.desc, gd.view, 2, 2, 4) > 0

"""Pins for the oracle's cache compaction (CPU only).  Alg. 1 names the cache update that
ends a round without defining it; what it has to mean is fixed by what the next round computes:
attention over the compacted cache must equal attention over the old cache restricted to
the accepted path.  Further pins: position-coded caches read back as the accepted
sequence, chains are left untouched, paged and contiguous layouts agree, nothing outside
the moved entries changes."""
import numpy as np
import pytest

from oracle import specexit_oracle as O
from workloads import gen


def tree_case(index=0, B=3, seed=0, n_q=None):
    shape = gen.scaled(gen.config(index), B=B, tree=True, n_q=n_q or 12, k=5)
    parent = gen.random_tree_parents(shape, seed)
    case = gen.accept_case(shape, seed, parent=parent)
    ref = O.accept_exit(O.ExitCfg(stop_think_token=1), case.block_tok, parent, case.target_argmax,
                        np.zeros((B, 3)), np.full(B, 10, np.int32), case.split_tok,
                        np.zeros((B, 3)), np.zeros(B, np.int32), np.ones(B, np.int32))
    return shape, parent, ref


def test_position_coded_cache_reads_back_as_the_accepted_sequence():
    # every entry stores its own position: after compaction positions L .. L+len hold
    # L, L+path[0], L+path[1], ...
    B, Hkv, l_max, d = 2, 2, 40, 4
    k = np.broadcast_to(np.arange(l_max, dtype=np.float32)[None, None, :, None], (B, Hkv, l_max, d)).copy()
    v = -k
    ctx = np.array([10, 20], np.int32)
    path = np.array([[2, 5, 7, -1, -1, -1, -1, -1], [1, 2, -1, -1, -1, -1, -1, -1]], np.int32)
    ln = np.array([3, 2], np.int32)
    k2, v2 = O.kv_compact(k, v, ctx, path, ln)
    assert k2[0, 1, 10:14, 0].tolist() == [10, 12, 15, 17]
    assert k2[1, 0, 20:23, 3].tolist() == [20, 21, 22]
    np.testing.assert_array_equal(v2, -k2)
    # nothing but positions L+1 .. L+len was written
    untouched = np.ones((B, l_max), bool)
    untouched[0, 11:14] = False
    untouched[1, 21:23] = False
    for b in range(B):
        np.testing.assert_array_equal(k2[b][:, untouched[b]], k[b][:, untouched[b]])


def test_overlapping_moves_read_the_old_cache():
    # path (2, 3): entry L+2 is both a target (of node 3) and a source (node 2)
    k = np.arange(8, dtype=np.float32).reshape(1, 1, 8, 1).copy()
    k2, _ = O.kv_compact(k, k.copy(), np.array([1]), np.array([[2, 3, -1, -1]]), np.array([2]))
    assert k2[0, 0, :, 0].tolist() == [0, 1, 3, 4, 4, 5, 6, 7]


def test_a_chain_is_left_as_it_is():
    shape = gen.scaled(gen.config(0), B=3)
    L = gen.context_lengths(shape, 0)
    kv = gen.kv_cache(shape, L, shape.n_q, 0)
    for m in range(shape.n_q):
        path = np.full((3, shape.n_q), -1, np.int32)
        path[:, :m] = np.arange(1, m + 1)
        k2, v2 = O.kv_compact(kv.k, kv.v, L, path, np.full(3, m, np.int32))
        np.testing.assert_array_equal(k2, kv.k)
        np.testing.assert_array_equal(v2, kv.v)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_next_round_attention_sees_exactly_the_accepted_path(seed):
    shape, parent, acc = tree_case(seed=seed)
    B, n_q = shape.B, shape.n_q
    assert acc["accept_len"].max() >= 2
    L = gen.context_lengths(shape, seed)
    kv = gen.kv_cache(shape, L, n_q, seed)
    q = gen.queries(shape, seed)
    mask = gen.ancestor_masks(parent)
    old = O.verify_attn(q, kv.k, kv.v, L, mask, shape.d ** -0.5)
    k2, v2 = O.kv_compact(kv.k, kv.v, L, acc["accept_path"], acc["accept_len"])
    for b in range(B):
        m = int(acc["accept_len"][b])
        last = int(acc["last_node"][b])
        # the last accepted node's query, now looking at a plain cache of length L + 1 + m
        # (its own entry included, as its ancestor mask included it before)
        qb = q[b:b + 1, last:last + 1]
        new = O.verify_attn(qb, k2[b:b + 1], v2[b:b + 1], np.array([L[b] + m]), None, shape.d ** -0.5)
        np.testing.assert_allclose(new[0, 0], old[b, last], rtol=1e-12, atol=1e-12)


def test_paged_and_contiguous_layouts_agree():
    shape, parent, acc = tree_case(seed=3)
    L = gen.context_lengths(shape, 3)
    kv = gen.kv_cache(shape, L, shape.n_q, 3)
    pg = gen.to_paged(shape, kv, shape.n_q, 3)
    k2, v2 = O.kv_compact(kv.k, kv.v, L, acc["accept_path"], acc["accept_len"])
    pk2, pv2 = O.kv_compact(pg.k, pg.v, L, acc["accept_path"], acc["accept_len"], pg.page_table, pg.page_size)
    for b in range(shape.B):
        n = int(L[b]) + shape.n_q
        pos = np.arange(n)
        pages = pg.page_table[b, pos // pg.page_size]
        np.testing.assert_array_equal(np.transpose(pk2[pages, :, pos % pg.page_size, :], (1, 0, 2)), k2[b, :, :n])
        np.testing.assert_array_equal(np.transpose(pv2[pages, :, pos % pg.page_size, :], (1, 0, 2)), v2[b, :, :n])


def test_hidden_state_of_the_last_accepted_node_is_handed_on():
    shape, parent, acc = tree_case(seed=4)
    L = gen.context_lengths(shape, 4)
    kv = gen.kv_cache(shape, L, shape.n_q, 4)
    hid = gen.hidden_rows(shape, shape.B * shape.n_q, 4).reshape(shape.B, shape.n_q, shape.D)
    _, _, nxt = O.kv_compact(kv.k, kv.v, L, acc["accept_path"], acc["accept_len"], block_hidden=hid,
                             last_node=acc["last_node"])
    for b in range(shape.B):
        np.testing.assert_array_equal(nxt[b], hid[b, acc["last_node"][b]])
    # nothing accepted: the root's own state
    _, _, nxt = O.kv_compact(kv.k, kv.v, L, acc["accept_path"], np.zeros(shape.B, np.int32), block_hidden=hid,
                             last_node=np.zeros(shape.B, np.int32))
    np.testing.assert_array_equal(nxt, hid[:, 0])

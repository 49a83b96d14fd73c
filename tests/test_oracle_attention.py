"""Pins for the oracle's verification attention (CPU only).

The oracle walks an explicit list of visible keys with a two-pass softmax.  It is
pinned against (a) the library's dense masked attention on small shapes, (b)
closed-form special cases and (c) structural invariants of the block mask."""
import numpy as np
import pytest
import torch

from oracle import specexit_oracle as O
from workloads import gen


def small_shape(**kw):
    base = dict(B=2, Hq=4, Hkv=2, d=16, n_q=5, ctx=(3, 40), V=64, D=32, I=64)
    base.update(kw)
    return gen.scaled(gen.config(0), **base)


def make_case(shape, seed=0, tree=False):
    L = gen.context_lengths(shape, seed)
    kv = gen.kv_cache(shape, L, shape.n_q, seed, paged=False)
    q = gen.queries(shape, seed)
    if tree:
        par = gen.random_tree_parents(gen.scaled(shape, k=min(3, shape.n_q - 1)), seed)
        mask = gen.ancestor_masks(par)
    else:
        par, mask = None, None
    return L, kv, q, par, mask


def dense_reference(q, kv, L, mask, scale):
    """softmax(QK^T*scale + additive mask) V through torch's library attention."""
    B, n_q, Hq, d = q.shape
    out = np.zeros((B, n_q, Hq, d))
    for b in range(B):
        n = int(L[b]) + n_q
        allow = torch.zeros(n_q, n, dtype=torch.bool)
        allow[:, :int(L[b])] = True
        for i in range(n_q):
            row = int(mask[b, i]) if mask is not None else (1 << (i + 1)) - 1
            for j in range(n_q):
                if (row >> j) & 1:
                    allow[i, int(L[b]) + j] = True
        qq = torch.tensor(q[b], dtype=torch.float64).permute(1, 0, 2)[None]      # [1,Hq,n_q,d]
        kk = torch.tensor(kv.k[b, :, :n], dtype=torch.float64)[None]
        vv = torch.tensor(kv.v[b, :, :n], dtype=torch.float64)[None]
        o = torch.nn.functional.scaled_dot_product_attention(
            qq, kk, vv, attn_mask=allow, scale=scale, enable_gqa=True)
        out[b] = o[0].permute(1, 0, 2).numpy()
    return out


@pytest.mark.parametrize("tree", [False, True])
@pytest.mark.parametrize("seed", [0, 1])
def test_matches_library_dense_attention(tree, seed):
    shape = small_shape()
    L, kv, q, par, mask = make_case(shape, seed, tree)
    scale = 0.37
    got = O.verify_attn(q, kv.k, kv.v, L, mask, scale)
    ref = dense_reference(q, kv, L, mask, scale)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)


def test_default_scale_is_inverse_sqrt_head_dim():
    shape = small_shape()
    L, kv, q, _, _ = make_case(shape, 3)
    a = O.verify_attn(q, kv.k, kv.v, L)
    b = O.verify_attn(q, kv.k, kv.v, L, scale=shape.d ** -0.5)
    np.testing.assert_array_equal(a, b)


def test_softmax_rows_sum_to_one_and_shift_invariant():
    r = np.random.default_rng(0)
    for n in (1, 2, 17, 300):
        s = r.standard_normal(n) * 30
        p = O.softmax_two_pass(s)
        assert abs(p.sum() - 1.0) < 1e-12
        assert np.all(p >= 0)
        np.testing.assert_allclose(O.softmax_two_pass(s + 1234.5), p, atol=1e-12)
    # huge scores do not overflow
    p = O.softmax_two_pass(np.array([1e4, 1e4 - 1.0]))
    np.testing.assert_allclose(p, [1 / (1 + np.exp(-1)), np.exp(-1) / (1 + np.exp(-1))], atol=1e-12)


def test_equal_value_rows_give_that_row():
    shape = small_shape()
    L, kv, q, par, mask = make_case(shape, 4, tree=True)
    row = np.linspace(-1, 1, shape.d).astype(np.float32)
    kv.v[:] = row
    out = O.verify_attn(q, kv.k, kv.v, L, mask)
    np.testing.assert_allclose(out, np.broadcast_to(row, out.shape), atol=1e-12)


def test_zero_query_gives_mean_of_visible_values():
    shape = small_shape()
    L, kv, q, par, mask = make_case(shape, 5, tree=True)
    q[:] = 0
    out = O.verify_attn(q, kv.k, kv.v, L, mask)
    G = shape.G
    for b in range(shape.B):
        for i in range(shape.n_q):
            vis = O.visible_positions(int(L[b]), int(mask[b, i]), shape.n_q)
            for h in range(shape.Hq):
                np.testing.assert_allclose(out[b, i, h], kv.v[b, h // G, vis].astype(np.float64).mean(axis=0), atol=1e-12)


def test_empty_context_self_only_returns_own_value():
    shape = small_shape(ctx=(0, 0))
    L, kv, q, _, _ = make_case(shape, 6)
    self_only = np.array([[1 << i for i in range(shape.n_q)]] * shape.B, dtype=np.uint64)
    out = O.verify_attn(q, kv.k, kv.v, L, self_only)
    for i in range(shape.n_q):
        for h in range(shape.Hq):
            np.testing.assert_allclose(out[:, i, h], kv.v[:, h // shape.G, i], atol=1e-12)


def test_visible_set_is_context_plus_masked_block_entries():
    vis = O.visible_positions(7, 0b10101, 5)
    assert vis.tolist() == [0, 1, 2, 3, 4, 5, 6, 7, 9, 11]
    assert O.visible_positions(0, 0b1, 4).tolist() == [0]
    assert O.chain_mask(4).tolist() == [1, 3, 7, 15]


def test_mask_invariants_of_generated_trees():
    shape = gen.config(3)
    par = gen.random_tree_parents(shape, 0)
    m = gen.ancestor_masks(par)
    dep = gen.node_depths(par)
    assert dep.max(axis=1).tolist() == [shape.k] * shape.B
    for b in range(shape.B):
        assert int(m[b, 0]) == 1
        counts = np.bincount(par[b, 1:], minlength=shape.n_q)
        assert counts.max() <= 3
        for i in range(shape.n_q):
            assert (int(m[b, i]) >> i) & 1
            assert int(m[b, i]) < (1 << (i + 1))          # never sees later nodes
            if i:
                assert 0 <= par[b, i] < i
                assert int(m[b, i]) == int(m[b, par[b, i]]) | (1 << i)
                assert bin(int(m[b, i])).count("1") == dep[b, i] + 1
    chain = gen.ancestor_masks(gen.chain_parents(2, 6))
    assert chain[0].tolist() == O.chain_mask(6).tolist()


def test_path_shaped_tree_equals_chain():
    shape = small_shape()
    L, kv, q, _, _ = make_case(shape, 7)
    mask = gen.ancestor_masks(gen.chain_parents(shape.B, shape.n_q))
    a = O.verify_attn(q, kv.k, kv.v, L, mask)
    b = O.verify_attn(q, kv.k, kv.v, L, None)
    np.testing.assert_array_equal(a, b)


def test_non_ancestor_block_entries_do_not_matter():
    shape = small_shape(n_q=6)
    L, kv, q, par, mask = make_case(shape, 8, tree=True)
    base = O.verify_attn(q, kv.k, kv.v, L, mask)
    k2, v2 = kv.k.copy(), kv.v.copy()
    b, i = 1, 3
    for j in range(shape.n_q):
        if not (int(mask[b, i]) >> j) & 1:
            k2[b, :, int(L[b]) + j] += 5.0
            v2[b, :, int(L[b]) + j] -= 3.0
    pert = O.verify_attn(q, k2, v2, L, mask)
    np.testing.assert_array_equal(pert[b, i], base[b, i])
    changed = [j for j in range(shape.n_q) if j != i and
               int(mask[b, j]) & ~int(mask[b, i]) & ((1 << shape.n_q) - 1)]
    assert changed, "case must contain a query that does see a perturbed entry"
    assert any(not np.array_equal(pert[b, j], base[b, j]) for j in changed)


def test_context_keys_all_matter():
    """A key at any context position changes every query's output (no off-by-one at L)."""
    shape = small_shape(B=1, ctx=(9, 9))
    L, kv, q, _, _ = make_case(shape, 9)
    base = O.verify_attn(q, kv.k, kv.v, L)
    for pos in (0, 8):
        v2 = kv.v.copy()
        v2[0, :, pos] += 1.0
        assert np.all(np.abs(O.verify_attn(q, kv.k, v2, L) - base).max(axis=-1) > 0)
    # position L + n_q - 1 (last block entry) matters only to the last query of a chain
    v2 = kv.v.copy()
    v2[0, :, 9 + shape.n_q - 1] += 1.0
    diff = np.abs(O.verify_attn(q, kv.k, v2, L) - base).max(axis=(-1, -2))[0]
    assert np.all(diff[:-1] == 0) and diff[-1] > 0


def test_paged_layout_equals_contiguous():
    shape = small_shape(ctx=(5, 70))
    L, kv, q, par, mask = make_case(shape, 10, tree=True)
    paged = gen.to_paged(shape, kv, shape.n_q, seed=3)
    assert paged.paged and paged.page_table is not None
    # pages really are shuffled: not the identity layout
    assert not np.array_equal(np.sort(paged.page_table[0, :2]), paged.page_table[0, :2]) or \
        paged.page_table[0, 0] != 0
    a = O.verify_attn(q, kv.k, kv.v, L, mask)
    b = O.verify_attn(q, paged.k, paged.v, L, mask, page_table=paged.page_table,
                      page_size=paged.page_size)
    np.testing.assert_array_equal(a, b)


def test_single_query_is_plain_decode_attention():
    shape = small_shape(n_q=1, B=1, ctx=(33, 33))
    L, kv, q, _, _ = make_case(shape, 11)
    out = O.verify_attn(q, kv.k, kv.v, L)
    for h in range(shape.Hq):
        k = kv.k[0, h // shape.G, :34].astype(np.float64)
        v = kv.v[0, h // shape.G, :34].astype(np.float64)
        s = k @ q[0, 0, h].astype(np.float64) / np.sqrt(shape.d)
        p = np.exp(s - s.max())
        p /= p.sum()
        np.testing.assert_allclose(out[0, 0, h], p @ v, atol=1e-12)


def test_gqa_head_mapping():
    """Query heads of one group read the same KV head: identical queries give identical rows."""
    shape = small_shape(Hq=6, Hkv=2)
    L, kv, q, _, _ = make_case(shape, 12)
    q[:, :, 1] = q[:, :, 0]
    q[:, :, 2] = q[:, :, 0]
    q[:, :, 3] = q[:, :, 0]
    out = O.verify_attn(q, kv.k, kv.v, L)
    np.testing.assert_array_equal(out[:, :, 1], out[:, :, 0])
    np.testing.assert_array_equal(out[:, :, 2], out[:, :, 0])
    assert not np.array_equal(out[:, :, 3], out[:, :, 0])      # head 3 is in the second group


def test_only_selects_entries():
    shape = small_shape()
    L, kv, q, _, _ = make_case(shape, 13)
    full = O.verify_attn(q, kv.k, kv.v, L)
    part = O.verify_attn(q, kv.k, kv.v, L, only=[(1, 2, 3)])
    np.testing.assert_array_equal(part[1, 2, 3], full[1, 2, 3])
    assert np.isnan(part[0, 0, 0]).all()

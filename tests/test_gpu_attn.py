"""GPU parity: specexit_verify_attn against the oracle."""
import numpy as np
import pytest

from workloads import gen

from harness import TOL, gpu_verify_attn, oracle_verify_attn, rel_err

pytestmark = pytest.mark.gpu


def case(shape, seed, tree=False, paged=None):
    L = gen.context_lengths(shape, seed)
    kv = gen.kv_cache(shape, L, shape.n_q, seed, paged=paged)
    q = gen.queries(shape, seed)
    mask = None
    if tree:
        mask = gen.ancestor_masks(gen.random_tree_parents(shape, seed))
    return L, kv, q, mask


def check(shape, L, kv, q, mask, only=None, label=""):
    print(f"verify_attn {label}: dtype={shape.dtype} B={shape.B} n_q={shape.n_q} Hq={shape.Hq} Hkv={shape.Hkv} "
          f"d={shape.d} L={L.tolist()[:8]} paged={kv.paged} tree={mask is not None}", flush=True)
    got = gpu_verify_attn(shape, kv, q, L, mask)
    ref = oracle_verify_attn(kv, q, L, mask, only=only)
    if only is not None:
        sel = tuple(np.array(only).T)
        got, ref = got[sel], ref[sel]
    assert np.isfinite(got).all()
    err = rel_err(got, ref)
    assert err < TOL[shape.dtype], err
    return err


def test_tiny_fp32_config():
    shape = gen.config(0)
    L, kv, q, mask = case(shape, 0)
    check(shape, L, kv, q, mask, label="config 0")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("d", [64, 128])
def test_small_chain_ragged_lengths(dtype, d):
    shape = gen.scaled(gen.config(1), dtype=dtype, B=5, Hq=8, Hkv=2, d=d, n_q=7, ctx=(0, 700))
    L, kv, q, mask = case(shape, 1)
    L[0] = 0                       # empty context: only the block itself is visible
    L[1] = 121                     # not a multiple of any tile
    check(shape, L, kv, q, mask, label="chain ragged")


@pytest.mark.parametrize("paged", [False, True])
def test_small_tree(paged):
    shape = gen.scaled(gen.config(3), B=3, Hq=8, Hkv=2, ctx=(100, 900))
    L, kv, q, mask = case(shape, 2, tree=True, paged=paged)
    check(shape, L, kv, q, mask, label="tree")


@pytest.mark.parametrize("dtype,B,paged", [("bf16", 1024, False), ("bf16", 333, True), ("f32", 1024, False)])
def test_many_short_sequences(dtype, B, paged):
    # the most sequences a launch takes (the length table spans sixteen 64-lane rounds) and an odd
    # count: every workgroup's share of the keys crosses several (sequence, KV head) units, some empty
    shape = gen.scaled(gen.config(2), dtype=dtype, B=B, Hq=4, Hkv=2, n_q=2, ctx=(0, 150))
    L, kv, q, mask = case(shape, 7, paged=paged)
    L[0] = 0
    L[B - 1] = 150
    check(shape, L, kv, q, mask, label="many sequences")


def test_paged_equals_contiguous_on_gpu():
    shape = gen.scaled(gen.config(2), B=4, Hq=8, Hkv=2, ctx=(30, 1200))
    L, kv, q, mask = case(shape, 3, paged=False)
    paged = gen.to_paged(shape, kv, shape.n_q, seed=1)
    a = gpu_verify_attn(shape, kv, q, L, mask)
    b = gpu_verify_attn(shape, paged, q, L, mask)
    np.testing.assert_array_equal(a, b)
    check(shape, L, paged, q, mask, label="paged")


@pytest.mark.parametrize("n_q,Hq,Hkv", [(1, 8, 2), (64, 4, 2), (16, 16, 2), (9, 8, 1)])
def test_block_size_extremes(n_q, Hq, Hkv):
    shape = gen.scaled(gen.config(1), B=2, Hq=Hq, Hkv=Hkv, n_q=n_q, k=min(5, max(n_q - 1, 1)), ctx=(50, 400))
    L, kv, q, mask = case(shape, 4, tree=n_q > 1)
    check(shape, L, kv, q, mask, label="extremes")


def test_self_only_mask_with_empty_context_returns_own_value():
    shape = gen.scaled(gen.config(1), B=2, Hq=4, Hkv=2, n_q=5, ctx=(0, 0))
    L, kv, q, _ = case(shape, 5)
    mask = np.array([[1 << i for i in range(5)]] * 2, dtype=np.uint64)
    got = gpu_verify_attn(shape, kv, q, L, mask)
    for i in range(5):
        for h in range(4):
            np.testing.assert_allclose(got[:, i, h], kv.v[:, h // 2, i], atol=1e-2)


def sample_triples(shape, n, seed):
    r = np.random.default_rng(seed)
    return [(int(r.integers(shape.B)), int(r.integers(shape.n_q)), int(r.integers(shape.Hq))) for _ in range(n)]


def test_full_size_config_1():
    shape = gen.config(1)
    L, kv, q, mask = case(shape, 0)
    check(shape, L, kv, q, mask, label="config 1 full")


@pytest.mark.parametrize("index", [2, 3, 4])
def test_full_size_sampled(index):
    """Full shapes; a sample of (sequence, query, head) outputs against the oracle."""
    shape = gen.config(index)
    L, kv, q, mask = case(shape, 0, tree=shape.tree)
    only = sample_triples(shape, 48, index)
    only += [(int(np.argmax(L)), shape.n_q - 1, 0), (int(np.argmin(L)), 0, shape.Hq - 1)]
    check(shape, L, kv, q, mask, only=only, label=f"config {index} sampled")

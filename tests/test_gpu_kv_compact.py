"""GPU parity: specexit_kv_compact against the oracle, bit-exact on every cache entry (moved,
kept and dead ones alike: the call may write nothing but the moved rows) and on the hidden
rows handed to the next round."""
import numpy as np
import pytest
import torch

from oracle import specexit_oracle as O
from workloads import gen

from harness import dev, host, sx, tdtype

pytestmark = pytest.mark.gpu


def random_paths(B, n_q, seed, p_keep=0.5):
    """Strictly increasing node lists starting after the root: what acceptance can produce."""
    r = np.random.default_rng(seed)
    path = np.full((B, n_q), -1, np.int32)
    ln = np.zeros(B, np.int32)
    for b in range(B):
        nodes = [c for c in range(1, n_q) if r.random() < p_keep]
        path[b, :len(nodes)] = nodes
        ln[b] = len(nodes)
    last = np.array([path[b, ln[b] - 1] if ln[b] else 0 for b in range(B)], np.int32)
    return path, ln, last


def run_case(shape, kv, L, path, ln, last, n_layers=1, with_hidden=True, seed=0):
    lib = sx()
    B, n_q = shape.B, shape.n_q
    layers_k = [kv.k] + [np.ascontiguousarray(np.roll(kv.k, 3 * i + 1, axis=-1)) for i in range(1, n_layers)]
    layers_v = [kv.v] + [np.ascontiguousarray(np.roll(kv.v, 5 * i + 2, axis=-1)) for i in range(1, n_layers)]
    k_dev = torch.stack([dev(a, shape) for a in layers_k])
    v_dev = torch.stack([dev(a, shape) for a in layers_v])
    pt = dev(kv.page_table) if kv.paged else None
    view = lib.kv_view(k_dev[0], v_dev[0], pt)
    stride = k_dev[0].numel() * k_dev.element_size()
    hid = gen.hidden_rows(shape, B * n_q, seed).reshape(B, n_q, shape.D)
    hid_dev = dev(hid, shape)
    nxt = torch.full((B, shape.D), 7.0, dtype=tdtype(shape), device="cuda")
    i32 = lambda a: dev(np.asarray(a, np.int32))
    lib.specexit_kv_compact(view, n_layers, stride, B, n_q, i32(L), i32(path), i32(ln),
                            i32(last) if with_hidden else None, hid_dev if with_hidden else None,
                            shape.D if with_hidden else 0, nxt if with_hidden else None)
    torch.cuda.synchronize()
    for i in range(n_layers):
        rk, rv, rh = O.kv_compact(layers_k[i], layers_v[i], L, path, ln, kv.page_table if kv.paged else None,
                                  kv.page_size, block_hidden=hid, last_node=last)
        np.testing.assert_array_equal(host(k_dev[i]), rk, err_msg=f"K layer {i}")
        np.testing.assert_array_equal(host(v_dev[i]), rv, err_msg=f"V layer {i}")
    if with_hidden:
        np.testing.assert_array_equal(host(nxt), rh)
    else:
        assert float(nxt.float().min()) == 7.0


@pytest.mark.parametrize("index", [0, 1, 3])
def test_tree_paths_contiguous(index):
    base = gen.config(index)
    shape = gen.scaled(base, B=max(base.B, 3), tree=True, n_q=16, k=5)
    for seed in range(2):
        print(f"kv_compact contiguous config={index} seed={seed}", flush=True)
        L = gen.context_lengths(shape, seed)
        kv = gen.kv_cache(shape, L, shape.n_q, seed)
        path, ln, last = random_paths(shape.B, shape.n_q, seed)
        run_case(shape, kv, L, path, ln, last, seed=seed)


@pytest.mark.parametrize("index", [2, 4])
def test_tree_paths_paged_shuffled_pages(index):
    base = gen.config(index)
    shape = gen.scaled(base, B=4, tree=True, n_q=16, k=5, ctx=(1000, 3000))
    print(f"kv_compact paged config={index}", flush=True)
    L = gen.context_lengths(shape, 1)
    L[0] = 1024 - 3                      # the block straddles a page boundary
    kv = gen.kv_cache(shape, L, shape.n_q, 1)
    assert kv.paged
    path, ln, last = random_paths(shape.B, shape.n_q, 11)
    run_case(shape, kv, L, path, ln, last, seed=1)


def test_accepted_paths_of_generated_trees_at_full_size():
    shape = gen.config(3)                # B=4, 16-node trees, 8192-token contiguous caches
    parent = gen.random_tree_parents(shape, 0)
    case = gen.accept_case(shape, 0, parent=parent)
    B = shape.B
    acc = O.accept_exit(O.ExitCfg(stop_think_token=1), case.block_tok, parent, case.target_argmax,
                        np.zeros((B, 3)), np.zeros(B, np.int32), case.split_tok,
                        np.zeros((B, 3)), np.zeros(B, np.int32), np.ones(B, np.int32))
    assert acc["accept_len"].max() >= 2
    L = gen.context_lengths(shape, 0)
    kv = gen.kv_cache(shape, L, shape.n_q, 0)
    print("kv_compact generated trees config=3 full size", flush=True)
    run_case(shape, kv, L, acc["accept_path"], acc["accept_len"], acc["last_node"])


def test_every_layer_of_a_stacked_cache():
    shape = gen.scaled(gen.config(1), B=2, tree=True, n_q=12, k=5, ctx=(300, 700))
    L = gen.context_lengths(shape, 2)
    kv = gen.kv_cache(shape, L, shape.n_q, 2)
    path, ln, last = random_paths(shape.B, shape.n_q, 5)
    print("kv_compact 5 layers", flush=True)
    run_case(shape, kv, L, path, ln, last, n_layers=5)


def test_chains_and_empty_acceptance_move_nothing():
    shape = gen.scaled(gen.config(1), B=3, ctx=(100, 200))
    L = gen.context_lengths(shape, 3)
    kv = gen.kv_cache(shape, L, shape.n_q, 3)
    n_q = shape.n_q
    path = np.full((3, n_q), -1, np.int32)
    path[0, :n_q - 1] = np.arange(1, n_q)          # everything accepted
    path[1, :2] = [1, 2]
    ln = np.array([n_q - 1, 2, 0], np.int32)
    last = np.array([n_q - 1, 2, 0], np.int32)
    print("kv_compact chains", flush=True)
    run_case(shape, kv, L, path, ln, last)
    run_case(shape, kv, L, path, ln, last, with_hidden=False)


def test_largest_block_and_fp32_rows():
    for index, d in ((0, 64), (0, 128), (1, 64), (1, 128)):
        shape = gen.scaled(gen.config(index), B=2, tree=True, n_q=64, k=5, d=d, ctx=(50, 90))
        L = gen.context_lengths(shape, 4)
        kv = gen.kv_cache(shape, L, shape.n_q, 4)
        path, ln, last = random_paths(shape.B, shape.n_q, 6, p_keep=0.9)
        path[1, :63] = np.arange(1, 64)
        path[1, 10:62] = np.arange(12, 64)           # 62 nodes, all but ten of them moving
        ln[1], last[1] = 62, 63
        print(f"kv_compact n_q=64 dtype={shape.dtype} d={d}", flush=True)
        run_case(shape, kv, L, path, ln, last)


def test_rejected_arguments():
    lib = sx()
    shape = gen.scaled(gen.config(1), B=1, ctx=(20, 30))
    L = gen.context_lengths(shape, 0)
    kv = gen.kv_cache(shape, L, shape.n_q, 0)
    k, v = dev(kv.k, shape), dev(kv.v, shape)
    view = lib.kv_view(k, v, None)
    z = torch.zeros(64, dtype=torch.int32, device="cuda")
    with pytest.raises(RuntimeError):
        lib.specexit_kv_compact(view, 0, 0, 1, shape.n_q, z, z, z)
    with pytest.raises(RuntimeError):
        lib.specexit_kv_compact(view, 2, 8, 1, shape.n_q, z, z, z)
    with pytest.raises(RuntimeError):
        lib.specexit_kv_compact(view, 1, 0, 1, 65, z, z, z)
    with pytest.raises(RuntimeError):
        lib.specexit_kv_compact(view, 1, 0, 1, shape.n_q, z, z, z, None, k, shape.D, None)

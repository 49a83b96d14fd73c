"""GPU parity: specexit_lmhead_argmax against the oracle (argmax bit-exact, logits within tolerance)."""
import numpy as np
import pytest

from oracle import specexit_oracle as O
from workloads import gen

from harness import TOL, force_gap, gpu_lmhead, rel_err

pytestmark = pytest.mark.gpu


def run_case(shape, M, n_extra, seed, label):
    print(f"lmhead {label}: dtype={shape.dtype} M={M} D={shape.D} V={shape.V} n_extra={n_extra} seed={seed}", flush=True)
    hidden = gen.hidden_rows(shape, M, seed)
    w = gen.lm_head(shape, seed, n_extra=n_extra)
    V = shape.V
    tok_rows, am_ref, z_ref = force_gap(hidden, w[:V], V, 0.05, shape)
    w = np.concatenate([tok_rows, w[V:]], axis=0)
    _, z_ref, extra_ref = O.lmhead_argmax(hidden, w, n_extra)
    assert O.top2_gap(z_ref).min() > 0.05
    am, mx, extra, logits = gpu_lmhead(shape, hidden, w, n_extra)
    np.testing.assert_array_equal(am, am_ref)
    tol = TOL[shape.dtype]
    assert rel_err(logits, z_ref) < tol
    assert rel_err(mx, z_ref.max(axis=1)) < tol
    if n_extra:
        assert rel_err(extra, extra_ref) < tol
    # the call as the round makes it, without the debug logits (the kernels then take their
    # check-free epilogues where they can): token ids against the oracle again
    am2, mx2, extra2, _ = gpu_lmhead(shape, hidden, w, n_extra, want_logits=False)
    np.testing.assert_array_equal(am2, am_ref)
    assert rel_err(mx2, z_ref.max(axis=1)) < tol
    if n_extra:
        assert rel_err(extra2, extra_ref) < tol
    return rel_err(logits, z_ref)


def test_tiny_fp32_config():
    shape = gen.config(0)
    run_case(shape, shape.n_q, 0, 0, "config 0")
    run_case(shape, 1, 3, 1, "config 0 widened")
    run_case(gen.scaled(shape, V=4099, D=520), 11, 2, 2, "fp32 ragged")


@pytest.mark.parametrize("M", [1, 7, 16, 17, 56, 64, 65, 100, 144])
def test_bf16_mfma_ragged_vocab(M):
    # 5003 rows: 312 full 16-row tiles and a 11-row tail that also holds the signal rows;
    # D = 384 is an odd number of 128-wide k blocks (the kernels take them in pairs)
    shape = gen.scaled(gen.config(1), V=5000, D=384)
    err = run_case(shape, M, 3, M, "mfma")
    assert err < 1e-3          # bf16 inputs are exact; only fp32 summation order differs


@pytest.mark.parametrize("M,D", [(33, 128), (72, 128), (144, 512), (96, 1280)])
def test_bf16_mfma_many_rows_other_depths(M, D):
    # one block, an even count, and ten blocks: the staged-activation buffers of the many-row kernels
    shape = gen.scaled(gen.config(1), V=3001, D=D)
    err = run_case(shape, M, 1, M + D, "mfma many rows")
    assert err < 1e-3


def test_bf16_alu_fallback_when_k_is_not_a_multiple_of_128():
    shape = gen.scaled(gen.config(1), V=1000, D=200)
    run_case(shape, 3, 3, 0, "alu bf16")
    run_case(shape, 19, 0, 1, "alu bf16")


@pytest.mark.parametrize("M,V,rows", [(4, 4096, (77, 1300, 4000)),        # per-tile candidates of the kernel for few rows
                                      (40, 4096, (77, 1300, 4000)),       # many-row kernel: three workgroups' shares
                                      (40, 40000, (5, 140, 30000))])      # ... two halves of one share and a far one
def test_tie_takes_lowest_index_across_tiles(M, V, rows):
    shape = gen.scaled(gen.config(1), V=V, D=256)
    hidden = gen.hidden_rows(shape, M, 5)
    w = gen.lm_head(shape, 5)
    win = gen.store(shape, (hidden[2] / np.abs(hidden[2]).max()).astype(np.float32))
    for row in rows:                      # three identical winning rows in different tiles
        w[row] = win
    am_ref, z_ref, _ = O.lmhead_argmax(hidden, w)
    assert am_ref[2] == rows[0] and z_ref[2, rows[0]] == z_ref[2, rows[2]]
    am, _, _, logits = gpu_lmhead(shape, hidden, w)
    assert am[2] == rows[0] and logits[2, rows[0]] == logits[2, rows[1]] == logits[2, rows[2]]


@pytest.mark.parametrize("M", [16, 72, 144])
def test_repeated_calls_give_identical_bits(M):
    # fixed summation and merge orders: no atomics, no dependence on which workgroup finishes first
    shape = gen.scaled(gen.config(1), V=20000, D=512)
    hidden = gen.hidden_rows(shape, M, 11)
    w = gen.lm_head(shape, 11)
    first = gpu_lmhead(shape, hidden, w)
    for _ in range(3):
        again = gpu_lmhead(shape, hidden, w)
        np.testing.assert_array_equal(again[0], first[0])
        np.testing.assert_array_equal(again[1], first[1])
        np.testing.assert_array_equal(again[3], first[3])


def test_workspace_and_argument_errors():
    from harness import sx, dev, workspace
    import torch
    lib = sx()
    shape = gen.scaled(gen.config(1), V=512, D=256)
    h, w = dev(gen.hidden_rows(shape, 2, 0), shape), dev(gen.lm_head(shape, 0), shape)
    am = torch.empty(2, dtype=torch.int32, device="cuda")
    with pytest.raises(lib.SpecExitError) as e:
        lib.specexit_lmhead_argmax(lib.BF16, 2, 256, 512, 0, h, w, am, workspace=workspace(256))
    assert e.value.code == lib.EWORKSPACE
    with pytest.raises(lib.SpecExitError) as e:
        lib.specexit_lmhead_argmax(lib.BF16, 2, 256, 512, 0, h, None, am, workspace=workspace(1 << 20))
    assert e.value.code == lib.EINVAL


@pytest.mark.timeout(1200)
@pytest.mark.parametrize("index", [1, 2, 3, 4])
def test_full_size_configs(index):
    """Full vocabulary and hidden size of every bf16 configuration, M = B * n_q rows (7, 56, 64, 144:
    the last three run the kernel form for more than 32 rows); argmax bit-exact, every logit compared."""
    shape = gen.config(index)
    run_case(shape, shape.B * shape.n_q, 0, 0, f"config {index} full size")

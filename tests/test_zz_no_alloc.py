"""specexit_lmhead_argmax_noalloc (scratch in a buffer built into the library) against
specexit_lmhead_argmax (scratch in the caller's workspace): same bits, call after call, also when
the second call is smaller than the first and so leaves part of the shared scratch stale."""
import numpy as np
import pytest
import torch

from workloads import gen
import harness as H

pytestmark = pytest.mark.gpu


def both(shape, M, n_extra, seed):
    lib = H.sx()
    dt = lib.BF16 if shape.dtype == "bf16" else lib.F32
    V, D = shape.V, shape.D
    hid = H.dev(gen.hidden_rows(shape, M, seed), shape)
    w = H.dev(gen.lm_head(shape, seed, n_extra=n_extra), shape)
    i32 = lambda: torch.full((M,), -7, dtype=torch.int32, device="cuda")
    f32 = lambda *s: torch.full(s, -7.0, dtype=torch.float32, device="cuda")
    ref = dict(am=i32(), mx=f32(M), ex=f32(M, max(n_extra, 1)), lg=f32(M, V))
    got = dict(am=i32(), mx=f32(M), ex=f32(M, max(n_extra, 1)), lg=f32(M, V))
    ws = H.workspace(lib.specexit_lmhead_argmax_workspace_bytes(dt, M, D, V, n_extra))
    lib.specexit_lmhead_argmax(dt, M, D, V, n_extra, hid, w, ref["am"], ref["mx"], ref["ex"] if n_extra else None, ref["lg"], ws)
    lib.specexit_lmhead_argmax_noalloc(dt, M, D, V, n_extra, hid, w, got["am"], got["mx"], got["ex"] if n_extra else None, got["lg"])
    torch.cuda.synchronize()
    for k in ref:
        np.testing.assert_array_equal(H.host(got[k]), H.host(ref[k]), err_msg=f"M={M} V={V} D={D}: {k}")
    assert (H.host(got["am"]) >= 0).all()


def test_two_calls_in_a_row_second_one_smaller():
    big = gen.scaled(gen.config(1), V=40000, D=1024)
    small = gen.scaled(gen.config(1), V=3001, D=384)
    print("no-alloc LM head: M=96 V=40000, then M=5 V=3001", flush=True)
    both(big, 96, 3, 1)          # matrix-core path, many rows
    both(small, 5, 0, 2)         # smaller input: most of the shared scratch keeps the first call's candidates
    both(big, 17, 0, 3)
    tiny = gen.scaled(gen.config(0), V=2000, D=200)
    both(tiny, 3, 2, 4)          # fp32: the ALU path keeps whole logit rows in the scratch


def test_shapes_beyond_the_built_in_buffer_are_refused():
    lib = H.sx()
    shape = gen.config(0)
    M, V, D = 144, 151936, 512           # fp32 ALU path: M * V * 4 bytes of logits, far beyond 12 MiB
    assert lib.specexit_lmhead_argmax_workspace_bytes(lib.F32, M, D, V, 0) > lib.NOALLOC_SCRATCH_BYTES
    hid = torch.zeros((M, D), dtype=torch.float32, device="cuda")
    w = torch.zeros((8, D), dtype=torch.float32, device="cuda")       # never read: the call is refused on the host
    am = torch.zeros(M, dtype=torch.int32, device="cuda")
    with pytest.raises(lib.SpecExitError) as e:
        lib.specexit_lmhead_argmax_noalloc(lib.F32, M, D, V, 0, hid, w, am)
    assert e.value.code == lib.EWORKSPACE and "built-in buffer holds" in str(e.value)
    with pytest.raises(lib.SpecExitError) as e:
        lib.specexit_lmhead_argmax_noalloc(lib.BF16, 500, 512, 4096, 0, hid, w, am)
    assert e.value.code == lib.EINVAL

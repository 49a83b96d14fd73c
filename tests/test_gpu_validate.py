"""Out-of-range device data: page ids, token ids and lengths are forced into range by the kernels
(nothing faults, every kernel ends normally), and with SPECEXIT_FLAG_VALIDATE the first problem is
reported in the caller's device status word.  Sequences whose data is sound still match the oracle."""
import numpy as np
import pytest
import torch

from workloads import gen
import harness as H

pytestmark = pytest.mark.gpu


def status_word():
    return torch.zeros(1, dtype=torch.int32, device="cuda")


def test_bad_page_id_and_length_in_verify_attn_are_reported_and_contained():
    lib = H.sx()
    shape = gen.scaled(gen.config(2), B=3, Hq=8, Hkv=2, ctx=(200, 900))
    L = gen.context_lengths(shape, 3)
    kv = gen.kv_cache(shape, L, shape.n_q, 3, paged=True)
    q = gen.queries(shape, 3)
    ref = H.oracle_verify_attn(kv, q, L, None)
    view, keep = H.kv_view_of(shape, kv)
    qd = H.dev(q, shape)
    ws = H.workspace(lib.specexit_verify_attn_workspace_bytes(view, shape.B, shape.n_q, shape.Hq))
    word = status_word()
    lib.specexit_set_dev_status(word)
    try:
        def run(table, lengths):
            keep[2].copy_(H.dev(table))
            out = torch.zeros_like(qd)
            lib.specexit_verify_attn(view, shape.B, shape.n_q, shape.Hq, qd, H.dev(lengths.astype(np.int32)), None,
                                     shape.d ** -0.5, out, ws, flags=lib.FLAG_VALIDATE)
            torch.cuda.synchronize()
            code = int(word.item())
            word.zero_()
            return H.host(out), code
        out, code = run(kv.page_table, L)
        assert code == lib.STATUS_OK and H.rel_err(out, ref) < H.TOL[shape.dtype]
        # one page id far outside the pool, one negative, in sequence 1
        bad = kv.page_table.copy()
        bad[1, 2], bad[1, 5] = 1 << 30, -7
        print("verify_attn with two bad page ids", flush=True)
        out, code = run(bad, L)
        assert code == lib.STATUS_BAD_PAGE
        assert np.isfinite(out).all()
        assert H.rel_err(out[[0, 2]], ref[[0, 2]]) < H.TOL[shape.dtype]      # the other sequences are untouched
        # a length beyond the cache capacity and a negative one
        badL = L.copy()
        badL[0], badL[2] = 10_000_000, -5
        print("verify_attn with two bad lengths", flush=True)
        out, code = run(kv.page_table, badL)
        assert code == lib.STATUS_BAD_LENGTH
        assert np.isfinite(out).all()
        assert H.rel_err(out[1], ref[1]) < H.TOL[shape.dtype]
        # without the flag nothing is reported, and nothing faults either
        keep[2].copy_(H.dev(bad))
        out2 = torch.zeros_like(qd)
        lib.specexit_verify_attn(view, shape.B, shape.n_q, shape.Hq, qd, H.dev(badL.astype(np.int32)), None,
                                 shape.d ** -0.5, out2, ws)
        torch.cuda.synchronize()
        assert int(word.item()) == lib.STATUS_OK and torch.isfinite(out2.float()).all()
    finally:
        lib.specexit_set_dev_status(None)


@pytest.mark.parametrize("B", [2, 6])
def test_bad_token_id_and_page_id_in_draft_step_are_reported_and_contained(B):
    """B = 2 takes the row-streaming projections, B = 6 the matrix-core ones."""
    lib = H.sx()
    shape = gen.scaled(gen.config(2), D=512, Hq=8, Hkv=2, d=128, I=1024, V=5000, B=B, ctx=(10, 400), k=2)
    w = gen.draft_weights(shape, 5, std=0.05)
    pos = gen.context_lengths(shape, 5)
    kv = gen.kv_cache(shape, pos, shape.k + 1, 5, paged=True)
    tok, g = gen.token_ids(shape, B, 5), gen.hidden_rows(shape, B, 5)
    gd = H.GpuDraft(shape, w, kv)
    good = gd.step(tok, g, pos)
    word = status_word()
    lib.specexit_set_dev_status(word)
    try:
        bad_tok = tok.copy()
        bad_tok[1] = shape.V + 12345
        print(f"draft_step B={B} with a bad token id", flush=True)
        out = gd.step(bad_tok, g, pos, flags=lib.FLAG_VALIDATE)
        assert int(word.item()) == lib.STATUS_BAD_TOKEN
        word.zero_()
        assert np.isfinite(out["hidden_out"]).all()
        np.testing.assert_array_equal(out["hidden_out"][0], good["hidden_out"][0])     # row 0 is sound
        bad_table = kv.page_table.copy()
        bad_table[1, int(pos[1]) // kv.page_size] = -3          # the page the new entry of sequence 1 goes to
        gd.keep[2].copy_(H.dev(bad_table))
        print(f"draft_step B={B} with a bad page id", flush=True)
        out = gd.step(tok, g, pos, flags=lib.FLAG_VALIDATE)
        assert int(word.item()) == lib.STATUS_BAD_PAGE
        assert np.isfinite(out["hidden_out"]).all()
        np.testing.assert_array_equal(out["next_tok"][0], good["next_tok"][0])
    finally:
        lib.specexit_set_dev_status(None)

"""GPU parity: specexit_draft_step against the oracle."""
import numpy as np
import pytest

from oracle import specexit_oracle as O
from workloads import gen

from harness import TOL, GpuDraft, force_draft_gap, oracle_dims, oracle_draft_rows, rel_err

pytestmark = pytest.mark.gpu


def setup(shape, seed, paged=False, norms=True, std=0.02):
    w = gen.draft_weights(shape, seed, std=std)
    if norms:
        w.update(gen.perturbed_norm_vectors(shape, seed))
    pos = gen.context_lengths(shape, seed)
    kv = gen.kv_cache(shape, pos, shape.k + 1, seed, paged=paged)
    tok = gen.token_ids(shape, shape.B, seed)
    g = gen.hidden_rows(shape, shape.B, seed)
    return w, kv, tok, g, pos


def one_step(shape, w, kv, tok, g, pos, gd=None, label=""):
    print(f"draft_step {label}: dtype={shape.dtype} B={shape.B} D={shape.D} I={shape.I} V={shape.V} "
          f"pos={pos.tolist()[:8]} paged={kv.paged}", flush=True)
    kc, vc = kv.k.astype(np.float64), kv.v.astype(np.float64)
    ref = O.draft_step(oracle_dims(shape), w, kc, vc, tok, g, pos, kv.page_table if kv.paged else None,
                       kv.page_size, store=lambda a: gen.store(shape, a.astype(np.float32)))
    assert O.top2_gap(ref["logits"]).min() > 0.05
    gd = gd or GpuDraft(shape, w, kv)
    got = gd.step(tok, g, pos)
    tol = TOL[shape.dtype]
    np.testing.assert_array_equal(got["next_tok"], ref["next_tok"])
    assert rel_err(got["hidden_out"], ref["hidden_out"]) < tol
    assert rel_err(got["sig_raw"], ref["sig_raw"]) < tol
    assert rel_err(got["sig"][:, :2], ref["sig"][:, :2]) < tol
    assert rel_err(got["sig"][:, 2], ref["sig"][:, 2]) < tol
    # the cache entry written at pos
    gk, gv = gd.cache()
    for b in range(shape.B):
        p = int(pos[b])
        if kv.paged:
            pg, sl = kv.page_table[b, p // kv.page_size], p % kv.page_size
            assert rel_err(gk[pg, :, sl], kc[pg, :, sl]) < tol and rel_err(gv[pg, :, sl], vc[pg, :, sl]) < tol
        else:
            assert rel_err(gk[b, :, p], kc[b, :, p]) < tol and rel_err(gv[b, :, p], vc[b, :, p]) < tol
    return ref, got, gd, (kc, vc)


def test_tiny_fp32_config_chain_of_steps():
    shape = gen.config(0)
    w, kv, tok, g, pos = setup(shape, 0)
    gd = None
    for step in range(shape.k):
        w2 = force_draft_gap(shape, w, kv, tok, g, pos)
        if gd is None or not np.array_equal(w2["w_head"], w["w_head"]):
            gd = None                      # weights changed: rebuild the device copy (cache contents carry over)
        w = w2
        ref, got, gd, (kc, vc) = one_step(shape, w, kv, tok, g, pos, gd, label=f"config 0 step {step}")
        kv.k[:], kv.v[:] = kc, vc           # oracle's cache after the step feeds the next one
        tok = ref["next_tok"].astype(np.int32)
        g = ref["hidden_out"].astype(np.float32)
        pos = pos + 1
        gd = None


@pytest.mark.parametrize("B,paged", [(1, False), (3, True), (9, False), (16, True)])
def test_small_bf16_mfma(B, paged):
    shape = gen.scaled(gen.config(2), D=256, Hq=4, Hkv=2, d=64, I=512, V=3000, B=B, ctx=(0, 300), k=2)
    w, kv, tok, g, pos = setup(shape, B, paged=paged, std=0.05)
    pos[0] = 0
    w = force_draft_gap(shape, w, kv, tok, g, pos)
    one_step(shape, w, kv, tok, g, pos, label="small mfma")


def test_small_bf16_alu_fallback():
    shape = gen.scaled(gen.config(1), D=192, Hq=4, Hkv=2, d=64, I=320, V=1000, B=2, ctx=(5, 90), k=2)
    w, kv, tok, g, pos = setup(shape, 1, std=0.05)
    w = force_draft_gap(shape, w, kv, tok, g, pos)
    one_step(shape, w, kv, tok, g, pos, label="small alu bf16")


def test_rem_activation_variants():
    shape = gen.scaled(gen.config(0), V=512)
    w, kv, tok, g, pos = setup(shape, 2)
    w = force_draft_gap(shape, w, kv, tok, g, pos)
    raw = GpuDraft(shape, w, kv, rem_activation=2).step(tok, g, pos)
    sg = GpuDraft(shape, w, kv, rem_activation=1).step(tok, g, pos)
    np.testing.assert_allclose(raw["sig"][:, 2], raw["sig_raw"][:, 2], rtol=1e-6)
    np.testing.assert_allclose(sg["sig"][:, 2], 1 / (1 + np.exp(-sg["sig_raw"][:, 2].astype(np.float64))), rtol=1e-5)


def test_full_size_config_1():
    shape = gen.config(1)
    w, kv, tok, g, pos = setup(shape, 0, norms=False)
    w = force_draft_gap(shape, w, kv, tok, g, pos)
    ref, got, gd, _ = one_step(shape, w, kv, tok, g, pos, label="config 1 full size")
    # the launch configuration bench.py times: workspace zero-filled once, flag set; same bits,
    # call after call
    prep = GpuDraft(shape, w, kv)
    prep.lib.specexit_workspace_prepare(prep.ws)
    for it in range(6):
        out = prep.step(tok, g, pos, flags=prep.lib.FLAG_WORKSPACE_PREPARED)
        for k in out:
            np.testing.assert_array_equal(out[k], got[k], err_msg=f"prepared call {it}: {k}")


def sampled_rows_step(shape, w, kv, tok, g, pos, rows, label):
    """The step runs over all B rows on the GPU; the oracle computes the sampled rows (rows of a step are
    independent of one another) and those are compared: token bit-exact, floats within tolerance."""
    print(f"draft_step {label}: dtype={shape.dtype} B={shape.B} D={shape.D} I={shape.I} V={shape.V} "
          f"pos={pos.tolist()} paged={kv.paged} oracle rows={rows}", flush=True)
    gd = GpuDraft(shape, w, kv)                       # device copies are taken before the oracle writes its entries
    got = gd.step(tok, g, pos)
    gk, gv = gd.cache()
    ref = oracle_draft_rows(shape, w, kv, tok, g, pos, rows, progress=label)
    tol = TOL[shape.dtype]
    for b in rows:
        r = ref[b]
        assert O.top2_gap(r["logits"][None, :])[0] > 0.05
        assert got["next_tok"][b] == O.argmax_lowest(r["logits"]), f"row {b}"
        assert rel_err(got["hidden_out"][b], r["hidden_out"]) < tol, f"row {b}"
        assert rel_err(got["sig_raw"][b], r["sig_raw"]) < tol, f"row {b}"
        assert rel_err(got["sig"][b], O.signal_activations(r["sig_raw"][None, :])[0]) < tol, f"row {b}"
        p = int(pos[b])
        if kv.paged:
            pg, sl = kv.page_table[b, p // kv.page_size], p % kv.page_size
            assert rel_err(gk[pg, :, sl], kv.k[pg, :, sl]) < tol and rel_err(gv[pg, :, sl], kv.v[pg, :, sl]) < tol
        else:
            assert rel_err(gk[b, :, p], kv.k[b, :, p]) < tol and rel_err(gv[b, :, p], kv.v[b, :, p]) < tol
    assert np.isfinite(got["hidden_out"]).all() and (got["next_tok"] >= 0).all() and (got["next_tok"] < shape.V).all()


@pytest.mark.timeout(1500)
def test_full_size_config_2_all_eight_rows():
    """Qwen3-8B-like sizes, B = 8, paged cache: the split-K matrix-core projections with their reducing
    epilogues at full width (steps of up to four rows take the row-streaming path); every row compared."""
    shape = gen.config(2)
    w, kv, tok, g, pos = setup(shape, 0, paged=True, norms=False)
    rows = list(range(shape.B))
    w = force_draft_gap(shape, w, kv, tok, g, pos, rows=rows)
    sampled_rows_step(shape, w, kv, tok, g, pos, rows, "config 2 full size")


@pytest.mark.timeout(1500)
def test_full_size_config_4_sixteen_rows():
    """32B-like sizes (D = 5120, I = 25600, 64 query heads, paged caches of 8k-32k entries), B = 16 rows in
    the launch shapes bench.py times; the oracle checks the longest and the shortest sequence's rows and one more."""
    shape = gen.config(4)
    w, kv, tok, g, pos = setup(shape, 0, paged=True, norms=False)
    rows = sorted({int(np.argmax(pos)), int(np.argmin(pos)), 7})
    w = force_draft_gap(shape, w, kv, tok, g, pos, rows=rows)
    sampled_rows_step(shape, w, kv, tok, g, pos, rows, "config 4 full size")


def test_prepared_workspace_flag_gives_the_same_results_call_after_call():
    """With the workspace zero-filled once and the flag set, the call skips clearing its
    arrival counters; every kernel must leave them at zero for the next call."""
    shape = gen.scaled(gen.config(2), D=512, Hq=8, Hkv=2, d=128, I=1024, V=5000, B=3, ctx=(10, 400), k=2)
    w, kv, tok, g, pos = setup(shape, 7, std=0.05)
    w = force_draft_gap(shape, w, kv, tok, g, pos)
    plain = GpuDraft(shape, w, kv)
    prep = GpuDraft(shape, w, kv)
    prep.ws.fill_(0x5A)                                   # garbage first: prepare must clear it
    prep.lib.specexit_workspace_prepare(prep.ws)
    for it in range(12):
        a = plain.step(tok, g, pos + it % 3)
        b = prep.step(tok, g, pos + it % 3, flags=prep.lib.FLAG_WORKSPACE_PREPARED)
        for k in a:
            np.testing.assert_array_equal(a[k], b[k], err_msg=f"call {it} {k}")


def test_reducing_epilogues_give_identical_bits_every_time():
    """The split-K sums are finished by whichever workgroup arrives last, always in the same
    order: forty repetitions of one step (six rows: the matrix-core path) must agree bit for bit,
    outputs and cache entry alike."""
    shape = gen.scaled(gen.config(2), D=1024, Hq=8, Hkv=2, d=128, I=2560, V=9000, B=6, ctx=(100, 900), k=2)
    w, kv, tok, g, pos = setup(shape, 11, paged=True, std=0.05)
    gd = GpuDraft(shape, w, kv)
    first, cache0 = None, None
    for it in range(40):
        out = gd.step(tok, g, pos)
        gk, gv = gd.cache()
        if first is None:
            first, cache0 = out, (gk, gv)
            continue
        for k in out:
            np.testing.assert_array_equal(out[k], first[k], err_msg=f"repetition {it}: {k}")
        np.testing.assert_array_equal(gk, cache0[0])
        np.testing.assert_array_equal(gv, cache0[1])

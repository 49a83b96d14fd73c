"""GPU parity: specexit_accept_exit against the oracle, bit-exact on every integer output."""
import numpy as np
import pytest

from oracle import specexit_oracle as O
from workloads import gen

from harness import gpu_accept_exit, gpu_state, host

pytestmark = pytest.mark.gpu

INT_KEYS = ("accept_len", "accept_path", "recover_tok", "last_node", "exit_flag", "new_ctx_len")


def oracle_round(cfg_kwargs, case, parent, sig, ctx, state):
    return O.accept_exit(O.ExitCfg(**cfg_kwargs), case.block_tok, parent, case.target_argmax, sig, ctx,
                         case.split_tok, *state)


def compare(got, ref):
    for k in INT_KEYS:
        np.testing.assert_array_equal(got[k], ref[k], err_msg=k)


@pytest.mark.parametrize("index", [0, 1, 2, 3, 4])
@pytest.mark.parametrize("variant", ["default", "latest_split", "check_root", "raw", "conf_only", "rem_only"])
def test_single_round_all_configs(index, variant):
    shape = gen.scaled(gen.config(index), B=max(gen.config(index).B, 32))
    kw = dict(stop_think_token=shape.V - 1)
    if variant == "latest_split":
        kw["split_pick"] = 1
    elif variant == "check_root":
        kw["check_root"] = 1
    elif variant == "raw":
        kw["smoother"] = 1
    elif variant == "conf_only":
        kw.update(signal_mask=1, thr_conf=0.9)
    elif variant == "rem_only":
        kw.update(signal_mask=4, thr_rem=100.0)
    for seed in range(3):
        print(f"accept_exit single round config={index} variant={variant} seed={seed}", flush=True)
        parent = gen.random_tree_parents(shape, seed) if shape.tree else None
        case = gen.accept_case(shape, seed, parent=parent, p_split=0.8)
        if variant == "check_root":
            case.block_tok[::3, 0] = case.split_tok[0]
        r = gen.rng_for(shape, 40, seed)
        sig = np.stack([r.random(shape.B), r.random(shape.B), r.random(shape.B) * 400], axis=1).astype(np.float32)
        sig[::2] = [0.95, 0.9, 20.0]
        ctx = gen.context_lengths(shape, seed)
        ost = (np.zeros((shape.B, 3)), np.zeros(shape.B, np.int32), np.ones(shape.B, np.int32))
        ost[2][1::5] = 0                                # some sequences already left thinking
        gst = gpu_state(shape.B)
        gst[2][1::5] = 0
        ref = oracle_round(kw, case, parent, sig, ctx, ost)
        got = gpu_accept_exit(kw, case.block_tok, parent, case.target_argmax, sig, ctx, case.split_tok, gst)
        compare(got, ref)
        assert ref["exit_flag"].sum() > 0
        np.testing.assert_array_equal(host(gst[2]), ost[2])
        np.testing.assert_array_equal(host(gst[1]), ost[1])
        np.testing.assert_allclose(host(gst[0]), ost[0], rtol=1e-6)


def test_edge_shapes():
    for n_q, B, S in [(1, 1, 0), (1, 5, 3), (64, 4, 8), (2, 257, 1)]:
        print(f"accept_exit edge n_q={n_q} B={B} S={S}", flush=True)
        shape = gen.scaled(gen.config(2), B=B, n_q=n_q, k=max(n_q - 1, 1), V=977)
        case = gen.accept_case(shape, 3, p_split=0.5, n_split=max(S, 1), p_accept=0.97)
        split = case.split_tok[:S]
        case.split_tok = split
        sig = np.tile(np.array([0.9, 0.9, 10.0], np.float32), (B, 1))
        ctx = np.arange(B, dtype=np.int32)
        kw = dict(stop_think_token=5)
        ost = (np.zeros((B, 3)), np.zeros(B, np.int32), np.ones(B, np.int32))
        gst = gpu_state(B)
        ref = oracle_round(kw, case, None, sig, ctx, ost)
        got = gpu_accept_exit(kw, case.block_tok, None, case.target_argmax, sig, ctx, split, gst)
        compare(got, ref)
        if n_q == 64:
            assert ref["accept_len"].max() > 20


def series_with_margin(shape, kw, seed0):
    """Signal series whose float64 smoothed values never come within 1e-4*max(1,|thr|) of a threshold."""
    cfg = O.ExitCfg(**kw)
    for seed in range(seed0, seed0 + 50):
        series, _ = gen.signal_series(shape, seed)
        x = series[0].astype(np.float64).copy()
        ok = True
        for t in range(series.shape[0]):
            if t:
                x = cfg.alpha * series[t].astype(np.float64) + (1 - cfg.alpha) * x
            for j, thr in enumerate((cfg.thr_conf, cfg.thr_prog, cfg.thr_rem)):
                if np.any(np.abs(x[:, j] - thr) < 1e-4 * max(1.0, abs(thr))):
                    ok = False
        if ok:
            return series, seed
    raise AssertionError("no series with a safe margin found")


def conditioned_round(cfg_kw, case, series_t, ctx, ost, hist):
    """One oracle round on signals nudged, where needed, so that no smoothed value of a thinking
    sequence lies within 1e-4*max(1,|thr|) of its threshold (float32 on the GPU must not be able to
    flip a flag).  Input conditioning only: returns the signals used and the oracle's result."""
    cfg = O.ExitCfg(**cfg_kw)
    sig = np.array(series_t, dtype=np.float32)
    thr = (cfg.thr_conf, cfg.thr_prog, cfg.thr_rem)
    for attempt in range(8):
        saved = ([a.copy() for a in ost], [(len(h.values), h.par_start) for h in hist])
        was_thinking = ost[2].copy()
        ref = O.accept_exit(cfg, case.block_tok, None, case.target_argmax, sig, ctx, case.split_tok, *ost, hist=hist)
        near = [(b, j) for b in range(sig.shape[0]) if was_thinking[b] for j in range(3)
                if abs(ost[0][b, j] - thr[j]) < 1e-4 * max(1.0, abs(thr[j]))]
        if not near:
            return sig, ref
        for a, c in zip(ost, saved[0]):
            a[...] = c
        for h, (n, p) in zip(hist, saved[1]):
            del h.values[n:]
            h.par_start = p
        for b, j in near:
            sig[b, j] += np.float32(7e-3 * max(1.0, abs(thr[j])) * (attempt + 1))
    raise AssertionError("could not move the smoothed signals away from the thresholds")


@pytest.mark.parametrize("index", [1, 4])
@pytest.mark.parametrize("smoother", ["window", "momentum", "paragraph", "window4"])
def test_other_smoothers_over_many_rounds(index, smoother):
    """Sliding window, momentum and paragraph mean (Appendix): every round of a whole signal series
    matches the oracle: integer outputs bit-exact, smoothed values to float32 accuracy."""
    shape = gen.config(index)
    kw = dict(stop_think_token=shape.V - 1,
              smoother={"window": 2, "momentum": 3, "paragraph": 4, "window4": 2}[smoother])
    if smoother == "window4":
        kw["window"] = 4
    rounds = shape.n_rounds
    series, _ = gen.signal_series(shape, 5)
    print(f"controller series config={index} smoother={smoother} rounds={rounds}", flush=True)
    ost = (np.zeros((shape.B, 3)), np.zeros(shape.B, np.int32), np.ones(shape.B, np.int32))
    hist = O.new_histories(shape.B)
    gst = gpu_state(shape.B, history=True)
    ctx = gen.context_lengths(shape, 5)
    n_exit = 0
    for t in range(rounds):
        case = gen.accept_case(shape, 3000 + t, p_split=0.3)
        sig, ref = conditioned_round(kw, case, series[t], ctx, ost, hist)
        got = gpu_accept_exit(kw, case.block_tok, None, case.target_argmax, sig, ctx, case.split_tok, gst)
        compare(got, ref)
        np.testing.assert_array_equal(host(gst[2]), ost[2])
        np.testing.assert_allclose(host(gst[0]), ost[0], rtol=2e-5, atol=2e-5, err_msg=f"round {t}")
        n_exit += int(ref["exit_flag"].sum())
        ctx = ref["new_ctx_len"]
    assert n_exit == shape.B, "every sequence should leave thinking within the series"
    np.testing.assert_array_equal(host(gst[1]), ost[1])


def test_smoothers_need_their_state_and_a_valid_window():
    shape = gen.scaled(gen.config(1), B=2)
    case = gen.accept_case(shape, 0)
    sig = np.zeros((2, 3), np.float32)
    ctx = np.array([5, 6], np.int32)
    with pytest.raises(RuntimeError):
        gpu_accept_exit(dict(smoother=2), case.block_tok, None, case.target_argmax, sig, ctx, case.split_tok, gpu_state(2))
    with pytest.raises(RuntimeError):
        gpu_accept_exit(dict(smoother=2, window=17), case.block_tok, None, case.target_argmax, sig, ctx,
                        case.split_tok, gpu_state(2, history=True))
    with pytest.raises(RuntimeError):
        gpu_accept_exit(dict(smoother=5), case.block_tok, None, case.target_argmax, sig, ctx, case.split_tok,
                        gpu_state(2, history=True))


@pytest.mark.parametrize("index", [1, 4])
def test_controller_over_many_rounds(index):
    """Whole signal series: exit round, lengths and state match the oracle at every round."""
    shape = gen.config(index)
    kw = dict(stop_think_token=shape.V - 1)
    series, seed = series_with_margin(shape, kw, 0)
    print(f"controller series config={index} rounds={shape.n_rounds} seed={seed}", flush=True)
    ost = (np.zeros((shape.B, 3)), np.zeros(shape.B, np.int32), np.ones(shape.B, np.int32))
    gst = gpu_state(shape.B)
    ctx = gen.context_lengths(shape, seed)
    exited_o = np.full(shape.B, -1)
    exited_g = np.full(shape.B, -1)
    for t in range(shape.n_rounds):
        case = gen.accept_case(shape, 1000 + t, p_split=0.5)
        ref = oracle_round(kw, case, None, series[t], ctx, ost)
        got = gpu_accept_exit(kw, case.block_tok, None, case.target_argmax, series[t], ctx, case.split_tok, gst)
        compare(got, ref)
        exited_o[(ref["exit_flag"] == 1) & (exited_o < 0)] = t
        exited_g[(got["exit_flag"] == 1) & (exited_g < 0)] = t
        ctx = ref["new_ctx_len"]
    np.testing.assert_array_equal(exited_g, exited_o)
    assert (exited_o >= 0).all(), "every sequence should leave thinking within the series"
    np.testing.assert_allclose(host(gst[0]), ost[0], rtol=1e-4)
    np.testing.assert_array_equal(host(gst[1]), ost[1])

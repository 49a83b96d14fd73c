"""Pins for the oracle's acceptance, smoothing and exit rule (CPU only).

Acceptance: hand-built chains and brute force over all root paths of small
trees.  Smoothing: closed form of the EWMA recurrence and the worked crossing
points stored in tests/golden/exit_rule_constants.txt (constants from the
paper's Appendix).  Exit rule: truth table of Alg. 1's gate and its effects."""
import itertools
import os

import numpy as np
import pytest

from oracle import specexit_oracle as O
from workloads import gen

GOLD = {}
with open(os.path.join(os.path.dirname(__file__), "golden", "exit_rule_constants.txt")) as fh:
    for line in fh:
        line = line.split("#")[0].split()
        if len(line) == 2:
            GOLD[line[0]] = float(line[1])


def fresh_state(B):
    return np.zeros((B, 3)), np.zeros(B, np.int32), np.ones(B, np.int32)


def run(cfg, tok, a, sig=None, parent=None, split=(), ctx=None, state=None):
    tok, a = np.atleast_2d(np.array(tok, np.int32)), np.atleast_2d(np.array(a, np.int32))
    B = tok.shape[0]
    sig = np.zeros((B, 3)) if sig is None else np.atleast_2d(np.array(sig, np.float64))
    ctx = np.full(B, 100, np.int32) if ctx is None else np.array(ctx, np.int32)
    ewma, n_obs, thinking = fresh_state(B) if state is None else state
    par = None if parent is None else np.atleast_2d(np.array(parent, np.int32))
    out = O.accept_exit(cfg, tok, par, a, sig, ctx, np.array(sorted(split), np.int32), ewma, n_obs, thinking)
    out.update(ewma=ewma, n_obs=n_obs, is_thinking=thinking)
    return out


def test_default_constants_are_the_papers():
    c = O.ExitCfg()
    assert c.alpha == GOLD["alpha"]
    assert (c.thr_conf, c.thr_prog, c.thr_rem) == (GOLD["combined_thr_conf"], GOLD["combined_thr_prog"], GOLD["combined_thr_rem"])


# ----------------------------------------------------------------------------- acceptance

def test_chain_all_match_gives_bonus_token():
    out = run(O.ExitCfg(), [9, 1, 2, 3, 4], [1, 2, 3, 4, 77])
    assert out["accept_len"][0] == 4 and out["recover_tok"][0] == 77 and out["last_node"][0] == 4
    assert out["accept_path"][0].tolist() == [1, 2, 3, 4, -1]
    assert out["new_ctx_len"][0] == 100 + 1 + 4 and out["exit_flag"][0] == 0


def test_chain_first_mismatch():
    out = run(O.ExitCfg(), [9, 1, 2, 3, 4], [5, 2, 3, 4, 77])
    assert out["accept_len"][0] == 0 and out["recover_tok"][0] == 5 and out["last_node"][0] == 0
    assert out["accept_path"][0].tolist() == [-1] * 5 and out["new_ctx_len"][0] == 101


def test_chain_match_mismatch_match():
    out = run(O.ExitCfg(), [9, 1, 2, 3, 4], [1, 8, 3, 4, 77])
    assert out["accept_len"][0] == 1 and out["recover_tok"][0] == 8
    assert out["accept_path"][0].tolist() == [1, -1, -1, -1, -1]


def all_root_paths(parent):
    n = len(parent)
    kids = [[c for c in range(n) if parent[c] == p] for p in range(n)]
    paths = [[0]]
    out = []
    while paths:
        p = paths.pop()
        out.append(p)
        for c in kids[p[-1]]:
            paths.append(p + [c])
    return out


@pytest.mark.parametrize("seed", range(6))
def test_tree_walk_equals_longest_matching_root_path(seed):
    shape = gen.scaled(gen.config(3), B=6, V=40)
    par = gen.random_tree_parents(shape, seed)
    case = gen.accept_case(shape, seed, parent=par)
    out = run(O.ExitCfg(), case.block_tok, case.target_argmax, parent=par)
    for b in range(shape.B):
        best = [0]
        for path in all_root_paths(par[b]):
            ok = all(case.block_tok[b, path[j + 1]] == case.target_argmax[b, path[j]] for j in range(len(path) - 1))
            if ok and len(path) > len(best):
                best = path
        # sibling tokens are distinct, so the longest matching path is unique
        assert out["accept_len"][b] == len(best) - 1 == case.planted_len[b]
        assert out["accept_path"][b, :len(best) - 1].tolist() == best[1:]
        assert out["last_node"][b] == best[-1]
        assert out["recover_tok"][b] == case.target_argmax[b, best[-1]]
        assert out["accept_len"][b] <= shape.k
        # accept_path is a root path
        prev = 0
        for node in out["accept_path"][b, :out["accept_len"][b]]:
            assert par[b, node] == prev
            prev = node


def test_generated_chains_have_the_planted_length():
    shape = gen.scaled(gen.config(2), B=64, V=1000)
    case = gen.accept_case(shape, 1)
    out = run(O.ExitCfg(), case.block_tok, case.target_argmax)
    np.testing.assert_array_equal(out["accept_len"], case.planted_len)
    assert case.planted_len.min() == 0 and case.planted_len.max() == shape.n_q - 1


def test_duplicate_sibling_tokens_take_lowest_index():
    # root has children 1, 2 (same token 5); only node 2 has a matching child
    out = run(O.ExitCfg(), [0, 5, 5, 6], [5, 1, 6, 9], parent=[-1, 0, 0, 2])
    assert out["accept_path"][0].tolist() == [1, -1, -1, -1] and out["recover_tok"][0] == 1


# ----------------------------------------------------------------------------- smoothing

def test_ewma_closed_form():
    r = np.random.default_rng(0)
    s = r.random(40)
    cfg = O.ExitCfg(alpha=0.1)
    state = fresh_state(1)
    for t in range(40):
        out = run(cfg, [1, 2], [3, 4], sig=[s[t], -s[t], 1000 * s[t]], state=state)
        x = 0.9 ** t * s[0] + 0.1 * sum(0.9 ** (t - i) * s[i] for i in range(1, t + 1))
        np.testing.assert_allclose(out["ewma"][0], [x, -x, 1000 * x], rtol=1e-13)
        assert out["n_obs"][0] == t + 1


def test_ewma_constant_is_fixed_point_and_alpha_weights_the_new_value():
    state = fresh_state(1)
    for _ in range(5):
        out = run(O.ExitCfg(), [1, 2], [3, 4], sig=[0.37, 0.37, 0.37], state=state)
    np.testing.assert_allclose(out["ewma"][0], 0.37, atol=1e-15)
    out = run(O.ExitCfg(alpha=0.25), [1, 2], [3, 4], sig=[1.37, 0.37, 0.37], state=state)
    np.testing.assert_allclose(out["ewma"][0, 0], 0.37 + 0.25, atol=1e-15)
    assert O.ewma_update(2.0, 12.0, 0.1) == pytest.approx(3.0)


def rounds_until_pass(cfg, first, rest, idx, limit=100):
    """Feed `first` once then `rest`; return n = number of `rest` observations at the first exit."""
    state = fresh_state(1)
    base = [1.0, 1.0, 0.0]                # the two other signals always pass
    for n in range(limit):
        sig = list(base)
        sig[idx] = first if n == 0 else rest
        out = run(cfg, [7, 3, 4], [3, 9, 9], sig=sig, split=[3], state=state)
        if out["exit_flag"][0]:
            return n
    return None


def test_worked_threshold_cases():
    """Series 0,1,1,... crosses x > thr after n ones; 2000,0,0,... drops below after n zeros."""
    assert rounds_until_pass(O.ExitCfg(), 0.0, 1.0, 1) == GOLD["ones_cross_0.3"]
    assert rounds_until_pass(O.ExitCfg(), 0.0, 1.0, 0) == GOLD["ones_cross_0.8"]
    assert rounds_until_pass(O.ExitCfg(), 2000.0, 0.0, 2) == GOLD["decay_below_200"]
    single = dict(thr_conf=GOLD["single_thr_conf"], thr_prog=GOLD["single_thr_prog"], thr_rem=GOLD["single_thr_rem"])
    assert rounds_until_pass(O.ExitCfg(signal_mask=1, **single), 0.0, 1.0, 0) == GOLD["ones_cross_0.9"]
    assert rounds_until_pass(O.ExitCfg(signal_mask=2, **single), 0.0, 1.0, 1) == GOLD["ones_cross_0.8"]
    assert rounds_until_pass(O.ExitCfg(signal_mask=4, **single), 2000.0, 0.0, 2) == GOLD["decay_below_100"]


def test_thresholds_are_strict_and_directed():
    cfg = O.ExitCfg()
    assert O.signals_pass([0.81, 0.31, 199.0], cfg)
    assert not O.signals_pass([0.8, 0.31, 199.0], cfg)        # confidence must exceed
    assert not O.signals_pass([0.81, 0.3, 199.0], cfg)        # progress must exceed
    assert not O.signals_pass([0.81, 0.31, 200.0], cfg)       # remaining must be below
    assert not O.signals_pass([0.81, 0.31, 5000.0], cfg)
    assert O.signals_pass([0.0, 0.0, 50.0], O.ExitCfg(signal_mask=4, thr_rem=100))
    assert O.signals_pass([0.95, 0.0, 1e9], O.ExitCfg(signal_mask=1, thr_conf=0.9))
    assert not O.signals_pass([0.95, 0.0, 1e9], O.ExitCfg(signal_mask=3, thr_conf=0.9, thr_prog=0.8))


def test_no_smoothing_mode_uses_the_raw_signal():
    state = fresh_state(1)
    run(O.ExitCfg(smoother=1), [7, 3], [3, 9], sig=[0, 0, 9999], split=[3], state=state)
    out = run(O.ExitCfg(smoother=1), [7, 3], [3, 9], sig=[0.9, 0.9, 1.0], split=[3], state=state)
    assert out["exit_flag"][0] == 1


# ----------------------------------------------------------------------------- exit rule

PASS, FAIL = [0.9, 0.9, 10.0], [0.9, 0.9, 900.0]


@pytest.mark.parametrize("thinking,has_split,passes", itertools.product([0, 1], repeat=3))
def test_gate_truth_table(thinking, has_split, passes):
    state = fresh_state(1)
    state[2][0] = thinking
    out = run(O.ExitCfg(stop_think_token=555), [7, 3, 4, 5], [3, 4, 8, 8], sig=PASS if passes else FAIL,
              split=[4] if has_split else [6], state=state)
    fired = thinking and has_split and passes
    assert out["exit_flag"][0] == int(fired)
    if fired:
        assert out["accept_len"][0] == 2 and out["recover_tok"][0] == 555 and out["is_thinking"][0] == 0
        assert out["accept_path"][0].tolist() == [1, 2, -1, -1] and out["last_node"][0] == 2
        assert out["new_ctx_len"][0] == 103
    else:
        assert out["accept_len"][0] == 2 and out["recover_tok"][0] == 8 and out["is_thinking"][0] == thinking


def test_truncation_keeps_the_split_token_and_drops_the_rest():
    # all four drafts accepted; split token is the 2nd accepted draft
    out = run(O.ExitCfg(stop_think_token=1), [7, 3, 4, 5, 6], [3, 4, 5, 6, 9], sig=PASS, split=[4])
    assert out["accept_len"][0] == 2 and out["accept_path"][0].tolist() == [1, 2, -1, -1, -1]
    assert out["recover_tok"][0] == 1 and out["new_ctx_len"][0] == 103


def test_earliest_or_latest_split_token():
    args = dict(tok=[7, 3, 4, 5, 6], a=[3, 4, 5, 6, 9], sig=PASS, split=[3, 5])
    assert run(O.ExitCfg(split_pick=0), **args)["accept_len"][0] == 1
    assert run(O.ExitCfg(split_pick=1), **args)["accept_len"][0] == 3


def test_split_token_beyond_accepted_prefix_never_triggers():
    out = run(O.ExitCfg(), [7, 3, 4, 5], [3, 0, 5, 9], sig=PASS, split=[5])
    assert out["exit_flag"][0] == 0 and out["accept_len"][0] == 1 and out["recover_tok"][0] == 0


def test_root_and_recover_token_are_not_accepted_draft_tokens():
    # root (7) and the target's own next token (9) are in the split set but no accepted draft is
    out = run(O.ExitCfg(), [7, 3, 4], [3, 4, 9], sig=PASS, split=[7, 9])
    assert out["exit_flag"][0] == 0 and out["accept_len"][0] == 2
    out = run(O.ExitCfg(check_root=1, stop_think_token=2), [7, 3, 4], [3, 4, 9], sig=PASS, split=[7, 9])
    assert out["exit_flag"][0] == 1 and out["accept_len"][0] == 0 and out["recover_tok"][0] == 2
    assert out["last_node"][0] == 0 and out["new_ctx_len"][0] == 101


def test_exit_fires_once_and_state_freezes():
    state = fresh_state(1)
    first = run(O.ExitCfg(), [7, 3], [3, 9], sig=PASS, split=[3], state=state)
    assert first["exit_flag"][0] == 1
    snap = state[0].copy()
    second = run(O.ExitCfg(), [7, 3], [3, 9], sig=[0.1, 0.2, 0.3], split=[3], state=state)
    assert second["exit_flag"][0] == 0 and second["accept_len"][0] == 1 and second["recover_tok"][0] == 9
    np.testing.assert_array_equal(state[0], snap)
    assert state[1][0] == 1


def test_exit_in_a_tree_cuts_the_accepted_path():
    par = [-1, 0, 0, 2, 2, 3]
    out = run(O.ExitCfg(stop_think_token=99), [7, 1, 2, 3, 4, 5], [2, 0, 3, 5, 0, 8], sig=PASS, parent=par, split=[3])
    # matching root path 0 -> 2 -> 3 -> 5 ; split token sits on node 3 (2nd accepted)
    assert out["accept_len"][0] == 2 and out["accept_path"][0].tolist() == [2, 3, -1, -1, -1, -1]
    assert out["last_node"][0] == 3 and out["recover_tok"][0] == 99


def test_sequences_are_independent():
    shape = gen.scaled(gen.config(2), B=16, V=500)
    case = gen.accept_case(shape, 5, p_split=0.7)
    sig = np.tile(np.array(PASS), (16, 1))
    sig[::2] = FAIL
    cfg = O.ExitCfg(stop_think_token=case.stop_think_token)
    full = run(cfg, case.block_tok, case.target_argmax, sig=sig, split=case.split_tok)
    assert 0 < full["exit_flag"].sum() < 16
    for b in (0, 3, 15):
        one = run(cfg, case.block_tok[b], case.target_argmax[b], sig=sig[b], split=case.split_tok)
        for key in ("accept_len", "recover_tok", "exit_flag", "last_node", "new_ctx_len"):
            assert one[key][0] == full[key][b]

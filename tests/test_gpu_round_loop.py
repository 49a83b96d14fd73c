"""Several decode rounds in a row with every entry point's outputs feeding the next call on the
device: draft chain -> block -> verification attention -> LM-head argmax -> acceptance / exit ->
cache compaction -> the next round's start token, start hidden state and context lengths.  The
oracle runs the same loop on the host; every integer of every round must agree (Alg. 1).

There is no target model here.  Its stand-in (`target_rows`) builds the target's final hidden row
of each block node from the LM-head row of the token the target is said to prefer there: the next
draft token with probability 0.7, another seeded token otherwise.  That is input preparation, done
the same way for both sides from the block's token ids."""
import numpy as np
import pytest
import torch

from oracle import specexit_oracle as O
from workloads import gen
import harness as H

pytestmark = pytest.mark.gpu

N_ROUNDS = 6
GAP = 0.05


def loop_shape(dtype, B):
    s = gen.scaled(gen.config(0), dtype=dtype, B=B, ctx=(150, 200))
    return s


def wanted_tokens(shape, block_tok, rnd, seed):
    """Token the stand-in target prefers after each block node ([B, n_q])."""
    B, n_q = block_tok.shape
    r = gen.rng_for(shape, 40 + rnd, seed)
    agree = r.random((B, n_q)) < 0.7
    other = r.integers(0, shape.V - 1, size=(B, n_q))
    want = other.copy()
    for b in range(B):
        for i in range(n_q):
            if i + 1 < n_q and agree[b, i]:
                want[b, i] = block_tok[b, i + 1]
            elif i + 1 < n_q and other[b, i] == block_tok[b, i + 1]:
                want[b, i] = (other[b, i] + 1) % (shape.V - 1)
    return want


def target_rows(shape, lm, block_tok, rnd, seed):
    """[B, n_q, D] hidden rows in the storage type whose LM-head argmax is wanted_tokens by a wide margin."""
    want = wanted_tokens(shape, block_tok, rnd, seed)
    rows = 8.0 * lm[want].astype(np.float64)
    return gen.store(shape, rows.astype(np.float32)), want


class Inputs:
    def __init__(self, shape, seed, std=0.02, big_embeddings=False):
        self.shape, self.seed = shape, seed
        self.w = gen.draft_weights(shape, seed, std=std)
        if big_embeddings:
            # token embeddings as large as the hidden states: sibling nodes of a tree (same parent
            # state, different token) must not come out with nearly the same logits
            self.w.update(gen.perturbed_norm_vectors(shape, seed))
            self.w["embed"] = gen.store(shape, self.w["embed"] * np.float32(1.0 / std))
        self.lm = gen.lm_head(shape, seed)
        self.L0 = gen.context_lengths(shape, seed)
        room = N_ROUNDS * shape.n_q + 2
        self.dkv = gen.kv_cache(shape, self.L0, room, seed, stream=17)
        self.tkv = gen.kv_cache(shape, self.L0, room, seed)
        self.tok0 = gen.token_ids(shape, shape.B, seed)
        self.g0 = gen.hidden_rows(shape, shape.B, seed, stream=18)
        self.q = [gen.queries(shape, seed + 100 + r) for r in range(N_ROUNDS)]
        r = gen.rng_for(shape, 39, seed)
        self.split = np.sort(r.choice(shape.V - 1, size=shape.V // 3, replace=False)).astype(np.int32)
        self.stop = shape.V - 1


def oracle_loop(inp: Inputs, cfg: O.ExitCfg, w=None):
    """The loop on the host.  Returns one record per round (plus, per draft step, what the gap forcing needs)."""
    s = inp.shape
    w = inp.w if w is None else w
    dims = H.oracle_dims(s)
    store = lambda a: gen.store(s, np.asarray(a, np.float32))
    kc, vc = inp.dkv.k.astype(np.float64), inp.dkv.v.astype(np.float64)
    tk, tv = inp.tkv.k.copy(), inp.tkv.v.copy()
    tok, g, L = inp.tok0.copy(), inp.g0.copy(), inp.L0.astype(np.int32).copy()
    ewma, n_obs, thinking = np.zeros((s.B, 3)), np.zeros(s.B, np.int32), np.ones(s.B, np.int32)
    recs = []
    for rnd in range(N_ROUNDS):
        block = np.zeros((s.B, s.n_q), np.int32)
        block[:, 0] = tok
        t, h, sig0, steps = tok, g, None, []
        for j in range(s.k):
            out = O.draft_step(dims, w, kc, vc, t, h, L + j, store=store)
            t, h = out["next_tok"].astype(np.int32), store(out["hidden_out"])
            block[:, j + 1] = t
            sig0 = out["sig"] if sig0 is None else sig0
            steps.append((out["h_final"], out["logits"]))
        hid, want = target_rows(s, inp.lm, block, rnd, inp.seed)
        attn = O.verify_attn(inp.q[rnd], tk, tv, L)
        am, z, _ = O.lmhead_argmax(hid.reshape(s.B * s.n_q, s.D), inp.lm)
        assert np.array_equal(am.reshape(s.B, s.n_q), want) and O.top2_gap(z).min() > 4 * GAP
        sig32 = sig0.astype(np.float32)
        o = O.accept_exit(cfg, block, None, am.reshape(s.B, s.n_q), sig32, L, inp.split, ewma, n_obs, thinking)
        tk, tv, g = O.kv_compact(tk, tv, L, o["accept_path"], o["accept_len"], block_hidden=hid,
                                 last_node=o["last_node"])
        recs.append(dict(block_tok=block, target_argmax=am.reshape(s.B, s.n_q), sig=sig0, attn=attn,
                         accept_len=o["accept_len"].copy(), recover_tok=o["recover_tok"].copy(),
                         exit_flag=o["exit_flag"].copy(), new_ctx_len=o["new_ctx_len"].copy(),
                         last_node=o["last_node"].copy(), smoothed=ewma.copy(), thinking=thinking.copy(),
                         hidden_next=g.copy(), steps=steps))
        tok, L = o["recover_tok"].astype(np.int32), o["new_ctx_len"].astype(np.int32)
    return recs


def force_loop_gap(inp: Inputs, cfg: O.ExitCfg, w=None, max_iter=12):
    """Bump the winners' token rows of w_head until every draft argmax of the whole loop has a top-2
    gap above GAP in the oracle's logits (a bump can change later steps, hence the iteration)."""
    s, w = inp.shape, dict(inp.w if w is None else w)
    for _ in range(max_iter):
        recs = oracle_loop(inp, cfg, w)
        head, bad = w["w_head"].copy(), 0
        for rec in recs:
            for h_fin, z in rec["steps"]:
                gaps = O.top2_gap(z)
                for b in np.flatnonzero(gaps < 1.2 * GAP):
                    bad += 1
                    h = h_fin[b]
                    big = np.argsort(-np.abs(h))[:64]       # a bump spread thinner would round away in bf16
                    win = O.argmax_lowest(z[b])
                    row = head[win].astype(np.float64)
                    row[big] += (2.0 * GAP - gaps[b]) * h[big] / (h[big] @ h[big])
                    head[win] = gen.store(s, row.astype(np.float32))
        if bad == 0:
            return w, recs
        w["w_head"] = head
    raise AssertionError("could not force the draft logit gaps of the loop")


def clear_of(recs, thr, margin):
    sm = np.concatenate([r["smoothed"] for r in recs])           # [rounds * B, 3]
    return all(np.min(np.abs(sm[:, j] - thr[j])) > margin * max(1.0, abs(thr[j])) for j in range(3))


def thresholds_off_the_values(recs, margin):
    """Thresholds that three quarters of the smoothed scores seen in the loop pass, moved until no
    observed value lies within `margin` of them: the exit decision must not hinge on rounding."""
    sm = np.concatenate([r["smoothed"] for r in recs])
    thr = []
    for j in range(3):
        vals = np.sort(sm[:, j])
        t = float(np.quantile(vals, 0.75 if j == 2 else 0.25))
        for _ in range(200):
            if np.min(np.abs(vals - t)) > margin * max(1.0, abs(t)):
                break
            t += (0.37 if j == 2 else -0.37) * margin * max(1.0, abs(t))
        else:
            raise AssertionError("no threshold clear of the observed scores")
        thr.append(t)
    return thr


def gpu_loop(inp: Inputs, cfg: O.ExitCfg, w):
    """The same loop through the C ABI.  Device buffers written by one call are read by the next;
    only the stand-in target takes the block's token ids to the host."""
    lib, s = H.sx(), inp.shape
    B, n_q, k = s.B, s.n_q, s.k
    dt = lib.BF16 if s.dtype == "bf16" else lib.F32
    draft = H.GpuDraft(s, w, inp.dkv)
    tview, tkeep = H.kv_view_of(s, inp.tkv)
    lm = H.dev(inp.lm, s)
    split = H.dev(inp.split)
    i32 = lambda *sh: torch.empty(sh, dtype=torch.int32, device="cuda")
    f32 = lambda *sh: torch.empty(sh, dtype=torch.float32, device="cuda")
    ws_attn = H.workspace(lib.specexit_verify_attn_workspace_bytes(tview, B, n_q, s.Hq))
    ws_head = H.workspace(lib.specexit_lmhead_argmax_workspace_bytes(dt, B * n_q, s.D, s.V, 0))
    ewma, n_obs, thinking = H.gpu_state(B)
    ecfg = lib.exit_cfg(alpha=cfg.alpha, thr_conf=cfg.thr_conf, thr_prog=cfg.thr_prog, thr_rem=cfg.thr_rem,
                        stop_think_token=cfg.stop_think_token)
    tok, g, ctx = H.dev(inp.tok0.astype(np.int32)), H.dev(inp.g0, s), H.dev(inp.L0.astype(np.int32))
    recs = []
    for rnd in range(N_ROUNDS):
        print(f"  round {rnd}", flush=True)
        block = i32(B, n_q)
        block[:, 0] = tok
        hid2 = [torch.empty_like(g) for _ in range(2)]
        nt, sr, sg = [i32(B) for _ in range(k)], [f32(B, 3) for _ in range(k)], [f32(B, 3) for _ in range(k)]
        t, h = tok, g
        for j in range(k):
            lib.specexit_draft_step(draft.desc, draft.w, draft.view, B, t, h, (ctx + j).contiguous(), hid2[j & 1],
                                    nt[j], sr[j], sg[j], draft.ws)
            t, h = nt[j], hid2[j & 1]
            block[:, j + 1] = nt[j]
        hid_np, _ = target_rows(s, inp.lm, H.host(block), rnd, inp.seed)
        hid = H.dev(hid_np, s)
        q = H.dev(inp.q[rnd], s)
        attn = torch.empty_like(q)
        lib.specexit_verify_attn(tview, B, n_q, s.Hq, q, ctx, None, s.d ** -0.5, attn, ws_attn)
        am = i32(B * n_q)
        lib.specexit_lmhead_argmax(dt, B * n_q, s.D, s.V, 0, hid.reshape(B * n_q, s.D), lm, am, workspace=ws_head)
        o = {n: i32(B) for n in ("accept_len", "recover_tok", "last_node", "exit_flag", "new_ctx_len")}
        path = i32(B, n_q)
        lib.specexit_accept_exit(ecfg, B, n_q, block, None, am, sg[0], ctx, split, len(inp.split), ewma, n_obs,
                                 thinking, None, o["accept_len"], path, o["recover_tok"], o["last_node"],
                                 o["exit_flag"], o["new_ctx_len"])
        g_next = torch.empty_like(g)
        lib.specexit_kv_compact(tview, 1, 0, B, n_q, ctx, path, o["accept_len"], o["last_node"], hid, s.D, g_next)
        torch.cuda.synchronize()
        rec = {n: H.host(v) for n, v in o.items()}
        rec.update(block_tok=H.host(block), target_argmax=H.host(am).reshape(B, n_q), sig=H.host(sg[0]),
                   attn=H.host(attn), smoothed=H.host(ewma), thinking=H.host(thinking), hidden_next=H.host(g_next))
        recs.append(rec)
        tok, g, ctx = o["recover_tok"], g_next, o["new_ctx_len"]
    return recs


@pytest.mark.parametrize("dtype,B", [("f32", 3), ("bf16", 3), ("bf16", 6)])
def test_rounds_chained_on_the_device(dtype, B):
    shape = loop_shape(dtype, B)
    inp = Inputs(shape, seed=3)
    probe = O.ExitCfg(thr_conf=2.0, stop_think_token=inp.stop)       # never exits: shows the scores' range
    w, recs = force_loop_gap(inp, probe)
    thr = thresholds_off_the_values(recs, 2.5 * H.TOL[dtype])
    cfg = O.ExitCfg(thr_conf=thr[0], thr_prog=thr[1], thr_rem=thr[2], stop_think_token=inp.stop)
    w, ref = force_loop_gap(inp, cfg, w)
    assert clear_of(ref, thr, 2 * H.TOL[dtype])
    got = gpu_loop(inp, cfg, w)
    assert sum(int(r["exit_flag"].sum()) for r in ref) >= 1, "the loop should see an exit"
    assert sum(int(r["accept_len"].sum()) for r in ref) >= N_ROUNDS, "and accepted drafts"
    tol = H.TOL[dtype]
    for rnd, (a, b) in enumerate(zip(got, ref)):
        for name in ("block_tok", "target_argmax", "accept_len", "recover_tok", "last_node", "exit_flag",
                     "new_ctx_len", "thinking"):
            assert np.array_equal(a[name], b[name]), (rnd, name, a[name], b[name])
        assert H.rel_err(a["sig"], b["sig"]) < tol, rnd
        assert H.rel_err(a["smoothed"], b["smoothed"]) < tol, rnd
        assert H.rel_err(a["attn"], b["attn"]) < tol, rnd
        assert np.array_equal(a["hidden_next"], b["hidden_next"]), rnd


# ----------------------------------------------------------------------------- the same loop over a drafted tree

def tree_wanted_tokens(shape, block_tok, parent, rnd, seed):
    """With a tree the stand-in target prefers, after a node, the token of one of the node's
    children (a seeded pick, probability 0.7) or a token that none of them carries."""
    B, n = block_tok.shape
    r = gen.rng_for(shape, 60 + rnd, seed)
    agree = r.random((B, n)) < 0.7
    pick = r.integers(0, 1 << 30, size=(B, n))
    want = r.integers(0, shape.V - 1, size=(B, n))
    for b in range(B):
        for i in range(n):
            kids = [c for c in range(1, n) if int(parent[c]) == i]
            if kids and agree[b, i]:
                want[b, i] = block_tok[b, kids[int(pick[b, i]) % len(kids)]]
            else:
                taken = {int(block_tok[b, c]) for c in kids}
                while int(want[b, i]) in taken:
                    want[b, i] = (want[b, i] + 1) % (shape.V - 1)
    return want


def tree_target_rows(shape, lm, block_tok, parent, rnd, seed):
    want = tree_wanted_tokens(shape, block_tok, parent, rnd, seed)
    return gen.store(shape, (8.0 * lm[want].astype(np.float64)).astype(np.float32)), want


def oracle_tree_loop(inp: Inputs, cfg: O.ExitCfg, parent, rank, w=None):
    """Tree rounds on the host.  After acceptance both caches are compacted along the accepted path:
    the target layer's (its block K/V came with the inputs) and the draft layer's own.  The draft
    cache holds entries only for nodes that were run through the draft forward; for an accepted leaf
    the compaction moves whatever its slot held, which a full decoder would overwrite by feeding the
    accepted tokens again -- outside this path, and the same on both sides."""
    s = inp.shape
    w = inp.w if w is None else w
    dims = H.oracle_dims(s)
    store = lambda a: gen.store(s, np.asarray(a, np.float32))
    kc, vc = inp.dkv.k.astype(np.float64), inp.dkv.v.astype(np.float64)
    tk, tv = inp.tkv.k.copy(), inp.tkv.v.copy()
    tok, g, L = inp.tok0.copy(), inp.g0.copy(), inp.L0.astype(np.int32).copy()
    ewma, n_obs, thinking = np.zeros((s.B, 3)), np.zeros(s.B, np.int32), np.ones(s.B, np.int32)
    par_b = np.tile(np.asarray(parent, np.int32), (s.B, 1))
    mask = gen.ancestor_masks(par_b)
    recs = []
    for rnd in range(N_ROUNDS):
        out = O.draft_tree(dims, w, kc, vc, tok, g, L, parent, rank, store=store)
        block = out["block_tok"].astype(np.int32)
        hid, want = tree_target_rows(s, inp.lm, block, parent, rnd, inp.seed)
        attn = O.verify_attn(inp.q[rnd], tk, tv, L, mask)
        am, z, _ = O.lmhead_argmax(hid.reshape(s.B * s.n_q, s.D), inp.lm)
        assert np.array_equal(am.reshape(s.B, s.n_q), want) and O.top2_gap(z).min() > 4 * GAP
        sig0 = out["sig"][:, 0]
        o = O.accept_exit(cfg, block, par_b, am.reshape(s.B, s.n_q), sig0.astype(np.float32), L, inp.split,
                          ewma, n_obs, thinking)
        tk, tv, g = O.kv_compact(tk, tv, L, o["accept_path"], o["accept_len"], block_hidden=hid,
                                 last_node=o["last_node"])
        kc, vc = O.kv_compact(kc, vc, L, o["accept_path"], o["accept_len"])
        recs.append(dict(block_tok=block, target_argmax=am.reshape(s.B, s.n_q), sig=sig0, attn=attn,
                         accept_len=o["accept_len"].copy(), accept_path=o["accept_path"].copy(),
                         recover_tok=o["recover_tok"].copy(), exit_flag=o["exit_flag"].copy(),
                         new_ctx_len=o["new_ctx_len"].copy(), last_node=o["last_node"].copy(),
                         smoothed=ewma.copy(), thinking=thinking.copy(), hidden_next=g.copy(),
                         tree=out, target_k=tk.copy()))
        tok, L = o["recover_tok"].astype(np.int32), o["new_ctx_len"].astype(np.int32)
    return recs


def force_tree_loop_gap(inp: Inputs, cfg: O.ExitCfg, parent, rank, top_b, w=None, max_iter=16):
    """As force_loop_gap, for the top_b + 1 best logits of every expanded node of every round."""
    s, w = inp.shape, dict(inp.w if w is None else w)
    for _ in range(max_iter):
        recs = oracle_tree_loop(inp, cfg, parent, rank, w)
        head, bad = w["w_head"].copy(), 0
        for rec in recs:
            out = rec["tree"]
            for b in range(s.B):
                for c in np.flatnonzero(out["expanded"]):
                    z = out["logits"][b, c]
                    order = O.top_b_lowest(z, top_b + 1)
                    if (z[order[:-1]] - z[order[1:]]).min() >= 1.2 * GAP:
                        continue
                    bad += 1
                    h = out["h_final"][b, c]
                    big = np.argsort(-np.abs(h))[:64]
                    inc = 0.0                                  # raise only what is missing, from the bottom up
                    for r in range(top_b - 1, -1, -1):
                        inc += max(0.0, 1.6 * GAP - (z[order[r]] - z[order[r + 1]]))
                        if inc > 0.0:
                            row = head[order[r]].astype(np.float64)
                            row[big] += inc * h[big] / (h[big] @ h[big])
                            head[order[r]] = gen.store(s, row.astype(np.float32))
        if bad == 0:
            return w, recs
        w["w_head"] = head
    raise AssertionError("could not force the logit gaps of the tree loop")


def gpu_tree_loop(inp: Inputs, cfg: O.ExitCfg, w, parent, rank, top_b):
    lib, s = H.sx(), inp.shape
    B, n_q = s.B, s.n_q
    dt = lib.BF16 if s.dtype == "bf16" else lib.F32
    draft = H.GpuDraft(s, w, inp.dkv)
    tview, tkeep = H.kv_view_of(s, inp.tkv)
    lm, split = H.dev(inp.lm, s), H.dev(inp.split)
    par_b = np.tile(np.asarray(parent, np.int32), (B, 1))
    par_d, mask_d = H.dev(par_b), H.dev(gen.ancestor_masks(par_b))
    i32 = lambda *sh: torch.empty(sh, dtype=torch.int32, device="cuda")
    ws_attn = H.workspace(lib.specexit_verify_attn_workspace_bytes(tview, B, n_q, s.Hq))
    ws_head = H.workspace(lib.specexit_lmhead_argmax_workspace_bytes(dt, B * n_q, s.D, s.V, 0))
    ewma, n_obs, thinking = H.gpu_state(B)
    ecfg = lib.exit_cfg(alpha=cfg.alpha, thr_conf=cfg.thr_conf, thr_prog=cfg.thr_prog, thr_rem=cfg.thr_rem,
                        stop_think_token=cfg.stop_think_token)
    tok, g, ctx = H.dev(inp.tok0.astype(np.int32)), H.dev(inp.g0, s), H.dev(inp.L0.astype(np.int32))
    recs = []
    for rnd in range(N_ROUNDS):
        print(f"  tree round {rnd}", flush=True)
        t = draft.tree(tok, g, ctx, parent, rank, top_b)
        block = t["block_tok_dev"]
        hid_np, _ = tree_target_rows(s, inp.lm, t["block_tok"], parent, rnd, inp.seed)
        hid, q = H.dev(hid_np, s), H.dev(inp.q[rnd], s)
        attn = torch.empty_like(q)
        lib.specexit_verify_attn(tview, B, n_q, s.Hq, q, ctx, mask_d, s.d ** -0.5, attn, ws_attn)
        am = i32(B * n_q)
        lib.specexit_lmhead_argmax(dt, B * n_q, s.D, s.V, 0, hid.reshape(B * n_q, s.D), lm, am, workspace=ws_head)
        o = {n: i32(B) for n in ("accept_len", "recover_tok", "last_node", "exit_flag", "new_ctx_len")}
        path = i32(B, n_q)
        lib.specexit_accept_exit(ecfg, B, n_q, block, par_d, am, t["sig_dev"][0], ctx, split, len(inp.split), ewma,
                                 n_obs, thinking, None, o["accept_len"], path, o["recover_tok"], o["last_node"],
                                 o["exit_flag"], o["new_ctx_len"])
        g_next = torch.empty_like(g)
        lib.specexit_kv_compact(tview, 1, 0, B, n_q, ctx, path, o["accept_len"], o["last_node"], hid, s.D, g_next)
        lib.specexit_kv_compact(draft.view, 1, 0, B, n_q, ctx, path, o["accept_len"])
        torch.cuda.synchronize()
        rec = {n: H.host(v) for n, v in o.items()}
        rec.update(block_tok=t["block_tok"], target_argmax=H.host(am).reshape(B, n_q), sig=H.host(t["sig_dev"][0]),
                   attn=H.host(attn), smoothed=H.host(ewma), thinking=H.host(thinking),
                   hidden_next=H.host(g_next), accept_path=H.host(path), target_k=H.host(tkeep[0]))
        recs.append(rec)
        tok, g, ctx = o["recover_tok"], g_next, o["new_ctx_len"]
    return recs


@pytest.mark.parametrize("dtype,B", [("f32", 2), ("bf16", 2)])
def test_tree_rounds_chained_on_the_device(dtype, B):
    shape = gen.scaled(gen.config(0), dtype=dtype, B=B, tree=True, n_q=8, k=3, ctx=(150, 200))
    parent, rank = gen.level_ordered_tree(shape, 1)
    top_b = int(rank.max()) + 1
    inp = Inputs(shape, seed=5, std=0.05, big_embeddings=True)
    probe = O.ExitCfg(thr_conf=2.0, stop_think_token=inp.stop)
    w, recs = force_tree_loop_gap(inp, probe, parent, rank, top_b)
    thr = thresholds_off_the_values(recs, 2.5 * H.TOL[dtype])
    cfg = O.ExitCfg(thr_conf=thr[0], thr_prog=thr[1], thr_rem=thr[2], stop_think_token=inp.stop)
    w, ref = force_tree_loop_gap(inp, cfg, parent, rank, top_b, w)
    assert clear_of(ref, thr, 2 * H.TOL[dtype])
    got = gpu_tree_loop(inp, cfg, w, parent, rank, top_b)
    assert sum(int(r["accept_len"].sum()) for r in ref) >= N_ROUNDS
    assert any((r["accept_path"][b, :r["accept_len"][b]] != np.arange(1, r["accept_len"][b] + 1)).any()
               for r in ref for b in range(B)), "some accepted path should need its cache rows moved"
    tol = H.TOL[dtype]
    for rnd, (a, b) in enumerate(zip(got, ref)):
        for name in ("block_tok", "target_argmax", "accept_len", "accept_path", "recover_tok", "last_node",
                     "exit_flag", "new_ctx_len", "thinking"):
            assert np.array_equal(a[name], b[name]), (rnd, name, a[name], b[name])
        assert H.rel_err(a["sig"], b["sig"]) < tol, rnd
        assert H.rel_err(a["smoothed"], b["smoothed"]) < tol, rnd
        assert H.rel_err(a["attn"], b["attn"]) < tol, rnd
        assert np.array_equal(a["hidden_next"], b["hidden_next"]), rnd
        assert np.array_equal(a["target_k"], b["target_k"]), rnd       # copies of input bytes: exact

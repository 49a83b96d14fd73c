"""A decode round recorded with specexit_graph_begin / _end and replayed with specexit_graph_launch
matches the oracle's round on the same inputs (integers bit-exact, floats within tolerance), and
gives, replay after replay, the bits of the same calls launched one by one -- also after the caller
has refilled the input buffers, and with other work of the process in between."""
import numpy as np
import pytest
import torch

from oracle import specexit_oracle as O
from workloads import gen
import harness as H

pytestmark = pytest.mark.gpu


class DeviceRound:
    """Buffers of one small round (two draft steps, verification attention, LM head, acceptance,
    cache compaction) and the calls that make it up, all on one stream."""

    def __init__(self, shape, seed, w=None, lm=None):
        lib = self.lib = H.sx()
        self.s = s = shape
        B, n_q = s.B, s.n_q
        self.dt = lib.BF16 if s.dtype == "bf16" else lib.F32
        # the host copies stay as they were generated: the oracle's round reads them
        self.h = h = dict(w=gen.draft_weights(s, seed) if w is None else w, L=gen.context_lengths(s, seed),
                          lm=gen.lm_head(s, seed) if lm is None else lm, tok0=gen.token_ids(s, B, seed),
                          g0=gen.hidden_rows(s, B, seed, stream=18), q=gen.queries(s, seed),
                          hid=gen.hidden_rows(s, B * n_q, seed), case=gen.accept_case(s, seed, p_split=1.0))
        L = h["L"]
        h["dkv"], h["tkv"] = gen.kv_cache(s, L, n_q + 2, seed, stream=17), gen.kv_cache(s, L, n_q + 2, seed)
        self.draft = H.GpuDraft(s, h["w"], h["dkv"])
        self.tview, self.tkeep = H.kv_view_of(s, h["tkv"])
        self.k0, self.v0 = self.tkeep[0].clone(), self.tkeep[1].clone()
        self.lm = H.dev(h["lm"], s)
        self.tok0 = H.dev(h["tok0"])
        self.g0 = H.dev(h["g0"], s)
        self.ctx = H.dev(L.astype(np.int32))
        self.pos = [H.dev((L + j).astype(np.int32)) for j in range(2)]
        self.q = H.dev(h["q"], s)
        self.hid = H.dev(h["hid"], s)
        case = h["case"]
        self.block = H.dev(case.block_tok)
        self.split = H.dev(case.split_tok)
        self.exit_kw = dict(thr_conf=0.0, thr_prog=0.0, thr_rem=1e9, stop_think_token=case.stop_think_token)
        self.cfg = lib.exit_cfg(**self.exit_kw)
        i32 = lambda *sh: torch.zeros(sh, dtype=torch.int32, device="cuda")
        f32 = lambda *sh: torch.zeros(sh, dtype=torch.float32, device="cuda")
        self.hout = [torch.zeros_like(self.g0) for _ in range(2)]
        self.nt = [i32(B) for _ in range(2)]
        self.sr, self.sg = [f32(B, 3) for _ in range(2)], [f32(B, 3) for _ in range(2)]
        self.attn = torch.zeros_like(self.q)
        self.am = i32(B * n_q)
        self.state = H.gpu_state(B)
        self.o = {n: i32(B) for n in ("accept_len", "recover_tok", "last_node", "exit_flag", "new_ctx_len")}
        self.path = i32(B, n_q)
        self.g_next = torch.zeros_like(self.g0)
        self.ws_attn = H.workspace(lib.specexit_verify_attn_workspace_bytes(self.tview, B, n_q, s.Hq))
        self.ws_head = H.workspace(lib.specexit_lmhead_argmax_workspace_bytes(self.dt, B * n_q, s.D, s.V, 0))

    def reset(self):
        """What a round changes beyond its outputs goes back to the start: the controller's state and
        the target cache rows the compaction moved."""
        self.state[0].zero_(); self.state[1].zero_(); self.state[2].fill_(1)
        self.tkeep[0].copy_(self.k0); self.tkeep[1].copy_(self.v0)

    def run(self, st):
        lib, s, d = self.lib, self.s, self.draft
        B, n_q = s.B, s.n_q
        tok, hin = self.tok0, self.g0
        for j in range(2):
            lib.specexit_draft_step(d.desc, d.w, d.view, B, tok, hin, self.pos[j], self.hout[j], self.nt[j], self.sr[j],
                                    self.sg[j], d.ws, stream=st)
            tok, hin = self.nt[j], self.hout[j]
        lib.specexit_verify_attn(self.tview, B, n_q, s.Hq, self.q, self.ctx, None, s.d ** -0.5, self.attn, self.ws_attn,
                                 stream=st)
        lib.specexit_lmhead_argmax(self.dt, B * n_q, s.D, s.V, 0, self.hid, self.lm, self.am, workspace=self.ws_head,
                                   stream=st)
        o = self.o
        lib.specexit_accept_exit(self.cfg, B, n_q, self.block, None, self.am, self.sg[0], self.ctx, self.split,
                                 self.split.numel(), *self.state, None, o["accept_len"], self.path, o["recover_tok"],
                                 o["last_node"], o["exit_flag"], o["new_ctx_len"], stream=st)
        lib.specexit_kv_compact(self.tview, 1, 0, B, n_q, self.ctx, self.path, o["accept_len"], o["last_node"],
                                self.hid.reshape(B, n_q, s.D), s.D, self.g_next, stream=st)

    def outputs(self):
        torch.cuda.synchronize()
        out = {n: H.host(v) for n, v in self.o.items()}
        out.update(nt0=H.host(self.nt[0]), nt1=H.host(self.nt[1]), sig=H.host(self.sg[0]), hout=H.host(self.hout[1]),
                   attn=H.host(self.attn), am=H.host(self.am), path=H.host(self.path), g_next=H.host(self.g_next),
                   ewma=H.host(self.state[0]), thinking=H.host(self.state[2]), target_k=H.host(self.tkeep[0]))
        return out


def oracle_round(shape, h, exit_kw):
    """The round DeviceRound.run makes, on the host: two chained draft steps, verification attention,
    LM-head argmax, acceptance / exit on the generated block, cache compaction."""
    s = shape
    B, n_q = s.B, s.n_q
    store = lambda a: gen.store(s, np.asarray(a, np.float32))
    dims = H.oracle_dims(s)
    dkv, tkv, L, case = h["dkv"], h["tkv"], h["L"], h["case"]
    kc, vc = dkv.k.astype(np.float64), dkv.v.astype(np.float64)
    o0 = O.draft_step(dims, h["w"], kc, vc, h["tok0"], h["g0"], L, store=store)
    o1 = O.draft_step(dims, h["w"], kc, vc, o0["next_tok"].astype(np.int32), store(o0["hidden_out"]), L + 1, store=store)
    attn = O.verify_attn(h["q"], tkv.k, tkv.v, L)
    am, z, _ = O.lmhead_argmax(h["hid"], h["lm"])
    ewma, n_obs, thinking = np.zeros((B, 3)), np.zeros(B, np.int32), np.ones(B, np.int32)
    o = O.accept_exit(O.ExitCfg(**exit_kw), case.block_tok, None, am.reshape(B, n_q), o0["sig"].astype(np.float32), L,
                      case.split_tok, ewma, n_obs, thinking)
    tk, tv, g_next = O.kv_compact(tkv.k.copy(), tkv.v.copy(), L, o["accept_path"], o["accept_len"],
                                  block_hidden=h["hid"].reshape(B, n_q, s.D), last_node=o["last_node"])
    ints = dict(nt0=o0["next_tok"], nt1=o1["next_tok"], am=am, path=o["accept_path"], thinking=thinking,
                **{n: o[n] for n in ("accept_len", "recover_tok", "last_node", "exit_flag", "new_ctx_len")})
    floats = dict(sig=o0["sig"], hout=o1["hidden_out"], attn=attn, ewma=ewma)
    exact = dict(g_next=g_next, target_k=tk)          # copies of input bytes
    gaps = dict(step0=O.top2_gap(o0["logits"]), step1=O.top2_gap(o1["logits"]), lm=O.top2_gap(z),
                h0=o0["h_final"], h1=o1["h_final"], z0=o0["logits"], z1=o1["logits"])
    return ints, floats, exact, gaps


def forced_inputs(shape, seed, gap=0.05):
    """Weights whose draft argmaxes (both steps) and LM-head argmaxes have a top-2 gap above `gap` in the
    oracle's logits.  A bump for the second step can move the first one's logits, hence the iteration."""
    w, lm = gen.draft_weights(shape, seed), gen.lm_head(shape, seed)
    hid = gen.hidden_rows(shape, shape.B * shape.n_q, seed)
    lm, _, _ = H.force_gap(hid, lm, shape.V, gap, shape)
    L = gen.context_lengths(shape, seed)
    h = dict(w=w, L=L, lm=lm, tok0=gen.token_ids(shape, shape.B, seed), g0=gen.hidden_rows(shape, shape.B, seed, stream=18),
             q=gen.queries(shape, seed), hid=hid, case=gen.accept_case(shape, seed, p_split=1.0),
             dkv=gen.kv_cache(shape, L, shape.n_q + 2, seed, stream=17), tkv=gen.kv_cache(shape, L, shape.n_q + 2, seed))
    kw = dict(thr_conf=0.0, thr_prog=0.0, thr_rem=1e9, stop_think_token=h["case"].stop_think_token)
    for _ in range(12):
        _, _, _, g = oracle_round(shape, h, kw)
        head, bad = h["w"]["w_head"].copy(), 0
        for gaps, hf, z in ((g["step0"], g["h0"], g["z0"]), (g["step1"], g["h1"], g["z1"])):
            for b in np.flatnonzero(gaps < 1.2 * gap):
                bad += 1
                win = O.argmax_lowest(z[b])
                row = head[win].astype(np.float64) + (2.0 * gap - gaps[b]) * hf[b] / (hf[b] @ hf[b])
                head[win] = gen.store(shape, row.astype(np.float32))
        if bad == 0:
            return h["w"], lm
        h["w"] = dict(h["w"], w_head=head)
    raise AssertionError("could not force the logit gaps of the round")


@pytest.mark.parametrize("dtype,B", [("f32", 2), ("bf16", 3), ("bf16", 6)])
def test_replayed_round_matches_the_oracle(dtype, B):
    """Parity of the replayed graph itself: what a replay leaves in the output buffers is compared
    with the oracle's round on the same inputs, not with other launches of the library."""
    shape = gen.scaled(gen.config(0), dtype=dtype, B=B, ctx=(100, 250))
    w, lm = forced_inputs(shape, seed=4)
    r = DeviceRound(shape, seed=4, w=w, lm=lm)
    ints, floats, exact, gaps = oracle_round(shape, r.h, r.exit_kw)
    assert min(gaps["step0"].min(), gaps["step1"].min(), gaps["lm"].min()) > 0.05
    lib = r.lib
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        r.reset()
        r.run(st)                                   # the warm-up the capture needs
        torch.cuda.synchronize()
        r.reset()
        lib.specexit_graph_begin(st)
        r.run(st)
        graph = lib.specexit_graph_end(st)
        try:
            for rep in range(2):
                print(f"  replay {rep} against the oracle", flush=True)
                for t in (r.nt[0], r.nt[1], r.am, r.attn, r.g_next, r.hout[1]):
                    t.zero_()
                r.reset()
                lib.specexit_graph_launch(graph, st)
                got = r.outputs()
                for n, ref in ints.items():
                    np.testing.assert_array_equal(got[n], np.asarray(ref).reshape(got[n].shape), err_msg=f"replay {rep}: {n}")
                for n, ref in floats.items():
                    assert H.rel_err(got[n], ref) < H.TOL[dtype], (rep, n)
                for n, ref in exact.items():
                    np.testing.assert_array_equal(got[n], np.asarray(ref, np.float32).reshape(got[n].shape), err_msg=f"replay {rep}: {n}")
        finally:
            lib.specexit_graph_destroy(graph)


def same(a, b, what):
    for n in a:
        np.testing.assert_array_equal(a[n], b[n], err_msg=f"{what}: {n}")


@pytest.mark.parametrize("dtype,B", [("f32", 2), ("bf16", 3), ("bf16", 6)])
def test_recorded_round_replays_to_the_same_bits(dtype, B):
    shape = gen.scaled(gen.config(0), dtype=dtype, B=B, ctx=(100, 250))
    r = DeviceRound(shape, seed=4)
    lib = r.lib
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        r.reset()
        r.run(st)                                   # also the warm-up the capture needs
        eager = r.outputs()
        r.reset()
        torch.cuda.synchronize()
        lib.specexit_graph_begin(st)
        r.run(st)
        graph = lib.specexit_graph_end(st)
        try:
            for rep in range(3):
                print(f"  replay {rep}", flush=True)
                for t in (r.nt[0], r.nt[1], r.am, r.attn, r.g_next):      # stale results must not pass for fresh ones
                    t.zero_()
                r.reset()
                lib.specexit_graph_launch(graph, st)
                same(r.outputs(), eager, f"replay {rep}")
                # other work of the process between replays: an eager call on different inputs
                lib.specexit_lmhead_argmax(r.dt, B * shape.n_q, shape.D, shape.V, 0, r.hid.flip(0).contiguous(), r.lm,
                                           torch.empty_like(r.am), workspace=r.ws_head, stream=st)
                torch.cuda.synchronize()
            # the graph reads its buffers when it runs: new inputs, same graph
            r.tok0.copy_(H.dev(gen.token_ids(shape, B, 9)))
            r.q.copy_(H.dev(gen.queries(shape, 9), shape))
            r.reset()
            lib.specexit_graph_launch(graph, st)
            replayed = r.outputs()
            r.reset()
            r.run(st)
            fresh = r.outputs()
            same(replayed, fresh, "refilled inputs")
            assert not np.array_equal(fresh["attn"], eager["attn"])
        finally:
            lib.specexit_graph_destroy(graph)


def test_graph_argument_errors():
    lib = H.sx()
    assert lib.LIB.specexit_graph_begin(None) == lib.EINVAL          # the null stream cannot be captured
    assert "null stream" in lib.last_error()
    with pytest.raises(lib.SpecExitError) as e:
        lib.specexit_graph_launch(None, torch.cuda.Stream())
    assert e.value.code == lib.EINVAL
    lib.specexit_graph_destroy(None)               # nothing to release: not an error

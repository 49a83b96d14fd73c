#!/usr/bin/env python3
"""Benchmark of the SpecExit decode-round hot path on one MI355X.

A "step" is one decode round: k x specexit_draft_step (chained), one
specexit_verify_attn call (one target layer), one specexit_lmhead_argmax over the
B*n_q block rows and one specexit_accept_exit.  Inputs are seeded synthetic tensors of
the workload's shapes, resident in HBM before the timed region.  The default workload is
the largest configuration (32B-like shapes, 16 sequences, paged caches of 8k-32k entries).
One JSON line is printed: rounds/s (value), draft tokens verified/s, the roofline of the
kernel that takes the largest share of the round (durations measured live with HIP events
the library records around its own launches; every other heavy kernel is listed beside it
with its HBM and matrix-core fractions), and the CPU oracle timed on the host cores on a
stated sample of the same workload."""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0        # dense bf16
RIDGE = MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)   # FLOP per byte where the two rooflines meet
DEFAULT_CONFIG = 4


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=DEFAULT_CONFIG,
                    help="index into the workload configurations (default: the largest one)")
    ap.add_argument("--no-graph", action="store_true", help="time eager launches instead of a HIP graph replay")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run the library's copy kernel over the head weights (both load paths) once, "
                         "so that a counter-collecting profiler run holds a kernel of known traffic")
    return ap.parse_args()


class Round:
    """Device-resident state of one decode round and the calls that run it."""

    def __init__(self, shape, seed, keep_host=False):
        import torch
        from paper_2509_24248_amd import binding as sx
        from workloads import gen
        self.torch, self.sx, self.shape = torch, sx, shape
        dt = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
        self.code = sx.BF16 if shape.dtype == "bf16" else sx.F32
        B, n_q, k = shape.B, shape.n_q, shape.k
        dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
        fdev = lambda a: dev(a).to(dt).contiguous()
        host = {}
        w = gen.draft_weights(shape, seed)
        self.wt = {n: fdev(w[n]) for n in sx.WEIGHT_NAMES}
        self.w = sx.draft_weights(self.wt)
        lm = gen.lm_head(shape, seed)
        self.lm = fdev(lm)
        L = gen.context_lengths(shape, seed)
        self.L = L
        tkv = gen.kv_cache(shape, L, n_q, seed)                       # target layer cache, block K/V in place
        dkv = gen.kv_cache(shape, L, n_q if shape.tree else k + 1, seed, stream=17)   # the draft layer's own cache (a tree keeps one entry per node)
        self.tk, self.tv = fdev(tkv.k), fdev(tkv.v)
        self.dk, self.dv = fdev(dkv.k), fdev(dkv.v)
        self.tpt = dev(tkv.page_table) if tkv.paged else None
        self.dpt = dev(dkv.page_table) if dkv.paged else None
        self.tview = sx.kv_view(self.tk, self.tv, self.tpt)
        self.dview = sx.kv_view(self.dk, self.dv, self.dpt)
        q = gen.queries(shape, seed)
        self.q = fdev(q)
        self.attn_out = torch.empty_like(self.q)
        hid = gen.hidden_rows(shape, B * n_q, seed)
        self.block_hidden = fdev(hid)                                   # target's final hidden rows of the block
        g0 = gen.hidden_rows(shape, B, seed, stream=18)
        self.g0 = fdev(g0)
        tok0 = gen.token_ids(shape, B, seed)
        self.tok0 = dev(tok0)
        if shape.tree:
            # one topology for all sequences, numbered level by level; the drafted tree and the
            # verified block share it
            par1, rank1 = gen.level_ordered_tree(shape, seed)
            parent = np.tile(par1, (B, 1)).astype(np.int32)
            mask = gen.ancestor_masks(parent)
            self.parent = dev(parent)
            self.mask = dev(mask.view(np.int64))
            self.n_draft_steps = shape.k                                # one call per tree level
        else:
            par1 = rank1 = None
            self.parent, self.mask = None, None
            self.n_draft_steps = shape.k
        case = gen.accept_case(shape, seed, parent=parent if shape.tree else None)
        self.block_tok = dev(case.block_tok)
        self.planted_len = case.planted_len
        self.split = dev(case.split_tok)
        self.S = len(case.split_tok)
        series, _ = gen.signal_series(shape, seed)
        self.ctx = dev(L.astype(np.int32))
        self.pos = [dev((L + j).astype(np.int32)) for j in range(self.n_draft_steps)]
        i32 = lambda *s: torch.empty(s, dtype=torch.int32, device="cuda")
        f32 = lambda *s: torch.empty(s, dtype=torch.float32, device="cuda")
        self.hid = [torch.empty_like(self.g0) for _ in range(2)]
        self.next_tok = [i32(B) for _ in range(self.n_draft_steps)]
        self.sig_raw = [f32(B, 3) for _ in range(self.n_draft_steps)]
        self.sig = [f32(B, 3) for _ in range(self.n_draft_steps)]
        self.target_argmax = i32(B * n_q)
        self.ewma = torch.zeros((B, 3), dtype=torch.float32, device="cuda")
        self.n_obs = torch.zeros(B, dtype=torch.int32, device="cuda")
        self.thinking = torch.ones(B, dtype=torch.int32, device="cuda")
        self.accept_len, self.recover, self.last_node, self.exit_flag, self.new_ctx = (i32(B) for _ in range(5))
        self.accept_path = i32(B, n_q)
        self.desc = sx.model_desc(self.code, shape.D, shape.Hq, shape.Hkv, shape.d, shape.I, shape.V,
                                  shape.rms_eps, shape.rope_theta, 0)
        self.cfg = sx.exit_cfg(stop_think_token=case.stop_think_token)
        ws = lambda n: torch.empty(max(n, 256), dtype=torch.uint8, device="cuda")
        self.ws_draft = ws(sx.specexit_draft_step_workspace_bytes(self.desc, self.dview, B))
        sx.specexit_workspace_prepare(self.ws_draft)      # kept to the draft step: its counters stay zero
        self.ws_attn = ws(sx.specexit_verify_attn_workspace_bytes(self.tview, B, n_q, shape.Hq))
        self.ws_head = ws(sx.specexit_lmhead_argmax_workspace_bytes(self.code, B * n_q, shape.D, shape.V, 0))
        self.scale = shape.d ** -0.5
        self.levels = self.plan_tree(par1, rank1) if shape.tree else None
        if keep_host:
            host.update(w=w, lm=lm, tkv=tkv, dkv=dkv, q=q, hid=hid, g0=g0, tok0=tok0, case=case, series=series,
                        parent=parent if shape.tree else None, mask=mask if shape.tree else None)
        self.host = host

    def plan_tree(self, parent, rank):
        """Index arrays and buffers of tree drafting, level by level: the nodes of a level that have
        children are the rows of that level's specexit_draft_tree_level call; specexit_tree_gather
        then fills the block's token row and hands tokens and hidden states to the next level."""
        torch, sx, s = self.torch, self.sx, self.shape
        from workloads import gen
        B, n, D = s.B, s.n_q, s.D
        dt = torch.bfloat16 if s.dtype == "bf16" else torch.float32
        depth = np.zeros(n, np.int64)
        for c in range(1, n):
            depth[c] = depth[parent[c]] + 1
        expanded = [any(int(parent[c]) == p for c in range(1, n)) for p in range(n)]
        masks = gen.ancestor_masks(np.asarray(parent)[None, :])[0]
        self.top_b = int(rank.max()) + 1
        i32 = lambda a: torch.from_numpy(np.asarray(a, np.int32)).cuda()
        self.block_drafted = torch.zeros((B, n), dtype=torch.int32, device="cuda")
        self.block_drafted[:, 0] = self.tok0
        levels, rows = [], [0]
        tok, hid = self.tok0.reshape(B, 1).contiguous(), self.g0.reshape(B, 1, D).contiguous()
        for level in range(int(depth.max())):
            W = len(rows)
            kids = [c for c in range(n) if depth[c] == level + 1]
            nxt = [c for c in kids if expanded[c]]
            lv = dict(level=level, W=W, tok=tok, hid=hid, node=i32(rows),
                      amask=torch.from_numpy(np.ascontiguousarray(masks[rows]).view(np.int64)).cuda(), n_blk=max(rows) + 1,
                      hout=torch.empty((B, W, D), dtype=dt, device="cuda"),
                      ct=torch.empty((B, W, self.top_b), dtype=torch.int32, device="cuda"),
                      sr=torch.empty((B, W, 3), dtype=torch.float32, device="cuda"),
                      sg=torch.empty((B, W, 3), dtype=torch.float32, device="cuda"),
                      kids=i32(kids), n_kids=len(kids), kid_src=i32([rows.index(int(parent[c])) for c in kids]),
                      kid_rank=i32([rank[c] for c in kids]),
                      kid_tok=torch.empty((B, len(kids)), dtype=torch.int32, device="cuda"),
                      n_next=len(nxt))
            # a workspace of its own per level: the prepared-workspace flag wants one shape per workspace
            lv["ws"] = torch.empty(max(sx.specexit_draft_tree_level_workspace_bytes(self.desc, self.dview, B, W, self.top_b), 256),
                                   dtype=torch.uint8, device="cuda")
            sx.specexit_workspace_prepare(lv["ws"])
            if nxt:
                lv.update(nxt=i32(nxt), nxt_src=i32([rows.index(int(parent[c])) for c in nxt]), nxt_rank=i32([rank[c] for c in nxt]))
                tok = torch.empty((B, len(nxt)), dtype=torch.int32, device="cuda")
                hid = torch.empty((B, len(nxt), D), dtype=dt, device="cuda")
                lv.update(tok_next=tok, hid_next=hid)
            levels.append(lv)
            if not nxt:
                break
            rows = nxt
        return levels

    def draft_tree(self):
        sx, s = self.sx, self.shape
        for lv in self.levels:
            sx.specexit_draft_tree_level(self.desc, self.w, self.dview, s.B, lv["W"], lv["tok"], lv["hid"], self.ctx,
                                         lv["level"], lv["node"], lv["amask"], lv["n_blk"], self.top_b, lv["hout"],
                                         lv["ct"], None, lv["sr"], lv["sg"], lv["ws"], flags=sx.FLAG_WORKSPACE_PREPARED)
            sx.specexit_tree_gather(self.code, s.B, lv["W"], self.top_b, lv["n_kids"], s.D, s.n_q, lv["kid_src"],
                                    lv["kid_rank"], lv["kids"], lv["ct"], lv["hout"], lv["kid_tok"], None, self.block_drafted)
            if lv["n_next"]:
                sx.specexit_tree_gather(self.code, s.B, lv["W"], self.top_b, lv["n_next"], s.D, s.n_q, lv["nxt_src"],
                                        lv["nxt_rank"], lv["nxt"], lv["ct"], lv["hout"], lv["tok_next"], lv["hid_next"], None)

    def run(self):
        sx, s = self.sx, self.shape
        tok, hin = self.tok0, self.g0
        if self.levels is not None:
            self.draft_tree()
        for j in range(0 if self.levels is not None else self.n_draft_steps):
            hout = self.hid[j & 1]
            sx.specexit_draft_step(self.desc, self.w, self.dview, s.B, tok, hin, self.pos[j], hout,
                                   self.next_tok[j], self.sig_raw[j], self.sig[j], self.ws_draft,
                                   flags=sx.FLAG_WORKSPACE_PREPARED)
            tok, hin = self.next_tok[j], hout
        sx.specexit_verify_attn(self.tview, s.B, s.n_q, s.Hq, self.q, self.ctx, self.mask, self.scale,
                                self.attn_out, self.ws_attn)
        sx.specexit_lmhead_argmax(self.code, s.B * s.n_q, s.D, s.V, 0, self.block_hidden, self.lm,
                                  self.target_argmax, workspace=self.ws_head)
        sig0 = self.sig[0] if self.levels is None else self.levels[0]["sg"]      # [B, 3] either way (the root level has one row)
        sx.specexit_accept_exit(self.cfg, s.B, s.n_q, self.block_tok, self.parent, self.target_argmax,
                                sig0, self.ctx, self.split, self.S, self.ewma, self.n_obs, self.thinking, None,
                                self.accept_len, self.accept_path, self.recover, self.last_node, self.exit_flag,
                                self.new_ctx)


def plant_acceptance(rnd: Round):
    """Rewrite the block's draft tokens so that, against the argmaxes the LM head really produces for the
    block's hidden rows, each sequence accepts the generator's planted number of drafts (a root path of
    lowest-index children) and the next one differs.  Input preparation, outside every timed region."""
    torch, s = rnd.torch, rnd.shape
    am = rnd.target_argmax.cpu().numpy().reshape(s.B, s.n_q)
    tok = rnd.block_tok.cpu().numpy().copy()
    par = rnd.parent.cpu().numpy() if rnd.parent is not None else np.tile(np.arange(-1, s.n_q - 1), (s.B, 1))
    for b in range(s.B):
        cur = 0
        for step in range(int(rnd.planted_len[b]) + 1):
            kids = [c for c in range(1, s.n_q) if par[b, c] == cur]
            for c in kids:                                   # nobody matches by accident
                if tok[b, c] == am[b, cur]:
                    tok[b, c] = (tok[b, c] + 1) % (s.V - 1)
            if not kids or step == int(rnd.planted_len[b]):
                break
            tok[b, kids[0]] = am[b, cur]
            cur = kids[0]
    rnd.block_tok.copy_(torch.from_numpy(tok).cuda())


def cpu_baseline(rnd: Round):
    """The oracle, as it stands, on the same inputs and the host cores.  Small workloads: one
    full round.  Large ones: a stated sample of the round's parts, each scaled to the whole
    (the oracle walks rows, queries and heads one by one, so its time is linear in them).
    Returns (seconds per round, description of the sample)."""
    from oracle import specexit_oracle as O
    from workloads import gen
    s, h = rnd.shape, rnd.host
    store = lambda a: gen.store(s, a.astype(np.float32))
    dims = O.DraftDims(s.D, s.Hq, s.Hkv, s.d, s.V, s.rms_eps, s.rope_theta)
    c = h["case"]
    dkv, tk = h["dkv"], h["tkv"]
    if s.index <= 1:
        t0 = time.perf_counter()
        kc, vc = dkv.k.astype(np.float64), dkv.v.astype(np.float64)
        tok, g, sig0 = h["tok0"], h["g0"], None
        for j in range(rnd.n_draft_steps):
            out = O.draft_step(dims, h["w"], kc, vc, tok, g, rnd.L + j, dkv.page_table if dkv.paged else None,
                               dkv.page_size, store=store)
            tok, g = out["next_tok"], store(out["hidden_out"])
            sig0 = out["sig"] if sig0 is None else sig0
        O.verify_attn(h["q"], tk.k, tk.v, rnd.L, h["mask"], rnd.scale, tk.page_table if tk.paged else None, tk.page_size)
        am, _, _ = O.lmhead_argmax(h["hid"], h["lm"])
        O.accept_exit(O.ExitCfg(stop_think_token=c.stop_think_token), c.block_tok, h["parent"],
                      am.reshape(s.B, s.n_q), sig0, rnd.L, c.split_tok, np.zeros((s.B, 3)), np.zeros(s.B, np.int32),
                      np.ones(s.B, np.int32))
        sec = time.perf_counter() - t0
        return sec, f"one full round of the same workload and inputs ({sec:.1f} s of numpy float64)"
    # ---- draft forward: the first row of the first step (the cache is read in place: float32 values
    # of the storage type; the row's own entry is written into it)
    n_sample = min(6, s.B)
    t0 = time.perf_counter()
    out = O.draft_step(dims, h["w"], dkv.k, dkv.v, h["tok0"][:n_sample], h["g0"][:n_sample], rnd.L[:n_sample],
                       dkv.page_table if dkv.paged else None, dkv.page_size, store=store)
    t_rows = time.perf_counter() - t0
    t_row = t_rows / n_sample
    n_rows = s.B * (sum(lv["W"] for lv in rnd.levels) if s.tree else rnd.n_draft_steps)
    # ---- verification attention: a sample of (sequence, query, head) outputs, scaled by visible keys
    r = np.random.default_rng(7)
    only = [(int(r.integers(s.B)), int(r.integers(s.n_q)), int(r.integers(s.Hq))) for _ in range(256)]
    t0 = time.perf_counter()
    O.verify_attn(h["q"], tk.k, tk.v, rnd.L, h["mask"], rnd.scale, tk.page_table if tk.paged else None, tk.page_size, only)
    t_attn_s = time.perf_counter() - t0
    keys_all = float((rnd.L.astype(np.int64) + s.n_q).sum()) * s.n_q * s.Hq
    keys_s = float(sum(int(rnd.L[b]) + s.n_q for b, _, _ in only))
    # ---- LM head over all block rows, acceptance and exit rule over all sequences
    t0 = time.perf_counter()
    am, _, _ = O.lmhead_argmax(h["hid"], h["lm"])
    O.accept_exit(O.ExitCfg(stop_think_token=c.stop_think_token), c.block_tok, h["parent"],
                  am.reshape(s.B, s.n_q), np.resize(out["sig"], (s.B, 3)), rnd.L, c.split_tok, np.zeros((s.B, 3)),
                  np.zeros(s.B, np.int32), np.ones(s.B, np.int32))
    t_head = time.perf_counter() - t0
    sec = t_row * n_rows + t_attn_s * keys_all / keys_s + t_head
    what = (f"measured {t_rows + t_attn_s + t_head:.1f} s of numpy float64: {n_sample} of the {n_rows} draft-forward rows of the round "
            f"({t_rows:.1f} s, scaled by {n_rows / n_sample:.1f}), {len(only)} of the {s.B * s.n_q * s.Hq} verification-attention outputs "
            f"({t_attn_s:.1f} s, scaled by visible keys x{keys_all / keys_s:.0f}), the whole LM head and accept/exit ({t_head:.1f} s); "
            f"extrapolated round: {sec:.0f} s")
    return sec, what


def threads_used():
    try:
        from threadpoolctl import threadpool_info
        n = [p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"]
        if n:
            return int(max(n))
    except Exception:
        pass
    return int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))


def stored_traffic(kernel_key, shape_name):
    """HBM bytes per launch of a kernel from the committed counter summary (FETCH_SIZE + WRITE_SIZE
    runs of this same command, scaled by the copy probe), if present."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{kernel_key}_{shape_name}.txt")
    try:
        with open(path) as fh:
            for line in fh:
                if line.startswith("bytes_per_launch"):
                    return int(line.split()[1])
    except Exception:
        pass
    return None


def round_bytes(shape, rnd, n_steps, rows, draft_keys, keys_ctx):
    """Algorithmic HBM bytes of one round: per draft launch the layer's and the head's weights and the
    draft cache; once the target layer's cache and the LM head."""
    e = 2 if shape.dtype == "bf16" else 4
    D, Hd, Hk, I, V = shape.D, shape.Hq * shape.d, shape.Hkv * shape.d, shape.I, shape.V
    layer = e * (2 * D * D + D * Hd + 2 * D * Hk + Hd * D + 3 * D * I)
    per_step = layer + e * (V + 3) * D + 2 * e * shape.Hkv * shape.d * draft_keys
    return n_steps * per_step + 2 * e * shape.Hkv * shape.d * (keys_ctx + shape.B * shape.n_q) + e * V * D


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one MI355X only: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch
    from workloads import gen
    from paper_2509_24248_amd import binding as sx
    assert torch.cuda.is_available(), "a GPU is required"
    torch.cuda.set_device(0)
    shape = gen.config(args.config)
    want_cpu = not args.no_cpu_baseline
    rnd = Round(shape, args.seed, keep_host=want_cpu)
    stream = torch.cuda.current_stream()

    for _ in range(max(args.warmup, 1)):
        rnd.run()
    torch.cuda.synchronize()
    plant_acceptance(rnd)
    if args.copy_probe:
        src = rnd.wt["w_head"]
        dst = torch.empty_like(src)
        nbytes = (src.numel() * src.element_size()) // 16 * 16
        for nt in (False, True):
            sx.specexit_copy_probe(src, dst, nbytes, nt)
        torch.cuda.synchronize()
        del dst

    # ---- eager leg with per-kernel events: durations of the heavy kernels, live
    K = args.steps
    n_steps = rnd.n_draft_steps if rnd.levels is None else len(rnd.levels)
    mk = lambda n: [torch.cuda.Event(enable_timing=True) for _ in range(n)]
    prof = {"draft_head_gemm": (sx.PROF_DRAFT_HEAD_GEMM, K * n_steps), "draft_attn_split": (sx.PROF_DRAFT_ATTN, K * n_steps),
            "lmhead_gemm": (sx.PROF_LMHEAD_GEMM, K), "verify_attn_split": (sx.PROF_VERIFY_ATTN, K),
            "draft_proj_in": (sx.PROF_DRAFT_PROJ_IN, K * n_steps), "draft_proj_out": (sx.PROF_DRAFT_PROJ_OUT, K * n_steps)}
    evs = {}
    for name, (kid, n) in prof.items():
        e0, e1 = mk(n), mk(n)
        for e in e0 + e1:
            e.record(stream)                                # creates the underlying handles
        evs[name] = (e0, e1)
    torch.cuda.synchronize()
    for name, (kid, n) in prof.items():
        sx.specexit_profile_events(kid, *evs[name])
    e_start, e_stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e_start.record(stream)
    for _ in range(K):
        rnd.run()
    e_stop.record(stream)
    torch.cuda.synchronize()
    eager_ms = e_start.elapsed_time(e_stop) / K
    kernel_ms = {}
    for name, (kid, n) in prof.items():
        used = sx.specexit_profile_events_used(kid)
        sx.specexit_profile_events(kid)
        assert used == n, f"{name}: {used} of {n} event pairs were recorded"
        kernel_ms[name] = float(np.mean([a.elapsed_time(b) for a, b in zip(*evs[name])]))

    # ---- timed region for `value`: K rounds, replayed from a HIP graph unless --no-graph
    graph_ms = None
    if not args.no_graph:
        graph = None
        try:
            gstream = torch.cuda.Stream()
            gstream.wait_stream(stream)
            with torch.cuda.stream(gstream):
                rnd.run()
                torch.cuda.synchronize()
                sx.specexit_graph_begin(gstream)            # the library's own record / replay calls
                try:
                    rnd.run()
                finally:
                    graph = sx.specexit_graph_end(gstream)
                torch.cuda.synchronize()
                for _ in range(max(args.warmup, 1)):
                    sx.specexit_graph_launch(graph, gstream)
                torch.cuda.synchronize()
                g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                g0.record(gstream)
                for _ in range(K):
                    sx.specexit_graph_launch(graph, gstream)
                g1.record(gstream)
                torch.cuda.synchronize()
            graph_ms = g0.elapsed_time(g1) / K
        except Exception as exc:                                # report eager numbers if capture is refused
            print(f"[bench] HIP graph capture unavailable ({exc}); reporting eager timing", file=sys.stderr)
            graph_ms = None
        finally:
            if graph is not None:
                sx.specexit_graph_destroy(graph)
    ms = graph_ms if graph_ms is not None else eager_ms

    # ---- time per call of each export (back-to-back calls of one export, outside the timed region)
    def per_call(fn, n=20):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fn()
        torch.cuda.synchronize()
        a.record(stream)
        for _ in range(n):
            fn()
        b.record(stream)
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n
    s_ = rnd.shape
    # the verify-attention call alone re-reads a cache of a few MB .. GB: cycle through copies that
    # together exceed the 256 MB last-level cache, so that no call is served from it
    kv_alloc = (rnd.tk.numel() + rnd.tv.numel()) * rnd.tk.element_size()
    n_copies = 1 if kv_alloc >= (512 << 20) else min(64, -(-(512 << 20) // kv_alloc))
    kv_keep = [(rnd.tk.clone(), rnd.tv.clone()) for _ in range(n_copies - 1)]
    kv_views = [rnd.tview] + [sx.kv_view(k_, v_, rnd.tpt) for k_, v_ in kv_keep]
    turn = [0]

    def attn_call():
        turn[0] = (turn[0] + 1) % n_copies
        sx.specexit_verify_attn(kv_views[turn[0]], s_.B, s_.n_q, s_.Hq, rnd.q, rnd.ctx, rnd.mask, rnd.scale,
                                rnd.attn_out, rnd.ws_attn)
    calls = {
        "specexit_draft_step": per_call(lambda: sx.specexit_draft_step(
            rnd.desc, rnd.w, rnd.dview, s_.B, rnd.tok0, rnd.g0, rnd.pos[0], rnd.hid[0], rnd.next_tok[0], rnd.sig_raw[0],
            rnd.sig[0], rnd.ws_draft, flags=sx.FLAG_WORKSPACE_PREPARED)),
        "specexit_verify_attn": per_call(attn_call, n=max(20, n_copies)),
        "specexit_lmhead_argmax": per_call(lambda: sx.specexit_lmhead_argmax(
            rnd.code, s_.B * s_.n_q, s_.D, s_.V, 0, rnd.block_hidden, rnd.lm, rnd.target_argmax, workspace=rnd.ws_head)),
        "specexit_accept_exit": per_call(lambda: sx.specexit_accept_exit(
            rnd.cfg, s_.B, s_.n_q, rnd.block_tok, rnd.parent, rnd.target_argmax, rnd.sig[0], rnd.ctx, rnd.split, rnd.S,
            rnd.ewma, rnd.n_obs, rnd.thinking, None, rnd.accept_len, rnd.accept_path, rnd.recover, rnd.last_node,
            rnd.exit_flag, rnd.new_ctx)),
    }
    # after the round: cache compaction along the accepted paths of the last round (one layer here)
    calls["specexit_kv_compact"] = per_call(lambda: sx.specexit_kv_compact(
        rnd.tview, 1, 0, s_.B, s_.n_q, rnd.ctx, rnd.accept_path, rnd.accept_len, rnd.last_node, rnd.block_hidden, s_.D,
        rnd.hid[0]))
    if rnd.levels is not None:
        wide = max(rnd.levels, key=lambda lv: lv["W"])
        calls[f"specexit_draft_tree_level (W={wide['W']}, top_b={rnd.top_b})"] = per_call(lambda: sx.specexit_draft_tree_level(
            rnd.desc, rnd.w, rnd.dview, s_.B, wide["W"], wide["tok"], wide["hid"], rnd.ctx, wide["level"], wide["node"],
            wide["amask"], wide["n_blk"], rnd.top_b, wide["hout"], wide["ct"], None, wide["sr"], wide["sg"], wide["ws"],
            flags=sx.FLAG_WORKSPACE_PREPARED))
        calls["tree drafting, all levels (draft_tree_level + tree_gather)"] = per_call(rnd.draft_tree)
    n_layers = {"tiny_f32": 4, "qwen3_4b_chain": 36, "qwen3_8b_paged": 36, "tree_8b": 36, "qwen3_32b_paged": 64}[shape.name]

    # ---- algorithmic bytes and FLOPs per launch of the heavy kernels
    e = 2 if shape.dtype == "bf16" else 4
    rows = shape.B if rnd.levels is None else float(np.mean([lv["W"] for lv in rnd.levels])) * shape.B   # draft rows per launch
    keys_ctx = int(rnd.L.astype(np.int64).sum())
    pages = lambda extra: int(sum(-(-(int(l) + extra) // shape.page_size) for l in rnd.L)) if shape.paged else 0
    draft_keys = keys_ctx + shape.B * ((n_steps + 1) / 2.0 if rnd.levels is None else shape.n_q / 2.0)   # mean over the steps
    spec = {
        # weights once + fp32 rows in, bf16 rows out + one (value, index) candidate per 16-row tile
        "draft_head_gemm": dict(bytes=e * (shape.V + 3) * shape.D + e * 2 * rows * shape.D + 8 * rows * ((shape.V + 18) // 16),
                                flops=2.0 * rows * (shape.V + 3) * shape.D, launches=n_steps,
                                what="widened-head GEMM + argmax of the draft step"),
        # K and V of every cache entry once + q in, out out + page ids
        "draft_attn_split": dict(bytes=2 * e * shape.Hkv * shape.d * draft_keys + 2 * e * rows * shape.Hq * shape.d + 4 * pages(n_steps),
                                 flops=4.0 * (rows / shape.B) * shape.Hq * shape.d * draft_keys, launches=n_steps,
                                 what="split-KV attention of the draft layer over its own cache"),
        "lmhead_gemm": dict(bytes=e * shape.V * shape.D + e * shape.B * shape.n_q * shape.D + 8 * shape.B * shape.n_q * ((shape.V + 15) // 16),
                            flops=2.0 * shape.B * shape.n_q * shape.D * shape.V, launches=1,
                            what="target LM-head GEMM + argmax over the block rows"),
        "verify_attn_split": dict(bytes=2 * e * shape.Hkv * shape.d * (keys_ctx + shape.B * shape.n_q) + 2 * e * shape.B * shape.n_q * shape.Hq * shape.d + 4 * pages(shape.n_q),
                                  flops=4.0 * shape.n_q * shape.Hq * shape.d * (keys_ctx + shape.B * shape.n_q), launches=1,
                                  what="split-KV verification attention of one target layer"),
    }
    # the layer's projections as two spans of consecutive launches (the weights once; rows and split-K partial sums are small)
    qkv_cols = (shape.Hq + 2 * shape.Hkv) * shape.d
    spec["draft_proj_in"] = dict(bytes=e * (2 * shape.D * shape.D + shape.D * qkv_cols), flops=2.0 * rows * (2 * shape.D * shape.D + shape.D * qkv_cols),
                                 launches=n_steps, what="span of launches: fuse projection, q|k|v projection with rotary embedding and cache write")
    spec["draft_proj_out"] = dict(bytes=e * (shape.Hq * shape.d * shape.D + 3 * shape.D * shape.I),
                                  flops=2.0 * rows * (shape.Hq * shape.d * shape.D + 3 * shape.D * shape.I), launches=n_steps,
                                  what="span of launches: o projection, gate|up projection, SiLU gate, down projection")
    kernels = {}
    for name, sp in spec.items():
        ms_k = kernel_ms[name]
        gbs = sp["bytes"] / (ms_k * 1e-3) / 1e9
        tfl = sp["flops"] / (ms_k * 1e-3) / 1e12
        ai = sp["flops"] / sp["bytes"]
        kernels[name] = {"what": sp["what"], "avg_launch_ms": ms_k, "launches_per_round": sp["launches"],
                         "share_of_round": ms_k * sp["launches"] / eager_ms,
                         "bytes_per_launch": int(sp["bytes"]), "achieved_GBs": gbs, "frac_hbm_peak": gbs / HBM_PEAK_GBS,
                         "flops_per_launch": sp["flops"], "achieved_TFLOPs": tfl, "frac_mfma_bf16_peak": tfl / MFMA_BF16_PEAK_TFLOPS,
                         # the most the matrix cores can be used while the weights / cache stream at HBM peak
                         "mfma_ceiling_at_hbm_peak": min(1.0, ai / RIDGE),
                         "traffic_bytes_per_launch": stored_traffic(name, shape.name)}
    top = max((n for n in kernels if not n.startswith("draft_proj")), key=lambda n: kernels[n]["share_of_round"])   # single kernels only
    kt = kernels[top]
    out = {
        "metric": "verify rounds/sec (and draft tokens verified/sec) per MI355X",
        "value": 1000.0 / ms,
        "unit": "rounds/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": shape.dtype, "data": "synthetic",
        "config": {"workload": f"configs[{shape.index}] {shape.name}: B={shape.B} {'tree depth' if shape.tree else 'chain'} k={shape.k} n_q={shape.n_q} "
                               f"ctx={shape.ctx} D={shape.D} Hq/Hkv/d={shape.Hq}/{shape.Hkv}/{shape.d} V={shape.V} I={shape.I}; " +
                               ("round = k tree-drafting levels" if shape.tree else "round = k draft steps") +
                               " + 1 target-layer verify attention + LM-head argmax + accept/exit",
                   "launch": "hip-graph replay" if graph_ms is not None else "eager"},
        "draft_tokens_verified_per_s": shape.B * (shape.n_q - 1) * 1000.0 / ms,
        # tokens the planted acceptance pattern yields per round: accepted drafts + the recover token
        "accepted_tokens_per_s": float(rnd.accept_len.float().sum().item() + shape.B) * 1000.0 / ms,
        "eager_ms_per_step": eager_ms, "graph_ms_per_step": graph_ms,
        "round_bytes": {"what": "algorithmic HBM bytes of the whole round (draft layers, heads, both caches) over its time",
                        "bytes": int(round_bytes(shape, rnd, n_steps, rows, draft_keys, keys_ctx)),
                        "achieved_GBs": round_bytes(shape, rnd, n_steps, rows, draft_keys, keys_ctx) / (ms * 1e-3) / 1e9},
        "roofline": {"kernel": f"{top}: {kt['what']} ({kt['share_of_round'] * 100:.0f} % of the round's time)",
                     "bound": "hbm", "achieved": kt["achieved_GBs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": kt["frac_hbm_peak"], "traffic": kt["traffic_bytes_per_launch"],
                     "bytes_per_launch": kt["bytes_per_launch"], "avg_launch_ms": kt["avg_launch_ms"]},
        "kernels": kernels,
        "other_kernels": {n: v for n, v in kernels.items() if n != top},     # everything but the roofline object's kernel
        "eager_ms_per_call": calls,
        # algorithmic bytes of one call of the three streaming exports over the per-call times above
        "eager_GBs_per_call": {
            "specexit_draft_step": sum(spec[n]["bytes"] for n in ("draft_proj_in", "draft_attn_split", "draft_proj_out", "draft_head_gemm"))
                                   / (calls["specexit_draft_step"] * 1e-3) / 1e9,
            "specexit_verify_attn": spec["verify_attn_split"]["bytes"] / (calls["specexit_verify_attn"] * 1e-3) / 1e9,
            "specexit_lmhead_argmax": spec["lmhead_gemm"]["bytes"] / (calls["specexit_lmhead_argmax"] * 1e-3) / 1e9},
        "per_call_note": f"back-to-back calls of one export; verify_attn cycles through {n_copies} copies of the KV cache "
                         f"({n_copies * kv_alloc / 1e6:.0f} MB in all)" +
                         (" so that no call is served from the 256 MB last-level cache" if n_copies * kv_alloc >= (512 << 20)
                          else ": small enough to stay in the 256 MB last-level cache, a cache-resident figure"),
        "projection": {"what": "verify attention call time x target layers (the round above holds one target layer's attention "
                               "and no target MLP / projection GEMMs)", "n_layers": n_layers,
                       "verify_attn_ms_all_layers": calls["specexit_verify_attn"] * n_layers},
    }
    if want_cpu:
        sec, what = cpu_baseline(rnd)
        out["cpu_baseline"] = {"value": 1.0 / sec, "unit": "rounds/s", "cores": threads_used(), "kind": "oracle",
                               "sample": what}
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out))


if __name__ == "__main__":
    main()

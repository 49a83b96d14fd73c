"""Test-side plumbing: numpy inputs -> device tensors -> C-ABI calls -> numpy outputs.

The same seeded arrays (workloads.gen) go to the oracle as float values and to
the HIP library in the configuration's storage type."""
from __future__ import annotations

import numpy as np
import torch

from oracle import specexit_oracle as O
from workloads import gen

TOL = {"f32": 1e-4, "bf16": 2e-2}      # max abs error relative to max(|ref|_inf, 1)


def sx():
    from paper_2509_24248_amd import binding
    return binding


def tdtype(shape):
    return torch.bfloat16 if shape.dtype == "bf16" else torch.float32


def dev(x, shape=None, dtype=None):
    """numpy -> cuda tensor; float arrays go to the storage type (values are representable)."""
    x = np.ascontiguousarray(x)
    if x.dtype == np.uint64:
        return torch.from_numpy(x.view(np.int64)).cuda()
    t = torch.from_numpy(x).cuda()
    if x.dtype.kind == "f":
        t = t.to(dtype if dtype is not None else tdtype(shape))
    return t.contiguous()


def host(t):
    return t.detach().float().cpu().numpy() if t.dtype in (torch.bfloat16, torch.float32) else t.cpu().numpy()


def rel_err(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.max(np.abs(np.asarray(got, dtype=np.float64) - ref)) / max(float(np.max(np.abs(ref))), 1.0))


def workspace(nbytes):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda")


class Guarded:
    """Output buffers with canary regions: every buffer handed to the library sits between two
    512-byte pads filled with a byte pattern; check() fails if a kernel wrote outside its output."""
    PAD, BYTE = 512, 0xA5

    def __init__(self):
        self.bufs = []

    def empty(self, shape, dtype):
        shape = tuple(int(x) for x in (shape if isinstance(shape, (tuple, list)) else (shape,)))
        esz = torch.empty((), dtype=dtype).element_size()
        nbytes = int(np.prod(shape)) * esz
        body = (nbytes + 255) // 256 * 256
        raw = torch.full((self.PAD + body + self.PAD,), self.BYTE, dtype=torch.uint8, device="cuda")
        view = raw[self.PAD:self.PAD + nbytes].view(dtype).reshape(shape)
        self.bufs.append((raw, nbytes))
        return view

    def empty_like(self, t):
        return self.empty(tuple(t.shape), t.dtype)

    def check(self):
        torch.cuda.synchronize()
        for raw, nbytes in self.bufs:
            assert bool((raw[:self.PAD] == self.BYTE).all()), "a kernel wrote in front of its output buffer"
            assert bool((raw[self.PAD + nbytes:] == self.BYTE).all()), "a kernel wrote behind its output buffer"


# ----------------------------------------------------------------------------- attention

def kv_view_of(shape, kv: gen.KVCache):
    lib = sx()
    k, v = dev(kv.k, shape), dev(kv.v, shape)
    pt = dev(kv.page_table) if kv.paged else None
    return lib.kv_view(k, v, pt), (k, v, pt)


def gpu_verify_attn(shape, kv, q, ctx_len, mask, scale=None):
    lib = sx()
    view, keep = kv_view_of(shape, kv)
    B, n_q, Hq, d = q.shape
    qd = dev(q, shape)
    guard = Guarded()
    out = guard.empty_like(qd)
    ws = workspace(lib.specexit_verify_attn_workspace_bytes(view, B, n_q, Hq))
    lib.specexit_verify_attn(view, B, n_q, Hq, qd, dev(ctx_len.astype(np.int32)),
                             None if mask is None else dev(mask), d ** -0.5 if scale is None else scale, out, ws)
    guard.check()
    return host(out)


def oracle_verify_attn(kv, q, ctx_len, mask, scale=None, only=None):
    return O.verify_attn(q, kv.k, kv.v, ctx_len, mask, scale, kv.page_table if kv.paged else None, kv.page_size, only)


# ----------------------------------------------------------------------------- LM head

def force_gap(hidden, w, V, gap=0.05, shape=None, max_iter=20):
    """Raise the winner's weight row until every hidden row has a top-2 logit gap > gap
    (done with the oracle's logits; the bump keeps the storage type)."""
    w = w.copy()
    h64 = hidden.astype(np.float64)
    for _ in range(max_iter):
        am, z, _ = O.lmhead_argmax(hidden, w[:V])
        g = O.top2_gap(z)
        bad = np.flatnonzero(g < gap * 1.2)
        if bad.size == 0:
            return w, am, z
        for r in bad:
            bump = (gap * 2.0 - g[r]) * h64[r] / (h64[r] @ h64[r])
            new = w[am[r]].astype(np.float64) + bump
            w[am[r]] = gen.store(shape, new.astype(np.float32)) if shape is not None else new
    raise AssertionError("could not force the logit gap")


def gpu_lmhead(shape, hidden, w, n_extra=0, want_logits=True):
    lib = sx()
    M, D = hidden.shape
    V = w.shape[0] - n_extra
    dt = lib.BF16 if shape.dtype == "bf16" else lib.F32
    hd, wd = dev(hidden, shape), dev(w, shape)
    guard = Guarded()
    am = guard.empty(M, torch.int32)
    mx = guard.empty(M, torch.float32)
    ex = guard.empty((M, max(n_extra, 1)), torch.float32)
    lg = guard.empty((M, V), torch.float32) if want_logits else None
    ws = workspace(lib.specexit_lmhead_argmax_workspace_bytes(dt, M, D, V, n_extra))
    lib.specexit_lmhead_argmax(dt, M, D, V, n_extra, hd, wd, am, mx, ex if n_extra else None, lg, ws)
    guard.check()
    return host(am), host(mx), host(ex)[:, :n_extra], (host(lg) if want_logits else None)


# ----------------------------------------------------------------------------- draft step

class GpuDraft:
    """Device-resident draft model + cache for repeated specexit_draft_step calls."""

    def __init__(self, shape, w, kv: gen.KVCache, rem_activation=0):
        lib = sx()
        self.lib, self.shape = lib, shape
        dt = lib.BF16 if shape.dtype == "bf16" else lib.F32
        self.desc = lib.model_desc(dt, shape.D, shape.Hq, shape.Hkv, shape.d, shape.I, shape.V, shape.rms_eps,
                                   shape.rope_theta, rem_activation)
        self.wt = {n: dev(w[n], shape) for n in lib.WEIGHT_NAMES}
        self.w = lib.draft_weights(self.wt)
        self.view, self.keep = kv_view_of(shape, kv)
        self.ws = workspace(lib.specexit_draft_step_workspace_bytes(self.desc, self.view, shape.B))
        assert self.ws.numel() > 256, lib.last_error()

    def step(self, tok, hidden_in, pos, flags=0):
        shape, B = self.shape, self.shape.B
        hin = dev(hidden_in, shape)
        guard = Guarded()
        hout = guard.empty_like(hin)
        nt = guard.empty(B, torch.int32)
        sr = guard.empty((B, 3), torch.float32)
        sg = guard.empty((B, 3), torch.float32)
        self.lib.specexit_draft_step(self.desc, self.w, self.view, B, dev(tok.astype(np.int32)), hin,
                                     dev(pos.astype(np.int32)), hout, nt, sr, sg, self.ws, flags=flags)
        guard.check()
        return {"hidden_out": host(hout), "next_tok": host(nt), "sig_raw": host(sr), "sig": host(sg)}

    def cache(self):
        return host(self.keep[0]), host(self.keep[1])

    def tree(self, tok0, g0, ctx_len, parent, rank, top_b):
        """Draft a whole tree level by level through specexit_draft_tree_level / specexit_tree_gather.
        Only index arrays are prepared here; every value comes out of the library.  tok0, g0 and
        ctx_len may be device tensors (outputs of earlier calls), which are then used as they are."""
        lib, shape, B = self.lib, self.shape, self.shape.B
        n = len(parent)
        depth = O.tree_depths(parent)
        expanded = [any(int(parent[c]) == p for c in range(1, n)) for p in range(n)]
        masks = gen.ancestor_masks(np.asarray(parent)[None, :])[0]
        i32 = lambda a: dev(np.asarray(a, np.int32))
        dt = lib.BF16 if shape.dtype == "bf16" else lib.F32
        Wmax = max(sum(1 for c in range(n) if depth[c] == l and expanded[c]) for l in range(int(depth.max()) + 1))
        ws = workspace(lib.specexit_draft_tree_level_workspace_bytes(self.desc, self.view, B, Wmax, top_b))
        assert ws.numel() > 256, lib.last_error()
        as_i32 = lambda a: a if torch.is_tensor(a) else i32(a)
        ctx, tok0 = as_i32(ctx_len), as_i32(tok0)
        block_tok = torch.zeros((B, n), dtype=torch.int32, device="cuda")
        block_tok[:, 0] = tok0
        tok = tok0.reshape(B, 1).contiguous()
        hid = (g0 if torch.is_tensor(g0) else dev(g0, shape)).reshape(B, 1, shape.D).contiguous()
        rows = [0]
        res = {"hidden_out": {}, "cand_tok": {}, "cand_logit": {}, "sig_raw": {}, "sig": {}, "sig_dev": {}}
        for level in range(int(depth.max())):
            W = len(rows)
            hout = torch.empty((B, W, shape.D), dtype=tdtype(shape), device="cuda")
            ct = torch.empty((B, W, top_b), dtype=torch.int32, device="cuda")
            cl = torch.empty((B, W, top_b), dtype=torch.float32, device="cuda")
            sr = torch.empty((B, W, 3), dtype=torch.float32, device="cuda")
            sg = torch.empty((B, W, 3), dtype=torch.float32, device="cuda")
            lib.specexit_draft_tree_level(self.desc, self.w, self.view, B, W, tok, hid, ctx, level, i32(rows),
                                          dev(masks[rows]), max(rows) + 1, top_b, hout, ct, cl, sr, sg, ws)
            torch.cuda.synchronize()
            for j, c in enumerate(rows):
                res["hidden_out"][c], res["cand_tok"][c], res["cand_logit"][c] = host(hout[:, j]), host(ct[:, j]), host(cl[:, j])
                res["sig_raw"][c], res["sig"][c] = host(sr[:, j]), host(sg[:, j])
                res["sig_dev"][c] = sg[:, j].contiguous()
            kids = [c for c in range(n) if depth[c] == level + 1]
            src = [rows.index(int(parent[c])) for c in kids]
            all_tok = torch.empty((B, len(kids)), dtype=torch.int32, device="cuda")
            lib.specexit_tree_gather(dt, B, W, top_b, len(kids), shape.D, n, i32(src), i32([rank[c] for c in kids]),
                                     i32(kids), ct, hout, all_tok, None, block_tok)
            nxt = [c for c in kids if expanded[c]]
            if not nxt:
                break
            src = [rows.index(int(parent[c])) for c in nxt]
            tok = torch.empty((B, len(nxt)), dtype=torch.int32, device="cuda")
            hid = torch.empty((B, len(nxt), shape.D), dtype=tdtype(shape), device="cuda")
            lib.specexit_tree_gather(dt, B, W, top_b, len(nxt), shape.D, n, i32(src), i32([rank[c] for c in nxt]),
                                     i32(nxt), ct, hout, tok, hid, None)
            rows = nxt
        torch.cuda.synchronize()
        res["block_tok"], res["block_tok_dev"] = host(block_tok), block_tok
        return res


def oracle_dims(shape):
    return O.DraftDims(shape.D, shape.Hq, shape.Hkv, shape.d, shape.V, shape.rms_eps, shape.rope_theta)


def oracle_tree(shape, w, kv, tok0, g0, L, parent, rank):
    kc, vc = kv.k.astype(np.float64), kv.v.astype(np.float64)
    out = O.draft_tree(oracle_dims(shape), w, kc, vc, tok0, g0, L, parent, rank, kv.page_table if kv.paged else None,
                       kv.page_size, store=lambda a: gen.store(shape, np.asarray(a, np.float32)))
    return out, kc, vc


def force_tree_gap(shape, w, kv, tok0, g0, L, parent, rank, top_b, gap=0.05, max_iter=12):
    """Bump w_head until, at every expanded node, the top_b + 1 best logits lie more than `gap`
    apart (with the oracle's logits), so that float32 / bf16 arithmetic cannot reorder them."""
    w = dict(w)
    V = shape.V
    for _ in range(max_iter):
        out, kc, vc = oracle_tree(shape, w, kv, tok0, g0, L, parent, rank)
        head = w["w_head"].copy()
        bad = 0
        for b in range(shape.B):
            for c in np.flatnonzero(out["expanded"]):
                z = out["logits"][b, c]
                order = O.top_b_lowest(z, top_b + 1)
                gaps = z[order[:-1]] - z[order[1:]]
                if gaps.min() >= gap * 1.2:
                    continue
                bad += 1
                h = out["h_final"][b, c]
                inc = 0.0                                # raise only what is missing, from the bottom up
                for r in range(top_b - 1, -1, -1):
                    inc += max(0.0, 1.6 * gap - (z[order[r]] - z[order[r + 1]]))
                    if inc > 0.0:
                        # spend the bump on the 64 largest components of h: spread over all of
                        # them it would be below the storage type's rounding step
                        big = np.argsort(-np.abs(h))[:64]
                        row = head[order[r]].astype(np.float64)
                        row[big] += inc * h[big] / (h[big] @ h[big])
                        head[order[r]] = gen.store(shape, row.astype(np.float32))
        if bad == 0:
            return w, out, kc, vc
        w["w_head"] = head
    raise AssertionError("could not force the logit gaps of the tree")


def oracle_draft_rows(shape, w, kv, tok, g, pos, rows, kc=None, vc=None, progress=None):
    """The oracle's draft forward for a sample of the step's rows (the rows of a step are independent:
    row b reads and writes sequence b's cache only).  Returns {row: result of the oracle's row routine};
    the cache arrays (kc, vc; default: kv's own, modified in place) receive the rows' new entries."""
    kc = kv.k if kc is None else kc
    vc = kv.v if vc is None else vc
    out = {}
    for b in rows:
        if progress:
            print(f"  oracle {progress}: row {b}", flush=True)
        p = int(pos[b])
        out[b] = O._draft_row(oracle_dims(shape), w, kc, vc, b, tok[b], g[b], p, p, np.arange(p + 1),
                              kv.page_table if kv.paged else None, kv.page_size,
                              lambda a: gen.store(shape, np.asarray(a, np.float32)))
    return out


def force_draft_gap(shape, w, kv, tok, g, pos, gap=0.05, rows=None):
    """Run the oracle once to get the final-normed hidden rows, then bump w_head's winners
    (rows: only these rows of the step are looked at)."""
    if rows is not None:
        res = oracle_draft_rows(shape, w, kv, tok, g, pos, rows, kv.k.copy(), kv.v.copy(), progress="gap forcing")
        out = {"h_final": np.stack([res[b]["h_final"] for b in rows])}
    else:
        kc, vc = kv.k.astype(np.float64), kv.v.astype(np.float64)
        out = O.draft_step(oracle_dims(shape), w, kc, vc, tok, g, pos, kv.page_table if kv.paged else None,
                           kv.page_size, store=lambda a: gen.store(shape, a.astype(np.float32)))
    head = w["w_head"]
    V = shape.V
    new_tok_rows, _, _ = force_gap(out["h_final"].astype(np.float32), head[:V], V, gap, shape)
    w = dict(w)
    w["w_head"] = np.concatenate([new_tok_rows, head[V:]], axis=0)
    return w


# ----------------------------------------------------------------------------- controller

def gpu_accept_exit(cfg_kwargs, block_tok, parent, target_argmax, sig, ctx_len, split_tok, state):
    """state = (ewma [B,3] f32, n_obs [B] i32, is_thinking [B] i32[, smooth_state [B,48] f32]) device
    tensors, updated in place."""
    lib = sx()
    B, n_q = block_tok.shape
    cfg = lib.exit_cfg(**cfg_kwargs)
    i32 = lambda a: dev(np.asarray(a, dtype=np.int32))
    guard = Guarded()
    outs = {k: guard.empty(B, torch.int32)
            for k in ("accept_len", "recover_tok", "last_node", "exit_flag", "new_ctx_len")}
    outs["accept_path"] = guard.empty((B, n_q), torch.int32)
    split = i32(split_tok) if len(split_tok) else None
    lib.specexit_accept_exit(cfg, B, n_q, i32(block_tok), None if parent is None else i32(parent),
                             i32(target_argmax), dev(np.asarray(sig, np.float32), dtype=torch.float32),
                             i32(ctx_len), split, len(split_tok), state[0], state[1], state[2],
                             state[3] if len(state) > 3 else None,
                             outs["accept_len"], outs["accept_path"], outs["recover_tok"], outs["last_node"],
                             outs["exit_flag"], outs["new_ctx_len"])
    guard.check()
    return {k: host(v) for k, v in outs.items()}


def gpu_state(B, history=False):
    st = (torch.zeros((B, 3), dtype=torch.float32, device="cuda"),
          torch.zeros(B, dtype=torch.int32, device="cuda"),
          torch.ones(B, dtype=torch.int32, device="cuda"))
    if history:
        st += (torch.zeros((B, sx().SMOOTH_WORDS), dtype=torch.float32, device="cuda"),)
    return st

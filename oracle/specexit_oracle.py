"""CPU oracle for one SpecExit decode round.  TEST INFRASTRUCTURE ONLY.

Plain, slow, obviously-correct numpy code in float64: it is what the GPU
library is checked against, it shares no code with it, and only the tests, the
smoke check and the benchmark's host-baseline leg may import it.  The product
path never routes through this file.

What is computed (SpecExit, arXiv 2509.24248):

* draft_step      - the draft ("MTP") forward whose output projection is widened
                    by three signal rows, Sec. 3.1 Eq. 1; signal activations as
                    used by the training losses, Sec. 3.2 Eqs. 3-5.
* draft_tree      - the same forward run over a candidate tree of fixed topology
                    (children = the parent's top-ranked tokens), producing the
                    block that tree attention verifies, Alg. 1.
* verify_attn     - the target's attention over [last accepted token | draft
                    candidates] with a tree (ancestor) mask: the target pass
                    of Alg. 1 that verifies the drafted block.
* lmhead_argmax   - target logits -> next token per block position (greedy),
                    Alg. 1, the target's own token at each block position.
* kv_compact      - what the round leaves behind for the next one: the accepted
                    path's K/V entries moved next to the context and the
                    hidden state of the last accepted node: the cache and
                    hidden-state update that closes a round of Alg. 1.
* accept_exit     - accepted tokens / accept length / recover token (Alg. 1),
                    EWMA smoothing (Sec. 3.3 "Signal Smoothing", Appendix
                    "Signal Smoothing" EWMA equation, alpha = 0.1; the sliding
                    window, momentum and paragraph-mean smoothers of the same
                    appendix, N = 10, as alternatives), the stop
                    thresholds (Appendix "Stop Threshold") and the step-split
                    gate with truncation (Sec. 3.3 "Stopping Conditions",
                    Alg. 1 inner if-block).

The paper fixes the widened head, the activations, the smoother, the thresholds
and the gate; it does not spell out the draft layer, which follows the
EAGLE-style structure named by this build's target (fuse of token embedding and
target hidden state, one pre-norm decoder layer, final norm, head).  That part
is a reading, pinned only through special cases and library building blocks:
against a trained checkpoint it is "parity unpinned" (no weights exist here).

Every method result here is the plain definition: two-pass softmax over an
explicit list of visible keys, dot products as numpy matmuls, strict '>' scans
for argmax.  The only blocking is memory management (the vocabulary is walked
in row blocks so the float64 copy of a weight matrix need not exist at once).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

F64 = np.float64


# ---------------------------------------------------------------------------
# stage 2: verification attention  (Alg. 1, "tree attention")
# ---------------------------------------------------------------------------

def chain_mask(n_q: int) -> np.ndarray:
    """Block-causal mask of a chain: query i sees block entries 0..i."""
    return np.array([(1 << (i + 1)) - 1 for i in range(n_q)], dtype=np.uint64)


def visible_positions(ctx_len: int, mask_row: int, n_q: int) -> np.ndarray:
    """Cache positions one query attends to: the whole context [0, L) and the
    block entries L+j whose bit j is set in the query's ancestor mask."""
    blk = [ctx_len + j for j in range(n_q) if (int(mask_row) >> j) & 1]
    return np.concatenate([np.arange(ctx_len, dtype=np.int64), np.array(blk, dtype=np.int64)])


def softmax_two_pass(s: np.ndarray) -> np.ndarray:
    m = np.max(s)
    e = np.exp(s - m)
    return e / np.sum(e)


def _kv_rows(pool, page_table, page_size, b, head, positions):
    """Resolve cache positions to stored rows; contiguous [B,Hkv,L,d] or paged
    [n_pages,Hkv,page,d] with page_table[b, pos // page]."""
    if page_table is None:
        return np.asarray(pool[b, head, positions, :], dtype=F64)
    pages = page_table[b, positions // page_size]
    return np.asarray(pool[pages, head, positions % page_size, :], dtype=F64)


def verify_attn(q, k, v, ctx_len, mask=None, scale=None, page_table=None, page_size=16,
                only: Optional[Sequence] = None):
    """softmax(scale * q.K^T over the visible set) . V per (sequence, query, head).

    q [B, n_q, Hq, d]; k, v contiguous [B, Hkv, l_max, d] or paged
    [n_pages, Hkv, page_size, d] (+ page_table [B, max_pages]); ctx_len [B];
    mask [B, n_q] uint64 (None = chain).  The block's own K/V sit at cache
    positions L_b .. L_b+n_q-1.  Query head h reads KV head h // (Hq/Hkv).
    Returns out [B, n_q, Hq, d] float64 (entries not in `only` stay NaN)."""
    q = np.asarray(q)
    B, n_q, Hq, d = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    scale = 1.0 / np.sqrt(d) if scale is None else float(scale)
    out = np.full((B, n_q, Hq, d), np.nan, dtype=F64)
    triples = only if only is not None else [(b, i, h) for b in range(B)
                                             for i in range(n_q) for h in range(Hq)]
    for (b, i, h) in triples:
        row = int(mask[b, i]) if mask is not None else (1 << (i + 1)) - 1
        vis = visible_positions(int(ctx_len[b]), row, n_q)
        kk = _kv_rows(k, page_table, page_size, b, h // G, vis)
        vv = _kv_rows(v, page_table, page_size, b, h // G, vis)
        s = scale * (kk @ np.asarray(q[b, i, h], dtype=F64))
        p = softmax_two_pass(s)
        out[b, i, h] = p @ vv
    return out


# ---------------------------------------------------------------------------
# stage 3: LM head -> argmax  (Alg. 1, recover token; greedy)
# ---------------------------------------------------------------------------

def argmax_lowest(z: np.ndarray) -> int:
    """Index of the maximum with a strict '>' scan from 0 (lowest index on ties)."""
    m = np.max(z)
    return int(np.flatnonzero(z == m)[0])


def linear(x: np.ndarray, w: np.ndarray, row_block: int = 16384) -> np.ndarray:
    """x [M,K] @ w[N,K]^T in float64; w is walked in row blocks only so that its
    float64 copy stays small."""
    x = np.asarray(x, dtype=F64)
    N = w.shape[0]
    out = np.empty((x.shape[0], N), dtype=F64)
    for lo in range(0, N, row_block):
        hi = min(N, lo + row_block)
        out[:, lo:hi] = x @ np.asarray(w[lo:hi], dtype=F64).T
    return out


def lmhead_argmax(hidden, w, n_extra: int = 0):
    """z = hidden . w^T; argmax over the first V rows of w, per hidden row.

    With n_extra > 0 the last n_extra rows of w are the widened head's signal
    rows (Eq. 1): they are excluded from the argmax and returned raw.
    Returns (argmax [M] int64, logits [M, V] float64, extra [M, n_extra])."""
    z = linear(hidden, w)
    V = w.shape[0] - n_extra
    logits = z[:, :V]
    extra = z[:, V:]
    am = np.array([argmax_lowest(logits[r]) for r in range(logits.shape[0])], dtype=np.int64)
    return am, logits, extra


def top2_gap(logits: np.ndarray) -> np.ndarray:
    part = np.partition(logits, -2, axis=-1)
    return part[..., -1] - part[..., -2]


# ---------------------------------------------------------------------------
# stage 1: draft step  (Sec. 3.1 Eq. 1; Sec. 3.2 Eqs. 3-5; Alg. 1 first line)
# ---------------------------------------------------------------------------

def rmsnorm(u: np.ndarray, w: np.ndarray, eps: float) -> np.ndarray:
    u = np.asarray(u, dtype=F64)
    return u / np.sqrt(np.mean(u * u, axis=-1, keepdims=True) + eps) * np.asarray(w, dtype=F64)


def rope_rotate_half(x: np.ndarray, pos: int, theta: float) -> np.ndarray:
    """Rotary embedding on the last axis, pairing (c, c + d/2):
    angle_c = pos * theta^(-2c/d);  out_c = x_c cos - x_{c+d/2} sin,
    out_{c+d/2} = x_{c+d/2} cos + x_c sin."""
    x = np.asarray(x, dtype=F64)
    d = x.shape[-1]
    half = d // 2
    c = np.arange(half, dtype=F64)
    ang = float(pos) * theta ** (-2.0 * c / d)
    cs, sn = np.cos(ang), np.sin(ang)
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * cs - x2 * sn, x2 * cs + x1 * sn], axis=-1)


def sigmoid(t):
    return 1.0 / (1.0 + np.exp(-np.asarray(t, dtype=F64)))


def silu(t):
    t = np.asarray(t, dtype=F64)
    return t * sigmoid(t)


def signal_activations(sig_raw: np.ndarray) -> np.ndarray:
    """Raw head outputs -> signals in their natural units.

    Confidence and progress are trained through a sigmoid (Eqs. 3-4).  The
    remaining-length output is trained to equal log(1 + r) (Eq. 5), so the
    token count is expm1 of it, floored at zero."""
    sig_raw = np.asarray(sig_raw, dtype=F64)
    conf = sigmoid(sig_raw[..., 0])
    prog = sigmoid(sig_raw[..., 1])
    rem = np.maximum(0.0, np.expm1(sig_raw[..., 2]))
    return np.stack([conf, prog, rem], axis=-1)


@dataclass
class DraftDims:
    D: int
    Hq: int
    Hkv: int
    d: int
    V: int
    rms_eps: float = 1e-6
    rope_theta: float = 1e6


def top_b_lowest(z: np.ndarray, b: int) -> np.ndarray:
    """The b largest entries of z, largest first, lower index first among equals."""
    z = np.asarray(z, dtype=F64)
    order = sorted(range(len(z)), key=lambda i: (-z[i], i)) if len(z) <= 4096 else \
        np.lexsort((np.arange(len(z)), -z))
    return np.asarray(order[:b], dtype=np.int64)


def _draft_row(dims: DraftDims, w: dict, k_cache, v_cache, b, tok, g, rope_pos, slot, visible,
               page_table, page_size, store):
    """The draft forward of one row of sequence b (steps 1-5 of draft_step): the
    row's K/V are rotated for position rope_pos, stored in cache entry `slot`,
    and its query attends to the cache entries listed in `visible` (which
    include `slot`)."""
    D, Hq, Hkv, d, V = dims.D, dims.Hq, dims.Hkv, dims.d, dims.V
    G = Hq // Hkv
    e = np.asarray(w["embed"][int(tok)], dtype=F64)
    g = np.asarray(g, dtype=F64)
    x = linear(np.concatenate([e, g])[None, :], w["w_fc"])[0]
    n = rmsnorm(x, w["ln_attn"], dims.rms_eps)
    qv = linear(n[None, :], w["w_q"])[0].reshape(Hq, d)
    kv = linear(n[None, :], w["w_k"])[0].reshape(Hkv, d)
    vv = linear(n[None, :], w["w_v"])[0].reshape(Hkv, d)
    qv = rope_rotate_half(qv, rope_pos, dims.rope_theta)
    kv = rope_rotate_half(kv, rope_pos, dims.rope_theta)
    k_new = kv if store is None else store(kv)
    v_new = vv if store is None else store(vv)
    if page_table is None:
        k_cache[b, :, slot, :] = k_new
        v_cache[b, :, slot, :] = v_new
    else:
        pg = page_table[b, slot // page_size]
        k_cache[pg, :, slot % page_size, :] = k_new
        v_cache[pg, :, slot % page_size, :] = v_new
    positions = np.asarray(visible, dtype=np.int64)
    attn = np.empty(Hq * d, dtype=F64)
    for h in range(Hq):
        kk = _kv_rows(k_cache, page_table, page_size, b, h // G, positions)
        vs = _kv_rows(v_cache, page_table, page_size, b, h // G, positions)
        s = (kk @ qv[h]) / np.sqrt(d)
        attn[h * d:(h + 1) * d] = softmax_two_pass(s) @ vs
    a = x + linear(attn[None, :], w["w_o"])[0]
    m = rmsnorm(a, w["ln_mlp"], dims.rms_eps)
    act = silu(linear(m[None, :], w["w_gate"])[0]) * linear(m[None, :], w["w_up"])[0]
    y = a + linear(act[None, :], w["w_down"])[0]
    h_fin = rmsnorm(y, w["ln_final"], dims.rms_eps)
    z = linear(h_fin[None, :], w["w_head"])[0]
    return {"hidden_out": y, "h_final": h_fin, "logits": z[:V], "sig_raw": z[V:V + 3], "attn_out": attn}


def draft_step(dims: DraftDims, w: dict, k_cache, v_cache, tok, hidden_in, pos,
               page_table=None, page_size=16, store=None):
    """One draft step for B rows (one per sequence).

    1. e = embed[tok];  x = W_fc [e ; g]   (g = hidden_in: the target's final
       hidden state of the last accepted token at the first step of a round,
       the draft's own hidden_out afterwards).
    2. n = RMSNorm(x; ln_attn);  q, k, v = W_q n, W_k n, W_v n;  RoPE(q, k) at
       position pos;  k, v written into the draft's own cache at pos.
    3. causal GQA attention of q over cache positions 0..pos.
    4. a = x + W_o attn;  y = a + W_down( silu(W_gate m) * (W_up m) ),
       m = RMSNorm(a; ln_mlp).
    5. hidden_out = y;  h = RMSNorm(y; ln_final);  z = W_head h with W_head =
       [W_tok; W_conf; W_prog; W_rem]  (Eq. 1);  next_tok = argmax z[:V];
       sig_raw = z[V:V+3];  sig = activations (Eqs. 3-5).

    k_cache / v_cache are modified in place (float arrays laid out as for
    verify_attn).  `store` optionally rounds what is written to the cache to the
    storage type (the GPU keeps the cache in that type)."""
    B = len(tok)
    D, Hq, d, V = dims.D, dims.Hq, dims.d, dims.V
    hidden_out = np.empty((B, D), dtype=F64)
    logits = np.empty((B, V), dtype=F64)
    sig_raw = np.empty((B, 3), dtype=F64)
    next_tok = np.empty(B, dtype=np.int64)
    attn_out = np.empty((B, Hq * d), dtype=F64)
    h_final = np.empty((B, D), dtype=F64)
    for b in range(B):
        p = int(pos[b])
        r = _draft_row(dims, w, k_cache, v_cache, b, tok[b], hidden_in[b], p, p, np.arange(p + 1),
                       page_table, page_size, store)
        hidden_out[b], h_final[b], logits[b] = r["hidden_out"], r["h_final"], r["logits"]
        sig_raw[b], attn_out[b] = r["sig_raw"], r["attn_out"]
        next_tok[b] = argmax_lowest(r["logits"])
    return {"hidden_out": hidden_out, "next_tok": next_tok, "sig_raw": sig_raw,
            "sig": signal_activations(sig_raw), "logits": logits, "attn_out": attn_out,
            "h_final": h_final}


def tree_depths(parent) -> np.ndarray:
    depth = np.zeros(len(parent), dtype=np.int64)
    for c in range(1, len(parent)):
        depth[c] = depth[int(parent[c])] + 1
    return depth


def draft_tree(dims: DraftDims, w: dict, k_cache, v_cache, tok0, g0, ctx_len, parent, rank,
               page_table=None, page_size=16, store=None):
    """Draft a whole candidate tree of fixed topology for every sequence (the
    block that verification with tree attention consumes, Alg. 1).

    parent[c] < c is the parent of node c (node 0 = the last accepted token,
    parent -1), rank[c] says which of the parent's continuations node c holds:
    its token is the rank[c]-th most likely token (0 = argmax) of the draft's
    output at the parent.  Every node that has children is run through the
    draft forward (the row of draft_step): its inputs are its token and the
    hidden state its parent's forward produced (node 0: the target's hidden
    state g0), its rotary position is L + depth, its K/V go to draft cache
    entry L + node, and it attends to the context 0..L-1 plus the entries of
    its ancestors and itself.  Hidden states are handed from parent to child in
    the storage type (`store`).  Nodes are processed in index order, which is a
    topological order.

    Returns block_tok [B, n], hidden_out / h_final / logits / sig_raw / sig per
    expanded node (NaN rows elsewhere), and `expanded` [n] bool."""
    n = len(parent)
    B = len(tok0)
    depth = tree_depths(parent)
    children = [[c for c in range(1, n) if int(parent[c]) == p] for p in range(n)]
    expanded = np.array([len(ch) > 0 for ch in children])
    block_tok = np.zeros((B, n), dtype=np.int64)
    hidden_out = np.full((B, n, dims.D), np.nan, dtype=F64)
    h_final = np.full((B, n, dims.D), np.nan, dtype=F64)
    logits = np.full((B, n, dims.V), np.nan, dtype=F64)
    sig_raw = np.full((B, n, 3), np.nan, dtype=F64)
    keep = (lambda a: a) if store is None else store
    for b in range(B):
        L = int(ctx_len[b])
        block_tok[b, 0] = int(tok0[b])
        for c in range(n):
            if c > 0:
                p = int(parent[c])
                need = max(int(rank[k]) for k in children[p]) + 1
                block_tok[b, c] = int(top_b_lowest(logits[b, p], need)[int(rank[c])])
            if not expanded[c]:
                continue
            g = g0[b] if c == 0 else keep(hidden_out[b, int(parent[c])])
            anc, a = [], c
            while a >= 0:
                anc.append(a)
                a = int(parent[a])
            visible = list(range(L)) + [L + a for a in sorted(anc)]
            r = _draft_row(dims, w, k_cache, v_cache, b, block_tok[b, c], g, L + int(depth[c]), L + c,
                           visible, page_table, page_size, store)
            hidden_out[b, c], h_final[b, c], logits[b, c] = r["hidden_out"], r["h_final"], r["logits"]
            sig_raw[b, c] = r["sig_raw"]
    return {"block_tok": block_tok, "hidden_out": hidden_out, "h_final": h_final, "logits": logits,
            "sig_raw": sig_raw, "sig": signal_activations(sig_raw), "expanded": expanded}


# ---------------------------------------------------------------------------
# stages 4 + 5: acceptance, smoothing, exit rule  (Alg. 1; Appendix)
# ---------------------------------------------------------------------------

@dataclass
class ExitCfg:
    alpha: float = 0.1          # Appendix, EWMA
    thr_conf: float = 0.8       # Appendix "Stop Threshold", combined rule
    thr_prog: float = 0.3
    thr_rem: float = 200.0
    signal_mask: int = 0b111    # bit 0 confidence, 1 progress, 2 remaining
    smoother: int = 0           # 0 EWMA, 1 none, 2 sliding window, 3 momentum, 4 paragraph mean
    window: int = 10            # N of the sliding-window and momentum smoothers (Appendix)
    split_pick: int = 0         # 0 earliest split token in the accepted path, 1 latest
    check_root: int = 0         # also look at the block root (not an accepted draft token)
    stop_think_token: int = 0


def ewma_update(x_prev: float, s: float, alpha: float) -> float:
    """x_t = alpha s_t + (1 - alpha) x_{t-1}   (Appendix, EWMA)."""
    return alpha * s + (1.0 - alpha) * x_prev


SMOOTH_EWMA, SMOOTH_NONE, SMOOTH_WINDOW, SMOOTH_MOMENTUM, SMOOTH_PARAGRAPH = 0, 1, 2, 3, 4


@dataclass
class SignalHistory:
    """Everything one sequence has observed while thinking: `values[i]` is the
    3-vector of round i, `par_start` the index of the first round of the
    current paragraph (a paragraph ends in a round that accepts a step-split
    token without leaving thinking)."""
    values: list
    par_start: int = 0


def new_histories(B: int):
    return [SignalHistory(values=[]) for _ in range(B)]


def smooth_series(s: Sequence[float], cfg: ExitCfg, par_start: int = 0) -> float:
    """Smoothed score after the observations s[0..t] of one signal, s[t] being
    this round's (Appendix "Signal Smoothing").

    none       the latest observation.
    EWMA       x_0 = s_0, then x_i = alpha s_i + (1 - alpha) x_{i-1}.
    window     mean of the last N observations.
    momentum   forecast of the next score: the latest observation plus the mean
               of the N-1 differences between the last N consecutive
               observations.  (The paper indexes the forecast by the step it
               predicts, so its s_{t-1} is the latest value seen here.)
    paragraph  mean of every observation of the current paragraph,
               s[par_start..t].
    While fewer than N observations exist, window and momentum use those there
    are (a single observation is its own forecast); the paper does not say."""
    s = [float(v) for v in s]
    t = len(s)
    assert t >= 1
    if cfg.smoother == SMOOTH_NONE:
        return s[-1]
    if cfg.smoother == SMOOTH_EWMA:
        x = s[0]
        for v in s[1:]:
            x = ewma_update(x, v, cfg.alpha)
        return x
    if cfg.smoother == SMOOTH_WINDOW:
        last = s[-min(cfg.window, t):]
        return sum(last) / len(last)
    if cfg.smoother == SMOOTH_MOMENTUM:
        last = s[-min(cfg.window, t):]
        if len(last) == 1:
            return last[0]
        diffs = [last[i] - last[i - 1] for i in range(1, len(last))]
        return last[-1] + sum(diffs) / len(diffs)
    if cfg.smoother == SMOOTH_PARAGRAPH:
        seg = s[par_start:]
        return sum(seg) / len(seg)
    raise ValueError(f"unknown smoother {cfg.smoother}")


def greedy_accept(block_tok, parent, a):
    """Walk from the root: at node c go to the lowest-index child whose token
    equals the target's argmax at c; stop when no child matches.  A chain is the
    tree parent[i] = i - 1.  Returns (path of accepted nodes, last node)."""
    n = len(block_tok)
    cur, path = 0, []
    while True:
        nxt = -1
        for c in range(cur + 1, n):
            p = (c - 1) if parent is None else int(parent[c])
            if p == cur and int(block_tok[c]) == int(a[cur]):
                nxt = c
                break
        if nxt < 0:
            break
        path.append(nxt)
        cur = nxt
    return path, cur


def signals_pass(x, cfg: ExitCfg) -> bool:
    """Confidence above, progress above, remaining below their thresholds
    (strict), ANDed over the enabled signals (Appendix "Stop Threshold")."""
    ok = True
    if cfg.signal_mask & 1:
        ok = ok and (x[0] > cfg.thr_conf)
    if cfg.signal_mask & 2:
        ok = ok and (x[1] > cfg.thr_prog)
    if cfg.signal_mask & 4:
        ok = ok and (x[2] < cfg.thr_rem)
    return bool(ok)


def accept_exit(cfg: ExitCfg, block_tok, parent, target_argmax, sig, ctx_len, split_tok,
                ewma, n_obs, is_thinking, hist=None):
    """Per sequence, one decode round of the controller (Alg. 1).

    State (ewma [B,3] = the smoothed scores, n_obs [B], is_thinking [B], and for the
    window / momentum / paragraph smoothers the list `hist` of SignalHistory) is
    updated in place.
    1. smoothing: the first observation initialises the state, later ones follow
       the EWMA recurrence (or, with `hist`, smooth_series over the stored
       observations); frozen once thinking has ended.
    2. acceptance: greedy walk (see greedy_accept); recover token = target argmax
       at the last accepted node.
    3. exit: if thinking, signals pass, and an accepted draft token is a step
       split token: keep the path up to and including that token, recover token
       becomes the stop-think token, thinking ends.
    4. new context length = L + 1 (root) + accepted drafts."""
    block_tok = np.asarray(block_tok)
    B, n_q = block_tok.shape
    split = set(int(t) for t in np.asarray(split_tok).ravel())
    accept_len = np.zeros(B, np.int32)
    accept_path = np.full((B, n_q), -1, np.int32)
    recover = np.zeros(B, np.int32)
    last_node = np.zeros(B, np.int32)
    exit_flag = np.zeros(B, np.int32)
    new_ctx = np.zeros(B, np.int32)
    for b in range(B):
        if is_thinking[b]:
            if cfg.smoother in (SMOOTH_EWMA, SMOOTH_NONE):
                for j in range(3):
                    s = float(sig[b, j])
                    if cfg.smoother == SMOOTH_NONE or n_obs[b] == 0:
                        ewma[b, j] = s
                    else:
                        ewma[b, j] = ewma_update(float(ewma[b, j]), s, cfg.alpha)
            else:
                h = hist[b]
                h.values.append([float(sig[b, j]) for j in range(3)])
                for j in range(3):
                    ewma[b, j] = smooth_series([v[j] for v in h.values], cfg, h.par_start)
            n_obs[b] += 1
        par = None if parent is None else parent[b]
        path, cur = greedy_accept(block_tok[b], par, target_argmax[b])
        t_rec = int(target_argmax[b, cur])
        # candidate cut lengths: keep the path up to and including a split token
        cuts = [j + 1 for j, node in enumerate(path) if int(block_tok[b, node]) in split]
        if cfg.check_root and int(block_tok[b, 0]) in split:
            cuts.append(0)                # exit right after the root: nothing accepted
        hit = -1
        if cuts:
            hit = min(cuts) if cfg.split_pick == 0 else max(cuts)
        if is_thinking[b] and hit >= 0 and signals_pass(ewma[b], cfg):
            path = path[:hit]
            cur = path[-1] if path else 0
            t_rec = int(cfg.stop_think_token)
            is_thinking[b] = 0
            exit_flag[b] = 1
        elif is_thinking[b] and hit >= 0 and hist is not None:
            hist[b].par_start = len(hist[b].values)     # a step-split token closed the paragraph
        accept_len[b] = len(path)
        accept_path[b, :len(path)] = path
        recover[b] = t_rec
        last_node[b] = cur
        new_ctx[b] = int(ctx_len[b]) + 1 + len(path)
    return {"accept_len": accept_len, "accept_path": accept_path, "recover_tok": recover,
            "last_node": last_node, "exit_flag": exit_flag, "new_ctx_len": new_ctx}


# ---------------------------------------------------------------------------
# after the round: cache compaction  (Alg. 1, last step of a round)
# ---------------------------------------------------------------------------

def kv_compact(k, v, ctx_len, accept_path, accept_len, page_table=None, page_size=16,
               block_hidden=None, last_node=None):
    """The cache as the next round must find it: the block root stays at position
    L, the accepted node path[j] (stored at L + path[j] during verification)
    becomes entry L + 1 + j, so that positions 0 .. L + accept_len hold exactly
    the accepted sequence; whatever lies beyond is dead.  Every moved row is
    read from the cache as it was before the call.  Returns new (k, v) arrays,
    and with block_hidden [B, n_q, D] also the rows block_hidden[b, last_node[b]]
    (the target's hidden state the next round's first draft step starts from)."""
    k_new, v_new = np.array(k, copy=True), np.array(v, copy=True)
    B = len(ctx_len)
    Hkv = k.shape[1]

    def row(b, head, pos):
        if page_table is None:
            return (b, head, pos)
        return (int(page_table[b, pos // page_size]), head, pos % page_size)

    for b in range(B):
        L = int(ctx_len[b])
        for j in range(int(accept_len[b])):
            src, dst = L + int(accept_path[b, j]), L + 1 + j
            for head in range(Hkv):
                k_new[row(b, head, dst)] = k[row(b, head, src)]
                v_new[row(b, head, dst)] = v[row(b, head, src)]
    if block_hidden is None:
        return k_new, v_new
    hidden_next = np.stack([block_hidden[b, int(last_node[b])] for b in range(B)])
    return k_new, v_new, hidden_next

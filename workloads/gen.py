"""Seeded synthetic inputs for one SpecExit decode round (numpy only).

This module serves both the CPU oracle's tests and the HIP path's tests and
benchmark.  It holds *no arithmetic of the method*: it draws random tensors of
the stated shapes and distributions, rounds them to the storage type, lays KV
caches out contiguously or in pages, and draws draft-block structure (chains,
trees, token ids, signal series).  Anything that needs the method's results
(forcing a top-2 logit gap, keeping a smoothed signal off its threshold) is done
by the tests, which call the oracle.

Shapes follow the five workload descriptions of this build (tiny fp32 round;
Qwen3-4B-like; Qwen3-8B-like paged batch; 8B tree draft; 32B-like long paged
batch).  The paper's own workloads (its reasoning benchmarks on
Qwen3-4B-Thinking-2507 / DeepSeek-R1-Distill-Llama-8B, Sec. 4.1) are not
available; only their shapes and generation lengths (Table 1: about 0.3k-26k
tokens) are mirrored.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Optional, Tuple

import numpy as np

BASE_SEED = 20250924


@dataclass(frozen=True)
class Shape:
    name: str
    index: int              # position in the list of workload configurations
    dtype: str              # "f32" or "bf16": storage type of weights / KV / activations
    D: int                  # hidden size
    Hq: int                 # query heads
    Hkv: int                # KV heads
    d: int                  # head dim
    V: int                  # vocabulary
    I: int                  # MLP intermediate size of the draft layer
    B: int                  # sequences
    k: int                  # chain draft length (tree: depth)
    n_q: int                # verification block size (root + drafts / tree nodes)
    tree: bool = False
    ctx: Tuple[int, int] = (256, 256)   # inclusive range of per-sequence context length
    paged: bool = False
    page_size: int = 16
    n_rounds: int = 1       # length of the controller's signal series
    rope_theta: float = 1.0e6
    rms_eps: float = 1.0e-6

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv


CONFIGS = [
    Shape("tiny_f32", 0, "f32", 512, 8, 2, 64, 4096, 2048, 1, 4, 5, ctx=(256, 256), n_rounds=8),
    Shape("qwen3_4b_chain", 1, "bf16", 2560, 32, 8, 128, 151936, 9728, 1, 6, 7,
          ctx=(4096, 4096), n_rounds=64),
    Shape("qwen3_8b_paged", 2, "bf16", 4096, 32, 8, 128, 151936, 12288, 8, 6, 7,
          ctx=(2048, 16384), paged=True, n_rounds=64),
    Shape("tree_8b", 3, "bf16", 4096, 32, 8, 128, 151936, 12288, 4, 5, 16, tree=True,
          ctx=(8192, 8192), n_rounds=64),
    Shape("qwen3_32b_paged", 4, "bf16", 5120, 64, 8, 128, 151936, 25600, 16, 8, 9,
          ctx=(8192, 32768), paged=True, n_rounds=2048),
]


def config(index: int) -> Shape:
    return CONFIGS[index]


def scaled(shape: Shape, **kw) -> Shape:
    """A reduced copy of a configuration (same structure, smaller extents)."""
    return replace(shape, **kw)


def rng_for(shape: Shape, stream: int, seed: int = 0) -> np.random.Generator:
    return np.random.default_rng(BASE_SEED + 1000 * shape.index + stream + 1_000_003 * seed)


# ---------------------------------------------------------------------------
# storage-type rounding (an encoding of the inputs, not part of the method)
# ---------------------------------------------------------------------------

def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    r = ((u + bias) >> 16) << 16
    return r.astype(np.uint32).view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of fp32 values that are already bf16-representable."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "values are not bf16-representable"
    return (u >> 16).astype(np.uint16)


def bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32)


def store(shape: Shape, x: np.ndarray) -> np.ndarray:
    """Round to the configuration's storage type (values kept as fp32)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return round_to_bf16(x) if shape.dtype == "bf16" else x


def normal(rng: np.random.Generator, size, std: float, shape: Shape) -> np.ndarray:
    """N(0, std^2) in the storage type, drawn in row blocks to bound memory."""
    size = tuple(int(s) for s in (size if isinstance(size, (tuple, list)) else (size,)))
    out = np.empty(size, dtype=np.float32)
    flat = out.reshape(-1)
    step = 1 << 24
    for lo in range(0, flat.size, step):
        hi = min(flat.size, lo + step)
        blk = rng.standard_normal(hi - lo, dtype=np.float32) * np.float32(std)
        flat[lo:hi] = round_to_bf16(blk) if shape.dtype == "bf16" else blk
    return out


# ---------------------------------------------------------------------------
# weights
# ---------------------------------------------------------------------------

def draft_weights(shape: Shape, seed: int = 0, std: float = 0.02) -> dict:
    """Draft model parameters, all N(0, std^2); norm vectors are ones.

    Row-major [out, in].  w_head has V+3 rows: token rows first, then the
    confidence, progress and remaining-length rows (Eq. 1)."""
    r = rng_for(shape, 1, seed)
    D, Hq, Hkv, d, I, V = shape.D, shape.Hq, shape.Hkv, shape.d, shape.I, shape.V
    w = {
        "embed": normal(r, (V, D), std, shape),
        "w_fc": normal(r, (D, 2 * D), std, shape),
        "ln_attn": np.ones(D, np.float32),
        "ln_mlp": np.ones(D, np.float32),
        "ln_final": np.ones(D, np.float32),
        "w_q": normal(r, (Hq * d, D), std, shape),
        "w_k": normal(r, (Hkv * d, D), std, shape),
        "w_v": normal(r, (Hkv * d, D), std, shape),
        "w_o": normal(r, (D, Hq * d), std, shape),
        "w_gate": normal(r, (I, D), std, shape),
        "w_up": normal(r, (I, D), std, shape),
        "w_down": normal(r, (D, I), std, shape),
        "w_head": normal(r, (V + 3, D), std, shape),
    }
    return w


def perturbed_norm_vectors(shape: Shape, seed: int = 0) -> dict:
    """Non-trivial norm gains (1 + N(0, 0.1^2)) so that tests see them act."""
    r = rng_for(shape, 2, seed)
    return {n: store(shape, 1.0 + 0.1 * r.standard_normal(shape.D).astype(np.float32))
            for n in ("ln_attn", "ln_mlp", "ln_final")}


def lm_head(shape: Shape, seed: int = 0, std: float = 0.02, n_extra: int = 0) -> np.ndarray:
    r = rng_for(shape, 3, seed)
    return normal(r, (shape.V + n_extra, shape.D), std, shape)


def hidden_rows(shape: Shape, M: int, seed: int = 0, stream: int = 4) -> np.ndarray:
    r = rng_for(shape, stream, seed)
    return normal(r, (M, shape.D), 1.0, shape)


def token_ids(shape: Shape, n: int, seed: int = 0, stream: int = 5) -> np.ndarray:
    r = rng_for(shape, stream, seed)
    return r.integers(0, shape.V, size=n, dtype=np.int32)


# ---------------------------------------------------------------------------
# KV caches
# ---------------------------------------------------------------------------

def context_lengths(shape: Shape, seed: int = 0) -> np.ndarray:
    r = rng_for(shape, 6, seed)
    lo, hi = shape.ctx
    return r.integers(lo, hi + 1, size=shape.B, dtype=np.int32)


@dataclass
class KVCache:
    """K and V of one attention layer.

    contiguous: k, v are [B, Hkv, l_max, d].
    paged:      k, v are [n_pages, Hkv, page_size, d]; page_table[b, j] is the
                pool page that holds tokens j*page_size .. of sequence b
                (entries past a sequence's last page are 0 and must not matter).
    Positions L_b .. L_b+extra-1 (the verification block / the draft's own new
    entries) are allocated and, for attention tests, filled."""
    paged: bool
    k: np.ndarray
    v: np.ndarray
    ctx_len: np.ndarray
    l_max: int
    page_size: int = 16
    page_table: Optional[np.ndarray] = None
    n_pages: int = 0

    def rows(self, which: str, b: int, head: int, positions: np.ndarray) -> np.ndarray:
        """Gather rows [len(positions), d] of K or V (a layout lookup, no arithmetic)."""
        pool = self.k if which == "k" else self.v
        positions = np.asarray(positions, dtype=np.int64)
        if not self.paged:
            return pool[b, head, positions, :]
        pages = self.page_table[b, positions // self.page_size]
        return pool[pages, head, positions % self.page_size, :]


def kv_cache(shape: Shape, ctx_len: np.ndarray, extra: int, seed: int = 0, stream: int = 7,
             paged: Optional[bool] = None, fill: bool = True) -> KVCache:
    """KV entries ~ N(0,1) for positions 0 .. L_b+extra-1 of every sequence."""
    r = rng_for(shape, stream, seed)
    paged = shape.paged if paged is None else paged
    B, Hkv, d, ps = shape.B, shape.Hkv, shape.d, shape.page_size
    need = ctx_len.astype(np.int64) + extra
    if not paged:
        l_max = int(need.max())
        if fill:
            k = normal(r, (B, Hkv, l_max, d), 1.0, shape)
            v = normal(r, (B, Hkv, l_max, d), 1.0, shape)
        else:
            k = np.zeros((B, Hkv, l_max, d), np.float32)
            v = np.zeros((B, Hkv, l_max, d), np.float32)
        return KVCache(False, k, v, ctx_len.copy(), l_max, ps)
    pages_per_seq = (need + ps - 1) // ps
    used = int(pages_per_seq.sum())
    n_pages = used + max(1, used // 10)
    perm = r.permutation(n_pages)[:used].astype(np.int32)
    max_pages = int(pages_per_seq.max())
    table = np.zeros((B, max_pages), np.int32)
    off = 0
    for b in range(B):
        n = int(pages_per_seq[b])
        table[b, :n] = perm[off:off + n]
        off += n
    if fill:
        k = normal(r, (n_pages, Hkv, ps, d), 1.0, shape)
        v = normal(r, (n_pages, Hkv, ps, d), 1.0, shape)
    else:
        k = np.zeros((n_pages, Hkv, ps, d), np.float32)
        v = np.zeros((n_pages, Hkv, ps, d), np.float32)
    return KVCache(True, k, v, ctx_len.copy(), max_pages * ps, ps, table, n_pages)


def to_paged(shape: Shape, kv: KVCache, extra: int, seed: int = 0) -> KVCache:
    """The same cache contents re-laid into shuffled pages."""
    assert not kv.paged
    out = kv_cache(shape, kv.ctx_len, extra, seed=seed, stream=8, paged=True, fill=True)
    ps = out.page_size
    for b in range(kv.k.shape[0]):
        n = int(kv.ctx_len[b]) + extra
        pos = np.arange(n)
        pages = out.page_table[b, pos // ps]
        out.k[pages, :, pos % ps, :] = np.transpose(kv.k[b, :, :n, :], (1, 0, 2))
        out.v[pages, :, pos % ps, :] = np.transpose(kv.v[b, :, :n, :], (1, 0, 2))
    return out


def queries(shape: Shape, seed: int = 0, n_q: Optional[int] = None) -> np.ndarray:
    r = rng_for(shape, 9, seed)
    n_q = shape.n_q if n_q is None else n_q
    return normal(r, (shape.B, n_q, shape.Hq, shape.d), 1.0, shape)


# ---------------------------------------------------------------------------
# draft blocks: chains, trees, masks
# ---------------------------------------------------------------------------

def chain_parents(B: int, n_q: int) -> np.ndarray:
    p = np.tile(np.arange(-1, n_q - 1, dtype=np.int32), (B, 1))
    return p


def random_tree_parents(shape: Shape, seed: int = 0, max_children: int = 3) -> np.ndarray:
    """Per sequence: node 0 is the root; node i>0 hangs under a uniformly chosen
    earlier node that has depth < shape.k and fewer than max_children children;
    topologies are redrawn until the deepest node has depth shape.k."""
    r = rng_for(shape, 10, seed)
    n, depth_cap = shape.n_q, shape.k
    out = np.empty((shape.B, n), np.int32)
    for b in range(shape.B):
        while True:
            parent = np.full(n, -1, np.int32)
            depth = np.zeros(n, np.int32)
            nchild = np.zeros(n, np.int32)
            for i in range(1, n):
                cand = [j for j in range(i) if depth[j] < depth_cap and nchild[j] < max_children]
                j = cand[int(r.integers(0, len(cand)))]
                parent[i] = j
                depth[i] = depth[j] + 1
                nchild[j] += 1
            if depth.max() == depth_cap:
                break
        out[b] = parent
    return out


def level_ordered_tree(shape: Shape, seed: int = 0, max_children: int = 3):
    """One draft-tree topology for tree drafting, shared by the sequences: a random tree as
    above, renumbered level by level (parents keep their relative order), with rank[c] = the
    position of c among its siblings.  Returns (parent [n], rank [n])."""
    one = replace(shape, B=1)
    old = random_tree_parents(one, seed, max_children)[0]
    n = len(old)
    depth = np.zeros(n, np.int64)
    for c in range(1, n):
        depth[c] = depth[old[c]] + 1
    order = sorted(range(n), key=lambda c: (depth[c], c))
    new_id = {c: i for i, c in enumerate(order)}
    parent = np.full(n, -1, np.int32)
    for c in range(1, n):
        parent[new_id[c]] = new_id[int(old[c])]
    rank = np.zeros(n, np.int32)
    seen = {}
    for c in range(1, n):
        rank[c] = seen.get(int(parent[c]), 0)
        seen[int(parent[c])] = rank[c] + 1
    return parent, rank


def ancestor_masks(parent: np.ndarray) -> np.ndarray:
    """mask[b, i] bit j set iff node j is node i or one of its ancestors."""
    B, n = parent.shape
    m = np.zeros((B, n), np.uint64)
    for b in range(B):
        for i in range(n):
            p = int(parent[b, i])
            m[b, i] = (m[b, p] if p >= 0 else np.uint64(0)) | (np.uint64(1) << np.uint64(i))
    return m


def node_depths(parent: np.ndarray) -> np.ndarray:
    B, n = parent.shape
    dep = np.zeros((B, n), np.int32)
    for b in range(B):
        for i in range(1, n):
            dep[b, i] = dep[b, parent[b, i]] + 1
    return dep


@dataclass
class AcceptCase:
    block_tok: np.ndarray       # [B, n_q] int32, node 0 = last accepted token
    parent: Optional[np.ndarray]  # [B, n_q] int32 or None for a chain
    target_argmax: np.ndarray   # [B, n_q] int32
    planted_len: np.ndarray     # [B] number of draft tokens built to match
    split_tok: np.ndarray       # [S] sorted int32
    stop_think_token: int


def accept_case(shape: Shape, seed: int = 0, parent: Optional[np.ndarray] = None,
                p_accept: float = 0.75, p_split: float = 0.3, n_split: int = 8) -> AcceptCase:
    """Block tokens and target argmaxes with a planted matching prefix / root path.

    Chain: m = min(Geometric - 1, k) draft tokens match (per-token acceptance
    p_accept, an assumption: the paper prints no acceptance rates), the next one
    is built to differ.  Tree: one root path is built to match for m edges
    (m uniform in 0..depth); all other children differ from their parent's
    argmax and siblings carry distinct tokens.  With probability p_split one
    matching draft token is replaced by a step-split id (in both arrays)."""
    r = rng_for(shape, 11, seed)
    B, n, V = shape.B, shape.n_q, shape.V
    is_tree = parent is not None
    par = parent if is_tree else chain_parents(B, n)
    split = np.sort(r.choice(V - 1, size=n_split, replace=False).astype(np.int32))
    stop_tok = V - 1            # never drawn into the split set
    a = r.integers(0, V - 1, size=(B, n), dtype=np.int32)
    tok = r.integers(0, V - 1, size=(B, n), dtype=np.int32)
    planted = np.zeros(B, np.int32)
    in_split = set(int(s) for s in split)
    for b in range(B):
        children = [[] for _ in range(n)]
        for i in range(1, n):
            children[par[b, i]].append(i)
        # keep every drawn id out of the split set unless planted below
        for i in range(n):
            while int(a[b, i]) in in_split:
                a[b, i] = (a[b, i] + 1) % (V - 1)
            while int(tok[b, i]) in in_split:
                tok[b, i] = (tok[b, i] + 1) % (V - 1)
        if is_tree:
            m = int(r.integers(0, shape.k + 1))
        else:
            m = min(int(r.geometric(1.0 - p_accept)) - 1, n - 1)
        # walk a root path of up to m edges
        path = []
        cur = 0
        for _ in range(m):
            if not children[cur]:
                break
            nxt = children[cur][int(r.integers(0, len(children[cur])))]
            path.append(nxt)
            cur = nxt
        planted[b] = len(path)
        if path and r.random() < p_split:
            j = int(r.integers(0, len(path)))
            a[b, par[b, path[j]]] = split[int(r.integers(0, n_split))]
        on_path = set(path)
        for c in range(n):
            sib_used = set()
            for ch in children[c]:
                if ch in on_path:
                    tok[b, ch] = a[b, c]
                    sib_used.add(int(tok[b, ch]))
            for ch in children[c]:
                if ch in on_path:
                    continue
                t = int(tok[b, ch])
                while t == int(a[b, c]) or t in sib_used or t in in_split:
                    t = (t + 1) % (V - 1)
                tok[b, ch] = t
                sib_used.add(t)
    return AcceptCase(tok, par if is_tree else None, a, planted, split, stop_tok)


# ---------------------------------------------------------------------------
# exit-signal series (confidence, progress, remaining tokens)
# ---------------------------------------------------------------------------

def signal_series(shape: Shape, seed: int = 0, noise: float = 0.05):
    """[n_rounds, B, 3] fp32 raw (activated) signals per decode round.

    Short series (<= 64 rounds): noisy monotone ramps that level off after 60 % of the rounds.  Long series: per sequence
    a logistic ramp centred on a round tau_b ~ U{200..2000} (width 20 rounds),
    the long-reasoning regime.  Returns (series, tau) with tau None for ramps."""
    r = rng_for(shape, 12, seed)
    T, B = shape.n_rounds, shape.B
    t = np.arange(T, dtype=np.float64)[:, None]
    eps = r.standard_normal((T, B, 3)) * noise
    if T <= 64:
        f = np.minimum(1.0, t / (0.6 * T))      # ramp over the first 60 % of the rounds, then flat
        conf = np.clip(0.4 + 0.6 * f + eps[:, :, 0], 0.0, 1.0)
        prog = np.clip(f + eps[:, :, 1], 0.0, 1.0)
        rem = np.maximum(0.0, 2000.0 * (1.0 - f) * (1.0 + eps[:, :, 2]))
        tau = None
    else:
        tau = r.integers(200, min(2000, T - 40) + 1, size=B)
        g = 1.0 / (1.0 + np.exp(-(t - tau[None, :]) / 20.0))
        conf = np.clip(0.3 + 0.68 * g + eps[:, :, 0], 0.0, 1.0)
        prog = np.clip(g + eps[:, :, 1], 0.0, 1.0)
        rem = np.maximum(0.0, 4000.0 * (1.0 - g) * (1.0 + eps[:, :, 2]))
    s = np.stack([conf, prog, rem], axis=-1).astype(np.float32)
    return s, tau

"""Pins for the oracle's LM-head argmax and draft step (CPU only).

LM head: textbook dot products (brute-force loops on tiny inputs), planted
winners with a known gap, lowest index on ties, signal rows excluded (Eq. 1).
Draft step: the decoder layer is rebuilt from torch library routines (rms_norm,
linear, silu, scaled_dot_product_attention) with the rotary embedding written as
a complex multiplication; special cases isolate each sub-block."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import specexit_oracle as O
from workloads import gen


# ----------------------------------------------------------------------------- LM head

def test_logits_are_dot_products_brute_force():
    r = np.random.default_rng(1)
    H = r.standard_normal((3, 7))
    W = r.standard_normal((11, 7))
    am, z, extra = O.lmhead_argmax(H, W)
    for m in range(3):
        for v in range(11):
            assert abs(z[m, v] - math.fsum(H[m, c] * W[v, c] for c in range(7))) < 1e-13
        assert am[m] == max(range(11), key=lambda v: z[m, v])
    assert extra.shape == (3, 0)


def test_row_blocking_does_not_change_values():
    r = np.random.default_rng(2)
    x, w = r.standard_normal((2, 9)), r.standard_normal((50, 9))
    np.testing.assert_allclose(O.linear(x, w, row_block=7), O.linear(x, w, row_block=1000), rtol=0, atol=1e-13)


def test_planted_winner_and_gap():
    shape = gen.scaled(gen.config(0), V=300, D=48)
    H = gen.hidden_rows(shape, 4, 0).astype(np.float64)
    W = gen.lm_head(shape, 0).astype(np.float64)
    wins = [17, 0, 299, 123]
    for m, v in enumerate(wins):
        # make row v's logit for hidden m equal to 5 while others stay N(0, small)
        others = np.delete(np.arange(4), m)
        W[v] = 5.0 * H[m] / (H[m] @ H[m])
    am, z, _ = O.lmhead_argmax(H, W)
    assert am.tolist() == wins
    for m, v in enumerate(wins):
        assert abs(z[m, v] - 5.0) < 1e-12
    gap = O.top2_gap(z)
    for m in range(4):
        srt = np.sort(z[m])
        assert abs(gap[m] - (srt[-1] - srt[-2])) < 1e-15 and gap[m] > 1.0


def test_tie_returns_lowest_index():
    r = np.random.default_rng(3)
    H = r.standard_normal((2, 8))
    W = r.standard_normal((20, 8)) * 0.01
    W[13] = W[5] = 3.0 * H[0] / (H[0] @ H[0])
    am, z, _ = O.lmhead_argmax(H, W)
    assert z[0, 5] == z[0, 13] and am[0] == 5
    assert O.argmax_lowest(np.array([1.0, 7.0, 7.0, 7.0, -2.0])) == 1
    assert O.argmax_lowest(np.array([4.0])) == 0


def test_signal_rows_are_not_vocabulary():
    """Eq. 1: the last three rows are signals; a huge value there never becomes a token."""
    r = np.random.default_rng(4)
    H = r.standard_normal((3, 8))
    W = r.standard_normal((23, 8))
    W[20:] = 100.0 * np.sign(H[0])
    am, z, extra = O.lmhead_argmax(H, W, n_extra=3)
    assert z.shape == (3, 20) and extra.shape == (3, 3)
    assert np.all(am < 20)
    np.testing.assert_allclose(extra, H @ W[20:].T, atol=1e-12)
    am_all, _, _ = O.lmhead_argmax(H, W, n_extra=0)
    assert am_all[0] >= 20          # the same rows would win if they were tokens


# ----------------------------------------------------------------------------- draft sub-blocks

def test_rmsnorm_against_library():
    r = np.random.default_rng(5)
    u, w = r.standard_normal((3, 40)), r.standard_normal(40)
    ref = F.rms_norm(torch.tensor(u), (40,), torch.tensor(w), eps=1e-6).numpy()
    np.testing.assert_allclose(O.rmsnorm(u, w, 1e-6), ref, atol=1e-13)
    # unit-RMS output for unit gain, and eps really is inside the square root
    out = O.rmsnorm(u, np.ones(40), 0.0)
    np.testing.assert_allclose(np.mean(out * out, axis=-1), 1.0, atol=1e-13)
    z = O.rmsnorm(np.full((1, 4), 1e-3), np.ones(4), 1.0)
    np.testing.assert_allclose(z, 1e-3 / np.sqrt(1e-6 + 1.0), atol=1e-15)


def rope_complex(x, pos, theta):
    d = x.shape[-1]
    half = d // 2
    z = torch.complex(torch.tensor(x[..., :half]), torch.tensor(x[..., half:]))
    ang = pos * theta ** (-2.0 * torch.arange(half, dtype=torch.float64) / d)
    z = z * torch.polar(torch.ones(half, dtype=torch.float64), ang)
    return np.concatenate([z.real.numpy(), z.imag.numpy()], axis=-1)


def test_rope_properties():
    r = np.random.default_rng(6)
    x, y = r.standard_normal((4, 16)), r.standard_normal((4, 16))
    theta = 1.0e4
    np.testing.assert_array_equal(O.rope_rotate_half(x, 0, theta), x)
    for pos in (1, 7, 1000):
        rx = O.rope_rotate_half(x, pos, theta)
        np.testing.assert_allclose(rx, rope_complex(x, pos, theta), atol=1e-12)
        np.testing.assert_allclose(np.linalg.norm(rx, axis=-1), np.linalg.norm(x, axis=-1), atol=1e-12)
    # relative-position property: <R_p x, R_q y> depends on p - q only
    a = np.sum(O.rope_rotate_half(x, 12, theta) * O.rope_rotate_half(y, 5, theta), axis=-1)
    b = np.sum(O.rope_rotate_half(x, 107, theta) * O.rope_rotate_half(y, 100, theta), axis=-1)
    np.testing.assert_allclose(a, b, atol=1e-10)
    # d = 2, pos = 1, theta irrelevant (c = 0): a plain rotation by one radian
    out = O.rope_rotate_half(np.array([1.0, 0.0]), 1, 123.0)
    np.testing.assert_allclose(out, [math.cos(1.0), math.sin(1.0)], atol=1e-15)
    # the frequency of pair c is theta^(-2c/d): the last pair turns slowest
    out = O.rope_rotate_half(np.array([0.0, 1.0, 0.0, 0.0]), 3, 100.0)
    np.testing.assert_allclose(out, [0, math.cos(3 / 10.0), 0, math.sin(3 / 10.0)], atol=1e-15)


def test_activations():
    np.testing.assert_allclose(O.sigmoid(0.0), 0.5)
    np.testing.assert_allclose(O.sigmoid(np.array([2.0, -2.0])).sum(), 1.0, atol=1e-15)
    np.testing.assert_allclose(O.silu(np.array([0.0, 1.0])), [0.0, 1 / (1 + math.exp(-1))], atol=1e-15)
    np.testing.assert_allclose(O.silu(np.array([-3.0, 3.0])), F.silu(torch.tensor([-3.0, 3.0], dtype=torch.float64)).numpy())
    s = O.signal_activations(np.array([[0.0, 0.0, 0.0], [2.0, -1.0, math.log(1 + 150.0)], [0, 0, -4.0]]))
    np.testing.assert_allclose(s[0], [0.5, 0.5, 0.0])
    np.testing.assert_allclose(s[1], [1 / (1 + math.exp(-2)), 1 / (1 + math.e), 150.0], rtol=1e-12)
    assert s[2, 2] == 0.0                       # a negative token count is floored
    # remaining-length is the inverse of the training target log(1 + r)  (Eq. 5)
    for rr in (0.0, 3.0, 199.0, 20000.0):
        assert abs(O.signal_activations(np.array([0, 0, math.log1p(rr)]))[2] - rr) < 1e-9 * max(1, rr)


# ----------------------------------------------------------------------------- whole draft step

def tiny_draft(seed=0, B=3, ctx=(0, 9), norms=True):
    shape = gen.scaled(gen.config(0), D=32, Hq=4, Hkv=2, d=8, V=50, I=48, B=B, ctx=ctx, rope_theta=1.0e4)
    w = gen.draft_weights(shape, seed, std=0.3)
    if norms:
        w.update(gen.perturbed_norm_vectors(shape, seed))
    pos = gen.context_lengths(shape, seed)
    kv = gen.kv_cache(shape, pos, 1, seed, paged=False)
    tok = gen.token_ids(shape, B, seed)
    g = gen.hidden_rows(shape, B, seed)
    dims = O.DraftDims(shape.D, shape.Hq, shape.Hkv, shape.d, shape.V, shape.rms_eps, shape.rope_theta)
    return shape, dims, w, kv, tok, g, pos


def torch_draft_step(shape, w, kv, tok, g, pos):
    """The same layer from library routines, float64."""
    T = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))
    outs = []
    for b in range(len(tok)):
        x = F.linear(torch.cat([T(w["embed"][tok[b]]), T(g[b])]), T(w["w_fc"]))
        n = F.rms_norm(x, (shape.D,), T(w["ln_attn"]), eps=shape.rms_eps)
        q = F.linear(n, T(w["w_q"])).reshape(shape.Hq, shape.d).numpy()
        k = F.linear(n, T(w["w_k"])).reshape(shape.Hkv, shape.d).numpy()
        v = F.linear(n, T(w["w_v"])).reshape(shape.Hkv, shape.d)
        p = int(pos[b])
        q = T(rope_complex(q, p, shape.rope_theta))
        k = T(rope_complex(k, p, shape.rope_theta))
        kc = torch.cat([T(kv.k[b, :, :p]), k[:, None, :]], dim=1)
        vc = torch.cat([T(kv.v[b, :, :p]), v[:, None, :]], dim=1)
        att = F.scaled_dot_product_attention(q[None, :, None, :], kc[None], vc[None], enable_gqa=True)
        a = x + F.linear(att.reshape(-1), T(w["w_o"]))
        m = F.rms_norm(a, (shape.D,), T(w["ln_mlp"]), eps=shape.rms_eps)
        y = a + F.linear(F.silu(F.linear(m, T(w["w_gate"]))) * F.linear(m, T(w["w_up"])), T(w["w_down"]))
        h = F.rms_norm(y, (shape.D,), T(w["ln_final"]), eps=shape.rms_eps)
        z = F.linear(h, T(w["w_head"]))
        outs.append((y.numpy(), z.numpy(), k.numpy(), v.numpy()))
    return outs


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_draft_step_against_library_layer(seed):
    shape, dims, w, kv, tok, g, pos = tiny_draft(seed)
    ref = torch_draft_step(shape, w, kv, tok, g, pos)
    k_cache, v_cache = kv.k.astype(np.float64), kv.v.astype(np.float64)
    out = O.draft_step(dims, w, k_cache, v_cache, tok, g, pos)
    for b in range(shape.B):
        y, z, k_new, v_new = ref[b]
        np.testing.assert_allclose(out["hidden_out"][b], y, atol=1e-11)
        np.testing.assert_allclose(out["logits"][b], z[:shape.V], atol=1e-11)
        np.testing.assert_allclose(out["sig_raw"][b], z[shape.V:], atol=1e-11)
        assert out["next_tok"][b] == int(np.argmax(z[:shape.V]))
        np.testing.assert_allclose(k_cache[b, :, pos[b]], k_new, atol=1e-12)
        np.testing.assert_allclose(v_cache[b, :, pos[b]], v_new, atol=1e-12)
    np.testing.assert_allclose(out["sig"][:, 0], 1 / (1 + np.exp(-out["sig_raw"][:, 0])), atol=1e-15)
    np.testing.assert_allclose(out["sig"][:, 2], np.maximum(0, np.expm1(out["sig_raw"][:, 2])), atol=1e-12)


def test_widened_head_equals_four_separate_products():
    """Eq. 1: W h = [W_tok h, W_conf h, W_prog h, W_rem h]."""
    shape, dims, w, kv, tok, g, pos = tiny_draft(3)
    out = O.draft_step(dims, w, kv.k.astype(np.float64), kv.v.astype(np.float64), tok, g, pos)
    h = O.rmsnorm(out["hidden_out"], w["ln_final"], dims.rms_eps)
    V = shape.V
    np.testing.assert_allclose(out["logits"], h @ w["w_head"][:V].astype(np.float64).T, atol=1e-12)
    for j in range(3):
        np.testing.assert_allclose(out["sig_raw"][:, j], h @ w["w_head"][V + j].astype(np.float64), atol=1e-12)
    # the signal rows do not touch the token prediction
    w2 = dict(w)
    w2["w_head"] = w["w_head"].copy()
    w2["w_head"][V:] *= -7.0
    out2 = O.draft_step(dims, w2, kv.k.astype(np.float64), kv.v.astype(np.float64), tok, g, pos)
    np.testing.assert_array_equal(out2["logits"], out["logits"])
    np.testing.assert_array_equal(out2["next_tok"], out["next_tok"])


def test_zero_output_projections_leave_the_fused_input():
    shape, dims, w, kv, tok, g, pos = tiny_draft(4)
    w = dict(w)
    w["w_o"] = np.zeros_like(w["w_o"])
    w["w_down"] = np.zeros_like(w["w_down"])
    out = O.draft_step(dims, w, kv.k.astype(np.float64), kv.v.astype(np.float64), tok, g, pos)
    for b in range(shape.B):
        cat = np.concatenate([w["embed"][tok[b]], g[b]]).astype(np.float64)
        np.testing.assert_allclose(out["hidden_out"][b], w["w_fc"].astype(np.float64) @ cat, atol=1e-12)
    # order inside the fuse: embedding first, hidden state second
    g2 = g.copy()
    g2[:, 0] += 1.0
    out2 = O.draft_step(dims, w, kv.k.astype(np.float64), kv.v.astype(np.float64), tok, g2, pos)
    np.testing.assert_allclose(out2["hidden_out"] - out["hidden_out"],
                               np.broadcast_to(w["w_fc"][:, shape.D].astype(np.float64), (shape.B, shape.D)), atol=1e-12)


def test_position_zero_attends_to_itself_only():
    shape, dims, w, kv, tok, g, pos = tiny_draft(5, ctx=(0, 0))
    k_cache, v_cache = kv.k.astype(np.float64), kv.v.astype(np.float64)
    out = O.draft_step(dims, w, k_cache, v_cache, tok, g, pos)
    for b in range(shape.B):
        own_v = v_cache[b, :, 0]                                   # [Hkv, d] just written
        expect = np.repeat(own_v, shape.G, axis=0).reshape(-1)     # each query head sees its KV head
        np.testing.assert_allclose(out["attn_out"][b], expect, atol=1e-13)


def test_draft_cache_positions_beyond_pos_do_not_matter():
    shape, dims, w, kv, tok, g, pos = tiny_draft(6, ctx=(4, 4))
    kv_big = gen.kv_cache(shape, pos, 5, 6, paged=False)
    a = O.draft_step(dims, w, kv_big.k.astype(np.float64), kv_big.v.astype(np.float64), tok, g, pos)
    k2, v2 = kv_big.k.astype(np.float64), kv_big.v.astype(np.float64)
    k2[:, :, 5:] += 9.0
    v2[:, :, 5:] -= 9.0
    b = O.draft_step(dims, w, k2, v2, tok, g, pos)
    np.testing.assert_array_equal(a["hidden_out"], b["hidden_out"])
    # ... while an earlier position does
    k3 = kv_big.k.astype(np.float64)
    k3[:, :, 0] += 1.0
    c = O.draft_step(dims, w, k3, kv_big.v.astype(np.float64), tok, g, pos)
    assert np.abs(c["hidden_out"] - a["hidden_out"]).max() > 1e-6


def test_draft_step_paged_cache_equals_contiguous():
    shape, dims, w, kv, tok, g, pos = tiny_draft(7, ctx=(3, 40))
    paged = gen.to_paged(shape, kv, 1, seed=1)
    a = O.draft_step(dims, w, kv.k.astype(np.float64), kv.v.astype(np.float64), tok, g, pos)
    pk, pv = paged.k.astype(np.float64), paged.v.astype(np.float64)
    b = O.draft_step(dims, w, pk, pv, tok, g, pos, page_table=paged.page_table, page_size=paged.page_size)
    np.testing.assert_array_equal(a["hidden_out"], b["hidden_out"])
    np.testing.assert_array_equal(a["next_tok"], b["next_tok"])


def test_storage_rounding_helpers():
    x = np.array([1.0, 1.00390625, 1.005859375, -3.1415927, 1e-30, 65504.0], np.float32)
    r = gen.round_to_bf16(x)
    assert r[0] == 1.0
    assert r[1] == 1.0                     # exactly halfway between 1.0 and 1.0078125: ties to even
    assert r[2] == 1.0078125               # above halfway rounds up
    bits = gen.bf16_bits(r)
    np.testing.assert_array_equal(gen.bits_to_f32(bits), r)
    ref = torch.tensor(x).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(r, ref)

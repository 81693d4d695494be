"""Pins for the oracle's decoder forward: special cases that reduce to torch library routines,
closed-form properties of its pieces, and cache / mask invariances."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import s2d2_oracle as O
from s2d2_inputs import ModelCfg, gen_weights

CFG = ModelCfg("pin", n_layers=2, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=96, vocab=50,
               dtype="f32", rope_theta=10000.0)
MOE = ModelCfg("pin-moe", n_layers=2, d_model=32, n_q_heads=2, n_kv_heads=1, head_dim=16, d_ffn=0, vocab=40,
               n_experts=4, top_k=2, d_expert=24, dtype="f32", rope_theta=10000.0)


def weights(cfg, seed=3):
    # large-ish gain and jittered norm gains so that every operand matters
    return gen_weights(cfg, seed=seed, unembed_gain=8.0, norm_jitter=0.2)


def empty_cache(cfg):
    z = np.zeros((0, cfg.n_kv_heads, cfg.head_dim))
    return [z] * cfg.n_layers, [z] * cfg.n_layers


def torch_library_causal_lm(cfg, W, tokens):
    """Plain causal LM forward built from torch library ops (fp64), RoPE via complex rotation."""
    t = lambda n: W[n].to(torch.float64)
    n, Hq, Hkv, D = len(tokens), cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    h = F.embedding(torch.as_tensor(tokens, dtype=torch.long), t("embed"))
    pos = torch.arange(n, dtype=torch.float64)
    freqs = torch.outer(pos, cfg.rope_theta ** (-torch.arange(0, D, 2, dtype=torch.float64) / D))
    rot = torch.polar(torch.ones_like(freqs), freqs)  # e^{i pos w_k}

    def rotate(x):  # x [n, H, D]; pair (x_k, x_{k+D/2}) is one complex number
        z = torch.complex(x[..., : D // 2], x[..., D // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    for l in range(cfg.n_layers):
        a = F.rms_norm(h, (cfg.d_model,), t(f"l{l}.norm1"), cfg.rms_eps)
        q, k, v = F.linear(a, t(f"l{l}.wqkv")).split([Hq * D, Hkv * D, Hkv * D], dim=-1)
        q, k, v = rotate(q.view(n, Hq, D)), rotate(k.view(n, Hkv, D)), v.view(n, Hkv, D)
        k = k.repeat_interleave(Hq // Hkv, dim=1)
        v = v.repeat_interleave(Hq // Hkv, dim=1)
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None],
                                           v.transpose(0, 1)[None], is_causal=True)[0]
        h = h + F.linear(o.transpose(0, 1).reshape(n, Hq * D), t(f"l{l}.wo"))
        b = F.rms_norm(h, (cfg.d_model,), t(f"l{l}.norm2"), cfg.rms_eps)
        wgu = t(f"l{l}.wgu")
        h = h + F.linear(F.silu(F.linear(b, wgu[0])) * F.linear(b, wgu[1]), t(f"l{l}.wdown"))
    return F.linear(F.rms_norm(h, (cfg.d_model,), t("norm_f"), cfg.rms_eps), t("unembed")).numpy()


def test_forward_no_prefix_causal_equals_torch_library_lm():
    W = weights(CFG)
    tok = np.array([3, 17, 17, 49, 0, 22, 8, 41, 5])
    ck, cv = empty_cache(CFG)
    out = O.forward(CFG, W, tok, np.arange(len(tok)), O.causal_mask(len(tok)), ck, cv)
    ref = torch_library_causal_lm(CFG, W, tok)
    assert np.abs(ref).max() > 1.0
    np.testing.assert_allclose(out.logits, ref, rtol=0, atol=1e-10)


def test_cache_split_equals_concatenated_causal_forward():
    """Causal invariance: prefix in the cache + causal window == one causal forward over both."""
    W = weights(CFG)
    tok = np.array([1, 9, 30, 2, 44, 13, 27, 6, 31, 12, 7])
    ck, cv = empty_cache(CFG)
    full = O.forward(CFG, W, tok, np.arange(len(tok)), O.causal_mask(len(tok)), ck, cv)
    s = 6
    pk, pv = O.prefill(CFG, W, tok[:s], chunk=4)
    for l in range(CFG.n_layers):
        np.testing.assert_allclose(pk[l], full.k[l][:s], atol=1e-12)
        np.testing.assert_allclose(pv[l], full.v[l][:s], atol=1e-12)
    tail = O.forward(CFG, W, tok[s:], s + np.arange(len(tok) - s), O.causal_mask(len(tok) - s), pk, pv)
    np.testing.assert_allclose(tail.logits, full.logits[s:], atol=1e-10)


def test_window_mask_is_respected_row_by_row():
    """A row's logits depend only on the rows it can see (checked by perturbing invisible tokens)."""
    W = weights(CFG)
    pk, pv = O.prefill(CFG, W, np.array([4, 8, 15, 16, 23]))
    rng = np.random.default_rng(0)
    vis = rng.random((5, 5)) < 0.5
    np.fill_diagonal(vis, True)
    vis = np.tril(vis)  # lower-triangular: dependence is then exactly the reachable set
    tok = np.array([11, 12, 13, 14, 15])
    base = O.forward(CFG, W, tok, 5 + np.arange(5), vis, pk, pv).logits
    reach = vis.copy()
    for _ in range(5):
        reach = reach | ((reach.astype(int) @ reach.astype(int)) > 0)
    for c in range(5):
        t2 = tok.copy()
        t2[c] = 33
        alt = O.forward(CFG, W, t2, 5 + np.arange(5), vis, pk, pv).logits
        for r in range(5):
            changed = np.abs(alt[r] - base[r]).max() > 1e-9
            assert changed == bool(reach[r, c]), (r, c)


def test_bidirectional_rows_with_equal_tokens_and_positions_are_exchangeable():
    W = weights(CFG)
    pk, pv = O.prefill(CFG, W, np.array([4, 8, 15]))
    tok = np.array([CFG.mask_id, 7, CFG.mask_id])
    out = O.forward(CFG, W, tok, np.array([3, 4, 3]), np.ones((3, 3), bool), pk, pv).logits
    np.testing.assert_allclose(out[0], out[2], atol=1e-12)
    assert np.abs(out[0] - out[1]).max() > 1e-3


def test_gqa_head_mapping_against_expanded_mha():
    """GQA with Hkv < Hq equals MHA whose K/V projections repeat each KV head Hq/Hkv times."""
    W = weights(CFG)
    D, Hq, Hkv = CFG.head_dim, CFG.n_q_heads, CFG.n_kv_heads
    mha = ModelCfg("mha", CFG.n_layers, CFG.d_model, Hq, Hq, D, CFG.d_ffn, CFG.vocab, dtype="f32", rope_theta=CFG.rope_theta)
    W2 = dict(W)
    for l in range(CFG.n_layers):
        w = W[f"l{l}.wqkv"]
        q, k, v = w[:Hq * D], w[Hq * D:(Hq + Hkv) * D], w[(Hq + Hkv) * D:]
        rep = lambda x: x.view(Hkv, D, -1).repeat_interleave(Hq // Hkv, dim=0).reshape(Hq * D, -1)
        W2[f"l{l}.wqkv"] = torch.cat([q, rep(k), rep(v)], dim=0)
    tok = np.array([5, 6, 7, 8])
    z = np.zeros((0, Hq, D))
    a = O.forward(CFG, W, tok, np.arange(4), np.ones((4, 4), bool), *empty_cache(CFG)).logits
    b = O.forward(mha, W2, tok, np.arange(4), np.ones((4, 4), bool), [z] * 2, [z] * 2).logits
    np.testing.assert_allclose(a, b, atol=1e-11)


def test_rope_is_a_rotation_with_relative_phase():
    rng = np.random.default_rng(1)
    q, k = rng.standard_normal((1, 1, 16)), rng.standard_normal((1, 1, 16))
    dots = []
    for m, n in [(0, 0), (5, 5), (100, 100)]:
        dots.append(np.sum(O.rope(q, [m], 1e4) * O.rope(k, [n], 1e4)))
    np.testing.assert_allclose(dots, dots[0], atol=1e-12)  # depends on m-n only
    a = np.sum(O.rope(q, [7], 1e4) * O.rope(k, [3], 1e4))
    b = np.sum(O.rope(q, [4], 1e4) * k)
    np.testing.assert_allclose(a, b, atol=1e-12)
    np.testing.assert_allclose(np.linalg.norm(O.rope(q, [9], 1e4)), np.linalg.norm(q), atol=1e-12)
    np.testing.assert_allclose(O.rope(q, [0], 1e4), q, atol=0)
    # first pair (i=0, i+D/2) rotates by exactly pos radians (frequency theta^0 = 1)
    e = np.zeros((1, 1, 16)); e[0, 0, 0] = 1.0
    r = O.rope(e, [2], 1e4)[0, 0]
    np.testing.assert_allclose([r[0], r[8]], [np.cos(2.0), np.sin(2.0)], atol=1e-15)
    # last pair uses frequency theta^{-(D-2)/D}
    e = np.zeros((1, 1, 16)); e[0, 0, 7] = 1.0
    r = O.rope(e, [3], 1e4)[0, 0]
    w = 1e4 ** (-14.0 / 16.0)
    np.testing.assert_allclose([r[7], r[15]], [np.cos(3 * w), np.sin(3 * w)], atol=1e-15)


def test_rmsnorm_unit_rms_and_softmax_rows():
    x = np.random.default_rng(2).standard_normal((3, 64)) * 5
    y = O.rmsnorm(x, np.ones(64), 0.0)
    np.testing.assert_allclose(np.sqrt((y * y).mean(-1)), 1.0, atol=1e-12)
    np.testing.assert_allclose(O.rmsnorm(x, np.full(64, 2.0), 0.0), 2 * y, atol=1e-12)
    s = O.softmax_rows(x)
    np.testing.assert_allclose(s, torch.softmax(torch.from_numpy(x), -1).numpy(), atol=1e-14)


def test_moe_identical_experts_is_the_dense_ffn():
    W = weights(MOE)
    dense = ModelCfg("d", MOE.n_layers, MOE.d_model, MOE.n_q_heads, MOE.n_kv_heads, MOE.head_dim, MOE.d_expert,
                     MOE.vocab, dtype="f32", rope_theta=MOE.rope_theta)
    Wd = dict(W)
    for l in range(MOE.n_layers):
        W[f"l{l}.e_wgu"] = W[f"l{l}.e_wgu"][:1].expand(MOE.n_experts, -1, -1, -1).contiguous()
        W[f"l{l}.e_wdown"] = W[f"l{l}.e_wdown"][:1].expand(MOE.n_experts, -1, -1).contiguous()
        Wd[f"l{l}.wgu"], Wd[f"l{l}.wdown"] = W[f"l{l}.e_wgu"][0], W[f"l{l}.e_wdown"][0]
    tok = np.array([1, 2, 3])
    a = O.forward(MOE, W, tok, np.arange(3), O.causal_mask(3), *empty_cache(MOE)).logits
    b = O.forward(dense, Wd, tok, np.arange(3), O.causal_mask(3), *empty_cache(MOE)).logits
    np.testing.assert_allclose(a, b, atol=1e-11)


def test_moe_all_experts_equal_router_is_the_mean_of_experts():
    rng = np.random.default_rng(5)
    b = rng.standard_normal((3, 8))
    router = np.zeros((4, 8))
    wgu, wd = rng.standard_normal((4, 2, 6, 8)), rng.standard_normal((4, 8, 6))
    y, chosen = O.moe_ffn(b, router, wgu, wd, top_k=4)
    ref = np.mean([O.dense_ffn(b, wgu[e], wd[e]) for e in range(4)], axis=0)
    np.testing.assert_allclose(y, ref, atol=1e-12)
    assert (chosen == np.arange(4)).all()  # all tied: lowest index first


def test_moe_topk_picks_largest_router_scores_and_renormalises():
    b = np.eye(4)[:1] * 1.0
    router = np.array([[0.0], [3.0], [1.0], [2.0]]) * np.eye(4)[0][None, :]
    rng = np.random.default_rng(6)
    wgu, wd = rng.standard_normal((4, 2, 5, 4)), rng.standard_normal((4, 4, 5))
    y, chosen = O.moe_ffn(b, router, wgu, wd, top_k=2)
    assert list(chosen[0]) == [1, 3]
    w = np.exp([3.0, 2.0]); w /= w.sum()
    ref = w[0] * O.dense_ffn(b, wgu[1], wd[1]) + w[1] * O.dense_ffn(b, wgu[3], wd[3])
    np.testing.assert_allclose(y, ref, atol=1e-12)


def test_dense_ffn_against_torch():
    rng = np.random.default_rng(7)
    b, wgu, wd = rng.standard_normal((2, 8)), rng.standard_normal((2, 6, 8)), rng.standard_normal((8, 6))
    tb, tg, td = map(torch.from_numpy, (b, wgu, wd))
    ref = F.linear(F.silu(F.linear(tb, tg[0])) * F.linear(tb, tg[1]), td).numpy()
    np.testing.assert_allclose(O.dense_ffn(b, wgu, wd), ref, atol=1e-12)

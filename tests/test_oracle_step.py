"""Pins for the oracle's S2D2 logic: masks (Eq. 3, Eq. 4), windows, SampleFromLogits,
the accept / residual law, the threshold rule, cache append and block roll-over."""
import itertools
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import s2d2_oracle as O
from s2d2_inputs import ModelCfg, gen_weights

CFG = ModelCfg("pin", n_layers=2, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=96, vocab=50,
               dtype="f32", rope_theta=10000.0)
MASK = CFG.mask_id


@pytest.fixture(scope="module")
def model():
    W = gen_weights(CFG, seed=11, unembed_gain=10.0, norm_jitter=0.2)
    prefix = np.array([4, 8, 15, 16, 23, 42, 7])
    ck, cv = O.prefill(CFG, W, prefix)
    return W, prefix, ck, cv


def fresh(prefix_len, B):
    return O.SeqState(seq_len=prefix_len, pos0=prefix_len, block=np.full(B, MASK, dtype=np.int64))


# ---------------------------------------------------------------- masks
def test_eq3_literal_blocks():
    for L in range(1, 5):
        m = O.verify_mask(L)
        for r, c in itertools.product(range(L), range(L)):
            assert m[r, c] == (c <= r)            # A_L
            assert not m[r, L + c]                # 0_L
            assert m[L + r, c] == (c < r)         # strictly lower part of A_L
            assert m[L + r, L + c] == (r == c)    # I_L
    assert O.verify_mask(2).astype(int).tolist() == [[1, 0, 0, 0], [1, 1, 0, 0], [0, 0, 1, 0], [1, 0, 0, 1]]


def test_eq4_limits_and_blocks():
    B = 5
    assert O.draft_mask(B, 0).all()
    assert (O.draft_mask(B, B) == O.causal_mask(B)).all()
    m = O.draft_mask(B, 2)
    assert m.astype(int).tolist() == [[1, 0, 0, 0, 0], [1, 1, 0, 0, 0], [1, 1, 1, 1, 1], [1, 1, 1, 1, 1], [1, 1, 1, 1, 1]]


def test_fresh_block_windows_are_eq4_j0_and_eq3():
    st = fresh(7, 4)
    dw = O.draft_window(st, MASK)
    assert dw.vis.all() and (dw.tokens == MASK).all() and list(dw.pos) == [7, 8, 9, 10]
    assert (dw.j, dw.L) == (0, 4) and list(dw.logit_rows) == [0, 1, 2, 3]
    vw = O.verify_window(st, np.array([10, 11, 12, 13]), MASK)
    assert (vw.vis == O.verify_mask(4)).all()
    assert list(vw.tokens) == [10, 11, 12, 13] + [MASK] * 4
    assert list(vw.pos) == [7, 8, 9, 10, 7, 8, 9, 10]      # MASK copies sit at the same positions
    assert list(vw.logit_rows) == [4, 5, 6, 7] and vw.n_causal == 4


def test_windows_mid_block_with_pending_and_carry():
    # block of 6: index 0 cached, 1..2 committed but uncached, 3..4 masked, 5 committed (earlier fallback step)
    st = O.SeqState(seq_len=11, pos0=10, block=np.array([9, 8, 7, MASK, MASK, 6]))
    assert O.first_span(st.block, MASK) == (3, 2)
    dw = O.draft_window(st, MASK)
    assert list(dw.tokens) == [8, 7, MASK, MASK, 6] and list(dw.pos) == [11, 12, 13, 14, 15]
    assert (dw.vis == O.draft_mask(6, 3)[1:, 1:]).all()
    assert list(dw.logit_rows) == [2, 3] and list(dw.logit_index) == [3, 4]
    assert O.draft_window(st, MASK, ar_mask=False).vis.all()
    vw = O.verify_window(st, np.array([-1, -1, -1, 30, 31, -1]), MASK)
    assert list(vw.tokens) == [8, 7, 30, 31, MASK, MASK] and list(vw.pos) == [11, 12, 13, 14, 13, 14]
    exp = np.array([[1, 0, 0, 0, 0, 0], [1, 1, 0, 0, 0, 0], [1, 1, 1, 0, 0, 0], [1, 1, 1, 1, 0, 0],
                    [1, 1, 0, 0, 1, 0], [1, 1, 1, 0, 0, 1]], dtype=bool)
    assert (vw.vis == exp).all() and vw.n_causal == 4
    # carried tokens of the previous block: causal among themselves, visible to the whole block
    st2 = O.SeqState(seq_len=8, pos0=10, block=np.array([MASK, MASK]), carry=np.array([5, 6]))
    dw2 = O.draft_window(st2, MASK)
    assert list(dw2.tokens) == [5, 6, MASK, MASK] and list(dw2.pos) == [8, 9, 10, 11]
    assert dw2.vis.astype(int).tolist() == [[1, 0, 0, 0], [1, 1, 0, 0], [1, 1, 1, 1], [1, 1, 1, 1]]
    vw2 = O.verify_window(st2, np.array([20, 21]), MASK)
    assert list(vw2.tokens) == [5, 6, 20, 21, MASK, MASK] and list(vw2.pos) == [8, 9, 10, 11, 10, 11]
    assert vw2.vis[4].astype(int).tolist() == [1, 1, 0, 0, 1, 0]
    assert vw2.vis[5].astype(int).tolist() == [1, 1, 1, 0, 0, 1]


# ---------------------------------------------------------------- drafter == verifier at block size 1
def test_block_size_one_draft_equals_verify_and_is_accepted(model):
    W, prefix, ck, cv = model
    st = fresh(len(prefix), 1)
    d = O.draft(CFG, W, st, ck, cv, tau=0.9)
    vo = O.verify(CFG, W, st, ck, cv, d.xhat)
    np.testing.assert_allclose(vo.logits, d.logits, atol=1e-12)
    np.testing.assert_allclose(vo.q, d.p[:1], atol=1e-14)
    for seed in range(20):
        a = O.accept(st, d, vo, seed=seed, step=0, seq=0)
        assert a.n_accept == 1 and a.resampled == -1 and a.block[0] == d.xhat[0]


def test_2L_parallel_verify_equals_sequential_block_size_one_decoding(model):
    """Verifier row i must equal a literal block-size-1 forward: [MASK] at position i with the
    causally computed K/V of the drafted tokens left of i appended to the cache."""
    W, prefix, ck, cv = model
    st = fresh(len(prefix), 4)
    d = O.draft(CFG, W, st, ck, cv, tau=0.9)
    vo = O.verify(CFG, W, st, ck, cv, d.xhat)
    k, v = [c.copy() for c in ck], [c.copy() for c in cv]
    S = len(prefix)
    for i in range(4):
        one = O.forward(CFG, W, np.array([MASK]), np.array([S + i]), np.ones((1, 1), bool), k, v)
        np.testing.assert_allclose(one.logits[0], vo.logits[i], atol=1e-10)
        tok = O.forward(CFG, W, np.array([d.xhat[i]]), np.array([S + i]), np.ones((1, 1), bool), k, v)
        for l in range(CFG.n_layers):
            np.testing.assert_allclose(tok.k[l][0], vo.k[l][i], atol=1e-12)
            k[l] = np.concatenate([k[l], tok.k[l]]); v[l] = np.concatenate([v[l], tok.v[l]])
    # draft (bidirectional over MASKs) is a different view from the verifier except at ... nowhere in general
    assert np.abs(vo.logits - d.logits).max() > 1e-6


def test_append_then_forward_equals_forward_over_concatenation(model):
    W, prefix, ck, cv = model
    st = fresh(len(prefix), 4)
    d = O.draft(CFG, W, st, ck, cv, tau=0.9)
    vo = O.verify(CFG, W, st, ck, cv, d.xhat)
    k, v = list(ck), list(cv)
    rows = O.kv_append(st, k, v, vo, n_accept=3)
    assert rows == 3 and st.seq_len == len(prefix) + 3
    seq = np.concatenate([prefix, d.xhat[:3]])
    k2, v2 = O.prefill(CFG, W, seq, chunk=5)
    for l in range(CFG.n_layers):
        np.testing.assert_allclose(k[l], k2[l], atol=1e-11)
        np.testing.assert_allclose(v[l], v2[l], atol=1e-11)


# ---------------------------------------------------------------- SampleFromLogits / ScoreFromLogits
def test_sample_from_logits_greedy_against_torch():
    rng = np.random.default_rng(0)
    l = rng.standard_normal(97) * 3
    s = O.sample_from_logits(l)
    P = torch.softmax(torch.from_numpy(l), 0)
    assert s["xhat"] == int(torch.argmax(P))
    np.testing.assert_allclose(s["p"], float(P.max()), atol=1e-14)
    np.testing.assert_allclose(s["lse"], float(torch.logsumexp(torch.from_numpy(l), 0)), atol=1e-12)
    top2 = torch.topk(P, 2).values
    np.testing.assert_allclose(s["margin"], float(top2[0] - top2[1]), atol=1e-14)
    H = float(torch.distributions.Categorical(probs=P).entropy())
    np.testing.assert_allclose(s["entropy_n"], H / np.log(97), atol=1e-12)
    q, lse = O.score_from_logits(l, 5)
    np.testing.assert_allclose(q, float(P[5]), atol=1e-14)


def test_sample_from_logits_special_rows():
    u = O.sample_from_logits(np.zeros(8))                       # uniform row
    assert u["xhat"] == 0 and abs(u["p"] - 1 / 8) < 1e-15 and abs(u["entropy_n"] - 1) < 1e-12 and u["margin"] == 0
    t = O.sample_from_logits(np.array([0.0, 5.0, 5.0, 1.0]))      # tie: lowest index
    assert t["xhat"] == 1 and t["margin"] == 0
    o = O.sample_from_logits(np.array([0.0, 800.0, 0.0]))        # one-hot, no overflow
    assert o["xhat"] == 1 and o["p"] == 1.0 and o["entropy_n"] == 0.0


def test_sample_mode_inverse_cdf_law():
    l = np.array([0.3, -1.0, 2.0, 0.0])
    for T in (1.0, 0.5):
        P = np.exp(l / T) / np.exp(l / T).sum()
        us = (np.arange(20000) + 0.5) / 20000
        xs = np.array([O.sample_from_logits(l, O.SAMPLE, T, u)["xhat"] for u in us])
        np.testing.assert_allclose(np.bincount(xs, minlength=4) / len(us), P, atol=1e-4)
        s = O.sample_from_logits(l, O.SAMPLE, T, 0.999)
        assert s["xhat"] == 3 and abs(s["p"] - P[3]) < 1e-15
    assert O.inverse_cdf(np.array([0.0, 1.0, 0.0, 1.0]), 0.5) == 3       # boundary: strictly greater
    assert O.inverse_cdf(np.array([0.0, 1.0, 0.0, 1.0]), 0.4999) == 1
    assert O.inverse_cdf(np.array([0.0, 0.0, 2.0]), 1e-9) == 2


# ---------------------------------------------------------------- accept / residual
def test_q_equals_p_accepts_everything_and_ratio_above_one_too():
    p = np.array([0.3, 0.9, 1e-6, 0.5])
    for u in (1e-9, 0.5, 1 - 2 ** -24):
        assert O.accept_scan(p, p * (1 + 1e-12), np.full(4, u)) == 4
        assert O.accept_scan(p, np.minimum(1.0, p * 3), np.full(4, u)) == 4
    assert O.accept_scan(p, p, np.full(4, 1 - 2 ** -24)) == 4  # u < 1 = min(1, q/p)


def test_accept_scan_stops_at_first_failure_and_energy_identity():
    rng = np.random.default_rng(1)
    for _ in range(200):
        L = rng.integers(1, 8)
        p, q, u = rng.uniform(0.01, 1, L), rng.uniform(0.01, 1, L), rng.uniform(0, 1, L)
        n = O.accept_scan(p, q, u)
        ratio_rule = [ui < min(1.0, qi / pi) for pi, qi, ui in zip(p, q, u)]
        energy_rule = [ui < min(1.0, np.exp(-(-np.log(qi) + np.log(pi)))) for pi, qi, ui in zip(p, q, u)]  # Eq. 8
        assert ratio_rule == energy_rule
        first_fail = ratio_rule.index(False) if False in ratio_rule else L
        assert n == first_fail
        # gamma = 1 through the tempered branch gives the same count
        assert O.accept_scan(p, q, u, gamma=1.0 + 1e-15) == n


def test_tempered_ratio_is_the_plain_rule_on_transformed_uniforms():
    """Ratio tempering (appendix on tempering the acceptance ratio): u < min(1, (q/p)^gamma) holds exactly when
    u^(1/gamma) < min(1, q/p), so the tempered scan on u is the plain scan on u^(1/gamma); gamma = 0 accepts
    everything; for a fixed u a larger gamma never accepts more."""
    rng = np.random.default_rng(5)
    for _ in range(300):
        L = int(rng.integers(1, 8))
        p, q, u = rng.uniform(0.01, 1, L), rng.uniform(0.01, 1, L), rng.uniform(1e-6, 1, L)
        for gamma, root in ((2.0, np.sqrt(u)), (0.5, u * u), (4.0, np.sqrt(np.sqrt(u)))):
            # (skip draws where the two sides of a comparison round to the same number)
            if np.any(np.abs(root * p - q) < 1e-12):
                continue
            assert O.accept_scan(p, q, u, gamma=gamma) == O.accept_scan(p, q, root)
        assert O.accept_scan(p, q, u, gamma=0.0) == L
        counts = [O.accept_scan(p, q, u, gamma=g) for g in (0.0, 0.25, 0.5, 1.0, 2.0, 8.0)]
        assert counts == sorted(counts, reverse=True)


def test_tempered_acceptance_frequency_on_a_uniform_grid():
    """One position, u on the midpoint grid of (0, 1): the accepted share is min(1, (q/p)^gamma) to 1/K; the
    exponent is written as repeated multiplication / square roots, not as the oracle's power."""
    K = 4000
    u = (np.arange(K) + 0.5) / K
    for p1, q1 in ((0.8, 0.2), (0.5, 0.45), (0.3, 0.9)):
        r = min(1.0, q1 / p1)
        for gamma, want in ((2.0, r * r), (3.0, r * r * r), (0.5, np.sqrt(r)), (1.0, r)):
            share = np.mean([O.accept_scan(np.array([p1]), np.array([q1]), np.array([ui]), gamma=gamma) for ui in u])
            assert abs(share - want) <= 1.0 / K + 1e-12


def test_reject_only_keeps_the_accepted_prefix_and_commits_nothing_else(model):
    """Reject-only variant (no residual resample): same accepted prefix as the full rule, the rejected position stays
    masked, nothing is drawn, and the committed count is the accepted count (possibly zero)."""
    W, prefix, ck, cv = model
    seen_reject = 0
    for seed in range(12):
        st = fresh(len(prefix), 4)
        d = O.draft(CFG, W, st, ck, cv, tau=0.9)
        xhat = np.array(d.xhat, copy=True)
        xhat[1] = (xhat[1] + 1 + seed) % (CFG.vocab - 1)      # a drafted token the verifier will mostly refuse
        d.xhat = xhat
        d.p = np.array(d.p, copy=True)
        d.p[1] = 0.999
        vo = O.verify(CFG, W, st, ck, cv, xhat)
        full = O.accept(st, d, vo, seed, 0, 0)
        ro = O.accept(st, d, vo, seed, 0, 0, resample=False)
        j, L = vo.win.j, vo.win.L
        assert ro.n_accept == full.n_accept and ro.resampled == -1 and ro.n_commit == ro.n_accept
        assert np.array_equal(ro.block[j:j + ro.n_accept], xhat[j:j + ro.n_accept])
        assert np.all(ro.block[j + ro.n_accept:] == MASK)
        assert np.array_equal(ro.u, full.u)
        if full.n_accept < L:
            seen_reject += 1
            assert full.n_commit == ro.n_commit + 1 and full.block[j + full.n_accept] == full.resampled
    assert seen_reject >= 6


def test_speculative_step_preserves_the_verifier_law_exact_rational():
    """First-position law: sum_x P(x) min(1,Q/P)(x) 1[x=v] + P(reject) * residual(v) == Q(v), exactly."""
    rng = np.random.default_rng(2)
    for V in range(2, 9):
        a, b = rng.integers(1, 20, V), rng.integers(0, 20, V)
        b[rng.integers(V)] += 1
        P = [Fraction(int(x), int(a.sum())) for x in a]
        Q = [Fraction(int(x), int(b.sum())) for x in b]
        acc = [P[v] * min(Fraction(1), Q[v] / P[v]) for v in range(V)]
        rej = 1 - sum(acc)
        res = [max(Fraction(0), Q[v] - P[v]) for v in range(V)]
        Z = sum(res)
        law = [acc[v] + (rej * res[v] / Z if Z else 0) for v in range(V)]
        assert law == Q
        # the oracle's residual is that same vector (fp64), and its normaliser equals P(reject)
        r = O.residual_distribution(np.log([float(x) for x in P]), np.log(np.maximum([float(x) for x in Q], 1e-300)))
        np.testing.assert_allclose(r, [float(x) for x in res], atol=1e-15)
        np.testing.assert_allclose(r.sum(), float(rej), atol=1e-14)


def test_speculative_step_law_by_enumerating_uniforms_through_the_oracle():
    """Drive the oracle's own accept_scan / residual_resample / sample_from_logits over a grid of
    (u_draft, u_accept, u_resample): the committed first token must follow softmax(l_ver)."""
    ld = np.array([0.2, 1.5, -0.7, 0.9, 0.0])
    lv = np.array([1.1, 0.3, 0.4, -0.5, 0.8])
    P, Q = np.exp(ld) / np.exp(ld).sum(), np.exp(lv) / np.exp(lv).sum()
    G = 64
    grid = (np.arange(G) + 0.5) / G
    counts = np.zeros(5)
    for ud in grid:
        s = O.sample_from_logits(ld, O.SAMPLE, 1.0, ud)
        q, _ = O.score_from_logits(lv, s["xhat"])
        for ua in grid:
            if O.accept_scan([s["p"]], [q], [ua]) == 1:
                counts[s["xhat"]] += G
            else:
                for ur in grid:
                    counts[O.residual_resample(ld, lv, ur)] += 1
    np.testing.assert_allclose(counts / G ** 3, Q, atol=2.5 / G)
    assert np.abs(P - Q).max() > 0.1  # the test distinguishes Q from P


def test_residual_one_hot_verifier_and_rejection_has_mass():
    ld = np.array([2.0, 0.0, 1.0, -1.0])
    lv = np.array([-50.0, -50.0, -50.0, 50.0])  # verifier ~ one-hot on 3, drafter proposed 0
    for u in (1e-6, 0.3, 0.999999):
        assert O.residual_resample(ld, lv, u) == 3
    rng = np.random.default_rng(3)
    for _ in range(100):
        ld, lv = rng.standard_normal(6) * 2, rng.standard_normal(6) * 2
        s = O.sample_from_logits(ld)
        q, _ = O.score_from_logits(lv, s["xhat"])
        if q < s["p"]:
            r = O.residual_distribution(ld, lv)
            assert r.sum() >= s["p"] - q - 1e-15 and r[s["xhat"]] == 0.0
            assert O.residual_resample(ld, lv, 0.5) != s["xhat"]


# ---------------------------------------------------------------- threshold rule (Alg. 2)
def test_threshold_set_monotone_nonempty_and_static_limit():
    rng = np.random.default_rng(4)
    for _ in range(100):
        B = rng.integers(1, 12)
        p = rng.uniform(0, 1, B)
        masked = rng.uniform(size=B) < 0.7
        prev = None
        for tau in (0.0, 0.3, 0.7, 0.9, 0.95, 1.0):
            S, n_hi = O.threshold_set(p, masked, tau)
            assert not (S & ~masked).any()
            assert S.sum() >= (1 if masked.any() else 0)
            assert n_hi == int((masked & (p > tau)).sum())
            if prev is not None:
                assert not (S & ~prev).any()  # tau1 < tau2  =>  S(tau1) contains S(tau2)
            prev = S
        S1, n1 = O.threshold_set(p, masked, 1.0)  # static decoding: exactly the arg-max position
        if masked.any():
            assert S1.sum() == 1 and n1 == 0 and S1[np.argmax(np.where(masked, p, -1))]
    S, _ = O.threshold_set(np.array([0.5, 0.5, 0.2]), np.array([True, True, True]), 0.9)
    assert S.tolist() == [True, False, False]  # tie: lowest index


# ---------------------------------------------------------------- full step bookkeeping
def test_step_commits_at_least_one_token_and_keeps_invariants(model):
    W, prefix, ck0, cv0 = model
    for seed in range(6):
        st = fresh(len(prefix), 4)
        ck, cv = list(ck0), list(cv0)
        toks = list(prefix)
        for s in range(7):
            before_masks = int((st.block == MASK).sum())
            d, vo, a = O.step(CFG, W, st, ck, cv, tau=0.9, seed=seed, step_idx=s)
            assert a.n_commit >= 1 and a.n_commit == a.n_accept + (a.resampled >= 0)
            assert a.n_accept <= vo.win.L
            assert (a.resampled >= 0) == (a.n_accept < vo.win.L)
            if a.resampled >= 0:
                assert a.resampled != d.xhat[vo.win.j + a.n_accept]
            assert ck[0].shape[0] == st.seq_len
            assert st.seq_len + len(st.carry) == st.pos0 or (len(st.carry) == 0 and st.seq_len >= st.pos0)
            # the cache always holds causally computed K of the committed sequence
        committed = int(st.seq_len)
        assert committed > len(prefix)


def test_cache_after_steps_equals_causal_prefill_of_committed_tokens(model):
    """AR caching: whatever was appended over several steps (including carried tokens across a
    block boundary) equals a causal prefill of the committed token sequence."""
    W, prefix, ck0, cv0 = model
    st = fresh(len(prefix), 3)
    ck, cv = list(ck0), list(cv0)
    seq = list(prefix)
    for s in range(9):
        pos0_before, block_before = st.pos0, None
        d, vo, a = O.step(CFG, W, st, ck, cv, tau=0.9, seed=5, step_idx=s)
        # reconstruct committed sequence: cached tokens are the causal verify rows appended
        n_lead = vo.win.n_causal - vo.win.L
        seq += list(vo.win.tokens[: n_lead + a.n_accept])
    assert len(seq) == st.seq_len
    k2, v2 = O.prefill(CFG, W, np.array(seq), chunk=6)
    for l in range(CFG.n_layers):
        np.testing.assert_allclose(ck[l], k2[l], atol=1e-10)
        np.testing.assert_allclose(cv[l], v2[l], atol=1e-10)
    assert st.pos0 > len(prefix)  # at least one block boundary was crossed


def test_block_advance_carries_uncached_tokens():
    st = O.SeqState(seq_len=12, pos0=10, block=np.array([1, 2, 3, 4]))
    assert O.block_advance(st, MASK)
    assert list(st.carry) == [3, 4] and st.pos0 == 14 and (st.block == MASK).all()
    st = O.SeqState(seq_len=10, pos0=10, block=np.array([1, MASK, 3, 4]))
    assert not O.block_advance(st, MASK)


def test_fallback_branch_commits_threshold_set(model):
    W, prefix, ck, cv = model
    st = fresh(len(prefix), 4)
    d = O.draft(CFG, W, st, ck, cv, tau=0.0)
    n = O.commit_threshold(st, d)
    assert n == 4 and (st.block == d.xhat).all()
    st = fresh(len(prefix), 4)
    d = O.draft(CFG, W, st, ck, cv, tau=1.0)
    assert O.commit_threshold(st, d) == 1
    i = int(np.argmax(d.p))
    assert st.block[i] == d.xhat[i] and (np.delete(st.block, i) == MASK).all()

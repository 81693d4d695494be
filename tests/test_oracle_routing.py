"""Pins for the oracle's verification routing (Section 4.3: expected accepted prefix length Eq. 5,
static / dynamic score, and the minimum-span, score-threshold and hysteresis policies of the
DoVerify algorithm).  Each pin is something other than the oracle's own formula: the definition of
an expectation enumerated over all outcomes, closed forms, library routines, hand-traced state
sequences."""
import copy
import itertools
import math

import numpy as np
import pytest

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


# ---------------------------------------------------------------- Eq. 5
def test_expected_prefix_length_is_the_expectation_over_all_accept_reject_outcomes():
    # If position i is accepted independently with probability alpha_i and the scan stops at the first
    # failure, the number of accepted tokens is the index of the first failure.  Enumerate all 2^L outcomes.
    rng = np.random.default_rng(5)
    for L in range(0, 9):
        alpha = rng.uniform(0.0, 1.0, L)
        expect = 0.0
        for outcome in itertools.product([0, 1], repeat=L):
            pr = 1.0
            for i, ok in enumerate(outcome):
                pr *= alpha[i] if ok else 1.0 - alpha[i]
            prefix = next((i for i, ok in enumerate(outcome) if not ok), L)
            expect += pr * prefix
        assert O.expected_prefix_length(alpha) == pytest.approx(expect, abs=1e-12)


def test_expected_prefix_length_closed_forms():
    assert O.expected_prefix_length(np.ones(7)) == 7.0                      # every product is 1
    assert O.expected_prefix_length(np.zeros(0)) == 0.0
    assert O.expected_prefix_length(np.array([0.0, 1.0, 1.0])) == 0.0       # a zero first factor kills every product
    assert O.expected_prefix_length(np.array([1.0, 1.0, 0.0, 1.0])) == 2.0  # products 1, 1, 0, 0
    for a, L in [(0.5, 6), (0.9, 12), (0.25, 3)]:                           # geometric sum
        assert O.expected_prefix_length(np.full(L, a)) == pytest.approx(a * (1 - a ** L) / (1 - a), rel=1e-13)
    # library routine: cumulative products summed
    al = np.random.default_rng(1).uniform(0.2, 1.0, 16)
    assert O.expected_prefix_length(al) == pytest.approx(float(np.cumprod(al).sum()), rel=1e-13)
    # order matters: the weak position first costs more than the weak position last
    assert O.expected_prefix_length(np.array([0.1, 1.0, 1.0])) < O.expected_prefix_length(np.array([1.0, 1.0, 0.1]))


def test_acceptance_proxies():
    V = 64
    # entropy proxy on the two extreme distributions, through the oracle's own draft statistics
    uniform_row = O.sample_from_logits(np.zeros(V))
    peaked_row = O.sample_from_logits(np.array([200.0] + [0.0] * (V - 1)))
    assert uniform_row["entropy_n"] == pytest.approx(1.0, abs=1e-12)   # H = ln V
    assert peaked_row["entropy_n"] == pytest.approx(0.0, abs=1e-12)
    ent = np.array([uniform_row["entropy_n"], peaked_row["entropy_n"], 0.5])
    a = O.acceptance_proxy(np.zeros(3), ent, O.EST_ENTROPY, 0.5, beta=2.0)
    assert a == pytest.approx([math.exp(-2.0), 1.0, math.exp(-1.0)], rel=1e-13)
    assert (O.acceptance_proxy(np.zeros(3), ent, O.EST_ENTROPY, 0.5, beta=0.0) == 1.0).all()
    # margin proxy: indicator with a closed threshold; K is then the count of leading confident positions
    m = np.array([0.9, 0.5, 0.49999, 0.8])
    a = O.acceptance_proxy(m, np.zeros(4), O.EST_MARGIN, 0.5, beta=1.0)
    assert a.tolist() == [1.0, 1.0, 0.0, 1.0]
    assert O.expected_prefix_length(a) == 2.0
    # top-1 minus top-2 probability of a three-way row, by hand
    row = O.sample_from_logits(np.log(np.array([0.6, 0.3, 0.1])))
    assert row["margin"] == pytest.approx(0.3, abs=1e-12)


def test_scores():
    assert O.verify_score(3.5, n_hi=4, c=0.5, dynamic=False) == 3.0
    assert O.verify_score(3.5, n_hi=4, c=0.5, dynamic=True) == 1.5
    assert O.verify_score(3.5, n_hi=0, c=7.0, dynamic=True) == 3.5


# ---------------------------------------------------------------- policies
def test_minimum_span_policy_special_settings():
    B = 8
    always = O.RouteParams(policy=O.ROUTE_MIN_SPAN, tau_span=1)
    first_only = O.RouteParams(policy=O.ROUTE_MIN_SPAN, tau_span=B)
    for L in range(1, B + 1):
        assert O.do_verify(always, L, -1e9, O.H_OFF) == (True, O.H_OFF)     # ignores score and state
        assert O.do_verify(first_only, L, 1e9, O.H_ON)[0] == (L == B)
    assert O.do_verify(always, 0, 0.0, O.H_ON)[0] is False                   # nothing masked: nothing to verify


def test_score_threshold_policy_is_closed_at_the_threshold():
    rp = O.RouteParams(policy=O.ROUTE_SCORE, tau_score=1.25)
    assert O.do_verify(rp, 3, 1.25, O.H_OFF)[0] is True
    assert O.do_verify(rp, 3, np.nextafter(1.25, 0.0), O.H_ON)[0] is False


def test_hysteresis_trace_and_reduction_to_a_plain_threshold():
    rp = O.RouteParams(policy=O.ROUTE_HYSTERESIS, tau_on=1.0, tau_off=-5.0)
    scores = [2.0, 0.0, -5.0, -5.000001, 0.0, 0.999, 1.0, -4.9, -6.0, 3.0]
    want = [1, 1, 1, 0, 0, 0, 1, 1, 0, 1]          # traced by hand: leaves ON only below -5, returns at >= 1
    h, got = O.H_ON, []
    for s in scores:
        dec, h = O.do_verify(rp, 4, s, h)
        got.append(int(dec))
        assert dec == (h == O.H_ON)
    assert got == want
    # equal thresholds: the state carries no memory, the policy is the score threshold
    eq = O.RouteParams(policy=O.ROUTE_HYSTERESIS, tau_on=0.3, tau_off=0.3)
    th = O.RouteParams(policy=O.ROUTE_SCORE, tau_score=0.3)
    rng = np.random.default_rng(2)
    for h0 in (O.H_ON, O.H_OFF):
        h = h0
        for s in rng.normal(0.3, 1.0, 200):
            dec, h = O.do_verify(eq, 2, s, h)
            assert dec == O.do_verify(th, 2, s, 0)[0]
    # the band holds the state: scores strictly inside (tau_off, tau_on) never change it
    for h0 in (O.H_ON, O.H_OFF):
        h = h0
        for s in rng.uniform(-4.99, 0.99, 100):
            _, h = O.do_verify(rp, 4, s, h)
            assert h == h0


# ---------------------------------------------------------------- the routed step
def test_routed_step_with_always_verify_is_the_verified_step(model):
    W, prefix, ck, cv = model
    a_st, b_st = fresh(len(prefix), 4), fresh(len(prefix), 4)
    a_k, a_v, b_k, b_v = list(ck), list(cv), list(ck), list(cv)
    rp = O.RouteParams(policy=O.ROUTE_MIN_SPAN, tau_span=1)
    for t in range(3):
        d1, v1, acc1 = O.step(CFG, W, a_st, a_k, a_v, 0.9, seed=3, step_idx=t)
        d2, r, v2, acc2 = O.step_routed(CFG, W, b_st, b_k, b_v, 0.9, seed=3, step_idx=t, rp=rp)
        assert r["verify"] and acc2.n_accept == acc1.n_accept and acc2.resampled == acc1.resampled
        assert (a_st.block == b_st.block).all() and a_st.seq_len == b_st.seq_len
        assert all(np.array_equal(x, y) for x, y in zip(a_k, b_k))


def test_routed_step_that_never_verifies_is_threshold_decoding(model):
    W, prefix, ck, cv = model
    st = fresh(len(prefix), 4)
    k, v = list(ck), list(cv)
    rp = O.RouteParams(policy=O.ROUTE_MIN_SPAN, tau_span=5)        # longer than any span of a 4-block
    before = copy.deepcopy(st)
    d, r, vo, acc = O.step_routed(CFG, W, st, k, v, 0.9, seed=3, step_idx=0, rp=rp)
    assert not r["verify"] and vo is None and acc is None
    want = np.where(d.unmask, d.xhat, before.block)                 # Alg. 2: exactly the threshold set is written
    if (want != MASK).all():                                        # a finished block rolls over
        assert (st.block == MASK).all() and st.pos0 == before.pos0 + 4
    else:
        assert (st.block == want).all()
    assert st.seq_len == before.seq_len and all(np.array_equal(x, y) for x, y in zip(k, ck))   # nothing appended
    assert d.unmask.sum() >= 1                                      # progress: the arg-max position is always in the set


def test_route_record_matches_its_parts(model):
    W, prefix, ck, cv = model
    st = fresh(len(prefix), 4)
    st.block[0] = 9                                                  # span starts at 1
    d = O.draft(CFG, W, st, ck, cv, 0.5)
    rp = O.RouteParams(policy=O.ROUTE_SCORE, estimator=O.EST_ENTROPY, dynamic=True, c=0.25, beta=3.0, tau_score=0.1)
    r = O.route(st, d, MASK, rp, O.H_ON)
    al = np.exp(-3.0 * d.entropy_n[1:4])
    assert r["L"] == 3 and r["khat"] == pytest.approx(float(np.cumprod(al).sum()), rel=1e-12)
    assert r["score"] == pytest.approx(r["khat"] - 0.25 * d.n_hi, rel=1e-12)
    assert r["verify"] == (r["score"] >= 0.1)


# ---------------------------------------------------------------- block completion and the outer loop (Alg. 1)
def test_block_complete_equals_one_forward_over_prefix_and_block(model):
    # K/V appended for a finished block = K/V of the same tokens in a single forward over [prefix, block] from an
    # empty cache whose mask is causal on the prefix and block-bidirectional on the block.
    W, prefix, ck, cv = model
    B = 4
    st = fresh(len(prefix), B)
    st.block = np.array([3, 17, 29, 5], dtype=np.int64)
    k, v = list(ck), list(cv)
    assert O.block_complete(CFG, W, st, k, v) == B and st.seq_len == len(prefix) + B
    toks = np.concatenate([prefix, [3, 17, 29, 5]])
    n, P = len(toks), len(prefix)
    vis = np.tril(np.ones((n, n), dtype=bool))
    vis[P:, P:] = True
    empty = [np.zeros((0, CFG.n_kv_heads, CFG.head_dim)) for _ in range(CFG.n_layers)]
    fo = O.forward(CFG, W, toks, np.arange(n), vis, empty, empty, logit_rows=np.zeros(0, dtype=np.int64))
    for l in range(CFG.n_layers):
        np.testing.assert_allclose(k[l][P:], fo.k[l][P:], rtol=0, atol=1e-12)
        np.testing.assert_allclose(v[l][P:], fo.v[l][P:], rtol=0, atol=1e-12)
        np.testing.assert_allclose(k[l][:P], ck[l], rtol=0, atol=0)        # the prefix rows are untouched
    # the first layer's K/V do not depend on the mask; deeper layers do (the block is not cached causally)
    causal_k, _ = O.prefill(CFG, W, toks)
    np.testing.assert_allclose(k[0][P:], causal_k[0][P:], rtol=0, atol=1e-12)
    assert np.abs(k[1][P:P + B - 1] - causal_k[1][P:P + B - 1]).max() > 1e-6


def test_block_complete_of_a_one_token_block_is_causal_append_and_unfinished_blocks_are_left(model):
    W, prefix, ck, cv = model
    st = fresh(len(prefix), 1)
    st.block = np.array([33], dtype=np.int64)
    k, v = list(ck), list(cv)
    O.block_complete(CFG, W, st, k, v)
    ref_k, ref_v = O.prefill(CFG, W, np.concatenate([prefix, [33]]))
    for l in range(CFG.n_layers):
        np.testing.assert_allclose(k[l], ref_k[l], rtol=0, atol=1e-12)
        np.testing.assert_allclose(v[l], ref_v[l], rtol=0, atol=1e-12)
    st2 = fresh(len(prefix), 4)
    st2.block[1] = 9
    k2 = list(ck)
    assert O.block_complete(CFG, W, st2, k2, list(cv)) == 0 and st2.seq_len == len(prefix) and k2[0] is ck[0]


def test_generate_commits_whole_blocks_and_both_cachings_end_with_a_full_cache(model):
    W, prefix, ck, cv = model
    B, nb = 4, 3
    rp = O.RouteParams(policy=O.ROUTE_MIN_SPAN, tau_span=2)
    for caching in ("causal", "block"):
        st = fresh(len(prefix), B)
        k, v = list(ck), list(cv)
        toks, log = O.generate(CFG, W, st, k, v, nb, 0.9, seed=5, rp=rp, max_steps_per_block=6, caching=caching)
        assert len(toks) == nb * B and all(0 <= t < CFG.vocab and t != MASK for t in toks)
        assert st.pos0 == len(prefix) + nb * B and (st.block == MASK).all()
        assert sum(c for _, _, c in log) == nb * B                       # every step's commits add up to the blocks
        assert all(kind == "threshold" or c >= 1 for kind, _, c in log)   # a verified step always commits something
        if caching == "block":
            assert st.seq_len == st.pos0 and k[0].shape[0] == st.pos0     # every finished block is cached whole
            # cached K/V of the generated blocks = block-diffusion forward over the final text
            full = np.concatenate([prefix, toks])
            n, P = len(full), len(prefix)
            vis = np.tril(np.ones((n, n), dtype=bool))
            for b in range(nb):
                vis[P + b * B:P + (b + 1) * B, P + b * B:P + (b + 1) * B] = True
            empty = [np.zeros((0, CFG.n_kv_heads, CFG.head_dim)) for _ in range(CFG.n_layers)]
            fo = O.forward(CFG, W, full, np.arange(n), vis, empty, empty, logit_rows=np.zeros(0, dtype=np.int64))
            np.testing.assert_allclose(k[1], fo.k[1], rtol=0, atol=1e-10)
        else:
            assert st.seq_len + len(st.carry) == st.pos0                  # causal caching may trail by carried tokens
            ref_k, _ = O.prefill(CFG, W, np.concatenate([prefix, toks])[:st.seq_len])
            np.testing.assert_allclose(k[1], ref_k[1], rtol=0, atol=1e-10)   # AR caching = causal prefill of the text


def test_generate_step_cap_forces_completion(model):
    W, prefix, ck, cv = model
    st = fresh(len(prefix), 4)
    rp = O.RouteParams(policy=O.ROUTE_MIN_SPAN, tau_span=99)              # never verify
    toks, log = O.generate(CFG, W, st, list(ck), list(cv), 1, 2.0, seed=1, rp=rp, max_steps_per_block=1, caching="block")
    # tau above 1: a threshold step commits only the arg-max position; the cap then commits the rest at once
    assert [c for _, _, c in log] == [1, 3] and len(toks) == 4


def test_causal_block_completion_appends_what_a_causal_prefill_of_the_text_gives(model):
    # Section 4.2: K/V cached under the causal mask depend only on the tokens to their left, so caching a finished
    # block (and tokens carried in front of it) in one causal forward = a plain causal prefill of prefix + text.
    W, prefix, ck, cv = model
    B = 4
    st = fresh(len(prefix), B)
    st.carry = np.array([11, 42], dtype=np.int64)                     # two uncached tokens of the block before
    st.pos0 = len(prefix) + 2
    st.block = np.array([3, 17, 29, 5], dtype=np.int64)
    k, v = list(ck), list(cv)
    assert O.block_complete(CFG, W, st, k, v, causal=True) == 6 and st.seq_len == st.pos0 + B and len(st.carry) == 0
    ref_k, ref_v = O.prefill(CFG, W, np.concatenate([prefix, [11, 42, 3, 17, 29, 5]]))
    for l in range(CFG.n_layers):
        np.testing.assert_allclose(k[l], ref_k[l], rtol=0, atol=1e-12)
        np.testing.assert_allclose(v[l], ref_v[l], rtol=0, atol=1e-12)
    # and it differs from the block-diffusion completion in the deeper layer (the mask matters there)
    st2 = fresh(len(prefix), B)
    st2.block = np.array([3, 17, 29, 5], dtype=np.int64)
    k2, k3 = list(ck), list(ck)
    O.block_complete(CFG, W, st2, k2, list(cv))
    st3 = fresh(len(prefix), B)
    st3.block = st2.block.copy()
    O.block_complete(CFG, W, st3, k3, list(cv), causal=True)
    assert np.abs(k2[1][-B:-1] - k3[1][-B:-1]).max() > 1e-6


def test_generate_without_any_verified_step_keeps_the_carry_bounded_and_the_tokens_unchanged(model):
    # A policy that never verifies: no verifier forward ever caches anything.  The carry may defer Alg. 1's per-block
    # cache update but not beyond its capacity; the committed tokens do not depend on the capacity (causal K/V are
    # the same whenever they are computed), and whatever is cached equals a causal prefill of the text.
    W, prefix, ck, cv = model
    B, nb = 4, 4
    rp = O.RouteParams(policy=O.ROUTE_MIN_SPAN, tau_span=99)
    runs = {}
    for cap in (None, 0, 10 ** 6):
        st = fresh(len(prefix), B)
        k, v = list(ck), list(cv)
        toks, log = O.generate(CFG, W, st, k, v, nb, 0.5, seed=3, rp=rp, max_steps_per_block=3, caching="causal", carry_cap=cap)
        assert all(kind == "threshold" for kind, _, _ in log) and len(toks) == nb * B
        assert st.seq_len + len(st.carry) == st.pos0 == len(prefix) + nb * B
        ref_k, _ = O.prefill(CFG, W, np.concatenate([prefix, toks])[:st.seq_len])
        np.testing.assert_allclose(k[1], ref_k[1], rtol=0, atol=1e-10)
        runs[cap] = (toks, len(st.carry))
    assert runs[None][0] == runs[0][0] == runs[10 ** 6][0]
    assert runs[None][1] <= B and runs[0][1] == 0 and runs[10 ** 6][1] == nb * B   # default capacity B; none; unbounded

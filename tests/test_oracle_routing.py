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

"""Pins for the oracle's right-shifted variant (Section 4.2: for models whose output at position i-1 scores token i
the plain causal mask already gives the verifier view): windows written out by hand, verifier probabilities against
teacher-forced scoring by one plain causal forward, block size 1 against textbook greedy decoding, cache contents
against a causal prefill of the committed text."""
import dataclasses

import numpy as np
import pytest

from oracle import s2d2_oracle as O
from s2d2_inputs import ModelCfg, gen_weights

CFG = ModelCfg("pin-shifted", n_layers=2, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=96, vocab=50,
               dtype="f32", rope_theta=10000.0, right_shifted=True)
PLAIN = dataclasses.replace(CFG, right_shifted=False)
MASK = CFG.mask_id
PREFIX = np.array([4, 8, 15, 16, 23, 42, 7])


@pytest.fixture(scope="module")
def model():
    W = gen_weights(CFG, seed=11, unembed_gain=10.0, norm_jitter=0.2)
    ck, cv = O.prefill(CFG, W, PREFIX[:-1])     # the cache lags: the last prompt token is carried
    return W, ck, cv


def start(B):
    return O.shifted_prefill_state(len(PREFIX), int(PREFIX[-1]), B, MASK)


def causal_logits(W, tokens):
    """Textbook language-model scoring: one causal forward over the whole text, no cache, no windows."""
    t = np.asarray(tokens, dtype=np.int64)
    nocache = [np.zeros((0, CFG.n_kv_heads, CFG.head_dim)) for _ in range(CFG.n_layers)]
    return O.forward(PLAIN, W, t, np.arange(len(t)), O.causal_mask(len(t)), nocache, list(nocache), np.arange(len(t))).logits


def test_windows_written_out():
    st = start(4)
    assert (st.seq_len, st.pos0, list(st.carry)) == (6, 7, [7])
    dw = O.shifted_draft_window(st, MASK)
    assert list(dw.tokens) == [7, MASK, MASK, MASK, MASK] and list(dw.pos) == [6, 7, 8, 9, 10]
    assert list(dw.logit_rows) == [0, 1, 2, 3] and list(dw.logit_index) == [0, 1, 2, 3]
    # the carried token is causal (sees only itself in the window); block rows see it and the whole block
    assert dw.vis.astype(int).tolist() == [[1, 0, 0, 0, 0]] + [[1, 1, 1, 1, 1]] * 4
    vw = O.shifted_verify_window(st, np.array([10, 11, 12, 13]), MASK)
    assert list(vw.tokens) == [7, 10, 11, 12] and list(vw.pos) == [6, 7, 8, 9]      # no row for the last draft
    assert (vw.vis == O.causal_mask(4)).all()
    assert list(vw.logit_rows) == [0, 1, 2, 3] and (vw.n_lead, vw.n_causal, vw.L, vw.j) == (1, 4, 4, 0)
    # mid-block: two committed tokens (first one cached), span of two, a committed token right of it
    st = O.SeqState(seq_len=8, pos0=7, block=np.array([21, 22, MASK, MASK, 25]))
    dw = O.shifted_draft_window(st, MASK)
    assert list(dw.tokens) == [22, MASK, MASK, 25] and list(dw.logit_rows) == [0, 1] and list(dw.logit_index) == [2, 3]
    vw = O.shifted_verify_window(st, np.array([-1, -1, 31, 32, -1]), MASK)
    assert list(vw.tokens) == [22, 31] and list(vw.pos) == [8, 9] and list(vw.logit_rows) == [0, 1]
    assert (vw.n_lead, vw.n_causal) == (1, 2)


def test_windows_refuse_a_cached_front_token():
    st = O.SeqState(seq_len=7, pos0=7, block=np.full(3, MASK, dtype=np.int64))    # front token already cached
    with pytest.raises(ValueError):
        O.shifted_draft_window(st, MASK)
    with pytest.raises(ValueError):
        O.shifted_verify_window(st, np.array([1, 2, 3]), MASK)


def test_verifier_probabilities_are_teacher_forced_scores(model):
    W, ck, cv = model
    st = start(4)
    xhat = np.array([10, 11, 12, 13])
    vo = O.verify(CFG, W, st, ck, cv, xhat)
    ref = causal_logits(W, list(PREFIX) + list(xhat))
    for r in range(4):   # token at position 7 + r is scored by the row of position 6 + r
        row = ref[len(PREFIX) - 1 + r]
        np.testing.assert_allclose(vo.logits[r], row, atol=1e-9)
        lp = row - np.log(np.exp(row - row.max()).sum()) - row.max()
        assert vo.q[r] == pytest.approx(float(np.exp(lp[xhat[r]])), rel=1e-9)


def test_draft_reads_the_row_in_front(model):
    """The draft logits of block index i are the plain model's output at the row of position i-1 of the same
    window (the non-shifted oracle, pinned elsewhere, read one row to the left)."""
    W, ck, cv = model
    st = O.SeqState(seq_len=6, pos0=7, block=np.array([30, MASK, MASK, 5]), carry=np.array([7]))
    d = O.draft(CFG, W, st, ck, cv, tau=0.9)
    win = O.draft_window(st, MASK)
    full = O.forward(PLAIN, W, win.tokens, win.pos, win.vis, ck, cv, np.arange(len(win.tokens))).logits
    assert list(d.win.logit_index) == [1, 2]
    np.testing.assert_allclose(d.logits[0], full[1], atol=1e-12)    # window rows: [carry, 30, M, M, 5]
    np.testing.assert_allclose(d.logits[1], full[2], atol=1e-12)


def test_block_size_one_is_greedy_autoregressive_decoding(model):
    """B = 1: the drafting row and the verifying row are the same causal row, so every draft is accepted and the
    text is what textbook greedy decoding produces."""
    W, ck0, cv0 = model
    st = start(1)
    ck, cv = list(ck0), list(cv0)
    text = list(PREFIX)
    for s in range(6):
        d, vo, a = O.step(CFG, W, st, ck, cv, tau=0.9, seed=3, step_idx=s)
        assert (a.n_accept, a.n_commit, a.resampled) == (1, 1, -1)
        assert vo.q[0] == pytest.approx(d.p[0], rel=1e-9)
        nxt = int(np.argmax(causal_logits(W, text)[-1]))
        assert int(d.xhat[0]) == nxt
        text.append(nxt)
        assert st.seq_len == len(text) - 1 and list(st.carry) == [nxt]


def test_cache_lags_one_token_and_equals_causal_prefill(model):
    W, ck0, cv0 = model
    for seed in range(4):
        st = start(3)
        ck, cv = list(ck0), list(cv0)
        seq = list(PREFIX[:-1])
        all_accepted = 0
        for s in range(10):
            d, vo, a = O.step(CFG, W, st, ck, cv, tau=0.9, seed=seed, step_idx=s)
            rows = vo.win.n_lead + min(a.n_accept, vo.win.L - 1)
            seq += list(vo.win.tokens[:rows])
            all_accepted += a.n_accept == vo.win.L
            assert a.n_commit >= 1 and ck[0].shape[0] == st.seq_len == len(seq)
            # the token in front of the next [MASK] is never cached
            j, L = O.first_span(st.block, MASK)
            assert st.seq_len <= st.pos0 + j - 1
        k2, v2 = O.prefill(CFG, W, np.array(seq), chunk=5)
        for l in range(CFG.n_layers):
            np.testing.assert_allclose(ck[l], k2[l], atol=1e-10)
            np.testing.assert_allclose(cv[l], v2[l], atol=1e-10)
        assert st.pos0 > len(PREFIX)


def test_whole_block_append_is_refused(model):
    W, ck, cv = model
    st = O.SeqState(seq_len=6, pos0=7, block=np.array([1, 2]), carry=np.array([7]))
    with pytest.raises(ValueError):
        O.block_complete(CFG, W, st, list(ck), list(cv))

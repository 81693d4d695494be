"""GPU parity of the right-shifted variant (Section 4.2: models whose output at position i-1 scores token i): the
draft reads its logits one row to the left, the verifier runs plain causal rows without [MASK] copies, the cache
lags one token behind the committed text.  Same harness and tolerances as the other parity tests."""
import dataclasses

import numpy as np
import pytest
import torch

import s2d2_inputs as I
from paper_2603_25702_amd import Params
from paper_2603_25702_amd.binding import S2D2Error

S2D2_EINVAL = -1
from tests import harness as H
from tests.test_gpu_parity import SMALL_BF16, SMALL_MOE, TINY, run_steps

pytestmark = pytest.mark.gpu


def shifted(cfg):
    return dataclasses.replace(cfg, right_shifted=True)


def test_tiny_fp32_many_steps_cross_block_boundaries():
    case = H.make_case(shifted(TINY), 2, 3, [37, 64], seed=5, synthetic_kv=False, norm_jitter=0.2, page_size=8, room=64)
    run, rep = run_steps(case, 8)
    print("shifted tiny multi-step:", rep)
    assert max(s.pos0 for s in case.states) > 64     # some block was completed and rolled
    assert rep.max_logit_err_draft < 1e-4 and rep.max_logit_err_verify < 1e-4
    for s in case.states:                             # the token in front of the first [MASK] is never cached
        j, L = H.O.first_span(s.block, case.cfg.mask_id)
        assert s.seq_len <= s.pos0 + j - 1


def test_block_size_one_accepts_every_draft():
    """B = 1: the drafting row and the verifying row are the same causal row (p = q up to rounding)."""
    case = H.make_case(shifted(TINY), 2, 1, [20, 33], seed=3, synthetic_kv=False, page_size=8, room=32)
    run, rep = run_steps(case, 5)
    assert rep.n_accept == [1] * 10 and rep.n_commit == [1] * 10


def test_small_bf16_ragged_batch_narrow_and_wide_windows():
    case = H.make_case(shifted(SMALL_BF16), 3, 8, [100, 257, 31], seed=2, synthetic_kv=True, page_size=16, room=64)
    run, rep = run_steps(case, 3)
    print("shifted small bf16:", rep)
    assert rep.max_logit_err_draft <= H.LOGIT_RTOL and rep.max_logit_err_verify <= H.LOGIT_RTOL
    case = H.make_case(shifted(SMALL_BF16), 3, 16, [100, 257, 31], seed=11, synthetic_kv=True, page_size=16, room=96, norm_jitter=0.1)
    run, rep = run_steps(case, 3)       # windows of up to 3 * (1 + 2 * 16) rows: the tiled GEMM and the wide attention
    print("shifted small bf16, wide windows:", rep)
    assert rep.max_logit_err_draft <= H.LOGIT_RTOL and rep.max_logit_err_verify <= H.LOGIT_RTOL


def test_sampling_mode_and_moe():
    case = H.make_case(shifted(SMALL_BF16), 2, 8, [64, 90], seed=4, synthetic_kv=True, page_size=16, room=64)
    run, rep = run_steps(case, 3, prm_kw=dict(mode=1, temperature=0.5))
    print("shifted sampling:", rep)
    case = H.make_case(shifted(SMALL_MOE), 2, 8, [64, 90], seed=7, synthetic_kv=True, page_size=16, room=64)
    run, rep = run_steps(case, 2)
    print("shifted moe:", rep)


def test_cached_front_token_is_reported_and_the_sequence_skipped():
    cfg = shifted(SMALL_BF16)
    case = H.make_case(cfg, 2, 4, [70, 33], seed=6, synthetic_kv=True, page_size=16, room=64)
    # sequence 1 breaks the precondition: its front token counts as cached, nothing is carried
    case.states[1] = H.O.SeqState(33, 33, np.full(4, cfg.mask_id, dtype=np.int64))
    case.seq_len[1] = 33
    run = H.DeviceRun(case)
    before = run.st.block_tokens.clone()
    prm = Params(step=0, seed=9)
    run.step(prm, advance=False)
    g = run.fetch()
    assert int(g["status"][1]) == S2D2_EINVAL and int(g["status"][0]) == 0
    assert int(g["span_len"][1]) == 0 and int(g["n_commit"][1]) == 0 and int(g["seq_len"][1]) == 33
    assert torch.equal(run.st.block_tokens[1], before[1])
    H.check_step(case, run, g, prm, seqs=[0])         # the other sequence is unaffected


def test_whole_block_append_is_refused():
    cfg = shifted(SMALL_BF16)
    case = H.make_case(cfg, 1, 4, [40], seed=1, synthetic_kv=True, page_size=16, room=64)
    run = H.DeviceRun(case)
    with pytest.raises(S2D2Error):
        run.eng.s2d2_block_complete(run.kv, run.st, 1, 4, run.v)


def test_session_prefill_carries_the_last_prompt_token_and_steps_match_the_oracle():
    """The runner's session: a prompt prefilled through the library leaves the cache one token behind, the steps that
    follow are checked against the oracle on the GPU's own cache contents."""
    from paper_2603_25702_amd.runner import Session
    cfg, N, B = shifted(SMALL_BF16), 2, 4
    W = I.gen_weights(cfg, 3)
    lens = np.array([90, 41], dtype=np.int32)
    ids = [I.gen_prefix_ids(cfg, int(lens[n]), 3, n) for n in range(N)]
    table = I.gen_page_table(N, 512 // 16, 3)
    ses = Session(cfg, W, N, B, 512, 16, "cuda:0", page_table=table)
    ses.prefill(ids)
    torch.cuda.synchronize()
    assert ses.kv.seq_len.tolist() == [89, 40] and ses.st.block_pos0.tolist() == [90, 41]
    assert ses.st.carry_tokens[:, 0].tolist() == [int(ids[0][-1]), int(ids[1][-1])]
    case = H.Case(cfg, W, N, B, 16, table, [], [], lens - 1)
    case.states = [H.O.shifted_prefill_state(int(lens[n]), int(ids[n][-1]), B, cfg.mask_id) for n in range(N)]
    run = H.DeviceRun(case, session=ses)
    H.sync_case_from_gpu(case, run)
    rep = H.Report()
    for s in range(4):
        prm = Params(step=s, seed=77)
        run.step(prm, advance=False)
        g = run.fetch()
        H.check_step(case, run, g, prm, rep=rep)
        run.eng.s2d2_block_advance(run.kv, run.st, N, B, None)
        H.sync_case_from_gpu(case, run)
    print("shifted session:", rep)
    assert int(ses.kv.status.abs().sum()) == 0 and sum(rep.n_commit) >= 8

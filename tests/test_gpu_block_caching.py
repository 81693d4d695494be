"""Alg. 1's cache update of a finished block on the MFMA path (bf16 dense and MoE models): the whole-block append of
decoding that caches nothing inside a block, and the causal completion of blocks that fallback steps finished when
the carry list cannot take them.  Staged protocol as everywhere (the oracle follows the device's committed tokens);
appended K/V rows are compared layer by layer."""
import numpy as np
import pytest
import torch

import s2d2_inputs as I
from paper_2603_25702_amd import Params
from tests import harness as H

pytestmark = pytest.mark.gpu

SMALL_BF16 = I.ModelCfg("small-bf16", 2, 512, 8, 4, 128, 1536, 32000)
SMALL_MOE = I.ModelCfg("small-moe", 2, 512, 8, 4, 128, 0, 32000, n_experts=8, top_k=2, d_expert=256)
MODELS = {"small_bf16": SMALL_BF16, "small_moe": SMALL_MOE}


def _finished(case):
    return [not (np.asarray(s.block) == case.cfg.mask_id).any() for s in case.states]


@pytest.mark.parametrize("model", ["small_bf16", "small_moe"])
def test_whole_block_append_under_block_diffusion_attention(model):
    """caching = "block": drafting fully bidirectional (ar_mask = 0), nothing appended inside a block, every finished
    block cached by s2d2_block_complete (its rows attend to the whole block), for several blocks of two ragged
    sequences; the next block's logits then read those rows through the cache."""
    cfg = MODELS[model]
    case = H.make_case(cfg, 2, 4, [37, 64], seed=21, synthetic_kv=True, page_size=16, room=64, norm_jitter=0.1)
    run, rep = H.DeviceRun(case), H.Report()
    completed = 0
    for s in range(14):
        prm = Params(step=s, seed=55, ar_mask=0)
        if s % 3 == 2:    # a fallback step now and then: non-contiguous commits inside the block
            run.step_fallback(prm)
            H.check_step(case, run, run.fetch(), prm, rep=rep, verified=False)
        else:
            run.step(prm, advance=False, append=False)
            H.check_step(case, run, run.fetch(), prm, rep=rep, append=False)
        if any(_finished(case)):
            completed += sum(_finished(case))
            H.check_block_complete(case, run, causal=False, rep=rep)
        run.eng.s2d2_block_advance(run.kv, run.st, case.N, case.B, None)
        H.sync_case_from_gpu(case, run)
        assert all(len(st.carry) == 0 and st.seq_len == st.pos0 for st in case.states if (np.asarray(st.block) == cfg.mask_id).all())
    print(model, "whole-block caching:", rep, "blocks completed:", completed)
    assert completed >= 4 and rep.max_kv_err > 0


@pytest.mark.parametrize("model", ["small_bf16", "small_moe"])
def test_blocks_finished_without_a_verified_step_are_cached_causally_once_the_carry_is_full(model):
    """A policy that never verifies (every step is draft + threshold commit): finished blocks ride in the carry list;
    the second finished block does not fit (capacity B) and is cached by s2d2_block_complete(causal = 1) together
    with the carried one.  Four blocks per sequence; the block always rolls over and no token is lost."""
    cfg = MODELS[model]
    B = 4
    case = H.make_case(cfg, 2, B, [30, 48], seed=23, synthetic_kv=True, page_size=16, room=64, norm_jitter=0.1)
    run, rep = H.DeviceRun(case), H.Report()
    flushed, blocks, text = 0, [0, 0], [[], []]
    for s in range(40):
        prm = Params(step=s, seed=56, tau=0.05)        # a low threshold: several tokens per step
        run.step_fallback(prm)
        H.check_step(case, run, run.fetch(), prm, rep=rep, verified=False)
        fin = _finished(case)
        for n in range(2):
            if fin[n]:
                blocks[n] += 1
                text[n] += [int(x) for x in case.states[n].block]
        over = [fin[n] and len(case.states[n].carry) + B - case.states[n].n_cached_in_block() > B for n in range(2)]
        if any(over):
            flushed += sum(over)
            H.check_block_complete(case, run, causal=True, rep=rep)
        run.eng.s2d2_block_advance(run.kv, run.st, case.N, case.B, None)
        torch.cuda.synchronize()
        assert int(run.kv.status.abs().sum()) == 0          # every finished block rolled over
        pos0_before = [st.pos0 for st in case.states]
        H.sync_case_from_gpu(case, run)
        for n in range(2):
            assert case.states[n].pos0 == pos0_before[n] + (B if fin[n] else 0)
            assert len(case.states[n].carry) <= B
        if min(blocks) >= 4:
            break
    print(model, "never verified:", rep, "blocks", blocks, "causal completions", flushed)
    assert min(blocks) >= 4 and flushed >= 2
    # the carried tokens are the tail of the committed text
    for n in range(2):
        nc = len(case.states[n].carry)
        assert nc == 0 or [int(x) for x in case.states[n].carry] == text[n][-nc:]


def test_block_advance_flags_a_finished_block_that_the_carry_cannot_take():
    """Without the causal completion the block is left in place and the status word says so (no silent stall)."""
    cfg, B = SMALL_BF16, 4
    case = H.make_case(cfg, 1, B, [20], seed=24, synthetic_kv=True, page_size=16, room=64)
    case.states[0].carry = np.array([5, 6, 7], dtype=np.int64)   # three uncached tokens of the block before
    case.states[0].pos0 += 3
    case.states[0].block = np.array([1, 2, 3, 4], dtype=np.int64)
    run = H.DeviceRun(case)
    run.eng.s2d2_block_advance(run.kv, run.st, 1, B, None)
    torch.cuda.synchronize()
    assert int(run.kv.status[0]) == -2 and int(run.st.block_pos0[0]) == 23
    assert run.st.block_tokens.cpu().tolist() == [[1, 2, 3, 4]]

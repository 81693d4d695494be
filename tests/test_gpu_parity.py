"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle (see harness.py)."""
import numpy as np
import pytest
import torch

import s2d2_inputs as I
from paper_2603_25702_amd import Params
from tests import harness as H

pytestmark = pytest.mark.gpu

TINY = I.CONFIGS[1].cfg
SMALL_BF16 = I.ModelCfg("small-bf16", 2, 512, 8, 4, 128, 1536, 32000)


def run_steps(case, steps, prm_kw=None, check_logits=True, seqs=None, advance=True, packed=True, act_planes=0):
    run = H.DeviceRun(case, packed=packed, act_planes=act_planes)
    rep = H.Report()
    for s in range(steps):
        prm = Params(step=s, seed=1234, **(prm_kw or {}))
        run.step(prm, advance=False)
        g = run.fetch()
        H.check_step(case, run, g, prm, seqs=seqs, rep=rep, check_logits=check_logits)
        if advance:
            run.eng.s2d2_block_advance(run.kv, run.st, case.N, case.B, None)
        H.sync_case_from_gpu(case, run)
    return run, rep


def test_config1_tiny_fp32_one_step_free_running():
    wl = I.CONFIGS[1]
    case = H.make_case(wl.cfg, wl.batch, wl.block, [wl.prefix_min], seed=0, synthetic_kv=False)
    run, rep = run_steps(case, 1)
    print("config1:", rep)
    assert rep.max_logit_err_draft < 1e-4 and rep.max_logit_err_verify < 1e-4
    assert rep.exempt_xhat == rep.exempt_ratio == rep.exempt_resample == rep.exempt_tau == 0
    assert rep.n_commit[0] >= 1


def test_tiny_fp32_many_steps_cross_block_boundaries_with_jittered_norms():
    cfg = TINY
    case = H.make_case(cfg, 2, 3, [37, 64], seed=5, synthetic_kv=False, norm_jitter=0.2, page_size=8, room=64)
    run, rep = run_steps(case, 8)
    print("tiny multi-step:", rep)
    assert max(s.pos0 for s in case.states) > 64  # some block was completed and rolled
    assert rep.max_logit_err_draft < 1e-4


def test_small_bf16_ragged_batch_paged():
    case = H.make_case(SMALL_BF16, 3, 8, [100, 257, 31], seed=2, synthetic_kv=True, page_size=16, room=64)
    run, rep = run_steps(case, 3)
    print("small bf16:", rep)
    assert rep.max_logit_err_draft <= H.LOGIT_RTOL


def test_small_bf16_canonical_weight_layout_path():
    """Same model without the packed weight copy: the plain (unfused) kernels."""
    case = H.make_case(SMALL_BF16, 2, 4, [70, 33], seed=6, synthetic_kv=True, page_size=16, room=64, norm_jitter=0.1)
    run, rep = run_steps(case, 2, packed=False)
    print("small bf16 unpacked:", rep)


def test_small_bf16_jittered_norm_gains_fused_path():
    case = H.make_case(SMALL_BF16, 2, 8, [40, 90], seed=9, synthetic_kv=True, page_size=16, room=64, norm_jitter=0.2)
    run, rep = run_steps(case, 3)
    print("small bf16 jitter:", rep)


def test_small_bf16_real_prefill_b4():
    case = H.make_case(SMALL_BF16, 1, 4, [96], seed=3, synthetic_kv=False, page_size=16, room=64)
    run, rep = run_steps(case, 4)
    print("small bf16 prefill:", rep)


def test_degenerate_batch_empty_prefix_page_boundary_and_a_finished_block():
    """Edge cases in one ragged batch: a sequence with an empty cache, one whose prefix ends exactly on a page
    boundary, and one whose block holds no [MASK] when the step starts (no span, no logit rows, nothing drafted or
    accepted; its committed, uncached tokens ride through the verifier as causal rows and are appended)."""
    case = H.make_case(TINY, 3, 4, [0, 16, 37], seed=4, synthetic_kv=True, page_size=8, room=64)
    case.states[2].block[:] = [5, 6, 7, 8]
    run = H.DeviceRun(case)
    rep = H.Report()
    for s in range(3):
        prm = Params(step=s, seed=77)
        run.push_state()
        run.step(prm, advance=False)
        g = run.fetch()
        H.check_step(case, run, g, prm, rep=rep)
        if s == 0:
            assert g["span_len"][2] == 0 and g["n_accept"][2] == 0 and g["n_commit"][2] == 0
            assert int(run.kv.seq_len[2]) == 41      # the four pending tokens were appended
        run.eng.s2d2_block_advance(run.kv, run.st, case.N, case.B, None)
        H.sync_case_from_gpu(case, run)
    print("degenerate batch:", rep)
    assert rep.max_logit_err_draft < 1e-4 and rep.max_logit_err_verify < 1e-4
    assert case.states[0].seq_len >= 1 and case.states[2].pos0 == 41


@pytest.mark.parametrize("model", ["tiny_fp32", "small_bf16"])
def test_maximum_block_size_of_64(model):
    """B = 64, the largest block the boundary admits (per-sequence sets are 64-bit masks): 128 draft rows and 192
    verifier rows per sequence, spans of up to 64 positions in the accept scan, several steps inside one block."""
    if model == "tiny_fp32":
        case = H.make_case(TINY, 2, 64, [40, 9], seed=12, synthetic_kv=True, page_size=8, room=256)
    else:
        case = H.make_case(SMALL_BF16, 1, 64, [150], seed=13, synthetic_kv=True, page_size=16, room=256)
    run, rep = run_steps(case, 3)
    print("B=64", model, rep)
    assert rep.max_logit_err_draft <= (1e-4 if model == "tiny_fp32" else H.LOGIT_RTOL)
    assert all(0 <= n <= 64 for n in rep.n_commit)


def test_maximum_batch_of_1024_ragged_sequences():
    """N = 1024, the largest batch the boundary admits (one planning thread per sequence), ragged prefixes from
    1 to 60 tokens; the oracle follows the first, the last and 22 sampled sequences over two steps."""
    rng = np.random.default_rng(3)
    lens = rng.integers(1, 61, size=1024)
    case = H.make_case(TINY, 1024, 2, lens, seed=14, synthetic_kv=True, page_size=8, room=32)
    seqs = sorted({0, 1023, *rng.choice(1024, size=22, replace=False).tolist()})
    run, rep = run_steps(case, 2, seqs=seqs)
    print("N=1024:", rep)
    assert rep.max_logit_err_draft < 1e-4 and rep.max_logit_err_verify < 1e-4


def test_narrow_windows_with_k_shares_that_end_in_a_partial_batch_of_loads():
    """d_model 1280 and d_ffn 2560 (40 and 80 K tiles): the K share of a streaming-GEMM wavefront is 5 or 10 tiles,
    i.e. full batches of four loads followed by a partial one, which none of the five configurations' shapes has."""
    cfg = I.ModelCfg("mid-bf16", 2, 1280, 8, 4, 128, 2560, 32000)
    case = H.make_case(cfg, 1, 4, [70], seed=21, synthetic_kv=True, page_size=16, room=64, norm_jitter=0.1)
    run, rep = run_steps(case, 2)
    print("partial batches:", rep)
    assert rep.max_logit_err_draft <= H.LOGIT_RTOL and rep.max_logit_err_verify <= H.LOGIT_RTOL
    case = H.make_case(cfg, 2, 8, [33, 90], seed=22, synthetic_kv=True, page_size=16, room=64, norm_jitter=0.1)
    run, rep = run_steps(case, 2)       # 32 draft rows: two row tiles of the streaming kernel
    assert rep.max_logit_err_draft <= H.LOGIT_RTOL and rep.max_logit_err_verify <= H.LOGIT_RTOL


def test_draft_mask_flag_and_block_size_one():
    # B = 1: drafter and verifier see the same thing, every token is accepted (q == p up to rounding)
    case = H.make_case(TINY, 2, 1, [20, 33], seed=7, synthetic_kv=False, page_size=8, room=32)
    run = H.DeviceRun(case)
    prm = Params(step=0, seed=9)
    run.step(prm, advance=False)
    g = run.fetch()
    np.testing.assert_allclose(g["logits_ver"][:2], g["logits"][:2], rtol=0, atol=1e-4)
    np.testing.assert_allclose(g["q"], g["p"], atol=1e-5)
    H.check_step(case, run, g, prm)
    # ar_mask = 0: committed in-block prefix sees the whole block
    case = H.make_case(TINY, 1, 4, [16], seed=8, synthetic_kv=False, page_size=8, room=32)
    case.states[0].block[:2] = [5, 6]
    run = H.DeviceRun(case)
    for ar in (1, 0):
        prm = Params(step=0, seed=9, ar_mask=ar)
        run.push_state()
        run.eng.s2d2_draft(run.kv, run.st, 1, 4, prm, run.d)
        g = run.fetch()
        st = case.states[0]
        ck, cv = case.oracle_cache(0)
        from oracle import s2d2_oracle as O
        od = O.draft(TINY, case.W, st, ck, cv, 0.9, bool(ar))
        rows = [g["logit_row_of"][0][i] for i in od.win.logit_index]
        np.testing.assert_allclose(g["logits"][rows], od.logits, atol=2e-4 * np.abs(od.logits).max())


@pytest.mark.parametrize("d_ffn", [1536, 4096])   # 4096: down projection with K shared between pairs of workgroups
def test_same_inputs_give_bit_identical_outputs(d_ffn):
    cfg = I.ModelCfg("small-bf16-det", 2, 512, 8, 4, 128, d_ffn, 32000)
    case = H.make_case(cfg, 2, 4, [50, 70], seed=4, synthetic_kv=True, page_size=16, room=32)
    outs = []
    for _ in range(2):
        run = H.DeviceRun(case)
        run.step(Params(step=3, seed=77), advance=True)
        g = run.fetch()
        outs.append(g)
    for k in outs[0]:
        if k in ("logits", "logits_ver"):  # rows beyond the planned count are unspecified
            n = int((outs[0]["logit_row_of"] >= 0).sum()) if k == "logits" else int((outs[0]["logit_row_of_ver"] >= 0).sum())
            assert np.array_equal(outs[0][k][:n], outs[1][k][:n]), k
        else:
            assert np.array_equal(outs[0][k], outs[1][k]), k


def test_token_ids_outside_the_vocabulary_are_read_as_mask_and_nothing_else_changes():
    """Device-side ids cannot be checked by the host.  A committed block token with an id outside [0, vocab)
    must embed as [MASK]: the step equals, bit for bit, the step of a model whose token T has the [MASK]
    embedding row, run with T at that position."""
    cfg = I.ModelCfg("small-bf16-ids", 2, 512, 8, 4, 128, 1536, 32000)
    W = I.gen_weights(cfg, 6)
    T = 1234
    W["embed"][T] = W["embed"][cfg.mask_id]
    outs = []
    for bad in (T, 2 ** 30, -7):
        case = H.make_case(cfg, 2, 4, [50, 70], seed=6, synthetic_kv=True, page_size=16, room=32, W=W)
        case.states[0].block[0] = bad          # a committed position in front of the masked span
        case.states[1].block[:2] = [17, bad]
        run = H.DeviceRun(case)
        run.step(Params(step=1, seed=5), advance=False)
        g = run.fetch()
        assert (g["status"] == 0).all()
        outs.append(g)
    for other in outs[1:]:
        for k in outs[0]:
            if k in ("block_tokens",):
                continue   # holds the id itself
            if k in ("logits", "logits_ver"):
                n = int((outs[0]["logit_row_of" if k == "logits" else "logit_row_of_ver"] >= 0).sum())
                assert np.isfinite(other[k][:n]).all() and np.array_equal(outs[0][k][:n], other[k][:n]), k
            else:
                assert np.array_equal(outs[0][k], other[k]), k


def test_kv_append_reports_enospc_without_writing():
    case = H.make_case(TINY, 1, 4, [30], seed=1, synthetic_kv=True, page_size=8, room=1)  # capacity 32
    run = H.DeviceRun(case)
    before = run.kv.k.clone()
    run.step(Params(step=0, seed=2), advance=False)
    g = run.fetch()
    lead_plus_acc = int(g["n_accept"][0])
    if 30 + lead_plus_acc > 32:
        assert g["status"][0] == -2 and g["seq_len"][0] == 30 and torch.equal(before, run.kv.k)
    else:
        assert g["status"][0] == 0 and g["seq_len"][0] == 30 + lead_plus_acc


def test_config2_full_size_consecutive_steps_in_the_benchmark_launch_configuration():
    """Full-size dense 1.7B-shaped model, the session bench.py times: prefix prefilled through the library, then
    ten consecutive draft+verify+accept+append steps, each one a replay of the captured HIP graph of a step as in
    the benchmark, each checked against the oracle (all logit rows, K/V appended in three layers): carried tokens,
    mid-block leading rows, block roll-over and a growing cache at full size.  Plus the first prefix positions of
    the prefilled cache."""
    from oracle import s2d2_oracle as O
    from paper_2603_25702_amd.runner import Session
    wl = I.CONFIGS[2]
    cfg, N, B = wl.cfg, wl.batch, wl.block
    W = I.gen_weights(cfg, 0)
    lens = I.gen_prefix_lengths(wl, 0)
    ids = [I.gen_prefix_ids(cfg, int(lens[n]), 0, n) for n in range(N)]
    max_seq = int(lens.max()) + 66 * B + 64
    table = I.gen_page_table(N, (max_seq + wl.page_size - 1) // wl.page_size, 0)
    ses = Session(cfg, W, N, B, max_seq, wl.page_size, "cuda:0", page_table=table)
    ses.prefill(ids)
    case = H.Case(cfg, W, N, B, wl.page_size, table, [], [], lens.copy())
    case.states = [O.SeqState(int(lens[n]), int(lens[n]), np.full(B, cfg.mask_id, dtype=np.int64)) for n in range(N)]
    run = H.DeviceRun(case, session=ses)
    H.sync_case_from_gpu(case, run)
    # sampled prefix check: the first positions of the prefilled cache against an oracle prefill
    ck, cv = O.prefill(cfg, W, ids[0][:12])
    for l in (0, cfg.n_layers // 2, cfg.n_layers - 1):
        gk, gv = run.cache_rows(0, 0, 12, l)
        assert np.abs(gk - ck[l]).max() <= H.LOGIT_RTOL * np.abs(ck[l]).max()
        assert np.abs(gv - cv[l]).max() <= H.LOGIT_RTOL * np.abs(cv[l]).max()
    graph = ses.capture_step(Params(tau=0.9, seed=0, step=0, step_dev=ses.step_dev), advance=False)
    rep = H.Report()
    pos0 = case.states[0].pos0
    for s in range(10):
        graph.replay()
        prm = Params(tau=0.9, seed=0, step=s)          # the device's step word is 0 + *step_dev = s
        rep = H.check_step(case, run, run.fetch(), prm, rep=rep, check_kv_layers=(0, 13, 27))
        ses.eng.s2d2_block_advance(ses.kv, ses.st, N, B, ses.step_dev)
        H.sync_case_from_gpu(case, run)
        print(f"config2 step {s}: committed {rep.n_commit[-1]}, seq_len {case.states[0].seq_len}, pos0 {case.states[0].pos0}", flush=True)
    print("config2 full, 10 steps:", rep)
    assert case.states[0].pos0 >= pos0 + 2 * B      # at least two blocks were completed and rolled over
    assert int(ses.tot_commit[0]) == sum(rep.n_commit) and rep.max_kv_err > 0


SMALL_MOE = I.ModelCfg("small-moe", 2, 512, 8, 4, 128, 0, 32000, n_experts=8, top_k=2, d_expert=256)


@pytest.mark.parametrize("tile_wc", ["4", "2"])
def test_small_bf16_wide_windows_run_the_tiled_gemm(monkeypatch, tile_wc):
    """Windows of up to 3*3*16 = 144 rows: the LDS-tiled GEMM with every fused epilogue, ragged row tiles; with
    the default workgroup of eight wavefronts and with the four-wavefront shape kept as a tuning aid."""
    monkeypatch.setenv("S2D2_TILE_WC", tile_wc)
    case = H.make_case(SMALL_BF16, 3, 16, [100, 257, 31], seed=11, synthetic_kv=True, page_size=16, room=96, norm_jitter=0.1)
    run, rep = run_steps(case, 3)
    print("small bf16 wide:", rep)
    assert rep.max_logit_err_draft <= H.LOGIT_RTOL


def test_tiled_gemm_with_k_that_ends_in_half_a_step():
    """d_model 480 and d_ffn 1504 are multiples of 32 but not of the tiled GEMM's K step of 64: every projection ends
    in a half-filled step (columns past K zeroed when the activation tile is staged, the weight tile index clamped),
    on full 128-row tiles (8 x 32 verifier rows) as on the ragged draft tile."""
    cfg = I.ModelCfg("small-bf16-k-tail", 2, 480, 8, 4, 128, 1504, 32000)
    case = H.make_case(cfg, 8, 16, [60, 33, 97, 16, 70, 41, 52, 85], seed=17, synthetic_kv=True, page_size=16, room=96, norm_jitter=0.1)
    run, rep = run_steps(case, 2)
    print("k tail:", rep)
    assert rep.max_logit_err_draft <= H.LOGIT_RTOL and rep.max_logit_err_verify <= H.LOGIT_RTOL


def test_k_split_hand_over_when_no_split_waits(monkeypatch):
    """The K splits of a tile of the tiled GEMM share its merge after a bounded wait; a split whose wait runs out
    hands its share to the split that arrives last.  With the wait set to zero polls every split but the last gives
    up at once, so the hand-over path (and the late give-up of a split that finds everybody there) does all the
    merging; results are sums in split order either way.  Several steps with carried tokens: row counts above and
    below the expected ones (workgroups that walk on to further row tiles, workgroups without rows)."""
    monkeypatch.setenv("S2D2_TILE_SPINS", "0")
    case = H.make_case(SMALL_BF16, 3, 16, [100, 257, 31], seed=13, synthetic_kv=True, page_size=16, room=96, norm_jitter=0.1)
    run, rep = run_steps(case, 3)
    print("hand-over:", rep)
    assert rep.max_logit_err_draft <= H.LOGIT_RTOL and rep.max_logit_err_verify <= H.LOGIT_RTOL
    run.eng.s2d2_status()


def test_long_k_down_projection_shared_by_pairs_of_workgroups():
    """d_ffn = 4096: the residual-add GEMM of the down projection splits K over pairs of workgroups that hand
    their partial over through tagged words (narrow windows only); one and two 16-row tiles, several steps so
    that the hand-over words are re-armed and reused, and the device status stays clean."""
    cfg = I.ModelCfg("small-long-k", 2, 512, 8, 4, 128, 4096, 32000)
    case = H.make_case(cfg, 1, 8, [70], seed=8, synthetic_kv=True, page_size=16, room=64, norm_jitter=0.1)
    run, rep = run_steps(case, 4)
    print("long K, paired:", rep)
    assert rep.max_logit_err_draft <= H.LOGIT_RTOL and rep.max_logit_err_verify <= H.LOGIT_RTOL
    run.eng.s2d2_status()
    case = H.make_case(cfg, 2, 4, [33, 90], seed=9, synthetic_kv=True, page_size=16, room=64)
    run, rep = run_steps(case, 3)
    run.eng.s2d2_status()


def test_one_and_a_half_rounds_of_tiles_and_several_row_tiles_per_column():
    """Launch forms of the tiled GEMM that only larger windows reach: 32 x 16 verifier rows against d_ffn = 6144 give
    the gate / up projection 48 x 8 = 384 tiles, 1.5 per compute unit: pairs of workgroups take one tile each and
    share a third one as two K splits; the same launch with the draft's 512 rows (192 tiles, four row tiles per
    column) and the unembedding (several row tiles) deal their tiles XCD by XCD.  Two steps: the partial buffers and
    tile counters are reused; the device status stays clean."""
    cfg = I.ModelCfg("small-wide-ffn", 2, 512, 8, 4, 128, 6144, 32000)
    lens = [20 + 7 * (n % 9) for n in range(32)]
    case = H.make_case(cfg, 32, 16, lens, seed=31, synthetic_kv=True, page_size=16, room=64, norm_jitter=0.1)
    run, rep = run_steps(case, 2, seqs=[0, 13, 31])
    print("wide FFN, 384 tiles:", rep)
    assert rep.max_logit_err_draft <= H.LOGIT_RTOL and rep.max_logit_err_verify <= H.LOGIT_RTOL
    run.eng.s2d2_status()


@pytest.mark.parametrize("act_planes", [1, 2, 3])
def test_operand_modes_narrow_wide_long_k_and_moe(act_planes):
    """`act_planes` of the model description: GEMM inputs as one bf16 plane (1), as a high + low bf16 plane (2), or as
    IEEE half values against a half copy of the weights (3, which the default 0 also selects and every other test
    runs).  Each mode through the streaming GEMM (narrow windows, also the paired K split of a long down projection),
    the tiled GEMM (wide windows), both attention kernels and the MoE FFN.  Two layers keep even the single bf16
    plane inside the tolerance; the 28- and 36-layer configurations need 11 bits or more."""
    case = H.make_case(SMALL_BF16, 3, 4, [100, 257, 31], seed=21, synthetic_kv=True, page_size=16, room=64)
    run, rep = run_steps(case, 2, act_planes=act_planes)
    print("planes", act_planes, "narrow:", rep)
    case = H.make_case(SMALL_BF16, 3, 16, [100, 257, 31], seed=22, synthetic_kv=True, page_size=16, room=96, norm_jitter=0.1)
    run, rep2 = run_steps(case, 2, act_planes=act_planes)
    print("planes", act_planes, "wide:", rep2)
    cfg = I.ModelCfg("small-long-k", 2, 512, 8, 4, 128, 4096, 32000)
    case = H.make_case(cfg, 1, 8, [70], seed=8, synthetic_kv=True, page_size=16, room=64, norm_jitter=0.1)
    run, rep3 = run_steps(case, 2, act_planes=act_planes)
    run.eng.s2d2_status()
    case = H.make_case(SMALL_MOE, 2, 8, [40, 90], seed=12, synthetic_kv=True, page_size=16, room=64, norm_jitter=0.1)
    run, rep4 = run_steps(case, 2, act_planes=act_planes)
    print("planes", act_planes, "long K:", rep3.max_logit_err_draft, "moe:", rep4.max_logit_err_draft)
    errs = [r.max_logit_err_draft for r in (rep, rep2, rep3, rep4)] + [r.max_logit_err_verify for r in (rep, rep2, rep3, rep4)]
    assert max(errs) <= H.LOGIT_RTOL
    if act_planes != 1:
        assert max(errs) <= 0.5 * H.LOGIT_RTOL


def test_small_moe_routing_grouped_gemm_and_combine():
    """MoE FFN: the oracle is held to the GPU's expert choices; the free-running router agreement is reported."""
    case = H.make_case(SMALL_MOE, 3, 8, [40, 90, 65], seed=12, synthetic_kv=True, page_size=16, room=64, norm_jitter=0.1)
    run = H.DeviceRun(case)
    rep = H.Report()
    for s in range(2):
        prm = Params(step=s, seed=99)
        run.step(prm, advance=False)
        g = run.fetch()
        H.check_step(case, run, g, prm, rep=rep, free_router=(s == 0))
        run.eng.s2d2_block_advance(run.kv, run.st, case.N, case.B, None)
        H.sync_case_from_gpu(case, run)
    print("small moe:", rep)
    assert rep.router_rows > 0 and rep.router_agree >= 0.9 * rep.router_rows


def test_vocab_and_accept_kernels_on_synthetic_logit_pairs_at_full_vocabulary():
    """The vocabulary stage alone on draft / verifier logit pairs shaped like the paper's confidence-by-ratio
    table (about three quarters agreeing rows, the rest independent), at V = 151936: statistics, scores, the
    accept scan with accepted runs of every length, and the residual draw, against the oracle on the same rows."""
    from oracle import s2d2_oracle as O
    from paper_2603_25702_amd import BlockState
    cfg = I.shrink(I.CONFIGS[2].cfg, n_layers=1, d_model=64, n_q_heads=1, n_kv_heads=1, head_dim=64, d_ffn=64)  # only V matters here
    N, B, V = 6, 8, cfg.vocab
    W = I.gen_weights(cfg, 0, unembed_gain=1.0)
    from paper_2603_25702_amd import Engine
    eng = Engine(cfg, W, N, B)
    dev = eng.device
    ld, lv, agree = I.gen_logit_pairs(N * B, V, seed=5)
    d, v, a = eng.alloc_draft_out(N, B), eng.alloc_verify_out(N, B), eng.alloc_accept_out(N, B)
    d.logits.copy_(torch.from_numpy(ld))
    v.logits_ver.copy_(torch.from_numpy(lv))
    ident = torch.arange(N * B, dtype=torch.int32, device=dev).view(N, B)
    d.logit_row_of.copy_(ident)
    v.logit_row_of.copy_(ident)
    st_d = eng.s2d2_vocab_draft_stats(d.logits)
    for k in ("xhat", "p", "lse", "margin", "entropy_n"):
        d.t[k].copy_(st_d[k].view(N, B))
    q, lse_v = eng.s2d2_vocab_score(v.logits_ver, d.xhat.view(-1))
    v.q.copy_(q.view(N, B))
    v.lse_ver.copy_(lse_v.view(N, B))
    starts = np.array([0, 1, 0, 2, 0, 3], dtype=np.int32)
    lens = np.array([8, 7, 8, 5, 8, 1], dtype=np.int32)
    d.span_start.copy_(torch.from_numpy(starts))
    d.span_len.copy_(torch.from_numpy(lens))
    blk = torch.full((N, B), cfg.mask_id, dtype=torch.int32, device=dev)
    st = BlockState(blk, torch.zeros(N, dtype=torch.int32, device=dev), torch.zeros((N, B), dtype=torch.int32, device=dev))
    hist = []
    for step in range(6):
        blk.fill_(cfg.mask_id)
        prm = Params(seed=31, step=step)
        eng.s2d2_accept(st, N, B, prm, d, v, a)
        torch.cuda.synchronize()
        g = {k: t.cpu().numpy() for k, t in list(d.t.items()) + list(a.t.items()) if k != "logits"}
        gq = v.q.cpu().numpy()
        for n in range(N):
            j, L = int(starts[n]), int(lens[n])
            rows = range(n * B + j, n * B + j + L)
            # oracle statistics on the same fp32 rows
            for r, i in zip(rows, range(j, j + L)):
                s = O.sample_from_logits(ld[r].astype(np.float64))
                assert s["xhat"] == g["xhat"][n, i] and abs(s["p"] - g["p"][n, i]) < 1e-3
                assert abs(s["margin"] - g["margin"][n, i]) < 2e-3 and abs(s["entropy_n"] - g["entropy_n"][n, i]) < 1e-3
                qq, _ = O.score_from_logits(lv[r].astype(np.float64), s["xhat"])
                assert abs(qq - gq[n, i]) < 1e-3
            u = np.array([O.uniform(31, step, n, j + r, O.STREAM_ACCEPT) for r in range(L)])
            p64, q64 = g["p"][n, j:j + L].astype(np.float64), gq[n, j:j + L].astype(np.float64)
            n_acc = O.accept_scan(p64, q64, u)
            if n_acc != g["n_accept"][n]:
                upto = min(L, max(n_acc, int(g["n_accept"][n])) + 1)
                assert (np.abs(q64[:upto] / p64[:upto] - u[:upto]) < H.TIE).any()
                n_acc = int(g["n_accept"][n])
            hist.append(n_acc)
            if n_acc < L:
                r = n * B + j + n_acc
                u2 = O.uniform(31, step, n, j + n_acc, O.STREAM_RESAMPLE)
                tok = O.residual_resample(ld[r].astype(np.float64), lv[r].astype(np.float64), u2)
                got = int(g["resampled"][n])
                if tok != got:
                    res = O.residual_distribution(ld[r].astype(np.float64), lv[r].astype(np.float64))
                    cdf = np.cumsum(res) / res.sum()
                    assert abs(cdf[min(tok, got)] - u2) < H.TIE, (n, step, tok, got)
                assert g["n_commit"][n] == n_acc + 1
            else:
                assert g["resampled"][n] == -1 and g["n_commit"][n] == L
    print("accepted-run histogram:", np.bincount(hist, minlength=9).tolist(), "agreeing rows:", int(agree.sum()), "of", N * B)
    assert max(hist) >= 2 and min(hist) == 0   # both long accepted runs and immediate rejections occurred


@pytest.mark.parametrize("d_ffn", [1536, 4096])
def test_captured_step_graph_replays_match_eager_steps(d_ffn):
    """A HIP graph of one step, replayed with eager work and synchronisations between the replays: every replay
    must leave exactly the state the same steps leave when enqueued call by call.  d_ffn = 4096 puts the down
    projection on the streaming GEMM that shares K between pairs of workgroups (hand-over words re-armed inside
    the kernel, no memset nodes)."""
    from paper_2603_25702_amd.runner import Session
    cfg = I.ModelCfg("small-bf16-graph", 2, 512, 8, 4, 128, d_ffn, 32000)
    W = I.gen_weights(cfg, 3)
    ids = [I.gen_prefix_ids(cfg, 90, 3, 0), I.gen_prefix_ids(cfg, 41, 3, 1)]

    def session():
        ses = Session(cfg, W, 2, 4, 512, 16, "cuda:0", max_block=16)
        ses.prefill(ids)
        return ses

    eager, states = session(), []
    prm_e = Params(seed=5, step=0, step_dev=eager.step_dev)
    for _ in range(4):
        eager.step(prm_e)
        torch.cuda.synchronize()
        states.append((eager.st.block_tokens.clone(), eager.kv.seq_len.clone(), eager.a.n_commit.clone(), eager.d.p.clone()))
    cap = session()
    prm_c = Params(seed=5, step=0, step_dev=cap.step_dev)
    graph = cap.capture_step(prm_c)
    cap.reset_blocks([90, 41])
    scratch = torch.zeros(1 << 20, device="cuda:0")
    for k in range(4):
        graph.replay()
        torch.cuda.synchronize()
        cap.eng.s2d2_status()
        scratch.add_(1.0).sum().item()       # eager work between replays
        blk, sl, nc, p = states[k]
        assert torch.equal(cap.st.block_tokens, blk) and torch.equal(cap.kv.seq_len, sl), f"replay {k}"
        assert torch.equal(cap.a.n_commit, nc) and torch.equal(cap.d.p, p), f"replay {k}"
    assert int(cap.tot_commit.sum()) == sum(int(s[2].sum()) for s in states)


def test_routing_scores_decisions_and_the_routed_step():
    """Section 4.3 on the device: K, score and decision of every policy against the oracle's routing applied to the
    same fp32 draft statistics; then one routed step (some sequences verified, the others committed by the
    threshold rule) against the oracle's routed step."""
    from oracle import s2d2_oracle as O
    from paper_2603_25702_amd.binding import DraftOut, RouteOut, RouteParams
    N, B = 5, 8
    case = H.make_case(SMALL_BF16, N, B, [100, 57, 31, 80, 64], seed=4, synthetic_kv=True, page_size=16, room=64)
    run, rep = run_steps(case, 1, advance=True)             # one verified step leaves blocks with different spans
    prm = Params(step=1, seed=1234)
    e = run.eng
    e.s2d2_draft(run.kv, run.st, N, B, prm, run.d)
    g = run.fetch()
    ro = RouteOut.alloc(N, run.dev)
    spans = [(int(g["span_start"][n]), int(g["span_len"][n])) for n in range(N)]
    assert len({L for _, L in spans}) > 1, spans

    def oracle_route(rp_or, h0):
        out = []
        for n in range(N):
            j, L = spans[n]
            al = O.acceptance_proxy(g["margin"][n, j:j + L].astype(np.float64), g["entropy_n"][n, j:j + L].astype(np.float64),
                                    rp_or.estimator, rp_or.tau_margin, rp_or.beta)
            k = O.expected_prefix_length(al)
            s = O.verify_score(k, int(g["n_hi"][n]), rp_or.c, rp_or.dynamic)
            dec, h = O.do_verify(rp_or, L, s, int(h0[n]))
            out.append((k, s, dec, h))
        return out

    policies = [
        dict(policy=0, tau_span=1), dict(policy=0, tau_span=4), dict(policy=0, tau_span=B + 1),
        dict(policy=1, estimator=1, dynamic=0, c=1.0, beta=2.0, tau_score=0.5),
        dict(policy=1, estimator=1, dynamic=1, c=0.5, beta=4.0, tau_score=0.0),
        dict(policy=1, estimator=0, dynamic=0, c=1.0, tau_margin=0.25, tau_score=1.0),
        dict(policy=2, estimator=1, dynamic=1, c=1.0, beta=1.0, tau_on=1.0, tau_off=-5.0),
        dict(policy=2, estimator=0, dynamic=0, c=2.0, tau_margin=0.5, tau_on=2.0, tau_off=0.0),
    ]
    near = 0
    for kw in policies:
        rp = RouteParams(**kw)
        rp_or = O.RouteParams(**{**kw, "dynamic": bool(kw.get("dynamic", 1))})
        h0 = np.array([1, 0, 1, 0, 1], dtype=np.int32)
        hyst = torch.as_tensor(h0, device=run.dev)
        e.s2d2_route(N, B, rp, run.d, hyst, ro)
        torch.cuda.synchronize()
        want = oracle_route(rp_or, h0)
        for n in range(N):
            k, s, dec, h = want[n]
            assert abs(float(ro.khat[n]) - k) <= 1e-5 * max(1.0, k), (kw, n)
            assert abs(float(ro.score[n]) - s) <= 1e-5 * max(1.0, abs(s)), (kw, n)
            thresholds = {1: [rp.tau_score], 2: [rp.tau_on, rp.tau_off]}.get(rp.policy, [])
            if any(abs(s - t) < 1e-4 for t in thresholds):
                near += 1
                continue
            assert int(ro.do_verify[n]) == int(dec), (kw, n, s)
            if rp.policy == 2:
                assert int(hyst[n]) == h, (kw, n)
            else:
                assert int(hyst[n]) == h0[n]
            assert int(ro.unmask_fallback[n]) == (0 if dec else int(g["unmask"][n]))
    assert near <= 2
    # error paths are host-side
    with pytest.raises(Exception):
        e.s2d2_route(N, B, RouteParams(policy=7), run.d, None, ro)
    with pytest.raises(Exception):
        e.s2d2_route(N, B, RouteParams(policy=2), run.d, None, ro)

    # ---- a routed step: a score threshold at the median sends about half of the sequences to the verifier ----
    rp0 = RouteParams(policy=1, estimator=1, dynamic=0, c=0.0, beta=2.0, tau_score=0.0)
    e.s2d2_route(N, B, rp0, run.d, None, ro)
    med = float(np.sort(ro.score.cpu().numpy())[N // 2])
    rp = RouteParams(policy=1, estimator=1, dynamic=0, c=0.0, beta=2.0, tau_score=med)
    e.s2d2_route(N, B, rp, run.d, None, ro)
    dv = ro.do_verify.cpu().numpy().astype(bool)
    assert dv.any() and (~dv).any(), dv
    prm_r = Params(step=1, seed=1234, active=ro.do_verify)
    before = [np.array(s.block, copy=True) for s in case.states]
    seq_before = [s.seq_len for s in case.states]
    e.s2d2_verify(run.kv, run.st, N, B, prm_r, run.d, run.v)
    e.s2d2_accept(run.st, N, B, prm_r, run.d, run.v, run.a)
    e.s2d2_kv_append(run.kv, N, B, run.d, run.v, run.a.n_accept)
    e.s2d2_commit_threshold(run.st, N, B, DraftOut({**run.d.t, "unmask": ro.unmask_fallback}))
    g2 = run.fetch()
    verified = [n for n in range(N) if dv[n]]
    H.check_step(case, run, g2, prm, seqs=verified, rep=rep)       # these went through Alg. 3's verify branch
    for n in range(N):
        if dv[n]:
            continue
        S = np.array([(int(g2["unmask"][n]) >> i) & 1 for i in range(B)], dtype=bool)
        want = np.where(S, g2["xhat"][n], before[n])
        np.testing.assert_array_equal(g2["block_tokens"][n], want)   # Alg. 2 commit, nothing else
        assert S.sum() >= 1 and (before[n][S] == SMALL_BF16.mask_id).all()
        assert int(g2["seq_len"][n]) == seq_before[n] and int(g2["n_accept"][n]) == 0 and int(g2["n_commit"][n]) == 0
        assert int(g2["resampled"][n]) == -1 and int(g2["stage_lead"][n]) == 0
        gp = g2["p"][n].astype(np.float64)
        S_or, _ = O.threshold_set(gp, before[n] == SMALL_BF16.mask_id, float(np.float32(prm.tau)))
        assert (S == S_or).all() or (np.abs(gp[before[n] == SMALL_BF16.mask_id] - prm.tau) < H.TIE).any()
    print("routing: decisions", dv.astype(int).tolist(), "scores", np.round(ro.score.cpu().numpy(), 3).tolist(), "near-threshold skips", near)


def test_accept_variants_ratio_tempering_and_reject_only():
    """Ablation flags of the accept step (appendix on acceptance variants): u < min(1, (q/p)^gamma) with gamma != 1,
    and rejection without the residual draw."""
    for kw in (dict(gamma=0.5), dict(gamma=2.0), dict(resample=0), dict(gamma=0.25, resample=0)):
        case = H.make_case(SMALL_BF16, 3, 8, [60, 45, 90], seed=8, synthetic_kv=True, page_size=16, room=64)
        run, rep = run_steps(case, 2, prm_kw=kw, check_logits=False)
        print("accept variant", kw, "n_accept", rep.n_accept, "n_commit", rep.n_commit)
        if kw.get("resample", 1) == 0:
            assert rep.n_commit == rep.n_accept          # nothing is committed at the rejected position
        else:
            assert all(c >= 1 for c in rep.n_commit)


def test_sampling_mode_drafting_at_temperature_half():
    """SAMPLE-mode drafting (the paper's T = 0.5 ablation): proposals drawn from softmax(logits / T) with the stream-2
    uniforms, p, q and the residual all at that temperature."""
    from paper_2603_25702_amd.binding import S2D2_SAMPLE
    for T in (0.5, 1.0):
        case = H.make_case(SMALL_BF16, 3, 8, [60, 45, 90], seed=12, synthetic_kv=True, page_size=16, room=64)
        run, rep = run_steps(case, 3, prm_kw=dict(mode=S2D2_SAMPLE, temperature=T), check_logits=(T == 0.5))
        print(f"sampling T={T}:", rep)
        assert all(c >= 1 for c in rep.n_commit)
    # the proposals really are samples: at T = 1 on near-uniform rows they differ from the arg-max somewhere
    case = H.make_case(SMALL_BF16, 2, 8, [40, 41], seed=13, synthetic_kv=True, page_size=16, room=64)
    run = H.DeviceRun(case)
    run.eng.s2d2_draft(run.kv, run.st, 2, 8, Params(step=0, seed=5), run.d)
    greedy = run.fetch()["xhat"].copy()
    run.eng.s2d2_draft(run.kv, run.st, 2, 8, Params(step=0, seed=5, mode=S2D2_SAMPLE, temperature=4.0), run.d)
    sampled = run.fetch()
    assert (sampled["xhat"] != greedy).any()
    assert (sampled["p"] > 0).all() and (sampled["p"] <= 1).all()


@pytest.mark.parametrize("tau_span", [2, 99])
def test_generate_loop_routed_with_step_cap_under_both_cachings(tau_span):
    """Alg. 1's outer loop on the device (draft, DoVerify, verify+accept or threshold commit, cache append per step or
    per finished block, block roll-over) against the oracle's generate, free-running on the tiny fp32 model; with a
    minimum-span policy that verifies most fresh blocks, and with one that never verifies (four blocks finished by
    fallback steps only: the carry fills up and is cached by the causal block completion)."""
    from oracle import s2d2_oracle as O
    from paper_2603_25702_amd.binding import RouteParams
    from paper_2603_25702_amd.runner import Session
    cfg, N, B, nb, cap = TINY, 2, 3, 4, 4
    for caching in ("causal", "block"):
        W = I.gen_weights(cfg, 15, norm_jitter=0.1)
        prefixes = [I.gen_prefix_ids(cfg, L, 15, n) for n, L in enumerate([21, 34])]
        sess = Session(cfg, W, N, B, max_seq=34 + nb * B + 16, page_size=8)
        sess.prefill(prefixes)
        rp = RouteParams(policy=0, tau_span=tau_span)
        toks, log = sess.generate(Params(seed=77), rp, nb, cap, caching)
        sl, p0 = sess.kv.seq_len.cpu().numpy(), sess.st.block_pos0.cpu().numpy()
        for n in range(N):
            ck, cv = O.prefill(cfg, W, np.asarray(prefixes[n]))
            st = O.SeqState(seq_len=len(prefixes[n]), pos0=len(prefixes[n]), block=np.full(B, cfg.mask_id, dtype=np.int64))
            ot, ol = O.generate(cfg, W, st, ck, cv, nb, float(np.float32(0.9)), seed=77,
                                rp=O.RouteParams(policy=O.ROUTE_MIN_SPAN, tau_span=tau_span), max_steps_per_block=cap,
                                caching=caching, seq=n)
            assert toks[n] == ot, (caching, n, toks[n], ot)
            assert log[n] == ol, (caching, n, log[n], ol)
            assert len(ot) == nb * B and (int(sl[n]), int(p0[n])) == (st.seq_len, st.pos0), (caching, n, sl[n], p0[n], st.seq_len, st.pos0)
            if tau_span == 99:
                assert all(kind == "threshold" for kind, _, _ in ol)
        if caching == "block":
            assert [int(x) for x in sl] == [len(p) + nb * B for p in prefixes]
        print("generate", caching, "tau_span", tau_span, "tokens", toks, "steps", [len(l) for l in log])

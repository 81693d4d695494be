"""s2d2_accept_static (the accept step for callers that cannot allocate: scratch in a device array of the library)
against s2d2_accept (scratch in the caller's workspace) on the same inputs, through the C ABI: every output bit
for bit, on two calls in a row, the second with a smaller input, so that what the first call left in the shared
array is in the way of the second."""
import numpy as np
import pytest
import torch

import s2d2_inputs as I
from paper_2603_25702_amd import BlockState, Engine, Params
from paper_2603_25702_amd.binding import S2D2_ENOSPC, S2D2Error, s2d2_accept_static

pytestmark = pytest.mark.gpu


def _inputs(eng, cfg, N, B, seed, starts, lens):
    dev, V = eng.device, cfg.vocab
    ld, lv, _ = I.gen_logit_pairs(N * B, V, seed=seed)
    d, v = eng.alloc_draft_out(N, B), eng.alloc_verify_out(N, B)
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
    d.span_start.copy_(torch.tensor(starts, dtype=torch.int32))
    d.span_len.copy_(torch.tensor(lens, dtype=torch.int32))
    return d, v


def _state(cfg, N, B, dev):
    blk = torch.full((N, B), cfg.mask_id, dtype=torch.int32, device=dev)
    return BlockState(blk, torch.zeros(N, dtype=torch.int32, device=dev), torch.zeros((N, B), dtype=torch.int32, device=dev))


def test_accept_without_allocation_matches_the_workspace_entry_point_on_two_calls_in_a_row():
    cfg = I.shrink(I.CONFIGS[2].cfg, n_layers=1, d_model=64, n_q_heads=1, n_kv_heads=1, head_dim=64, d_ffn=64)  # only V matters
    W = I.gen_weights(cfg, 0, unembed_gain=1.0)
    eng = Engine(cfg, W, 6, 8)
    dev = eng.device
    cases = [(6, 8, 5, [0, 1, 0, 2, 0, 3], [8, 7, 8, 5, 8, 1]),      # 8 workgroups share each sequence's vocabulary
             (3, 4, 6, [0, 1, 2], [4, 3, 1])]                          # smaller: fewer sequences, shorter blocks
    rejected = 0
    for N, B, seed, starts, lens in cases:
        d, v = _inputs(eng, cfg, N, B, seed, starts, lens)
        for step in range(3):
            prm = Params(seed=31, step=step)
            got = {}
            for name in ("workspace", "static"):
                st, a = _state(cfg, N, B, dev), eng.alloc_accept_out(N, B)
                for t in a.t.values():
                    t.fill_(-7)
                if name == "workspace":
                    eng.s2d2_accept(st, N, B, prm, d, v, a)
                else:
                    s2d2_accept_static(None, cfg.vocab, st, N, B, prm, d, v, a)
                torch.cuda.synchronize()
                got[name] = {k: t.cpu().numpy() for k, t in a.t.items()}
                got[name]["block_tokens"] = st.block_tokens.cpu().numpy()
            for k in got["workspace"]:
                np.testing.assert_array_equal(got["static"][k].view(np.int32), got["workspace"][k].view(np.int32), err_msg=f"N={N} step={step} {k}")
            rejected += int((got["static"]["resampled"] >= 0).sum())
    assert rejected >= 4      # the residual draw, which is what uses the scratch, ran in both shapes
    eng.close()


def test_sizes_beyond_the_static_scratch_are_refused_before_anything_is_launched():
    cfg = I.shrink(I.CONFIGS[1].cfg, n_layers=1)
    dev = torch.device("cuda:0")
    from paper_2603_25702_amd.binding import AcceptOut, DraftOut, VerifyOut
    N, B, V = 2, 4, 64
    d = DraftOut.alloc(N, B, V, dev)
    v = VerifyOut.alloc(N, B, V, 1, 8, 1, 8, torch.float32, dev)
    a = AcceptOut.alloc(N, B, dev)
    st = _state(cfg, N, B, dev)
    for kw in (dict(N=129, vocab=V), dict(N=N, vocab=(1 << 18) + 1)):
        with pytest.raises(S2D2Error) as e:
            s2d2_accept_static(None, kw["vocab"], st, kw["N"], B, Params(), d, v, a)
        assert e.value.code == S2D2_ENOSPC

"""Parity harness: runs the HIP path through the C ABI and the fp64 oracle on the same seeded
inputs and compares them stage by stage.

Protocol (bf16 vs fp64 cannot be compared free-running, an arg-max may flip inside the logit
tolerance), every stage on the same inputs:
  1. draft logits:    max |gpu - oracle| <= 2e-2 * max |oracle logit|
  2. draft vocab:     the oracle's SampleFromLogits / threshold rule is fed the GPU's fp32 logits;
                      x_hat exact unless the top-1/top-2 probability gap < 1e-3, p/margin/entropy
                      within 1e-3, threshold set exact unless |p - tau| < 1e-3
  3. verifier logits: the oracle verifies the GPU's x_hat (teacher forcing); same logit bound
  4. accept:          the oracle's accept loop is fed the GPU's logits and the same uniforms;
                      n_accept exact unless some |q/p - u| < 1e-3 at or before the decision; the
                      resampled token exact unless the residual CDF is within 1e-3 of u' at it
  5. cache append:    appended K/V rows equal the oracle's causal verify rows within the storage
                      rounding; seq_len and page placement exact
Every exemption that fires is counted and returned.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np
import torch

import s2d2_inputs as I
from oracle import s2d2_oracle as O
from paper_2603_25702_amd import BlockState, Engine, KvCache, Params

LOGIT_RTOL = 2e-2
PROB_ATOL = 1e-3
TIE = 1e-3


def round_to_storage(x: np.ndarray, cfg) -> torch.Tensor:
    return torch.from_numpy(np.asarray(x)).to(cfg.torch_dtype)


@dataclass
class Case:
    cfg: I.ModelCfg
    W: Dict[str, torch.Tensor]
    N: int
    B: int
    page_size: int
    page_table: np.ndarray            # [N, max_pages]
    k_pages: List[torch.Tensor]       # per layer CPU [n_pages, Hkv, ps, D] storage dtype
    v_pages: List[torch.Tensor]       # per layer CPU [n_pages, Hkv, D, ps] (the cache keeps V key-minor)
    seq_len: np.ndarray               # [N]
    states: List[O.SeqState] = field(default_factory=list)

    def oracle_cache(self, n: int):
        """Logical cache of sequence n gathered from the physical pages (stored values)."""
        S, ps = int(self.seq_len[n]), self.page_size
        npg = (S + ps - 1) // ps
        pages = torch.as_tensor(self.page_table[n, :npg].astype(np.int64))
        ck, cv = [], []
        for l in range(self.cfg.n_layers):
            k = self.k_pages[l][pages].permute(0, 2, 1, 3).reshape(npg * ps, self.cfg.n_kv_heads, self.cfg.head_dim)[:S]
            v = self.v_pages[l][pages].permute(0, 3, 1, 2).reshape(npg * ps, self.cfg.n_kv_heads, self.cfg.head_dim)[:S]
            ck.append(k)
            cv.append(v)
        return ck, cv


def make_case(cfg: I.ModelCfg, N: int, B: int, prefix_lens, seed: int = 0, page_size: int = 16,
              synthetic_kv: bool = True, norm_jitter: float = 0.0, gain: Optional[float] = None,
              room: int = 0, W: Optional[Dict[str, torch.Tensor]] = None) -> Case:
    """Weights, prefix cache (real causal prefill by the oracle, or synthetic pages) and fresh blocks."""
    if W is None:
        W = I.gen_weights(cfg, seed, unembed_gain=gain, norm_jitter=norm_jitter)
    prefix_lens = np.asarray(prefix_lens, dtype=np.int32)
    room = room or 3 * B + page_size
    max_pages = int((prefix_lens.max() + room + page_size - 1) // page_size)
    table = I.gen_page_table(N, max_pages, seed)
    n_pages = N * max_pages
    if synthetic_kv:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=8) as ex:  # independent keyed generators per (layer, k/v)
            k_pages = list(ex.map(lambda l: I.gen_synth_kv_pages(cfg, n_pages, page_size, seed, l, "k"), range(cfg.n_layers)))
            v_pages = list(ex.map(lambda l: I.gen_synth_kv_pages(cfg, n_pages, page_size, seed, l, "v").permute(0, 1, 3, 2).contiguous(),
                                  range(cfg.n_layers)))
    else:
        shape = (n_pages, cfg.n_kv_heads, page_size, cfg.head_dim)
        k_pages = [torch.zeros(shape, dtype=cfg.torch_dtype) for _ in range(cfg.n_layers)]
        v_pages = [torch.zeros(shape, dtype=cfg.torch_dtype).permute(0, 1, 3, 2).contiguous() for _ in range(cfg.n_layers)]
        for n in range(N):
            ids = I.gen_prefix_ids(cfg, int(prefix_lens[n]), seed, n)
            ck, cv = O.prefill(cfg, W, ids)
            for l in range(cfg.n_layers):
                for s in range(len(ids)):
                    pg, sl = int(table[n, s // page_size]), s % page_size
                    k_pages[l][pg, :, sl, :] = round_to_storage(ck[l][s], cfg)
                    v_pages[l][pg, :, :, sl] = round_to_storage(cv[l][s], cfg)
    case = Case(cfg, W, N, B, page_size, table, k_pages, v_pages, prefix_lens.copy())
    case.states = [O.SeqState(int(prefix_lens[n]), int(prefix_lens[n]), np.full(B, cfg.mask_id, dtype=np.int64)) for n in range(N)]
    if getattr(cfg, "right_shifted", False):   # the cache lags: the last prompt token is carried, its cache row unused
        case.seq_len = prefix_lens - 1
        case.states = [O.shifted_prefill_state(int(prefix_lens[n]), int(I.gen_prefix_ids(cfg, int(prefix_lens[n]), seed, n)[-1]),
                                               B, cfg.mask_id) for n in range(N)]
    return case


LazyF64Weights = O.LazyF64Weights


class DeviceRun:
    """Device-side mirror of a Case plus output buffers; methods call the C ABI."""

    def __init__(self, case: Case, device: str = "cuda:0", session=None, packed: bool = True, act_planes: int = 0):
        cfg, N, B = case.cfg, case.N, case.B
        self.case, self.dev = case, torch.device(device)
        if session is not None:  # wrap the buffers of a runner.Session (cache already on the device)
            self.eng, self.kv, self.st = session.eng, session.kv, session.st
            self.d, self.v, self.a = session.d, session.v, session.a
            return
        self.eng = Engine(cfg, case.W, N, B, device, packed=packed, act_planes=act_planes)
        i32 = torch.int32
        kdev = torch.empty((cfg.n_layers,) + tuple(case.k_pages[0].shape), dtype=cfg.torch_dtype, device=self.dev)
        vdev = torch.empty((cfg.n_layers,) + tuple(case.v_pages[0].shape), dtype=cfg.torch_dtype, device=self.dev)
        for l in range(cfg.n_layers):  # layer by layer: no second host copy of a multi-GB cache
            kdev[l].copy_(case.k_pages[l])
            vdev[l].copy_(case.v_pages[l])
        self.kv = KvCache(kdev, vdev,
                          torch.as_tensor(case.page_table, dtype=i32, device=self.dev),
                          torch.as_tensor(case.seq_len, dtype=i32, device=self.dev),
                          torch.zeros(N, dtype=i32, device=self.dev))
        self.st = BlockState(torch.empty((N, B), dtype=i32, device=self.dev), torch.empty(N, dtype=i32, device=self.dev),
                             torch.zeros((N, B), dtype=i32, device=self.dev))
        self.push_state()
        self.d = self.eng.alloc_draft_out(N, B)
        self.v = self.eng.alloc_verify_out(N, B)
        self.a = self.eng.alloc_accept_out(N, B)

    def push_state(self):
        c = self.case
        blk = np.stack([s.block for s in c.states]).astype(np.int32)
        car = np.zeros((c.N, c.B), dtype=np.int32)
        for n, s in enumerate(c.states):
            car[n, :len(s.carry)] = s.carry
        self.st.block_tokens.copy_(torch.from_numpy(blk))
        self.st.carry_tokens.copy_(torch.from_numpy(car))
        self.st.block_pos0.copy_(torch.as_tensor([s.pos0 for s in c.states], dtype=torch.int32))
        self.kv.seq_len.copy_(torch.as_tensor([s.seq_len for s in c.states], dtype=torch.int32))

    def step_fallback(self, prm: Params):
        """The else-branch of Alg. 3 for every sequence: draft, then the threshold commit of Alg. 2."""
        N, B, e = self.case.N, self.case.B, self.eng
        e.s2d2_draft(self.kv, self.st, N, B, prm, self.d)
        if self.case.cfg.is_moe:
            self.choices_draft = e.s2d2_moe_choices(2 * N * B)
        e.s2d2_commit_threshold(self.st, N, B, self.d)

    def step(self, prm: Params, advance: bool = True, append: bool = True):
        N, B, e = self.case.N, self.case.B, self.eng
        moe = self.case.cfg.is_moe
        e.s2d2_draft(self.kv, self.st, N, B, prm, self.d)
        if moe:
            self.choices_draft = e.s2d2_moe_choices(2 * N * B)
        e.s2d2_verify(self.kv, self.st, N, B, prm, self.d, self.v)
        if moe:
            self.choices_verify = e.s2d2_moe_choices(3 * N * B)
        e.s2d2_accept(self.st, N, B, prm, self.d, self.v, self.a)
        if append:
            e.s2d2_kv_append(self.kv, N, B, self.d, self.v, self.a.n_accept)
        if advance:
            e.s2d2_block_advance(self.kv, self.st, N, B, prm.step_dev)

    def fetch(self) -> Dict[str, np.ndarray]:
        torch.cuda.synchronize(self.dev)
        self.eng.s2d2_status()   # raises if a device-side barrier of the fused forward timed out
        out = {}
        for src in (self.d.t, self.v.t, self.a.t):
            for k, t in src.items():
                if k in ("k_stage", "v_stage"):
                    continue
                key = k if k not in out else k + "_ver"
                out[key] = t.detach().cpu().numpy()
        out["block_tokens"] = self.st.block_tokens.cpu().numpy()
        out["block_pos0"] = self.st.block_pos0.cpu().numpy()
        out["carry_tokens"] = self.st.carry_tokens.cpu().numpy()
        out["seq_len"] = self.kv.seq_len.cpu().numpy()
        out["status"] = self.kv.status.cpu().numpy()
        return out

    def cache_rows(self, n: int, s0: int, s1: int, layer: int):
        """K, V of logical positions [s0, s1) of sequence n, layer `layer`, from device pages (fp64)."""
        ps = self.case.page_size
        ks, vs = [], []
        for s in range(s0, s1):
            pg = int(self.case.page_table[n, s // ps])
            ks.append(self.kv.k[layer, pg, :, s % ps, :].to(torch.float64).cpu().numpy())
            vs.append(self.kv.v[layer, pg, :, :, s % ps].to(torch.float64).cpu().numpy())
        return np.stack(ks), np.stack(vs)


@dataclass
class Report:
    max_logit_err_draft: float = 0.0      # relative to max |logit|
    max_logit_err_verify: float = 0.0
    max_prob_err: float = 0.0
    max_kv_err: float = 0.0
    exempt_xhat: int = 0
    exempt_tau: int = 0
    exempt_ratio: int = 0
    exempt_resample: int = 0
    n_commit: List[int] = field(default_factory=list)
    n_accept: List[int] = field(default_factory=list)
    rows_checked: int = 0
    router_rows: int = 0                  # MoE: (layer, row) pairs compared with the oracle's own routing
    router_agree: int = 0


def draft_window_of(cfg):
    return O.shifted_draft_window if getattr(cfg, "right_shifted", False) else O.draft_window


def verify_window_of(cfg):
    return O.shifted_verify_window if getattr(cfg, "right_shifted", False) else O.verify_window


def check_step(case: Case, run: DeviceRun, g: Dict[str, np.ndarray], prm: Params, seqs=None,
               rep: Optional[Report] = None, check_logits: bool = True, check_kv_layers=None,
               pre_seq_len: Optional[np.ndarray] = None, free_router: bool = False, append: bool = True,
               verified: bool = True) -> Report:
    """Compares one GPU step (outputs `g`, taken after the step with advance=False) with the oracle.
    case.states must still hold the state from BEFORE the step; on return they hold the oracle's
    state after accept + append (not advanced).  append=False: a step of decoding that appends nothing inside a
    block (no s2d2_kv_append was called).  verified=False: a fallback step (draft, then s2d2_commit_threshold)."""
    cfg, B = case.cfg, case.B
    rep = rep or Report()
    seqs = range(case.N) if seqs is None else seqs
    tau = float(np.float32(prm.tau))
    mode, T = int(prm.mode), (float(np.float32(prm.temperature)) if int(prm.mode) == O.SAMPLE else 1.0)
    # MoE: window rows are packed sequence after sequence; the oracle is held to the GPU's expert choices
    moe = cfg.is_moe
    if moe:
        ch_d = run.choices_draft.cpu().numpy()
        ch_v = run.choices_verify.cpu().numpy() if verified else None
        row0_d, row0_v, rd, rv = [], [], 0, 0
        for n in range(case.N):
            wd = draft_window_of(cfg)(case.states[n], cfg.mask_id, bool(prm.ar_mask))
            row0_d.append(rd)
            row0_v.append(rv)
            rd += len(wd.tokens)
            rv += len(verify_window_of(cfg)(case.states[n], np.zeros(B, dtype=np.int64), cfg.mask_id).tokens)
    for n in seqs:
        st = case.states[n]
        ck, cv = case.oracle_cache(n)
        # ---- stage 1 + 2: draft -------------------------------------------------------------
        win = draft_window_of(cfg)(st, cfg.mask_id, bool(prm.ar_mask))
        assert g["span_start"][n] == win.j and g["span_len"][n] == win.L
        rows_d = g["logit_row_of"][n]
        assert [(rows_d[i] >= 0) for i in range(B)] == [i in set(win.logit_index) for i in range(B)]
        V = g["logits"].shape[1]
        # (a block without [MASK] has no logit rows: the comparisons below then run over empty arrays)
        gl = np.stack([g["logits"][rows_d[i]] for i in win.logit_index] or [np.zeros((0, V))]).astype(np.float64).reshape(-1, V)
        if check_logits:
            forced = None
            if moe:
                forced = [ch_d[l, row0_d[n]:row0_d[n] + len(win.tokens)] for l in range(cfg.n_layers)]
                if free_router:
                    free = O.draft(cfg, case.W, st, ck, cv, tau, bool(prm.ar_mask))
                    for l in range(cfg.n_layers):
                        rep.router_rows += len(win.tokens)
                        rep.router_agree += int((np.sort(free.fwd.experts[l], axis=1) == np.sort(forced[l], axis=1)).all(axis=1).sum())
            od = O.draft(cfg, case.W, st, ck, cv, tau, bool(prm.ar_mask), forced_experts=forced)
            scale = np.abs(od.logits).max() if od.logits.size else 1.0
            err = np.abs(gl - od.logits).max() / scale if od.logits.size else 0.0
            rep.max_logit_err_draft = max(rep.max_logit_err_draft, err)
            assert err <= LOGIT_RTOL, f"seq {n}: draft logits off by {err:.3e} of max|logit|"
        d = O.draft_from_logits(st, win, gl, cfg.mask_id, tau, mode, T, prm.seed, prm.step, n)
        xhat = g["xhat"][n].astype(np.int64).copy()
        for r, i in enumerate(win.logit_index):
            P, _ = O.log_softmax_stats(gl[r], T)
            top2 = np.sort(P)[-2:]
            if xhat[i] != d.xhat[i]:
                if mode == O.SAMPLE:   # the inverse CDF lands within rounding of a boundary between the two tokens
                    cdf = np.cumsum(P)
                    ud = O.uniform(prm.seed, prm.step, n, int(i), O.STREAM_DRAFT)
                    assert abs(cdf[min(xhat[i], d.xhat[i])] - ud) < TIE, f"seq {n} pos {i}: sampled x_hat {xhat[i]} vs {d.xhat[i]}"
                else:
                    assert top2[1] - top2[0] < TIE and abs(P[xhat[i]] - top2[1]) < TIE, f"seq {n} pos {i}: x_hat {xhat[i]} vs {d.xhat[i]}"
                rep.exempt_xhat += 1
                d.xhat[i] = xhat[i]
                d.p[i] = P[xhat[i]]
            for name, tol in (("p", PROB_ATOL), ("margin", 2 * PROB_ATOL), ("entropy_n", PROB_ATOL)):
                e = abs(float(g[name][n, i]) - float(getattr(d, name)[i]))
                rep.max_prob_err = max(rep.max_prob_err, e)
                assert e <= tol, f"seq {n} pos {i}: {name} {g[name][n, i]} vs {getattr(d, name)[i]}"
            assert abs(float(g["lse"][n, i]) - d.lse[i]) <= 1e-3 * max(1.0, abs(d.lse[i]))
        committed = np.asarray(st.block) != cfg.mask_id
        assert (g["xhat"][n][committed] == -1).all() and (g["p"][n][committed] == 0).all()
        # threshold set, decided on the GPU's own fp32 p (same precision on both sides)
        gp = g["p"][n].astype(np.float64)
        S_or, n_hi = O.threshold_set(gp, ~committed, tau)
        S_gpu = np.array([(int(g["unmask"][n]) >> i) & 1 for i in range(B)], dtype=bool)
        if not (S_gpu == S_or).all() or g["n_hi"][n] != n_hi:
            assert (np.abs(gp[~committed] - tau) < TIE).any(), f"seq {n}: threshold set differs"
            rep.exempt_tau += 1
        if not verified:   # Alg. 2 commit of the (GPU's) threshold set; nothing is appended
            want = np.array(st.block, copy=True)
            want[S_gpu] = xhat[S_gpu]
            np.testing.assert_array_equal(g["block_tokens"][n], want)
            assert int(g["seq_len"][n]) == st.seq_len
            st.block = want
            rep.n_commit.append(int(S_gpu.sum()))
            rep.rows_checked += len(win.logit_index)
            continue
        # ---- stage 3: verifier logits with the GPU's proposals ----------------------------------
        vwin = verify_window_of(cfg)(st, xhat, cfg.mask_id)
        rows_v = g["logit_row_of_ver"][n]
        gv = np.stack([g["logits_ver"][rows_v[i]] for i in vwin.logit_index] or [np.zeros((0, V))]).astype(np.float64).reshape(-1, V)
        assert g["stage_lead"][n] == vwin.n_lead
        ov = None
        if check_logits:
            forced = None
            if moe:
                forced = [ch_v[l, row0_v[n]:row0_v[n] + len(vwin.tokens)] for l in range(cfg.n_layers)]
            ov = O.verify(cfg, case.W, st, ck, cv, xhat, forced_experts=forced)
            err = np.abs(gv - ov.logits).max() / np.abs(ov.logits).max() if ov.logits.size else 0.0
            rep.max_logit_err_verify = max(rep.max_logit_err_verify, err)
            assert err <= LOGIT_RTOL, f"seq {n}: verifier logits off by {err:.3e} of max|logit|"
        vo = O.verify_from_logits(vwin, gv, xhat, ov.k if ov else None, ov.v if ov else None, mode, T)
        for r, i in enumerate(vwin.logit_index):
            e = abs(float(g["q"][n, i]) - vo.q[r])
            rep.max_prob_err = max(rep.max_prob_err, e)
            assert e <= PROB_ATOL, f"seq {n} pos {i}: q {g['q'][n, i]} vs {vo.q[r]}"
        # ---- stage 4: accept ---------------------------------------------------------------------
        d.xhat, d.logits = xhat, gl
        a = O.accept(st, d, vo, prm.seed, prm.step, n, mode=mode, temperature=T, gamma=prm.gamma, resample=bool(prm.resample))
        j, L = vwin.j, vwin.L
        np.testing.assert_array_equal(g["u_used"][n, j:j + min(L, int(g["n_accept"][n]) + 1)].astype(np.float64),
                                      a.u[:min(L, int(g["n_accept"][n]) + 1)])
        ratios = vo.q / d.p[j:j + L]
        n_acc_gpu = int(g["n_accept"][n])
        if n_acc_gpu != a.n_accept:
            upto = min(L, max(n_acc_gpu, a.n_accept) + 1)
            assert (np.abs(ratios[:upto] - a.u[:upto]) < TIE).any(), f"seq {n}: n_accept {n_acc_gpu} vs {a.n_accept}"
            rep.exempt_ratio += 1
            # continue the comparison along the GPU's branch
            a = _accept_forced(st, d, vo, prm, n, n_acc_gpu, T)
        res_gpu = int(g["resampled"][n])
        if res_gpu != a.resampled:
            assert a.resampled >= 0 and res_gpu >= 0
            i = j + a.n_accept
            r = O.residual_distribution(gl[list(win.logit_index).index(i)], gv[a.n_accept], T)
            cdf = np.cumsum(r) / r.sum()
            u2 = O.uniform(prm.seed, prm.step, n, i, O.STREAM_RESAMPLE)
            assert abs(cdf[min(res_gpu, a.resampled)] - u2) < TIE, f"seq {n}: resampled {res_gpu} vs {a.resampled}"
            rep.exempt_resample += 1
            a.block[i] = res_gpu
        assert int(g["n_commit"][n]) == a.n_commit
        np.testing.assert_array_equal(g["block_tokens"][n], a.block)
        rep.n_commit.append(a.n_commit)
        rep.n_accept.append(a.n_accept)
        if not append:
            assert int(g["seq_len"][n]) == st.seq_len
            st.block = a.block
            rep.rows_checked += len(win.logit_index) + L
            continue
        # ---- stage 5: cache append -----------------------------------------------------------------
        n_lead = vwin.n_lead
        rows = n_lead + min(a.n_accept, vwin.n_causal - n_lead)   # (a right-shifted window has no row for the last draft)
        S0 = st.seq_len
        assert int(g["seq_len"][n]) == S0 + rows and int(g["status"][n]) == 0
        if ov is not None and rows:
            layers = range(cfg.n_layers) if check_kv_layers is None else check_kv_layers
            for l in layers:
                gk, gvv = run.cache_rows(n, S0, S0 + rows, l)
                for got, want in ((gk, ov.k[l][:rows]), (gvv, ov.v[l][:rows])):
                    err = np.abs(got - want).max() / max(np.abs(want).max(), 1e-30)
                    rep.max_kv_err = max(rep.max_kv_err, err)
                    assert err <= LOGIT_RTOL, f"seq {n} layer {l}: appended K/V off by {err:.3e}"
        st.block = a.block
        st.seq_len = S0 + rows
        st.carry = np.zeros(0, dtype=np.int64)
        rep.rows_checked += len(win.logit_index) + L
    return rep


def check_block_complete(case: Case, run: DeviceRun, causal: bool, rep: Optional[Report] = None) -> Report:
    """s2d2_block_complete on the device against the oracle's block_complete, sequence by sequence, on the state
    and cache held in `case` (synchronised with the device before the call).  Compares seq_len and the appended
    K/V rows of every layer; MoE: the oracle is held to the device's expert choices.  On return case.states hold
    the state after the append (not advanced)."""
    cfg, N, B = case.cfg, case.N, case.B
    rep = rep or Report()
    S0 = [s.seq_len for s in case.states]
    run.eng.s2d2_block_complete(run.kv, run.st, N, B, run.v, int(causal))
    choices = run.eng.s2d2_moe_choices(3 * N * B).cpu().numpy() if cfg.is_moe else None
    torch.cuda.synchronize(run.dev)
    run.eng.s2d2_status()
    sl = run.kv.seq_len.cpu().numpy()
    assert int(run.kv.status.abs().sum()) == 0
    row0 = 0
    for n, st in enumerate(case.states):
        finished = not (np.asarray(st.block) == cfg.mask_id).any()
        rows = len(st.carry) + (B - st.n_cached_in_block()) if finished else 0
        if causal and rows <= B:
            rows = 0
        if rows == 0:
            assert int(sl[n]) == S0[n]
            continue
        ck, cv = case.oracle_cache(n)
        forced = [choices[l, row0:row0 + rows] for l in range(cfg.n_layers)] if choices is not None else None
        k, v = [O.f64(x) for x in ck], [O.f64(x) for x in cv]
        assert O.block_complete(cfg, case.W, st, k, v, forced_experts=forced, causal=causal) == rows
        assert int(sl[n]) == S0[n] + rows == st.seq_len
        for l in range(cfg.n_layers):
            gk, gvv = run.cache_rows(n, S0[n], S0[n] + rows, l)
            for got, want in ((gk, k[l][S0[n]:]), (gvv, v[l][S0[n]:])):
                err = np.abs(got - want).max() / max(np.abs(want).max(), 1e-30)
                rep.max_kv_err = max(rep.max_kv_err, err)
                assert err <= LOGIT_RTOL, f"seq {n} layer {l}: completed-block K/V off by {err:.3e}"
        rep.rows_checked += rows
        row0 += rows
    return rep


def _accept_forced(st, d, vo, prm, n, n_acc, T=1.0):
    """Oracle accept along a prescribed accepted count (used after a near-tie exemption)."""
    j, L = vo.win.j, vo.win.L
    u = np.array([O.uniform(prm.seed, prm.step, n, j + r, O.STREAM_ACCEPT) for r in range(L)])
    block = np.array(st.block, copy=True)
    block[j:j + n_acc] = d.xhat[j:j + n_acc]
    resampled, n_commit = -1, n_acc
    if n_acc < L and prm.resample:
        i = j + n_acc
        row_d = int(np.nonzero(d.win.logit_index == i)[0][0])
        resampled = O.residual_resample(d.logits[row_d], vo.logits[n_acc], O.uniform(prm.seed, prm.step, n, i, O.STREAM_RESAMPLE), T)
        block[i] = resampled
        n_commit = n_acc + 1
    return O.AcceptOut(n_acc, n_commit, resampled, block, u)


def sync_case_from_gpu(case: Case, run: DeviceRun, seqs=None):
    """Adopts the GPU's cache contents and state as the stored inputs of the next step.  With `seqs`, only
    the pages of those sequences are copied back (full-size caches are tens of GB)."""
    torch.cuda.synchronize(run.dev)
    if seqs is None:
        k, v = run.kv.k.cpu(), run.kv.v.cpu()
        case.k_pages = [k[l] for l in range(case.cfg.n_layers)]
        case.v_pages = [v[l] for l in range(case.cfg.n_layers)]
    else:
        pages = torch.as_tensor(np.unique(case.page_table[list(seqs)].reshape(-1)).astype(np.int64))
        for l in range(case.cfg.n_layers):
            case.k_pages[l][pages] = run.kv.k[l][pages.to(run.dev)].cpu()
            case.v_pages[l][pages] = run.kv.v[l][pages.to(run.dev)].cpu()
    case.seq_len = run.kv.seq_len.cpu().numpy().copy()
    blk, pos0, car = run.st.block_tokens.cpu().numpy(), run.st.block_pos0.cpu().numpy(), run.st.carry_tokens.cpu().numpy()
    for n, s in enumerate(case.states):
        s.seq_len, s.pos0, s.block = int(case.seq_len[n]), int(pos0[n]), blk[n].astype(np.int64)
        s.carry = car[n, :max(0, s.pos0 - s.seq_len)].astype(np.int64)

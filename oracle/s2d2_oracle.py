"""CPU oracle for one S2D2 draft + verify + accept + cache-append step.  TEST INFRASTRUCTURE.

A plain, slow, fp64 numpy statement of what the step computes, written from the paper
(Section 4.1-4.2, Eq. 3, Eq. 4, Algorithms 1-3) and, for the decoder architecture the paper
leaves open, from the benchmark configurations (pre-norm, RMSNorm, RoPE, GQA, SwiGLU / MoE).
It shares no code with the HIP path and must never be imported by the product; only tests,
the smoke check and the benchmark's cpu_baseline leg call it.  Library primitives used as
steps: numpy matmul / einsum, exp, argsort.  No blocking, fusion or reordering.

Every function is pinned by tests/test_oracle_*.py against something other than itself
(library routines on special cases, closed forms, brute-force enumeration, published
known-answer vectors).  Not pinned ("parity unpinned"): none of the functions below; the
paper's *empirical* numbers (acceptance shares, speed-ups) need trained weights and are
not reproduced.

Readings taken where the paper is silent (each is listed in the design notes):
  * SampleFromLogits: greedy = arg-max token with its softmax probability at temperature 1;
    sample = inverse-CDF draw from softmax(logits / T) with its probability.
  * ratio and residual use the softmax distributions of draft and verifier logits.
  * ties: lowest index wins (token arg-max, position arg-max, expert top-k).
  * uniforms: Philox-4x32-10, u = (top 23 bits + 0.5) / 2^23 (odd multiples of 2^-24: exact in fp32), accept iff u * p < q.
  * residual draw: inverse CDF in ascending vocabulary order.
  * right-shifted models (cfg.right_shifted): logits of block index i are read at the row of position i-1 in both
    forwards; the verifier window is plain causal without [MASK] copies; the cache lags one token behind the
    committed text so that this row is always a window row.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional, Sequence, Tuple

import numpy as np

# --------------------------------------------------------------------------------------
# Counter-based uniforms: Philox-4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11).
# --------------------------------------------------------------------------------------
_PH_M0, _PH_M1 = 0xD2511F53, 0xCD9E8D57
_PH_W0, _PH_W1 = 0x9E3779B9, 0xBB67AE85
_U32 = 0xFFFFFFFF

STREAM_ACCEPT, STREAM_RESAMPLE, STREAM_DRAFT = 0, 1, 2


def philox4x32_10(ctr: Sequence[int], key: Sequence[int]) -> Tuple[int, int, int, int]:
    c0, c1, c2, c3 = (int(c) & _U32 for c in ctr)
    k0, k1 = (int(k) & _U32 for k in key)
    for _ in range(10):
        p0 = _PH_M0 * c0
        p1 = _PH_M1 * c2
        hi0, lo0 = p0 >> 32, p0 & _U32
        hi1, lo1 = p1 >> 32, p1 & _U32
        c0, c1, c2, c3 = (hi1 ^ c1 ^ k0) & _U32, lo1, (hi0 ^ c3 ^ k1) & _U32, lo0
        k0 = (k0 + _PH_W0) & _U32
        k1 = (k1 + _PH_W1) & _U32
    return c0, c1, c2, c3


def uniform(seed: int, step: int, seq: int, index: int, stream: int) -> float:
    """u in (0,1): key = 64-bit seed, counter = (step, sequence, block index, stream)."""
    out = philox4x32_10((step, seq, index, stream), (seed & _U32, (seed >> 32) & _U32))
    return ((out[0] >> 9) + 0.5) / 8388608.0


# --------------------------------------------------------------------------------------
# Decoder forward (the black box x_theta of Algorithms 1-3) with a prefix cache and an
# arbitrary in-window visibility matrix.
# --------------------------------------------------------------------------------------
def f64(x) -> np.ndarray:
    """Up-cast a stored tensor (torch bf16/fp32 or numpy) to fp64 without changing its value."""
    if hasattr(x, "detach"):
        import torch
        return x.detach().to(torch.float64).cpu().numpy()
    return np.asarray(x, dtype=np.float64)


class LazyF64Weights(dict):
    """The same stored weights, with the expert tensors of the most recently used layer kept up-cast to
    fp64 so that the oracle's per-(row, expert) up-casts become no-ops.  Values are unchanged."""

    def __init__(self, W):
        super().__init__(W)
        self._key, self._val = {}, {}

    def __getitem__(self, k):
        base = k.split(".")[-1]
        if base in ("e_wgu", "e_wdown"):
            if self._key.get(base) != k:
                self._key[base], self._val[base] = k, f64(super().__getitem__(k))
            return self._val[base]
        return super().__getitem__(k)


def take_rows(table, idx: np.ndarray) -> np.ndarray:
    if hasattr(table, "detach"):
        import torch
        return f64(table[torch.as_tensor(np.asarray(idx), dtype=torch.long)])
    return f64(np.asarray(table)[np.asarray(idx)])


def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * g


def rope(x: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotary embedding, half-split pairing: element i is rotated with element i + D/2."""
    D = x.shape[-1]
    half = D // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / D)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv_freq[None, :]  # [n, half]
    cos, sin = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * cos - x2 * sin, x2 * cos + x1 * sin], axis=-1)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def softmax_rows(s: np.ndarray) -> np.ndarray:
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def dense_ffn(b: np.ndarray, wgu: np.ndarray, wdown: np.ndarray) -> np.ndarray:
    return (silu(b @ wgu[0].T) * (b @ wgu[1].T)) @ wdown.T


def topk_lowest_index(scores: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k largest entries of each row, ties to the lower index, largest first."""
    order = np.argsort(-scores, axis=-1, kind="stable")
    return order[..., :k]


def moe_ffn(b: np.ndarray, router: np.ndarray, e_wgu, e_wdown, top_k: int,
            forced: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Softmax router over all experts, top-k, weights renormalised to sum 1, no shared expert."""
    s = softmax_rows(b @ router.T)  # [n, E]
    chosen = topk_lowest_index(s, top_k) if forced is None else np.asarray(forced)
    out = np.zeros_like(b)
    for r in range(b.shape[0]):
        w = s[r, chosen[r]]
        w = w / np.sum(w)
        for e, we in zip(chosen[r], w):
            out[r] += we * dense_ffn(b[r:r + 1], f64(e_wgu[e]), f64(e_wdown[e]))[0]
    return out, chosen


@dataclass
class ForwardOut:
    logits: np.ndarray                 # [len(logit_rows), V]
    k: List[np.ndarray]                # per layer [n, Hkv, D] post-RoPE keys of the window rows
    v: List[np.ndarray]                # per layer [n, Hkv, D]
    experts: List[np.ndarray] = field(default_factory=list)  # per layer [n, top_k] (MoE)
    hidden: Optional[np.ndarray] = None


def forward(cfg, W: Dict, tokens: np.ndarray, pos: np.ndarray, vis: np.ndarray,
            cache_k: Sequence, cache_v: Sequence, logit_rows: Optional[np.ndarray] = None,
            forced_experts: Optional[Sequence[np.ndarray]] = None) -> ForwardOut:
    """One forward over the `n` window rows of ONE sequence.

    tokens[n], pos[n]: ids and absolute positions of the window rows.
    vis[n, n]: vis[r, c] true iff row r attends to window row c.  Every row additionally
    attends to all cached positions cache_k[l][0:S] (prefix cache, fully visible).
    cache_k[l], cache_v[l]: [S, Hkv, D] stored (post-RoPE) keys / values of layer l.
    """
    n = len(tokens)
    Hq, Hkv, D = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    grp = Hq // Hkv
    pos = np.asarray(pos)
    vis = np.asarray(vis, dtype=bool)
    h = take_rows(W["embed"], tokens)
    ks, vs, ex = [], [], []
    for l in range(cfg.n_layers):
        a = rmsnorm(h, f64(W[f"l{l}.norm1"]), cfg.rms_eps)
        qkv = a @ f64(W[f"l{l}.wqkv"]).T
        q = qkv[:, :Hq * D].reshape(n, Hq, D)
        k = qkv[:, Hq * D:(Hq + Hkv) * D].reshape(n, Hkv, D)
        v = qkv[:, (Hq + Hkv) * D:].reshape(n, Hkv, D)
        q = rope(q, pos, cfg.rope_theta)
        k = rope(k, pos, cfg.rope_theta)
        ks.append(k)
        vs.append(v)
        kc, vc = f64(cache_k[l]), f64(cache_v[l])  # [S, Hkv, D]
        o = np.zeros((n, Hq, D))
        for hq in range(Hq):
            g = hq // grp  # query head hq reads KV head floor(hq / (Hq/Hkv))
            s_c = q[:, hq, :] @ kc[:, g, :].T                       # [n, S]
            s_w = np.where(vis, q[:, hq, :] @ k[:, g, :].T, -np.inf)  # [n, n]
            p = softmax_rows(np.concatenate([s_c, s_w], axis=1) / np.sqrt(D))
            o[:, hq, :] = p[:, :kc.shape[0]] @ vc[:, g, :] + p[:, kc.shape[0]:] @ v[:, g, :]
        h = h + o.reshape(n, Hq * D) @ f64(W[f"l{l}.wo"]).T
        b = rmsnorm(h, f64(W[f"l{l}.norm2"]), cfg.rms_eps)
        if cfg.is_moe:
            y, chosen = moe_ffn(b, f64(W[f"l{l}.router"]), W[f"l{l}.e_wgu"], W[f"l{l}.e_wdown"],
                                cfg.top_k, None if forced_experts is None else forced_experts[l])
            ex.append(chosen)
        else:
            y = dense_ffn(b, f64(W[f"l{l}.wgu"]), f64(W[f"l{l}.wdown"]))
        h = h + y
    rows = np.arange(n) if logit_rows is None else np.asarray(logit_rows, dtype=np.int64)
    hf = rmsnorm(h[rows], f64(W["norm_f"]), cfg.rms_eps)
    logits = hf @ f64(W["unembed"]).T if len(rows) else np.zeros((0, cfg.vocab))
    return ForwardOut(logits=logits, k=ks, v=vs, experts=ex, hidden=h)


# --------------------------------------------------------------------------------------
# Attention masks of the method.
# --------------------------------------------------------------------------------------
def causal_mask(n: int) -> np.ndarray:
    return np.tril(np.ones((n, n), dtype=bool))


def draft_mask(B: int, j: int) -> np.ndarray:
    """Eq. 4: the committed in-block prefix (< j) is causal, every other row sees the whole block."""
    m = np.ones((B, B), dtype=bool)
    m[:j, :j] = causal_mask(j)
    m[:j, j:] = False
    return m


def verify_mask(L: int) -> np.ndarray:
    """Eq. 3: [[A_L, 0], [A_L strictly lower, I_L]] over [drafted tokens, MASK copies]."""
    A = causal_mask(L)
    top = np.concatenate([A, np.zeros((L, L), dtype=bool)], axis=1)
    bot = np.concatenate([np.tril(np.ones((L, L), dtype=bool), k=-1), np.eye(L, dtype=bool)], axis=1)
    return np.concatenate([top, bot], axis=0)


# --------------------------------------------------------------------------------------
# Per-sequence decoding state and the two windows built from it.
# --------------------------------------------------------------------------------------
@dataclass
class SeqState:
    """State of one sequence between steps.

    seq_len: number of tokens whose K/V are in the cache (positions 0..seq_len-1).
    pos0:    absolute position of block index 0.
    block:   [B] committed token id or mask_id.
    carry:   committed tokens of earlier blocks that are not cached yet; they sit at
             positions seq_len .. pos0-1 (non-empty only if seq_len < pos0).
    Invariant: either carry is empty and seq_len - pos0 = number of cached block tokens,
    or seq_len + len(carry) = pos0.
    """
    seq_len: int
    pos0: int
    block: np.ndarray
    carry: np.ndarray = field(default_factory=lambda: np.zeros(0, dtype=np.int64))

    def n_cached_in_block(self) -> int:
        return max(0, self.seq_len - self.pos0)


@dataclass
class Window:
    tokens: np.ndarray
    pos: np.ndarray
    vis: np.ndarray
    logit_rows: np.ndarray      # window rows whose logits are needed
    logit_index: np.ndarray     # block index each of those rows scores
    j: int                      # first masked block index (B if none)
    L: int                      # length of the first contiguous masked span C_t
    n_causal: int = 0           # verify window: number of leading causal rows (pending + drafted)
    n_lead: int = 0             # verify window: uncached committed tokens left of C_t (the first rows)


def first_span(block: np.ndarray, mask_id: int) -> Tuple[int, int]:
    """(j, L): start and length of the first maximal run of [MASK] in the block (Alg. 3, C_t)."""
    B = len(block)
    masked = np.asarray(block) == mask_id
    if not masked.any():
        return B, 0
    j = int(np.argmax(masked))
    L = 0
    while j + L < B and masked[j + L]:
        L += 1
    return j, L


def draft_window(st: SeqState, mask_id: int, ar_mask: bool = True) -> Window:
    """Window of the draft forward: every block position not yet in the cache, preceded by the
    uncached committed tokens of earlier blocks.  Visibility: carried tokens are causal
    (they belong to finished blocks); inside the block Eq. 4 with j = first masked index
    (ar_mask) or all-ones (plain block diffusion).  The prefix cache is always visible."""
    B = len(st.block)
    c = st.n_cached_in_block()
    j, L = first_span(st.block, mask_id)
    nc = len(st.carry)
    tokens = np.concatenate([np.asarray(st.carry, dtype=np.int64), np.asarray(st.block[c:], dtype=np.int64)])
    pos = st.seq_len + np.arange(len(tokens))
    n = len(tokens)
    full = draft_mask(B, j if ar_mask else 0)[c:, c:]
    vis = np.zeros((n, n), dtype=bool)
    vis[:nc, :nc] = causal_mask(nc)
    vis[nc:, :nc] = True
    vis[nc:, nc:] = full
    masked_idx = np.nonzero(np.asarray(st.block) == mask_id)[0]
    return Window(tokens, pos, vis, logit_rows=nc + masked_idx - c, logit_index=masked_idx, j=j, L=L)


def shifted_draft_window(st: SeqState, mask_id: int, ar_mask: bool = True) -> Window:
    """Draft window of a right-shifted model (Section 4.2, last sentence before the related-work remark: models
    whose output at position i-1 is the distribution of token i).  Same rows and visibility as draft_window; the
    logits of a masked block index are read from the row of the position in front of it.  That row must be in the
    window: the committed token in front of the first [MASK] is not cached yet (the cache of such a model lags one
    token behind the committed text; shifted_prefill_state sets a prefilled sequence up that way)."""
    w = draft_window(st, mask_id, ar_mask)
    rows = w.logit_rows - 1
    if len(rows) and rows.min() < 0:
        raise ValueError("right-shifted drafting needs the token in front of the first [MASK] as a window row")
    return Window(w.tokens, w.pos, w.vis, logit_rows=rows, logit_index=w.logit_index, j=w.j, L=w.L)


def verify_window(st: SeqState, xhat: np.ndarray, mask_id: int) -> Window:
    """Window of the verifier forward (2L trick): all uncached committed tokens left of C_t and
    the drafted tokens of C_t as causal rows, then one [MASK] copy per drafted token at the
    same position, which sees the causal rows strictly left of its position and itself
    (Eq. 3 with the leading committed tokens riding along as ordinary causal rows)."""
    c = st.n_cached_in_block()
    j, L = first_span(st.block, mask_id)
    nc = len(st.carry)
    pend = np.asarray(st.block[c:j], dtype=np.int64)
    drafted = np.asarray(xhat[j:j + L], dtype=np.int64)
    causal_tokens = np.concatenate([np.asarray(st.carry, dtype=np.int64), pend, drafted])
    na = len(causal_tokens)
    n_lead = na - L
    tokens = np.concatenate([causal_tokens, np.full(L, mask_id, dtype=np.int64)])
    pos_causal = st.seq_len + np.arange(na)
    pos = np.concatenate([pos_causal, pos_causal[n_lead:]])
    n = na + L
    vis = np.zeros((n, n), dtype=bool)
    vis[:na, :na] = causal_mask(na)
    vm = verify_mask(L)
    vis[na:, :n_lead] = True
    vis[na:, n_lead:na] = vm[L:, :L]
    vis[na:, na:] = vm[L:, L:]
    return Window(tokens, pos, vis, logit_rows=na + np.arange(L), logit_index=j + np.arange(L),
                  j=j, L=L, n_causal=na, n_lead=n_lead)


def shifted_verify_window(st: SeqState, xhat: np.ndarray, mask_id: int) -> Window:
    """Verifier window of a right-shifted model: the plain causal mask already gives the verifier view (Section 4.2),
    so there are no [MASK] copies.  Rows: the uncached committed tokens left of C_t, then the first L-1 drafted
    tokens, all causal; the row at position i-1 yields the verifier distribution of the drafted token at i, i.e.
    the L logit rows start at the last leading row.  The last drafted token needs no row of its own."""
    c = st.n_cached_in_block()
    j, L = first_span(st.block, mask_id)
    pend = np.asarray(st.block[c:j], dtype=np.int64)
    lead_tokens = np.concatenate([np.asarray(st.carry, dtype=np.int64), pend])
    n_lead = len(lead_tokens)
    if L > 0 and n_lead == 0:
        raise ValueError("right-shifted verification needs the token in front of C_t as a window row")
    tokens = np.concatenate([lead_tokens, np.asarray(xhat[j:j + max(L - 1, 0)], dtype=np.int64)])
    na = len(tokens)
    pos = st.seq_len + np.arange(na)
    return Window(tokens, pos, causal_mask(na), logit_rows=n_lead - 1 + np.arange(L), logit_index=j + np.arange(L),
                  j=j, L=L, n_causal=na, n_lead=n_lead)


def shifted_prefill_state(seq_len: int, last_token: int, B: int, mask_id: int) -> SeqState:
    """State of a right-shifted model after a prompt of seq_len tokens: its last token stays out of the cache and is
    carried in front of the first block (cache rows at or past seq_len - 1 are not part of the state)."""
    return SeqState(seq_len=seq_len - 1, pos0=seq_len, block=np.full(B, mask_id, dtype=np.int64),
                    carry=np.array([last_token], dtype=np.int64))


# --------------------------------------------------------------------------------------
# Vocabulary-wide sampling primitives (SampleFromLogits, ScoreFromLogits, residual).
# --------------------------------------------------------------------------------------
GREEDY, SAMPLE = 0, 1


def log_softmax_stats(logits: np.ndarray, temperature: float = 1.0):
    """(P, lse) of softmax(logits / T); lse is the log normaliser of the scaled logits."""
    z = np.asarray(logits, dtype=np.float64) / temperature
    m = np.max(z)
    lse = m + np.log(np.sum(np.exp(z - m)))
    return np.exp(z - lse), lse


def inverse_cdf(weights: np.ndarray, u: float) -> int:
    """Smallest index v with sum_{w<=v} weights[w] > u * sum(weights) (ascending index order)."""
    cdf = np.cumsum(weights)
    v = int(np.searchsorted(cdf, u * cdf[-1], side="right"))
    return min(v, len(weights) - 1)


def sample_from_logits(logits: np.ndarray, mode: int = GREEDY, temperature: float = 1.0,
                       u: Optional[float] = None) -> Dict[str, float]:
    """SampleFromLogits (Alg. 2/3): proposal x_hat, its probability p, plus the statistics the
    routing proxies need (Section 4.3): top-1 minus top-2 probability and H / log V."""
    T = 1.0 if mode == GREEDY else temperature
    P, lse = log_softmax_stats(logits, T)
    order = np.argsort(-P, kind="stable")
    if mode == GREEDY:
        x = int(order[0])  # arg-max, lowest index on ties
    else:
        x = inverse_cdf(P, u)
    nz = P > 0
    H = -np.sum(P[nz] * np.log(P[nz]))
    return dict(xhat=x, p=float(P[x]), lse=float(lse), margin=float(P[order[0]] - P[order[1]]),
                entropy_n=float(H / np.log(len(P))), top1=int(order[0]))


def score_from_logits(logits_ver: np.ndarray, token: int, temperature: float = 1.0) -> Tuple[float, float]:
    """ScoreFromLogits (Alg. 3): verifier probability q of a given token, and the row's lse."""
    Q, lse = log_softmax_stats(logits_ver, temperature)
    return float(Q[token]), float(lse)


def threshold_set(p: np.ndarray, masked: np.ndarray, tau: float) -> Tuple[np.ndarray, int]:
    """Alg. 2: S = {i in M : p_i > tau} united with the arg-max-confidence masked position."""
    masked = np.asarray(masked, dtype=bool)
    S = masked & (np.asarray(p) > tau)
    n_hi = int(S.sum())
    if masked.any():
        pm = np.where(masked, p, -np.inf)
        S = S.copy()
        S[int(np.argmax(pm))] = True  # np.argmax returns the lowest index among ties
    return S, n_hi


def accept_scan(p: np.ndarray, q: np.ndarray, u: np.ndarray, gamma: float = 1.0) -> int:
    """Left-to-right speculative acceptance (Alg. 3): position i passes iff u_i < min(1, (q_i/p_i)^gamma),
    decided as u_i * p_i < q_i for gamma = 1.  Returns the number of positions passed before
    the first failure."""
    n = 0
    for pi, qi, ui in zip(p, q, u):
        ok = (ui * pi < qi) if gamma == 1.0 else (ui < min(1.0, (qi / pi) ** gamma))
        if not ok:
            break
        n += 1
    return n


def residual_distribution(logits_draft: np.ndarray, logits_ver: np.ndarray, temperature: float = 1.0) -> np.ndarray:
    """(P_ver - P_draft)_+, unnormalised."""
    P, _ = log_softmax_stats(logits_draft, temperature)
    Q, _ = log_softmax_stats(logits_ver, temperature)
    return np.maximum(Q - P, 0.0)


def residual_resample(logits_draft: np.ndarray, logits_ver: np.ndarray, u2: float,
                      temperature: float = 1.0) -> int:
    r = residual_distribution(logits_draft, logits_ver, temperature)
    assert r.sum() > 0.0, "a rejection implies q < p at the drafted token, so the residual has mass"
    return inverse_cdf(r, u2)


# --------------------------------------------------------------------------------------
# The step: draft, verify, accept, cache append, next block.
# --------------------------------------------------------------------------------------
@dataclass
class DraftOut:
    win: Window
    logits: np.ndarray        # [len(win.logit_rows), V] draft logits of the masked positions
    xhat: np.ndarray          # [B] proposal per block index (-1 where the position is committed)
    p: np.ndarray             # [B] its draft probability (0 where committed)
    lse: np.ndarray
    margin: np.ndarray
    entropy_n: np.ndarray
    unmask: np.ndarray        # [B] bool threshold set S_t^tau (the fallback branch of Alg. 3)
    n_hi: int
    fwd: Optional[ForwardOut] = None


@dataclass
class VerifyOut:
    win: Window
    logits: np.ndarray        # [L, V] verifier logits of the MASK copies
    q: np.ndarray             # [L]
    lse: np.ndarray           # [L]
    k: List[np.ndarray]       # per layer [n_causal, Hkv, D]: K of the causal (drafted-half) rows
    v: List[np.ndarray]
    fwd: Optional[ForwardOut] = None


@dataclass
class AcceptOut:
    n_accept: int
    n_commit: int
    resampled: int            # -1 if no rejection happened
    block: np.ndarray
    u: np.ndarray             # uniforms consumed by the scan, [L]


def draft_from_logits(st: SeqState, win: Window, logits: np.ndarray, mask_id: int, tau: float,
                      mode: int = GREEDY, temperature: float = 1.0, seed: int = 0, step: int = 0,
                      seq: int = 0) -> DraftOut:
    """Everything in s2d2 drafting that follows the forward: proposals, M_t, threshold set."""
    B = len(st.block)
    xhat = np.full(B, -1, dtype=np.int64)
    p, lse, margin, ent = (np.zeros(B) for _ in range(4))
    for r, i in enumerate(win.logit_index):
        u = uniform(seed, step, seq, int(i), STREAM_DRAFT) if mode == SAMPLE else None
        s = sample_from_logits(logits[r], mode, temperature, u)
        xhat[i], p[i], lse[i], margin[i], ent[i] = s["xhat"], s["p"], s["lse"], s["margin"], s["entropy_n"]
    masked = np.asarray(st.block) == mask_id
    unmask, n_hi = threshold_set(p, masked, tau)
    return DraftOut(win, logits, xhat, p, lse, margin, ent, unmask, n_hi)


def draft(cfg, W, st: SeqState, cache_k, cache_v, tau: float, ar_mask: bool = True, mode: int = GREEDY,
          temperature: float = 1.0, seed: int = 0, step: int = 0, seq: int = 0,
          forced_experts=None) -> DraftOut:
    """Alg. 3, draft forward + SampleFromLogits + M_t, C_t (+ the threshold set of its else-branch)."""
    win = (shifted_draft_window if getattr(cfg, "right_shifted", False) else draft_window)(st, cfg.mask_id, ar_mask)
    fo = forward(cfg, W, win.tokens, win.pos, win.vis, cache_k, cache_v, win.logit_rows, forced_experts)
    out = draft_from_logits(st, win, fo.logits, cfg.mask_id, tau, mode, temperature, seed, step, seq)
    out.fwd = fo
    return out


def verify_from_logits(win: Window, logits_ver: np.ndarray, xhat: np.ndarray, k, v, mode: int = GREEDY,
                       temperature: float = 1.0) -> VerifyOut:
    T = 1.0 if mode == GREEDY else temperature
    q, lse = np.zeros(win.L), np.zeros(win.L)
    for r, i in enumerate(win.logit_index):
        q[r], lse[r] = score_from_logits(logits_ver[r], int(xhat[i]), T)
    return VerifyOut(win, logits_ver, q, lse, k, v)


def verify(cfg, W, st: SeqState, cache_k, cache_v, xhat: np.ndarray, mode: int = GREEDY,
           temperature: float = 1.0, forced_experts=None) -> VerifyOut:
    """Alg. 3, verifier forward under block-size-1 masking (2L trick; plain causal rows for a right-shifted
    model) + ScoreFromLogits."""
    win = (shifted_verify_window if getattr(cfg, "right_shifted", False) else verify_window)(st, xhat, cfg.mask_id)
    fo = forward(cfg, W, win.tokens, win.pos, win.vis, cache_k, cache_v, win.logit_rows, forced_experts)
    na = win.n_causal
    out = verify_from_logits(win, fo.logits, xhat, [k[:na] for k in fo.k], [v[:na] for v in fo.v],
                             mode, temperature)
    out.fwd = fo
    return out


def accept(st: SeqState, d: DraftOut, vo: VerifyOut, seed: int, step: int, seq: int,
           mode: int = GREEDY, temperature: float = 1.0, gamma: float = 1.0,
           resample: bool = True) -> AcceptOut:
    """Alg. 3 accept loop: scan C_t left to right; the first failing position gets a token drawn
    from the residual (P_ver - P_draft)_+ and ends the scan.  Writes the committed tokens."""
    T = 1.0 if mode == GREEDY else temperature
    j, L = vo.win.j, vo.win.L
    u = np.array([uniform(seed, step, seq, j + r, STREAM_ACCEPT) for r in range(L)])
    n_acc = accept_scan(d.p[j:j + L], vo.q, u, gamma)
    block = np.array(st.block, copy=True)
    block[j:j + n_acc] = d.xhat[j:j + n_acc]
    resampled, n_commit = -1, n_acc
    if n_acc < L and resample:
        i = j + n_acc
        row_d = int(np.nonzero(d.win.logit_index == i)[0][0])
        u2 = uniform(seed, step, seq, i, STREAM_RESAMPLE)
        resampled = residual_resample(d.logits[row_d], vo.logits[n_acc], u2, T)
        block[i] = resampled
        n_commit = n_acc + 1
    return AcceptOut(n_acc, n_commit, resampled, block, u)


def kv_append(st: SeqState, cache_k: List[np.ndarray], cache_v: List[np.ndarray], vo: VerifyOut,
              n_accept: int) -> int:
    """Append to the cache the K/V of every causal verify row up to the accepted prefix:
    the uncached committed tokens left of C_t and C_t[0:n_accept).  Those rows were computed
    under a causal mask (AR caching, Section 4.2), so they are final.  A right-shifted verifier window holds no
    row for the last drafted token: if all of C_t is accepted that token stays uncached, as the token in front
    of the next [MASK] must be.  Returns rows appended; updates cache lists in place and st.seq_len."""
    n_lead = vo.win.n_lead
    rows = n_lead + min(n_accept, vo.win.n_causal - n_lead)
    for l in range(len(cache_k)):
        cache_k[l] = np.concatenate([f64(cache_k[l]), vo.k[l][:rows]], axis=0)
        cache_v[l] = np.concatenate([f64(cache_v[l]), vo.v[l][:rows]], axis=0)
    st.seq_len += rows
    st.carry = np.zeros(0, dtype=np.int64)
    return rows


def commit_threshold(st: SeqState, d: DraftOut) -> int:
    """Else-branch of Alg. 3 / body of Alg. 2: write the proposals of the threshold set."""
    st.block = np.where(d.unmask, d.xhat, st.block)
    return int(d.unmask.sum())


# --------------------------------------------------------------------------------------
# Verification routing (Section 4.3: Eq. 5 and the score below it; Algorithm "DoVerify").
# --------------------------------------------------------------------------------------
ROUTE_MIN_SPAN, ROUTE_SCORE, ROUTE_HYSTERESIS = 0, 1, 2
EST_MARGIN, EST_ENTROPY = 0, 1
H_OFF, H_ON = 0, 1


@dataclass
class RouteParams:
    policy: int = ROUTE_MIN_SPAN
    estimator: int = EST_ENTROPY
    dynamic: bool = True          # s = K - c N_hi (dynamic) or s = K - c (static)
    tau_span: int = 1
    tau_score: float = 0.0
    tau_on: float = 1.0
    tau_off: float = -5.0
    c: float = 1.0
    beta: float = 1.0             # entropy proxy alpha = exp(-beta H / ln V)
    tau_margin: float = 0.5       # margin proxy alpha = 1[m >= tau_margin]


def acceptance_proxy(margin: np.ndarray, entropy_n: np.ndarray, estimator: int, tau_margin: float,
                     beta: float) -> np.ndarray:
    """alpha_i of Section 4.3 for the positions given: indicator of the top-1 minus top-2 margin, or
    exp(-beta * normalised entropy)."""
    if estimator == EST_MARGIN:
        return (f64(margin) >= tau_margin).astype(np.float64)
    return np.exp(-beta * f64(entropy_n))


def expected_prefix_length(alpha: np.ndarray) -> float:
    """Eq. 5: K = sum over k = 1..L of the product of alpha_1 .. alpha_k (each product taken anew)."""
    total = 0.0
    for k in range(1, len(alpha) + 1):
        prod = 1.0
        for i in range(k):
            prod *= float(alpha[i])
        total += prod
    return total


def verify_score(khat: float, n_hi: int, c: float, dynamic: bool) -> float:
    """Static score K - c, dynamic score K - c * N_hi (Section 4.3)."""
    return khat - c * n_hi if dynamic else khat - c


def do_verify(rp: RouteParams, L: int, score: float, h: int) -> Tuple[bool, int]:
    """Algorithm DoVerify: returns (decision, hysteresis state after the call).  A block without a
    masked span (L = 0) has nothing to verify under any policy."""
    if L <= 0:
        return False, h
    if rp.policy == ROUTE_MIN_SPAN:
        return bool(L >= rp.tau_span), h
    if rp.policy == ROUTE_SCORE:
        return bool(score >= rp.tau_score), h
    if h == H_ON and score < rp.tau_off:
        h = H_OFF
    elif h == H_OFF and score >= rp.tau_on:
        h = H_ON
    return h == H_ON, h


def route(st: SeqState, d: DraftOut, mask_id: int, rp: RouteParams, h: int = H_ON):
    """K, score and decision for one sequence from the draft's statistics over C_t."""
    j, L = first_span(np.asarray(st.block), mask_id)
    alpha = acceptance_proxy(d.margin[j:j + L], d.entropy_n[j:j + L], rp.estimator, rp.tau_margin, rp.beta)
    khat = expected_prefix_length(alpha)
    score = verify_score(khat, d.n_hi, rp.c, rp.dynamic)
    decision, h2 = do_verify(rp, L, score, h)
    return dict(khat=khat, score=score, verify=decision, h=h2, L=L)


def block_advance(st: SeqState, mask_id: int) -> bool:
    """Alg. 1: once the block holds no [MASK], start a fresh [MASK]^B block right after it.
    Committed tokens of the finished block that are not cached yet are carried."""
    B = len(st.block)
    if (np.asarray(st.block) == mask_id).any():
        return False
    c = st.n_cached_in_block()
    st.carry = np.concatenate([np.asarray(st.carry, dtype=np.int64), np.asarray(st.block[c:], dtype=np.int64)])
    st.pos0 += B
    st.block = np.full(B, mask_id, dtype=np.int64)
    return True


def step(cfg, W, st: SeqState, cache_k, cache_v, tau: float, seed: int, step_idx: int, seq: int = 0,
         ar_mask: bool = True, mode: int = GREEDY, temperature: float = 1.0):
    """One always-verified S2D2 step on one sequence: draft, verify, accept, append, roll."""
    d = draft(cfg, W, st, cache_k, cache_v, tau, ar_mask, mode, temperature, seed, step_idx, seq)
    vo = verify(cfg, W, st, cache_k, cache_v, d.xhat, mode, temperature)
    a = accept(st, d, vo, seed, step_idx, seq, mode, temperature)
    st.block = a.block
    kv_append(st, cache_k, cache_v, vo, a.n_accept)
    block_advance(st, cfg.mask_id)
    return d, vo, a


def step_routed(cfg, W, st: SeqState, cache_k, cache_v, tau: float, seed: int, step_idx: int, rp: RouteParams,
                h: int = H_ON, seq: int = 0, ar_mask: bool = True, mode: int = GREEDY, temperature: float = 1.0):
    """Alg. 3 in full: draft; DoVerify; then either verify + accept + append, or the threshold-set
    commit of Alg. 2.  Returns (draft, route record, verify or None, accept or None)."""
    d = draft(cfg, W, st, cache_k, cache_v, tau, ar_mask, mode, temperature, seed, step_idx, seq)
    r = route(st, d, cfg.mask_id, rp, h)
    vo = a = None
    if r["verify"]:
        vo = verify(cfg, W, st, cache_k, cache_v, d.xhat, mode, temperature)
        a = accept(st, d, vo, seed, step_idx, seq, mode, temperature)
        st.block = a.block
        kv_append(st, cache_k, cache_v, vo, a.n_accept)
    else:
        commit_threshold(st, d)
    block_advance(st, cfg.mask_id)
    return d, r, vo, a


# --------------------------------------------------------------------------------------
# Alg. 1, lines after SampleBlock: forward over the finished block, whole-block cache append.
# --------------------------------------------------------------------------------------
def block_complete(cfg, W, st: SeqState, cache_k: List[np.ndarray], cache_v: List[np.ndarray],
                   forced_experts=None, causal: bool = False) -> int:
    """Once the block holds no [MASK]: one forward over its tokens that are not cached yet (and over
    carried tokens of earlier blocks, which stay causal), with the block's rows attending to the whole
    block (block-diffusion attention), and append of all their K/V.  Returns the rows appended (0 if the
    block is unfinished).  This is the cache update of the variant that does not cache causally inside a
    block (Section 4.2 describes the causal alternative the incremental append relies on).
    causal=True is that alternative applied to a whole finished block: every row sees only the rows left of it, so
    the appended K/V are those a causal prefill of the text would give (used by generate when a block was finished
    without a verifier forward that could have cached it).  forced_experts (MoE): expert choices per layer."""
    if getattr(cfg, "right_shifted", False):
        raise ValueError("whole-block append is not defined here for right-shifted models (their cache lags one token)")
    block = np.asarray(st.block)
    if (block == cfg.mask_id).any():
        return 0
    c = st.n_cached_in_block()
    carry = np.asarray(st.carry, dtype=np.int64)
    toks = np.concatenate([carry, block[c:].astype(np.int64)])
    n, nc = len(toks), len(carry)
    if n == 0:
        return 0
    pos = st.seq_len + np.arange(n)
    vis = np.zeros((n, n), dtype=bool)
    for r in range(n):
        if r < nc or causal:
            vis[r, :r + 1] = True          # carried tokens: causal
        else:
            vis[r, :] = True               # block rows: everything in the window
    fo = forward(cfg, W, toks, pos, vis, cache_k, cache_v, logit_rows=np.zeros(0, dtype=np.int64),
                 forced_experts=forced_experts)
    for l in range(cfg.n_layers):
        cache_k[l] = np.concatenate([f64(cache_k[l]), fo.k[l]], axis=0)
        cache_v[l] = np.concatenate([f64(cache_v[l]), fo.v[l]], axis=0)
    st.seq_len += n
    st.carry = np.zeros(0, dtype=np.int64)
    return n


def generate(cfg, W, st: SeqState, cache_k, cache_v, n_blocks: int, tau: float, seed: int, rp: RouteParams,
             max_steps_per_block: int, caching: str = "causal", seq: int = 0, mode: int = GREEDY,
             temperature: float = 1.0, carry_cap: Optional[int] = None):
    """Alg. 1's outer loop around the block sampler of Alg. 3, for n_blocks blocks, at most max_steps_per_block
    denoising steps per block (a block that runs out of steps commits the threshold set of a tau = 0 pass, i.e.
    every remaining proposal).  caching = "causal": the accepted prefix is appended after every verified step
    (Section 4.2); "block": nothing is appended inside a block (drafting then sees the block fully
    bidirectionally) and the finished block is appended by block_complete.  Under causal caching a block that
    fallback steps finished has tokens no verifier forward cached; they are carried in front of the next block
    and cached by its first verified step.  Alg. 1 appends every block's K/V before the next block is sampled; the
    carry only defers that, and it is bounded: when the carried tokens plus the finished block's uncached ones
    would exceed carry_cap (default B, the carry capacity of the C boundary), they are cached at once by one
    causal forward (block_complete with causal=True), which is Alg. 1's per-block cache update under the causal
    mask of Section 4.2.  The committed tokens do not depend on carry_cap (causal K/V are the same whenever they
    are computed); only seq_len bookkeeping does.  Returns the committed tokens and the per-step records."""
    assert caching in ("causal", "block")
    out, log, h, step_idx = [], [], H_ON, 0
    B = len(st.block)
    for _ in range(n_blocks):
        for t in range(max_steps_per_block + 1):
            last = t == max_steps_per_block
            ar = caching == "causal"
            d = draft(cfg, W, st, cache_k, cache_v, 0.0 if last else tau, ar, mode, temperature, seed, step_idx, seq)
            r = route(st, d, cfg.mask_id, rp, h)
            h = r["h"]
            if last:
                r = dict(r, verify=False)
                d.unmask = np.asarray(st.block) == cfg.mask_id     # out of steps: commit every proposal
            if r["verify"]:
                vo = verify(cfg, W, st, cache_k, cache_v, d.xhat, mode, temperature)
                a = accept(st, d, vo, seed, step_idx, seq, mode, temperature)
                st.block = a.block
                if caching == "causal":
                    kv_append(st, cache_k, cache_v, vo, a.n_accept)
                log.append(("verify", a.n_accept, a.n_commit))
            else:
                log.append(("threshold", 0, commit_threshold(st, d)))
            step_idx += 1
            if not (np.asarray(st.block) == cfg.mask_id).any():
                break
        out.extend(int(x) for x in st.block)
        if caching == "block":
            block_complete(cfg, W, st, cache_k, cache_v)
        elif len(st.carry) + (B - st.n_cached_in_block()) > (B if carry_cap is None else carry_cap):
            block_complete(cfg, W, st, cache_k, cache_v, causal=True)
        block_advance(st, cfg.mask_id)
    return out, log


def prefill(cfg, W, ids: np.ndarray, chunk: int = 256):
    """Prefix cache by a plain causal forward over the prompt (not on the hot path)."""
    ck = [np.zeros((0, cfg.n_kv_heads, cfg.head_dim)) for _ in range(cfg.n_layers)]
    cv = [np.zeros((0, cfg.n_kv_heads, cfg.head_dim)) for _ in range(cfg.n_layers)]
    for s in range(0, len(ids), chunk):
        t = np.asarray(ids[s:s + chunk])
        fo = forward(cfg, W, t, s + np.arange(len(t)), causal_mask(len(t)), ck, cv, logit_rows=np.zeros(0, dtype=np.int64))
        for l in range(cfg.n_layers):
            ck[l] = np.concatenate([ck[l], fo.k[l]], axis=0)
            cv[l] = np.concatenate([cv[l], fo.v[l]], axis=0)
    return ck, cv

"""ctypes binding of libs2d2.so: argument marshalling only.

The C structs of include/s2d2.h are mirrored one to one; the Python entry points carry the
names of the C calls (s2d2_draft, s2d2_verify, s2d2_accept, s2d2_kv_append, ...).  torch is
used for device memory and streams, never for arithmetic of the method.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field
from typing import Dict, Optional

import torch

HERE = os.path.dirname(os.path.abspath(__file__))

S2D2_OK, S2D2_EINVAL, S2D2_ENOSPC, S2D2_EARCH, S2D2_ELAUNCH = 0, -1, -2, -3, -4
S2D2_F32, S2D2_BF16 = 0, 1
S2D2_GREEDY, S2D2_SAMPLE = 0, 1

EXPORTS = [
    "s2d2_last_error", "s2d2_version", "s2d2_stage_rows", "s2d2_workspace_bytes", "s2d2_packed_bytes", "s2d2_create", "s2d2_destroy",
    "s2d2_set_stream", "s2d2_draft", "s2d2_verify", "s2d2_accept", "s2d2_accept_static", "s2d2_kv_append", "s2d2_block_advance",
    "s2d2_commit_threshold", "s2d2_block_complete", "s2d2_route", "s2d2_moe_choices", "s2d2_debug_buffer", "s2d2_status", "s2d2_vocab_draft_stats", "s2d2_vocab_score", "s2d2_profile_start", "s2d2_profile_stop",
]
PROFILE_CLASSES = ("gemm", "attention", "vocab", "other", "gemm_qkv", "gemm_o", "gemm_gateup", "gemm_down", "gemm_unembed")


class S2D2Error(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"s2d2 error {code}: {msg}")
        self.code = code


class ModelDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn",
                                         "vocab", "n_experts", "top_k", "d_expert", "dtype", "mask_id", "act_planes",
                                         "right_shifted")] + \
               [("rope_theta", C.c_float), ("rms_eps", C.c_float)]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("norm1", "wqkv", "wo", "norm2", "wgu", "wdown", "router", "e_wgu", "e_wdown")]


class Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("unembed", C.c_void_p), ("norm_f", C.c_void_p), ("layers", C.POINTER(LayerWeights))]


class KvView(C.Structure):
    _fields_ = [("k_pages", C.c_void_p), ("v_pages", C.c_void_p), ("page_table", C.c_void_p), ("seq_len", C.c_void_p),
                ("status", C.c_void_p), ("n_pages", C.c_int32), ("page_size", C.c_int32), ("max_pages_per_seq", C.c_int32)]


class BlockStateC(C.Structure):
    _fields_ = [("block_tokens", C.c_void_p), ("block_pos0", C.c_void_p), ("carry_tokens", C.c_void_p)]


class ParamsC(C.Structure):
    _fields_ = [("tau", C.c_float), ("temperature", C.c_float), ("gamma", C.c_float), ("seed", C.c_uint64),
                ("step", C.c_uint32), ("mode", C.c_int32), ("ar_mask", C.c_int32), ("resample", C.c_int32),
                ("step_dev", C.c_void_p), ("active", C.c_void_p)]


class RouteParamsC(C.Structure):
    _fields_ = [("policy", C.c_int32), ("estimator", C.c_int32), ("dynamic", C.c_int32), ("tau_span", C.c_int32),
                ("tau_score", C.c_float), ("tau_on", C.c_float), ("tau_off", C.c_float), ("c", C.c_float),
                ("beta", C.c_float), ("tau_margin", C.c_float)]


class RouteOutC(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("do_verify", "khat", "score", "unmask_fallback")]


class DraftOutC(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("logits", "logit_row_of", "xhat", "p", "lse", "margin", "entropy_n", "unmask",
                                          "n_hi", "span_start", "span_len")]


class VerifyOutC(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("logits_ver", "logit_row_of", "q", "lse_ver", "k_stage", "v_stage",
                                          "stage_row0", "stage_lead")]


class AcceptOutC(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("n_accept", "n_commit", "resampled", "u_used")]


class ProfileC(C.Structure):
    _fields_ = [("launches", C.c_int64), ("ms", C.c_double), ("bytes", C.c_double), ("flops", C.c_double), ("max_ms", C.c_double)]


def lib_path() -> str:
    return os.path.join(HERE, "libs2d2.so")


_LIB = None


def load_library():
    """Loads libs2d2.so; raises if it has not been built (there is no fallback path)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is missing: build it with `python -m paper_2603_25702_amd.build`")
    lib = C.CDLL(path)
    lib.s2d2_last_error.restype = C.c_char_p
    lib.s2d2_version.restype = C.c_char_p
    lib.s2d2_stage_rows.restype = C.c_int64
    lib.s2d2_stage_rows.argtypes = [C.c_int32, C.c_int32]
    lib.s2d2_workspace_bytes.restype = C.c_int64
    lib.s2d2_workspace_bytes.argtypes = [C.POINTER(ModelDesc), C.c_int32, C.c_int32]
    lib.s2d2_create.restype = C.c_int32
    lib.s2d2_packed_bytes.restype = C.c_int64
    lib.s2d2_packed_bytes.argtypes = [C.POINTER(ModelDesc)]
    lib.s2d2_create.argtypes = [C.POINTER(ModelDesc), C.POINTER(Weights), C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                C.c_size_t, C.c_void_p, C.c_size_t, C.POINTER(C.c_void_p)]
    lib.s2d2_destroy.argtypes = [C.c_void_p]
    lib.s2d2_set_stream.argtypes = [C.c_void_p, C.c_void_p]
    lib.s2d2_draft.argtypes = [C.c_void_p, C.POINTER(KvView), C.POINTER(BlockStateC), C.c_int32, C.c_int32,
                               C.POINTER(ParamsC), C.POINTER(DraftOutC)]
    lib.s2d2_verify.argtypes = [C.c_void_p, C.POINTER(KvView), C.POINTER(BlockStateC), C.c_int32, C.c_int32,
                                C.POINTER(ParamsC), C.POINTER(DraftOutC), C.POINTER(VerifyOutC)]
    lib.s2d2_accept.argtypes = [C.c_void_p, C.POINTER(BlockStateC), C.c_int32, C.c_int32, C.POINTER(ParamsC),
                                C.POINTER(DraftOutC), C.POINTER(VerifyOutC), C.POINTER(AcceptOutC)]
    lib.s2d2_accept_static.argtypes = [C.c_void_p, C.c_int32, C.POINTER(BlockStateC), C.c_int32, C.c_int32, C.POINTER(ParamsC),
                                       C.POINTER(DraftOutC), C.POINTER(VerifyOutC), C.POINTER(AcceptOutC)]
    lib.s2d2_accept_static.restype = C.c_int32
    lib.s2d2_kv_append.argtypes = [C.c_void_p, C.POINTER(KvView), C.c_int32, C.c_int32, C.POINTER(DraftOutC),
                                   C.POINTER(VerifyOutC), C.c_void_p]
    lib.s2d2_block_advance.argtypes = [C.c_void_p, C.POINTER(KvView), C.POINTER(BlockStateC), C.c_int32, C.c_int32,
                                       C.c_void_p]
    lib.s2d2_commit_threshold.argtypes = [C.c_void_p, C.POINTER(BlockStateC), C.c_int32, C.c_int32, C.POINTER(DraftOutC)]
    lib.s2d2_block_complete.argtypes = [C.c_void_p, C.POINTER(KvView), C.POINTER(BlockStateC), C.c_int32, C.c_int32,
                                        C.POINTER(VerifyOutC), C.c_int32]
    lib.s2d2_route.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(RouteParamsC), C.POINTER(DraftOutC), C.c_void_p,
                               C.POINTER(RouteOutC)]
    lib.s2d2_status.argtypes = [C.c_void_p]
    lib.s2d2_status.restype = C.c_int32
    lib.s2d2_debug_buffer.argtypes = [C.c_void_p, C.c_char_p, C.POINTER(C.c_void_p)]
    lib.s2d2_debug_buffer.restype = C.c_int32
    lib.s2d2_moe_choices.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
    lib.s2d2_moe_choices.restype = C.c_int32
    lib.s2d2_vocab_draft_stats.argtypes = [C.c_void_p, C.c_void_p, C.c_int32] + [C.c_void_p] * 5
    lib.s2d2_vocab_score.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.s2d2_profile_start.argtypes = [C.c_void_p, C.c_int32]
    lib.s2d2_profile_stop.argtypes = [C.c_void_p, C.POINTER(ProfileC)]
    for name in ("s2d2_profile_start", "s2d2_profile_stop", "s2d2_destroy", "s2d2_set_stream", "s2d2_draft", "s2d2_verify", "s2d2_accept", "s2d2_kv_append",
                 "s2d2_block_advance", "s2d2_commit_threshold", "s2d2_block_complete", "s2d2_route", "s2d2_moe_choices", "s2d2_debug_buffer", "s2d2_status", "s2d2_vocab_draft_stats", "s2d2_vocab_score"):
        getattr(lib, name).restype = C.c_int32
    _LIB = lib
    return lib


def _check(lib, rc: int):
    if rc != 0:
        raise S2D2Error(rc, lib.s2d2_last_error().decode())


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def model_desc(cfg, act_planes: int = 0) -> ModelDesc:
    return ModelDesc(cfg.n_layers, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ffn, cfg.vocab,
                     cfg.n_experts, cfg.top_k, cfg.d_expert, S2D2_BF16 if cfg.dtype == "bf16" else S2D2_F32,
                     cfg.mask_id, act_planes, int(bool(getattr(cfg, "right_shifted", False))), cfg.rope_theta, cfg.rms_eps)


@dataclass
class Params:
    tau: float = 0.9
    temperature: float = 1.0
    gamma: float = 1.0
    seed: int = 0
    step: int = 0
    mode: int = S2D2_GREEDY
    ar_mask: int = 1
    resample: int = 1
    step_dev: Optional[torch.Tensor] = None  # uint32 counter on the device (as int32 storage)
    active: Optional[torch.Tensor] = None    # int32 [N] on the device: 0 = skipped by verify / accept

    def c(self) -> ParamsC:
        return ParamsC(self.tau, self.temperature, self.gamma, self.seed, self.step, self.mode, self.ar_mask,
                       self.resample, _ptr(self.step_dev), _ptr(self.active))


S2D2_ROUTE_MIN_SPAN, S2D2_ROUTE_SCORE, S2D2_ROUTE_HYSTERESIS = 0, 1, 2
S2D2_EST_MARGIN, S2D2_EST_ENTROPY = 0, 1


@dataclass
class RouteParams:
    policy: int = S2D2_ROUTE_MIN_SPAN
    estimator: int = S2D2_EST_ENTROPY
    dynamic: int = 1
    tau_span: int = 1
    tau_score: float = 0.0
    tau_on: float = 1.0
    tau_off: float = -5.0
    c: float = 1.0
    beta: float = 1.0
    tau_margin: float = 0.5

    def c_struct(self) -> RouteParamsC:
        return RouteParamsC(self.policy, self.estimator, int(self.dynamic), self.tau_span, self.tau_score, self.tau_on,
                            self.tau_off, self.c, self.beta, self.tau_margin)


@dataclass
class RouteOut:
    t: Dict[str, torch.Tensor]

    @staticmethod
    def alloc(N: int, device) -> "RouteOut":
        return RouteOut(_alloc([("do_verify", (N,), torch.int32), ("khat", (N,), torch.float32),
                                ("score", (N,), torch.float32), ("unmask_fallback", (N,), torch.int64)], device))

    def c(self) -> RouteOutC:
        return RouteOutC(*[self.t[n].data_ptr() for n, _ in RouteOutC._fields_])

    def __getattr__(self, k):
        try:
            return self.__dict__["t"][k]
        except KeyError:
            raise AttributeError(k)


@dataclass
class KvCache:
    """Paged cache tensors: k [n_layers, n_pages, Hkv, page_size, D], v [n_layers, n_pages, Hkv, D, page_size];
    page_table [N, max_pages]; seq_len [N]."""
    k: torch.Tensor
    v: torch.Tensor
    page_table: torch.Tensor
    seq_len: torch.Tensor
    status: torch.Tensor

    def c(self) -> KvView:
        return KvView(self.k.data_ptr(), self.v.data_ptr(), self.page_table.data_ptr(), self.seq_len.data_ptr(),
                      self.status.data_ptr(), self.k.shape[1], self.k.shape[3], self.page_table.shape[1])


@dataclass
class BlockState:
    block_tokens: torch.Tensor   # int32 [N, B]
    block_pos0: torch.Tensor     # int32 [N]
    carry_tokens: torch.Tensor   # int32 [N, B]

    def c(self) -> BlockStateC:
        return BlockStateC(self.block_tokens.data_ptr(), self.block_pos0.data_ptr(), self.carry_tokens.data_ptr())


def _alloc(names_shapes_dtypes, device):
    return {n: torch.empty(s, dtype=d, device=device) for n, s, d in names_shapes_dtypes}


@dataclass
class DraftOut:
    t: Dict[str, torch.Tensor]

    @staticmethod
    def alloc(N: int, B: int, V: int, device) -> "DraftOut":
        i32, f32 = torch.int32, torch.float32
        return DraftOut(_alloc([("logits", (N * B, V), f32), ("logit_row_of", (N, B), i32), ("xhat", (N, B), i32),
                                ("p", (N, B), f32), ("lse", (N, B), f32), ("margin", (N, B), f32),
                                ("entropy_n", (N, B), f32), ("unmask", (N,), torch.int64), ("n_hi", (N,), i32),
                                ("span_start", (N,), i32), ("span_len", (N,), i32)], device))

    def c(self) -> DraftOutC:
        return DraftOutC(*[self.t[n].data_ptr() for n, _ in DraftOutC._fields_])

    def __getattr__(self, k):
        try:
            return self.__dict__["t"][k]
        except KeyError:
            raise AttributeError(k)


@dataclass
class VerifyOut:
    t: Dict[str, torch.Tensor]

    @staticmethod
    def alloc(N: int, B: int, V: int, n_layers: int, stage_rows: int, Hkv: int, D: int, dtype, device) -> "VerifyOut":
        i32, f32 = torch.int32, torch.float32
        return VerifyOut(_alloc([("logits_ver", (N * B, V), f32), ("logit_row_of", (N, B), i32), ("q", (N, B), f32),
                                 ("lse_ver", (N, B), f32), ("k_stage", (n_layers, stage_rows, Hkv, D), dtype),
                                 ("v_stage", (n_layers, stage_rows, Hkv, D), dtype), ("stage_row0", (N,), i32),
                                 ("stage_lead", (N,), i32)], device))

    def c(self) -> VerifyOutC:
        return VerifyOutC(*[self.t[n].data_ptr() for n, _ in VerifyOutC._fields_])

    def __getattr__(self, k):
        try:
            return self.__dict__["t"][k]
        except KeyError:
            raise AttributeError(k)


@dataclass
class AcceptOut:
    t: Dict[str, torch.Tensor]

    @staticmethod
    def alloc(N: int, B: int, device) -> "AcceptOut":
        i32 = torch.int32
        return AcceptOut(_alloc([("n_accept", (N,), i32), ("n_commit", (N,), i32), ("resampled", (N,), i32),
                                 ("u_used", (N, B), torch.float32)], device))

    def c(self) -> AcceptOutC:
        return AcceptOutC(*[self.t[n].data_ptr() for n, _ in AcceptOutC._fields_])

    def __getattr__(self, k):
        try:
            return self.__dict__["t"][k]
        except KeyError:
            raise AttributeError(k)


def s2d2_accept_static(stream: Optional[torch.cuda.Stream], vocab: int, st: BlockState, N: int, B: int, prm: Params,
                       draft: DraftOut, ver: VerifyOut, out: AcceptOut):
    """The accept step without a context or a workspace (scratch inside the library; N <= 128, vocab <= 2^18)."""
    lib = load_library()
    s = stream if stream is not None else torch.cuda.current_stream(draft.logits.device)
    _check(lib, lib.s2d2_accept_static(C.c_void_p(s.cuda_stream), vocab, C.byref(st.c()), N, B, C.byref(prm.c()),
                                       C.byref(draft.c()), C.byref(ver.c()), C.byref(out.c())))


class Engine:
    """Owns a library context: weights on the device, workspace, stream.  Methods = C calls."""

    def __init__(self, cfg, weights: Dict[str, torch.Tensor], max_batch: int, max_block: int,
                 device: str = "cuda:0", stream: Optional[torch.cuda.Stream] = None, packed: bool = True,
                 act_planes: int = 0):
        self.lib = load_library()
        self.cfg, self.max_batch, self.max_block = cfg, max_batch, max_block
        self.device = torch.device(device)
        self.desc = model_desc(cfg, act_planes)
        self.w = {k: v.to(self.device).contiguous() for k, v in weights.items() if not k.startswith("__")}
        layers = (LayerWeights * cfg.n_layers)()
        for l in range(cfg.n_layers):
            g = lambda n: _ptr(self.w.get(f"l{l}.{n}"))
            layers[l] = LayerWeights(g("norm1"), g("wqkv"), g("wo"), g("norm2"), g("wgu"), g("wdown"), g("router"),
                                     g("e_wgu"), g("e_wdown"))
        self._layers = layers
        self._weights = Weights(self.w["embed"].data_ptr(), self.w["unembed"].data_ptr(), self.w["norm_f"].data_ptr(), layers)
        need = self.lib.s2d2_workspace_bytes(C.byref(self.desc), max_batch, max_block)
        if need < 0:
            raise S2D2Error(int(need), self.lib.s2d2_last_error().decode())
        self.workspace = torch.empty(int(need), dtype=torch.uint8, device=self.device)
        self.stream = stream
        pbytes = int(self.lib.s2d2_packed_bytes(C.byref(self.desc))) if packed else 0
        self.packed = torch.empty(pbytes, dtype=torch.uint8, device=self.device) if pbytes > 0 else None
        ctx = C.c_void_p()
        _check(self.lib, self.lib.s2d2_create(C.byref(self.desc), C.byref(self._weights), max_batch, max_block,
                                              self._stream_handle(), self.workspace.data_ptr(), int(need),
                                              _ptr(self.packed), pbytes, C.byref(ctx)))
        self.ctx = ctx
        self.stage_rows = int(self.lib.s2d2_stage_rows(max_batch, max_block))

    def _stream_handle(self):
        s = self.stream if self.stream is not None else torch.cuda.current_stream(self.device)
        return C.c_void_p(s.cuda_stream)

    def set_stream(self, stream: torch.cuda.Stream):
        self.stream = stream
        _check(self.lib, self.lib.s2d2_set_stream(self.ctx, C.c_void_p(stream.cuda_stream)))

    def close(self):
        if getattr(self, "ctx", None):
            self.lib.s2d2_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- buffers -------------------------------------------------------------------------
    def alloc_draft_out(self, N, B) -> DraftOut:
        return DraftOut.alloc(N, B, self.cfg.vocab, self.device)

    def alloc_verify_out(self, N, B) -> VerifyOut:
        return VerifyOut.alloc(N, B, self.cfg.vocab, self.cfg.n_layers, self.stage_rows, self.cfg.n_kv_heads,
                               self.cfg.head_dim, self.cfg.torch_dtype, self.device)

    def alloc_accept_out(self, N, B) -> AcceptOut:
        return AcceptOut.alloc(N, B, self.device)

    # ---- the C calls ----------------------------------------------------------------------
    def s2d2_draft(self, kv: KvCache, st: BlockState, N, B, prm: Params, out: DraftOut):
        _check(self.lib, self.lib.s2d2_draft(self.ctx, C.byref(kv.c()), C.byref(st.c()), N, B, C.byref(prm.c()), C.byref(out.c())))

    def s2d2_verify(self, kv: KvCache, st: BlockState, N, B, prm: Params, draft: DraftOut, out: VerifyOut):
        _check(self.lib, self.lib.s2d2_verify(self.ctx, C.byref(kv.c()), C.byref(st.c()), N, B, C.byref(prm.c()),
                                              C.byref(draft.c()), C.byref(out.c())))

    def s2d2_accept(self, st: BlockState, N, B, prm: Params, draft: DraftOut, ver: VerifyOut, out: AcceptOut):
        _check(self.lib, self.lib.s2d2_accept(self.ctx, C.byref(st.c()), N, B, C.byref(prm.c()), C.byref(draft.c()),
                                              C.byref(ver.c()), C.byref(out.c())))

    def s2d2_kv_append(self, kv: KvCache, N, B, draft: DraftOut, ver: VerifyOut, n_accept: torch.Tensor):
        _check(self.lib, self.lib.s2d2_kv_append(self.ctx, C.byref(kv.c()), N, B, C.byref(draft.c()), C.byref(ver.c()),
                                                 n_accept.data_ptr()))

    def s2d2_block_advance(self, kv: KvCache, st: BlockState, N, B, step_dev: Optional[torch.Tensor] = None):
        _check(self.lib, self.lib.s2d2_block_advance(self.ctx, C.byref(kv.c()), C.byref(st.c()), N, B, _ptr(step_dev)))

    def s2d2_commit_threshold(self, st: BlockState, N, B, draft: DraftOut):
        _check(self.lib, self.lib.s2d2_commit_threshold(self.ctx, C.byref(st.c()), N, B, C.byref(draft.c())))

    def s2d2_block_complete(self, kv: KvCache, st: BlockState, N, B, scratch: VerifyOut, causal: int = 0):
        _check(self.lib, self.lib.s2d2_block_complete(self.ctx, C.byref(kv.c()), C.byref(st.c()), N, B, C.byref(scratch.c()),
                                                      int(causal)))

    def s2d2_route(self, N, B, rp: RouteParams, draft: DraftOut, hysteresis: Optional[torch.Tensor], out: RouteOut):
        _check(self.lib, self.lib.s2d2_route(self.ctx, N, B, C.byref(rp.c_struct()), C.byref(draft.c()), _ptr(hysteresis),
                                             C.byref(out.c())))

    def s2d2_status(self):
        _check(self.lib, self.lib.s2d2_status(self.ctx))

    def s2d2_debug_buffer(self, name: str) -> int:
        p = C.c_void_p()
        _check(self.lib, self.lib.s2d2_debug_buffer(self.ctx, name.encode(), C.byref(p)))
        return int(p.value)

    def s2d2_moe_choices(self, rows: int) -> torch.Tensor:
        """[n_layers, rows, top_k] experts chosen in the most recent forward (device int32)."""
        out = torch.empty((self.cfg.n_layers, rows, self.cfg.top_k), dtype=torch.int32, device=self.device)
        _check(self.lib, self.lib.s2d2_moe_choices(self.ctx, rows, out.data_ptr()))
        return out

    def s2d2_profile_start(self, max_launches: int):
        _check(self.lib, self.lib.s2d2_profile_start(self.ctx, max_launches))

    def s2d2_profile_stop(self):
        out = (ProfileC * len(PROFILE_CLASSES))()
        _check(self.lib, self.lib.s2d2_profile_stop(self.ctx, out))
        return {n: dict(launches=int(out[i].launches), ms=float(out[i].ms), bytes=float(out[i].bytes), flops=float(out[i].flops),
                        max_ms=float(out[i].max_ms))
                for i, n in enumerate(PROFILE_CLASSES)}

    def s2d2_vocab_draft_stats(self, logits: torch.Tensor):
        rows = logits.shape[0]
        dev = logits.device
        o = dict(xhat=torch.empty(rows, dtype=torch.int32, device=dev))
        for n in ("p", "lse", "margin", "entropy_n"):
            o[n] = torch.empty(rows, dtype=torch.float32, device=dev)
        _check(self.lib, self.lib.s2d2_vocab_draft_stats(self.ctx, logits.data_ptr(), rows, o["xhat"].data_ptr(),
                                                         o["p"].data_ptr(), o["lse"].data_ptr(), o["margin"].data_ptr(),
                                                         o["entropy_n"].data_ptr()))
        return o

    def s2d2_vocab_score(self, logits_ver: torch.Tensor, token: torch.Tensor):
        rows = logits_ver.shape[0]
        q = torch.empty(rows, dtype=torch.float32, device=logits_ver.device)
        lse = torch.empty_like(q)
        _check(self.lib, self.lib.s2d2_vocab_score(self.ctx, logits_ver.data_ptr(), rows, token.data_ptr(), q.data_ptr(),
                                                   lse.data_ptr()))
        return q, lse

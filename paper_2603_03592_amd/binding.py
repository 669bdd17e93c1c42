from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch  # noqa: F401  -- first: the library must bind to the HIP runtime torch has loaded (one runtime per process)

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libstageverify.so")

SV_OK, SV_EINVAL, SV_EUNSUPPORTED, SV_ENOMEM, SV_EHIP = range(5)
SV_F32, SV_BF16 = 0, 1
SV_MLP_GELU, SV_MLP_SWIGLU = 0, 1
SV_NORM_LN, SV_NORM_RMS = 0, 1
SV_REDUCE_GLOBAL, SV_REDUCE_MAX_TOKEN = 0, 1
SV_FLAG_BACKWARD, SV_FLAG_PLAIN_KERNELS, SV_FLAG_SLICED_W, SV_FLAG_FUSE_NORM = 1, 2, 4, 8
SV_M_SW = 16
METRIC_NAMES = ("rel_l2", "l1", "zl2", "sfr")
METRIC_BITS = {n: 1 << i for i, n in enumerate(METRIC_NAMES)}
_STATUS = {1: "SV_EINVAL", 2: "SV_EUNSUPPORTED", 3: "SV_ENOMEM", 4: "SV_EHIP"}


class SVError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"{_STATUS.get(status, status)}: {msg}")
        self.status = status


class StageDescC(C.Structure):
    _fields_ = [("n_blocks", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("ffn_hidden", C.c_int32), ("mlp", C.c_int32), ("norm", C.c_int32), ("rope", C.c_int32),
                ("causal", C.c_int32), ("norm_eps", C.c_float), ("rope_theta", C.c_float), ("dtype", C.c_int32),
                ("n_experts", C.c_int32), ("top_k", C.c_int32), ("ffn_shared", C.c_int32), ("router_score", C.c_int32),
                ("router_norm", C.c_int32)]


_WNAMES = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "norm1_g", "norm1_b", "norm2_g", "norm2_b",
           "w_router", "ws_gate", "ws_up", "ws_down")


class BlockWeightsC(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _WNAMES]


OP_NAMES = ("norm", "gemm_qkv", "rope", "attn", "gemm_o", "gemm_gateup", "gemm_down", "score", "bwd_gemm_da",
            "bwd_gemm_dn2", "bwd_norm", "bwd_gemm_do", "bwd_attn", "bwd_rope", "bwd_gemm_dn1", "bwd_wtranspose",
            "sw_project", "sw_sort", "moe_route", "moe_permute", "bwd_moe", "norm_pieces")


class PolicyCfgC(C.Structure):
    _fields_ = [("c", C.c_int32), ("t_forgive", C.c_int32), ("window", C.c_int32), ("n_max", C.c_int32),
                ("k0", C.c_double), ("alpha", C.c_double), ("grow", C.c_double), ("shrink", C.c_double),
                ("min_dist_mult", C.c_double), ("eps", C.c_double), ("severe", C.c_double)]


class SentinelCfgC(C.Structure):
    _fields_ = [("n_stages", C.c_int32), ("n_workers", C.c_int32), ("T", C.c_int64), ("D", C.c_int32), ("metric_mask", C.c_uint32),
                ("n_dirs", C.c_int32), ("directions", C.c_void_p), ("beta_h", C.c_float), ("beta_g", C.c_float),
                ("policy_h", PolicyCfgC), ("policy_g", PolicyCfgC)]


class ProfileC(C.Structure):
    _fields_ = [("ms", C.c_double * len(OP_NAMES)), ("flop", C.c_double * len(OP_NAMES)),
                ("launches", C.c_int64 * len(OP_NAMES))]


RESULT_DTYPE = np.dtype([("score", np.float32, (4,)), ("flag", np.uint32), ("metric_mask", np.uint32),
                         ("max_token_rell2", np.float32), ("argmax_token", np.int32)])
assert RESULT_DTYPE.itemsize == 32


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2603_03592_amd.build` "
                          "(there is no CPU fallback)")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, u32, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_float
    L.sv_check_desc.restype = C.c_int
    L.sv_check_desc.argtypes = [C.POINTER(StageDescC), u32, C.c_char_p, i32]
    L.sv_workspace_bytes.restype = i64
    L.sv_workspace_bytes.argtypes = [C.POINTER(StageDescC), i64, i32, u32]
    L.sv_create.restype = C.c_int
    L.sv_create.argtypes = [C.POINTER(StageDescC), i64, i32, u32, C.POINTER(vp)]
    L.sv_destroy.restype = None
    L.sv_destroy.argtypes = [vp]
    L.sv_last_error.restype = C.c_char_p
    L.sv_last_error.argtypes = [vp]
    L.sv_last_routing.restype = C.c_int
    L.sv_last_routing.argtypes = [vp, i32, vp, vp, vp]
    L.sv_verify_forward.restype = C.c_int
    L.sv_verify_forward.argtypes = [vp, C.POINTER(BlockWeightsC), vp, i32, i32, vp, u32, C.POINTER(f32), i32, vp, vp, vp, vp]
    L.sv_verify_backward.restype = C.c_int
    L.sv_verify_backward.argtypes = [vp, C.POINTER(BlockWeightsC), vp, vp, i32, i32, vp, u32, C.POINTER(f32), i32, vp, vp, vp, vp, vp]
    L.sv_profile_select.restype = C.c_int
    L.sv_profile_select.argtypes = [vp, C.c_uint64]
    L.sv_score_and_flag.restype = C.c_int
    L.sv_score_and_flag.argtypes = [vp, vp, i64, i32, vp, i64, i32, i32, i64, i32, u32, C.POINTER(f32), i32, vp, vp, vp]
    L.sv_score_and_flag_noalloc.restype = C.c_int
    L.sv_score_and_flag_noalloc.argtypes = [vp, i64, i32, vp, i64, i32, i32, i64, i32, u32, C.POINTER(f32), i32, vp, vp, vp]
    L.sv_score_and_sum.restype = C.c_int
    L.sv_score_and_sum.argtypes = [vp, vp, i64, i32, vp, i32, i32, i64, i32, u32, C.POINTER(f32), i32, vp, vp, C.c_char_p, vp, vp]
    L.sv_ema_from_sum.restype = C.c_int
    L.sv_ema_from_sum.argtypes = [vp, vp, vp, i32, i64, i32, f32, vp]
    L.sv_sw_row_len.restype = i64
    L.sv_sw_row_len.argtypes = [i64]
    L.sv_sw_against_projection.restype = C.c_int
    L.sv_sw_against_projection.argtypes = [vp, vp, i64, i32, i32, i64, i32, vp, i32, vp, vp, f32, vp, vp, vp]
    L.sv_sw_projection_ema.restype = C.c_int
    L.sv_sw_projection_ema.argtypes = [vp, vp, vp, i32, C.c_char_p, i64, i32, f32, vp]
    L.sv_ema_update.restype = C.c_int
    L.sv_ema_update.argtypes = [vp, vp, vp, i64, i32, i32, vp, i64, i32, f32, vp]
    L.sv_profile_enable.restype = C.c_int
    L.sv_profile_enable.argtypes = [vp, i32]
    L.sv_profile_read.restype = C.c_int
    L.sv_profile_read.argtypes = [vp, C.POINTER(ProfileC)]
    L.sv_sliced_wasserstein.restype = C.c_int
    L.sv_sliced_wasserstein.argtypes = [vp, vp, i64, i32, vp, i64, i32, i32, i64, i32, vp, i32, f32, vp, vp, vp]
    dp, u8p = C.POINTER(C.c_double), C.POINTER(C.c_uint8)
    L.sv_adaptive_iqr.restype = C.c_int
    L.sv_adaptive_iqr.argtypes = [dp, i32, C.c_double, C.POINTER(PolicyCfgC), dp, dp, dp]
    L.sv_policy_create.restype = C.c_int
    L.sv_policy_create.argtypes = [i32, i32, C.POINTER(PolicyCfgC), C.POINTER(vp)]
    L.sv_policy_destroy.restype = None
    L.sv_policy_destroy.argtypes = [vp]
    L.sv_policy_warmup.restype = C.c_int
    L.sv_policy_warmup.argtypes = [vp, dp]
    L.sv_policy_step.restype = C.c_int
    L.sv_policy_step.argtypes = [vp, dp, u8p, u8p, u8p]
    L.sv_policy_state.restype = C.c_int
    L.sv_policy_state.argtypes = [vp, C.POINTER(i32), u8p, dp, dp, dp, C.POINTER(i32)]
    L.sv_replace_with_ema.restype = C.c_int
    L.sv_replace_with_ema.argtypes = [vp, vp, i64, i32, i32, vp, vp, i64, i32, vp]
    L.sv_sentinel_create.restype = C.c_int
    L.sv_sentinel_create.argtypes = [vp, C.POINTER(SentinelCfgC), C.POINTER(vp)]
    L.sv_sentinel_destroy.restype = None
    L.sv_sentinel_destroy.argtypes = [vp]
    L.sv_sentinel_last_error.restype = C.c_char_p
    L.sv_sentinel_last_error.argtypes = [vp]
    L.sv_sentinel_begin_iteration.restype = C.c_int
    L.sv_sentinel_begin_iteration.argtypes = [vp, i32]
    L.sv_sentinel_forward.restype = C.c_int
    L.sv_sentinel_forward.argtypes = [vp, i32, vp, i32, u8p, dp, vp]
    L.sv_sentinel_backward.restype = C.c_int
    L.sv_sentinel_backward.argtypes = [vp, i32, vp, i32, u8p, dp, vp]
    L.sv_sentinel_state.restype = C.c_int
    L.sv_sentinel_state.argtypes = [vp, i32, i32, C.POINTER(vp), C.POINTER(i32), u8p, dp, dp, dp]
    L.sv_sentinel_counters.restype = C.c_int
    L.sv_sentinel_counters.argtypes = [vp, C.POINTER(C.c_int64)]
    L.sv_sentinel_read_ema.restype = C.c_int
    L.sv_sentinel_read_ema.argtypes = [vp, i32, i32, C.POINTER(f32), vp]
    L.sv_prepare_weights.restype = C.c_int
    L.sv_prepare_weights.argtypes = [vp, C.POINTER(BlockWeightsC), vp]
    L.sv_gemm_bf16.restype = C.c_int
    L.sv_gemm_bf16.argtypes = [vp, i64, vp, i64, i32, vp, i64, i32, i32, i32, i32, vp]
    return L


lib = _load()


def sv_gemm_bf16(a, b, b_is_kn: bool = False, tile: int = 0, out=None):
    """C = a @ b.T (b stored [N,K]) or a @ b (b stored [K,N]) on the MFMA GEMM kernels; bf16 device tensors."""
    import torch
    M, K = a.shape
    N = b.shape[1] if b_is_kn else b.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=torch.bfloat16, device=a.device)
    st = lib.sv_gemm_bf16(a.data_ptr(), a.stride(0), b.data_ptr(), b.stride(0), int(b_is_kn), out.data_ptr(), out.stride(0),
                          M, N, K, tile, torch.cuda.current_stream().cuda_stream)
    if st != SV_OK:
        raise SVError(st, "sv_gemm_bf16")
    return out


def _policy_cfg(c=5, t_forgive=100, window=100, k0=1.5, alpha=0.01, grow=1.1, shrink=0.9, n_max=10, min_dist_mult=0.0,
                eps=1e-3, severe=100.0) -> PolicyCfgC:
    return PolicyCfgC(int(c), int(t_forgive), int(window), int(n_max), float(k0), float(alpha), float(grow), float(shrink),
                      float(min_dist_mult), float(eps), float(severe))


def _dbl(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(C.POINTER(C.c_double))


def adaptive_iqr(history, k_prev, alpha, grow, shrink, n_max, min_dist_mult, eps):
    """One run of the adaptive-multiplier algorithm on a host array; returns (lower, upper, k)."""
    h, hp = _dbl(history)
    cfg = _policy_cfg(alpha=alpha, grow=grow, shrink=shrink, n_max=n_max, min_dist_mult=min_dist_mult, eps=eps)
    lo, up, k = C.c_double(), C.c_double(), C.c_double()
    st = lib.sv_adaptive_iqr(hp, h.size, float(k_prev), C.byref(cfg), C.byref(lo), C.byref(up), C.byref(k))
    if st != SV_OK:
        raise SVError(st, "sv_adaptive_iqr")
    return lo.value, up.value, k.value


class Policy:
    """One sv_policy: violation counters, bans, histories and fences of one stage and one signal kind (host side)."""

    def __init__(self, n_workers: int, n_metrics: int, **cfg):
        self.d, self.m = n_workers, n_metrics
        self._p = C.c_void_p()
        c = _policy_cfg(**cfg)
        st = lib.sv_policy_create(n_workers, n_metrics, C.byref(c), C.byref(self._p))
        if st != SV_OK:
            raise SVError(st, "sv_policy_create")

    def close(self):
        if self._p:
            lib.sv_policy_destroy(self._p)
            self._p = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _gamma(self, gamma):
        g, gp = _dbl(gamma)
        assert g.shape == (self.d, self.m)
        return g, gp

    def warmup(self, gamma):
        g, gp = self._gamma(gamma)
        st = lib.sv_policy_warmup(self._p, gp)
        if st != SV_OK:
            raise SVError(st, "sv_policy_warmup")

    def step(self, gamma, skip=None, pre_tainted=None):
        """Returns the list of workers tainted at this stage in this iteration."""
        g, gp = self._gamma(gamma)
        out = np.zeros(self.d, dtype=np.uint8)
        u8p = C.POINTER(C.c_uint8)
        masks = [None if a is None else np.ascontiguousarray(a, dtype=np.uint8) for a in (skip, pre_tainted)]
        sk, pt = (None if a is None else a.ctypes.data_as(u8p) for a in masks)
        st = lib.sv_policy_step(self._p, gp, sk, pt, out.ctypes.data_as(u8p))
        if st != SV_OK:
            raise SVError(st, "sv_policy_step")
        return [int(r) for r in np.nonzero(out)[0]]

    def state(self):
        v = np.zeros(self.d, dtype=np.int32)
        b = np.zeros(self.d, dtype=np.uint8)
        lo, up, k = (np.zeros(self.m, dtype=np.float64) for _ in range(3))
        n = np.zeros(self.m, dtype=np.int32)
        dp, u8p, ip = C.POINTER(C.c_double), C.POINTER(C.c_uint8), C.POINTER(C.c_int32)
        st = lib.sv_policy_state(self._p, v.ctypes.data_as(ip), b.ctypes.data_as(u8p), lo.ctypes.data_as(dp), up.ctypes.data_as(dp),
                                 k.ctypes.data_as(dp), n.ctypes.data_as(ip))
        if st != SV_OK:
            raise SVError(st, "sv_policy_state")
        return dict(violations=v, banned=b.astype(bool), lower=lo, upper=up, k=k, history_len=n)


def _desc_c(desc) -> StageDescC:
    return StageDescC(int(desc.n_blocks), int(desc.d_model), int(desc.n_heads), int(desc.n_kv_heads), int(desc.ffn_hidden),
                      SV_MLP_SWIGLU if desc.mlp == "swiglu" else SV_MLP_GELU,
                      SV_NORM_RMS if desc.norm == "rms" else SV_NORM_LN, int(bool(desc.rope)), int(bool(desc.causal)),
                      float(desc.norm_eps), float(desc.rope_theta), SV_BF16 if desc.dtype == "bf16" else SV_F32,
                      int(getattr(desc, "n_experts", 0)), int(getattr(desc, "top_k", 0)),
                      int(getattr(desc, "n_shared", 0)) * int(desc.ffn_hidden) if getattr(desc, "n_experts", 0) else 0,
                      1 if getattr(desc, "router_score", "sigmoid") == "softmax" and getattr(desc, "n_experts", 0) else 0,
                      int(bool(getattr(desc, "router_norm", False))) if getattr(desc, "n_experts", 0) else 0)


def sv_check_desc(desc, flags: int = 0):
    buf = C.create_string_buffer(256)
    d = _desc_c(desc)
    st = lib.sv_check_desc(C.byref(d), flags, buf, 256)
    return st, buf.value.decode()


def sv_workspace_bytes(desc, max_tokens: int, max_seq: int, flags: int = 0) -> int:
    d = _desc_c(desc)
    return int(lib.sv_workspace_bytes(C.byref(d), max_tokens, max_seq, flags))


def _tau_array(tau) -> "C.Array":
    if isinstance(tau, dict):
        vals = [float(tau.get(n, 0.0)) for n in METRIC_NAMES]
    else:
        vals = [float(t) for t in tau]
    return (C.c_float * 4)(*vals)


def _mask(metrics) -> int:
    if isinstance(metrics, int):
        return metrics
    m = 0
    for n in metrics:
        m |= METRIC_BITS[n]
    return m


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _dt(t) -> int:
    import torch
    if t.dtype == torch.bfloat16:
        return SV_BF16
    if t.dtype == torch.float32:
        return SV_F32
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def score_and_flag_noalloc(claims, ref, results, metrics=("rel_l2",), tau=(0, 0, 0, 0), reduce="max_token", token_scores=None):
    """sv_score_and_flag_noalloc: the statistic without a context and without any allocation, here or in the library.
    claims [n, T, D]; ref [T, D] shared or [n, T, D]; results: caller's uint8 [n, 32] device tensor (one sv_result per
    submission); token_scores: caller's float32 [n, T] device tensor or None.  Enqueued on the current stream."""
    import torch
    n, D = claims.shape[0], claims.shape[-1]
    T = claims[0].numel() // D
    shared = ref.numel() == T * D
    assert claims.is_contiguous() and ref.is_contiguous() and results.is_contiguous()
    assert results.dtype == torch.uint8 and results.numel() == 32 * n
    assert token_scores is None or (token_scores.dtype == torch.float32 and token_scores.numel() == n * T and token_scores.is_contiguous())
    st = lib.sv_score_and_flag_noalloc(_ptr(claims), T * D, n, _ptr(ref), 0 if shared else T * D, _dt(claims), _dt(ref), T, D,
                                       _mask(metrics), _tau_array(tau),
                                       SV_REDUCE_MAX_TOKEN if reduce == "max_token" else SV_REDUCE_GLOBAL,
                                       _ptr(token_scores), _ptr(results), torch.cuda.current_stream().cuda_stream)
    if st != SV_OK:
        raise SVError(st, lib.sv_last_error(None).decode())
    return results


def fuse_norm_pays(desc) -> bool:
    """Whether SV_FLAG_FUSE_NORM made the stage check faster where it was measured (one MI355X): it saves the norm
    passes' HBM traffic and adds work to four epilogues, and the chip runs the products at its power limit either way.
    d_model 2048 (k loops of 32 slices, epilogues a tenth of a product): 0.6-0.9 % faster.  d_model 4096: 1.3 % slower
    (0.11 ms of norm passes saved, 0.2 ms more in the products, a third of it in their code and the rest with the
    unnormalised operand and without the pauses between products).  Dense bf16 stages with RMSNorm only (a mixture of
    experts can fold its first norm; that was not timed)."""
    return desc.dtype == "bf16" and desc.norm == "rms" and desc.n_experts == 0 and desc.d_model <= 2048


class Verifier:
    """One sv_ctx.  Tensors are torch tensors on the context's device, contiguous, in the stage dtype."""

    def __init__(self, desc, max_tokens: int, max_seq: int, backward: bool = False, plain_kernels: bool = False,
                 sliced_w: bool = False, fuse_norm: bool = False):
        import torch
        self.torch = torch
        self.desc = desc
        self.tdtype = torch.bfloat16 if desc.dtype == "bf16" else torch.float32
        self.flags = ((SV_FLAG_BACKWARD if backward else 0) | (SV_FLAG_PLAIN_KERNELS if plain_kernels else 0)
                      | (SV_FLAG_SLICED_W if sliced_w else 0) | (SV_FLAG_FUSE_NORM if fuse_norm else 0))
        self._ctx = C.c_void_p()
        d = _desc_c(desc)
        st = lib.sv_create(C.byref(d), max_tokens, max_seq, self.flags, C.byref(self._ctx))
        if st != SV_OK:
            raise SVError(st, lib.sv_last_error(None).decode())

    def close(self):
        if getattr(self, "_ctx", None) is not None and self._ctx.value:
            lib.sv_destroy(self._ctx)
            self._ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ------------------------------------------------------------------ helpers
    def _check(self, st: int):
        if st != SV_OK:
            raise SVError(st, lib.sv_last_error(self._ctx).decode())

    def _stream(self) -> int:
        return self.torch.cuda.current_stream().cuda_stream

    def pack_weights(self, blocks: Sequence[Dict[str, object]]):
        """Host array of sv_block_weights from per-block dicts of device tensors (kept alive by the caller)."""
        arr = (BlockWeightsC * len(blocks))()
        for i, b in enumerate(blocks):
            for n in _WNAMES:
                t = b.get(n)
                if t is not None:
                    assert t.is_cuda and t.is_contiguous() and t.dtype == self.tdtype, n
                setattr(arr[i], n, _ptr(t))
        return arr

    def last_routing(self, block: int, n_tokens: int):
        """(experts [T, top_k] int32, gates [T, top_k] float32) that the latest verify call used in `block`."""
        torch = self.torch
        k = int(self.desc.top_k)
        ex = torch.empty((n_tokens, k), dtype=torch.int32, device="cuda")
        gt = torch.empty((n_tokens, k), dtype=torch.float32, device="cuda")
        self._check(lib.sv_last_routing(self._ctx, block, _ptr(ex), _ptr(gt), self._stream()))
        return ex, gt

    def prepare_weights(self, weights_c):
        """Make the context's weight copies once (transposed for backward, gain-folded with fuse_norm); valid until the
        weights change (then call again)."""
        self._check(lib.sv_prepare_weights(self._ctx, weights_c, self._stream()))

    def _results(self, n: int):
        return self.torch.empty((n, 32), dtype=self.torch.uint8, device="cuda")

    @staticmethod
    def read_results(res_dev) -> np.ndarray:
        return res_dev.cpu().numpy().view(RESULT_DTYPE).reshape(-1)

    def profile_enable(self, on: bool = True):
        self._check(lib.sv_profile_enable(self._ctx, int(on)))

    def profile_select(self, ops=None):
        """Bracket only these operation classes (names of OP_NAMES) with events; None: all of them."""
        mask = 0 if ops is None else sum(1 << OP_NAMES.index(o) for o in ops)
        self._check(lib.sv_profile_select(self._ctx, mask))

    def profile_read(self) -> Dict[str, Dict[str, float]]:
        p = ProfileC()
        self._check(lib.sv_profile_read(self._ctx, C.byref(p)))
        return {n: dict(ms=p.ms[i], flop=p.flop[i], launches=int(p.launches[i])) for i, n in enumerate(OP_NAMES)}

    # ------------------------------------------------------------------ entry points
    def verify_forward(self, weights_c, h_in, claimed_h=None, metrics=("rel_l2",), tau=(0, 0, 0, 0), reduce="max_token",
                       want_h_hat=False, want_token_scores=False):
        B, S, D = h_in.shape
        torch = self.torch
        h_hat = torch.empty_like(h_in) if want_h_hat else None
        tok = torch.empty(B * S, dtype=torch.float32, device=h_in.device) if (want_token_scores and claimed_h is not None) else None
        res = self._results(1) if claimed_h is not None else None
        self._check(lib.sv_verify_forward(self._ctx, weights_c, _ptr(h_in), B, S, _ptr(claimed_h), _mask(metrics), _tau_array(tau),
                                          SV_REDUCE_MAX_TOKEN if reduce == "max_token" else SV_REDUCE_GLOBAL,
                                          _ptr(h_hat), _ptr(tok), _ptr(res), self._stream()))
        return dict(result=res, h_hat=h_hat, token_scores=tok)

    def verify_backward(self, weights_c, h_in, g_out, claimed_g=None, metrics=("rel_l2",), tau=(0, 0, 0, 0), reduce="max_token",
                        want_g_hat=False, want_h_hat=False, want_token_scores=False):
        B, S, D = h_in.shape
        torch = self.torch
        g_hat = torch.empty_like(h_in) if want_g_hat else None
        h_hat = torch.empty_like(h_in) if want_h_hat else None
        tok = torch.empty(B * S, dtype=torch.float32, device=h_in.device) if (want_token_scores and claimed_g is not None) else None
        res = self._results(1) if claimed_g is not None else None
        self._check(lib.sv_verify_backward(self._ctx, weights_c, _ptr(h_in), _ptr(g_out), B, S, _ptr(claimed_g), _mask(metrics),
                                           _tau_array(tau), SV_REDUCE_MAX_TOKEN if reduce == "max_token" else SV_REDUCE_GLOBAL,
                                           _ptr(g_hat), _ptr(h_hat), _ptr(tok), _ptr(res), self._stream()))
        return dict(result=res, g_hat=g_hat, h_hat=h_hat, token_scores=tok)

    def score_and_flag(self, claims, ref, metrics=("rel_l2",), tau=(0, 0, 0, 0), reduce="max_token", want_token_scores=False):
        """claims [n, T, D] (or [n, B, S, D]); ref [T, D] shared or [n, T, D] per claim."""
        torch = self.torch
        n, D = claims.shape[0], claims.shape[-1]
        T = claims[0].numel() // D
        shared = ref.numel() == T * D
        assert claims.is_contiguous() and ref.is_contiguous()
        tok = torch.empty((n, T), dtype=torch.float32, device=claims.device) if want_token_scores else None
        res = self._results(n)
        self._check(lib.sv_score_and_flag(self._ctx, _ptr(claims), T * D, n, _ptr(ref), 0 if shared else T * D, _dt(claims), _dt(ref),
                                          T, D, _mask(metrics), _tau_array(tau),
                                          SV_REDUCE_MAX_TOKEN if reduce == "max_token" else SV_REDUCE_GLOBAL,
                                          _ptr(tok), _ptr(res), self._stream()))
        return dict(result=res, token_scores=tok)

    def score_and_sum(self, claims, ref, skip=None, metrics=("rel_l2",), tau=(0, 0, 0, 0), reduce="max_token", want_token_scores=False):
        """score_and_flag against one shared reference [T, D] that also returns sum [T, D] float32 = the sum of the
        claims whose entry in `skip` (host sequence of n flags, or None) is zero."""
        torch = self.torch
        n, D = claims.shape[0], claims.shape[-1]
        T = claims[0].numel() // D
        assert claims.is_contiguous() and ref.is_contiguous() and ref.numel() == T * D
        tok = torch.empty((n, T), dtype=torch.float32, device=claims.device) if want_token_scores else None
        res = self._results(n)
        total = torch.empty((T, D), dtype=torch.float32, device=claims.device)
        skip_b = None if skip is None else bytes(bytearray(int(bool(x)) for x in skip))
        assert skip_b is None or len(skip_b) == n
        self._check(lib.sv_score_and_sum(self._ctx, _ptr(claims), T * D, n, _ptr(ref), _dt(claims), _dt(ref), T, D, _mask(metrics),
                                         _tau_array(tau), SV_REDUCE_MAX_TOKEN if reduce == "max_token" else SV_REDUCE_GLOBAL,
                                         _ptr(tok), _ptr(res), skip_b, _ptr(total), self._stream()))
        return dict(result=res, token_scores=tok, sum=total)

    def ema_from_sum(self, m, total, n_summed: int, beta: float):
        """m [T, D] float32 updated in place from the sum of n_summed claims that score_and_sum returned."""
        D = m.shape[-1]
        T = m.numel() // D
        assert m.dtype == self.torch.float32 and total.dtype == self.torch.float32 and total.numel() == m.numel()
        assert m.is_contiguous() and total.is_contiguous()
        self._check(lib.sv_ema_from_sum(self._ctx, _ptr(m), _ptr(total), int(n_summed), T, D, float(beta), self._stream()))
        return m

    def sliced_wasserstein(self, claims, ref, directions, tau: float, results=None):
        """claims [n, T, D]; ref [T, D] shared or [n, T, D]; directions bf16 [L, D].  Returns sw [n] float32 (device);
        with `results` (the sv_result tensor of an earlier scoring call) the flag is OR-ed into it."""
        torch = self.torch
        n, D = claims.shape[0], claims.shape[-1]
        T = claims[0].numel() // D
        shared = ref.numel() == T * D
        assert claims.is_contiguous() and ref.is_contiguous() and directions.is_contiguous()
        assert directions.dtype == torch.bfloat16 and directions.shape[1] == D
        sw = torch.empty((n,), dtype=torch.float32, device=claims.device)
        self._check(lib.sv_sliced_wasserstein(self._ctx, _ptr(claims), T * D, n, _ptr(ref), 0 if shared else T * D, _dt(claims), _dt(ref),
                                              T, D, _ptr(directions), directions.shape[0], float(tau), _ptr(sw), _ptr(results),
                                              self._stream()))
        return sw

    def sw_against_projection(self, claims, ref_proj, directions, tau: float, results=None):
        """claims [n, T, D]; ref_proj [L, Tpad] float32: unsorted projections of the reference; directions bf16 [L, D].
        Returns (sw [n] float32, claim_proj [n, L, Tpad] float32), both on the device."""
        torch = self.torch
        n, D = claims.shape[0], claims.shape[-1]
        T = claims[0].numel() // D
        L, Tpad = directions.shape[0], lib.sv_sw_row_len(T)
        assert claims.is_contiguous() and ref_proj.is_contiguous() and directions.is_contiguous()
        assert directions.dtype == torch.bfloat16 and ref_proj.dtype == torch.float32 and tuple(ref_proj.shape) == (L, Tpad)
        sw = torch.empty((n,), dtype=torch.float32, device=claims.device)
        proj = torch.empty((n, L, Tpad), dtype=torch.float32, device=claims.device)
        self._check(lib.sv_sw_against_projection(self._ctx, _ptr(claims), T * D, n, _dt(claims), T, D, _ptr(directions), L, _ptr(ref_proj),
                                                 _ptr(proj), float(tau), _ptr(sw), _ptr(results), self._stream()))
        return sw, proj

    def sw_projection_ema(self, ref_proj, claim_proj, T: int, skip, beta: float):
        """ref_proj [L, Tpad] updated in place from claim_proj [n, L, Tpad]; skip: host sequence of n flags or None."""
        n, L = claim_proj.shape[0], claim_proj.shape[1]
        skip_b = None if skip is None else bytes(bytearray(int(bool(x)) for x in skip))
        assert ref_proj.is_contiguous() and claim_proj.is_contiguous() and (skip_b is None or len(skip_b) == n)
        self._check(lib.sv_sw_projection_ema(self._ctx, _ptr(ref_proj), _ptr(claim_proj), n, skip_b, int(T), L, float(beta), self._stream()))
        return ref_proj

    def replace_with_ema(self, signals, mask_dev, m):
        """signals [n, T, D] updated in place: signal i becomes m (rounded) where mask_dev[i] != 0."""
        n, D = signals.shape[0], signals.shape[-1]
        T = signals[0].numel() // D
        assert signals.is_contiguous() and m.dtype == self.torch.float32 and m.numel() == T * D and mask_dev.dtype == self.torch.uint8
        self._check(lib.sv_replace_with_ema(self._ctx, _ptr(signals), T * D, n, _dt(signals), _ptr(mask_dev), _ptr(m), T, D, self._stream()))
        return signals

    def ema_update(self, m, claims, flags_dev, beta: float):
        """m [T, D] float32 updated in place from claims [n, T, D]; flags_dev: uint8 [n] on the device or None."""
        n, D = claims.shape[0], claims.shape[-1]
        T = claims[0].numel() // D
        assert m.dtype == self.torch.float32 and m.numel() == T * D and m.is_contiguous() and claims.is_contiguous()
        self._check(lib.sv_ema_update(self._ctx, _ptr(m), _ptr(claims), T * D, n, _dt(claims), _ptr(flags_dev), T, D, float(beta),
                                      self._stream()))
        return m


METRIC_ORDER = ("rel_l2", "l1", "zl2", "sfr", "sw")


class Sentinel:
    """One sv_sentinel: the verifier loop over n_stages x n_workers with EMAs on the device and the policy on the host."""

    def __init__(self, verifier: Verifier, n_stages: int, n_workers: int, T: int, D: int, metrics, directions=None,
                 beta_h: float = 0.9, beta_g: float = 0.8, policy_h=None, policy_g=None):
        self.ver, self.p, self.d, self.T, self.D = verifier, n_stages, n_workers, T, D
        self.metrics = [m for m in METRIC_ORDER if m in metrics]
        mask = sum(1 << METRIC_ORDER.index(m) for m in self.metrics)
        self._dirs = directions                      # kept alive: the library retains the pointer
        cfg = SentinelCfgC(n_stages, n_workers, T, D, mask, 0 if directions is None else directions.shape[0],
                           None if directions is None else directions.data_ptr(), beta_h, beta_g,
                           _policy_cfg(**(policy_h or {})), _policy_cfg(**(policy_g or {})))
        self._s = C.c_void_p()
        st = lib.sv_sentinel_create(verifier._ctx, C.byref(cfg), C.byref(self._s))
        if st != SV_OK:
            raise SVError(st, "sv_sentinel_create")

    def close(self):
        if self._s:
            lib.sv_sentinel_destroy(self._s)
            self._s = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st):
        if st != SV_OK:
            raise SVError(st, lib.sv_sentinel_last_error(self._s).decode())

    def begin_iteration(self, warmup: bool):
        self._check(lib.sv_sentinel_begin_iteration(self._s, int(bool(warmup))))

    def _call(self, fn, stage, signals):
        assert signals.is_contiguous() and signals.shape[0] == self.d and signals[0].numel() == self.T * self.D
        tainted = np.zeros(self.d, dtype=np.uint8)
        gamma = np.zeros((self.d, len(self.metrics)), dtype=np.float64)
        self._check(fn(self._s, stage, _ptr(signals), _dt(signals), tainted.ctypes.data_as(C.POINTER(C.c_uint8)),
                       gamma.ctypes.data_as(C.POINTER(C.c_double)), self.ver._stream()))
        return [int(r) for r in np.nonzero(tainted)[0]], gamma

    def forward(self, stage: int, h):
        """h [n_workers, T, D]; returns (workers tainted at this stage, Gamma)."""
        return self._call(lib.sv_sentinel_forward, stage, h)

    def backward(self, stage: int, g):
        """g [n_workers, T, D], tainted workers' gradients are replaced in place; returns (tainted, Gamma)."""
        return self._call(lib.sv_sentinel_backward, stage, g)

    def state(self, stage: int, kind: str):
        v = np.zeros(self.d, dtype=np.int32)
        b = np.zeros(self.d, dtype=np.uint8)
        lo, up, k = (np.zeros(len(self.metrics), dtype=np.float64) for _ in range(3))
        ema = C.c_void_p()
        dp, u8p, ip = C.POINTER(C.c_double), C.POINTER(C.c_uint8), C.POINTER(C.c_int32)
        self._check(lib.sv_sentinel_state(self._s, stage, 0 if kind == "h" else 1, C.byref(ema), v.ctypes.data_as(ip), b.ctypes.data_as(u8p),
                                          lo.ctypes.data_as(dp), up.ctypes.data_as(dp), k.ctypes.data_as(dp)))
        return dict(ema_ptr=ema.value, violations=v, banned=b.astype(bool), lower=lo, upper=up, k=k)

    def counters(self) -> dict:
        """How the stage calls were served: calls, EMA updates from the score pass's sum / from the signals, sliced
        Wasserstein checks against carried projections."""
        c = (C.c_int64 * 4)()
        self._check(lib.sv_sentinel_counters(self._s, c))
        return dict(calls=c[0], ema_from_sum=c[1], ema_from_signals=c[2], sw_carried=c[3])

    def ema(self, stage: int, kind: str) -> np.ndarray:
        """A host copy of the stage's EMA, [T, D] float32."""
        out = np.empty((self.T, self.D), dtype=np.float32)
        self._check(lib.sv_sentinel_read_ema(self._s, stage, 0 if kind == "h" else 1, out.ctypes.data_as(C.POINTER(C.c_float)),
                                             self.ver._stream()))
        return out

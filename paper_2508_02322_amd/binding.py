"""Thin ctypes binding over libcamera_hip.so (include/camera.h).

Argument marshalling only: every step of the path runs in the HIP kernels
behind the C ABI.  torch is used for device memory and the current stream.
There is no CPU fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libcamera_hip.so")

F32, BF16 = 0, 1
ACCUMULATE, NO_FINALIZE = 1, 2
K_ROUTE, K_BUCKET, K_GEMM, K_DOWN_NORM, K_FINALIZE, K_RANK, K_GATHER, K_DOWN_GEMM, K_COMBINE = range(9)
KERNEL_NAMES = ["route", "bucket", "gemm", "down_norm", "finalize", "rank", "gather", "down_gemm", "combine",
                "compact_hidden", "compact_down"]

EXPORTS = ["camera_create", "camera_destroy", "camera_last_error", "camera_version", "camera_route_topk",
           "camera_score_layer", "camera_select_prune", "camera_select_prune_noalloc", "camera_select_prune_multi", "camera_alloc_bits", "camera_rank_decisions",
           "camera_gather_micro_experts", "camera_input_channel_energy", "camera_layer_forward", "camera_layer_forward_compact", "camera_output_error", "camera_profile_enable",
           "camera_profile_read"]

_c = ctypes
_vp, _i, _i64, _f, _d = _c.c_void_p, _c.c_int, _c.c_int64, _c.c_float, _c.c_double


class CameraError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"camera status {code}: {message}")
        self.code = code
        self.message = message


def load_library(path: str = LIB_PATH) -> ctypes.CDLL:
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} is missing: build it with `python -m paper_2508_02322_amd.build` (there is no fallback path)")
    lib = ctypes.CDLL(path)
    lib.camera_create.argtypes = [_c.POINTER(_vp), _i]
    lib.camera_destroy.argtypes = [_vp]
    lib.camera_last_error.argtypes = [_vp]
    lib.camera_last_error.restype = _c.c_char_p
    lib.camera_version.argtypes = []
    lib.camera_route_topk.argtypes = [_vp, _vp, _vp, _i, _i64, _i64, _i64, _vp, _i64, _vp, _i, _i, _i, _vp, _vp]
    lib.camera_score_layer.argtypes = [_vp, _vp, _vp, _i, _i64, _i64, _i64, _vp, _vp, _i, _i, _i64, _vp, _vp, _i64,
                                       _vp, _i64, _f, _i, _vp, _vp, _vp, _vp]
    lib.camera_select_prune.argtypes = [_vp, _vp, _vp, _i64, _c.POINTER(_i64), _i, _d, _vp, _vp, _vp, _vp]
    lib.camera_select_prune_noalloc.argtypes = [_vp, _vp, _vp, _i64, _c.POINTER(_i64), _i, _d, _vp, _vp, _vp]
    lib.camera_select_prune_multi.argtypes = [_vp, _vp, _vp, _i64, _c.POINTER(_i64), _i, _i, _c.POINTER(_d), _vp, _vp]
    lib.camera_alloc_bits.argtypes = [_vp, _vp, _vp, _i64, _c.POINTER(_i64), _i, _i, _c.POINTER(_i),
                                      _c.POINTER(_d), _vp, _vp, _vp]
    lib.camera_rank_decisions.argtypes = [_vp, _vp, _vp, _i64, _c.POINTER(_i64), _i, _i, _c.POINTER(_d), _vp, _vp, _i,
                                          _c.POINTER(_i), _c.POINTER(_d), _vp, _vp, _vp]
    lib.camera_gather_micro_experts.argtypes = [_vp, _vp, _i, _i, _i64, _i64, _vp, _vp, _i64, _vp, _i64, _vp, _i64,
                                                _i64, _vp, _i, _vp, _vp, _vp]
    lib.camera_input_channel_energy.argtypes = [_vp, _vp, _vp, _i, _i64, _i64, _i64, _vp, _i, _i, _vp]
    lib.camera_layer_forward.argtypes = [_vp, _vp, _vp, _i, _i64, _i64, _i64, _vp, _vp, _i, _i, _i64, _vp, _vp, _i64,
                                         _vp, _i64, _vp, _i, _vp]
    lib.camera_layer_forward_compact.argtypes = [_vp, _vp, _vp, _i, _i64, _i64, _i64, _vp, _vp, _i, _i, _i,
                                                 _c.POINTER(_c.c_int32), _i, _vp, _vp, _vp, _i, _vp]
    lib.camera_output_error.argtypes = [_vp, _vp, _vp, _vp, _i64, _i64, _vp]
    lib.camera_profile_enable.argtypes = [_vp, _i]
    lib.camera_profile_read.argtypes = [_vp, _i, _c.POINTER(_d), _c.POINTER(_i64)]
    for name in EXPORTS:
        if name != "camera_last_error":
            getattr(lib, name).restype = _i
    return lib


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else _vp(t.data_ptr())


def _require(cond: bool, message: str):
    """Layouts the library cannot see from a pointer and one stride: refuse them here instead of reading wrong bytes."""
    if not cond:
        raise CameraError(-2, message)


def _check_matrix(t, name: str, like=None):
    """[rows, cols] with unit inner stride (the row stride is passed on)."""
    if t is None:
        return
    _require(t.dim() == 2 and t.stride(1) == 1, f"{name}: must be 2-D with unit inner stride (got strides {tuple(t.stride())})")
    if like is not None:
        _require(t.dtype == like.dtype and t.device == like.device, f"{name}: dtype / device differ from X")


def _check_experts(t, name: str, like=None):
    """[N_E, rows, cols] with contiguous rows exactly cols apart (the expert stride is passed on)."""
    if t is None:
        return
    _require(t.dim() == 3 and t.stride(2) == 1 and t.stride(1) == t.shape[2],
             f"{name}: must be [experts, rows, cols] with rows contiguous and cols apart (got strides {tuple(t.stride())})")
    if like is not None:
        _require(t.dtype == like.dtype and t.device == like.device, f"{name}: dtype / device differ from X")


def _check_flat(t, name: str, dtype=None, device=None):
    if t is None:
        return
    _require(t.is_contiguous(), f"{name}: must be contiguous")
    if dtype is not None:
        _require(t.dtype == dtype, f"{name}: must be {dtype}")
    if device is not None:
        _require(t.device == device, f"{name}: on another device")


def _stream_handle(device) -> _vp:
    return _vp(torch.cuda.current_stream(device).cuda_stream)


class Camera:
    """One library context on one GPU.  Methods mirror the C entry points and
    allocate their outputs with torch on the context's device."""

    def __init__(self, device: int = 0, lib_path: str = LIB_PATH):
        self.lib = load_library(lib_path)
        self.device = torch.device("cuda", device)
        self._ctx = _vp()
        rc = self.lib.camera_create(_c.byref(self._ctx), device)
        if rc != 0:
            raise CameraError(rc, self.lib.camera_last_error(None).decode())

    def close(self):
        if getattr(self, "_ctx", None) is not None and self._ctx.value:
            self.lib.camera_destroy(self._ctx)
            self._ctx = _vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int):
        if rc != 0:
            raise CameraError(rc, self.lib.camera_last_error(self._ctx).decode())

    @staticmethod
    def _check_layer(X, topk_idx, topk_w, W_gate, W_up, W_down):
        _check_matrix(X, "X")
        _check_experts(W_gate, "W_gate", like=X)
        _check_experts(W_up, "W_up", like=X)
        _check_experts(W_down, "W_down", like=X)
        _check_flat(topk_idx, "topk_idx", torch.int32, X.device)
        _check_flat(topk_w, "topk_w", torch.float32, X.device)
        if W_gate is not None and W_up is not None:
            _require(W_gate.shape == W_up.shape and W_gate.stride(0) == W_up.stride(0), "W_gate / W_up: shapes or expert strides differ")
        if W_gate is not None:
            _require(W_gate.shape[2] == X.shape[1], "W_gate: d_model differs from X")
        if W_gate is not None and W_down is not None:
            _require(W_down.shape[0] == W_gate.shape[0] and W_down.shape[1] == W_gate.shape[2] and W_down.shape[2] == W_gate.shape[1],
                     "W_down: must be [experts, d_model, d_ff]")

    # ---- entry points ------------------------------------------------------
    def route_topk(self, X, W_r, bias, top_k: int, renorm: bool = True):
        _check_matrix(X, "X")
        _check_matrix(W_r, "W_r", like=X)
        _check_flat(bias, "bias", torch.float32, X.device)
        n, d = X.shape
        n_experts = W_r.shape[0]
        idx = torch.empty((n, top_k), dtype=torch.int32, device=self.device)
        w = torch.empty((n, top_k), dtype=torch.float32, device=self.device)
        self._check(self.lib.camera_route_topk(
            self._ctx, _stream_handle(self.device), _ptr(X), _dtype_code(X), n, d, X.stride(0), _ptr(W_r),
            W_r.stride(0), _ptr(bias), n_experts, top_k, int(renorm), _ptr(idx), _ptr(w)))
        return idx, w

    def score_layer(self, X, topk_idx, topk_w, W_gate, W_up, W_down, alpha: float, flags: int = 0, out=None):
        """W_gate / W_up [N_E, d_ff, d_model], W_down [N_E, d_model, d_ff] (None with NO_FINALIZE).
        Returns dict(phi2, phi_inf, omega2, energy); pass `out` to reuse / accumulate into buffers."""
        self._check_layer(X, topk_idx, topk_w, W_gate, W_up, W_down)
        n, d = X.shape
        n_experts, d_ff, _ = W_gate.shape
        n_micro = n_experts * d_ff
        if out is not None:
            for k, v in out.items():
                _check_flat(v, k, torch.float32, X.device)
        if out is None:
            out = {k: torch.empty(n_micro, dtype=torch.float32, device=self.device)
                   for k in ("phi2", "phi_inf", "omega2", "energy")}
        top_k = 0 if topk_idx is None else topk_idx.shape[1]
        self._check(self.lib.camera_score_layer(
            self._ctx, _stream_handle(self.device), _ptr(X), _dtype_code(X), n, d, X.stride(0), _ptr(topk_idx),
            _ptr(topk_w), top_k, n_experts, d_ff, _ptr(W_gate), _ptr(W_up), W_gate.stride(0), _ptr(W_down),
            0 if W_down is None else W_down.stride(0), float(alpha), flags, _ptr(out["phi2"]), _ptr(out["phi_inf"]),
            _ptr(out.get("omega2")), _ptr(out.get("energy"))))
        return out

    def select_prune(self, energy, seg_offsets: Sequence[int], ratio: float, want_idx=False, want_rank=False):
        _check_flat(energy, "energy", torch.float32)
        n_micro = energy.numel()
        n_seg = len(seg_offsets) - 1
        seg = (_i64 * (n_seg + 1))(*seg_offsets)
        keep = torch.empty(n_micro, dtype=torch.uint8, device=self.device)
        per_expert = torch.empty(n_seg, dtype=torch.int32, device=self.device)
        # kept_idx is sized for the worst case; the caller trims it with per_expert.sum()
        kept_idx = torch.empty(n_micro, dtype=torch.int32, device=self.device) if want_idx else None
        rank = torch.empty(n_micro, dtype=torch.int32, device=self.device) if want_rank else None
        self._check(self.lib.camera_select_prune(
            self._ctx, _stream_handle(self.device), _ptr(energy), n_micro, seg, n_seg, float(ratio), _ptr(keep),
            _ptr(per_expert), _ptr(kept_idx), _ptr(rank)))
        return keep, per_expert, kept_idx, rank

    def select_prune_noalloc(self, energy, seg_offsets: Sequence[int], ratio: float, keep, per_expert, kept_idx=None):
        """camera_select_prune_noalloc: the caller brings every output (keep uint8 [n_micro], per_expert int32
        [n_seg], kept_idx int32 [>= kept] or None); the call itself allocates nothing on the device."""
        _check_flat(energy, "energy", torch.float32)
        _check_flat(keep, "keep", torch.uint8, energy.device)
        _check_flat(per_expert, "per_expert", torch.int32, energy.device)
        _check_flat(kept_idx, "kept_idx", torch.int32, energy.device)
        n_seg = len(seg_offsets) - 1
        seg = (_i64 * (n_seg + 1))(*seg_offsets)
        self._check(self.lib.camera_select_prune_noalloc(
            self._ctx, _stream_handle(self.device), _ptr(energy), energy.numel(), seg, n_seg, float(ratio), _ptr(keep),
            _ptr(per_expert), _ptr(kept_idx)))

    def select_prune_multi(self, energy, seg_offsets, ratios, out=None):
        """Masks at several rising ratios from one ranking pass: (keep_bits uint8 [n_micro] with bit k = kept at
        ratios[k], kept_per_expert int32 [len(ratios), n_seg])."""
        _check_flat(energy, "energy", torch.float32)
        n_micro = energy.numel()
        n_seg = len(seg_offsets) - 1
        seg = (_i64 * (n_seg + 1))(*seg_offsets)
        if out is None:
            out = (torch.empty(n_micro, dtype=torch.uint8, device=self.device),
                   torch.empty((len(ratios), n_seg), dtype=torch.int32, device=self.device))
        self._check(self.lib.camera_select_prune_multi(
            self._ctx, _stream_handle(self.device), _ptr(energy), n_micro, seg, n_seg, len(ratios),
            (_d * len(ratios))(*[float(r) for r in ratios]), _ptr(out[0]), _ptr(out[1])))
        return out

    def alloc_bits(self, energy, seg_offsets: Sequence[int], bits: Sequence[int], ratios: Sequence[float],
                   want_perm=False):
        _check_flat(energy, "energy", torch.float32)
        n_micro = energy.numel()
        n_seg = len(seg_offsets) - 1
        n_levels = len(bits)
        seg = (_i64 * (n_seg + 1))(*seg_offsets)
        bit_of = torch.empty(n_micro, dtype=torch.uint8, device=self.device)
        level_count = torch.empty((n_seg, n_levels), dtype=torch.int32, device=self.device)
        perm = torch.empty(n_micro, dtype=torch.int32, device=self.device) if want_perm else None
        self._check(self.lib.camera_alloc_bits(
            self._ctx, _stream_handle(self.device), _ptr(energy), n_micro, seg, n_seg, n_levels,
            (_i * n_levels)(*bits), (_d * len(ratios))(*ratios), _ptr(bit_of), _ptr(level_count), _ptr(perm)))
        return bit_of, level_count, perm

    def rank_decisions(self, energy, seg_offsets, prune_ratios, bits, level_ratios, want_perm=False, out=None):
        """The CAMERA-P masks at several rising ratios and one CAMERA-Q bit allocation from one pass over the
        ranking: (keep_bits, kept_per_expert [len(prune_ratios), n_seg], bit_of, level_count [n_seg, len(bits)], perm)."""
        _check_flat(energy, "energy", torch.float32)
        n_micro = energy.numel()
        n_seg = len(seg_offsets) - 1
        seg = (_i64 * (n_seg + 1))(*seg_offsets)
        if out is None:
            out = (torch.empty(n_micro, dtype=torch.uint8, device=self.device),
                   torch.empty((len(prune_ratios), n_seg), dtype=torch.int32, device=self.device),
                   torch.empty(n_micro, dtype=torch.uint8, device=self.device),
                   torch.empty((n_seg, len(bits)), dtype=torch.int32, device=self.device),
                   torch.empty(n_micro, dtype=torch.int32, device=self.device) if want_perm else None)
        self._check(self.lib.camera_rank_decisions(
            self._ctx, _stream_handle(self.device), _ptr(energy), n_micro, seg, n_seg, len(prune_ratios),
            (_d * len(prune_ratios))(*[float(r) for r in prune_ratios]), _ptr(out[0]), _ptr(out[1]), len(bits),
            (_i * len(bits))(*bits), (_d * len(level_ratios))(*[float(r) for r in level_ratios]), _ptr(out[2]), _ptr(out[3]),
            _ptr(out[4])))
        return out

    def gather_micro_experts(self, W_gate, W_up, W_down, index, count=None, index_base=0, out=None, down_row_align=1):
        """Kept gate / up rows and down columns of one group of experts (Algorithm 2, lines 10-13).
        W_gate, W_up [N_E, d_ff, d_model], W_down [N_E, d_model, d_ff] (any of them may be None: skipped);
        index int32 [n_index] global indices grouped by expert; count int32 [N_E] or None (d_ff each);
        down_row_align: the rows of every W_down block are padded with zeros to a multiple of it.
        Returns (gate_out [n_index, d_model], up_out, down_out flat: sized for the longest padding when
        allocated here, [d_model][ld(e)] blocks one after the other)."""
        ref = W_gate if W_gate is not None else (W_up if W_up is not None else W_down)
        for name, t in (("W_gate", W_gate), ("W_up", W_up), ("W_down", W_down)):
            _check_experts(t, name)
        _check_flat(index, "index", torch.int32, ref.device)
        _check_flat(count, "count", torch.int32, ref.device)
        n_experts = ref.shape[0]
        d_ff, d_model = (ref.shape[1], ref.shape[2]) if ref is not W_down else (ref.shape[2], ref.shape[1])
        n_index = index.numel()
        stride_gu = (W_gate if W_gate is not None else W_up).stride(0) if (W_gate is not None or W_up is not None) else 0
        if out is None:
            mk = lambda src, shape: None if src is None else torch.empty(shape, dtype=src.dtype, device=self.device)
            padded = n_index + n_experts * (int(down_row_align) - 1)
            out = (mk(W_gate, (n_index, d_model)), mk(W_up, (n_index, d_model)), mk(W_down, (padded * d_model,)))
        self._check(self.lib.camera_gather_micro_experts(
            self._ctx, _stream_handle(self.device), _dtype_code(ref), n_experts, d_ff, d_model, _ptr(W_gate), _ptr(W_up),
            stride_gu, _ptr(W_down), W_down.stride(0) if W_down is not None else 0, _ptr(index), n_index,
            int(index_base), _ptr(count), int(down_row_align), _ptr(out[0]), _ptr(out[1]), _ptr(out[2])))
        return out

    def input_channel_energy(self, X, topk_idx, n_experts: int, out=None):
        """h [n_experts, d_model] float32: per expert, the sum over its routed tokens of X[j, c]^2 (the statistic the
        column-wise comparison variant CAMERA-Q-dagger ranks the input channels of W_up / W_gate by)."""
        _check_matrix(X, "X")
        _check_flat(topk_idx, "topk_idx", torch.int32, X.device)
        n, d = X.shape
        if out is None:
            out = torch.empty((n_experts, d), dtype=torch.float32, device=self.device)
        _check_flat(out, "h", torch.float32, X.device)
        self._check(self.lib.camera_input_channel_energy(
            self._ctx, _stream_handle(self.device), _ptr(X), _dtype_code(X), n, d, X.stride(0), _ptr(topk_idx),
            0 if topk_idx is None else topk_idx.shape[1], int(n_experts), _ptr(out)))
        return out

    def layer_forward(self, X, topk_idx, topk_w, W_gate, W_up, W_down, keep_mask=None, Y=None, accumulate=False):
        """Layer output over the kept micro-experts of one group of experts (Eq. 1-2); Y float32 [n, d_model]."""
        self._check_layer(X, topk_idx, topk_w, W_gate, W_up, W_down)
        _check_flat(keep_mask, "keep_mask", torch.uint8, X.device)
        _check_flat(Y, "Y", torch.float32, X.device)
        n, d = X.shape
        n_experts, d_ff, _ = W_gate.shape
        top_k = 0 if topk_idx is None else topk_idx.shape[1]
        if Y is None:
            Y = torch.empty((n, d), dtype=torch.float32, device=self.device)
        self._check(self.lib.camera_layer_forward(
            self._ctx, _stream_handle(self.device), _ptr(X), _dtype_code(X), n, d, X.stride(0), _ptr(topk_idx),
            _ptr(topk_w), top_k, n_experts, d_ff, _ptr(W_gate), _ptr(W_up), W_gate.stride(0), _ptr(W_down),
            W_down.stride(0), _ptr(keep_mask), ACCUMULATE if accumulate else 0, _ptr(Y)))
        return Y

    def layer_forward_compact(self, X, topk_idx, topk_w, count, W_gate_c, W_up_c, W_down_c, n_shared=0,
                              down_row_align=1, Y=None, accumulate=False):
        """Layer output from compacted weights (the outputs of gather_micro_experts, with the same
        down_row_align); count: per-expert kept micro-experts as a sequence of Python ints, the last n_shared
        of them shared experts (every token, weight 1).  Y float32 [n, d_model]."""
        _check_matrix(X, "X")
        for name, t in (("W_gate_c", W_gate_c), ("W_up_c", W_up_c), ("W_down_c", W_down_c)):
            # (a dtype other than bf16 is the library's to refuse: it names what it supports)
            _check_flat(t, name, X.dtype if X.dtype == torch.bfloat16 else None, X.device)
        _check_flat(topk_idx, "topk_idx", torch.int32, X.device)
        _check_flat(topk_w, "topk_w", torch.float32, X.device)
        _check_flat(Y, "Y", torch.float32, X.device)
        n, d = X.shape
        counts = [int(c) for c in count]
        top_k = 0 if topk_idx is None else topk_idx.shape[1]
        if Y is None:
            Y = torch.empty((n, d), dtype=torch.float32, device=self.device)
        self._check(self.lib.camera_layer_forward_compact(
            self._ctx, _stream_handle(self.device), _ptr(X), _dtype_code(X), n, d, X.stride(0), _ptr(topk_idx),
            _ptr(topk_w), top_k, len(counts) - int(n_shared), int(n_shared), (_c.c_int32 * len(counts))(*counts),
            int(down_row_align), _ptr(W_gate_c), _ptr(W_up_c), _ptr(W_down_c), ACCUMULATE if accumulate else 0, _ptr(Y)))
        return Y

    def output_error(self, Y, Y_hat):
        """Per-token [n, 4]: ||y - y_hat||^2, ||y||^2, ||y_hat||^2, <y, y_hat>."""
        _check_flat(Y, "Y", torch.float32)
        _check_flat(Y_hat, "Y_hat", torch.float32, Y.device)
        n, d = Y.shape
        out = torch.empty((n, 4), dtype=torch.float32, device=self.device)
        self._check(self.lib.camera_output_error(self._ctx, _stream_handle(self.device), _ptr(Y), _ptr(Y_hat), n, d,
                                                 _ptr(out)))
        return out

    # ---- profiling ---------------------------------------------------------
    def profile_enable(self, on: bool):
        self._check(self.lib.camera_profile_enable(self._ctx, int(on)))

    def profile_read(self, kernel_id: int):
        ms, count = _d(), _i64()
        self._check(self.lib.camera_profile_read(self._ctx, kernel_id, _c.byref(ms), _c.byref(count)))
        return ms.value, count.value

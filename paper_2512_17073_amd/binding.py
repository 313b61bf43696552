"""Thin ctypes binding of libmoe_lrc.so: argument marshalling only.

Every step of the layer runs in the library's HIP kernels; PyTorch appears here only as the owner
of device buffers and the source of the current HIP stream.  There is no fallback: if the shared
library is missing, importing a symbol raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoe_lrc.so")

RESIDENT, STAGED, POOLED = 0, 1, 2
STACK_PREFETCH, STACK_RESIDUAL = 1, 2

# every symbol include/moe_lrc.h declares
EXPORTS = [
    "moe_lrc_last_error", "moe_lrc_layer_create", "moe_lrc_layer_destroy", "moe_lrc_set_gate",
    "moe_lrc_set_expert", "moe_lrc_set_expert_ranked", "moe_lrc_set_expert_factors_quantized", "moe_lrc_workspace_bytes", "moe_lrc_route", "moe_lrc_permute",
    "moe_lrc_expert_ffn", "moe_lrc_combine", "moe_lrc_forward", "moe_lrc_forward_noalloc", "moe_lrc_debug_unpack",
    "moe_lrc_packed_bytes", "moe_lrc_pack_codes", "moe_lrc_unpack_codes", "moe_lrc_get_stats",
    "moe_lrc_profile_enable", "moe_lrc_profile_read", "moe_lrc_calibrate",
    "moe_lrc_selftest_decode_index", "moe_lrc_selftest_factor_pair",
    "moe_lrc_offline_quantize", "moe_lrc_offline_quantize_refined", "moe_lrc_offline_factors", "moe_lrc_offline_kurtosis", "moe_lrc_offline_allocate_ranks", "moe_lrc_selftest_half_rounding",
    "moe_lrc_stack_create", "moe_lrc_stack_destroy", "moe_lrc_stack_step", "moe_lrc_stack_get_stats", "moe_lrc_stack_reset",
]
STAGES = ["route", "permute", "prep", "xa13", "w13", "xa2", "w2", "shared", "combine"]


class Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "hidden", "ffn", "n_experts", "n_shared", "top_k", "top_n", "bits", "shared_bits", "group",
        "rank", "renormalize", "max_tokens", "residency")]


class Stats(C.Structure):
    _fields_ = [("bytes_codes", C.c_uint64), ("bytes_meta", C.c_uint64), ("bytes_factors", C.c_uint64),
                ("active_experts", C.c_int32), ("comp_experts", C.c_int32), ("path", C.c_int32),
                ("stage_ms", C.c_float)]


class StackStats(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("steps", "expert_uses", "hits", "misses", "prefetched", "prefetch_hits",
                                          "factor_copies", "bytes_h2d")] + [("last_step_ms", C.c_float), ("last_copy_ms", C.c_float)]


class MoeLrcError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"moe_lrc error {code}: {text}")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    """Loads the built library (raises if it has not been built: there is no other path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is not built; run `python -m paper_2512_17073_amd.build` "
                                    "(or __graft_entry__.build()) first")
        # torch ships its own HIP runtime; load it first so that this library binds to the same
        # runtime instance (two runtimes in one process do not share the device)
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        vp, i32, sz = C.c_void_p, C.c_int, C.c_size_t
        L.moe_lrc_last_error.restype = C.c_char_p
        L.moe_lrc_layer_create.argtypes = [C.POINTER(Config), C.POINTER(vp)]
        L.moe_lrc_layer_destroy.argtypes = [vp]
        L.moe_lrc_set_gate.argtypes = [vp, vp, vp]
        L.moe_lrc_set_expert.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp]
        L.moe_lrc_set_expert_ranked.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, i32]
        L.moe_lrc_set_expert_factors_quantized.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, vp, vp]
        L.moe_lrc_workspace_bytes.argtypes = [vp, i32]
        L.moe_lrc_workspace_bytes.restype = sz
        L.moe_lrc_route.argtypes = [vp, vp, i32, vp, vp, vp]
        L.moe_lrc_permute.argtypes = [vp, vp, i32, vp, vp, vp, vp, vp, vp]
        L.moe_lrc_expert_ffn.argtypes = [vp, vp, i32, vp, vp, vp, vp, sz, vp]
        L.moe_lrc_combine.argtypes = [vp, vp, vp, vp, vp, i32, vp, vp, sz, vp]
        L.moe_lrc_forward.argtypes = [vp, vp, i32, vp, vp, sz, vp]
        L.moe_lrc_forward_noalloc.argtypes = [vp, vp, i32, vp, vp]
        L.moe_lrc_debug_unpack.argtypes = [vp, i32, i32, vp, vp]
        L.moe_lrc_packed_bytes.argtypes = [i32, i32, i32]
        L.moe_lrc_packed_bytes.restype = sz
        L.moe_lrc_pack_codes.argtypes = [i32, i32, i32, vp, vp]
        L.moe_lrc_unpack_codes.argtypes = [i32, i32, i32, vp, vp]
        L.moe_lrc_get_stats.argtypes = [vp, C.POINTER(Stats)]
        L.moe_lrc_profile_enable.argtypes = [vp, i32]
        L.moe_lrc_profile_read.argtypes = [vp, C.POINTER(C.c_float)]
        L.moe_lrc_calibrate.argtypes = [i32, sz, i32, C.POINTER(C.c_double)]
        L.moe_lrc_selftest_decode_index.argtypes = [i32] * 14
        L.moe_lrc_offline_quantize.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, vp, vp]
        L.moe_lrc_offline_quantize_refined.argtypes = [vp, i32, i32, i32, i32, i32, C.c_double, C.c_double, C.c_double, vp, vp, vp, vp, vp]
        L.moe_lrc_offline_factors.argtypes = [vp, i32, i32, i32, vp, i32, i32, vp, vp, vp, vp, vp]
        L.moe_lrc_offline_kurtosis.argtypes = [vp, sz, C.POINTER(C.c_double)]
        L.moe_lrc_selftest_half_rounding.argtypes = [vp, sz, vp]
        L.moe_lrc_selftest_factor_pair.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp]
        L.moe_lrc_offline_allocate_ranks.argtypes = [vp, i32, i32, vp, i32, vp]
        L.moe_lrc_stack_create.argtypes = [C.POINTER(vp), i32, i32, i32, C.POINTER(vp)]
        L.moe_lrc_stack_destroy.argtypes = [vp]
        L.moe_lrc_stack_step.argtypes = [vp, vp, i32, vp, vp, vp]
        L.moe_lrc_stack_get_stats.argtypes = [vp, C.POINTER(StackStats)]
        L.moe_lrc_stack_reset.argtypes = [vp]
        _lib = L
    return _lib


def last_error() -> str:
    return lib().moe_lrc_last_error().decode()


def _check(rc: int) -> None:
    if rc != 0:
        raise MoeLrcError(rc, last_error())


def _host(a: Optional[np.ndarray], dtype) -> Optional[np.ndarray]:
    if a is None:
        return None
    return np.ascontiguousarray(a, dtype=dtype)


def _hp(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


CAL_HBM_READ, CAL_H2D, CAL_MFMA_F16, CAL_MFMA_F16_32, CAL_MFMA_VALU, CAL_SUBSTEP = 0, 1, 2, 3, 4, 5


def calibrate(kind: int, nbytes: int = 0, reps: int = 5) -> float:
    """moe_lrc_calibrate: GB/s (HBM read, pinned host -> device) or TFLOP/s (f16 MFMA) of this device."""
    out = C.c_double(0.0)
    _check(lib().moe_lrc_calibrate(kind, nbytes, reps, C.byref(out)))
    return out.value


def selftest_factor_pair(Aq: dict, Bq: dict):
    """moe_lrc_selftest_factor_pair (host only): (A [K][rank], B [rank][N]) float32 as the kernels rebuild a
    pair held at 3 bits; Aq / Bq as for Layer.set_expert_factors_quantized."""
    K, rank = Aq["codes"].shape
    N = Bq["codes"].shape[0]
    arrs = [_host(Aq["codes"], np.uint8), _host(Aq["scale"], np.uint16), _host(Aq["zero"], np.uint16),
            _host(Bq["codes"], np.uint8), _host(Bq["scale"], np.uint16), _host(Bq["zero"], np.uint16)]
    A = np.zeros((K, rank), np.float32)
    B = np.zeros((rank, N), np.float32)
    _check(lib().moe_lrc_selftest_factor_pair(K, N, rank, *[_hp(a) for a in arrs], _hp(A), _hp(B)))
    return A, B


def selftest_decode_index(hidden, ffn, bits, group, layer_rank, ranks, first_row, rows, total_rows,
                          blocks_w13, blocks_w2, kblocks_w2) -> None:
    """moe_lrc_selftest_decode_index (host only): raises MoeLrcError with the first violation."""
    _check(lib().moe_lrc_selftest_decode_index(hidden, ffn, bits, group, layer_rank, ranks[0], ranks[1], ranks[2],
                                               first_row, rows, total_rows, blocks_w13, blocks_w2, kblocks_w2))


# ---- host-only helpers (no device) ----------------------------------------------------------
def pack_codes(bits: int, codes: np.ndarray) -> np.ndarray:
    codes = _host(codes, np.uint8)
    K, N = codes.shape
    nbytes = lib().moe_lrc_packed_bytes(bits, K, N)
    if nbytes == 0:
        raise MoeLrcError(-2, "unsupported shape for packing")
    out = np.zeros(nbytes, dtype=np.uint8)
    _check(lib().moe_lrc_pack_codes(bits, K, N, _hp(codes), _hp(out)))
    return out


def unpack_codes(bits: int, K: int, N: int, packed: np.ndarray) -> np.ndarray:
    packed = _host(packed, np.uint8)
    out = np.empty((K, N), dtype=np.uint8)
    _check(lib().moe_lrc_unpack_codes(bits, K, N, _hp(packed), _hp(out)))
    return out


class Layer:
    """One MoE layer object of the library.  Methods mirror the C calls one to one."""

    def __init__(self, *, hidden, ffn, n_experts, top_k, top_n, bits, group, rank, max_tokens,
                 n_shared=0, shared_bits=4, renormalize=0, residency=RESIDENT):
        self.cfg = Config(hidden, ffn, n_experts, n_shared, top_k, top_n, bits, shared_bits, group,
                          rank, renormalize, max_tokens, residency)
        self._h = C.c_void_p()
        _check(lib().moe_lrc_layer_create(C.byref(self.cfg), C.byref(self._h)))
        self._ws = None

    @classmethod
    def from_config(cls, cfg, max_tokens=None, residency=RESIDENT) -> "Layer":
        """cfg: any object with the workload fields (hidden, ffn, n_experts, ...)."""
        return cls(hidden=cfg.hidden, ffn=cfg.ffn, n_experts=cfg.n_experts, top_k=cfg.top_k,
                   top_n=cfg.top_n, bits=cfg.bits, group=cfg.group, rank=cfg.rank,
                   max_tokens=max_tokens or cfg.tokens, n_shared=cfg.n_shared,
                   shared_bits=cfg.shared_bits, renormalize=cfg.renormalize, residency=residency)

    def close(self) -> None:
        if self._h:
            lib().moe_lrc_layer_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- uploads (host arrays) ----
    def set_gate(self, wg_bf16: np.ndarray, bias: Optional[np.ndarray] = None) -> None:
        wg = _host(wg_bf16, np.uint16)
        b = _host(bias, np.float32)
        _check(lib().moe_lrc_set_gate(self._h, _hp(wg), _hp(b)))

    def set_expert(self, expert: int, mat: int, codes, scale_f16, zero_f16, A_bf16=None, B_bf16=None,
                   rank: Optional[int] = None) -> None:
        """rank None: the layer's rank (moe_lrc_set_expert); an int: this projection's own rank
        (moe_lrc_set_expert_ranked), with A [K][rank] and B [rank][N], both None for rank 0."""
        arrs = [_host(codes, np.uint8), _host(scale_f16, np.uint16), _host(zero_f16, np.uint16),
                _host(A_bf16, np.uint16), _host(B_bf16, np.uint16)]
        if rank is None:
            _check(lib().moe_lrc_set_expert(self._h, expert, mat, *[_hp(a) for a in arrs]))
        else:
            _check(lib().moe_lrc_set_expert_ranked(self._h, expert, mat, *[_hp(a) for a in arrs], int(rank)))

    def set_expert_factors_quantized(self, expert: int, mat: int, rank: int, Aq: dict, Bq: dict) -> None:
        """Aq / Bq: {"codes", "scale", "zero"} of A [K][rank] and of B transposed [N][rank] at 3 bits."""
        arrs = [_host(Aq["codes"], np.uint8), _host(Aq["scale"], np.uint16), _host(Aq["zero"], np.uint16),
                _host(Bq["codes"], np.uint8), _host(Bq["scale"], np.uint16), _host(Bq["zero"], np.uint16)]
        _check(lib().moe_lrc_set_expert_factors_quantized(self._h, expert, mat, int(rank), *[_hp(a) for a in arrs]))

    def load(self, layer: dict) -> None:
        """layer = {"wg", "bias", "experts": [{mat: {"codes","scale","zero","A","B"}}]}."""
        self.set_gate(layer["wg"], layer.get("bias"))
        for e, ex in enumerate(layer["experts"]):
            for mat in (0, 1, 2):
                a = ex[mat]
                if a.get("Aq") is not None:          # factor pair at 3 bits
                    self.set_expert(e, mat, a["codes"], a["scale"], a["zero"], None, None, 0)
                    self.set_expert_factors_quantized(e, mat, a["Aq"]["codes"].shape[1], a["Aq"], a["Bq"])
                else:
                    self.set_expert(e, mat, a["codes"], a["scale"], a["zero"], a.get("A"), a.get("B"), a.get("rank"))

    # ---- workspace ----
    def workspace_bytes(self, T: int) -> int:
        return lib().moe_lrc_workspace_bytes(self._h, T)

    def workspace(self, T: int):
        import torch
        need = self.workspace_bytes(T)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
        return self._ws

    # ---- hot path (torch CUDA tensors in, torch CUDA tensors out) ----
    def route(self, x):
        import torch
        T, k = x.shape[0], self.cfg.top_k
        idx = torch.empty((T, k), dtype=torch.int32, device=x.device)
        w = torch.empty((T, k), dtype=torch.float32, device=x.device)
        _check(lib().moe_lrc_route(self._h, x.data_ptr(), T, idx.data_ptr(), w.data_ptr(), _stream()))
        return idx, w

    def permute(self, topk_idx):
        import torch
        T, k, E = topk_idx.shape[0], self.cfg.top_k, self.cfg.n_experts
        dev = topk_idx.device
        counts = torch.empty(E, dtype=torch.int32, device=dev)
        offsets = torch.empty(E + 1, dtype=torch.int32, device=dev)
        row_pair = torch.empty(T * k, dtype=torch.int32, device=dev)
        pair_row = torch.empty(T * k, dtype=torch.int32, device=dev)
        comp = torch.empty(E, dtype=torch.int32, device=dev)
        _check(lib().moe_lrc_permute(self._h, topk_idx.data_ptr(), T, counts.data_ptr(), offsets.data_ptr(),
                                     row_pair.data_ptr(), pair_row.data_ptr(), comp.data_ptr(), _stream()))
        return counts, offsets, row_pair, pair_row, comp

    def expert_ffn(self, x, offsets, row_pair):
        import torch
        T = x.shape[0]
        y = torch.empty((T * self.cfg.top_k, self.cfg.hidden), dtype=torch.bfloat16, device=x.device)
        ws = self.workspace(T)
        _check(lib().moe_lrc_expert_ffn(self._h, x.data_ptr(), T, offsets.data_ptr(), row_pair.data_ptr(),
                                        y.data_ptr(), ws.data_ptr(), ws.numel(), _stream()))
        return y

    def combine(self, y_rows, topk_w, pair_row, x):
        import torch
        T = x.shape[0]
        out = torch.empty((T, self.cfg.hidden), dtype=torch.bfloat16, device=x.device)
        ws = self.workspace(T)
        _check(lib().moe_lrc_combine(self._h, y_rows.data_ptr(), topk_w.data_ptr(), pair_row.data_ptr(),
                                     x.data_ptr(), T, out.data_ptr(), ws.data_ptr(), ws.numel(), _stream()))
        return out

    def forward(self, x, out=None):
        import torch
        T = x.shape[0]
        if out is None:
            out = torch.empty((T, self.cfg.hidden), dtype=torch.bfloat16, device=x.device)
        ws = self.workspace(T)
        _check(lib().moe_lrc_forward(self._h, x.data_ptr(), T, out.data_ptr(), ws.data_ptr(), ws.numel(), _stream()))
        return out

    def forward_noalloc(self, x, out) -> None:
        """moe_lrc_forward_noalloc: the workspace is the library's built-in device array."""
        _check(lib().moe_lrc_forward_noalloc(self._h, x.data_ptr(), x.shape[0], out.data_ptr(), _stream()))

    def forward_raw(self, x_ptr: int, T: int, out_ptr: int, ws_ptr: int, ws_bytes: int, stream: int) -> None:
        _check(lib().moe_lrc_forward(self._h, x_ptr, T, out_ptr, ws_ptr, ws_bytes, stream))

    # ---- hooks ----
    def debug_unpack(self, expert: int, mat: int):
        import torch
        K, N = (self.cfg.ffn, self.cfg.hidden) if mat == 2 else (self.cfg.hidden, self.cfg.ffn)
        codes = torch.empty((K, N), dtype=torch.uint8, device="cuda")
        _check(lib().moe_lrc_debug_unpack(self._h, expert, mat, codes.data_ptr(), _stream()))
        return codes

    def profile_enable(self, on: bool = True) -> None:
        _check(lib().moe_lrc_profile_enable(self._h, int(on)))

    def profile_read(self) -> dict:
        ms = (C.c_float * len(STAGES))()
        _check(lib().moe_lrc_profile_read(self._h, ms))
        return dict(zip(STAGES, list(ms)))

    def stats(self) -> dict:
        s = Stats()
        _check(lib().moe_lrc_get_stats(self._h, C.byref(s)))
        return {n: getattr(s, n) for n, _ in Stats._fields_}


# ---- offline pipeline (device tensors in, device tensors out) ---------------------------------
def offline_quantize(W, bits: int, group: int, want_residual: bool = True, refine: Optional[dict] = None):
    """moe_lrc_offline_quantize: W [K][N] torch.float64 on the device -> (codes uint8 [K][N],
    scale, zero as int16 views of fp16 bits [K/group][N], residual float64 [K][N] or None).
    refine = {"iters", "p", "beta", "kappa"} (any subset): moe_lrc_offline_quantize_refined."""
    import torch
    K, N = W.shape
    codes = torch.empty((K, N), dtype=torch.uint8, device=W.device)
    scale = torch.empty((K // group, N), dtype=torch.int16, device=W.device)
    zero = torch.empty((K // group, N), dtype=torch.int16, device=W.device)
    resid = torch.empty((K, N), dtype=torch.float64, device=W.device) if want_residual else None
    rp = resid.data_ptr() if want_residual else None
    if refine is None:
        _check(lib().moe_lrc_offline_quantize(W.data_ptr(), K, N, bits, group, codes.data_ptr(), scale.data_ptr(),
                                              zero.data_ptr(), rp, _stream()))
    else:
        _check(lib().moe_lrc_offline_quantize_refined(W.data_ptr(), K, N, bits, group, int(refine.get("iters", 20)),
                                                      float(refine.get("p", 0.7)), float(refine.get("beta", 10.0)),
                                                      float(refine.get("kappa", 1.01)), codes.data_ptr(), scale.data_ptr(),
                                                      zero.data_ptr(), rp, _stream()))
    return codes, scale, zero, resid


def offline_factors(E, rank: int, omega, power_iters: int = 2):
    """moe_lrc_offline_factors: E [K][N], omega [N][l] torch.float64 on the device ->
    (A [K][rank], B [rank][N] float64, sigma numpy [rank], A, B as int16 views of bf16 bits)."""
    import torch
    K, N = E.shape
    l = omega.shape[1]
    torch.cuda.synchronize()
    A = torch.empty((K, rank), dtype=torch.float64, device=E.device)
    B = torch.empty((rank, N), dtype=torch.float64, device=E.device)
    Ab = torch.empty((K, rank), dtype=torch.int16, device=E.device)
    Bb = torch.empty((rank, N), dtype=torch.int16, device=E.device)
    sigma = np.zeros(rank, dtype=np.float64)
    _check(lib().moe_lrc_offline_factors(E.data_ptr(), K, N, rank, omega.data_ptr(), l, power_iters, A.data_ptr(),
                                         B.data_ptr(), _hp(sigma), Ab.data_ptr(), Bb.data_ptr()))
    return A, B, sigma, Ab, Bb


def offline_kurtosis(W) -> float:
    import torch
    torch.cuda.synchronize()
    out = C.c_double(0.0)
    _check(lib().moe_lrc_offline_kurtosis(W.data_ptr(), W.numel(), C.byref(out)))
    return out.value


def allocate_ranks(kappas, r_avg: int, buckets=(0, 16, 32, 128, 256, 512, 1024)) -> np.ndarray:
    """moe_lrc_offline_allocate_ranks (host only)."""
    k = _host(np.asarray(kappas, dtype=np.float64).ravel(), np.float64)
    bk = _host(np.asarray(buckets), np.int32)
    out = np.zeros(k.size, dtype=np.int32)
    _check(lib().moe_lrc_offline_allocate_ranks(_hp(k), k.size, int(r_avg), _hp(bk), bk.size, _hp(out)))
    return out


def f64_to_f16_bits(a: np.ndarray) -> np.ndarray:
    """moe_lrc_selftest_half_rounding (host only)."""
    a = _host(a, np.float64).ravel()
    out = np.empty(a.size, dtype=np.uint16)
    _check(lib().moe_lrc_selftest_half_rounding(_hp(a), a.size, _hp(out)))
    return out


class Stack:
    """moe_lrc_stack: layers of residency POOLED decoding from host-resident experts through one
    device slot pool.  Keeps the Layer objects alive; closes before them."""

    def __init__(self, layers, slots: int, prefetch: bool = True, residual: bool = True):
        self.layers = list(layers)
        arr = (C.c_void_p * len(self.layers))(*[l._h for l in self.layers])
        self._h = C.c_void_p()
        flags = (STACK_PREFETCH if prefetch else 0) | (STACK_RESIDUAL if residual else 0)
        _check(lib().moe_lrc_stack_create(arr, len(self.layers), int(slots), flags, C.byref(self._h)))

    def close(self) -> None:
        if self._h:
            lib().moe_lrc_stack_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def step(self, x, out=None, layer_inputs=None):
        """x [T][hidden] bf16 (device).  layer_inputs: optional [n_layers][T][hidden] bf16 tensor that
        receives every layer's input."""
        import torch
        T = x.shape[0]
        if out is None:
            out = torch.empty_like(x)
        li = layer_inputs.data_ptr() if layer_inputs is not None else None
        _check(lib().moe_lrc_stack_step(self._h, x.data_ptr(), T, out.data_ptr(), li, _stream()))
        return out

    def stats(self) -> dict:
        s = StackStats()
        _check(lib().moe_lrc_stack_get_stats(self._h, C.byref(s)))
        return {n: getattr(s, n) for n, _ in StackStats._fields_}

    def reset(self) -> None:
        _check(lib().moe_lrc_stack_reset(self._h))


def bf16_tensor(bits: np.ndarray, device="cuda"):
    """uint16 bf16 bit patterns -> torch.bfloat16 tensor on `device` (a reinterpretation, no arithmetic)."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(device)

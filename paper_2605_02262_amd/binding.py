"""Thin ctypes binding over libwq.so: argument marshalling only.

PyTorch is used for device memory (``torch.empty(..., device="cuda")``, ``.data_ptr()``) and for the current
stream; every step of the path runs in the library's kernels.  Loading fails loudly when the library has
not been built (``python -m paper_2605_02262_amd.build``): there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

F32, BF16, F16 = 0, 1, 2
SCORE_AUTO, SCORE_PAIRWISE_MFMA, SCORE_POOLED = 0, 1, 2
MODE_QUOTA, MODE_THRESHOLD = 0, 1
DECODE_AUTO, DECODE_GENERIC, DECODE_MFMA = 0, 1, 2
DECODE_PARTIALS_ONLY = 0x100
DECODE_FIXED_SHARES = 0x200
DECODE_BY_LENGTH = 0x400
DECODE_SEPARATE_MERGE = 0x800
CLASS_BITS = (2, 4, 8)
DEV_CLASS_OVERFLOW, DEV_SEG16_OVERFLOW, DEV_APPEND_TIMEOUT, DEV_TOO_MANY_WINDOWS, DEV_BAD_ASSIGNMENT = 1, 2, 4, 16, 32

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libwq.so")
_lib = None


class WQError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"wq error {code}: {msg}")
        self.code = code


class _PackedKV(C.Structure):
    _fields_ = [("B", C.c_int32), ("Hkv", C.c_int32), ("hd", C.c_int32), ("group", C.c_int32),
                ("dtype16", C.c_int32), ("reserved", C.c_int32),
                ("codes", C.c_void_p * 3), ("meta", C.c_void_p * 3), ("cap", C.c_int64 * 3),
                ("cls_off", C.c_void_p * 3), ("cls_len", C.c_void_p * 3),
                ("k16", C.c_void_p), ("v16", C.c_void_p), ("cap16", C.c_int64),
                ("off16", C.c_void_p), ("len16", C.c_void_p), ("v_scale_max", C.c_void_p)]


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2605_02262_amd.build`")
        L = C.CDLL(_LIB_PATH)
        vp, i32, i64, f32 = C.c_void_p, C.c_int, C.c_int64, C.c_float
        L.wq_create.argtypes = [C.POINTER(vp), vp, vp, C.c_size_t]
        L.wq_destroy.argtypes = [vp]
        L.wq_set_stream.argtypes = [vp, vp]
        L.wq_last_error.argtypes = [vp]
        L.wq_last_error.restype = C.c_char_p
        L.wq_device_status.argtypes = [vp, C.POINTER(C.c_uint32)]
        L.wq_v_scale_floats.argtypes = [i32, i32, C.POINTER(C.c_int64)]
        L.wq_v_scale_floats.restype = C.c_size_t
        L.wq_workspace_bytes.argtypes = [i32, i32, i32, i32, i64, i64, i32]
        L.wq_workspace_bytes.restype = C.c_size_t
        L.wq_packed_bytes.argtypes = [i32, i64, i32, i32, i32, C.POINTER(C.c_size_t)]
        L.wq_packed_bytes.restype = C.c_size_t
        L.wq_auto_splits.argtypes = [i32, i32, i64]
        L.wq_auto_splits_ragged.argtypes = [i32, i32, i64, i64]
        L.wq_window_scores.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, i64, i64, i64, i32, vp]
        L.wq_assign_bits.argtypes = [vp, vp, i32, vp, i32, i32, vp, vp, i32, i32, vp, vp, vp]
        L.wq_layer_thresholds.argtypes = [C.POINTER(C.c_double), i32, C.c_double, C.POINTER(C.c_float), C.POINTER(C.c_float)]
        L.wq_vote_bits.argtypes = [vp, vp, i32, vp, i32, vp, vp, vp]
        L.wq_validate_assignment.argtypes = [vp, i32, vp, i32, vp, vp]
        L.wq_reorder_quantize.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, i64, C.POINTER(_PackedKV)]
        L.wq_append_kv.argtypes = [vp, vp, vp, i32, i32, C.POINTER(_PackedKV)]
        L.wq_dequantize.argtypes = [vp, i32, C.POINTER(_PackedKV), C.POINTER(_PackedKV)]
        L.wq_decode_append_attention.argtypes = [vp, vp, i32, i32, i32, C.POINTER(_PackedKV), vp, vp, i32, f32, i32, i64, i32, vp, vp]
        L.wq_decode_attention.argtypes = [vp, vp, i32, i32, i32, C.POINTER(_PackedKV), f32, i32, i64, i32, vp, vp]
        L.wq_decode_attention_static.argtypes = [vp, vp, i32, i32, i32, C.POINTER(_PackedKV), f32, i32, i64, i32, vp, vp]
        L.wq_static_last_error.argtypes = []
        L.wq_static_last_error.restype = C.c_char_p
        L.wq_probe_stream.argtypes = [vp, vp, vp, i64, i32]
        L.wq_probe_mfma.argtypes = [vp, i32, i32, i32, C.POINTER(C.c_double)]
        L.wq_decode_timing.argtypes = [vp, i32]
        L.wq_decode_times_us.argtypes = [vp, C.POINTER(C.c_float), i32]
        _lib = L
    return _lib


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    return t.data_ptr() if t.numel() > 0 else None


def _dtype_id(t: torch.Tensor) -> int:
    return {torch.float32: F32, torch.bfloat16: BF16, torch.float16: F16}[t.dtype]


def workspace_bytes(B=0, Hq=0, hd=0, max_splits=0, total_vis=0, total_txt=0, D=0) -> int:
    return int(lib().wq_workspace_bytes(B, Hq, hd, max_splits, total_vis, total_txt, D))


def packed_bytes(bits: int, cap_tokens: int, Hkv: int, hd: int, group: int):
    mb = C.c_size_t(0)
    cb = lib().wq_packed_bytes(bits, cap_tokens, Hkv, hd, group, C.byref(mb))
    return int(cb), int(mb.value)


def auto_splits(B: int, Hkv: int, max_seq_tokens: int) -> int:
    return int(lib().wq_auto_splits(B, Hkv, max_seq_tokens))


def auto_splits_ragged(B: int, Hkv: int, max_seq_tokens: int, total_tokens: int) -> int:
    return int(lib().wq_auto_splits_ragged(B, Hkv, max_seq_tokens, total_tokens))


class Context:
    """wq_ctx plus the torch tensor that backs its workspace (first 256 bytes zero = clean status word)."""

    def __init__(self, workspace_bytes_: int, device: str = "cuda", stream: Optional[torch.cuda.Stream] = None):
        self.device = torch.device(device)
        self.ws = torch.zeros(max(int(workspace_bytes_), 16384), dtype=torch.uint8, device=self.device)
        self.handle = C.c_void_p()
        st = (stream or torch.cuda.current_stream(self.device)).cuda_stream
        rc = lib().wq_create(C.byref(self.handle), C.c_void_p(st), self.ws.data_ptr(), self.ws.numel())
        if rc != 0:
            raise WQError(rc, "wq_create failed")

    def set_stream(self, stream: torch.cuda.Stream):
        lib().wq_set_stream(self.handle, C.c_void_p(stream.cuda_stream))

    def check(self, rc: int):
        if rc != 0:
            raise WQError(rc, lib().wq_last_error(self.handle).decode())

    def decode_timing(self, enable: bool = True):
        self.check(lib().wq_decode_timing(self.handle, 1 if enable else 0))

    def decode_times_us(self, n: int):
        buf = (C.c_float * n)()
        self.check(lib().wq_decode_times_us(self.handle, buf, n))
        return [float(x) for x in buf]

    def device_status(self) -> int:
        bits = C.c_uint32(0)
        self.check(lib().wq_device_status(self.handle, C.byref(bits)))
        return int(bits.value)

    def __del__(self):
        try:
            if self.handle:
                lib().wq_destroy(self.handle)
                self.handle = C.c_void_p()
        except Exception:
            pass


class PackedKV:
    """Device buffers of one layer's packed cache plus the C descriptor that points at them."""

    def __init__(self, B: int, Hkv: int, hd: int, group: int, dtype16: torch.dtype, cap: Sequence[int], off16: Sequence[int],
                 device: str = "cuda", fill: Optional[int] = None):
        dev = torch.device(device)
        self.B, self.Hkv, self.hd, self.group = B, Hkv, hd, group
        self.cap = [(int(c) + 31) // 32 * 32 for c in cap]
        self.dtype16 = dtype16
        G = hd // group
        mk = (lambda *s, dtype: torch.empty(*s, dtype=dtype, device=dev)) if fill is None else \
             (lambda *s, dtype: torch.full(s, fill, dtype=dtype, device=dev))
        self.codes = [mk(2, Hkv, self.cap[c] * hd * b // 8, dtype=torch.uint8) for c, b in enumerate(CLASS_BITS)]
        self.meta = [mk(2, Hkv, self.cap[c] * G, dtype=torch.int32) for c in range(3)]
        self.cls_off = [torch.zeros(B + 1, dtype=torch.int32, device=dev) for _ in range(3)]
        self.cls_len = [torch.zeros(B, dtype=torch.int32, device=dev) for _ in range(3)]
        self.off16 = torch.as_tensor(list(off16), dtype=torch.int32).to(dev)
        assert self.off16.numel() == B + 1
        self.cap16 = int(off16[-1]) if len(off16) else 0
        self.k16 = torch.zeros(self.cap16, Hkv, hd, dtype=dtype16, device=dev)
        self.v16 = torch.zeros(self.cap16, Hkv, hd, dtype=dtype16, device=dev)
        self.len16 = torch.zeros(B, dtype=torch.int32, device=dev)
        n_vs = lib().wq_v_scale_floats(B, Hkv, (C.c_int64 * 3)(*[int(c) for c in self.cap]))
        self.v_scale_max = torch.zeros(n_vs, dtype=torch.float32, device=dev)
        d = _PackedKV()
        d.B, d.Hkv, d.hd, d.group = B, Hkv, hd, group
        d.dtype16 = _dtype_id(self.k16)
        for c in range(3):
            d.codes[c] = _ptr(self.codes[c])
            d.meta[c] = _ptr(self.meta[c])
            d.cap[c] = self.cap[c]
            d.cls_off[c] = self.cls_off[c].data_ptr()
            d.cls_len[c] = _ptr(self.cls_len[c])
        d.k16, d.v16, d.cap16 = _ptr(self.k16), _ptr(self.v16), self.cap16
        d.off16, d.len16 = self.off16.data_ptr(), _ptr(self.len16)
        d.v_scale_max = _ptr(self.v_scale_max)
        self.desc = d

    def bytes_algorithmic(self) -> int:
        """Bytes a decode step has to read: codes + metadata of the real tokens and the 16-bit rows in use."""
        G = self.hd // self.group
        n = 0
        for c, b in enumerate(CLASS_BITS):
            t = int(self.cls_len[c].sum().item())
            n += t * self.Hkv * 2 * (self.hd * b // 8 + G * 4)
        n += int(self.len16.sum().item()) * self.Hkv * self.hd * 2 * 2
        return n


# ------------------------------------------------------------------------------------------------------------
# the four calls (same names as the C ABI)
# ------------------------------------------------------------------------------------------------------------
def wq_window_scores(ctx: Context, vis_emb, txt_emb, vis_off, txt_off, win_size, win_off, total_vis: int,
                     total_txt: int, total_win: int, algo: int = SCORE_AUTO, scores: Optional[torch.Tensor] = None):
    B = win_size.numel()
    D = vis_emb.shape[1] if vis_emb.numel() else txt_emb.shape[1]
    if scores is None:
        scores = torch.empty(total_win, dtype=torch.float32, device=ctx.device)
    ctx.check(lib().wq_window_scores(ctx.handle, _ptr(vis_emb), _ptr(txt_emb), _dtype_id(vis_emb), B, D, _ptr(vis_off),
                                     _ptr(txt_off), _ptr(win_size), _ptr(win_off), total_vis, total_txt, total_win, algo,
                                     _ptr(scores)))
    return scores


def wq_assign_bits(ctx: Context, scores, win_off, max_windows: int, mode: int = MODE_QUOTA, quota=None, thresholds=None,
                   top_bits: int = 8, pin_first: int = 1):
    B = win_off.numel() - 1
    W = scores.numel()
    bits = torch.empty(W, dtype=torch.uint8, device=ctx.device)
    perm = torch.empty(W, dtype=torch.int32, device=ctx.device)
    seg = torch.empty(B, 4, dtype=torch.int32, device=ctx.device)
    ctx.check(lib().wq_assign_bits(ctx.handle, _ptr(scores), B, _ptr(win_off), max_windows, mode, _ptr(quota),
                                   _ptr(thresholds), top_bits, pin_first, _ptr(bits), _ptr(perm), _ptr(seg)))
    return bits, perm, seg


def wq_layer_thresholds(s, alpha: float):
    """(T_low, T_high) per layer as fp32 lists (host-only call)."""
    n = len(s)
    sa = (C.c_double * n)(*[float(x) for x in s])
    lo, hi = (C.c_float * n)(), (C.c_float * n)()
    rc = lib().wq_layer_thresholds(sa, n, float(alpha), lo, hi)
    if rc != 0:
        raise WQError(rc, "wq_layer_thresholds: bad argument")
    return [float(x) for x in lo], [float(x) for x in hi]


def wq_vote_bits(ctx: Context, bits, win_off, max_windows: int):
    B = win_off.numel() - 1
    W = bits.numel()
    out = torch.empty(W, dtype=torch.uint8, device=ctx.device)
    perm = torch.empty(W, dtype=torch.int32, device=ctx.device)
    seg = torch.empty(B, 4, dtype=torch.int32, device=ctx.device)
    ctx.check(lib().wq_vote_bits(ctx.handle, _ptr(bits), B, _ptr(win_off), max_windows, _ptr(out), _ptr(perm), _ptr(seg)))
    return out, perm, seg


def wq_validate_assignment(ctx: Context, win_off, max_windows: int, perm, seg_windows):
    B = win_off.numel() - 1
    ctx.check(lib().wq_validate_assignment(ctx.handle, B, _ptr(win_off), max_windows, _ptr(perm), _ptr(seg_windows)))


def wq_reorder_quantize(ctx: Context, K, V, kv_off, win_size, win_off, perm, seg_windows, total_rows: int, out: PackedKV):
    B = win_size.numel()
    # a batch without any window has an empty perm: the library still wants a valid pointer (it cannot see the window
    # count on the host), which is never read then
    perm_ptr = _ptr(perm) if perm.numel() else _ptr(seg_windows)
    ctx.check(lib().wq_reorder_quantize(ctx.handle, _ptr(K), _ptr(V), _dtype_id(K), B, _ptr(kv_off), _ptr(win_size),
                                        _ptr(win_off), perm_ptr, _ptr(seg_windows), total_rows, C.byref(out.desc)))
    return out


def wq_append_kv(ctx: Context, k_new, v_new, kv: PackedKV):
    B = k_new.shape[0]
    ctx.check(lib().wq_append_kv(ctx.handle, _ptr(k_new), _ptr(v_new), _dtype_id(k_new), B, C.byref(kv.desc)))


def wq_decode_append_attention(ctx: Context, q, kv: PackedKV, k_new, v_new, sm_scale: float, num_splits: int = 0,
                               max_seq_tokens: int = 0, algo: int = DECODE_AUTO, out: Optional[torch.Tensor] = None,
                               lse: Optional[torch.Tensor] = None):
    B, Hq, hd = q.shape
    if out is None:
        out = torch.empty(B, Hq, hd, dtype=torch.float32, device=ctx.device)
    ctx.check(lib().wq_decode_append_attention(ctx.handle, _ptr(q), _dtype_id(q), B, Hq, C.byref(kv.desc), _ptr(k_new), _ptr(v_new),
                                               _dtype_id(k_new), sm_scale, num_splits, max_seq_tokens, algo, _ptr(out), _ptr(lse)))
    return out


def wq_dequantize(ctx: Context, src: PackedKV, dst: PackedKV):
    ctx.check(lib().wq_dequantize(ctx.handle, src.B, C.byref(src.desc), C.byref(dst.desc)))


def wq_decode_attention(ctx: Context, q, kv: PackedKV, sm_scale: float, num_splits: int = 0, max_seq_tokens: int = 0,
                        algo: int = DECODE_AUTO, out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None):
    B, Hq, hd = q.shape
    if out is None:
        out = torch.empty(B, Hq, hd, dtype=torch.float32, device=ctx.device)
    ctx.check(lib().wq_decode_attention(ctx.handle, _ptr(q), _dtype_id(q), B, Hq, C.byref(kv.desc), sm_scale, num_splits,
                                        max_seq_tokens, algo, _ptr(out), _ptr(lse)))
    return out


def wq_decode_attention_static(q, kv: PackedKV, sm_scale: float, num_splits: int = 0, max_seq_tokens: int = 0,
                               algo: int = DECODE_AUTO, out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                               stream: Optional[torch.cuda.Stream] = None):
    """wq_decode_attention without a context: the library's own static scratch array is the workspace."""
    B, Hq, hd = q.shape
    if out is None:
        out = torch.empty(B, Hq, hd, dtype=torch.float32, device=q.device)
    st = (stream or torch.cuda.current_stream(q.device)).cuda_stream
    rc = lib().wq_decode_attention_static(C.c_void_p(st), _ptr(q), _dtype_id(q), B, Hq, C.byref(kv.desc), sm_scale, num_splits,
                                          max_seq_tokens, algo, _ptr(out), _ptr(lse))
    if rc != 0:
        raise WQError(rc, lib().wq_static_last_error().decode())
    return out


def wq_probe_mfma(ctx: Context, random_operands: bool, workgroups: int = 2048, iters: int = 1000) -> float:
    """Launches the matrix-core rate probe; returns the floating-point operations of the launch."""
    fl = C.c_double(0.0)
    ctx.check(lib().wq_probe_mfma(ctx.handle, int(random_operands), workgroups, iters, C.byref(fl)))
    return fl.value


def wq_probe_stream(ctx: Context, src: torch.Tensor, dst: Optional[torch.Tensor] = None, blocks: int = 4096):
    nbytes = src.numel() * src.element_size() // 16 * 16
    ctx.check(lib().wq_probe_stream(ctx.handle, src.data_ptr(), None if dst is None else dst.data_ptr(), nbytes, blocks))
    return nbytes

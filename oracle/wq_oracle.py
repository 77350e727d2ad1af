"""ctypes front end of ``wq_oracle.c`` (test infrastructure, see that file's header).

Every function takes and returns numpy arrays; floating inputs are float32
arrays that hold the storage-type (bf16 / fp16 / fp32) values exactly.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import List, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "wq_oracle.c")
_LIB = os.path.join(_HERE, "libwq_oracle.so")
CLASS_BITS = (2, 4, 8)


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared",
                               "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.wqo_f16_bits_to_f64.restype = C.c_double
        _lib.wqo_f16_bits_to_f64.argtypes = [C.c_uint16]
        _lib.wqo_f32_to_f16_bits.restype = C.c_uint16
        _lib.wqo_f32_to_f16_bits.argtypes = [C.c_float]
        _lib.wqo_num_threads.restype = C.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def num_threads() -> int:
    return int(lib().wqo_num_threads())


def f32_to_f16_bits(x: float) -> int:
    return int(lib().wqo_f32_to_f16_bits(C.c_float(x)))


def f16_bits_to_f64(h: int) -> float:
    return float(lib().wqo_f16_bits_to_f64(C.c_uint16(h)))


# ----------------------------------------------------------------------------- O1
def window_scores(Ev, Et, vis_off, txt_off, win_size, win_off, form: str = "pooled") -> np.ndarray:
    Ev, Et = _f32(Ev), _f32(Et)
    D = Ev.shape[1] if Ev.size else Et.shape[1]
    vis_off, txt_off, win_size, win_off = map(_i32, (vis_off, txt_off, win_size, win_off))
    B = len(win_size)
    out = np.zeros(int(win_off[-1]), dtype=np.float64)
    fn = lib().wqo_scores_pairwise if form == "pairwise" else lib().wqo_scores_pooled
    fn(_p(Ev), _p(Et), C.c_int(D), C.c_int(B), _p(vis_off), _p(txt_off), _p(win_size), _p(win_off), _p(out))
    return out


# ----------------------------------------------------------------------------- O2
def assign_bits(scores, win_off, mode: int, quota=None, thresholds=None, top_bits: int = 8, pin_first: int = 1):
    scores = _f32(scores)
    win_off = _i32(win_off)
    B = len(win_off) - 1
    W = int(win_off[-1])
    quota = _i32(quota if quota is not None else np.zeros((B, 3)))
    thresholds = _f32(thresholds if thresholds is not None else np.zeros((B, 2)))
    bits = np.zeros(W, dtype=np.uint8)
    perm = np.zeros(W, dtype=np.int32)
    seg = np.zeros((B, 4), dtype=np.int32)
    lib().wqo_assign_bits(_p(scores), C.c_int(B), _p(win_off), C.c_int(mode), _p(quota), _p(thresholds),
                          C.c_int(top_bits), C.c_int(pin_first), _p(bits), _p(perm), _p(seg))
    return bits, perm, seg


def rank_by_counting(scores, first: int = 0) -> np.ndarray:
    s = _f32(scores)
    r = np.full(len(s), -1, dtype=np.int32)
    lib().wqo_rank_by_counting(_p(s), C.c_int(len(s)), C.c_int(first), _p(r))
    return r


def layer_thresholds(s, alpha: float):
    """Sec. 3.2.3 threshold functions, fp64, written out as printed:
    T_low = f1(s) = (e^{alpha s} - 1) / (e^alpha - 1),  T_high = f2(s) = (e^{-alpha s} - 1) / (e^{-alpha} - 1).
    alpha = 0 is the limit of both (the identity).  Pins: f(0) = 0, f(1) = 1, f1 <= f2 on [0, 1] (all stated by the
    paper), f1(s) + f2(1 - s) = 1, and f1(1/2) = 1 / (1 + e) at the paper's default alpha = 2."""
    s = np.asarray(s, dtype=np.float64)
    if alpha == 0.0:
        return s.copy(), s.copy()
    lo = (np.exp(alpha * s) - 1.0) / (np.exp(alpha) - 1.0)
    hi = (np.exp(-alpha * s) - 1.0) / (np.exp(-alpha) - 1.0)
    return lo, hi


def class_order(bits_seq) -> tuple:
    """Stable class order of one sequence's windows (Alg. 2 prefill loop: windows are appended to their class
    buffer in index order; classes are laid out 2-, 4-, 8-, 16-bit): (perm, counts)."""
    bits_seq = list(int(x) for x in bits_seq)
    perm = [i for width in (2, 4, 8, 16) for i, x in enumerate(bits_seq) if x == width]
    return np.asarray(perm, dtype=np.int32), np.asarray([bits_seq.count(w) for w in (2, 4, 8, 16)], dtype=np.int32)


def vote_bits(bits, win_off):
    """Batch-shared configuration (last paragraph of Sec. 3.2.3): for every window position the width that occurs
    most often among the requests that have that position is given to all of them.  The paper does not say what
    happens on a tie; the higher precision wins here.  Plain loops; returns (bits, perm, seg_windows)."""
    bits = np.asarray(bits, dtype=np.uint8)
    win_off = np.asarray(win_off, dtype=np.int64)
    B = len(win_off) - 1
    out = bits.copy()
    n_pos = int(np.diff(win_off).max()) if B else 0
    for p in range(n_pos):
        have = [b for b in range(B) if win_off[b + 1] - win_off[b] > p]
        votes = {}
        for b in have:
            w = int(bits[win_off[b] + p])
            votes[w] = votes.get(w, 0) + 1
        best = max(votes.items(), key=lambda kv: (kv[1], kv[0]))[0]      # most votes, then the wider
        for b in have:
            out[win_off[b] + p] = best
    perm = np.zeros(len(bits), dtype=np.int32)
    seg = np.zeros((B, 4), dtype=np.int32)
    for b in range(B):
        pb, cb = class_order(out[win_off[b]:win_off[b + 1]])
        perm[win_off[b]:win_off[b + 1]] = pb
        seg[b] = cb
    return out, perm, seg


# ----------------------------------------------------------------------------- O3
def quantize_group(x, bits: int):
    x = _f32(x)
    codes = np.zeros(len(x), dtype=np.uint8)
    s = C.c_uint16(0)
    m = C.c_uint16(0)
    lib().wqo_quantize_group(_p(x), C.c_int(len(x)), C.c_int(bits), _p(codes), C.byref(s), C.byref(m))
    return codes, int(s.value), int(m.value)


@dataclass
class PackedOracle:
    """Reordered, quantized cache in logical (unpacked) form plus the packed byte images."""
    B: int
    Hkv: int
    hd: int
    group: int
    cls_off: np.ndarray            # [3][B+1]
    cls_len: np.ndarray            # [3][B]
    cap: List[int]                 # tokens per class buffer (multiple of 32)
    src_row: List[np.ndarray]      # [cap_c] source row of each slot, -1 = padding
    codes: List[np.ndarray]        # [2][Hkv][cap_c][hd] uint8
    sbits: List[np.ndarray]        # [2][Hkv][cap_c][G] uint16
    mbits: List[np.ndarray]
    off16: np.ndarray              # [B]
    len16: np.ndarray              # [B]
    rows16: np.ndarray             # [cap16] source rows (-1 unused)
    k16: np.ndarray                # [cap16][Hkv][hd] float32 (16-bit values)
    v16: np.ndarray

    def packed_codes(self, c: int) -> np.ndarray:
        """Byte image [2][Hkv][cap_c*hd*b/8] of class c in the storage layout."""
        b = CLASS_BITS[c]
        cap, hd = self.cap[c], self.hd
        out = np.zeros((2, self.Hkv, cap * hd * b // 8), dtype=np.uint8)
        for pl in range(2):
            fn = lib().wqo_pack_k if pl == 0 else lib().wqo_pack_v
            for h in range(self.Hkv):
                src = np.ascontiguousarray(self.codes[c][pl, h])
                dst = np.zeros(cap * hd * b // 8, dtype=np.uint8)
                if cap:
                    fn(_p(src), C.c_int64(cap), C.c_int(hd), C.c_int(b), _p(dst))
                out[pl, h] = dst
        return out

    def packed_meta(self, c: int) -> np.ndarray:
        """Word image [2][Hkv][cap_c*G] uint32 of class c."""
        G = self.hd // self.group
        cap = self.cap[c]
        out = np.zeros((2, self.Hkv, cap * G), dtype=np.uint32)
        for pl in range(2):
            for h in range(self.Hkv):
                s = np.ascontiguousarray(self.sbits[c][pl, h])
                m = np.ascontiguousarray(self.mbits[c][pl, h])
                dst = np.zeros(cap * G, dtype=np.uint32)
                if cap:
                    lib().wqo_pack_meta(_p(s), _p(m), C.c_int64(cap), C.c_int(G), _p(dst))
                out[pl, h] = dst
        return out


def plan(kv_off, win_size, win_off, seg_windows):
    kv_off, win_size, win_off = map(_i32, (kv_off, win_size, win_off))
    seg = _i32(seg_windows)
    B = len(win_size)
    cls_off = np.zeros((3, B + 1), dtype=np.int32)
    cls_len = np.zeros((3, B), dtype=np.int32)
    len16 = np.zeros(B, dtype=np.int32)
    lib().wqo_plan(C.c_int(B), _p(kv_off), _p(win_size), _p(win_off), _p(seg), _p(cls_off), _p(cls_len), _p(len16))
    return cls_off, cls_len, len16


def reorder_quantize(K, V, kv_off, win_size, win_off, perm, seg_windows, group: int, off16=None,
                     cap: Optional[List[int]] = None, cap16: Optional[int] = None) -> PackedOracle:
    K, V = _f32(K), _f32(V)
    _, Hkv, hd = K.shape
    kv_off, win_size, win_off, perm = map(_i32, (kv_off, win_size, win_off, perm))
    seg = _i32(seg_windows)
    B = len(win_size)
    cls_off, cls_len, len16 = plan(kv_off, win_size, win_off, seg)
    if off16 is None:
        off16 = np.concatenate([[0], np.cumsum(len16)[:-1]]).astype(np.int32)
    off16 = _i32(off16)
    cap = [int(cls_off[c, B]) for c in range(3)] if cap is None else list(cap)
    cap16 = int((off16 + len16).max()) if cap16 is None and B else (cap16 or 0)
    # the C routines below trust these sizes (the GPU library reports an overflow instead): refuse what does not fit
    for c in range(3):
        if cap[c] < int(cls_off[c, B]):
            raise ValueError(f"class {CLASS_BITS[c]}-bit needs {int(cls_off[c, B])} token slots, cap is {cap[c]}")
    if B and int((off16 + len16).max()) > cap16:
        raise ValueError(f"the 16-bit segment needs {int((off16 + len16).max())} rows, cap16 is {cap16}")
    if B > 1 and np.any(off16[1:] < off16[:-1] + len16[:-1]):
        raise ValueError("16-bit segments overlap")
    src = [np.full(max(cap[c], 1), -1, dtype=np.int64) for c in range(3)]
    rows16 = np.full(max(cap16, 1), -1, dtype=np.int64)
    lib().wqo_gather_rows(C.c_int(B), _p(kv_off), _p(win_size), _p(win_off), _p(perm), _p(seg), _p(cls_off),
                          _p(off16), _p(src[0]), _p(src[1]), _p(src[2]), _p(rows16))
    G = hd // group
    codes, sb, mb = [], [], []
    for c in range(3):
        cc = np.zeros((2, Hkv, cap[c], hd), dtype=np.uint8)
        ss = np.zeros((2, Hkv, cap[c], G), dtype=np.uint16)
        mm = np.zeros((2, Hkv, cap[c], G), dtype=np.uint16)
        if cap[c]:
            for pl, X in enumerate((K, V)):
                lib().wqo_quantize_class(_p(X), C.c_int(Hkv), C.c_int(hd), C.c_int(group), C.c_int(CLASS_BITS[c]),
                                         C.c_int64(cap[c]), _p(src[c]), _p(cc[pl]), _p(ss[pl]), _p(mm[pl]))
        codes.append(cc)
        sb.append(ss)
        mb.append(mm)
    k16 = np.zeros((cap16, Hkv, hd), dtype=np.float32)
    v16 = np.zeros((cap16, Hkv, hd), dtype=np.float32)
    used = rows16[:cap16] >= 0
    k16[used] = K[rows16[:cap16][used]]
    v16[used] = V[rows16[:cap16][used]]
    return PackedOracle(B, Hkv, hd, group, cls_off, cls_len, cap, [s[:cap[c]] for c, s in enumerate(src)], codes,
                        sb, mb, off16, len16, rows16[:cap16], k16, v16)


# ----------------------------------------------------------------------------- O4
def decode_attention(q, pk: PackedOracle, sm_scale: float, Hq: Optional[int] = None, want_lse: bool = False):
    q = _f32(q)
    B, Hq, hd = q.shape
    out = np.zeros((B, Hq, hd), dtype=np.float64)
    lse = np.zeros((B, Hq), dtype=np.float64)
    args = [_p(q), C.c_int(B), C.c_int(Hq), C.c_int(pk.Hkv), C.c_int(hd), C.c_int(pk.group)]
    keep = []
    for c in range(3):
        arrs = [np.ascontiguousarray(pk.codes[c]), np.ascontiguousarray(pk.sbits[c]),
                np.ascontiguousarray(pk.mbits[c]), np.ascontiguousarray(pk.cls_off[c]),
                np.ascontiguousarray(pk.cls_len[c])]
        keep += arrs
        args += [_p(a) for a in arrs] + [C.c_int64(pk.cap[c])]
    k16, v16 = _f32(pk.k16), _f32(pk.v16)
    off16, len16 = _i32(pk.off16), _i32(pk.len16)
    args += [_p(k16), _p(v16), _p(off16), _p(len16), C.c_double(sm_scale), _p(out), _p(lse)]
    lib().wqo_decode_attention(*args)
    return (out, lse) if want_lse else out


def attention_dense(q, K, V, sm_scale: float) -> np.ndarray:
    """Textbook softmax(q K^T) V in fp64 on an explicit cache [T, Hkv, hd]; q [Hq, hd]."""
    q, K, V = _f32(q), _f32(K), _f32(V)
    Hq, hd = q.shape
    T, Hkv, _ = K.shape
    out = np.zeros((Hq, hd), dtype=np.float64)
    lib().wqo_attention_dense(_p(q), _p(K), _p(V), C.c_int(T), C.c_int(Hq), C.c_int(Hkv), C.c_int(hd),
                              C.c_double(sm_scale), _p(out))
    return out

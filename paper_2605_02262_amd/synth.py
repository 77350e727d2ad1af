"""Seeded synthetic workloads shaped like LLaVA-OneVision video requests.

This module only *draws inputs*: embeddings, keys/values, queries and the
descriptor tables of a batch.  It contains none of the method's arithmetic
(no scoring, ranking, quantization or attention) and is the one module that
both the GPU path's tests and the CPU oracle's tests are allowed to share.

Everything is drawn on the host with ``numpy.random.Generator(PCG64(seed))``
in a fixed order per sequence:

    text embedding -> alpha -> visual embedding -> channel scales -> K -> V -> q

Values are rounded to the run's storage type right away (bf16 / fp16 by
round-to-nearest-even, kept in float32 containers plus a uint16 bit image) so
that every consumer sees bit-identical numbers.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

F32, BF16, F16 = 0, 1, 2           # storage type ids, same numbering as the C ABI
CLASS_BITS = (2, 4, 8)             # class index c -> bit width
TOKEN_PAD = 32                     # class segments are padded to this many tokens


# --------------------------------------------------------------------------- #
# storage-type rounding (input preparation only)
# --------------------------------------------------------------------------- #
def round_bf16(x: np.ndarray) -> np.ndarray:
    """float32 -> nearest bf16 (ties to even), returned as float32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u.astype(np.uint64) + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint32) << 16
    return r.astype(np.uint32).view(np.float32).reshape(x.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 holding bf16-representable values -> uint16 bit image."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return (u >> 16).astype(np.uint16).reshape(x.shape)


def round_f16(x: np.ndarray) -> np.ndarray:
    return np.asarray(x, dtype=np.float32).astype(np.float16).astype(np.float32)


def f16_bits(x: np.ndarray) -> np.ndarray:
    return np.asarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)


def round_to(x: np.ndarray, dtype: int) -> np.ndarray:
    if dtype == BF16:
        return round_bf16(x)
    if dtype == F16:
        return round_f16(x)
    return np.asarray(x, dtype=np.float32)


def storage_bits(x: np.ndarray, dtype: int) -> np.ndarray:
    """Array in the byte image the device expects for ``dtype``."""
    if dtype == BF16:
        return bf16_bits(x)
    if dtype == F16:
        return f16_bits(x)
    return np.ascontiguousarray(x, dtype=np.float32)


# --------------------------------------------------------------------------- #
# workload description
# --------------------------------------------------------------------------- #
@dataclass
class SeqSpec:
    frames: int            # number of video frames
    tok_per_frame: int     # visual tokens per frame
    win_size: int          # S: tokens per window
    n_text: int            # text tokens (kept 16-bit)
    quota: tuple           # (n_top, n4, n2) windows
    tail: int = 0          # extra visual tokens that do not fill a window

    @property
    def n_vis(self) -> int:
        return self.frames * self.tok_per_frame + self.tail

    @property
    def n_win(self) -> int:
        return (self.frames * self.tok_per_frame + self.tail) // self.win_size


@dataclass
class Workload:
    name: str
    dtype: int             # storage type of embeddings, K, V, q
    dtype16: int           # storage type of the 16-bit segment
    Hq: int
    Hkv: int
    hd: int
    group: int
    D: int
    sigma_k: float
    seqs: List[SeqSpec]
    seed: int
    top_bits: int = 8
    pin_first: int = 1
    layers: int = 1
    logit_std: float = 2.0

    @property
    def B(self) -> int:
        return len(self.seqs)


def mix_to_quota(n_win: int, p8: int, p4: int) -> tuple:
    """Integer-only conversion of a percentage mix to window counts."""
    n8 = (p8 * n_win + 50) // 100
    c = ((p8 + p4) * n_win + 50) // 100
    return (n8, c - n8, n_win - c)


def workload(cfg: int, seed: Optional[int] = None) -> Workload:
    """The five configurations of the build's measurement plan, plus the paper's own operating point (5)."""
    if cfg == 0:
        s = SeqSpec(8, 16, 16, 16, mix_to_quota(8, 25, 50))
        return Workload("cfg0-tiny", F32, F16, 14, 2, 64, 32, 896, 1.0, [s], 0 if seed is None else seed)
    if cfg == 1:
        s = SeqSpec(32, 196, 196, 128, mix_to_quota(32, 25, 50))
        return Workload("cfg1-ov0.5b-layer", BF16, BF16, 14, 2, 64, 32, 896, 1.0, [s],
                        1000 if seed is None else seed)
    if cfg == 2:
        s = [SeqSpec(64, 196, 196, 256, mix_to_quota(64, 20, 50)) for _ in range(8)]
        return Workload("cfg2-ov7b-28layers", BF16, BF16, 28, 4, 128, 64, 3584, 1.5, s,
                        2000 if seed is None else seed, layers=28)
    if cfg == 3:
        s = [SeqSpec(256, 196, 196, 512, mix_to_quota(256, 10, 40)) for _ in range(4)]
        return Workload("cfg3-ov7b-longvideo", BF16, BF16, 28, 4, 128, 64, 3584, 1.5, s,
                        3000 if seed is None else seed)
    if cfg == 4:
        sd = 4000 if seed is None else seed
        rng = np.random.Generator(np.random.PCG64(sd + 77))
        seqs = []
        for b in range(32):
            frames = int(rng.integers(8, 129))
            S = int(rng.choice([98, 196]))
            n_win = frames * 196 // S
            share = rng.dirichlet([1.0, 1.0, 1.0])
            if b == 0:
                quota = (0, 0, n_win)
            elif b == 1:
                quota = (n_win, 0, 0)
            else:
                p8 = int(round(100 * share[0]))
                p4 = min(100 - p8, int(round(100 * share[1])))
                quota = mix_to_quota(n_win, p8, p4)
            seqs.append(SeqSpec(frames, 196, S, 256, quota))
        return Workload("cfg4-ragged", BF16, BF16, 28, 4, 128, 64, 3584, 1.5, seqs, sd, pin_first=0)
    if cfg == 5:
        # the paper's own operating point (Sec. 4.1 defaults, Sec. 4.3 token counts): batch 1, 100 frames, windows of
        # 32 tokens, top tier kept 16-bit.  19600 visual tokens = 612 windows + a tail of 16; 2 / 217 / 393 windows at
        # 16 / 4 / 2 bits and 135 text tokens give 215 / 6944 / 12576 tokens (the paper counts 215 / 6956 / 12564).
        s = SeqSpec(100, 196, 32, 135, (2, 217, 393))
        return Workload("cfg5-paper-tiers", BF16, BF16, 28, 4, 128, 64, 3584, 1.5, [s],
                        5000 if seed is None else seed, top_bits=16)
    raise ValueError(f"unknown config {cfg}")


# --------------------------------------------------------------------------- #
# descriptor tables
# --------------------------------------------------------------------------- #
@dataclass
class Tables:
    vis_off: np.ndarray     # [B+1] visual-token offsets (embedding rows)
    txt_off: np.ndarray     # [B+1] text-token offsets (embedding rows)
    kv_off: np.ndarray      # [B+1] offsets into K/V rows: visual tokens then text tokens
    win_size: np.ndarray    # [B]
    win_off: np.ndarray     # [B+1] window offsets
    quota: np.ndarray       # [B,3] (n_top, n4, n2)


def tables(w: Workload) -> Tables:
    nv = np.array([s.n_vis for s in w.seqs], dtype=np.int64)
    nt = np.array([s.n_text for s in w.seqs], dtype=np.int64)
    nw = np.array([s.n_win for s in w.seqs], dtype=np.int64)
    cs = lambda a: np.concatenate([[0], np.cumsum(a)]).astype(np.int32)
    return Tables(cs(nv), cs(nt), cs(nv + nt), np.array([s.win_size for s in w.seqs], dtype=np.int32),
                  cs(nw), np.array([s.quota for s in w.seqs], dtype=np.int32).reshape(-1, 3))


# --------------------------------------------------------------------------- #
# draws
# --------------------------------------------------------------------------- #
def _rng(w: Workload, b: int, layer: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([w.seed, layer, b, stream]))


def embeddings(w: Workload, b: int):
    """(E_t [N,D], E_v [M,D]) of sequence b, rounded to the run's storage type.

    Each window i draws alpha_i ~ U(0,1); its tokens are alpha_i * u + N(0, I),
    u being the unit vector along the mean text token.
    """
    s = w.seqs[b]
    rng = _rng(w, b, 0, 0)
    et = rng.standard_normal((s.n_text, w.D), dtype=np.float32)
    if s.n_text > 0:
        u = et.astype(np.float64).mean(axis=0)
        u = (u / np.linalg.norm(u)).astype(np.float32)
    else:
        u = np.zeros(w.D, dtype=np.float32)
    n_rows = s.n_vis
    alpha = rng.random(max(s.n_win, 1), dtype=np.float32)
    ev = rng.standard_normal((n_rows, w.D), dtype=np.float32)
    a_tok = np.zeros(n_rows, dtype=np.float32)
    a_tok[: s.n_win * s.win_size] = np.repeat(alpha[: s.n_win], s.win_size)
    ev += a_tok[:, None] * u[None, :]
    return round_to(et, w.dtype), round_to(ev, w.dtype)


def keys_values(w: Workload, b: int, layer: int = 0):
    """(K, V) [n_vis + n_text, Hkv, hd] float32 holding storage-type values.

    K = c[h,ch] * N(0,1) with c ~ lognormal(0, sigma_k) (channel outliers),
    V = N(0,1).  Rows past the windowed visual tokens (tail, text) are the ones
    the method keeps 16-bit; they are rounded to ``dtype16`` as well so that a
    16-bit copy of them is lossless.
    """
    s = w.seqs[b]
    rng = _rng(w, b, layer, 1)
    n = s.n_vis + s.n_text
    c = rng.lognormal(0.0, w.sigma_k, size=(w.Hkv, w.hd)).astype(np.float32)
    k = rng.standard_normal((n, w.Hkv, w.hd), dtype=np.float32) * c[None]
    v = rng.standard_normal((n, w.Hkv, w.hd), dtype=np.float32)
    k, v = round_to(k, w.dtype), round_to(v, w.dtype)
    if w.dtype == F32:          # the whole cache must survive a 16-bit copy exactly
        k, v = round_to(k, w.dtype16), round_to(v, w.dtype16)
    return k, v


def query(w: Workload, b: int, k: np.ndarray, layer: int = 0, step: int = 0) -> np.ndarray:
    """q [Hq, hd]: N(0,1), rescaled per head so the scaled logits over this
    sequence's (unquantized) keys have standard deviation ``logit_std``."""
    rng = _rng(w, b, layer, 2 + step)
    q = rng.standard_normal((w.Hq, w.hd), dtype=np.float32).astype(np.float64)
    rep = w.Hq // w.Hkv
    sm = 1.0 / np.sqrt(w.hd)
    k64 = k.astype(np.float64)
    for h in range(w.Hq):
        lg = (k64[:, h // rep, :] @ q[h]) * sm
        sd = lg.std()
        if sd > 0:
            q[h] *= w.logit_std / sd
    return round_to(q.astype(np.float32), w.dtype)


@dataclass
class Batch:
    w: Workload
    t: Tables
    E_t: np.ndarray
    E_v: np.ndarray
    K: np.ndarray
    V: np.ndarray
    q: np.ndarray           # [B, Hq, hd]
    layer: int = 0


def batch(w: Workload, layer: int = 0, with_embeddings: bool = True) -> Batch:
    """Draw a whole batch (all sequences) for one layer."""
    t = tables(w)
    ets, evs, ks, vs, qs = [], [], [], [], []
    for b in range(w.B):
        if with_embeddings:
            et, ev = embeddings(w, b)
            ets.append(et)
            evs.append(ev)
        k, v = keys_values(w, b, layer)
        ks.append(k)
        vs.append(v)
        qs.append(query(w, b, k, layer))
    cat = lambda xs, d: (np.concatenate(xs, axis=0) if xs else np.zeros((0, d), np.float32))
    return Batch(w, t, cat(ets, w.D), cat(evs, w.D), np.concatenate(ks), np.concatenate(vs),
                 np.stack(qs), layer)

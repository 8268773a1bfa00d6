"""Seeded synthetic inputs and the named workload shapes.

This module serves both the CPU oracle's tests and the GPU path's tests and
benchmark.  It holds NO arithmetic of the attention method: only shapes, random
draws, rotary position encoding of the inputs, and rounding to the storage
dtype.  Everything is numpy on the host; callers move the arrays where they
need them.

The shapes stand in for Self-Forcing / Wan 2.1 activations (Sec. 5, kernel
latency tables): 480p latent grid h=30, w=52 (1560 tokens per frame), 3-frame
autoregressive chunks, 21 latent frames for an 81-frame video, 12 heads of 128;
720p: h=45, w=80.  No model weights or datasets are used.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Tuple

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    heads: int
    head_dim: int
    f_q: int
    f_kv: int
    h: int
    w: int
    b1: int
    b2: int
    tile: int            # 0 regular Monarch, 1 tiled (b1,b2 are tile-local block sizes)
    iters: int           # T
    causal_chunk: int    # frames per autoregressive chunk, 0 = no mask
    q_frame_offset: int  # absolute frame of query frame 0 inside the kv grid
    dtype: str           # "f32" | "bf16"
    scale: float         # logits multiplier
    rope: bool
    sigma_qk: float = 1.0
    sigma_v: float = 1.0
    seed: int = 0
    assign: str = "fh_w"  # aligned block assignment (Sec. 4.1): axes of the b1 side _ axes of the b2 side
    tile_h: int = 0       # n_h > 0: neighbourhood tiles of (b1 / n_h) frames x n_h rows x b2 columns (Sec. 4.2)

    def block_grid(self):
        """(rows_q, rows_kv, cols) of the block grid under the assignment."""
        size = lambda axes, f: int(np.prod([{"f": f, "h": self.h, "w": self.w}[c] for c in axes]))
        ra, ca = self.assign.split("_")
        cols_q, cols_k = size(ca, self.f_q), size(ca, self.f_kv)
        assert cols_q == cols_k, "frame axis on the b2 side needs f_q == f_kv"
        return size(ra, self.f_q), size(ra, self.f_kv), cols_q

    @property
    def n_q(self) -> int:
        return self.f_q * self.h * self.w

    @property
    def n_kv(self) -> int:
        return self.f_kv * self.h * self.w

    @property
    def ntq(self) -> int:
        rq, _, cols = self.block_grid()
        return 1 if self.tile == 0 else (rq // self.b1) * (cols // self.b2)

    @property
    def ntk(self) -> int:
        _, rk, cols = self.block_grid()
        return 1 if self.tile == 0 else (rk // self.b1) * (cols // self.b2)


_INV_SQRT128 = 1.0 / np.sqrt(128.0)

WORKLOADS: Dict[str, Workload] = {
    # tiny regular Monarch, fp32; inputs already carry 1/sqrt(d)
    "C0": Workload("C0", 1, 1, 64, 1, 1, 24, 24, 24, 24, 0, 1, 0, 0, "f32", 1.0, False,
                   sigma_qk=1.0 / 8.0, sigma_v=1.0 / 8.0),
    # Self-Forcing chunk shape, regular Monarch (f*h, w)
    "C1": Workload("C1", 1, 12, 128, 3, 3, 30, 52, 90, 52, 0, 2, 0, 0, "bf16", _INV_SQRT128, True),
    # same tensors, tiled Monarch with tiles (90, 26)
    "C2": Workload("C2", 1, 12, 128, 3, 3, 30, 52, 90, 26, 1, 2, 0, 0, "bf16", _INV_SQRT128, True),
    # KV-cache step: last 3-frame chunk against a 21-frame cache
    "C3": Workload("C3", 1, 12, 128, 3, 21, 30, 52, 90, 26, 1, 2, 3, 18, "bf16", _INV_SQRT128, True),
    # 720p stress
    "C4": Workload("C4", 1, 40, 128, 3, 21, 45, 80, 135, 40, 1, 3, 3, 18, "bf16", _INV_SQRT128, True),
    # Shapes of the paper's kernel-latency table for Self-Forcing final-chunk decoding (Tab. 6):
    # 480p with tile blocks (3h, w) [density 3 %] and (h, w) [5 %], 720p likewise; the paper does
    # not state T or the precision for those rows, so these run T = 1 (its finetuned setting).
    "T6-480-3hw": Workload("T6-480-3hw", 1, 12, 128, 3, 21, 30, 52, 90, 52, 1, 1, 3, 18, "bf16", _INV_SQRT128, True),
    "T6-480-hw": Workload("T6-480-hw", 1, 12, 128, 3, 21, 30, 52, 30, 52, 1, 1, 3, 18, "bf16", _INV_SQRT128, True),
    "T6-720-3hw": Workload("T6-720-3hw", 1, 12, 128, 3, 21, 45, 80, 135, 80, 1, 1, 3, 18, "bf16", _INV_SQRT128, True),
    "T6-720-hw": Workload("T6-720-hw", 1, 12, 128, 3, 21, 45, 80, 45, 80, 1, 1, 3, 18, "bf16", _INV_SQRT128, True),
    # Shapes of the paper's Wan 2.1 kernel-latency table (Tab. 5): full bidirectional attention
    # over the 21-frame latent video, same tile blocks; T = 1.
    "T5-480-3hw": Workload("T5-480-3hw", 1, 12, 128, 21, 21, 30, 52, 90, 52, 1, 1, 0, 0, "bf16", _INV_SQRT128, True),
    "T5-480-hw": Workload("T5-480-hw", 1, 12, 128, 21, 21, 30, 52, 30, 52, 1, 1, 0, 0, "bf16", _INV_SQRT128, True),
    "T5-720-3hw": Workload("T5-720-3hw", 1, 12, 128, 21, 21, 45, 80, 135, 80, 1, 1, 0, 0, "bf16", _INV_SQRT128, True),
    "T5-720-hw": Workload("T5-720-hw", 1, 12, 128, 21, 21, 45, 80, 45, 80, 1, 1, 0, 0, "bf16", _INV_SQRT128, True),
    # The whole 21-frame sequence under the block-causal mask (chunks of 3 frames), the shape a
    # training step of the autoregressive model runs (forward and backward): query tile row a sees
    # the key tile rows of chunks 0 .. a, so the stage L problems differ sevenfold in length.
    "BC-480-3hw": Workload("BC-480-3hw", 1, 12, 128, 21, 21, 30, 52, 90, 52, 1, 1, 3, 0, "bf16", _INV_SQRT128, True),
    # C1's tensors under the other aligned block assignments that fit the kernels' block limits
    # (Sec. 4.1): (w, fh) = (52, 90) and (fw, h) = (156, 30), regular Monarch, T = 2
    "C1-w_fh": Workload("C1-w_fh", 1, 12, 128, 3, 3, 30, 52, 52, 90, 0, 2, 0, 0, "bf16", _INV_SQRT128, True,
                        assign="w_fh"),
    "C1-fw_h": Workload("C1-fw_h", 1, 12, 128, 3, 3, 30, 52, 156, 30, 0, 2, 0, 0, "bf16", _INV_SQRT128, True,
                        assign="fw_h"),
    # KV-cache step with (frame, width) rows: tiles of one frame (52 rows) by 30 columns, chunk-causal
    "C3-fw_h": Workload("C3-fw_h", 1, 12, 128, 3, 21, 30, 52, 52, 30, 1, 2, 3, 18, "bf16", _INV_SQRT128, True,
                        assign="fw_h"),
    # neighbourhood tiles of half a frame: (n_f, n_h, n_w) = (1, 15, 26)
    "C3-half": Workload("C3-half", 1, 12, 128, 3, 21, 30, 52, 15, 26, 1, 2, 3, 18, "bf16", _INV_SQRT128, True),
    # neighbourhood tiles of 3 frames x 15 rows x 26 columns: (n_f, n_h, n_w) = (3, 15, 26), b1 = 45
    "C3-nbh": Workload("C3-nbh", 1, 12, 128, 3, 21, 30, 52, 45, 26, 1, 2, 3, 18, "bf16", _INV_SQRT128, True,
                       tile_h=15),
}


def variant(name: str, **kw) -> Workload:
    return replace(WORKLOADS[name], **kw)


# --------------------------------------------------------------------------
# storage rounding
# --------------------------------------------------------------------------
def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 -> nearest-even bfloat16, returned as fp32 holding exactly those values."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 values that are exactly representable in bf16 -> uint16 bit patterns."""
    return (np.ascontiguousarray(x, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)


# --------------------------------------------------------------------------
# 3-D rotary position encoding of the inputs (input generation only)
# --------------------------------------------------------------------------
def rope_pairs_split(head_dim: int) -> Tuple[int, int, int]:
    """Rotary pairs assigned to (frame, height, width); 64 pairs -> (22, 21, 21)."""
    pairs = head_dim // 2
    ph = pw = pairs // 3
    return pairs - ph - pw, ph, pw


def rope_angles(frames: np.ndarray, h: int, w: int, head_dim: int,
                theta: float = 10000.0) -> np.ndarray:
    """angles[token, pair] for tokens in row-major (frame, height, width) order;
    `frames` holds the absolute frame index of each frame of the grid."""
    pf, ph, pw = rope_pairs_split(head_dim)
    fr = np.repeat(np.asarray(frames, dtype=np.float64), h * w)
    hh = np.tile(np.repeat(np.arange(h, dtype=np.float64), w), len(frames))
    ww = np.tile(np.arange(w, dtype=np.float64), len(frames) * h)
    def freqs(n):
        return theta ** (-np.arange(n, dtype=np.float64) / n)
    return np.concatenate([fr[:, None] * freqs(pf)[None], hh[:, None] * freqs(ph)[None],
                           ww[:, None] * freqs(pw)[None]], axis=1)


def rope_tables(ang: np.ndarray):
    """(cos, sin) of the angles as fp32, the form apply_rope multiplies with."""
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def apply_rope(x: np.ndarray, ang: np.ndarray, tables=None) -> np.ndarray:
    """Rotate adjacent element pairs (2p, 2p+1) of x[..., token, d] by ang[token, p]
    (tables: rope_tables(ang) computed beforehand, to share them between heads)."""
    c, s = rope_tables(ang) if tables is None else tables
    xe, xo = x[..., 0::2], x[..., 1::2]
    out = np.empty_like(x)
    out[..., 0::2] = xe * c - xo * s
    out[..., 1::2] = xe * s + xo * c
    return out


# --------------------------------------------------------------------------
# generators
# --------------------------------------------------------------------------
def _draw(wl: Workload, tensor_id: int, b: int, hd: int, n: int, sigma: float) -> np.ndarray:
    rng = np.random.default_rng((wl.seed, tensor_id, b, hd))
    return (sigma * rng.standard_normal((n, wl.head_dim), dtype=np.float32)).astype(np.float32)


def _rope_tables_qk(wl: Workload):
    tq = rope_tables(rope_angles(wl.q_frame_offset + np.arange(wl.f_q), wl.h, wl.w, wl.head_dim))
    tk = rope_tables(rope_angles(np.arange(wl.f_kv), wl.h, wl.w, wl.head_dim))
    return tq, tk


def make_head(wl: Workload, b: int, hd: int, tables=None):
    """Q [n_q,d], K,V [n_kv,d] of one (batch, head) as fp32 arrays whose values are
    exactly representable in the workload's storage dtype.  Heads are drawn from
    independent streams keyed by (seed, tensor, batch, head), so any head can be
    regenerated alone.  tables: the rotary (cos, sin) tables of the query and key grids, if the
    caller already has them (they are the same for every head)."""
    Q = _draw(wl, 0, b, hd, wl.n_q, wl.sigma_qk)
    K = _draw(wl, 1, b, hd, wl.n_kv, wl.sigma_qk)
    V = _draw(wl, 2, b, hd, wl.n_kv, wl.sigma_v)
    if wl.rope:
        tq, tk = _rope_tables_qk(wl) if tables is None else tables
        Q = apply_rope(Q, None, tq)
        K = apply_rope(K, None, tk)
    if wl.dtype == "bf16":
        Q, K, V = round_to_bf16(Q), round_to_bf16(K), round_to_bf16(V)
    return Q, K, V


def make_inputs(wl: Workload):
    """All heads: Q [batch, heads, n_q, d], K, V [batch, heads, n_kv, d] (fp32 arrays
    holding storage-dtype-exact values).  Heads are generated by a few threads (every head has its
    own random stream, so the values do not depend on the schedule)."""
    from concurrent.futures import ThreadPoolExecutor
    Q = np.empty((wl.batch, wl.heads, wl.n_q, wl.head_dim), np.float32)
    K = np.empty((wl.batch, wl.heads, wl.n_kv, wl.head_dim), np.float32)
    V = np.empty_like(K)
    tables = _rope_tables_qk(wl) if wl.rope else None

    def one(bh):
        b, hd = divmod(bh, wl.heads)
        Q[b, hd], K[b, hd], V[b, hd] = make_head(wl, b, hd, tables)

    n = wl.batch * wl.heads
    if n == 1:
        one(0)
    else:
        with ThreadPoolExecutor(max_workers=min(8, n)) as pool:
            list(pool.map(one, range(n)))
    return Q, K, V


def make_separable_head(wl: Workload, b: int, hd: int):
    """Position-only inputs: one constant content vector per tensor, rotated by the
    3-D rotary encoding.  The logit between two tokens is then a sum of a
    (frame,height) term and a width term, which an aligned (f*h, w) Monarch
    structure represents exactly (Sec. 4.1), so MonarchRT must equal dense
    attention on them.  Values are NOT rounded to bf16 exactly separable any more
    after storage rounding, so callers compare with a tolerance."""
    rng = np.random.default_rng((wl.seed, 7, b, hd))
    q0 = rng.standard_normal(wl.head_dim).astype(np.float32)
    k0 = rng.standard_normal(wl.head_dim).astype(np.float32)
    Q = np.broadcast_to(q0, (wl.n_q, wl.head_dim)).copy()
    K = np.broadcast_to(k0, (wl.n_kv, wl.head_dim)).copy()
    V = _draw(wl, 2, b, hd, wl.n_kv, 1.0)
    Q = apply_rope(Q, rope_angles(wl.q_frame_offset + np.arange(wl.f_q), wl.h, wl.w, wl.head_dim))
    K = apply_rope(K, rope_angles(np.arange(wl.f_kv), wl.h, wl.w, wl.head_dim))
    if wl.dtype == "bf16":
        Q, K, V = round_to_bf16(Q), round_to_bf16(K), round_to_bf16(V)
    return Q, K, V


def make_structured_head(wl: Workload, b: int, hd: int, n_semantic: int = 8, strength: float = 4.0,
                         noise: float = 0.25):
    """Inputs whose attention map follows the paper's informal model (Sec. 3.1): a separable
    positional part (one content vector under the 3-D rotary encoding), a sparse semantic part
    (n_semantic keys that a random 2 % of the queries match whatever their position: a shared
    direction added to those rows after the rotation) and noise (independent N(0, noise^2)
    content added to every row).  V ~ N(0,1).  Values are rounded to the storage type."""
    rng = np.random.default_rng((wl.seed, 11, b, hd))
    d = wl.head_dim
    q0 = rng.standard_normal(d).astype(np.float32)
    k0 = rng.standard_normal(d).astype(np.float32)
    Q = np.broadcast_to(q0, (wl.n_q, d)).copy()
    K = np.broadcast_to(k0, (wl.n_kv, d)).copy()
    Q = apply_rope(Q, rope_angles(wl.q_frame_offset + np.arange(wl.f_q), wl.h, wl.w, d))
    K = apply_rope(K, rope_angles(np.arange(wl.f_kv), wl.h, wl.w, d))
    for _ in range(n_semantic):
        u = rng.standard_normal(d).astype(np.float32)
        u *= strength / np.linalg.norm(u)
        key = int(rng.integers(wl.n_kv))
        queries = rng.choice(wl.n_q, size=max(1, wl.n_q // 50), replace=False)
        K[key] += u
        Q[queries] += u
    Q += noise * rng.standard_normal(Q.shape).astype(np.float32)
    K += noise * rng.standard_normal(K.shape).astype(np.float32)
    V = rng.standard_normal((wl.n_kv, d)).astype(np.float32)
    if wl.dtype == "bf16":
        Q, K, V = round_to_bf16(Q), round_to_bf16(K), round_to_bf16(V)
    return Q, K, V

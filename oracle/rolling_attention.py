"""fp64 CPU oracle for rolling-cache chunk attention.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package.  It shares no code with the HIP path and never calls it.

What it computes follows the paper's statement of the streaming scheme:

* Sec. 3.2 "Rolling KV Cache with Frame Sinks": the context of a new chunk is
  the first S frames of the stream (sinks, kept for ever) plus the most recent
  frames of a rolling window; the model attends only to that context.
* Sec. 3.1 / Related Work: the generator is a block-causal transformer that
  conditions each new chunk on the KV cache of the preceding frames.
* Sec. 3.3 "Streaming Long Tuning": in the update the cache of the preceding
  frames is detached and gradients flow through the active window only.

The rolling cache is an exact reformulation of softmax attention over the
visible set, so the oracle is the plain definition: it keeps the WHOLE history
of every stream and masks out the frames the ring would have evicted; no ring,
no tiling, no online softmax.  numpy matmul serves as the contraction step.

The paper gives no attention formula, rotary embedding, chunk size or
eviction order; the readings taken are:
scaled dot-product softmax with 1/sqrt(D); every chunk query sees every chunk
key (or, with `block_frames`, the chunk keys of its own and earlier blocks of
that many frames: the block-causal mask at a finer block size, down to the
frame-by-frame factorisation p(x_i | x_<i) of Sec. 3.1);
the first S frames after a reset are the sinks; eviction is FIFO over
non-sink frames; attention runs over the residents first and the append comes
after; rotary embedding is 3-axis (frame, row, column) on interleaved adjacent
pairs with per-axis frequencies base**(-j/n_axis), temporal position = the
absolute frame index, keys cached after rotation, values never rotated;
gradients are returned for the un-rotated Q, K_chunk, V_chunk.

Window-relative temporal positions (`window_relative=True`).  Sec. 4.3 only
says that a positional-extrapolation method from another paper lets models
trained on short clips run for long videos, and defines nothing.  The reading
built here: the temporal position of a frame is its RANK in the sequence the
chunk attends to -- sinks first (0 .. S-1), then the resident window frames
from oldest to newest, then the chunk's own frames -- instead of its absolute
index.  Ranks never exceed C + n_frames - 1 however long the stream runs, and
the stream's start frame no longer matters.  Row and column positions are
unchanged.  Relative to absolute positions this only moves the sinks: window
and chunk frames are consecutive either way, while the distance from the
sinks to the window stays S instead of growing with every eviction.

Parity pins: tests/test_oracle_*.py (brute force, invariants, closed forms,
library SDPA, finite differences).  The rotary pair layout and the
attend-then-append order are fixed by this build, not by the paper: for those
two readings parity is unpinned by the paper.
"""
from __future__ import annotations

from typing import Iterable, List, Optional, Sequence, Tuple

import numpy as np


# ----------------------------------------------------------------------------
# rotary embedding
# ----------------------------------------------------------------------------

def rope_angles(frame: int, grid_h: int, grid_w: int, pairs: Sequence[int], base: float) -> np.ndarray:
    """Rotation angle of every (token, pair) of one frame: array [T, D/2].

    Token t = row * grid_w + col.  Pair i belongs to the frame axis if
    i < n_t, to the row axis if i < n_t + n_h, else to the column axis; with
    in-axis index j and n_a pairs on the axis, the frequency is base**(-j/n_a)
    and the angle is position * frequency.
    """
    n_t, n_h, n_w = (int(p) for p in pairs)
    rows = np.repeat(np.arange(grid_h, dtype=np.float64), grid_w)
    cols = np.tile(np.arange(grid_w, dtype=np.float64), grid_h)
    T = grid_h * grid_w
    out = np.empty((T, n_t + n_h + n_w), dtype=np.float64)
    base = np.float64(base)
    for j in range(n_t):
        out[:, j] = np.float64(frame) * base ** (-np.float64(j) / n_t)
    for j in range(n_h):
        out[:, n_t + j] = rows * base ** (-np.float64(j) / n_h)
    for j in range(n_w):
        out[:, n_t + n_h + j] = cols * base ** (-np.float64(j) / n_w)
    return out


def rope_rotate(x: np.ndarray, phi: np.ndarray) -> np.ndarray:
    """Rotate adjacent pairs (x[2i], x[2i+1]) of x [N, H, D] by phi [N, D/2].
    Dimensions beyond 2*phi.shape[1] (none when the split sums to D/2) pass."""
    x = np.asarray(x, dtype=np.float64)
    out = x.copy()
    npair = phi.shape[1]
    if npair == 0:
        return out
    c = np.cos(phi)[:, None, :]
    s = np.sin(phi)[:, None, :]
    x0 = x[..., 0:2 * npair:2]
    x1 = x[..., 1:2 * npair:2]
    out[..., 0:2 * npair:2] = x0 * c - x1 * s
    out[..., 1:2 * npair:2] = x0 * s + x1 * c
    return out


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Diagnostic only: round fp64 values to the nearest bf16 (ties to even)."""
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    u = f.view(np.uint32)
    u = (u + (((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF))) & np.uint32(0xFFFF0000)
    return u.view(np.float32).astype(np.float64)


# ----------------------------------------------------------------------------
# which frames a new chunk may see (Sec. 3.2)
# ----------------------------------------------------------------------------

def visible_history(n0: int, sink_frames: int, window_frames: int) -> List[int]:
    """Stream-local numbers n < n0 of the history frames a chunk starting at
    frame number n0 attends to: the sinks and the last `window_frames`
    non-sink frames."""
    vis = []
    for n in range(n0):
        if n < sink_frames:
            vis.append(n)
        elif n >= n0 - window_frames:
            vis.append(n)
    return vis


class RingTableSim:
    """Naive simulation of the resident-frame table of one stream: a list of C
    slots; a new frame takes the lowest empty slot, else the slot of the oldest
    non-sink frame, which is thereby evicted."""

    def __init__(self, capacity_frames: int, sink_frames: int, start_frame: int = 0):
        self.capacity = capacity_frames
        self.sinks = sink_frames
        self.start = start_frame
        self.next_n = 0
        self.slot_number: List[Optional[int]] = [None] * capacity_frames

    def append_frame(self) -> int:
        n = self.next_n
        if None in self.slot_number:
            slot = self.slot_number.index(None)
        else:
            candidates = [(m, s) for s, m in enumerate(self.slot_number) if m >= self.sinks]
            slot = min(candidates)[1]
        self.slot_number[slot] = n
        self.next_n += 1
        return slot

    def slot_frame(self) -> List[int]:
        return [-1 if m is None else self.start + m for m in self.slot_number]

    def slot_pos(self, window_relative: bool = False) -> List[int]:
        # temporal rotary position of the frame held by each slot; -1 for an empty slot.
        # Absolute: the frame's absolute index (reading 9).  Window-relative: its rank among
        # the resident frames in stream order.
        if not window_relative:
            return self.slot_frame()
        resident = sorted(m for m in self.slot_number if m is not None)
        return [-1 if m is None else resident.index(m) for m in self.slot_number]


# ----------------------------------------------------------------------------
# attention over the visible set
# ----------------------------------------------------------------------------

def _softmax_attention(qt, kt, v, visible=None):
    """qt [Nq, D], kt [Nk, D], v [Nk, D] -> P [Nq, Nk], O [Nq, D], LSE [Nq].
    visible: optional bool [Nq, Nk]; a hidden key gets score -inf (probability 0).
    Every row must see at least one key."""
    D = qt.shape[1]
    s = (qt @ kt.T) / np.sqrt(np.float64(D))
    if visible is not None:
        s = np.where(visible, s, -np.inf)
    m = s.max(axis=1, keepdims=True)
    e = np.exp(s - m)
    z = e.sum(axis=1, keepdims=True)
    p = e / z
    o = p @ v
    lse = (m + np.log(z))[:, 0]
    return p, o, lse


class RollingCacheOracle:
    """B independent streams; per stream the whole history of appended frames.

    Tensors are [B, n_frames*T, H, D] float64 (un-rotated), token
    n = (frame_in_chunk * grid_h + row) * grid_w + col.
    """

    def __init__(self, batch: int, heads: int, head_dim: int, grid_h: int, grid_w: int,
                 capacity_frames: int, sink_frames: int, rope_pairs: Sequence[int],
                 rope_base: float = 10000.0, start_frames: Optional[Iterable[int]] = None,
                 cache_rounding: bool = False, block_frames: Optional[int] = None,
                 window_relative: bool = False):
        assert 0 <= sink_frames < capacity_frames
        assert block_frames is None or block_frames >= 1
        assert sum(rope_pairs) in (0, head_dim // 2)
        self.B, self.H, self.D = batch, heads, head_dim
        self.gh, self.gw = grid_h, grid_w
        self.T = grid_h * grid_w
        self.C, self.S = capacity_frames, sink_frames
        self.Lw = capacity_frames - sink_frames
        self.pairs = tuple(int(p) for p in rope_pairs)
        self.base = float(rope_base)
        self.cache_rounding = cache_rounding  # diagnostic: bf16-round rotated cached keys
        # None: every chunk query sees the whole chunk.  k: the chunk's frames form blocks of
        # k frames (the last may be shorter); a query sees the chunk keys of its own block
        # and of earlier blocks only.  The history is visible to every query either way.
        self.block_frames = block_frames
        # temporal positions by rank in the attended sequence instead of absolute frame index
        self.window_relative = window_relative
        starts = [0] * batch if start_frames is None else [int(s) for s in start_frames]
        self.start = starts
        # per stream: list of (K_frame [T,H,D], V_frame [T,H,D]) by reference
        self.history: List[List[Tuple[np.ndarray, np.ndarray]]] = [[] for _ in range(batch)]
        self.tables = [RingTableSim(capacity_frames, sink_frames, s) for s in starts]

    # -- state ---------------------------------------------------------------
    def reset(self, stream: int, start_frame: int) -> None:
        which = range(self.B) if stream < 0 else [stream]
        for b in which:
            self.start[b] = int(start_frame)
            self.history[b] = []
            self.tables[b] = RingTableSim(self.C, self.S, int(start_frame))

    def append(self, k: np.ndarray, v: np.ndarray, n_frames: int) -> None:
        """Commit n_frames new frames per stream (un-rotated K, V)."""
        assert k.shape == v.shape == (self.B, n_frames * self.T, self.H, self.D)
        for b in range(self.B):
            self.append_stream(b, k[b], v[b], n_frames)

    def append_stream(self, b: int, k: np.ndarray, v: np.ndarray, n_frames: int) -> None:
        for i in range(n_frames):
            self.history[b].append((k[i * self.T:(i + 1) * self.T], v[i * self.T:(i + 1) * self.T]))
            self.tables[b].append_frame()

    def table_arrays(self):
        slot_frame = np.array([t.slot_frame() for t in self.tables], dtype=np.int32)
        slot_pos = np.array([t.slot_pos(self.window_relative) for t in self.tables], dtype=np.int32)
        next_n = np.array([t.next_n for t in self.tables], dtype=np.int32)
        return slot_frame, slot_pos, next_n

    # -- helpers ---------------------------------------------------------------
    def _phi(self, frame: int) -> np.ndarray:
        return rope_angles(frame, self.gh, self.gw, self.pairs, self.base)

    def _context(self, b: int, h: int):
        """Rotated keys and values of stream b's visible history for head h."""
        n0 = len(self.history[b])
        ks, vs = [], []
        for rank, n in enumerate(visible_history(n0, self.S, self.Lw)):
            kf, vf = self.history[b][n]
            pos = rank if self.window_relative else self.start[b] + n
            kt = rope_rotate(np.asarray(kf[:, h:h + 1, :], dtype=np.float64), self._phi(pos))[:, 0]
            if self.cache_rounding:
                kt = round_to_bf16(kt)
            ks.append(kt)
            vs.append(np.asarray(vf[:, h, :], dtype=np.float64))
        if ks:
            return np.concatenate(ks, 0), np.concatenate(vs, 0)
        return np.zeros((0, self.D)), np.zeros((0, self.D))

    def _chunk_phi(self, b: int, n_frames: int) -> np.ndarray:
        if self.window_relative:  # the chunk continues the ranks of the visible history
            f0 = len(visible_history(len(self.history[b]), self.S, self.Lw))
        else:
            f0 = self.start[b] + len(self.history[b])
        return np.concatenate([self._phi(f0 + i) for i in range(n_frames)], 0)

    def _visible(self, n_hist_rows: int, n_frames: int):
        """bool [Nq, n_hist_rows + Nq] of the keys each chunk query sees, or None when
        that is all of them."""
        if self.block_frames is None or self.block_frames >= n_frames:
            return None
        block = (np.arange(n_frames * self.T) // self.T) // self.block_frames  # block of each chunk token
        chunk = block[None, :] <= block[:, None]
        return np.concatenate([np.ones((n_frames * self.T, n_hist_rows), dtype=bool), chunk], axis=1)

    def _pairs(self, streams, heads):
        bs = range(self.B) if streams is None else streams
        hs = range(self.H) if heads is None else heads
        return [(b, h) for b in bs for h in hs]

    # -- forward ---------------------------------------------------------------
    def attn_fwd(self, q, k_chunk, v_chunk, n_frames: int, streams=None, heads=None,
                 return_probs: bool = False, rows=None):
        """O [B,Nq,H,D], LSE [B,H,Nq]; only the listed (stream, head) pairs are
        filled when `streams` / `heads` are given (the rest stay NaN).  `rows`: only
        these query rows are computed (a query's output depends on no other query),
        against all the keys it sees; the other rows stay NaN."""
        Nq = n_frames * self.T
        assert q.shape == k_chunk.shape == v_chunk.shape == (self.B, Nq, self.H, self.D)
        out = np.full((self.B, Nq, self.H, self.D), np.nan)
        lse = np.full((self.B, self.H, Nq), np.nan)
        probs = {}
        sel = slice(None) if rows is None else np.asarray(rows, dtype=np.int64)
        for b, h in self._pairs(streams, heads):
            phi = self._chunk_phi(b, n_frames)
            qt = rope_rotate(np.asarray(q[b, :, h:h + 1, :], dtype=np.float64), phi)[:, 0]
            kc = rope_rotate(np.asarray(k_chunk[b, :, h:h + 1, :], dtype=np.float64), phi)[:, 0]
            kh, vh = self._context(b, h)
            kt = np.concatenate([kh, kc], 0)
            vv = np.concatenate([vh, np.asarray(v_chunk[b, :, h, :], dtype=np.float64)], 0)
            vis = self._visible(kh.shape[0], n_frames)
            p, o, l = _softmax_attention(qt[sel], kt, vv, None if vis is None else vis[sel])
            out[b, sel, h, :] = o
            lse[b, h, sel] = l
            if return_probs:
                probs[(b, h)] = p
        if return_probs:
            return out, lse, probs
        return out, lse

    # -- backward (history detached) --------------------------------------------
    def attn_bwd(self, q, k_chunk, v_chunk, dout, n_frames: int, streams=None, heads=None,
                 return_dscores: bool = False, history_grads: bool = False):
        """dQ, dK_chunk, dV_chunk [B,Nq,H,D] w.r.t. the un-rotated inputs; the
        cached frames are constants (Sec. 3.3).  With `history_grads` the
        gradients w.r.t. the rotated cached keys and cached values are also
        returned per pair (used by pins only)."""
        Nq = n_frames * self.T
        scale = 1.0 / np.sqrt(np.float64(self.D))
        dq = np.full((self.B, Nq, self.H, self.D), np.nan)
        dk = np.full((self.B, Nq, self.H, self.D), np.nan)
        dv = np.full((self.B, Nq, self.H, self.D), np.nan)
        extra = {}
        for b, h in self._pairs(streams, heads):
            phi = self._chunk_phi(b, n_frames)
            qt = rope_rotate(np.asarray(q[b, :, h:h + 1, :], dtype=np.float64), phi)[:, 0]
            kc = rope_rotate(np.asarray(k_chunk[b, :, h:h + 1, :], dtype=np.float64), phi)[:, 0]
            kh, vh = self._context(b, h)
            nh = kh.shape[0]
            kt = np.concatenate([kh, kc], 0)
            vv = np.concatenate([vh, np.asarray(v_chunk[b, :, h, :], dtype=np.float64)], 0)
            do = np.asarray(dout[b, :, h, :], dtype=np.float64)
            p, o, _ = _softmax_attention(qt, kt, vv, self._visible(kh.shape[0], n_frames))
            delta = (do * o).sum(axis=1, keepdims=True)
            dp = do @ vv.T
            ds = p * (dp - delta)
            dqt = scale * (ds @ kt)
            dkt = scale * (ds[:, nh:].T @ qt)
            dvc = p[:, nh:].T @ do
            # d/dx of R(phi) x is R(phi)^T = R(-phi)
            dq[b, :, h, :] = rope_rotate(dqt[:, None, :], -phi)[:, 0]
            dk[b, :, h, :] = rope_rotate(dkt[:, None, :], -phi)[:, 0]
            dv[b, :, h, :] = dvc
            if return_dscores or history_grads:
                extra[(b, h)] = dict(ds=ds, dk_hist_rot=scale * (ds[:, :nh].T @ qt), dv_hist=p[:, :nh].T @ do)
        if return_dscores or history_grads:
            return dq, dk, dv, extra
        return dq, dk, dv

    # -- group-wise candidates over one shared, frozen context (Sec. 3.2) ------------------
    # Clip-level group sampling: G candidate continuations of stream b are generated from the
    # SAME rolling cache; candidate g's chunk attends to the stream's visible history and to
    # its own chunk only, never to another candidate's.  Tensors are [B*G, Nq, H, D] with
    # candidate c = b*G + g.  By definition this is attention of each candidate against its
    # stream's context, so it is written as exactly that loop.
    def _candidate_pairs(self, group: int, candidates, heads):
        cs = range(self.B * group) if candidates is None else candidates
        hs = range(self.H) if heads is None else heads
        return [(c, h) for c in cs for h in hs]

    def group_attn_fwd(self, q, k_chunk, v_chunk, n_frames: int, group: int, candidates=None, heads=None,
                       rows=None):
        """O [B*G,Nq,H,D], LSE [B*G,H,Nq]; unlisted (candidate, head) pairs stay NaN, and with
        `rows` only those query rows are computed (as in attn_fwd)."""
        Nq = n_frames * self.T
        assert group >= 1
        assert q.shape == k_chunk.shape == v_chunk.shape == (self.B * group, Nq, self.H, self.D)
        out = np.full((self.B * group, Nq, self.H, self.D), np.nan)
        lse = np.full((self.B * group, self.H, Nq), np.nan)
        sel = slice(None) if rows is None else np.asarray(rows, dtype=np.int64)
        context = {}
        for c, h in self._candidate_pairs(group, candidates, heads):
            b = c // group
            if (b, h) not in context:
                context[(b, h)] = self._context(b, h)
            kh, vh = context[(b, h)]
            phi = self._chunk_phi(b, n_frames)
            qt = rope_rotate(np.asarray(q[c, :, h:h + 1, :], dtype=np.float64), phi)[:, 0]
            kc = rope_rotate(np.asarray(k_chunk[c, :, h:h + 1, :], dtype=np.float64), phi)[:, 0]
            kt = np.concatenate([kh, kc], 0)
            vv = np.concatenate([vh, np.asarray(v_chunk[c, :, h, :], dtype=np.float64)], 0)
            vis = self._visible(kh.shape[0], n_frames)
            _, o, l = _softmax_attention(qt[sel], kt, vv, None if vis is None else vis[sel])
            out[c, sel, h, :] = o
            lse[c, h, sel] = l
        return out, lse

    def group_attn_bwd(self, q, k_chunk, v_chunk, dout, n_frames: int, group: int, candidates=None, heads=None):
        """dQ, dK_chunk, dV_chunk [B*G,Nq,H,D]; the shared context is a constant (Sec. 3.3)."""
        Nq = n_frames * self.T
        scale = 1.0 / np.sqrt(np.float64(self.D))
        shape = (self.B * group, Nq, self.H, self.D)
        assert q.shape == k_chunk.shape == v_chunk.shape == dout.shape == shape
        dq, dk, dv = (np.full(shape, np.nan) for _ in range(3))
        context = {}
        for c, h in self._candidate_pairs(group, candidates, heads):
            b = c // group
            if (b, h) not in context:
                context[(b, h)] = self._context(b, h)
            kh, vh = context[(b, h)]
            nh = kh.shape[0]
            phi = self._chunk_phi(b, n_frames)
            qt = rope_rotate(np.asarray(q[c, :, h:h + 1, :], dtype=np.float64), phi)[:, 0]
            kc = rope_rotate(np.asarray(k_chunk[c, :, h:h + 1, :], dtype=np.float64), phi)[:, 0]
            kt = np.concatenate([kh, kc], 0)
            vv = np.concatenate([vh, np.asarray(v_chunk[c, :, h, :], dtype=np.float64)], 0)
            do = np.asarray(dout[c, :, h, :], dtype=np.float64)
            p, o, _ = _softmax_attention(qt, kt, vv, self._visible(kh.shape[0], n_frames))
            delta = (do * o).sum(axis=1, keepdims=True)
            ds = p * (do @ vv.T - delta)
            dq[c, :, h, :] = rope_rotate((scale * (ds @ kt))[:, None, :], -phi)[:, 0]
            dk[c, :, h, :] = rope_rotate((scale * (ds[:, nh:].T @ qt))[:, None, :], -phi)[:, 0]
            dv[c, :, h, :] = p[:, nh:].T @ do
        return dq, dk, dv

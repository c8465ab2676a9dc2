"""Seeded synthetic inputs and the named workload shapes.

This module holds none of the method's arithmetic: it only names shapes and
draws seeded N(0,1) values rounded to bf16.  Both the CPU oracle's tests and
the GPU tests / benchmark take their inputs from here so that both sides see
identical bit patterns.

The real inputs of the paper's path are activations of a causal video
diffusion transformer at 480x832 resolution (Table S1); those weights are not
available, so i.i.d. unit-variance Gaussians of the same tensor shapes stand
in for them.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Tuple

import numpy as np

BASE_SEED = 20260317


@dataclass(frozen=True)
class Workload:
    """Shape of one streaming-attention workload.

    batch            B  independent streams, each with its own ring cache
    heads, head_dim  H, D
    grid_h, grid_w   latent grid of one frame; T = grid_h * grid_w tokens
    capacity_frames  C  ring capacity (frames resident before the chunk)
    sink_frames      S  first S frames of a stream are never evicted
    chunk_frames     Fc frames per new chunk
    resident_frames  R  frames already streamed before the measured chunk
    rope_pairs       rotary pairs given to the (frame, row, column) axes
    """

    name: str
    config_id: int
    batch: int
    heads: int
    head_dim: int
    grid_h: int
    grid_w: int
    capacity_frames: int
    sink_frames: int
    chunk_frames: int
    resident_frames: int
    rope_pairs: Tuple[int, int, int]
    rope_base: float = 10000.0

    @property
    def tokens_per_frame(self) -> int:
        return self.grid_h * self.grid_w

    @property
    def n_q(self) -> int:
        return self.chunk_frames * self.tokens_per_frame

    @property
    def n_k(self) -> int:
        r = min(self.resident_frames, self.capacity_frames)
        return (r + self.chunk_frames) * self.tokens_per_frame

    @property
    def seed(self) -> int:
        return BASE_SEED + self.config_id

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


def default_rope_pairs(head_dim: int) -> Tuple[int, int, int]:
    """Split of the D/2 rotary pairs over (frame, row, column): the two
    spatial axes get floor(D/6) pairs each and the frame axis the rest."""
    s = head_dim // 6
    return (head_dim // 2 - 2 * s, s, s)


# The five named configurations.
TINY_FWD = Workload("tiny_fwd", 1, 1, 2, 64, 8, 8, 4, 0, 1, 4, (12, 10, 10))
PROD_FWD = Workload("prod_fwd", 2, 1, 12, 128, 30, 52, 18, 0, 3, 18, (22, 21, 21))
GROUP_FWD_APPEND = Workload("group_fwd_append", 3, 8, 12, 128, 30, 52, 18, 0, 3, 18, (22, 21, 21))
STREAM_EVICT = Workload("stream_evict", 4, 1, 12, 128, 30, 52, 12, 1, 3, 0, (22, 21, 21))
RL_BWD = Workload("rl_bwd", 5, 4, 12, 128, 30, 52, 18, 0, 3, 18, (22, 21, 21))
# one stream whose frozen cache is shared by a group of candidate chunks (group size given at the call)
SHARED_PREFIX = Workload("shared_prefix", 6, 1, 12, 128, 30, 52, 18, 0, 3, 18, (22, 21, 21))

WORKLOADS = {w.name: w for w in (TINY_FWD, PROD_FWD, GROUP_FWD_APPEND, STREAM_EVICT, RL_BWD, SHARED_PREFIX)}


# ----------------------------------------------------------------------------
# bf16 bit patterns <-> wider floats (format conversion only)
# ----------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even), returned as uint16."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounding = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + rounding) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(bits).astype(np.float64)


# ----------------------------------------------------------------------------
# seeded generators
# ----------------------------------------------------------------------------

# tensor ids used as the second half of the generator key
T_Q, T_K, T_V, T_DO, T_HIST_K, T_HIST_V, T_OFFSETS = range(7)


def _rng(seed: int, tensor_id: int, index: int = 0) -> np.random.Generator:
    # Philox is counter based: the key fixes the stream, independent of draw order
    # of any other tensor.
    return np.random.Generator(np.random.Philox(key=[seed, (tensor_id << 32) | index]))


def normal_bf16(seed: int, tensor_id: int, shape, index: int = 0) -> np.ndarray:
    """i.i.d. N(0,1) rounded to bf16; uint16 bit patterns of the given shape."""
    x = _rng(seed, tensor_id, index).standard_normal(size=shape, dtype=np.float32)
    return f32_to_bf16_bits(x)


def normal_f32(seed: int, tensor_id: int, shape, index: int = 0) -> np.ndarray:
    """i.i.d. N(0,1) in float32 (for the fp32 debug path)."""
    return _rng(seed, tensor_id, index).standard_normal(size=shape, dtype=np.float32)


def stream_offsets(seed: int, batch: int, low: int = 0, high: int = 60) -> np.ndarray:
    """Per-stream number of frames already streamed, uniform on [low, high]."""
    return _rng(seed, T_OFFSETS).integers(low, high + 1, size=batch).astype(np.int64)


def chunk_inputs(w: Workload, step: int = 0, with_dout: bool = False):
    """bf16 bit patterns of Q, K_chunk, V_chunk (and dO) for chunk number `step`,
    each of shape [B, Fc*T, H, D]."""
    shape = (w.batch, w.n_q, w.heads, w.head_dim)
    q = normal_bf16(w.seed, T_Q, shape, step)
    k = normal_bf16(w.seed, T_K, shape, step)
    v = normal_bf16(w.seed, T_V, shape, step)
    if with_dout:
        return q, k, v, normal_bf16(w.seed, T_DO, shape, step)
    return q, k, v


def group_inputs(w: Workload, group: int, step: int = 0, with_dout: bool = False):
    """As chunk_inputs, for `group` candidate chunks per stream: [B*group, Fc*T, H, D],
    candidate c = b*group + g."""
    shape = (w.batch * group, w.n_q, w.heads, w.head_dim)
    ids = (T_Q, T_K, T_V, T_DO) if with_dout else (T_Q, T_K, T_V)
    return tuple(normal_bf16(w.seed + 1000 * group, t, shape, step) for t in ids)


def history_frame_pool(w: Workload, n_pool: int):
    """A pool of `n_pool` distinct random frames (K and V bit patterns), each
    [T, H, D].  History frames of every stream are taken from the pool by index
    so that long histories cost no extra generation time or memory."""
    shape = (n_pool, w.tokens_per_frame, w.heads, w.head_dim)
    return normal_bf16(w.seed, T_HIST_K, shape), normal_bf16(w.seed, T_HIST_V, shape)


def pool_index(stream: int, frame_number: int, n_pool: int) -> int:
    """Which pool frame stream `stream` uses as its `frame_number`-th history frame."""
    return (stream * 7 + frame_number * 5 + 3) % n_pool

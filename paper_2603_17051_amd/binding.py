"""ctypes binding of the C ABI in include/astro.h: argument marshalling only.

torch is used for device memory and streams; every computation happens in the
HIP library.  If libastro.so is missing the import of this module fails
loudly; there is no fallback.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, byref, c_double, c_float, c_int, c_int32, c_size_t, c_void_p

import torch

from .build import LIB_PATH

ASTRO_OK = 0
ASTRO_ERR_INVALID_ARG = -1
ASTRO_ERR_BAD_STATE = -2
ASTRO_ERR_UNSUPPORTED = -3
ASTRO_ERR_HIP = -4
ASTRO_ERR_WORKSPACE = -5
ASTRO_BF16 = 0
ASTRO_F32 = 1
ASTRO_FLAG_HOST_ONLY = 1
ASTRO_FLAG_WINDOW_RELATIVE = 2
ASTRO_FLAG_REUSE_STAGED = 4
ASTRO_MAX_BATCH = 64
ASTRO_MAX_CAPACITY_FRAMES = 256

EXPORTED = (
    "astro_kvcache_bytes", "astro_kvcache_sink_bytes", "astro_kvcache_create", "astro_kvcache_destroy", "astro_kvcache_reset",
    "astro_kvcache_append", "astro_kvcache_tables", "astro_chunk_attn_workspace_bytes",
    "astro_chunk_attn_fwd", "astro_chunk_attn_bwd", "astro_strerror",
    "astro_group_attn_workspace_bytes", "astro_group_attn_fwd", "astro_group_attn_bwd",
    "astro_nft_loss_workspace_bytes", "astro_nft_loss", "astro_nft_loss_static_bytes", "astro_nft_loss_static",
    "astro_chunk_attn_bwd_full_workspace_bytes", "astro_chunk_attn_bwd_full",
    "astro_profile_begin", "astro_profile_end", "astro_calib_mfma", "astro_calib_copy",
)


class astro_kvcache_desc_t(ctypes.Structure):
    _fields_ = [
        ("batch", c_int32), ("heads", c_int32), ("head_dim", c_int32),
        ("grid_h", c_int32), ("grid_w", c_int32),
        ("capacity_frames", c_int32), ("sink_frames", c_int32), ("max_chunk_frames", c_int32),
        ("rope_pairs_t", c_int32), ("rope_pairs_h", c_int32), ("rope_pairs_w", c_int32),
        ("dtype", c_int32), ("flags", c_int32), ("block_frames", c_int32),
        ("rope_base", c_double),
        ("k_storage", c_void_p), ("v_storage", c_void_p), ("k_sink_storage", c_void_p),
    ]


class astro_kernel_time_t(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char * 48), ("launches", c_int32), ("total_ms", c_float)]


class AstroError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {astro_strerror(code)} ({code})")


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    P = POINTER
    lib.astro_kvcache_bytes.argtypes = [P(astro_kvcache_desc_t), P(c_size_t), P(c_size_t)]
    lib.astro_kvcache_sink_bytes.argtypes = [P(astro_kvcache_desc_t), P(c_size_t)]
    lib.astro_kvcache_create.argtypes = [P(astro_kvcache_desc_t), P(c_void_p)]
    lib.astro_kvcache_destroy.argtypes = [c_void_p]
    lib.astro_kvcache_reset.argtypes = [c_void_p, c_int32, c_int32]
    lib.astro_kvcache_append.argtypes = [c_void_p, c_void_p, c_void_p, c_int32, c_void_p]
    lib.astro_kvcache_tables.argtypes = [c_void_p, P(c_int32), P(c_int32), P(c_int32)]
    lib.astro_chunk_attn_workspace_bytes.argtypes = [c_void_p, c_int32, P(c_size_t), P(c_size_t)]
    lib.astro_chunk_attn_fwd.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int32, c_void_p, c_void_p,
                                         c_void_p, c_size_t, c_void_p]
    lib.astro_chunk_attn_bwd.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                         c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    lib.astro_group_attn_workspace_bytes.argtypes = [c_void_p, c_int32, c_int32, P(c_size_t), P(c_size_t)]
    lib.astro_group_attn_fwd.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int32, c_int32, c_void_p, c_void_p,
                                         c_void_p, c_size_t, c_void_p]
    lib.astro_group_attn_bwd.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                         c_int32, c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    lib.astro_nft_loss_workspace_bytes.argtypes = [c_int32, ctypes.c_int64, P(c_size_t)]
    lib.astro_nft_loss.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int32, ctypes.c_int64,
                                   c_int32, c_float, c_float, c_float, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    lib.astro_nft_loss_static_bytes.argtypes = [P(c_size_t)]
    lib.astro_nft_loss_static.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int32, ctypes.c_int64,
                                          c_int32, c_float, c_float, c_float, c_void_p, c_void_p, c_void_p]
    lib.astro_chunk_attn_bwd_full_workspace_bytes.argtypes = [c_void_p, c_int32, P(c_size_t)]
    lib.astro_chunk_attn_bwd_full.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                              c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                              c_size_t, c_void_p]
    lib.astro_profile_begin.argtypes = []
    lib.astro_profile_end.argtypes = [P(astro_kernel_time_t), c_int32, P(c_int32)]
    lib.astro_calib_mfma.argtypes = [c_void_p, c_int32, c_int32, c_void_p, c_void_p]
    lib.astro_calib_copy.argtypes = [c_void_p, c_void_p, c_size_t, c_void_p]
    for name in EXPORTED:
        getattr(lib, name).restype = c_int
    lib.astro_strerror.argtypes = [c_int]
    lib.astro_strerror.restype = ctypes.c_char_p
    return lib


_lib = _load()


def library() -> ctypes.CDLL:
    return _lib


def astro_strerror(code: int) -> str:
    return _lib.astro_strerror(int(code)).decode()


def _check(code: int, where: str) -> None:
    if code != ASTRO_OK:
        raise AstroError(code, where)


def _ptr(t) -> c_void_p:
    return c_void_p(None if t is None else t.data_ptr())


def _stream(stream) -> c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return c_void_p(stream.cuda_stream)


def make_desc(batch, heads, head_dim, grid_h, grid_w, capacity_frames, sink_frames, max_chunk_frames,
              rope_pairs=(0, 0, 0), rope_base=10000.0, dtype=ASTRO_BF16, flags=0,
              k_storage=None, v_storage=None, block_frames=0, k_sink_storage=None) -> astro_kvcache_desc_t:
    return astro_kvcache_desc_t(batch, heads, head_dim, grid_h, grid_w, capacity_frames, sink_frames,
                                max_chunk_frames, rope_pairs[0], rope_pairs[1], rope_pairs[2], dtype, flags, block_frames,
                                float(rope_base), _ptr(k_storage), _ptr(v_storage), _ptr(k_sink_storage))


def astro_kvcache_bytes(desc: astro_kvcache_desc_t):
    kb, vb = c_size_t(0), c_size_t(0)
    _check(_lib.astro_kvcache_bytes(byref(desc), byref(kb), byref(vb)), "astro_kvcache_bytes")
    return kb.value, vb.value


def astro_kvcache_sink_bytes(desc: astro_kvcache_desc_t) -> int:
    n = c_size_t(0)
    _check(_lib.astro_kvcache_sink_bytes(byref(desc), byref(n)), "astro_kvcache_sink_bytes")
    return n.value


class KVCache:
    """Owner of one cache handle and of the torch tensors behind it."""

    def __init__(self, handle: c_void_p, desc: astro_kvcache_desc_t, k_storage, v_storage, k_sink_storage=None):
        self.handle = handle
        self.desc = desc
        self.k_storage = k_storage
        self.v_storage = v_storage
        self.k_sink_storage = k_sink_storage
        self._workspace = None

    @property
    def tokens_per_frame(self) -> int:
        return self.desc.grid_h * self.desc.grid_w

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.desc.dtype == ASTRO_BF16 else torch.float32

    def workspace(self, nbytes: int, device) -> torch.Tensor:
        if self._workspace is None or self._workspace.numel() < nbytes:
            self._workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
        return self._workspace

    def close(self) -> None:
        if self.handle is not None:
            astro_kvcache_destroy(self)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def astro_kvcache_create(batch, heads, head_dim, grid_h, grid_w, capacity_frames, sink_frames, max_chunk_frames,
                         rope_pairs=(0, 0, 0), rope_base=10000.0, dtype=ASTRO_BF16, host_only=False,
                         device="cuda:0", block_frames=0, window_relative=False, reuse_staged=False) -> KVCache:
    """Allocate the K/V storage with torch (unless host_only) and create the handle."""
    flags = ((ASTRO_FLAG_HOST_ONLY if host_only else 0) | (ASTRO_FLAG_WINDOW_RELATIVE if window_relative else 0)
             | (ASTRO_FLAG_REUSE_STAGED if reuse_staged else 0))
    desc = make_desc(batch, heads, head_dim, grid_h, grid_w, capacity_frames, sink_frames, max_chunk_frames,
                     rope_pairs, rope_base, dtype, flags, block_frames=block_frames)
    k_storage = v_storage = k_sink_storage = None
    if not host_only:
        kb, vb = astro_kvcache_bytes(desc)
        k_storage = torch.zeros(kb, dtype=torch.uint8, device=device)
        v_storage = torch.zeros(vb, dtype=torch.uint8, device=device)
        desc.k_storage, desc.v_storage = _ptr(k_storage), _ptr(v_storage)
        sb = astro_kvcache_sink_bytes(desc)
        if sb:
            k_sink_storage = torch.zeros(sb, dtype=torch.uint8, device=device)
            desc.k_sink_storage = _ptr(k_sink_storage)
    handle = c_void_p(None)
    _check(_lib.astro_kvcache_create(byref(desc), byref(handle)), "astro_kvcache_create")
    return KVCache(handle, desc, k_storage, v_storage, k_sink_storage)


def astro_kvcache_destroy(cache: KVCache) -> None:
    handle, cache.handle = cache.handle, None
    _check(_lib.astro_kvcache_destroy(handle), "astro_kvcache_destroy")


def astro_kvcache_reset(cache: KVCache, stream_index: int = -1, start_frame: int = 0) -> None:
    _check(_lib.astro_kvcache_reset(cache.handle, stream_index, start_frame), "astro_kvcache_reset")


def _check_chunk_tensor(cache: KVCache, t: torch.Tensor, n_frames: int, name: str, dtype=None, group: int = 1) -> None:
    d = cache.desc
    shape = (d.batch * group, n_frames * cache.tokens_per_frame, d.heads, d.head_dim)
    if tuple(t.shape) != shape or not t.is_contiguous() or t.dtype != (dtype or cache.torch_dtype):
        raise ValueError(f"{name}: expected contiguous {dtype or cache.torch_dtype} tensor of shape {shape}, "
                         f"got {t.dtype} {tuple(t.shape)}")
    if not t.is_cuda:
        raise ValueError(f"{name}: must be a device tensor")


def astro_kvcache_append(cache: KVCache, k=None, v=None, n_frames: int = 1, stream=None) -> None:
    host_only = bool(cache.desc.flags & ASTRO_FLAG_HOST_ONLY)
    if not host_only:
        _check_chunk_tensor(cache, k, n_frames, "k")
        _check_chunk_tensor(cache, v, n_frames, "v")
    _check(_lib.astro_kvcache_append(cache.handle, _ptr(k), _ptr(v), n_frames,
                                     c_void_p(None) if host_only else _stream(stream)), "astro_kvcache_append")


def astro_kvcache_tables(cache: KVCache):
    """(slot_frame [B, C], slot_pos [B, C], next_n [B]) as nested python lists."""
    B, C = cache.desc.batch, cache.desc.capacity_frames
    sf, sp, nn = (c_int32 * (B * C))(), (c_int32 * (B * C))(), (c_int32 * B)()
    _check(_lib.astro_kvcache_tables(cache.handle, sf, sp, nn), "astro_kvcache_tables")
    rows = lambda a: [list(a[b * C:(b + 1) * C]) for b in range(B)]
    return rows(sf), rows(sp), list(nn)


def astro_group_attn_workspace_bytes(cache: KVCache, n_frames: int, group: int):
    f, b = c_size_t(0), c_size_t(0)
    _check(_lib.astro_group_attn_workspace_bytes(cache.handle, n_frames, group, byref(f), byref(b)),
           "astro_group_attn_workspace_bytes")
    return f.value, b.value


def astro_group_attn_fwd(cache: KVCache, q, k_chunk, v_chunk, n_frames: int, group: int, out=None, lse=None,
                         workspace=None, stream=None):
    """`group` candidate chunks per cache stream, tensors [B*group, Nq, H, D].
    Returns (out [B*group, Nq, H, D], lse [B*group, H, Nq] fp32)."""
    for name, t in (("q", q), ("k_chunk", k_chunk), ("v_chunk", v_chunk)):
        _check_chunk_tensor(cache, t, n_frames, name, group=group)
    d = cache.desc
    if out is None:
        out = torch.empty_like(q)
    if lse is None:
        lse = torch.empty((d.batch * group, d.heads, q.shape[1]), dtype=torch.float32, device=q.device)
    _check_chunk_tensor(cache, out, n_frames, "out", group=group)
    if lse.dtype != torch.float32 or not lse.is_contiguous() or lse.numel() != d.batch * group * d.heads * q.shape[1]:
        raise ValueError("lse: expected contiguous fp32 [B*group, H, Nq]")
    if workspace is None:
        workspace = cache.workspace(astro_group_attn_workspace_bytes(cache, n_frames, group)[0], q.device)
    _check(_lib.astro_group_attn_fwd(cache.handle, _ptr(q), _ptr(k_chunk), _ptr(v_chunk), n_frames, group, _ptr(out),
                                     _ptr(lse), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                     _stream(stream)), "astro_group_attn_fwd")
    return out, lse


def astro_group_attn_bwd(cache: KVCache, q, k_chunk, v_chunk, out, lse, dout, n_frames: int, group: int,
                         dq=None, dk_chunk=None, dv_chunk=None, workspace=None, stream=None):
    """Returns fp32 (dq, dk_chunk, dv_chunk), each [B*group, Nq, H, D]."""
    for name, t in (("q", q), ("k_chunk", k_chunk), ("v_chunk", v_chunk), ("out", out), ("dout", dout)):
        _check_chunk_tensor(cache, t, n_frames, name, group=group)
    mk = lambda: torch.empty(q.shape, dtype=torch.float32, device=q.device)
    dq = mk() if dq is None else dq
    dk_chunk = mk() if dk_chunk is None else dk_chunk
    dv_chunk = mk() if dv_chunk is None else dv_chunk
    for name, t in (("dq", dq), ("dk_chunk", dk_chunk), ("dv_chunk", dv_chunk)):
        _check_chunk_tensor(cache, t, n_frames, name, torch.float32, group=group)
    d = cache.desc
    if lse.dtype != torch.float32 or not lse.is_contiguous() or lse.numel() != d.batch * group * d.heads * q.shape[1]:
        raise ValueError("lse: expected contiguous fp32 [B*group, H, Nq]")
    if workspace is None:
        workspace = cache.workspace(astro_group_attn_workspace_bytes(cache, n_frames, group)[1], q.device)
    _check(_lib.astro_group_attn_bwd(cache.handle, _ptr(q), _ptr(k_chunk), _ptr(v_chunk), _ptr(out), _ptr(lse),
                                     _ptr(dout), n_frames, group, _ptr(dq), _ptr(dk_chunk), _ptr(dv_chunk),
                                     _ptr(workspace), workspace.numel() * workspace.element_size(),
                                     _stream(stream)), "astro_group_attn_bwd")
    return dq, dk_chunk, dv_chunk


def astro_chunk_attn_workspace_bytes(cache: KVCache, n_frames: int):
    f, b = c_size_t(0), c_size_t(0)
    _check(_lib.astro_chunk_attn_workspace_bytes(cache.handle, n_frames, byref(f), byref(b)),
           "astro_chunk_attn_workspace_bytes")
    return f.value, b.value


def astro_chunk_attn_fwd(cache: KVCache, q, k_chunk, v_chunk, n_frames: int, out=None, lse=None,
                         workspace=None, stream=None):
    """Returns (out [B, Nq, H, D], lse [B, H, Nq] fp32)."""
    for name, t in (("q", q), ("k_chunk", k_chunk), ("v_chunk", v_chunk)):
        _check_chunk_tensor(cache, t, n_frames, name)
    d = cache.desc
    if out is None:
        out = torch.empty_like(q)
    if lse is None:
        lse = torch.empty((d.batch, d.heads, q.shape[1]), dtype=torch.float32, device=q.device)
    _check_chunk_tensor(cache, out, n_frames, "out")
    if workspace is None:
        workspace = cache.workspace(astro_chunk_attn_workspace_bytes(cache, n_frames)[0], q.device)
    _check(_lib.astro_chunk_attn_fwd(cache.handle, _ptr(q), _ptr(k_chunk), _ptr(v_chunk), n_frames, _ptr(out),
                                     _ptr(lse), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                     _stream(stream)), "astro_chunk_attn_fwd")
    return out, lse


def astro_chunk_attn_bwd(cache: KVCache, q, k_chunk, v_chunk, out, lse, dout, n_frames: int,
                         dq=None, dk_chunk=None, dv_chunk=None, workspace=None, stream=None):
    """Returns fp32 (dq, dk_chunk, dv_chunk), each [B, Nq, H, D]."""
    for name, t in (("q", q), ("k_chunk", k_chunk), ("v_chunk", v_chunk), ("out", out), ("dout", dout)):
        _check_chunk_tensor(cache, t, n_frames, name)
    mk = lambda: torch.empty(q.shape, dtype=torch.float32, device=q.device)
    dq = mk() if dq is None else dq
    dk_chunk = mk() if dk_chunk is None else dk_chunk
    dv_chunk = mk() if dv_chunk is None else dv_chunk
    for name, t in (("dq", dq), ("dk_chunk", dk_chunk), ("dv_chunk", dv_chunk)):
        _check_chunk_tensor(cache, t, n_frames, name, torch.float32)
    if lse.dtype != torch.float32 or not lse.is_contiguous():
        raise ValueError("lse: expected contiguous fp32")
    if workspace is None:
        workspace = cache.workspace(astro_chunk_attn_workspace_bytes(cache, n_frames)[1], q.device)
    _check(_lib.astro_chunk_attn_bwd(cache.handle, _ptr(q), _ptr(k_chunk), _ptr(v_chunk), _ptr(out), _ptr(lse),
                                     _ptr(dout), n_frames, _ptr(dq), _ptr(dk_chunk), _ptr(dv_chunk),
                                     _ptr(workspace), workspace.numel() * workspace.element_size(),
                                     _stream(stream)), "astro_chunk_attn_bwd")
    return dq, dk_chunk, dv_chunk


def astro_profile_begin() -> None:
    _check(_lib.astro_profile_begin(), "astro_profile_begin")


def astro_profile_end(max_entries: int = 32):
    """{kernel name: (launches, total_ms)} of the launches since astro_profile_begin."""
    buf = (astro_kernel_time_t * max_entries)()
    n = c_int32(0)
    _check(_lib.astro_profile_end(buf, max_entries, byref(n)), "astro_profile_end")
    return {buf[i].name.decode(): (buf[i].launches, float(buf[i].total_ms)) for i in range(n.value)}


def astro_calib_mfma(operands: torch.Tensor, workgroups: int, iters: int, sink: torch.Tensor, stream=None) -> None:
    """Launch the MFMA-only calibration kernel (timed via astro_profile_* as "calib_mfma_bf16")."""
    if operands.numel() * operands.element_size() < 8 * 256 * 16 or sink.numel() < workgroups * 256:
        raise ValueError("operand or sink buffer too small")
    _check(_lib.astro_calib_mfma(_ptr(operands), int(workgroups), int(iters), _ptr(sink), _stream(stream)),
           "astro_calib_mfma")


def astro_calib_copy(src: torch.Tensor, dst: torch.Tensor, stream=None) -> None:
    """Launch the streaming-copy calibration kernel (timed as "calib_copy")."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() < nbytes:
        raise ValueError("dst smaller than src")
    _check(_lib.astro_calib_copy(_ptr(src), _ptr(dst), c_size_t(nbytes), _stream(stream)), "astro_calib_copy")


def astro_nft_loss_workspace_bytes(n_samples: int, elems_per_sample: int) -> int:
    b = c_size_t(0)
    _check(_lib.astro_nft_loss_workspace_bytes(int(n_samples), int(elems_per_sample), byref(b)),
           "astro_nft_loss_workspace_bytes")
    return b.value


def astro_nft_loss(v_theta, v_old, v_ref, target, advantage, kl_mask, a_max: float, beta: float, lambda_kl: float,
                   loss=None, grad=None, workspace=None, stream=None):
    """Fused clip-level loss: tensors [n, ...] (bf16 or fp32, contiguous), advantage fp32 [n],
    kl_mask int32 [n].  Returns (loss [3] fp32 = total, policy, kl; grad fp32 like v_theta)."""
    n = v_theta.shape[0]
    elems = v_theta.numel() // n
    for name, t in (("v_old", v_old), ("v_ref", v_ref), ("target", target)):
        if t.shape != v_theta.shape or t.dtype != v_theta.dtype or not t.is_contiguous():
            raise ValueError(f"{name}: must match v_theta in shape and dtype and be contiguous")
    if v_theta.dtype not in (torch.bfloat16, torch.float32) or not v_theta.is_contiguous():
        raise ValueError("v_theta: expected contiguous bf16 or fp32")
    if advantage.dtype != torch.float32 or advantage.numel() != n or kl_mask.dtype != torch.int32 or kl_mask.numel() != n:
        raise ValueError("advantage: fp32 [n]; kl_mask: int32 [n]")
    dev = v_theta.device
    loss = torch.empty(3, dtype=torch.float32, device=dev) if loss is None else loss
    grad = torch.empty(v_theta.shape, dtype=torch.float32, device=dev) if grad is None else grad
    if grad.dtype != torch.float32 or grad.numel() != v_theta.numel() or loss.dtype != torch.float32 or loss.numel() < 3:
        raise ValueError("grad: fp32 like v_theta; loss: fp32 [3]")
    need = astro_nft_loss_workspace_bytes(n, elems)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    dtype = ASTRO_BF16 if v_theta.dtype == torch.bfloat16 else ASTRO_F32
    _check(_lib.astro_nft_loss(_ptr(v_theta), _ptr(v_old), _ptr(v_ref), _ptr(target), _ptr(advantage), _ptr(kl_mask),
                               n, elems, dtype, float(a_max), float(beta), float(lambda_kl), _ptr(loss), _ptr(grad),
                               _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)),
           "astro_nft_loss")
    return loss, grad


def astro_nft_loss_static_bytes() -> int:
    b = c_size_t(0)
    _check(_lib.astro_nft_loss_static_bytes(byref(b)), "astro_nft_loss_static_bytes")
    return b.value


def astro_nft_loss_static(v_theta, v_old, v_ref, target, advantage, kl_mask, a_max: float, beta: float, lambda_kl: float,
                          loss, grad, stream=None):
    """astro_nft_loss without a workspace (the library's static device array is the scratch).  `loss`
    (fp32 [3]) and `grad` (fp32 like v_theta) are the caller's: the call itself allocates nothing."""
    n = v_theta.shape[0]
    elems = v_theta.numel() // n
    for name, t in (("v_old", v_old), ("v_ref", v_ref), ("target", target)):
        if t.shape != v_theta.shape or t.dtype != v_theta.dtype or not t.is_contiguous():
            raise ValueError(f"{name}: must match v_theta in shape and dtype and be contiguous")
    if v_theta.dtype not in (torch.bfloat16, torch.float32) or not v_theta.is_contiguous():
        raise ValueError("v_theta: expected contiguous bf16 or fp32")
    if advantage.dtype != torch.float32 or advantage.numel() != n or kl_mask.dtype != torch.int32 or kl_mask.numel() != n:
        raise ValueError("advantage: fp32 [n]; kl_mask: int32 [n]")
    if grad.dtype != torch.float32 or grad.numel() != v_theta.numel() or loss.dtype != torch.float32 or loss.numel() < 3:
        raise ValueError("grad: fp32 like v_theta; loss: fp32 [3]")
    dtype = ASTRO_BF16 if v_theta.dtype == torch.bfloat16 else ASTRO_F32
    _check(_lib.astro_nft_loss_static(_ptr(v_theta), _ptr(v_old), _ptr(v_ref), _ptr(target), _ptr(advantage), _ptr(kl_mask),
                                      n, elems, dtype, float(a_max), float(beta), float(lambda_kl), _ptr(loss), _ptr(grad),
                                      _stream(stream)), "astro_nft_loss_static")
    return loss, grad


def astro_chunk_attn_bwd_full_workspace_bytes(cache: KVCache, n_frames: int) -> int:
    b = c_size_t(0)
    _check(_lib.astro_chunk_attn_bwd_full_workspace_bytes(cache.handle, n_frames, byref(b)),
           "astro_chunk_attn_bwd_full_workspace_bytes")
    return b.value


def astro_chunk_attn_bwd_full(cache: KVCache, q, k_chunk, v_chunk, out, lse, dout, n_frames: int,
                              dq=None, dk_chunk=None, dv_chunk=None, dk_cache=None, dv_cache=None,
                              workspace=None, stream=None):
    """The backward without the detach.  Returns fp32 (dq, dk_chunk, dv_chunk [B, Nq, H, D],
    dk_cache, dv_cache [B, C*T, H, D]); rows of empty slots of the last two stay as they were
    (zero when allocated here)."""
    for name, t in (("q", q), ("k_chunk", k_chunk), ("v_chunk", v_chunk), ("out", out), ("dout", dout)):
        _check_chunk_tensor(cache, t, n_frames, name)
    d = cache.desc
    mk = lambda: torch.empty(q.shape, dtype=torch.float32, device=q.device)
    dq = mk() if dq is None else dq
    dk_chunk = mk() if dk_chunk is None else dk_chunk
    dv_chunk = mk() if dv_chunk is None else dv_chunk
    ring_shape = (d.batch, d.capacity_frames * cache.tokens_per_frame, d.heads, d.head_dim)
    mkr = lambda: torch.zeros(ring_shape, dtype=torch.float32, device=q.device)
    dk_cache = mkr() if dk_cache is None else dk_cache
    dv_cache = mkr() if dv_cache is None else dv_cache
    for name, t in (("dq", dq), ("dk_chunk", dk_chunk), ("dv_chunk", dv_chunk)):
        _check_chunk_tensor(cache, t, n_frames, name, torch.float32)
    for name, t in (("dk_cache", dk_cache), ("dv_cache", dv_cache)):
        if tuple(t.shape) != ring_shape or t.dtype != torch.float32 or not t.is_contiguous() or not t.is_cuda:
            raise ValueError(f"{name}: expected contiguous fp32 device tensor of shape {ring_shape}")
    if lse.dtype != torch.float32 or not lse.is_contiguous():
        raise ValueError("lse: expected contiguous fp32")
    if workspace is None:
        workspace = cache.workspace(astro_chunk_attn_bwd_full_workspace_bytes(cache, n_frames), q.device)
    _check(_lib.astro_chunk_attn_bwd_full(cache.handle, _ptr(q), _ptr(k_chunk), _ptr(v_chunk), _ptr(out), _ptr(lse),
                                          _ptr(dout), n_frames, _ptr(dq), _ptr(dk_chunk), _ptr(dv_chunk),
                                          _ptr(dk_cache), _ptr(dv_cache), _ptr(workspace),
                                          workspace.numel() * workspace.element_size(), _stream(stream)),
           "astro_chunk_attn_bwd_full")
    return dq, dk_chunk, dv_chunk, dk_cache, dv_cache

"""ctypes binding of include/cacheclip.h: same calls, same argument order.

torch is used for device memory and the current HIP stream only.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libcacheclip.so"

CC_OK = 0
CC_ERR_NULL, CC_ERR_SHAPE, CC_ERR_IDX, CC_ERR_WORKSPACE, CC_ERR_HIP = -1, -2, -3, -4, -5
FLAG_NO_GROUPING, FLAG_CHECK_IDX = 1, 2
K_NAMES = ("colsum", "select", "gather_norm", "qkv", "attn", "oproj", "post_norm", "gate_up", "down",
           "assemble", "copy", "block_scores")

EXPORTS = (
    "cc_create", "cc_destroy", "cc_set_stream", "cc_last_error", "cc_select",
    "cc_step_column_scores", "cc_recompute_layer", "cc_step_gather_rmsnorm",
    "cc_step_qkv_rope_scatter", "cc_step_sparse_attention", "cc_step_oproj_residual",
    "cc_step_mlp", "cc_profile_enable", "cc_profile_read", "cc_calib_copy", "cc_assemble_cache",
    "cc_step_block_scores", "cc_select_blocks", "cc_debug_set_launch", "cc_select_noalloc",
)


class CacheClipError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"cacheclip status {status}: {msg}")
        self.status = status


class ModelDesc(C.Structure):
    _fields_ = [("d", C.c_int32), ("H_q", C.c_int32), ("H_kv", C.c_int32), ("d_h", C.c_int32),
                ("f", C.c_int32), ("rope_base", C.c_float), ("rms_eps", C.c_float),
                ("N_cap", C.c_int32), ("M_cap", C.c_int32), ("T_cap", C.c_int32)]


class _KV(C.Structure):
    _fields_ = [("K", C.c_void_p), ("V", C.c_void_p), ("stride_token", C.c_int64),
                ("stride_head", C.c_int64), ("N", C.c_int32)]


class _Chunk(C.Structure):
    _fields_ = [("K", C.c_void_p), ("V", C.c_void_p), ("len", C.c_int32)]


class _AuxBlock(C.Structure):
    _fields_ = [("attn", C.c_void_p), ("stride_head", C.c_int64), ("stride_row", C.c_int64),
                ("col0", C.c_int32), ("len", C.c_int32)]


class _Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("w_in_norm", "w_qkv", "b_qkv", "w_o", "w_post_norm",
                                          "w_gate", "w_up", "w_down")]


class LaunchOverride(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("gemm_tile", "gemm_staged", "gemm_mfma32", "gemm_gm",
                                         "gemm_splitk", "attn_splits")]


def lib_path() -> str:
    return os.path.join(_HERE, _LIB_NAME)


_lib = None


def load_library() -> C.CDLL:
    """Loads the in-tree shared library.  No fallback: a missing library is an error."""
    global _lib
    if _lib is not None:
        return _lib
    # torch first: the process must hold ONE HIP runtime, the one torch's
    # allocator and streams live in; the library binds to whichever
    # libamdhip64.so.7 is already mapped.
    import torch  # noqa: F401
    p = lib_path()
    if not os.path.exists(p):
        raise ImportError(
            f"{p} is missing: build it with `python -m paper_2510_10129_amd.build` "
            "(hipcc, gfx950). There is no CPU fallback.")
    lib = C.CDLL(p)
    vp, i32, i64, u32 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32
    lib.cc_create.argtypes = [C.POINTER(vp), C.POINTER(ModelDesc), vp]
    lib.cc_destroy.argtypes = [vp]
    lib.cc_set_stream.argtypes = [vp, vp]
    lib.cc_last_error.argtypes = [vp]
    lib.cc_last_error.restype = C.c_char_p
    lib.cc_select.argtypes = [vp, vp, i32, i32, i64, u32, i32, i32, i32, i32, i32, vp, vp,
                              C.POINTER(i32)]
    lib.cc_select_noalloc.argtypes = [vp, vp, i32, i32, i64, u32, i32, i32, i32, i32, i32, vp, vp]
    lib.cc_step_column_scores.argtypes = [vp, vp, i32, i32, i64, vp]
    lib.cc_recompute_layer.argtypes = [vp, vp, i64, vp, C.POINTER(_KV), vp, i32,
                                       C.POINTER(_Weights), vp, i32]
    lib.cc_step_gather_rmsnorm.argtypes = [vp, vp, i64, vp, i32, vp, vp]
    lib.cc_step_qkv_rope_scatter.argtypes = [vp, vp, i32, vp, vp, vp, C.POINTER(_KV), vp, i32]
    lib.cc_step_sparse_attention.argtypes = [vp, vp, i32, vp, C.POINTER(_KV), vp, i32]
    lib.cc_step_oproj_residual.argtypes = [vp, vp, i32, vp, vp, i64, vp, vp]
    lib.cc_step_mlp.argtypes = [vp, vp, i32, vp, vp, vp, vp, vp]
    lib.cc_calib_copy.argtypes = [vp, vp, vp, i64]
    lib.cc_assemble_cache.argtypes = [vp, C.POINTER(_Chunk), i32, i32, i64, i64, i32, C.POINTER(_KV)]
    lib.cc_step_block_scores.argtypes = [vp, C.POINTER(_AuxBlock), i32, i32, i32, vp]
    lib.cc_select_blocks.argtypes = [vp, C.POINTER(_AuxBlock), i32, i32, i32, u32, i32, i32, i32, i32, i32,
                                     vp, vp, C.POINTER(i32)]
    lib.cc_debug_set_launch.argtypes = [vp, C.POINTER(LaunchOverride)]
    lib.cc_profile_enable.argtypes = [vp, i32]
    lib.cc_profile_read.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(i32)]
    for name in EXPORTS:
        if name != "cc_last_error":
            getattr(lib, name).restype = i32
    _lib = lib
    return lib


def select_noalloc(attn, recomp_bp: int, window: int, tau: int, flags: int, idx_offset: int, n_tail: int,
                   idx_out, n_out, stream=None):
    """cc_select_noalloc: attn cuda fp32 [Q_a, T]; idx_out, n_out preallocated cuda int32.  Enqueues on
    `stream` (default: torch's current stream); raises CacheClipError on a non-zero status."""
    import torch
    lib = load_library()
    Q_a, T = attn.shape
    s = torch.cuda.current_stream().cuda_stream if stream is None else stream
    st = lib.cc_select_noalloc(C.c_void_p(s), attn.data_ptr(), Q_a, T, attn.stride(0), recomp_bp, window, tau,
                               flags, idx_offset, n_tail, idx_out.data_ptr(), n_out.data_ptr())
    if st != CC_OK:
        raise CacheClipError(st, (lib.cc_last_error(None) or b"").decode())


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


@dataclass
class KVLayer:
    """One layer's cache: K, V torch bf16 tensors [N, H_kv, d_h] (last dim contiguous)."""
    K: "object"
    V: "object"

    def c_struct(self) -> _KV:
        K, V = self.K, self.V
        assert K.shape == V.shape and K.stride() == V.stride() and K.stride(2) == 1
        return _KV(K.data_ptr(), V.data_ptr(), K.stride(0), K.stride(1), K.shape[0])


@dataclass
class LayerWeights:
    """Device bf16 tensors of one layer (b_qkv may be None)."""
    w_in_norm: "object"
    w_qkv: "object"
    b_qkv: "object"
    w_o: "object"
    w_post_norm: "object"
    w_gate: "object"
    w_up: "object"
    w_down: "object"

    def c_struct(self) -> _Weights:
        return _Weights(*[_ptr(getattr(self, n)) for n, _ in _Weights._fields_])


class Context:
    """Owns a cc_ctx.  Methods mirror the C entry points one to one."""

    def __init__(self, d, H_q, H_kv, d_h, f, rope_base, rms_eps, N_cap, M_cap, T_cap, stream=None):
        import torch
        self._lib = load_library()
        self.desc = ModelDesc(d, H_q, H_kv, d_h, f, rope_base, rms_eps, N_cap, M_cap, T_cap)
        self._h = C.c_void_p()
        s = torch.cuda.current_stream().cuda_stream if stream is None else stream
        st = self._lib.cc_create(C.byref(self._h), C.byref(self.desc), C.c_void_p(s))
        if st != CC_OK:
            raise CacheClipError(st, (self._lib.cc_last_error(None) or b"").decode())

    @classmethod
    def for_model(cls, model, N_cap, M_cap, T_cap, stream=None):
        return cls(model.d, model.H_q, model.H_kv, model.d_h, model.f, model.rope_base,
                   model.rms_eps, N_cap, M_cap, T_cap, stream)

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            self._lib.cc_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int):
        if st != CC_OK:
            raise CacheClipError(st, (self._lib.cc_last_error(self._h) or b"").decode())

    def set_stream(self, stream: int):
        self._check(self._lib.cc_set_stream(self._h, C.c_void_p(stream)))

    # ---- selection ----
    def select(self, attn, recomp_bp: int, window: int, tau: int = 0, flags: int = 0,
               idx_offset: int = 0, n_tail: int = 0, idx_out=None, n_out=None,
               sync: bool = True) -> Tuple["object", Optional[int]]:
        """attn: cuda fp32 [Q_a, T].  Returns (idx_out tensor, count or None)."""
        import torch
        Q_a, T = attn.shape
        if idx_out is None:
            idx_out = torch.empty(T + n_tail, dtype=torch.int32, device=attn.device)
        if n_out is None:
            n_out = torch.empty(1, dtype=torch.int32, device=attn.device)
        host = C.c_int32(-1)
        self._check(self._lib.cc_select(self._h, attn.data_ptr(), Q_a, T, attn.stride(0), recomp_bp,
                                        window, tau, flags, idx_offset, n_tail, idx_out.data_ptr(),
                                        n_out.data_ptr(), C.byref(host) if sync else None))
        return idx_out, (host.value if sync else None)

    def step_column_scores(self, attn, score):
        Q_a, T = attn.shape
        self._check(self._lib.cc_step_column_scores(self._h, attn.data_ptr(), Q_a, T, attn.stride(0),
                                                    score.data_ptr()))

    @staticmethod
    def _aux_blocks(blocks):
        """blocks: sequence of (attn cuda fp32 [H, Q_a, W], col0, len)."""
        arr = (_AuxBlock * len(blocks))()
        H = Q_a = None
        for i, (a, col0, ln) in enumerate(blocks):
            if a.dim() != 3 or a.stride(2) != 1:
                raise ValueError("a block must be [H, Q_a, W] with unit column stride")
            if H is None:
                H, Q_a = a.shape[0], a.shape[1]
            elif (a.shape[0], a.shape[1]) != (H, Q_a):
                raise ValueError("all blocks must have the same H and Q_a")
            if col0 + ln > a.shape[2]:
                raise ValueError("col0 + len exceeds the block's width")
            arr[i] = _AuxBlock(a.data_ptr(), a.stride(0), a.stride(1), col0, ln)
        return arr, H, Q_a

    def step_block_scores(self, blocks, score):
        arr, H, Q_a = self._aux_blocks(blocks)
        self._check(self._lib.cc_step_block_scores(self._h, arr, len(blocks), H, Q_a, score.data_ptr()))

    def select_blocks(self, blocks, recomp_bp: int, window: int, tau: int = 0, flags: int = 0,
                      idx_offset: int = 0, n_tail: int = 0, idx_out=None, n_out=None,
                      sync: bool = True) -> Tuple["object", Optional[int]]:
        """blocks: sequence of (attn cuda fp32 [H, Q_a, W], col0, len).  Returns (idx_out, count or None)."""
        import torch
        arr, H, Q_a = self._aux_blocks(blocks)
        T = sum(b[2] for b in blocks)
        dev = blocks[0][0].device
        if idx_out is None:
            idx_out = torch.empty(T + n_tail, dtype=torch.int32, device=dev)
        if n_out is None:
            n_out = torch.empty(1, dtype=torch.int32, device=dev)
        host = C.c_int32(-1)
        self._check(self._lib.cc_select_blocks(self._h, arr, len(blocks), H, Q_a, recomp_bp, window, tau,
                                               flags, idx_offset, n_tail, idx_out.data_ptr(),
                                               n_out.data_ptr(), C.byref(host) if sync else None))
        return idx_out, (host.value if sync else None)

    # ---- layer ----
    def recompute_layer(self, hidden, gather_idx, kv: KVLayer, idx, M: int, w: LayerWeights, out,
                        flags: int = 0):
        kvs, ws = kv.c_struct(), w.c_struct()
        self._check(self._lib.cc_recompute_layer(self._h, hidden.data_ptr(), hidden.shape[0],
                                                 _ptr(gather_idx), C.byref(kvs), idx.data_ptr(), M,
                                                 C.byref(ws), out.data_ptr(), flags))

    def step_gather_rmsnorm(self, hidden, gather_idx, M, w_norm, xn):
        self._check(self._lib.cc_step_gather_rmsnorm(self._h, hidden.data_ptr(), hidden.shape[0],
                                                     _ptr(gather_idx), M, w_norm.data_ptr(),
                                                     xn.data_ptr()))

    def step_qkv_rope_scatter(self, xn, M, idx, w_qkv, b_qkv, kv: KVLayer, q_out, flags: int = 0):
        kvs = kv.c_struct()
        self._check(self._lib.cc_step_qkv_rope_scatter(self._h, xn.data_ptr(), M, idx.data_ptr(),
                                                       w_qkv.data_ptr(), _ptr(b_qkv), C.byref(kvs),
                                                       q_out.data_ptr(), flags))

    def step_sparse_attention(self, q, M, idx, kv: KVLayer, o, flags: int = 0):
        kvs = kv.c_struct()
        self._check(self._lib.cc_step_sparse_attention(self._h, q.data_ptr(), M, idx.data_ptr(),
                                                       C.byref(kvs), o.data_ptr(), flags))

    def step_oproj_residual(self, o, M, w_o, hidden, gather_idx, y):
        self._check(self._lib.cc_step_oproj_residual(self._h, o.data_ptr(), M, w_o.data_ptr(),
                                                     hidden.data_ptr(), hidden.shape[0],
                                                     _ptr(gather_idx), y.data_ptr()))

    def step_mlp(self, y, M, w_post_norm, w_gate, w_up, w_down, out):
        self._check(self._lib.cc_step_mlp(self._h, y.data_ptr(), M, w_post_norm.data_ptr(),
                                          w_gate.data_ptr(), w_up.data_ptr(), w_down.data_ptr(),
                                          out.data_ptr()))

    # ---- cache assembly ----
    def assemble_cache(self, chunk_K: Sequence, chunk_V: Sequence, P: int, n_tail: int, dst: KVLayer):
        """chunk_K[c], chunk_V[c]: cuda bf16 [P + L_c, H_kv, d_h], all with the same strides."""
        n = len(chunk_K)
        arr = (_Chunk * n)()
        st = chunk_K[0].stride()
        for i, (K, V) in enumerate(zip(chunk_K, chunk_V)):
            assert K.shape == V.shape and K.stride() == st and V.stride() == st and st[2] == 1
            arr[i] = _Chunk(K.data_ptr(), V.data_ptr(), K.shape[0] - P)
        kvs = dst.c_struct()
        self._check(self._lib.cc_assemble_cache(self._h, arr, n, P, st[0], st[1], n_tail, C.byref(kvs)))

    # ---- measurement support ----
    def calib_copy(self, dst, src):
        self._check(self._lib.cc_calib_copy(self._h, dst.data_ptr(), src.data_ptr(),
                                            src.numel() * src.element_size()))

    # ---- test support ----
    def debug_set_launch(self, gemm_tile: str = "", gemm_staged: bool = False, gemm_mfma32: bool = False,
                         gemm_gm: int = 0, gemm_splitk: int = 0, attn_splits: int = 0):
        """Overrides the launch shapes until the next call; no arguments = the library's own choices."""
        o = LaunchOverride(ord(gemm_tile) if gemm_tile else 0, int(gemm_staged), int(gemm_mfma32), gemm_gm,
                           gemm_splitk, attn_splits)
        self._check(self._lib.cc_debug_set_launch(self._h, C.byref(o)))

    # ---- timing ----
    def profile_enable(self, on: bool):
        self._check(self._lib.cc_profile_enable(self._h, 1 if on else 0))

    def profile_read(self):
        n = len(K_NAMES)
        ms = (C.c_float * n)()
        cnt = (C.c_int32 * n)()
        self._check(self._lib.cc_profile_read(self._h, ms, cnt))
        return {K_NAMES[i]: (ms[i], cnt[i]) for i in range(n)}

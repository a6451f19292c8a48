"""ctypes binding of libflexsp.so: argument marshalling only.

Function names are those of include/flexsp.h.  Tensors are torch tensors living on the
GPU (torch is used for device memory and streams, nothing else); every step of the path
runs inside the library's HIP kernels.  There is no fallback: if the shared library is
missing the import of a symbol raises, and without a gfx950 device ``Context(0)`` raises.
"""
from __future__ import annotations

import ctypes
from ctypes import POINTER, Structure, byref, c_char_p, c_float, c_int, c_int32, c_int64, c_size_t, c_void_p
from pathlib import Path

import numpy as np

LIB_PATH = Path(__file__).resolve().parent / "libflexsp.so"

OK, INVALID_ARGUMENT, UNSUPPORTED, PLAN_MISMATCH, HIP_ERROR, OUT_OF_MEMORY, NO_DEVICE = 0, -1, -2, -3, -4, -5, -6
PASS_FWD, PASS_BWD_DKV, PASS_BWD_DQ = 0, 1, 2
BF16, F32 = 0, 1

EXPORTS = (
    "flexsp_strerror", "flexsp_last_hip_error", "flexsp_version",
    "flexsp_ctx_create", "flexsp_ctx_destroy", "flexsp_ctx_num_cu", "flexsp_ctx_num_xcd",
    "flexsp_plan_create", "flexsp_plan_destroy", "flexsp_plan_num_items", "flexsp_plan_get_items",
    "flexsp_plan_tile_rows", "flexsp_attn_bwd_workspace_bytes",
    "flexsp_pack", "flexsp_unpack", "flexsp_pack_many", "flexsp_unpack_many",
    "flexsp_attn_varlen_fwd", "flexsp_attn_varlen_bwd", "flexsp_attn_varlen_fwd_static",
    "flexsp_plan_create_kvshard", "flexsp_attn_varlen_fwd_kvshard", "flexsp_attn_varlen_fwd_kvshard_acc", "flexsp_attn_varlen_bwd_kvshard", "flexsp_lse_merge", "flexsp_lse_merge_acc",
    "flexsp_profile_start", "flexsp_profile_stop",
    "flexsp_bucket_dp", "flexsp_chunk_dp", "flexsp_min_microbatches",
)
KERNELS = ("pack", "unpack", "fwd", "bwd_delta", "bwd_dkv", "bwd_dq")


class FlexspError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().flexsp_strerror(status).decode()
        if status == HIP_ERROR:
            msg += " (hipError %d)" % lib().flexsp_last_hip_error()
        super().__init__(f"{where}: {msg} [{status}]")


class Tensor(Structure):
    _fields_ = [("ptr", c_void_p), ("stride_token", c_int64), ("stride_head", c_int64)]


class Item(Structure):
    _fields_ = [("seq_start", c_int32), ("seq_len", c_int32), ("tile", c_int32), ("head", c_int32),
                ("step_begin", c_int32), ("step_end", c_int32), ("slot", c_int32), ("parts", c_int32)]


class Profile(Structure):
    _fields_ = [("ms", ctypes.c_double * 6), ("launches", c_int64 * 6), ("dropped", c_int64)]


_lib = None


def lib() -> ctypes.CDLL:
    """Loads libflexsp.so (built in-tree by paper_2412_01523_amd.build); fails loudly if absent."""
    global _lib
    if _lib is None:
        if not LIB_PATH.exists():
            raise FileNotFoundError(
                f"{LIB_PATH} not built: run `python -m paper_2412_01523_amd.build` (needs hipcc)")
        # torch ships its own HIP runtime (soname libamdhip64.so.7).  Load it first so that this
        # library binds to the same runtime instance that owns torch's device memory and streams;
        # two runtimes in one process do not see each other's allocations.
        import torch  # noqa: F401
        L = ctypes.CDLL(str(LIB_PATH))
        L.flexsp_strerror.restype = c_char_p
        L.flexsp_strerror.argtypes = [c_int]
        L.flexsp_version.restype = c_char_p
        L.flexsp_last_hip_error.restype = c_int
        L.flexsp_ctx_create.argtypes = [POINTER(c_void_p), c_int]
        L.flexsp_ctx_destroy.argtypes = [c_void_p]
        L.flexsp_ctx_destroy.restype = None
        L.flexsp_ctx_num_cu.argtypes = [c_void_p]
        L.flexsp_ctx_num_xcd.argtypes = [c_void_p]
        L.flexsp_plan_create.argtypes = [c_void_p, c_void_p, c_int32, c_int32, c_int32, c_int32, c_int,
                                         POINTER(c_void_p)]
        L.flexsp_plan_destroy.argtypes = [c_void_p]
        L.flexsp_plan_destroy.restype = None
        L.flexsp_plan_num_items.argtypes = [c_void_p, c_int]
        L.flexsp_plan_num_items.restype = c_int64
        L.flexsp_plan_get_items.argtypes = [c_void_p, c_int, c_void_p, c_int64, c_void_p]
        L.flexsp_plan_tile_rows.argtypes = [c_void_p, c_int]
        L.flexsp_attn_bwd_workspace_bytes.argtypes = [c_void_p]
        L.flexsp_attn_bwd_workspace_bytes.restype = c_size_t
        perm = [c_void_p, c_void_p, c_void_p, c_int64, c_int32, c_int32, c_int32, c_int32, c_void_p]
        L.flexsp_pack.argtypes = perm
        L.flexsp_unpack.argtypes = perm
        many = [c_void_p, c_int32, POINTER(c_void_p), POINTER(c_void_p), c_int64, POINTER(c_int32), c_int32,
                c_int32, c_int32, c_void_p]
        L.flexsp_pack_many.argtypes = many
        L.flexsp_unpack_many.argtypes = many
        L.flexsp_attn_varlen_fwd.argtypes = [c_void_p, c_void_p, Tensor, Tensor, Tensor, c_void_p, c_int32,
                                             c_int32, c_int32, c_int32, c_int, c_float, Tensor, c_void_p,
                                             c_void_p]
        L.flexsp_attn_varlen_bwd.argtypes = [c_void_p, c_void_p, Tensor, Tensor, Tensor, Tensor, Tensor,
                                             c_void_p, c_void_p, c_int32, c_int32, c_int32, c_int32, c_int,
                                             c_float, Tensor, Tensor, Tensor, c_int32, c_void_p]
        L.flexsp_attn_varlen_fwd_static.argtypes = [c_void_p, Tensor, Tensor, Tensor, c_void_p, c_int32, c_int64,
                                                    c_int32, c_int32, c_int32, c_int32, c_int32, c_int, c_float,
                                                    Tensor, c_void_p, c_void_p]
        L.flexsp_plan_create_kvshard.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int32, c_int32, c_int32,
                                                 c_int32, c_int, POINTER(c_void_p)]
        L.flexsp_attn_varlen_fwd_kvshard.argtypes = [c_void_p, c_void_p, Tensor, Tensor, Tensor, c_int32, c_int32,
                                                     c_int32, c_int32, c_int, c_float, Tensor, c_void_p, c_void_p]
        L.flexsp_attn_varlen_fwd_kvshard_acc.argtypes = [c_void_p, c_void_p, Tensor, Tensor, Tensor, c_int32, c_int32,
                                                         c_int32, c_int32, c_int, c_float, Tensor, c_void_p, Tensor,
                                                         c_void_p]
        L.flexsp_attn_varlen_bwd_kvshard.argtypes = [c_void_p, c_void_p, Tensor, Tensor, Tensor, Tensor, Tensor, c_void_p,
                                                     c_int32, c_int32, c_int32, c_int32, c_int, c_float, Tensor, Tensor,
                                                     Tensor, c_int32, c_int32, c_void_p]
        L.flexsp_lse_merge.argtypes = [c_void_p, Tensor, c_void_p, Tensor, c_void_p, Tensor, c_void_p, c_int64,
                                       c_int32, c_int32, c_void_p]
        L.flexsp_lse_merge_acc.argtypes = [c_void_p, Tensor, c_void_p, Tensor, c_void_p, Tensor, c_int64, c_int32, c_int32,
                                           c_void_p]
        L.flexsp_bucket_dp.argtypes = [c_void_p, c_int64, c_int32, c_void_p, POINTER(c_int32), c_void_p,
                                       POINTER(c_int64)]
        L.flexsp_chunk_dp.argtypes = [c_void_p, c_int64, c_int32, c_void_p, POINTER(c_int64)]
        L.flexsp_min_microbatches.argtypes = [c_int64, c_int64]
        L.flexsp_min_microbatches.restype = c_int64
        L.flexsp_profile_start.argtypes = [c_void_p, c_int32]
        L.flexsp_profile_stop.argtypes = [c_void_p, POINTER(Profile)]
        _lib = L
    return _lib


def _check(status: int, where: str):
    if status != OK:
        raise FlexspError(status, where)


def _stream(stream) -> int:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return int(getattr(stream, "cuda_stream", stream))


def _view(t) -> Tensor:
    """[T, heads, D] torch tensor (2-byte elements, last dim contiguous) -> flexsp_tensor."""
    assert t.dim() == 3 and t.stride(2) == 1 and t.element_size() in (2, 4), "need [T,H,D], D contiguous"
    return Tensor(t.data_ptr(), t.stride(0), t.stride(1))


class Context:
    """flexsp_ctx.  device=-1 gives a host-only context (plan inspection without a GPU)."""

    def __init__(self, device: int = 0):
        self.handle = c_void_p()
        _check(lib().flexsp_ctx_create(byref(self.handle), device), "flexsp_ctx_create")
        self.device = device

    @property
    def num_cu(self) -> int:
        return lib().flexsp_ctx_num_cu(self.handle)

    @property
    def num_xcd(self) -> int:
        return lib().flexsp_ctx_num_xcd(self.handle)

    def profile_start(self, max_launches: int = 4096):
        _check(lib().flexsp_profile_start(self.handle, max_launches), "flexsp_profile_start")

    def profile_stop(self) -> dict:
        """{kernel: (total ms, launches)} for the launches since profile_start; synchronises."""
        p = Profile()
        _check(lib().flexsp_profile_stop(self.handle, byref(p)), "flexsp_profile_stop")
        out = {name: (p.ms[i], int(p.launches[i])) for i, name in enumerate(KERNELS)}
        out["dropped"] = int(p.dropped)
        return out

    def close(self):
        if self.handle:
            lib().flexsp_ctx_destroy(self.handle)
            self.handle = c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Plan:
    """flexsp_plan built from HOST cu_seqlens (int32 prefix sums)."""

    def __init__(self, ctx: Context, cu_seqlens_host, hq: int, hkv: int, d: int, causal: bool = True):
        cu = np.ascontiguousarray(cu_seqlens_host, dtype=np.int32)
        assert cu.ndim == 1 and len(cu) >= 1
        self.ctx = ctx
        self.handle = c_void_p()
        self.cu = cu
        self.hq, self.hkv, self.d, self.causal = hq, hkv, d, bool(causal)
        _check(lib().flexsp_plan_create(ctx.handle, cu.ctypes.data_as(c_void_p), len(cu) - 1, hq, hkv, d,
                                        int(bool(causal)), byref(self.handle)), "flexsp_plan_create")

    def num_items(self, which: int) -> int:
        n = lib().flexsp_plan_num_items(self.handle, which)
        if n < 0:
            raise FlexspError(int(n), "flexsp_plan_num_items")
        return int(n)

    def items(self, which: int):
        """(items as a structured numpy array, queue offsets)"""
        n = self.num_items(which)
        arr = np.zeros(n, dtype=np.dtype([("seq_start", "<i4"), ("seq_len", "<i4"), ("tile", "<i4"), ("head", "<i4"),
                                          ("step_begin", "<i4"), ("step_end", "<i4"), ("slot", "<i4"), ("parts", "<i4")]))
        offs = np.zeros(self.ctx.num_xcd + 1, dtype=np.int64)
        _check(lib().flexsp_plan_get_items(self.handle, which, arr.ctypes.data_as(c_void_p), n,
                                           offs.ctypes.data_as(c_void_p)), "flexsp_plan_get_items")
        # the packed `parts` field, unpacked for convenience
        out = np.zeros(n, dtype=np.dtype(arr.dtype.descr + [("part", "<i4"), ("nparts", "<i4")]))
        for name in arr.dtype.names:
            out[name] = arr[name]
        out["part"], out["nparts"] = arr["parts"] >> 16, arr["parts"] & 0xffff
        return out, offs

    def tile_rows(self, which: int) -> int:
        return lib().flexsp_plan_tile_rows(self.handle, which)

    @property
    def workspace_bytes(self) -> int:
        return int(lib().flexsp_attn_bwd_workspace_bytes(self.handle))

    def close(self):
        if self.handle:
            lib().flexsp_plan_destroy(self.handle)
            self.handle = c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class ShardPlan(Plan):
    """flexsp_plan for attention against one shard of the keys (flexsp_plan_create_kvshard)."""

    def __init__(self, ctx: Context, cu_q_host, cu_k_host, shift_host, hq: int, hkv: int, d: int, causal: bool = True):
        cu_q = np.ascontiguousarray(cu_q_host, dtype=np.int32)
        cu_k = np.ascontiguousarray(cu_k_host, dtype=np.int32)
        shift = np.ascontiguousarray(shift_host, dtype=np.int32)
        assert cu_q.ndim == 1 and len(cu_q) == len(cu_k) == len(shift) + 1
        self.ctx = ctx
        self.handle = c_void_p()
        self.cu, self.cu_k, self.shift = cu_q, cu_k, shift
        self.hq, self.hkv, self.d, self.causal = hq, hkv, d, bool(causal)
        _check(lib().flexsp_plan_create_kvshard(ctx.handle, cu_q.ctypes.data_as(c_void_p), cu_k.ctypes.data_as(c_void_p),
                                                shift.ctypes.data_as(c_void_p), len(shift), hq, hkv, d,
                                                int(bool(causal)), byref(self.handle)), "flexsp_plan_create_kvshard")


def flexsp_pack(ctx: Context, src, dst, P: int, stream=None):
    """src [T,H,D] -> dst [P,T,H/P,D] (dense torch tensors on the context's GPU)."""
    T, H, D = src.shape
    assert src.is_contiguous() and dst.is_contiguous() and dst.numel() == src.numel()
    _check(lib().flexsp_pack(ctx.handle, src.data_ptr(), dst.data_ptr(), T, H, D, P, src.element_size(),
                             _stream(stream)), "flexsp_pack")


def flexsp_unpack(ctx: Context, src, dst, stream=None):
    """src [P,T,Hp,D] -> dst [T,P*Hp,D]."""
    P, T, Hp, D = src.shape
    assert src.is_contiguous() and dst.is_contiguous() and dst.numel() == src.numel()
    _check(lib().flexsp_unpack(ctx.handle, src.data_ptr(), dst.data_ptr(), T, P * Hp, D, P,
                               src.element_size(), _stream(stream)), "flexsp_unpack")


def _many(fn, name, ctx, srcs, dsts, T, heads, D, P, stream):
    n = len(srcs)
    assert n == len(dsts) and all(s.is_contiguous() and d.is_contiguous() and s.numel() == d.numel()
                                  for s, d in zip(srcs, dsts))
    eb = srcs[0].element_size()
    assert all(s.element_size() == eb for s in srcs)
    sp = (c_void_p * n)(*[s.data_ptr() for s in srcs])
    dp = (c_void_p * n)(*[d.data_ptr() for d in dsts])
    hh = (c_int32 * n)(*heads)
    _check(fn(ctx.handle, n, sp, dp, T, hh, D, P, eb, _stream(stream)), name)


def flexsp_pack_many(ctx: Context, srcs, dsts, P: int, stream=None):
    """Several src [T,H_i,D] -> dst [P,T,H_i/P,D] in one launch (same T, D, element size)."""
    T, _, D = srcs[0].shape
    assert all(s.shape[0] == T and s.shape[2] == D for s in srcs)
    _many(lib().flexsp_pack_many, "flexsp_pack_many", ctx, srcs, dsts, T, [s.shape[1] for s in srcs], D, P, stream)


def flexsp_unpack_many(ctx: Context, srcs, dsts, stream=None):
    """Several src [P,T,Hp_i,D] -> dst [T,P*Hp_i,D] in one launch."""
    P, T, _, D = srcs[0].shape
    assert all(s.shape[0] == P and s.shape[1] == T and s.shape[3] == D for s in srcs)
    _many(lib().flexsp_unpack_many, "flexsp_unpack_many", ctx, srcs, dsts, T, [P * s.shape[2] for s in srcs], D, P,
          stream)


def flexsp_attn_varlen_fwd(ctx: Context, plan: Plan, q, k, v, cu_seqlens_dev, o, lse, *, head_begin=0,
                           head_count=None, kv_head_begin=0, kv_head_count=None, causal=True,
                           softmax_scale=0.0, stream=None):
    head_count = plan.hq if head_count is None else head_count
    kv_head_count = plan.hkv if kv_head_count is None else kv_head_count
    _check(lib().flexsp_attn_varlen_fwd(ctx.handle, plan.handle, _view(q), _view(k), _view(v),
                                        None if cu_seqlens_dev is None else cu_seqlens_dev.data_ptr(), head_begin,
                                        head_count, kv_head_begin,
                                        kv_head_count, int(bool(causal)), float(softmax_scale), _view(o),
                                        lse.data_ptr(), _stream(stream)), "flexsp_attn_varlen_fwd")


def flexsp_attn_varlen_bwd(ctx: Context, plan: Plan, q, k, v, o, dO, lse, cu_seqlens_dev, dq, dk, dv, *,
                           head_begin=0, head_count=None, kv_head_begin=0, kv_head_count=None, causal=True,
                           softmax_scale=0.0, stream=None):
    head_count = plan.hq if head_count is None else head_count
    kv_head_count = plan.hkv if kv_head_count is None else kv_head_count
    assert dq.element_size() == dk.element_size() == dv.element_size()
    grad_dtype = F32 if dq.element_size() == 4 else BF16      # gradient tensors are bf16 or fp32
    _check(lib().flexsp_attn_varlen_bwd(ctx.handle, plan.handle, _view(q), _view(k), _view(v), _view(o),
                                        _view(dO), lse.data_ptr(),
                                        None if cu_seqlens_dev is None else cu_seqlens_dev.data_ptr(), head_begin,
                                        head_count, kv_head_begin, kv_head_count, int(bool(causal)),
                                        float(softmax_scale), _view(dq), _view(dk), _view(dv),
                                        grad_dtype, _stream(stream)), "flexsp_attn_varlen_bwd")


def flexsp_attn_varlen_fwd_kvshard(ctx: Context, plan: ShardPlan, q, k, v, o, lse, *, head_begin=0, head_count=None,
                                   kv_head_begin=0, kv_head_count=None, causal=True, softmax_scale=0.0, stream=None):
    head_count = plan.hq if head_count is None else head_count
    kv_head_count = plan.hkv if kv_head_count is None else kv_head_count
    _check(lib().flexsp_attn_varlen_fwd_kvshard(ctx.handle, plan.handle, _view(q), _view(k), _view(v), head_begin,
                                                head_count, kv_head_begin, kv_head_count, int(bool(causal)),
                                                float(softmax_scale), _view(o), lse.data_ptr(), _stream(stream)),
           "flexsp_attn_varlen_fwd_kvshard")


def flexsp_attn_varlen_fwd_kvshard_acc(ctx: Context, plan: ShardPlan, q, k, v, o_acc, lse_acc, o_bf16=None, *, head_begin=0,
                                       head_count=None, kv_head_begin=0, kv_head_count=None, causal=True,
                                       softmax_scale=0.0, stream=None):
    """o_acc [Tq,Hq,D] fp32 view and lse_acc [Hq,Tq] fp32: the ring's running result, updated in place; o_bf16:
    optional bf16 [Tq,Hq,D] view that receives the merged rows rounded once."""
    import torch
    assert o_acc.dtype == torch.float32 and lse_acc.is_contiguous()
    head_count = plan.hq if head_count is None else head_count
    kv_head_count = plan.hkv if kv_head_count is None else kv_head_count
    _check(lib().flexsp_attn_varlen_fwd_kvshard_acc(ctx.handle, plan.handle, _view(q), _view(k), _view(v), head_begin,
                                                    head_count, kv_head_begin, kv_head_count, int(bool(causal)),
                                                    float(softmax_scale), _view(o_acc), lse_acc.data_ptr(),
                                                    Tensor(None, 0, 0) if o_bf16 is None else _view(o_bf16),
                                                    _stream(stream)), "flexsp_attn_varlen_fwd_kvshard_acc")


def flexsp_attn_varlen_bwd_kvshard(ctx: Context, plan: ShardPlan, q, k, v, o, dO, lse, dq, dk, dv, *, head_begin=0,
                                   head_count=None, kv_head_begin=0, kv_head_count=None, causal=True, softmax_scale=0.0,
                                   grad_dtype=None, accumulate=False, stream=None):
    """lse [Hq,Tq] and o: those of the COMPLETE attention; dq [Tq,Hq,D], dk / dv [Tk,Hkv,D] (see include/flexsp.h)."""
    import torch
    head_count = plan.hq if head_count is None else head_count
    kv_head_count = plan.hkv if kv_head_count is None else kv_head_count
    if grad_dtype is None:
        grad_dtype = F32 if dq.dtype == torch.float32 else BF16
    _check(lib().flexsp_attn_varlen_bwd_kvshard(ctx.handle, plan.handle, _view(q), _view(k), _view(v), _view(o), _view(dO),
                                                lse.data_ptr(), head_begin, head_count, kv_head_begin, kv_head_count,
                                                int(bool(causal)), float(softmax_scale), _view(dq), _view(dk), _view(dv),
                                                grad_dtype, int(bool(accumulate)), _stream(stream)),
           "flexsp_attn_varlen_bwd_kvshard")


def flexsp_lse_merge(ctx: Context, o_a, lse_a, o_b, lse_b, o_out, lse_out, stream=None):
    """o_* [T,H,D] bf16 views, lse_* [H,T] fp32 contiguous; o_out / lse_out may be one of the inputs."""
    T, H, D = o_a.shape
    assert o_b.shape == o_a.shape == o_out.shape and lse_a.shape == lse_b.shape == lse_out.shape == (H, T)
    assert lse_a.is_contiguous() and lse_b.is_contiguous() and lse_out.is_contiguous()
    _check(lib().flexsp_lse_merge(ctx.handle, _view(o_a), lse_a.data_ptr(), _view(o_b), lse_b.data_ptr(), _view(o_out),
                                  lse_out.data_ptr(), T, H, D, _stream(stream)), "flexsp_lse_merge")


def flexsp_lse_merge_acc(ctx: Context, o_acc, lse_acc, o_b, lse_b, o_bf16=None, stream=None):
    """o_acc [T,H,D] fp32 view and lse_acc [H,T] fp32: the running result, updated in place; o_b bf16 view, lse_b
    [H,T] fp32: the new part; o_bf16: optional bf16 [T,H,D] view that receives the merged rows rounded once."""
    import torch
    T, H, D = o_acc.shape
    assert o_acc.dtype == torch.float32 and o_b.shape == o_acc.shape and lse_acc.shape == lse_b.shape == (H, T)
    assert lse_acc.is_contiguous() and lse_b.is_contiguous()
    none = Tensor(None, 0, 0)
    _check(lib().flexsp_lse_merge_acc(ctx.handle, _view(o_acc), lse_acc.data_ptr(), _view(o_b), lse_b.data_ptr(),
                                      none if o_bf16 is None else _view(o_bf16), T, H, D, _stream(stream)),
           "flexsp_lse_merge_acc")


def flexsp_attn_varlen_fwd_static(ctx: Context, q, k, v, cu_seqlens_dev, o, lse, *, head_begin=0, head_count=None,
                                  kv_head_begin=0, kv_head_count=None, causal=True, softmax_scale=0.0,
                                  stream=None):
    """The forward without a plan and without any allocation (queues built on the device)."""
    head_count = q.shape[1] - head_begin if head_count is None else head_count
    kv_head_count = k.shape[1] - kv_head_begin if kv_head_count is None else kv_head_count
    _check(lib().flexsp_attn_varlen_fwd_static(ctx.handle, _view(q), _view(k), _view(v), cu_seqlens_dev.data_ptr(),
                                               cu_seqlens_dev.numel() - 1, q.shape[0], head_begin, head_count,
                                               kv_head_begin, kv_head_count, q.shape[2], int(bool(causal)),
                                               float(softmax_scale), _view(o), lse.data_ptr(), _stream(stream)),
           "flexsp_attn_varlen_fwd_static")


# ----------------------------------------------------------------------------- planner pieces (host only)
def flexsp_bucket_dp(lens, Q: int = 16):
    """(limits, bucket_of, error): at most Q buckets with minimal total deviation from the upper limits."""
    s = np.ascontiguousarray(lens, dtype=np.int64)
    limits = np.zeros(max(Q, 1), dtype=np.int64)
    bucket_of = np.zeros(len(s), dtype=np.int32)
    nb, err = c_int32(0), c_int64(0)
    _check(lib().flexsp_bucket_dp(s.ctypes.data, len(s), Q, limits.ctypes.data, byref(nb), bucket_of.ctypes.data,
                                  byref(err)), "flexsp_bucket_dp")
    return limits[:nb.value].copy(), bucket_of, int(err.value)


def flexsp_chunk_dp(lens, M: int):
    """(ends, max_tokens): M consecutive non-empty micro-batches with the smallest possible largest token count."""
    s = np.ascontiguousarray(lens, dtype=np.int64)
    ends = np.zeros(max(M, 1), dtype=np.int64)
    mx = c_int64(0)
    _check(lib().flexsp_chunk_dp(s.ctypes.data, len(s), M, ends.ctypes.data, byref(mx)), "flexsp_chunk_dp")
    return ends[:M].copy(), int(mx.value)


def flexsp_min_microbatches(batch_tokens: int, cluster_token_capacity: int) -> int:
    r = lib().flexsp_min_microbatches(batch_tokens, cluster_token_capacity)
    if r < 0:
        raise FlexspError(int(r), "flexsp_min_microbatches")
    return int(r)

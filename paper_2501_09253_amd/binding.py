"""ctypes binding of the C ABI in include/pserve.h: argument marshalling only.

Every step of the path runs in the HIP kernels of libpserve.so; torch is used for device
memory and streams.  There is no CPU fallback: if the library is missing, loading fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))

F32, BF16 = 0, 1
MSE_STATIC_MAX_PATCHES = 16384      # PSERVE_MSE_STATIC_MAX_PATCHES
STAGE_KIND = {"RES1": 1, "RES2": 2, "SATTN": 3, "XATTN": 4, "FFN": 5, "LSATTN": 6, "LXATTN": 7, "LFFN": 8, "RES2T": 9, "ASATTN": 10, "AMLP": 11, "MMDIT": 12}
TABLES = {"perm": 0, "request_offset": 1, "res_offset": 2, "res_hw": 3, "patch_owner": 4,
          "patch_rc": 5, "neighbour": 6, "halo_src": 7, "cu_seqlens": 8, "seq_len": 9}
SLOT_H1, SLOT_R, SLOT_K, SLOT_V, SLOT_Y = 0, 1, 2, 3, 4
MAX_STAGES, MAX_PARAMS = 8, 24

# parameter order per stage kind (same as the header)
PARAM_ORDER = {
    "RES1": ["gn_g", "gn_b", "conv_w", "conv_b"],
    "RES2": ["gn_a_g", "gn_a_b", "conv_a_w", "conv_a_b", "gn_b_g", "gn_b_b", "conv_b_w", "conv_b_b"],
    "SATTN": ["gn_g", "gn_b", "wq", "wk", "wv", "wo", "bo"],
    "XATTN": ["wq", "wk", "wv", "wo", "bo"],
    "FFN": ["w1", "b1", "w2", "b2"],
    "LSATTN": ["ln_g", "ln_b", "wq", "wk", "wv", "wo", "bo"],
    "LXATTN": ["ln_g", "ln_b", "wq", "wk", "wv", "wo", "bo"],
    "LFFN": ["ln_g", "ln_b", "w1", "b1", "w2", "b2"],
    "MMDIT": [X + "." + n for X in ("img", "txt") for n in ("wm", "bm", "wq", "wk", "wv", "wo", "bo", "w1", "b1", "w2", "b2")],
    "ASATTN": ["wm", "bm", "wq", "wk", "wv", "wo", "bo"],
    "AMLP": ["wm", "bm", "w1", "b1", "w2", "b2"],
    "RES2T": ["gn_a_g", "gn_a_b", "conv_a_w", "conv_a_b", "gn_b_g", "gn_b_b", "conv_b_w", "conv_b_b", "wt", "bt"],
}


class PserveError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"pserve status {status}: {msg}")
        self.status = status


class _PlanInfo(C.Structure):
    _fields_ = [("n", C.c_int32), ("R", C.c_int32), ("P", C.c_int32), ("ph", C.c_int32), ("pw", C.c_int32),
                ("ring", C.c_int32), ("T", C.c_int64), ("text_len", C.c_int32), ("text_patches", C.c_int32)]


class _BlockDesc(C.Structure):
    _fields_ = [("n_stages", C.c_int32), ("stages", C.c_int32 * MAX_STAGES), ("C", C.c_int32), ("G", C.c_int32),
                ("heads", C.c_int32), ("dtype", C.c_int32), ("eps", C.c_float), ("ctx_len", C.c_int32),
                ("ctx_dim", C.c_int32), ("ffn_mult", C.c_int32), ("temb_dim", C.c_int32)]


class _ProfEntry(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("calls", C.c_int32), ("total_ms", C.c_float)]


class _Task(C.Structure):
    _fields_ = [("id", C.c_int64), ("H", C.c_int32), ("W", C.c_int32), ("steps_left", C.c_int32),
                ("arrival", C.c_double), ("ddl", C.c_double), ("standalone", C.c_double)]


class _LatencyModel(C.Structure):
    _fields_ = [("w", C.c_double * 4)]


class _BlockParams(C.Structure):
    _fields_ = [("p", (C.c_void_p * MAX_PARAMS) * MAX_STAGES)]


def library_path() -> str:
    return os.path.join(_HERE, "libpserve.so")


_lib = None


def lib() -> C.CDLL:
    """Load libpserve.so (built by paper_2501_09253_amd.build); fails loudly if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} not found: build it with `python -m paper_2501_09253_amd.build` "
                          "(there is no CPU fallback)")
    L = C.CDLL(path)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    L.pserve_last_error.restype = C.c_char_p
    L.pserve_last_error.argtypes = []
    L.pserve_plan.argtypes = [C.POINTER(i32), i32, i32, i32, vp, C.POINTER(vp)]
    L.pserve_plan_free.argtypes = [vp]
    L.pserve_plan_free.restype = None
    L.pserve_plan_info.argtypes = [vp, C.POINTER(_PlanInfo)]
    L.pserve_plan_table.argtypes = [vp, C.c_int, C.c_int, C.POINTER(C.POINTER(i32)), C.POINTER(i64)]
    L.pserve_plan_text.argtypes = [C.POINTER(i32), i32, i32, i32, i32, vp, C.POINTER(vp)]
    L.pserve_text_scatter.argtypes = [vp, vp, i32, C.c_int, vp, vp]
    L.pserve_text_gather.argtypes = [vp, vp, i32, C.c_int, vp, vp]
    L.pserve_split.argtypes = [vp, C.POINTER(vp), i32, C.c_int, vp, vp]
    L.pserve_split_stats.argtypes = [vp, C.POINTER(vp), i32, C.c_int, vp, vp, vp]
    L.pserve_reassemble.argtypes = [vp, vp, i32, C.c_int, C.POINTER(vp), vp]
    L.pserve_block_create.argtypes = [C.POINTER(_BlockDesc), C.POINTER(_BlockParams), vp, C.POINTER(vp)]
    L.pserve_block_free.argtypes = [vp]
    L.pserve_block_free.restype = None
    L.pserve_cache_create.argtypes = [vp, vp, C.c_int, C.POINTER(vp)]
    L.pserve_cache_free.argtypes = [vp]
    L.pserve_cache_free.restype = None
    L.pserve_cache_load.argtypes = [vp, C.c_int, C.c_int, vp, vp]
    L.pserve_cache_read.argtypes = [vp, C.c_int, C.c_int, vp, vp]
    L.pserve_block_forward.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp]
    L.pserve_block_forward_temb.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp]
    L.pserve_set_kernel_mode.argtypes = [C.c_int]
    L.pserve_profile_enable.argtypes = [C.c_int]
    L.pserve_profile_select.argtypes = [C.c_char_p]
    L.pserve_profile_sample.argtypes = [C.c_int]
    L.pserve_patch_mse.argtypes = [vp, vp, vp, i32, C.c_int, vp, vp]
    L.pserve_patch_mse_static.argtypes = [vp, vp, vp, i32, C.c_int, vp, vp]
    L.pserve_probe_mfma_bf16.argtypes = [C.c_int, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double), vp]
    L.pserve_probe_mfma_mix.argtypes = [C.c_int, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double), vp]
    L.pserve_probe_copy.argtypes = [vp, vp, C.c_size_t, C.c_int, C.POINTER(C.c_double), vp]
    L.pserve_cache_sets.argtypes = [vp, C.POINTER(C.c_int64), vp, C.POINTER(C.c_int64), C.POINTER(i32),
                                    C.POINTER(C.c_uint8), vp, vp]
    L.pserve_cache_migrate.argtypes = [vp, vp, vp, vp, vp]
    L.pserve_profile_read.argtypes = [C.POINTER(_ProfEntry), i32, C.POINTER(i32)]
    L.pserve_latency_predict.argtypes = [C.POINTER(_LatencyModel), C.POINTER(_Task), i32, i32, i32, C.POINTER(C.c_double)]
    L.pserve_latency_fit.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_double), i32, C.POINTER(_LatencyModel)]
    L.pserve_slack.argtypes = [C.POINTER(_Task), C.c_double, C.c_double, C.POINTER(C.c_double)]
    L.pserve_schedule.argtypes = [C.POINTER(_Task), i32, C.POINTER(_Task), i32, C.c_double, C.POINTER(_LatencyModel), i32, i32,
                                  C.c_double, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]
    L.pserve_resample_create.argtypes = [C.c_int, i32, i32, C.c_int, vp, vp, vp, C.POINTER(vp)]
    L.pserve_resample_free.argtypes = [vp]
    L.pserve_resample_free.restype = None
    L.pserve_resample_workspace.argtypes = [vp, vp, C.POINTER(C.c_size_t)]
    L.pserve_resample_forward.argtypes = [vp, vp, vp, vp, vp, C.c_size_t, vp, vp]
    _lib = L
    return L


def _check(status: int):
    if status != 0:
        raise PserveError(status, lib().pserve_last_error().decode())


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _torch_dtype(dtype: int):
    import torch
    return torch.bfloat16 if dtype == BF16 else torch.float32


def set_kernel_mode(mode: int):
    """0 = fastest kernels for the shapes, 1 = plain reference kernels only."""
    _check(lib().pserve_set_kernel_mode(mode))


def profile_enable(on: bool):
    """Bracket every kernel of pserve_block_forward with HIP events (pserve_profile_enable)."""
    _check(lib().pserve_profile_enable(int(on)))


def profile_select(label: Optional[str]):
    """Time only the kernels with this label; None = all kernels (pserve_profile_select)."""
    _check(lib().pserve_profile_select(None if not label else label.encode()))


def profile_sample(every: int):
    """Bracket the kernels of every n-th forward call only (pserve_profile_sample)."""
    _check(lib().pserve_profile_sample(int(every)))


def probe_mfma_bf16(iters: int = 20000, random_operands: bool = False):
    """pserve_probe_mfma_bf16: (dense bf16 TFLOP/s of a register-resident MFMA stream, shader clock in MHz inside it)."""
    out, mhz = C.c_double(0.0), C.c_double(0.0)
    _check(lib().pserve_probe_mfma_bf16(iters, 1 if random_operands else 0, C.byref(out), C.byref(mhz), _stream()))
    return out.value, mhz.value


def probe_mfma_mix(mix: int, iters: int = 20000):
    """pserve_probe_mfma_mix: (bf16 TFLOP/s of the 32 x 32 x 16 MFMAs, shader clock in MHz) of an MFMA stream on
    standard-normal operands with the instruction mix `mix` between the MFMAs (19: attention inner loop, 8: convolution)."""
    out, mhz = C.c_double(0.0), C.c_double(0.0)
    _check(lib().pserve_probe_mfma_mix(iters, int(mix), C.byref(out), C.byref(mhz), _stream()))
    return out.value, mhz.value


def probe_copy(dst, src, reps: int = 5) -> float:
    """pserve_probe_copy: GB/s (read + written) of a plain copy between two equally sized device tensors."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes and src.is_contiguous() and dst.is_contiguous()
    out = C.c_double(0.0)
    _check(lib().pserve_probe_copy(dst.data_ptr(), src.data_ptr(), nbytes, reps, C.byref(out), _stream()))
    return out.value


def profile_read() -> Dict[str, Dict[str, float]]:
    """Collect {kernel label: {"calls": n, "total_ms": t}} since the last read (pserve_profile_read)."""
    buf = (_ProfEntry * 64)()
    n = C.c_int32()
    _check(lib().pserve_profile_read(buf, 64, C.byref(n)))
    return {buf[i].name.decode(): {"calls": int(buf[i].calls), "total_ms": float(buf[i].total_ms)}
            for i in range(n.value)}


class Plan:
    """pserve_plan: Compressed Sparse Patch tables of one batch composition."""

    def __init__(self, resolutions: Sequence[Sequence[int]], ph: int = 0, pw: int = 0, text_len: int = 0):
        res = np.ascontiguousarray(np.asarray(resolutions, dtype=np.int32).reshape(-1, 2))
        self._h = C.c_void_p()
        _check(lib().pserve_plan_text(res.ctypes.data_as(C.POINTER(C.c_int32)), res.shape[0], ph, pw, text_len, _stream(),
                                      C.byref(self._h)))
        info = _PlanInfo()
        _check(lib().pserve_plan_info(self._h, C.byref(info)))
        self.n, self.R, self.P, self.ph, self.pw, self.ring, self.T = (info.n, info.R, info.P, info.ph, info.pw,
                                                                      info.ring, info.T)
        self.text_len, self.text_patches = info.text_len, info.text_patches
        self.resolutions = [tuple(int(v) for v in r) for r in res]

    def text_scatter(self, text, x):
        """pserve_text_scatter: text [n, text_len, C] (caller order) into the text patches of x[T, C] (in place)."""
        assert text.is_contiguous() and x.is_contiguous() and text.dtype == x.dtype
        assert tuple(text.shape) == (self.n, self.text_len, x.shape[1]) and x.shape[0] == self.T
        import torch
        dt = BF16 if x.dtype == torch.bfloat16 else F32
        _check(lib().pserve_text_scatter(self._h, text.data_ptr(), x.shape[1], dt, x.data_ptr(), _stream()))
        return x

    def text_gather(self, x):
        """pserve_text_gather: the text tokens of every request out of x[T, C]: [n, text_len, C] in caller order."""
        import torch
        assert x.is_contiguous() and x.shape[0] == self.T
        out = torch.empty((self.n, self.text_len, x.shape[1]), dtype=x.dtype, device=x.device)
        dt = BF16 if x.dtype == torch.bfloat16 else F32
        _check(lib().pserve_text_gather(self._h, x.data_ptr(), x.shape[1], dt, out.data_ptr(), _stream()))
        return out

    def table(self, name: str) -> np.ndarray:
        """Host mirror of a table as a numpy int32 array (copy)."""
        ptr = C.POINTER(C.c_int32)()
        cnt = C.c_int64()
        _check(lib().pserve_plan_table(self._h, TABLES[name], 0, C.byref(ptr), C.byref(cnt)))
        a = np.ctypeslib.as_array(ptr, shape=(cnt.value,)).copy()
        shape = {"res_hw": (-1, 2), "patch_rc": (-1, 2), "neighbour": (-1, 8), "halo_src": (self.P, -1)}.get(name)
        return a.reshape(shape) if shape else a

    def table_device_ptr(self, name: str) -> int:
        ptr = C.POINTER(C.c_int32)()
        cnt = C.c_int64()
        _check(lib().pserve_plan_table(self._h, TABLES[name], 1, C.byref(ptr), C.byref(cnt)))
        return C.cast(ptr, C.c_void_p).value

    def split(self, images, out=None, cache=None):
        """Per-request NCHW device tensors (caller order) -> patch-major token matrix x[T, C].  With `cache` (a Cache of
        this plan) the pass also leaves the input's GroupNorm moments behind for the cache's next forward call on x
        (pserve_split_stats)."""
        import torch
        Cc = images[0].shape[0]
        dt = BF16 if images[0].dtype == torch.bfloat16 else F32
        if out is None:
            out = torch.empty((self.T, Cc), dtype=images[0].dtype, device=images[0].device)
        ptrs = (C.c_void_p * self.n)(*[im.data_ptr() for im in images])
        for im, (h, w) in zip(images, self.resolutions):
            assert im.is_contiguous() and tuple(im.shape) == (Cc, h, w) and im.dtype == images[0].dtype
        if cache is not None:
            _check(lib().pserve_split_stats(self._h, ptrs, Cc, dt, out.data_ptr(), cache._h, _stream()))
        else:
            _check(lib().pserve_split(self._h, ptrs, Cc, dt, out.data_ptr(), _stream()))
        return out

    def reassemble(self, y, images=None):
        """Patch-major y[T, C] -> per-request NCHW tensors in caller order."""
        import torch
        Cc = y.shape[1]
        dt = BF16 if y.dtype == torch.bfloat16 else F32
        assert y.is_contiguous() and y.shape[0] == self.T
        if images is None:
            images = [torch.empty((Cc, h, w), dtype=y.dtype, device=y.device) for h, w in self.resolutions]
        ptrs = (C.c_void_p * self.n)(*[im.data_ptr() for im in images])
        _check(lib().pserve_reassemble(self._h, y.data_ptr(), Cc, dt, ptrs, _stream()))
        return images

    def patch_mse(self, a, b):
        """pserve_patch_mse: per-patch mean squared error of two patch batches [T, C] -> float32 [P] (plan order)."""
        import torch
        assert a.shape == b.shape and a.dtype == b.dtype and a.is_contiguous() and b.is_contiguous() and a.shape[0] == self.T
        out = torch.empty(self.P, dtype=torch.float32, device=a.device)
        dt = BF16 if a.dtype == torch.bfloat16 else F32
        _check(lib().pserve_patch_mse(self._h, a.data_ptr(), b.data_ptr(), a.shape[1], dt, out.data_ptr(), _stream()))
        return out

    def patch_mse_static(self, a, b, out=None):
        """pserve_patch_mse_static: the same result through the library's fixed device scratch; allocates nothing when
        `out` (float32 [P]) is given."""
        import torch
        assert a.shape == b.shape and a.dtype == b.dtype and a.is_contiguous() and b.is_contiguous() and a.shape[0] == self.T
        if out is None:
            out = torch.empty(self.P, dtype=torch.float32, device=a.device)
        dt = BF16 if a.dtype == torch.bfloat16 else F32
        _check(lib().pserve_patch_mse_static(self._h, a.data_ptr(), b.data_ptr(), a.shape[1], dt, out.data_ptr(), _stream()))
        return out

    def cache_sets(self, ids, old_plan: "Plan", old_ids):
        """pserve_cache_sets with this plan as the new batch: returns (req_src, expired, patch_src device tensor)."""
        import torch
        new_ids = np.ascontiguousarray(np.asarray(ids, dtype=np.int64))
        prev_ids = np.ascontiguousarray(np.asarray(old_ids, dtype=np.int64))
        assert new_ids.shape == (self.n,) and prev_ids.shape == (old_plan.n,)
        req_src = np.empty(self.n, dtype=np.int32)
        expired = np.empty(old_plan.n, dtype=np.uint8)
        patch_src = torch.empty(self.P, dtype=torch.int32, device="cuda")
        _check(lib().pserve_cache_sets(old_plan._h, prev_ids.ctypes.data_as(C.POINTER(C.c_int64)), self._h,
                                       new_ids.ctypes.data_as(C.POINTER(C.c_int64)),
                                       req_src.ctypes.data_as(C.POINTER(C.c_int32)),
                                       expired.ctypes.data_as(C.POINTER(C.c_uint8)), patch_src.data_ptr(), _stream()))
        return req_src, expired, patch_src

    def close(self):
        if self._h:
            lib().pserve_plan_free(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Block:
    """pserve_block: block description + packed weights (params: per stage dict name -> device tensor)."""

    def __init__(self, stages: Sequence[str], params: List[Dict[str, "object"]], *, C_: int, G: int, heads: int,
                 dtype: int, eps: float = 1e-5, ctx_len: int = 0, ctx_dim: int = 0, ffn_mult: int = 4, temb_dim: int = 0):
        desc = _BlockDesc()
        desc.n_stages = len(stages)
        for i, s in enumerate(stages):
            desc.stages[i] = STAGE_KIND[s]
        desc.C, desc.G, desc.heads, desc.dtype, desc.eps = C_, G, heads, dtype, eps
        desc.ctx_len, desc.ctx_dim, desc.ffn_mult, desc.temb_dim = ctx_len, ctx_dim, ffn_mult, temb_dim
        bp = _BlockParams()
        keep = []
        for i, (s, p) in enumerate(zip(stages, params)):
            for k, name in enumerate(PARAM_ORDER[s]):
                t = p[name]
                assert t.is_contiguous() and t.dtype == _torch_dtype(dtype), (s, name, t.dtype)
                keep.append(t)
                bp.p[i][k] = t.data_ptr()
        self._h = C.c_void_p()
        _check(lib().pserve_block_create(C.byref(desc), C.byref(bp), _stream(), C.byref(self._h)))
        self.stages, self.C, self.dtype = tuple(stages), C_, dtype

    def close(self):
        if self._h:
            lib().pserve_block_free(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Cache:
    """pserve_cache: cached operand tensors + scratch of one (plan, block) pair."""

    def __init__(self, plan: Plan, block: Block, with_slots: bool = False):
        self._h = C.c_void_p()
        _check(lib().pserve_cache_create(plan._h, block._h, int(with_slots), C.byref(self._h)))
        self.plan, self.block = plan, block

    def load(self, stage: int, slot: int, src):
        assert src.is_contiguous() and tuple(src.shape) == (self.plan.T, self.block.C)
        _check(lib().pserve_cache_load(self._h, stage, slot, src.data_ptr(), _stream()))

    def read(self, stage: int, slot: int):
        import torch
        dst = torch.empty((self.plan.T, self.block.C), dtype=_torch_dtype(self.block.dtype), device="cuda")
        _check(lib().pserve_cache_read(self._h, stage, slot, dst.data_ptr(), _stream()))
        return dst

    def migrate_from(self, old_cache: "Cache", patch_src):
        """pserve_cache_migrate: take the Common Set's slots from the cache of the previous batch; returns valid[P]."""
        import torch
        assert patch_src.dtype == torch.int32 and patch_src.numel() == self.plan.P and patch_src.is_contiguous()
        valid = torch.empty(self.plan.P, dtype=torch.uint8, device="cuda")
        _check(lib().pserve_cache_migrate(old_cache._h, self._h, patch_src.data_ptr(), valid.data_ptr(), _stream()))
        return valid

    def forward(self, x, ctx=None, reuse_mask=None, y=None, temb=None):
        """pserve_block_forward (pserve_block_forward_temb when temb is given) on the current torch stream; returns y[T, C]."""
        import torch
        assert x.is_contiguous() and tuple(x.shape) == (self.plan.T, self.block.C)
        assert x.dtype == _torch_dtype(self.block.dtype)
        if y is None:
            y = torch.empty_like(x)
        if ctx is not None:
            assert ctx.is_contiguous() and ctx.dtype == x.dtype
        if reuse_mask is not None:
            assert reuse_mask.dtype == torch.uint8 and reuse_mask.numel() == self.plan.P and reuse_mask.is_contiguous()
        mask_p = reuse_mask.data_ptr() if reuse_mask is not None else None
        ctx_p = ctx.data_ptr() if ctx is not None else None
        if temb is not None:
            assert temb.is_contiguous() and temb.dtype == x.dtype
            _check(lib().pserve_block_forward_temb(self.plan._h, x.data_ptr(), ctx_p, temb.data_ptr(), self.block._h,
                                                   self._h, mask_p, y.data_ptr(), _stream()))
        else:
            _check(lib().pserve_block_forward(self.plan._h, x.data_ptr(), ctx_p, self.block._h, self._h, mask_p,
                                              y.data_ptr(), _stream()))
        return y

    def close(self):
        if self._h:
            lib().pserve_cache_free(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


DOWN2, UP2 = 1, 2


class Resample:
    """pserve_resample: stride-2 (DOWN2) or nearest-up (UP2) 3x3 convolution between two plans with the same patch grid."""

    def __init__(self, kind: int, w, b, dtype: int):
        assert w.is_contiguous() and b.is_contiguous() and w.dtype == _torch_dtype(dtype) and b.dtype == w.dtype
        self.kind, self.dtype, self.C_out, self.C_in = kind, dtype, int(w.shape[0]), int(w.shape[1])
        self._h = C.c_void_p()
        _check(lib().pserve_resample_create(kind, self.C_in, self.C_out, dtype, w.data_ptr(), b.data_ptr(), _stream(),
                                            C.byref(self._h)))
        self._ws = None

    def workspace_bytes(self, plan_in: "Plan") -> int:
        n = C.c_size_t()
        _check(lib().pserve_resample_workspace(self._h, plan_in._h, C.byref(n)))
        return int(n.value)

    def forward(self, plan_in: "Plan", plan_out: "Plan", x, y=None, workspace=None):
        import torch
        assert x.is_contiguous() and tuple(x.shape) == (plan_in.T, self.C_in) and x.dtype == _torch_dtype(self.dtype)
        if workspace is None:
            need = self.workspace_bytes(plan_in)
            if self._ws is None or self._ws.numel() < need:
                self._ws = torch.empty(need, dtype=torch.uint8, device=x.device)
            workspace = self._ws
        if y is None:
            y = torch.empty((plan_out.T, self.C_out), dtype=x.dtype, device=x.device)
        _check(lib().pserve_resample_forward(self._h, plan_in._h, plan_out._h, x.data_ptr(), workspace.data_ptr(),
                                             workspace.numel() * workspace.element_size(), y.data_ptr(), _stream()))
        return y

    def close(self):
        if self._h:
            lib().pserve_resample_free(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ---- host-side scheduler pieces (tasks are tuples (id, H, W, steps_left, arrival, ddl, standalone), times in ms)
def _tasks(ts):
    arr = (_Task * max(1, len(ts)))()
    for i, t in enumerate(ts):
        arr[i] = _Task(*t)
    return arr


def _model(w):
    m = _LatencyModel()
    for i in range(4):
        m.w[i] = float(w[i])
    return m


def latency_predict(w, batch, ph, pw) -> float:
    out = C.c_double()
    _check(lib().pserve_latency_predict(C.byref(_model(w)), _tasks(batch), len(batch), ph, pw, C.byref(out)))
    return out.value


def latency_fit(X, y):
    import numpy as np
    X = np.ascontiguousarray(X, dtype=np.float64)
    y = np.ascontiguousarray(y, dtype=np.float64)
    m = _LatencyModel()
    _check(lib().pserve_latency_fit(X.ctypes.data_as(C.POINTER(C.c_double)), y.ctypes.data_as(C.POINTER(C.c_double)),
                                    X.shape[0], C.byref(m)))
    return [m.w[i] for i in range(4)]


def slack(task, now, latency) -> float:
    out = C.c_double()
    _check(lib().pserve_slack(_tasks([task]), now, latency, C.byref(out)))
    return out.value


def schedule(wait, active, now, w, ph, pw, relaxed_slack):
    """pserve_schedule: returns (admitted, discarded), indices into `wait` in the order decided."""
    n = len(wait)
    adm, dis = (C.c_int32 * max(1, n))(), (C.c_int32 * max(1, n))()
    na, nd = C.c_int32(), C.c_int32()
    _check(lib().pserve_schedule(_tasks(wait), n, _tasks(active), len(active), now, C.byref(_model(w)), ph, pw,
                                 relaxed_slack, adm, C.byref(na), dis, C.byref(nd)))
    return list(adm[:na.value]), list(dis[:nd.value])

"""ctypes marshalling for include/calibatt.h."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG_DIR, "libcalibatt.so")
_lib = None


class CalibattError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


class _CStrides(C.Structure):
    _fields_ = [("b", C.c_int64), ("h", C.c_int64), ("n", C.c_int64)]


class _CFwdOptions(C.Structure):
    _fields_ = [("in_strides", C.POINTER(_CStrides)), ("out_strides", C.POINTER(_CStrides)),
                ("dtype", C.c_int32), ("lse", C.c_void_p), ("kernel", C.c_int32)]


KERNEL_AUTO, KERNEL_TWO_WORKGROUPS, KERNEL_INTERLEAVED = 0, 1, 2


class _CPattern(C.Structure):
    _fields_ = [
        ("H", C.c_int32), ("N", C.c_int32), ("block_q", C.c_int32), ("block_k", C.c_int32),
        ("nbq", C.c_int32), ("nbk", C.c_int32),
        ("n_work", C.c_int32), ("n_repeat", C.c_int32),
        ("order", C.c_int32), ("max_row", C.c_int32),
        ("nnz", C.c_int64),
        ("row_ptr", C.c_void_p), ("col_idx", C.c_void_p), ("repeat_src", C.c_void_p),
        ("work", C.c_void_p), ("fan_ptr", C.c_void_p), ("fan_dst", C.c_void_p),
        ("work_counter", C.c_void_p),
        ("n_groups", C.c_int32),
        ("group_ptr", C.c_int32 * 9),
        ("iv_ptr", C.c_void_p), ("iv", C.c_void_p),
        ("head_map", C.c_void_p),
    ]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libcalibatt.so (built by ``python -m paper_2603_05503_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2603_05503_amd.build` "
            "(there is no fallback path)"
        )
    # Device pointers and streams handed to the library come from torch, so both must sit on ONE HIP
    # runtime.  torch ships its own copy; loading torch first makes the dynamic linker resolve the
    # library's libamdhip64 dependency to that already loaded copy instead of a second runtime
    # (which would not see torch's device context).
    import torch  # noqa: F401

    lib = C.CDLL(_LIB_PATH)
    i32p, u8p, i64p = C.POINTER(C.c_int32), C.POINTER(C.c_uint8), C.POINTER(C.c_int64)
    lib.calibatt_pattern_sizes.restype = C.c_int
    lib.calibatt_pattern_sizes.argtypes = [u8p, i32p, C.c_int, C.c_int, C.c_int, C.c_int, i64p, i32p, i32p]
    lib.calibatt_compile_pattern.restype = C.c_int
    lib.calibatt_compile_pattern.argtypes = [
        u8p, i32p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
        i32p, i32p, C.c_int64, i32p, i32p, i32p, i32p, C.POINTER(_CPattern),
    ]
    lib.calibatt_sparse_attn_fwd.restype = C.c_int
    lib.calibatt_sparse_attn_fwd.argtypes = [
        C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
        C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
        C.POINTER(_CPattern), C.c_float, C.c_void_p,
    ]
    lib.calibatt_anchor_map.restype = C.c_int
    lib.calibatt_anchor_map.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, i32p, i32p, i32p, i32p]
    lib.calibatt_anchor_attn_fwd.restype = C.c_int
    lib.calibatt_anchor_attn_fwd.argtypes = [
        C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
        C.c_int, C.c_int, C.c_int, C.c_int,
        C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
        C.c_float, C.c_void_p,
    ]
    lib.calibatt_block_energy.restype = C.c_int
    lib.calibatt_block_energy.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int,
                                          C.c_int, C.c_int, C.c_float, C.c_void_p]
    lib.calibatt_select_blocks.restype = C.c_int
    lib.calibatt_select_blocks.argtypes = [C.POINTER(C.c_float), C.c_int64, C.c_int, C.c_double, u8p]
    lib.calibatt_vote_masks.restype = C.c_int
    lib.calibatt_vote_masks.argtypes = [u8p, C.c_int, C.c_int64, C.c_double, u8p]
    u16p = C.POINTER(C.c_uint16)
    lib.calibatt_vote_accumulate.restype = C.c_int
    lib.calibatt_vote_accumulate.argtypes = [u8p, C.c_int64, u16p]
    lib.calibatt_vote_finish.restype = C.c_int
    lib.calibatt_vote_finish.argtypes = [u16p, C.c_int, C.c_int64, C.c_double, u8p]
    lib.calibatt_epsilon_schedule.restype = C.c_double
    lib.calibatt_epsilon_schedule.argtypes = [C.c_int, C.c_int, C.c_double, C.c_double, C.c_double]
    lib.calibatt_schedule_base_level.restype = C.c_double
    lib.calibatt_schedule_base_level.argtypes = [C.c_int]
    u32p = C.POINTER(C.c_uint32)
    lib.calibatt_encode_intervals.restype = C.c_int
    lib.calibatt_encode_intervals.argtypes = [i32p, i32p, C.c_int64, i32p, u32p, C.c_int64, i64p]
    lib.calibatt_merge_intervals.restype = C.c_int
    lib.calibatt_merge_intervals.argtypes = [u8p, C.c_int64, C.c_int, C.c_double, u8p, i32p]
    lib.calibatt_share_timesteps.restype = C.c_int
    lib.calibatt_share_timesteps.argtypes = [u8p, C.c_int, C.c_int64, C.c_double, i32p, u8p, i32p]
    lib.calibatt_sparse_attn_fwd_strided.restype = C.c_int
    lib.calibatt_sparse_attn_fwd_strided.argtypes = [
        C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
        C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
        C.POINTER(_CPattern), C.c_float, C.POINTER(_CStrides), C.POINTER(_CStrides), C.c_void_p,
    ]
    lib.calibatt_schedule_constants.restype = C.c_int
    lib.calibatt_schedule_constants.argtypes = [C.c_int, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double),
                                                C.POINTER(C.c_double)]
    lib.calibatt_flag_heads.restype = C.c_int
    lib.calibatt_flag_heads.argtypes = [C.POINTER(C.c_float), C.c_int, C.c_int, C.c_double, C.POINTER(C.c_uint8),
                                        C.POINTER(C.c_double)]
    lib.calibatt_anchor_partner.restype = C.c_int
    lib.calibatt_anchor_partner.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, i32p]
    lib.calibatt_spatial_similarity.restype = C.c_int
    lib.calibatt_spatial_similarity.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int,
                                                C.c_void_p, C.c_int, C.c_int, C.c_float, C.c_void_p, C.c_void_p,
                                                C.c_void_p]
    lib.calibatt_spatial_similarity_static.restype = C.c_int
    lib.calibatt_spatial_similarity_static.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int,
                                                       C.c_void_p, C.c_int, C.c_int, C.c_float, C.c_void_p, C.c_void_p]
    lib.calibatt_sparse_attn_fwd_ex.restype = C.c_int
    lib.calibatt_sparse_attn_fwd_ex.argtypes = [
        C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
        C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
        C.POINTER(_CPattern), C.c_float, C.POINTER(_CFwdOptions), C.c_void_p,
    ]
    lib.calibatt_anchor_attn_fwd_strided.restype = C.c_int
    lib.calibatt_anchor_attn_fwd_strided.argtypes = lib.calibatt_anchor_attn_fwd.argtypes[:-1] + [
        C.POINTER(_CStrides), C.POINTER(_CStrides), C.c_void_p]
    lib.calibatt_anchor_attn_fwd_split.restype = C.c_int
    lib.calibatt_anchor_attn_fwd_split.argtypes = lib.calibatt_anchor_attn_fwd_strided.argtypes[:-1] + [
        C.c_void_p, C.c_int64, C.c_void_p]
    lib.calibatt_anchor_split_plan.restype = C.c_int
    lib.calibatt_anchor_split_plan.argtypes = [C.c_int] * 5 + [C.POINTER(C.c_int32), C.POINTER(C.c_int64)]
    lib.calibatt_block_energy_workspace_bytes.restype = C.c_int
    lib.calibatt_block_energy_workspace_bytes.argtypes = [C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int64)]
    lib.calibatt_block_energy_onepass.restype = C.c_int
    lib.calibatt_block_energy_onepass.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p] + [C.c_int] * 6 + [
        C.c_float, C.c_void_p, C.c_int64, C.c_void_p]
    lib.calibatt_select_blocks_device.restype = C.c_int
    lib.calibatt_select_blocks_device.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_double, C.c_void_p, C.c_void_p]
    lib.calibatt_vote_accumulate_device.restype = C.c_int
    lib.calibatt_vote_accumulate_device.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
    lib.calibatt_strerror.restype = C.c_char_p
    lib.calibatt_strerror.argtypes = [C.c_int]
    lib.calibatt_version.restype = C.c_int
    lib.calibatt_version.argtypes = []
    _lib = lib
    return lib


def strerror(status: int) -> str:
    return load_library().calibatt_strerror(int(status)).decode()


def version() -> int:
    return int(load_library().calibatt_version())


def _as_mask(mask, H, nbq, nbk):
    m = np.ascontiguousarray(mask, dtype=np.uint8)
    if m.size != H * nbq * nbk:
        raise ValueError(f"mask has {m.size} entries, expected {H}x{nbq}x{nbk}")
    return m


def _as_repeat(repeat, H, nbq):
    if repeat is None:
        return None
    r = np.ascontiguousarray(repeat, dtype=np.int32)
    if r.size != H * nbq:
        raise ValueError(f"repeat has {r.size} entries, expected {H}x{nbq}")
    return r


def _ptr(a, ctype):
    return None if a is None else a.ctypes.data_as(C.POINTER(ctype))


def pattern_sizes(mask, repeat, H, N, block_q, block_k):
    """(nnz, n_work, n_repeat) via calibatt_pattern_sizes."""
    lib = load_library()
    nbq, nbk = -(-N // block_q), -(-N // block_k)
    m, r = _as_mask(mask, H, nbq, nbk), _as_repeat(repeat, H, nbq)
    nnz, nw, nr = C.c_int64(0), C.c_int32(0), C.c_int32(0)
    st = lib.calibatt_pattern_sizes(_ptr(m, C.c_uint8), _ptr(r, C.c_int32), H, N, block_q, block_k,
                                    C.byref(nnz), C.byref(nw), C.byref(nr))
    if st != 0:
        raise CalibattError(st, "calibatt_pattern_sizes")
    return int(nnz.value), int(nw.value), int(nr.value)


@dataclass
class HostPattern:
    """Output of calibatt_compile_pattern in host (NumPy) buffers."""
    H: int
    N: int
    block_q: int
    block_k: int
    nbq: int
    nbk: int
    n_work: int
    n_repeat: int
    order: int
    max_row: int
    nnz: int
    row_ptr: np.ndarray
    col_idx: np.ndarray
    repeat_src: np.ndarray
    work: np.ndarray
    fan_ptr: np.ndarray
    fan_dst: np.ndarray
    n_groups: int = 1
    group_ptr: Optional[np.ndarray] = None

    def to_device(self, device="cuda", persistent=True, intervals=False, head_map=None) -> "DevicePattern":
        """``intervals=True`` uploads the interval form of the kept-block lists instead of col_idx;
        ``head_map`` (one tensor head per pattern head) makes the pattern act on a subset of heads."""
        return DevicePattern(self, device, persistent, intervals, head_map)

    def encode_intervals(self):
        """(iv_ptr int32 [rows + 1], iv uint32 words) via calibatt_encode_intervals."""
        return encode_intervals(self.row_ptr, self.col_idx)


def compile_pattern(mask, repeat, H, N, block_q, block_k, order=4) -> HostPattern:
    lib = load_library()
    if min(H, N, block_q, block_k) <= 0:
        raise CalibattError(-2, "calibatt_compile_pattern")
    nbq, nbk = -(-N // block_q), -(-N // block_k)
    m, r = _as_mask(mask, H, nbq, nbk), _as_repeat(repeat, H, nbq)
    nnz, _, _ = pattern_sizes(m, r, H, N, block_q, block_k)
    rows = H * nbq
    row_ptr = np.empty(rows + 1, np.int32)
    col_idx = np.empty(max(nnz, 1), np.int32)
    repeat_src = np.empty(rows, np.int32)
    work = np.empty(rows, np.int32)
    fan_ptr = np.empty(rows + 1, np.int32)
    fan_dst = np.empty(rows, np.int32)
    cp = _CPattern()
    st = lib.calibatt_compile_pattern(
        _ptr(m, C.c_uint8), _ptr(r, C.c_int32), H, N, block_q, block_k, order,
        _ptr(row_ptr, C.c_int32), _ptr(col_idx, C.c_int32), nnz, _ptr(repeat_src, C.c_int32),
        _ptr(work, C.c_int32), _ptr(fan_ptr, C.c_int32), _ptr(fan_dst, C.c_int32), C.byref(cp))
    if st != 0:
        raise CalibattError(st, "calibatt_compile_pattern")
    return HostPattern(
        H=cp.H, N=cp.N, block_q=cp.block_q, block_k=cp.block_k, nbq=cp.nbq, nbk=cp.nbk,
        n_work=cp.n_work, n_repeat=cp.n_repeat, order=cp.order, max_row=cp.max_row, nnz=cp.nnz,
        row_ptr=row_ptr, col_idx=col_idx[:nnz], repeat_src=repeat_src,
        work=work[: cp.n_work], fan_ptr=fan_ptr[: cp.n_work + 1], fan_dst=fan_dst[: cp.n_repeat],
        n_groups=cp.n_groups, group_ptr=np.array(list(cp.group_ptr), dtype=np.int32),
    )


class DevicePattern:
    """The six index arrays as int32 torch tensors on the GPU plus the C struct
    that points at them."""

    _NAMES = ("row_ptr", "col_idx", "repeat_src", "work", "fan_ptr", "fan_dst")

    def __init__(self, hp: HostPattern, device="cuda", persistent=True, intervals=False, head_map=None):
        import torch

        self.host = hp
        self.tensors = {}
        self.intervals = bool(intervals)
        for name in self._NAMES:
            if intervals and name == "col_idx":
                continue
            a = getattr(hp, name)
            t = torch.from_numpy(np.ascontiguousarray(a if a.size else np.zeros(1, np.int32)))
            self.tensors[name] = t.to(device)
        c = _CPattern()
        for f in ("H", "N", "block_q", "block_k", "nbq", "nbk", "n_work", "n_repeat", "order", "max_row", "nnz"):
            setattr(c, f, getattr(hp, f))
        for name in self._NAMES:
            setattr(c, name, self.tensors[name].data_ptr() if name in self.tensors else None)
        if intervals:
            iv_ptr, iv = hp.encode_intervals()
            self.tensors["iv_ptr"] = torch.from_numpy(iv_ptr).to(device)
            self.tensors["iv"] = torch.from_numpy(iv.view(np.int32)).to(device)
            c.iv_ptr = self.tensors["iv_ptr"].data_ptr()
            c.iv = self.tensors["iv"].data_ptr()
        else:
            c.iv_ptr = None
            c.iv = None
        if head_map is not None:
            hm = np.ascontiguousarray(head_map, dtype=np.int32).reshape(-1)
            if hm.size != hp.H:
                raise ValueError(f"head_map has {hm.size} entries, the pattern has {hp.H} heads")
            self.tensors["head_map"] = torch.from_numpy(hm).to(device)
            c.head_map = self.tensors["head_map"].data_ptr()
        else:
            c.head_map = None
        # int32[16] workspace of the persistent-workgroup scheduler (kept zero between calls)
        self.counter = torch.zeros(16, dtype=torch.int32, device=device) if persistent else None
        c.work_counter = self.counter.data_ptr() if persistent else None
        c.n_groups = hp.n_groups
        gp = hp.group_ptr if hp.group_ptr is not None else np.array([0] + [hp.n_work] * 8, np.int32)
        for i in range(9):
            c.group_ptr[i] = int(gp[i])
        self.c = c
        self._stream_of_c = None   # stream handle that uses self.c
        self._per_stream = {}      # other streams: (clone of the struct, its own counters)

    def c_for(self, stream_handle: int):
        """The C struct to pass for a call on ``stream_handle``.  Calls on different streams may overlap on
        the GPU, and overlapping calls must not share the scheduler's work counters: every stream after the
        first gets a clone of the struct that points at counters of its own (the index arrays are shared)."""
        if self.counter is None or self._stream_of_c is None or self._stream_of_c == stream_handle:
            self._stream_of_c = stream_handle
            return self.c
        if stream_handle not in self._per_stream:
            import torch

            clone = _CPattern()
            C.memmove(C.byref(clone), C.byref(self.c), C.sizeof(_CPattern))
            counter = torch.zeros(16, dtype=torch.int32, device=self.counter.device)
            clone.work_counter = counter.data_ptr()
            self._per_stream[stream_handle] = (clone, counter)
        return self._per_stream[stream_handle][0]

    @property
    def nnz(self) -> int:
        return self.host.nnz

    @property
    def index_bytes(self) -> int:
        """Bytes of the kept-block lists on the GPU (col_idx, or iv_ptr + iv in the interval form)."""
        names = ("iv_ptr", "iv") if self.intervals else ("col_idx",)
        return sum(self.tensors[n].numel() * 4 for n in names)


def sparse_attn_fwd(q, k, v, out, pattern: DevicePattern, scale: float,
                    block_q: Optional[int] = None, block_k: Optional[int] = None, stream=None, lse=None,
                    kernel: int = KERNEL_AUTO):
    """The sparse forward on torch CUDA tensors of logical shape [B, H, N, D], bf16 or fp16 (all four
    alike).  The tensors may be strided views (e.g. ``x.transpose(1, 2)`` of a [B, N, H, D] tensor, or
    slices of a fused [B, N, 3, H, D] projection) as long as D is contiguous and q, k, v share their
    strides.  ``lse``: optional contiguous fp32 CUDA tensor [B, H, N] that receives the log-sum-exp of
    every query's kept logits.  ``kernel``: KERNEL_AUTO, KERNEL_TWO_WORKGROUPS or KERNEL_INTERLEAVED (the
    ``kernel`` field of calibatt_fwd_options).  Packed bf16 calls without ``lse`` and with the automatic
    kernel choice go through calibatt_sparse_attn_fwd, everything else through calibatt_sparse_attn_fwd_ex."""
    import torch

    lib = load_library()
    for t in (q, k, v, out):
        if not (t.is_cuda and t.dtype in (torch.bfloat16, torch.float16) and t.dim() == 4 and t.stride(3) == 1):
            raise ValueError("q, k, v, out must be bf16 or fp16 CUDA tensors [B, H, N, D] with contiguous D")
        if t.shape != q.shape or t.dtype != q.dtype:
            raise ValueError("q, k, v, out must have the same shape and element type")
    if not (q.stride() == k.stride() == v.stride()):
        raise ValueError("q, k, v must share their strides")
    B, H, N, D = q.shape
    if lse is not None and not (lse.is_cuda and lse.dtype == torch.float32 and lse.is_contiguous()
                                and tuple(lse.shape) == (B, H, N)):
        raise ValueError("lse must be a contiguous fp32 CUDA tensor [B, H, N]")
    bq = pattern.host.block_q if block_q is None else block_q
    bk = pattern.host.block_k if block_k is None else block_k
    if stream is None:
        stream = torch.cuda.current_stream(q.device).cuda_stream
    packed = all(t.is_contiguous() for t in (q, k, v, out))
    if packed and lse is None and q.dtype == torch.bfloat16 and kernel == KERNEL_AUTO:
        st = lib.calibatt_sparse_attn_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(),
                                          B, H, N, D, bq, bk, C.byref(pattern.c_for(int(stream))), float(scale), C.c_void_p(stream))
    else:
        si = _CStrides(q.stride(0), q.stride(1), q.stride(2))
        so = _CStrides(out.stride(0), out.stride(1), out.stride(2))
        opt = _CFwdOptions(None if packed else C.pointer(si), None if packed else C.pointer(so),
                           0 if q.dtype == torch.bfloat16 else 1, None if lse is None else lse.data_ptr(), int(kernel))
        st = lib.calibatt_sparse_attn_fwd_ex(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(),
                                             B, H, N, D, bq, bk, C.byref(pattern.c_for(int(stream))), float(scale),
                                             C.byref(opt), C.c_void_p(stream))
    if st != 0:
        raise CalibattError(st, "calibatt_sparse_attn_fwd")
    return out


@dataclass
class HostAnchorMap:
    """Output of calibatt_anchor_map in host (NumPy) buffers."""
    N: int
    n_q: int
    q_index: np.ndarray
    dst_ptr: np.ndarray
    dst_idx: np.ndarray

    def to_device(self, device="cuda") -> "DeviceAnchorMap":
        return DeviceAnchorMap(self, device)


def anchor_map(N, F, Hs, Ws, k) -> HostAnchorMap:
    lib = load_library()
    n_q = C.c_int32(0)
    st = lib.calibatt_anchor_map(N, F, Hs, Ws, k, None, None, None, C.byref(n_q))
    if st != 0:
        raise CalibattError(st, "calibatt_anchor_map")
    q_index = np.empty(n_q.value, np.int32)
    dst_ptr = np.empty(n_q.value + 1, np.int32)
    dst_idx = np.empty(N, np.int32)
    st = lib.calibatt_anchor_map(N, F, Hs, Ws, k, _ptr(q_index, C.c_int32), _ptr(dst_ptr, C.c_int32),
                                 _ptr(dst_idx, C.c_int32), C.byref(n_q))
    if st != 0:
        raise CalibattError(st, "calibatt_anchor_map")
    return HostAnchorMap(N=N, n_q=int(n_q.value), q_index=q_index, dst_ptr=dst_ptr, dst_idx=dst_idx)


class DeviceAnchorMap:
    """The three lists of an anchor map as int32 torch tensors on the GPU."""

    def __init__(self, hm: HostAnchorMap, device="cuda"):
        import torch

        self.host = hm
        self.n_q = hm.n_q
        self.q_index = torch.from_numpy(np.ascontiguousarray(hm.q_index, dtype=np.int32)).to(device)
        self.dst_ptr = torch.from_numpy(np.ascontiguousarray(hm.dst_ptr, dtype=np.int32)).to(device)
        self.dst_idx = torch.from_numpy(np.ascontiguousarray(hm.dst_idx, dtype=np.int32)).to(device)


def anchor_split_plan(B: int, N: int, D: int, n_heads: int, n_q: int):
    """calibatt_anchor_split_plan on the current device: (n_split, workspace_bytes)."""
    lib = load_library()
    n_split, nbytes = C.c_int32(0), C.c_int64(0)
    st = lib.calibatt_anchor_split_plan(B, N, D, n_heads, n_q, C.byref(n_split), C.byref(nbytes))
    if st != 0:
        raise CalibattError(st, "calibatt_anchor_split_plan")
    return n_split.value, nbytes.value


def anchor_attn_fwd(q, k, v, out, head_ids, amap: DeviceAnchorMap, scale: float, stream=None, workspace=None):
    """calibatt_anchor_attn_fwd on torch bf16 CUDA tensors of logical shape [B, H, N, D] (strided views
    with contiguous D allowed, q, k, v sharing their strides); ``head_ids`` is an int32 CUDA tensor of
    the heads to process.  ``workspace``: a contiguous CUDA tensor of at least the bytes
    ``anchor_split_plan`` names for the shape selects calibatt_anchor_attn_fwd_split."""
    import torch

    lib = load_library()
    for t in (q, k, v, out):
        if not (t.is_cuda and t.dtype == torch.bfloat16 and t.dim() == 4 and t.stride(3) == 1):
            raise ValueError("q, k, v, out must be bf16 CUDA tensors [B, H, N, D] with contiguous D")
        if t.shape != q.shape:
            raise ValueError("q, k, v, out must have the same shape")
    if not (q.stride() == k.stride() == v.stride()):
        raise ValueError("q, k, v must share their strides")
    if not (head_ids.is_cuda and head_ids.dtype == torch.int32 and head_ids.is_contiguous() and head_ids.dim() == 1):
        raise ValueError("head_ids must be a contiguous 1-d int32 CUDA tensor")
    B, H, N, D = q.shape
    if stream is None:
        stream = torch.cuda.current_stream(q.device).cuda_stream
    args = (q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), B, H, N, D,
            head_ids.data_ptr(), head_ids.numel(), amap.q_index.data_ptr(),
            amap.dst_ptr.data_ptr(), amap.dst_idx.data_ptr(), amap.n_q, float(scale))
    if workspace is not None:
        if not (workspace.is_cuda and workspace.is_contiguous() and workspace.device == q.device):
            raise ValueError("workspace must be a contiguous CUDA tensor on the tensors' device")
        si = _CStrides(q.stride(0), q.stride(1), q.stride(2))
        so = _CStrides(out.stride(0), out.stride(1), out.stride(2))
        st = lib.calibatt_anchor_attn_fwd_split(*args, C.byref(si), C.byref(so), C.c_void_p(workspace.data_ptr()),
                                                workspace.numel() * workspace.element_size(), C.c_void_p(stream))
    elif all(t.is_contiguous() for t in (q, k, v, out)):
        st = lib.calibatt_anchor_attn_fwd(*args, C.c_void_p(stream))
    else:
        si = _CStrides(q.stride(0), q.stride(1), q.stride(2))
        so = _CStrides(out.stride(0), out.stride(1), out.stride(2))
        st = lib.calibatt_anchor_attn_fwd_strided(*args, C.byref(si), C.byref(so), C.c_void_p(stream))
    if st != 0:
        raise CalibattError(st, "calibatt_anchor_attn_fwd")
    return out


def block_energy_workspace_bytes(N: int, block_q: int, block_k: int) -> int:
    lib = load_library()
    n = C.c_int64(0)
    st = lib.calibatt_block_energy_workspace_bytes(N, block_q, block_k, C.byref(n))
    if st != 0:
        raise CalibattError(st, "calibatt_block_energy_workspace_bytes")
    return n.value


def block_energy(q, k, block_q: int, block_k: int, scale: float, out=None, stream=None, workspace=None):
    """calibatt_block_energy on torch bf16 CUDA tensors [B, H, N, D]; returns the fp32 CUDA tensor
    [B, H, ceil(N/block_q), ceil(N/block_k)] (``out`` if given).  ``workspace`` (a contiguous CUDA
    tensor, see ``block_energy_workspace_bytes``) selects calibatt_block_energy_onepass."""
    import torch

    lib = load_library()
    for t in (q, k):
        if not (t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous() and t.dim() == 4):
            raise ValueError("q, k must be contiguous bf16 CUDA tensors [B, H, N, D]")
    if q.shape != k.shape:
        raise ValueError("q and k must have the same shape")
    B, H, N, D = q.shape
    shape = (B, H, -(-N // block_q), -(-N // block_k))
    if out is None:
        out = torch.empty(shape, dtype=torch.float32, device=q.device)
    elif not (out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and tuple(out.shape) == shape):
        raise ValueError(f"out must be a contiguous fp32 CUDA tensor of shape {shape}")
    if stream is None:
        stream = torch.cuda.current_stream(q.device).cuda_stream
    if workspace is not None:
        if not (workspace.is_cuda and workspace.is_contiguous() and workspace.device == q.device):
            raise ValueError("workspace must be a contiguous CUDA tensor on the tensors' device")
        st = lib.calibatt_block_energy_onepass(q.data_ptr(), k.data_ptr(), out.data_ptr(), B, H, N, D, block_q, block_k,
                                               float(scale), workspace.data_ptr(),
                                               workspace.numel() * workspace.element_size(), C.c_void_p(stream))
    else:
        st = lib.calibatt_block_energy(q.data_ptr(), k.data_ptr(), out.data_ptr(), B, H, N, D, block_q, block_k,
                                       float(scale), C.c_void_p(stream))
    if st != 0:
        raise CalibattError(st, "calibatt_block_energy")
    return out


def select_blocks_device(energy, eps: float, out=None, stream=None):
    """calibatt_select_blocks_device on a contiguous fp32 CUDA tensor [..., nbk]: uint8 CUDA mask of the
    same shape (``out`` if given)."""
    import torch

    lib = load_library()
    if not (energy.is_cuda and energy.dtype == torch.float32 and energy.is_contiguous() and energy.dim() >= 1):
        raise ValueError("energy must be a contiguous fp32 CUDA tensor [..., nbk]")
    if out is None:
        out = torch.empty(energy.shape, dtype=torch.uint8, device=energy.device)
    elif not (out.is_cuda and out.dtype == torch.uint8 and out.is_contiguous() and out.shape == energy.shape):
        raise ValueError("out must be a contiguous uint8 CUDA tensor of the energies' shape")
    nbk = energy.shape[-1]
    if stream is None:
        stream = torch.cuda.current_stream(energy.device).cuda_stream
    st = lib.calibatt_select_blocks_device(energy.data_ptr(), energy.numel() // max(nbk, 1), nbk, float(eps),
                                           out.data_ptr(), C.c_void_p(stream))
    if st != 0:
        raise CalibattError(st, "calibatt_select_blocks_device")
    return out


def vote_accumulate_device(mask, counts, stream=None):
    """calibatt_vote_accumulate_device: ``mask`` uint8 CUDA tensor of n entries, ``counts`` int16 CUDA
    tensor of n entries holding uint16 counters (torch has no arithmetic on uint16; read them back with
    ``counts.cpu().numpy().view(numpy.uint16)``)."""
    import torch

    lib = load_library()
    if not (mask.is_cuda and mask.dtype == torch.uint8 and mask.is_contiguous()):
        raise ValueError("mask must be a contiguous uint8 CUDA tensor")
    if not (counts.is_cuda and counts.dtype == torch.int16 and counts.is_contiguous() and counts.numel() == mask.numel()):
        raise ValueError("counts must be a contiguous int16 CUDA tensor with one entry per mask entry")
    if stream is None:
        stream = torch.cuda.current_stream(mask.device).cuda_stream
    st = lib.calibatt_vote_accumulate_device(mask.data_ptr(), mask.numel(), counts.data_ptr(), C.c_void_p(stream))
    if st != 0:
        raise CalibattError(st, "calibatt_vote_accumulate_device")
    return counts


def select_blocks(energy, eps: float) -> np.ndarray:
    """calibatt_select_blocks on a host array [..., nbk] (converted to fp32): uint8 mask of the same shape."""
    lib = load_library()
    e = np.ascontiguousarray(energy, dtype=np.float32)
    if e.ndim < 1 or e.shape[-1] == 0:
        raise CalibattError(-2, "calibatt_select_blocks")
    mask = np.empty(e.shape, np.uint8)
    st = lib.calibatt_select_blocks(_ptr(e, C.c_float), e.size // e.shape[-1], e.shape[-1], float(eps),
                                    _ptr(mask, C.c_uint8))
    if st != 0:
        raise CalibattError(st, "calibatt_select_blocks")
    return mask


def vote_masks(masks, rho: float) -> np.ndarray:
    """calibatt_vote_masks on a host array [n_prompts, ...]: uint8 mask of the trailing shape."""
    lib = load_library()
    m = np.ascontiguousarray(masks, dtype=np.uint8)
    if m.ndim < 1 or m.shape[0] == 0:
        raise CalibattError(-2, "calibatt_vote_masks")
    out = np.empty(m.shape[1:], np.uint8)
    st = lib.calibatt_vote_masks(_ptr(m, C.c_uint8), m.shape[0], out.size, float(rho), _ptr(out, C.c_uint8))
    if st != 0:
        raise CalibattError(st, "calibatt_vote_masks")
    return out


def vote_accumulate(mask, counts: np.ndarray) -> None:
    """calibatt_vote_accumulate: adds one prompt's mask to the uint16 counters (same shape), in place."""
    lib = load_library()
    m = np.ascontiguousarray(mask, dtype=np.uint8)
    if not (counts.dtype == np.uint16 and counts.flags.c_contiguous and counts.shape == m.shape):
        raise ValueError("counts must be a C-contiguous uint16 array of the mask's shape")
    st = lib.calibatt_vote_accumulate(_ptr(m, C.c_uint8), m.size, _ptr(counts, C.c_uint16))
    if st != 0:
        raise CalibattError(st, "calibatt_vote_accumulate")


def vote_finish(counts: np.ndarray, n_prompts: int, rho: float) -> np.ndarray:
    """calibatt_vote_finish: uint8 mask of the counters' shape."""
    lib = load_library()
    c = np.ascontiguousarray(counts, dtype=np.uint16)
    out = np.empty(c.shape, np.uint8)
    st = lib.calibatt_vote_finish(_ptr(c, C.c_uint16), int(n_prompts), c.size, float(rho), _ptr(out, C.c_uint8))
    if st != 0:
        raise CalibattError(st, "calibatt_vote_finish")
    return out


def epsilon_schedule(t: int, T: int, A: float, Cc: float, k: float) -> float:
    return float(load_library().calibatt_epsilon_schedule(int(t), int(T), float(A), float(Cc), float(k)))


def schedule_base_level(N: int) -> float:
    return float(load_library().calibatt_schedule_base_level(int(N)))


REGIME_MANY_STEP, REGIME_DISTILLED = 0, 1


def schedule_constants(regime: int, N: int):
    """calibatt_schedule_constants: (A, C, k) of Eq. 7 for the many-step (0) or distilled (1) regime."""
    lib = load_library()
    A, Cc, k = C.c_double(), C.c_double(), C.c_double()
    st = lib.calibatt_schedule_constants(int(regime), int(N), C.byref(A), C.byref(Cc), C.byref(k))
    if st != 0:
        raise CalibattError(st, "calibatt_schedule_constants")
    return A.value, Cc.value, k.value


def flag_heads(scores, gamma: float):
    """calibatt_flag_heads: scores [n_prompts, H] -> (flags uint8 [H], mean float64 [H])."""
    lib = load_library()
    s = np.ascontiguousarray(scores, dtype=np.float32)
    if s.ndim != 2:
        raise ValueError("scores must be [n_prompts, H]")
    flags = np.zeros(s.shape[1], dtype=np.uint8)
    mean = np.zeros(s.shape[1], dtype=np.float64)
    st = lib.calibatt_flag_heads(s.ctypes.data_as(C.POINTER(C.c_float)), int(s.shape[0]), int(s.shape[1]), float(gamma),
                                 flags.ctypes.data_as(C.POINTER(C.c_uint8)), mean.ctypes.data_as(C.POINTER(C.c_double)))
    if st != 0:
        raise CalibattError(st, "calibatt_flag_heads")
    return flags, mean


def encode_intervals(row_ptr, col_idx):
    """calibatt_encode_intervals: (iv_ptr int32 [rows + 1], iv uint32 words)."""
    lib = load_library()
    rp = np.ascontiguousarray(row_ptr, dtype=np.int32)
    ci = np.ascontiguousarray(col_idx, dtype=np.int32)
    if ci.size == 0:
        ci = np.zeros(1, np.int32)
    n_rows = rp.size - 1
    n_words = C.c_int64(0)
    st = lib.calibatt_encode_intervals(_ptr(rp, C.c_int32), _ptr(ci, C.c_int32), n_rows, None, None, 0, C.byref(n_words))
    if st != 0:
        raise CalibattError(st, "calibatt_encode_intervals")
    iv_ptr = np.empty(n_rows + 1, np.int32)
    iv = np.empty(max(n_words.value, 1), np.uint32)
    st = lib.calibatt_encode_intervals(_ptr(rp, C.c_int32), _ptr(ci, C.c_int32), n_rows, _ptr(iv_ptr, C.c_int32),
                                       _ptr(iv, C.c_uint32), iv.size, C.byref(n_words))
    if st != 0:
        raise CalibattError(st, "calibatt_encode_intervals")
    return iv_ptr, iv[: n_words.value]


def merge_intervals(mask, pct: float):
    """calibatt_merge_intervals over all rows of ``mask[..., nbk]``: (merged uint8 mask, width)."""
    lib = load_library()
    m = np.ascontiguousarray(mask, dtype=np.uint8)
    if m.ndim < 1 or m.shape[-1] == 0:
        raise CalibattError(-2, "calibatt_merge_intervals")
    out = np.empty_like(m)
    width = C.c_int32(0)
    st = lib.calibatt_merge_intervals(_ptr(m, C.c_uint8), m.size // m.shape[-1], m.shape[-1], float(pct),
                                      _ptr(out, C.c_uint8), C.byref(width))
    if st != 0:
        raise CalibattError(st, "calibatt_merge_intervals")
    return out, int(width.value)


def share_timesteps(masks, tau: float):
    """calibatt_share_timesteps on ``masks[T, ...]`` of one (layer, head): (cluster ids int32 [T],
    shared masks uint8 [n_clusters, ...])."""
    lib = load_library()
    m = np.ascontiguousarray(masks, dtype=np.uint8)
    if m.ndim < 1 or m.shape[0] == 0:
        raise CalibattError(-2, "calibatt_share_timesteps")
    T = m.shape[0]
    n = m.size // T
    cluster = np.empty(T, np.int32)
    shared = np.empty_like(m)
    n_clusters = C.c_int32(0)
    st = lib.calibatt_share_timesteps(_ptr(m, C.c_uint8), T, n, float(tau), _ptr(cluster, C.c_int32),
                                      _ptr(shared, C.c_uint8), C.byref(n_clusters))
    if st != 0:
        raise CalibattError(st, "calibatt_share_timesteps")
    return cluster, shared[: n_clusters.value].copy()


def anchor_partner(F, Hs, Ws, k) -> np.ndarray:
    """calibatt_anchor_partner: int32 [F*Hs*Ws], the token each video token is compared with."""
    lib = load_library()
    if min(F, Hs, Ws) <= 0:
        raise CalibattError(-2, "calibatt_anchor_partner")
    partner = np.empty(F * Hs * Ws, np.int32)
    st = lib.calibatt_anchor_partner(F, Hs, Ws, k, _ptr(partner, C.c_int32))
    if st != 0:
        raise CalibattError(st, "calibatt_anchor_partner")
    return partner


def spatial_similarity(q, k, partner, row_len: int, scale: float, workspace=None, stream=None):
    """calibatt_spatial_similarity on torch bf16 CUDA tensors [B, H, N, D]; ``partner`` is an int32
    CUDA tensor [n_tok].  Returns the fp32 CUDA tensor [B, H] of scores."""
    import torch

    lib = load_library()
    for t in (q, k):
        if not (t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous() and t.dim() == 4):
            raise ValueError("q, k must be contiguous bf16 CUDA tensors [B, H, N, D]")
    if q.shape != k.shape:
        raise ValueError("q and k must have the same shape")
    if not (partner.is_cuda and partner.dtype == torch.int32 and partner.is_contiguous() and partner.dim() == 1):
        raise ValueError("partner must be a contiguous 1-d int32 CUDA tensor")
    B, H, N, D = q.shape
    n_tok = partner.numel()
    if workspace is None:
        workspace = torch.empty((B, H, max(n_tok, 1), 3), dtype=torch.float32, device=q.device)
    score = torch.empty((B, H), dtype=torch.float32, device=q.device)
    if stream is None:
        stream = torch.cuda.current_stream(q.device).cuda_stream
    st = lib.calibatt_spatial_similarity(q.data_ptr(), k.data_ptr(), B, H, N, D, partner.data_ptr(), n_tok,
                                         int(row_len), float(scale), workspace.data_ptr(), score.data_ptr(),
                                         C.c_void_p(stream))
    if st != 0:
        raise CalibattError(st, "calibatt_spatial_similarity")
    return score


SIMILARITY_STATIC_MAX_BYTES = 16 * 1024 * 1024


def spatial_similarity_static(q, k, partner, row_len: int, scale: float, score, stream=None):
    """calibatt_spatial_similarity_static: the call that allocates nothing.  ``score`` is the caller's
    fp32 CUDA tensor [B, H]; the per-token sums live in the library's own buffer (one per GPU, shared by
    all calls on it)."""
    import torch

    lib = load_library()
    for t in (q, k):
        if not (t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous() and t.dim() == 4):
            raise ValueError("q, k must be contiguous bf16 CUDA tensors [B, H, N, D]")
    if q.shape != k.shape:
        raise ValueError("q and k must have the same shape")
    if not (partner.is_cuda and partner.dtype == torch.int32 and partner.is_contiguous() and partner.dim() == 1):
        raise ValueError("partner must be a contiguous 1-d int32 CUDA tensor")
    B, H, N, D = q.shape
    if not (score.is_cuda and score.dtype == torch.float32 and score.is_contiguous() and tuple(score.shape) == (B, H)):
        raise ValueError("score must be a contiguous fp32 CUDA tensor [B, H]")
    if stream is None:
        stream = torch.cuda.current_stream(q.device).cuda_stream
    st = lib.calibatt_spatial_similarity_static(q.data_ptr(), k.data_ptr(), B, H, N, D, partner.data_ptr(),
                                                partner.numel(), int(row_len), float(scale), score.data_ptr(),
                                                C.c_void_p(stream))
    if st != 0:
        raise CalibattError(st, "calibatt_spatial_similarity_static")
    return score

"""ctypes binding of libntp.so: argument marshalling only.

Each function has the name of the C entry point it calls (include/ntp.h).  Tensors
are torch tensors used as device memory; the current torch stream is passed through.
There is no fallback: if the library is not built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libntp.so")

NTP_OK = 0
NTP_ERR_INVALID_ARG = -1
NTP_ERR_ALIGNMENT = -2
NTP_ERR_LAUNCH = -3
NTP_ERR_UNSUPPORTED = -4
NTP_ERR_NOT_PREPARED = -5
NTP_ERR_NO_DEVICE = -6
NTP_ERR_SCRATCH_TOO_SMALL = -7
NTP_STATIC_SCRATCH_BYTES = 32 << 20
NTP_OPT_GEMM_TILE = 0
NTP_OPT_GEMM_SPLIT = 1
NTP_OPT_GEMM_NO_RING_TAIL = 2
NTP_OPT_ATTN_PARTS = 3
NTP_OPT_RESHARD_BLOCK = 4
NTP_OPT_RESHARD_FLAT_BLOCK = 5
NTP_OPT_RESHARD_TABLE_BLOCK = 6
NTP_OPT_RESHARD_NO_FLAT = 7
NTP_OPT_RESHARD_NO_TABLE = 8
NTP_OPT_GEMM_SCHEDULE = 9
NTP_OPT_GEMM_WORKGROUPS = 10
NTP_OPT_ATTN_COPY = 11
NTP_OPT_ATTN_BWD_LAUNCHES = 12
NTP_PROBE_MFMA = 0
NTP_PROBE_LDS_B128 = 1
NTP_PROBE_LDS_TR_B64 = 2
NTP_PROBE_MFMA_LDS_B128 = 3
NTP_PROBE_MFMA_LDS_TR_B64 = 4
NTP_PROBE_MFMA_1WAVE = 5
NTP_PROBE_SOFTMAX_1WAVE = 6
NTP_PROBE_MFMA_AND_SOFTMAX = 7
NTP_CALL_MLP_SHARD = 0
NTP_CALL_ATTN_PROJ_SHARD = 1
NTP_CALL_ATTN_CORE_SHARD = 2
# NTP_OPT_GEMM_TILE values by name
GEMM_TILES = {"auto": 0, "generic": 1, "256x256": 2, "256x224": 3, "224x256": 4, "256x192": 5, "192x256": 6,
              "256x128": 7, "128x256": 8, "128x128": 9, "128x128w8": 10}
NTP_GELU_ERF = 0
NTP_GELU_TANH = 1
NTP_KIND_PLAIN = 0
NTP_KIND_QKV_GQA = 1

EXPORTS = (
    "ntp_version", "ntp_status_string", "ntp_shard_plan", "ntp_attn_shard_plan", "ntp_mlp_shard_fwd",
    "ntp_mlp_shard_bwd", "ntp_attn_proj_shard_fwd", "ntp_attn_proj_shard_bwd", "ntp_reshard_segments",
    "ntp_reshard_grad", "ntp_kernel_timing_enable", "ntp_kernel_timing_read", "ntp_calibration_copy",
    "ntp_comp_sync_plan", "ntp_reshard_plan_create", "ntp_reshard_plan_segments", "ntp_reshard_plan_splits",
    "ntp_reshard_plan_table", "ntp_reshard_plan_prepare", "ntp_reshard_plan_run", "ntp_reshard_plan_destroy", "ntp_reshard_row_segments",
    "ntp_mlp_shard_bwd_resharded", "ntp_attn_proj_shard_bwd_resharded", "ntp_attn_core_shard_fwd", "ntp_attn_core_shard_bwd",
    "ntp_set_workspace", "ntp_gemm_choice", "ntp_attn_core_choice", "ntp_create", "ntp_destroy", "ntp_device_info",
    "ntp_set_option", "ntp_workspace_bytes", "ntp_attn_proj_shard_fwd_static", "ntp_replica_sum", "ntp_probe_rates",
)


class GemmChoice(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("tile_m", "tile_n", "wavefronts", "ring", "k_splits", "persistent", "pingpong")]


class AttnCoreChoice(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("fwd_rows_per_wavefront", "fwd_parts", "dq_parts", "dkv_parts")]


class NtpError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


class AttnPlan(C.Structure):
    _fields_ = [("q_off", C.c_int32), ("q_cnt", C.c_int32), ("kv_off", C.c_int32), ("kv_cnt", C.c_int32),
                ("head_dim", C.c_int32), ("w_qkv", C.c_int32), ("w_o", C.c_int32)]


class MlpShape(C.Structure):
    _fields_ = [("M", C.c_int64), ("H", C.c_int64), ("n_r", C.c_int64), ("gelu_mode", C.c_int32)]


class AttnShape(C.Structure):
    _fields_ = [("M", C.c_int64), ("H", C.c_int64), ("w_qkv", C.c_int64), ("w_o", C.c_int64)]


class TensorSpec(C.Structure):
    _fields_ = [("rows", C.c_int64), ("cols", C.c_int64), ("partition_dim", C.c_int32), ("unit", C.c_int32),
                ("elem_size", C.c_int32), ("kind", C.c_int32), ("n_q", C.c_int32), ("n_kv", C.c_int32)]


class Segment(C.Structure):
    _fields_ = [("src_rank", C.c_int32), ("dst_rank", C.c_int32), ("src_unit", C.c_int64),
                ("dst_unit", C.c_int64), ("units", C.c_int64)]


class AttnCoreShape(C.Structure):
    _fields_ = [("n_seq", C.c_int32), ("seq_len", C.c_int32), ("q_cnt", C.c_int32), ("kv_cnt", C.c_int32),
                ("q_off", C.c_int32), ("kv_off", C.c_int32), ("group", C.c_int32), ("head_dim", C.c_int32),
                ("causal", C.c_int32)]


class RowSegment(C.Structure):
    _fields_ = [("row_begin", C.c_int64), ("rows", C.c_int64), ("dst", C.c_void_p), ("ld", C.c_int64)]


class UnitSource(C.Structure):
    _fields_ = [("src_rank", C.c_int32), ("src_unit", C.c_int32)]


class ProbeResult(C.Structure):
    _fields_ = [("ms", C.c_double), ("tflops", C.c_double), ("lds_gbps_per_cu", C.c_double), ("mfma_per_turn", C.c_int32),
                ("reads_per_turn", C.c_int32)]


class KernelTime(C.Structure):
    _fields_ = [("name", C.c_char * 48), ("flops", C.c_double), ("bytes", C.c_double), ("ms", C.c_float),
                ("pad_", C.c_int32)]


_lib = None


def lib() -> C.CDLL:
    """The loaded library.  Raises if it has not been built (python -m paper_2504_06095_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2504_06095_amd.build`")
        # PyTorch first: the library and PyTorch must share one HIP runtime in the process, and the one that is
        # loaded first is the one both use (PyTorch ships its own copy)
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        L.ntp_version.restype = C.c_int
        L.ntp_status_string.restype = C.c_char_p
        L.ntp_status_string.argtypes = [C.c_int]
        L.ntp_shard_plan.argtypes = [C.c_int64, C.c_int32, C.c_int32, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
        L.ntp_attn_shard_plan.argtypes = [C.c_int32] * 5 + [C.POINTER(AttnPlan)]
        vp, i64 = C.c_void_p, C.c_int64
        L.ntp_create.argtypes = [C.POINTER(vp)]
        L.ntp_destroy.argtypes = [vp]
        L.ntp_device_info.argtypes = [vp, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.ntp_set_option.argtypes = [vp, C.c_int32, i64]
        L.ntp_workspace_bytes.argtypes = [vp, C.c_int32, vp, C.POINTER(i64)]
        L.ntp_mlp_shard_fwd.argtypes = [vp, C.POINTER(MlpShape)] + [vp, i64] * 6 + [vp]
        L.ntp_mlp_shard_bwd.argtypes = [vp, C.POINTER(MlpShape)] + [vp, i64] * 10 + [C.c_int32, vp]
        L.ntp_attn_proj_shard_fwd.argtypes = [vp, C.POINTER(AttnShape)] + [vp, i64] * 6 + [vp]
        L.ntp_attn_proj_shard_bwd.argtypes = [vp, C.POINTER(AttnShape)] + [vp, i64] * 10 + [C.c_int32, vp]
        L.ntp_attn_proj_shard_fwd_static.argtypes = L.ntp_attn_proj_shard_fwd.argtypes
        L.ntp_reshard_segments.argtypes = [C.POINTER(TensorSpec), C.c_int32, C.c_int32, C.POINTER(Segment), i64,
                                           C.POINTER(i64)]
        L.ntp_probe_rates.argtypes = [vp, C.c_int32, vp, i64, C.POINTER(ProbeResult)]
        L.ntp_replica_sum.argtypes = [vp, C.POINTER(TensorSpec), C.c_int32, C.POINTER(vp), C.POINTER(i64), vp]
        L.ntp_reshard_grad.argtypes = [vp, C.POINTER(TensorSpec), C.c_int32, C.c_int32, C.POINTER(vp), C.POINTER(i64),
                                       C.POINTER(vp), C.POINTER(i64), vp]
        i32p = C.POINTER(C.c_int32)
        L.ntp_comp_sync_plan.argtypes = [i64, C.c_int32, C.c_int32, i32p, i32p]
        L.ntp_reshard_plan_create.argtypes = [C.POINTER(TensorSpec), i64, C.c_int32, i32p, C.c_int32, i32p, C.POINTER(vp)]
        L.ntp_reshard_plan_segments.argtypes = [vp, C.POINTER(Segment), i64, C.POINTER(i64)]
        L.ntp_reshard_plan_splits.argtypes = [vp, C.POINTER(i64)]
        L.ntp_reshard_plan_table.argtypes = [vp, C.POINTER(UnitSource), i64, C.POINTER(i64)]
        L.ntp_reshard_plan_prepare.argtypes = [vp]
        L.ntp_reshard_plan_run.argtypes = [vp, vp, C.POINTER(vp), C.POINTER(i64), C.POINTER(vp), C.POINTER(i64), vp]
        L.ntp_reshard_plan_destroy.argtypes = [vp]
        segp = C.POINTER(RowSegment)
        L.ntp_reshard_row_segments.argtypes = [C.POINTER(TensorSpec), C.c_int32, C.c_int32, C.c_int32, C.POINTER(vp),
                                               C.POINTER(i64), segp, i64, C.POINTER(i64)]
        L.ntp_mlp_shard_bwd_resharded.argtypes = ([vp, C.POINTER(MlpShape)] + [vp, i64] * 8 + [segp, C.c_int32, segp, C.c_int32]
                                                  + [C.c_int32, vp])
        L.ntp_attn_proj_shard_bwd_resharded.argtypes = ([vp, C.POINTER(AttnShape)] + [vp, i64] * 8
                                                        + [segp, C.c_int32, segp, C.c_int32] + [C.c_int32, vp])
        L.ntp_attn_core_shard_fwd.argtypes = [vp, C.POINTER(AttnCoreShape), vp, i64, vp, i64, vp, vp]
        L.ntp_attn_core_shard_bwd.argtypes = [vp, C.POINTER(AttnCoreShape), vp, i64, vp, i64, vp, i64, vp, vp, vp, i64, vp]
        L.ntp_kernel_timing_enable.argtypes = [vp, C.c_int32]
        L.ntp_kernel_timing_read.argtypes = [vp, C.POINTER(KernelTime), i64, C.POINTER(i64)]
        L.ntp_calibration_copy.argtypes = [vp, vp, vp, i64, vp]
        L.ntp_set_workspace.argtypes = [vp, vp, i64]
        L.ntp_gemm_choice.argtypes = [vp, C.c_int32, i64, i64, i64, C.POINTER(GemmChoice)]
        L.ntp_attn_core_choice.argtypes = [vp, C.POINTER(AttnCoreShape), C.POINTER(AttnCoreChoice)]
        for name in EXPORTS:
            getattr(L, name)  # AttributeError if a declared symbol is not exported
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().ntp_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != NTP_OK:
        raise NtpError(status, where)


def _stream() -> int:
    import torch
    return int(torch.cuda.current_stream().cuda_stream)


def _mat(t, dtype=None):
    """(device pointer, leading dimension in elements) of a 2-D row-major tensor, or (None, 0)."""
    if t is None:
        return None, 0
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError("expected a row-major 2-D tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {t.dtype}")
    if not t.is_cuda:
        raise ValueError("expected a device tensor")
    return t.data_ptr(), int(t.stride(0))


# ---- handle ----------------------------------------------------------------------
class Handle:
    """An ntp_handle_t (ntp_create / ntp_destroy); keeps the workspace tensor it was given alive."""

    def __init__(self):
        self._h = C.c_void_p()
        self.workspace = None
        _check(lib().ntp_create(C.byref(self._h)), "ntp_create")

    @property
    def ptr(self):
        return self._h

    def destroy(self) -> None:
        if self._h:
            _check(lib().ntp_destroy(self._h), "ntp_destroy")
            self._h = C.c_void_p()
            self.workspace = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


_default = None


def default_handle() -> Handle:
    """The handle that calls without a `handle=` argument use (created on first use, on the device that is
    current then)."""
    global _default
    if _default is None:
        _default = Handle()
    return _default


def _h(handle):
    return (handle or default_handle()).ptr


def ntp_create() -> Handle:
    return Handle()


def ntp_destroy(handle: Handle) -> None:
    handle.destroy()


def ntp_device_info(handle: Handle | None = None) -> dict:
    dev, cus = C.c_int32(), C.c_int32()
    _check(lib().ntp_device_info(_h(handle), C.byref(dev), C.byref(cus)), "ntp_device_info")
    return dict(device=dev.value, compute_units=cus.value)


def ntp_set_option(option: int, value, handle: Handle | None = None) -> None:
    """Tuning override of a handle; NTP_OPT_GEMM_TILE also takes a name from GEMM_TILES."""
    if option == NTP_OPT_GEMM_TILE and isinstance(value, str):
        value = GEMM_TILES[value]
    _check(lib().ntp_set_option(_h(handle), option, int(value)), "ntp_set_option")


def ntp_workspace_bytes(call: int, shape, handle: Handle | None = None) -> int:
    """Largest workspace the call of this shape (MlpShape, AttnShape or AttnCoreShape) can use."""
    n = C.c_int64()
    _check(lib().ntp_workspace_bytes(_h(handle), call, C.byref(shape), C.byref(n)), "ntp_workspace_bytes")
    return n.value


# ---- host-only calls -------------------------------------------------------------
def ntp_version() -> int:
    return int(lib().ntp_version())


def ntp_shard_plan(dim: int, tp: int, rank: int) -> tuple[int, int]:
    off, w = C.c_int64(), C.c_int64()
    _check(lib().ntp_shard_plan(dim, tp, rank, C.byref(off), C.byref(w)), "ntp_shard_plan")
    return off.value, w.value


def ntp_attn_shard_plan(n_q: int, n_kv: int, head_dim: int, tp: int, rank: int) -> dict:
    p = AttnPlan()
    _check(lib().ntp_attn_shard_plan(n_q, n_kv, head_dim, tp, rank, C.byref(p)), "ntp_attn_shard_plan")
    return {k: getattr(p, k) for k, _ in AttnPlan._fields_}


def tensor_spec(rows, cols, partition_dim, unit=1, elem_size=4, kind=NTP_KIND_PLAIN, n_q=0, n_kv=0) -> TensorSpec:
    return TensorSpec(rows, cols, partition_dim, unit, elem_size, kind, n_q, n_kv)


def ntp_reshard_segments(spec: TensorSpec, src_tp: int, dst_tp: int) -> list[tuple[int, int, int, int, int]]:
    """[(src_rank, dst_rank, src_unit, dst_unit, units)] in destination order."""
    n = C.c_int64()
    _check(lib().ntp_reshard_segments(C.byref(spec), src_tp, dst_tp, None, 0, C.byref(n)), "ntp_reshard_segments")
    buf = (Segment * max(1, n.value))()
    _check(lib().ntp_reshard_segments(C.byref(spec), src_tp, dst_tp, buf, n.value, C.byref(n)),
           "ntp_reshard_segments")
    return [(s.src_rank, s.dst_rank, s.src_unit, s.dst_unit, s.units) for s in buf[: n.value]]


# ---- device calls ----------------------------------------------------------------
def ntp_mlp_shard_fwd(X, A_t, B, P, Y, Zpart, n_r: int, gelu_mode: int = NTP_GELU_ERF, handle=None) -> None:
    """X [M,H], A_t [n_r,H], B [n_r,H] bf16 -> P, Y [M, >=n_r] and Zpart [M,H] bf16 (all preallocated)."""
    import torch
    bf = torch.bfloat16
    shape = MlpShape(X.shape[0], X.shape[1], n_r, gelu_mode)
    args = []
    for t in (X, A_t, B, P, Y, Zpart):
        args += list(_mat(t, bf))
    _check(lib().ntp_mlp_shard_fwd(_h(handle), C.byref(shape), *args, _stream()), "ntp_mlp_shard_fwd")


def ntp_mlp_shard_bwd(dZ, X, A_t, B, P, Y, dP, dXpart, dA_t, dB, n_r: int, gelu_mode: int = NTP_GELU_ERF,
                      accumulate: bool = False, handle=None) -> None:
    import torch
    bf, f32 = torch.bfloat16, torch.float32
    shape = MlpShape(X.shape[0], X.shape[1], n_r, gelu_mode)
    args = []
    for t in (dZ, X, A_t, B, P, Y, dP, dXpart):
        args += list(_mat(t, bf))
    for t in (dA_t, dB):
        args += list(_mat(t, f32))
    _check(lib().ntp_mlp_shard_bwd(_h(handle), C.byref(shape), *args, int(bool(accumulate)), _stream()), "ntp_mlp_shard_bwd")


def ntp_attn_proj_shard_fwd(M, H, w_qkv, w_o, X=None, Wqkv=None, QKV=None, C_=None, Wo=None, Zpart=None, handle=None) -> None:
    import torch
    bf = torch.bfloat16
    shape = AttnShape(M, H, w_qkv, w_o)
    args = []
    for t in (X, Wqkv, QKV, C_, Wo, Zpart):
        args += list(_mat(t, bf))
    _check(lib().ntp_attn_proj_shard_fwd(_h(handle), C.byref(shape), *args, _stream()), "ntp_attn_proj_shard_fwd")


def ntp_attn_proj_shard_fwd_static(M, H, w_qkv, w_o, X=None, Wqkv=None, QKV=None, C_=None, Wo=None, Zpart=None,
                                   handle=None) -> None:
    """ntp_attn_proj_shard_fwd with the split-K partial sums in the library's static device array."""
    import torch
    bf = torch.bfloat16
    shape = AttnShape(M, H, w_qkv, w_o)
    args = []
    for t in (X, Wqkv, QKV, C_, Wo, Zpart):
        args += list(_mat(t, bf))
    _check(lib().ntp_attn_proj_shard_fwd_static(_h(handle), C.byref(shape), *args, _stream()), "ntp_attn_proj_shard_fwd_static")


def ntp_attn_proj_shard_bwd(M, H, w_qkv, w_o, dZ=None, dQKV=None, X=None, C_=None, Wqkv=None, Wo=None, dC=None,
                            dXpart=None, dWqkv=None, dWo=None, accumulate: bool = False, handle=None) -> None:
    import torch
    bf, f32 = torch.bfloat16, torch.float32
    shape = AttnShape(M, H, w_qkv, w_o)
    args = []
    for t in (dZ, dQKV, X, C_, Wqkv, Wo, dC, dXpart):
        args += list(_mat(t, bf))
    for t in (dWqkv, dWo):
        args += list(_mat(t, f32))
    _check(lib().ntp_attn_proj_shard_bwd(_h(handle), C.byref(shape), *args, int(bool(accumulate)), _stream()),
           "ntp_attn_proj_shard_bwd")


def attn_core_shape(n_seq, seq_len, plan: dict, group: int, causal: bool = False) -> AttnCoreShape:
    """Shape of the attention core call from a rank's ntp_attn_shard_plan and the query heads per KV head."""
    return AttnCoreShape(n_seq, seq_len, plan["q_cnt"], plan["kv_cnt"], plan["q_off"], plan["kv_off"], group,
                         plan["head_dim"], int(bool(causal)))


def ntp_attn_core_shard_fwd(shape: AttnCoreShape, QKV, C_, LSE=None, handle=None) -> None:
    """QKV [M, (q_cnt + 2 kv_cnt) d] bf16 -> C_ [M, q_cnt d] bf16 and LSE [q_cnt, M] fp32 (optional)."""
    import torch
    q, ldq = _mat(QKV, torch.bfloat16)
    c, ldc = _mat(C_, torch.bfloat16)
    lse = None
    if LSE is not None:
        if LSE.dtype != torch.float32 or not LSE.is_contiguous():
            raise TypeError("LSE: contiguous fp32 expected")
        lse = LSE.data_ptr()
    _check(lib().ntp_attn_core_shard_fwd(_h(handle), C.byref(shape), q, ldq, c, ldc, lse, _stream()), "ntp_attn_core_shard_fwd")


def ntp_attn_core_shard_bwd(shape: AttnCoreShape, QKV, C_, dC, LSE, Delta, dQKV, handle=None) -> None:
    """Gradient of the attention core: dQKV (QKV's layout) from dC; LSE from the forward call, Delta scratch
    (both contiguous fp32 [q_cnt, M])."""
    import torch
    bf = torch.bfloat16
    q, ldq = _mat(QKV, bf)
    c, ldc = _mat(C_, bf)
    g, ldg = _mat(dC, bf)
    d, ldd = _mat(dQKV, bf)
    for t in (LSE, Delta):
        if t.dtype != torch.float32 or not t.is_contiguous() or not t.is_cuda:
            raise TypeError("LSE / Delta: contiguous fp32 device tensors expected")
    _check(lib().ntp_attn_core_shard_bwd(_h(handle), C.byref(shape), q, ldq, c, ldc, g, ldg, LSE.data_ptr(), Delta.data_ptr(), d, ldd,
                                         _stream()), "ntp_attn_core_shard_bwd")


def ntp_reshard_row_segments(spec: TensorSpec, src_tp: int, src_rank: int, dst_tp: int, dst_shards):
    """Row segments (a ctypes array of RowSegment) of source rank src_rank's gradient for src_tp -> dst_tp, given
    the destination shards (2-D fp32 device tensors; None where this rank sends nothing)."""
    vp, i64 = C.c_void_p, C.c_int64
    dp, dl = (vp * dst_tp)(), (i64 * dst_tp)()
    if len(dst_shards) != dst_tp:
        raise ValueError("one entry per destination rank expected")
    for i, t in enumerate(dst_shards):
        if t is None:
            dp[i], dl[i] = None, 0
        elif isinstance(t, tuple):  # (device address, leading dimension)
            dp[i], dl[i] = t
        elif t.numel() == 0:
            dp[i], dl[i] = None, 0
        else:
            dp[i], dl[i] = _mat(t)
    n = i64()
    _check(lib().ntp_reshard_row_segments(C.byref(spec), src_tp, src_rank, dst_tp, dp, dl, None, 0, C.byref(n)),
           "ntp_reshard_row_segments")
    buf = (RowSegment * max(1, n.value))()
    _check(lib().ntp_reshard_row_segments(C.byref(spec), src_tp, src_rank, dst_tp, dp, dl, buf, n.value, C.byref(n)),
           "ntp_reshard_row_segments")
    return (RowSegment * n.value)(*buf[: n.value]) if n.value else (RowSegment * 0)()


def row_segments(items):
    """A ctypes array of RowSegment from [(row_begin, rows, tensor_or_pointer, ld)]."""
    arr = (RowSegment * len(items))()
    for i, (b, r, d, ld) in enumerate(items):
        arr[i] = RowSegment(b, r, d if isinstance(d, int) or d is None else d.data_ptr(), ld)
    return arr


def ntp_mlp_shard_bwd_resharded(dZ, X, A_t, B, P, Y, dP, dXpart, dA_segs, dB_segs, n_r: int,
                                gelu_mode: int = NTP_GELU_ERF, accumulate: bool = False, handle=None) -> None:
    """As ntp_mlp_shard_bwd; dA_segs / dB_segs are ctypes arrays of RowSegment."""
    import torch
    bf = torch.bfloat16
    shape = MlpShape(X.shape[0], X.shape[1], n_r, gelu_mode)
    args = []
    for t in (dZ, X, A_t, B, P, Y, dP, dXpart):
        args += list(_mat(t, bf))
    _check(lib().ntp_mlp_shard_bwd_resharded(_h(handle), C.byref(shape), *args, dA_segs, len(dA_segs), dB_segs, len(dB_segs),
                                             int(bool(accumulate)), _stream()), "ntp_mlp_shard_bwd_resharded")


def ntp_attn_proj_shard_bwd_resharded(M, H, w_qkv, w_o, dZ=None, dQKV=None, X=None, C_=None, Wqkv=None, Wo=None, dC=None,
                                      dXpart=None, dWqkv_segs=None, dWo_segs=None, accumulate: bool = False,
                                      handle=None) -> None:
    """As ntp_attn_proj_shard_bwd; dWqkv_segs / dWo_segs are ctypes arrays of RowSegment."""
    import torch
    bf = torch.bfloat16
    shape = AttnShape(M, H, w_qkv, w_o)
    args = []
    for t in (dZ, dQKV, X, C_, Wqkv, Wo, dC, dXpart):
        args += list(_mat(t, bf))
    q = dWqkv_segs if dWqkv_segs is not None else (RowSegment * 0)()
    o = dWo_segs if dWo_segs is not None else (RowSegment * 0)()
    _check(lib().ntp_attn_proj_shard_bwd_resharded(_h(handle), C.byref(shape), *args, q, len(q), o, len(o), int(bool(accumulate)),
                                                   _stream()), "ntp_attn_proj_shard_bwd_resharded")


def _shard_arrays(spec: TensorSpec, src_tp: int, dst_tp: int, src_shards, dst_shards):
    vp, i64 = C.c_void_p, C.c_int64
    sp, sl = (vp * src_tp)(), (i64 * src_tp)()
    dp, dl = (vp * dst_tp)(), (i64 * dst_tp)()
    if len(src_shards) != src_tp or len(dst_shards) != dst_tp:
        raise ValueError("one entry per rank expected")
    for arr_p, arr_l, shards in ((sp, sl, src_shards), (dp, dl, dst_shards)):
        for i, t in enumerate(shards):
            if t is None or t.numel() == 0:
                arr_p[i], arr_l[i] = None, 0
                continue
            if t.element_size() != spec.elem_size:
                raise TypeError("element size of a shard differs from the spec")
            p, ld = _mat(t)
            arr_p[i], arr_l[i] = p, ld
    return sp, sl, dp, dl


def ntp_reshard_grad(spec: TensorSpec, src_tp: int, dst_tp: int, src_shards, dst_shards, handle=None) -> None:
    """src_shards / dst_shards: lists of 2-D device tensors (or None for "not on this GPU")."""
    sp, sl, dp, dl = _shard_arrays(spec, src_tp, dst_tp, src_shards, dst_shards)
    _check(lib().ntp_reshard_grad(_h(handle), C.byref(spec), src_tp, dst_tp, sp, sl, dp, dl, _stream()), "ntp_reshard_grad")


def ntp_replica_sum(spec: TensorSpec, tp: int, shards, handle=None) -> None:
    """shards: list of 2-D fp32 device tensors of the TP = tp layout (or None for "not on this GPU"), updated in place."""
    vp, i64 = C.c_void_p, C.c_int64
    if len(shards) != tp:
        raise ValueError("one entry per rank expected")
    sp, sl = (vp * tp)(), (i64 * tp)()
    for i, t in enumerate(shards):
        if t is None or t.numel() == 0:
            sp[i], sl[i] = None, 0
        else:
            sp[i], sl[i] = _mat(t)
    _check(lib().ntp_replica_sum(_h(handle), C.byref(spec), tp, sp, sl, _stream()), "ntp_replica_sum")


class ReshardPlan:
    """Handle of a reshard plan between two unit -> rank maps; the methods carry the names of the
    entry points they call.  Destroyed with the object (or by destroy())."""

    def __init__(self, spec: TensorSpec, src_tp: int, src_rank_of_unit, dst_tp: int, dst_rank_of_unit):
        n = len(src_rank_of_unit)
        if len(dst_rank_of_unit) != n:
            raise ValueError("the two maps must cover the same units")
        self.spec, self.src_tp, self.dst_tp, self.n_units = spec, src_tp, dst_tp, n
        a = (C.c_int32 * max(1, n))(*[int(x) for x in src_rank_of_unit])
        b = (C.c_int32 * max(1, n))(*[int(x) for x in dst_rank_of_unit])
        self._h = C.c_void_p()
        _check(lib().ntp_reshard_plan_create(C.byref(spec), n, src_tp, a, dst_tp, b, C.byref(self._h)),
               "ntp_reshard_plan_create")

    def ntp_reshard_plan_segments(self) -> list[tuple[int, int, int, int, int]]:
        n = C.c_int64()
        _check(lib().ntp_reshard_plan_segments(self._h, None, 0, C.byref(n)), "ntp_reshard_plan_segments")
        buf = (Segment * max(1, n.value))()
        _check(lib().ntp_reshard_plan_segments(self._h, buf, n.value, C.byref(n)), "ntp_reshard_plan_segments")
        return [(s.src_rank, s.dst_rank, s.src_unit, s.dst_unit, s.units) for s in buf[: n.value]]

    def ntp_reshard_plan_splits(self) -> list[list[int]]:
        buf = (C.c_int64 * max(1, self.src_tp * self.dst_tp))()
        _check(lib().ntp_reshard_plan_splits(self._h, buf), "ntp_reshard_plan_splits")
        return [[buf[r * self.dst_tp + s] for s in range(self.dst_tp)] for r in range(self.src_tp)]

    def ntp_reshard_plan_table(self) -> list[tuple[int, int]]:
        n = C.c_int64()
        buf = (UnitSource * max(1, self.n_units))()
        _check(lib().ntp_reshard_plan_table(self._h, buf, self.n_units, C.byref(n)), "ntp_reshard_plan_table")
        return [(e.src_rank, e.src_unit) for e in buf[: n.value]]

    def ntp_reshard_plan_prepare(self) -> None:
        """Make the plan ready to run on the current device (uploads its run table); needed once before the first run."""
        _check(lib().ntp_reshard_plan_prepare(self._h), "ntp_reshard_plan_prepare")

    def ntp_reshard_plan_run(self, src_shards, dst_shards, handle=None) -> None:
        sp, sl, dp, dl = _shard_arrays(self.spec, self.src_tp, self.dst_tp, src_shards, dst_shards)
        _check(lib().ntp_reshard_plan_run(_h(handle), self._h, sp, sl, dp, dl, _stream()), "ntp_reshard_plan_run")

    def destroy(self) -> None:
        if self._h:
            _check(lib().ntp_reshard_plan_destroy(self._h), "ntp_reshard_plan_destroy")
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def ntp_comp_sync_plan(k: int, full_tp: int, reduced_tp: int) -> tuple[list[int], list[int]]:
    """(comp_rank, sync_rank): rank of every unit in the compute and in the synchronisation layout."""
    comp, sync = (C.c_int32 * max(1, k))(), (C.c_int32 * max(1, k))()
    _check(lib().ntp_comp_sync_plan(k, full_tp, reduced_tp, comp, sync), "ntp_comp_sync_plan")
    return list(comp[:k]), list(sync[:k])


def ntp_reshard_plan_create(spec: TensorSpec, src_tp: int, src_rank_of_unit, dst_tp: int, dst_rank_of_unit) -> ReshardPlan:
    return ReshardPlan(spec, src_tp, src_rank_of_unit, dst_tp, dst_rank_of_unit)


# ---- measurement aid ---------------------------------------------------------------
def ntp_kernel_timing_enable(on: bool, handle=None) -> None:
    _check(lib().ntp_kernel_timing_enable(_h(handle), int(bool(on))), "ntp_kernel_timing_enable")


def ntp_kernel_timing_read(max_records: int = 4096, handle=None) -> list[dict]:
    """Waits for the recorded launches; returns [{name, flops, bytes, ms}] in launch order."""
    buf = (KernelTime * max_records)()
    n = C.c_int64()
    _check(lib().ntp_kernel_timing_read(_h(handle), buf, max_records, C.byref(n)), "ntp_kernel_timing_read")
    return [dict(name=r.name.decode(), flops=r.flops, bytes=r.bytes, ms=r.ms) for r in buf[: min(n.value, max_records)]]


def ntp_probe_rates(which: int, scratch, handle=None) -> dict:
    """Sustained matrix / LDS-read rates of the device (blocking measurement aid); scratch: a device tensor."""
    out = ProbeResult()
    _check(lib().ntp_probe_rates(_h(handle), which, scratch.data_ptr(), scratch.numel() * scratch.element_size(), C.byref(out)),
           "ntp_probe_rates")
    return {n: getattr(out, n) for n, _ in ProbeResult._fields_}


def ntp_calibration_copy(dst, src, handle=None) -> None:
    """Plain dense copy src -> dst (contiguous device tensors of equal byte size)."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes or not (src.is_contiguous() and dst.is_contiguous()):
        raise ValueError("expected two contiguous tensors of equal byte size")
    _check(lib().ntp_calibration_copy(_h(handle), dst.data_ptr(), src.data_ptr(), nbytes, _stream()), "ntp_calibration_copy")


def ntp_set_workspace(workspace, handle: Handle | None = None) -> None:
    """Give the handle a device tensor (any dtype, contiguous) as its workspace, or None to remove it."""
    hd = handle or default_handle()
    if workspace is None:
        _check(lib().ntp_set_workspace(hd.ptr, None, 0), "ntp_set_workspace")
        hd.workspace = None
        return
    if not workspace.is_contiguous():
        raise ValueError("expected a contiguous tensor")
    _check(lib().ntp_set_workspace(hd.ptr, workspace.data_ptr(), workspace.numel() * workspace.element_size()), "ntp_set_workspace")
    hd.workspace = workspace


def ntp_gemm_choice(layout: int, M: int, N: int, K: int, handle=None) -> dict:
    """Kernel variant a shard GEMM of this shape would run (host only); layout 0 nt, 1 nn, 2 tn."""
    out = GemmChoice()
    _check(lib().ntp_gemm_choice(_h(handle), layout, M, N, K, C.byref(out)), "ntp_gemm_choice")
    return {n: getattr(out, n) for n, _ in GemmChoice._fields_}


def ntp_attn_core_choice(shape, handle=None) -> dict:
    """Launch decisions of the attention core kernels for an AttnCoreShape (host only)."""
    out = AttnCoreChoice()
    _check(lib().ntp_attn_core_choice(_h(handle), C.byref(shape), C.byref(out)), "ntp_attn_core_choice")
    return {n: getattr(out, n) for n, _ in AttnCoreChoice._fields_}

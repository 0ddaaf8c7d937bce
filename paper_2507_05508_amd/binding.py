"""ctypes binding of libmlmc.so: the same entry points as include/mlmc.h, taking torch CUDA tensors.

Argument marshalling only -- every step of the method runs in the HIP kernels of the library.  torch is
used for device memory and for the current stream.  There is no CPU fallback: if the library has not
been built (python -m paper_2507_05508_amd.build) loading fails with an error.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libmlmc.so")

MLMC_OK, MLMC_EINVAL, MLMC_ENOMEM, MLMC_EHIP, MLMC_ELIMIT = 0, 1, 2, 3, 4
MLMC_STATIC_SCRATCH_BYTES = 1 << 20
MLMC_DEV_CAPACITY, MLMC_DEV_NONFINITE, MLMC_DEV_INTERNAL, MLMC_DEV_REDONE = 1, 2, 4, 8
MLMC_F32, MLMC_BF16 = 0, 1
MLMC_TOPK, MLMC_BITS, MLMC_FBITS, MLMC_STOPK, MLMC_VBITS, MLMC_RTN = 0, 1, 2, 3, 4, 5
MLMC_MAX_SLEVELS = 65536
MLMC_TILE = 4096
MLMC_MAX_LEVELS = 32

EXPORTS = ["mlmc_plan", "mlmc_plan_destroy", "mlmc_plan_set_sampling", "mlmc_plan_set_staging", "mlmc_plan_set_overlap", "mlmc_plan_num_tiles", "mlmc_plan_chunk", "mlmc_plan_num_planes", "mlmc_geometric_p",
           "mlmc_status_string", "mlmc_level_norms", "mlmc_compress_topk", "mlmc_compress_bits", "mlmc_compress_bits_static", "mlmc_compress_rtn", "mlmc_aggregate", "mlmc_aggregate_update", "mlmc_message_bits",
           "mlmc_profile_enable", "mlmc_profile_reset", "mlmc_profile_num_kernels", "mlmc_profile_kernel_name",
           "mlmc_profile_get"]

_lib = None


class MlmcError(RuntimeError):
    pass


def lib():
    """The loaded library (loads on first use; raises if it was not built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise MlmcError(f"{LIB_PATH} is missing: build it with `python -m paper_2507_05508_amd.build`")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, u64, dbl_p = C.c_void_p, C.c_int, C.c_int64, C.c_uint64, C.POINTER(C.c_double)
        L.mlmc_plan.restype = C.c_int
        L.mlmc_plan.argtypes = [C.POINTER(vp), i32, i32, i64, i32, i32, C.POINTER(i64), dbl_p,
                                C.POINTER(C.c_size_t), C.POINTER(i64)]
        L.mlmc_plan_destroy.restype = None
        L.mlmc_plan_destroy.argtypes = [vp]
        L.mlmc_plan_set_sampling.restype = C.c_int
        L.mlmc_plan_set_sampling.argtypes = [vp, i32]
        L.mlmc_plan_set_staging.restype = C.c_int
        L.mlmc_plan_set_staging.argtypes = [vp, i32]
        L.mlmc_plan_set_overlap.restype = C.c_int
        L.mlmc_plan_set_overlap.argtypes = [vp, i32]
        L.mlmc_plan_num_tiles.restype = i64
        L.mlmc_plan_num_tiles.argtypes = [vp]
        L.mlmc_plan_chunk.restype = i64
        L.mlmc_plan_chunk.argtypes = [vp]
        L.mlmc_plan_num_planes.restype = i32
        L.mlmc_plan_num_planes.argtypes = [vp]
        L.mlmc_geometric_p.restype = C.c_int
        L.mlmc_geometric_p.argtypes = [i32, dbl_p]
        L.mlmc_status_string.restype = C.c_char_p
        L.mlmc_status_string.argtypes = [i32]
        L.mlmc_level_norms.restype = C.c_int
        L.mlmc_level_norms.argtypes = [vp, vp, i64, vp, vp, vp, vp]
        L.mlmc_compress_topk.restype = C.c_int
        L.mlmc_compress_topk.argtypes = [vp, vp, i64, vp, i32, u64, u64, vp, vp, vp, vp, i64, vp, vp, vp, vp, vp]
        L.mlmc_compress_bits.restype = C.c_int
        L.mlmc_compress_bits.argtypes = [vp, vp, i64, u64, u64, vp, vp, vp, vp, vp, vp]
        L.mlmc_compress_rtn.restype = C.c_int
        L.mlmc_compress_rtn.argtypes = [vp, vp, i64, u64, u64, vp, vp, vp, vp, vp, vp, vp]
        L.mlmc_compress_bits_static.restype = C.c_int
        L.mlmc_compress_bits_static.argtypes = [vp, vp, i64, u64, u64, vp, vp, vp, vp, vp]
        L.mlmc_aggregate.restype = C.c_int
        L.mlmc_aggregate.argtypes = [vp, vp, vp, vp, vp, i64, vp, vp, vp, C.c_float, vp, vp, vp]
        L.mlmc_aggregate_update.restype = C.c_int
        L.mlmc_aggregate_update.argtypes = [vp, vp, vp, vp, vp, i64, vp, vp, vp, C.c_float, C.c_float, vp, vp, vp, vp]
        L.mlmc_message_bits.restype = C.c_int
        L.mlmc_message_bits.argtypes = [vp, vp, vp, vp]
        L.mlmc_profile_enable.restype = None
        L.mlmc_profile_enable.argtypes = [i32]
        L.mlmc_profile_reset.restype = None
        L.mlmc_profile_reset.argtypes = []
        L.mlmc_profile_num_kernels.restype = i32
        L.mlmc_profile_num_kernels.argtypes = []
        L.mlmc_profile_kernel_name.restype = C.c_char_p
        L.mlmc_profile_kernel_name.argtypes = [i32]
        L.mlmc_profile_get.restype = C.c_int
        L.mlmc_profile_get.argtypes = [i32, dbl_p, C.POINTER(i64)]
        _lib = L
    return _lib


def mlmc_profile_enable(on: bool):
    lib().mlmc_profile_enable(int(bool(on)))


def mlmc_profile_reset():
    lib().mlmc_profile_reset()


def mlmc_profile_get():
    """{kernel name: (total device ms, launches)} since the last reset (waits for the recorded events)."""
    out = {}
    for i in range(lib().mlmc_profile_num_kernels()):
        ms, n = C.c_double(), C.c_int64()
        _check(lib().mlmc_profile_get(i, C.byref(ms), C.byref(n)), "mlmc_profile_get")
        if n.value:
            out[lib().mlmc_profile_kernel_name(i).decode()] = (ms.value, n.value)
    return out


def _check(rc: int, what: str):
    if rc != MLMC_OK:
        raise MlmcError(f"{what}: {lib().mlmc_status_string(rc).decode()}")


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def mlmc_geometric_p(L: int):
    buf = (C.c_double * L)()
    _check(lib().mlmc_geometric_p(L, buf), "mlmc_geometric_p")
    return list(buf)


class Plan:
    """Host plan + the device workspace and status word the calls need (allocated once, reused)."""

    def __init__(self, kind: int, M: int, d: int, dtype: int, ladder: Sequence[int],
                 p_fixed: Optional[Sequence[float]], device="cuda:0", allocate: bool = True):
        if kind == MLMC_STOPK:   # ladder = [s]: segments of s entries of the sorted row, L = ceil(d / s) levels
            self.s = int(ladder[0])
            L = -(-d // self.s) if self.s >= 1 else 0
            self.ladder = [min(self.s * l, d) for l in range(L + 1)] if 1 <= L <= MLMC_MAX_SLEVELS else [self.s]
            lad = (C.c_int64 * 1)(self.s)
        else:
            L = len(ladder) - 1
            self.ladder = [int(x) for x in ladder]
            lad = (C.c_int64 * (L + 1))(*self.ladder)
        self.kind, self.M, self.d, self.dtype, self.L = kind, M, d, dtype, L
        self.p_fixed = None if p_fixed is None else [float(x) for x in p_fixed]
        pf = None if p_fixed is None else (C.c_double * L)(*self.p_fixed)
        handle, wsb, cap = C.c_void_p(), C.c_size_t(), C.c_int64()
        rc = lib().mlmc_plan(C.byref(handle), kind, M, d, dtype, L, lad, pf, C.byref(wsb), C.byref(cap))
        _check(rc, "mlmc_plan")
        self.handle = handle
        self.workspace_bytes = wsb.value
        self.sparse_capacity_worst = cap.value
        self.num_tiles = lib().mlmc_plan_num_tiles(handle)
        self.num_planes = lib().mlmc_plan_num_planes(handle)
        self.chunk = lib().mlmc_plan_chunk(handle)
        self.device = torch.device(device)
        self.ws = None
        self.dev_status = None
        if allocate:
            self.ws = torch.empty(self.workspace_bytes + 256, dtype=torch.uint8, device=self.device)
            assert self.ws.data_ptr() % 256 == 0
            self.dev_status = torch.zeros(1, dtype=torch.int32, device=self.device)

    def close(self):
        if getattr(self, "handle", None):
            lib().mlmc_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_sampling(self, shift: int):
        """Histogram sampling of the threshold search: one block out of 2^shift (run time only, never results)."""
        _check(lib().mlmc_plan_set_sampling(self.handle, int(shift)), "mlmc_plan_set_sampling")

    def set_staging(self, enable: bool):
        """Stage the drawn band's members during the selection read (run time only, never results)."""
        _check(lib().mlmc_plan_set_staging(self.handle, int(bool(enable))), "mlmc_plan_set_staging")

    def set_overlap(self, enable: bool):
        """Run the second read of unstaged rows on the plan's side stream, beside the assembly of the other rows' messages
        (run time only, never results)."""
        _check(lib().mlmc_plan_set_overlap(self.handle, int(bool(enable))), "mlmc_plan_set_overlap")

    def status(self, informational: bool = False) -> int:
        """Device status bits of the last call (synchronises).  MLMC_DEV_REDONE is not an error and is only
        reported when `informational` is set."""
        s = int(self.dev_status.item())
        return s if informational else s & ~MLMC_DEV_REDONE


def mlmc_plan(kind, M, d, dtype, ladder, p_fixed=None, device="cuda:0", allocate=True) -> Plan:
    return Plan(kind, M, d, dtype, ladder, p_fixed, device, allocate)


def _check_g(plan: Plan, g: torch.Tensor):
    want = torch.float32 if plan.dtype == MLMC_F32 else torch.bfloat16
    if g.dtype != want or g.dim() != 2 or g.shape[0] != plan.M or g.shape[1] != plan.d or g.stride(1) != 1 or not g.is_cuda:
        raise MlmcError(f"g must be a CUDA {want} tensor [M={plan.M}, d={plan.d}] with unit inner stride")
    return g.stride(0)


def mlmc_level_norms(plan: Plan, g: torch.Tensor, norms: Optional[torch.Tensor] = None) -> torch.Tensor:
    ld = _check_g(plan, g)
    if norms is None:
        norms = torch.empty((plan.M, plan.L), dtype=torch.float64, device=g.device)
    rc = lib().mlmc_level_norms(plan.handle, _ptr(g), ld, _ptr(norms), _ptr(plan.dev_status), _ptr(plan.ws), _stream())
    _check(rc, "mlmc_level_norms")
    return norms


class SparseMessage:
    """Device buffers of one mlmc_compress_topk call (reused across steps when passed back in)."""

    def __init__(self, plan: Plan, capacity: Optional[int] = None, with_norms: bool = False):
        dev = plan.device
        self.capacity = plan.sparse_capacity_worst if capacity is None else int(capacity)
        self.level = torch.empty(plan.M, dtype=torch.int32, device=dev)
        self.row_off = torch.empty(plan.M + 1, dtype=torch.int64, device=dev)
        self.idx = torch.empty(max(self.capacity, 1), dtype=torch.int32, device=dev)   # uint32 payload
        self.val = torch.empty(max(self.capacity, 1), dtype=torch.float32, device=dev)
        self.tile_off = torch.empty((plan.M, plan.num_tiles + 1), dtype=torch.int32, device=dev)
        self.norms = torch.empty((plan.M, plan.L), dtype=torch.float64, device=dev) if with_norms else None


def mlmc_compress_topk(plan: Plan, g: torch.Tensor, seed: int, step: int, p: Optional[torch.Tensor] = None,
                       p_is_norms: bool = False, out: Optional[SparseMessage] = None) -> SparseMessage:
    ld = _check_g(plan, g)
    if out is None:
        out = SparseMessage(plan, with_norms=(plan.p_fixed is None and p is None))
    if p is not None and (p.dtype != torch.float64 or tuple(p.shape) != (plan.M, plan.L) or not p.is_contiguous()):
        raise MlmcError("p must be a contiguous float64 CUDA tensor [M, L]")
    rc = lib().mlmc_compress_topk(plan.handle, _ptr(g), ld, _ptr(p), int(bool(p_is_norms)), seed, step,
                                  _ptr(out.level), _ptr(out.row_off), _ptr(out.idx), _ptr(out.val), out.capacity,
                                  _ptr(out.tile_off), _ptr(out.norms), _ptr(plan.dev_status), _ptr(plan.ws), _stream())
    _check(rc, "mlmc_compress_topk")
    return out


class BitsMessage:
    def __init__(self, plan: Plan):
        dev = plan.device
        self.nwords = (plan.d + 63) // 64
        self.level = torch.empty(plan.M, dtype=torch.int32, device=dev)
        # per row: the scale exponent (MLMC_BITS), the bits of the largest entry (MLMC_VBITS), or, for MLMC_RTN, two
        # words: the bits of c and of the coefficient
        self.scale_exp = torch.empty((plan.M, 2) if plan.kind == MLMC_RTN else (plan.M,), dtype=torch.int32, device=dev)
        self.norms = torch.empty((plan.M, plan.L), dtype=torch.float64, device=dev) if plan.kind == MLMC_RTN else None
        self.planes = torch.zeros((plan.M, plan.num_planes, self.nwords), dtype=torch.int64, device=dev)  # uint64 payload


def mlmc_compress_bits(plan: Plan, g: torch.Tensor, seed: int, step: int, out: Optional[BitsMessage] = None) -> BitsMessage:
    ld = _check_g(plan, g)
    if out is None:
        out = BitsMessage(plan)
    rc = lib().mlmc_compress_bits(plan.handle, _ptr(g), ld, seed, step, _ptr(out.level), _ptr(out.scale_exp),
                                  _ptr(out.planes), _ptr(plan.dev_status), _ptr(plan.ws), _stream())
    _check(rc, "mlmc_compress_bits")
    return out


def mlmc_compress_rtn(plan: Plan, g: torch.Tensor, seed: int, step: int, out: Optional[BitsMessage] = None) -> BitsMessage:
    ld = _check_g(plan, g)
    if out is None:
        out = BitsMessage(plan)
    rc = lib().mlmc_compress_rtn(plan.handle, _ptr(g), ld, seed, step, _ptr(out.level), _ptr(out.scale_exp), _ptr(out.planes),
                                 _ptr(out.norms), _ptr(plan.dev_status), _ptr(plan.ws), _stream())
    _check(rc, "mlmc_compress_rtn")
    return out


def mlmc_compress_bits_static(plan: Plan, g: torch.Tensor, seed: int, step: int, out: BitsMessage,
                              dev_status: torch.Tensor) -> BitsMessage:
    """mlmc_compress_bits without a workspace (the library's static device scratch).  `out` and `dev_status` are
    the caller's: this call allocates nothing."""
    ld = _check_g(plan, g)
    rc = lib().mlmc_compress_bits_static(plan.handle, _ptr(g), ld, seed, step, _ptr(out.level), _ptr(out.scale_exp),
                                         _ptr(out.planes), _ptr(dev_status), _stream())
    _check(rc, "mlmc_compress_bits_static")
    return out


def mlmc_aggregate(plan: Plan, msg, alpha: float, out: Optional[torch.Tensor] = None, use_tile_off: bool = True) -> torch.Tensor:
    if out is None:
        out = torch.empty(plan.d, dtype=torch.float32, device=plan.device)
    if plan.kind in (MLMC_TOPK, MLMC_STOPK):
        rc = lib().mlmc_aggregate(plan.handle, None, _ptr(msg.row_off), _ptr(msg.idx), _ptr(msg.val), msg.capacity,
                                  _ptr(msg.tile_off) if use_tile_off else None, None, None, float(alpha), _ptr(out),
                                  _ptr(plan.ws), _stream())
    else:
        rc = lib().mlmc_aggregate(plan.handle, _ptr(msg.level), None, None, None, 0, None, _ptr(msg.scale_exp),
                                  _ptr(msg.planes), float(alpha), _ptr(out), _ptr(plan.ws), _stream())
    _check(rc, "mlmc_aggregate")
    return out


def mlmc_aggregate_update(plan: Plan, msg, alpha: float, eta: float, x: torch.Tensor, out: Optional[torch.Tensor] = None,
                          use_tile_off: bool = True) -> torch.Tensor:
    """x <- x - eta * (alpha * sum of the workers' messages), in place; `out` (optional) also receives the update."""
    if x.dtype != torch.float32 or x.numel() != plan.d or not x.is_contiguous() or not x.is_cuda:
        raise MlmcError("x must be a contiguous float32 CUDA tensor [d]")
    if plan.kind in (MLMC_TOPK, MLMC_STOPK):
        rc = lib().mlmc_aggregate_update(plan.handle, None, _ptr(msg.row_off), _ptr(msg.idx), _ptr(msg.val), msg.capacity,
                                         _ptr(msg.tile_off) if use_tile_off else None, None, None, float(alpha), float(eta),
                                         _ptr(x), _ptr(out), _ptr(plan.ws), _stream())
    else:
        rc = lib().mlmc_aggregate_update(plan.handle, _ptr(msg.level), None, None, None, 0, None, _ptr(msg.scale_exp),
                                         _ptr(msg.planes), float(alpha), float(eta), _ptr(x), _ptr(out), _ptr(plan.ws), _stream())
    _check(rc, "mlmc_aggregate_update")
    return x


def mlmc_message_bits(plan: Plan, msg, bits: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Bits per worker that the message `msg` of this plan takes on the wire (int64 tensor [M])."""
    if bits is None:
        bits = torch.empty(plan.M, dtype=torch.int64, device=plan.device)
    _check(lib().mlmc_message_bits(plan.handle, _ptr(msg.level), _ptr(bits), _stream()), "mlmc_message_bits")
    return bits


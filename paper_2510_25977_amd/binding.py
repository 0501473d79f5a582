"""Thin ctypes binding of ``libsvdmlp.so`` (same names as ``include/svdmlp.h``).

Argument marshalling only: PyTorch supplies device memory and streams, every step of the forward
runs in the library's HIP kernels.  There is no CPU or PyTorch fallback: if the library is missing
or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
from pathlib import Path
from typing import Optional

import torch

HERE = Path(__file__).resolve().parent
LIB_PATH = HERE / "libsvdmlp.so"      # the in-tree build, nothing else

SVDMLP_BF16, SVDMLP_F32 = 0, 1
SVDMLP_GATED, SVDMLP_LINEAR = 0, 1
SVDMLP_OK = 0
SVDMLP_INVALID_ARGUMENT, SVDMLP_UNSUPPORTED, SVDMLP_WORKSPACE_TOO_SMALL, SVDMLP_HIP_ERROR, SVDMLP_NO_DEVICE = -1, -2, -3, -4, -5
SVDMLP_SCRATCH_TOO_SMALL, SVDMLP_OUT_OF_HOST_MEMORY, SVDMLP_TIMED_OUT = -6, -7, -8
FLAG_FORCE_TILED, FLAG_FORCE_STREAM, FLAG_SKIP_ARCH_CHECK, FLAG_STREAM_ONE_KERNEL, FLAG_TILED_FUSED, FLAG_TILE_128 = 1, 2, 4, 8, 16, 32
FLAG_PLAN_ROOM = 64
FIRST_S1, FIRST_IN, OUT_256, OUT_128 = 1, 2, 1, 2

EXPORTS = ["svdmlp_workspace_bytes", "svdmlp_create", "svdmlp_forward", "svdmlp_destroy", "svdmlp_status_string",
           "svdmlp_last_hip_error", "svdmlp_last_path", "svdmlp_abi_version", "svdmlp_profile_begin",
           "svdmlp_profile_end", "svdmlp_profile_kernel_name", "svdmlp_describe", "svdmlp_rank_for_ratio",
           "svdmlp_forward_static_scratch", "svdmlp_static_scratch_bytes",
           "svdmlp_roof_read", "svdmlp_roof_mfma", "svdmlp_roof_mfma_operands", "svdmlp_roof_pingpong", "svdmlp_roof_empty", "svdmlp_roof_empty_chain", "svdmlp_force_plan", "svdmlp_roof_coexec", "svdmlp_check", "svdmlp_debug_set_poll_limit"]


class svdmlp_desc(ctypes.Structure):
    _fields_ = [
        ("kind", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("max_M", ctypes.c_int64), ("d", ctypes.c_int64), ("ffn", ctypes.c_int64), ("r", ctypes.c_int64),
        ("r_down", ctypes.c_int64),
        ("Ug", ctypes.c_void_p), ("Vg", ctypes.c_void_p), ("Uu", ctypes.c_void_p), ("Vu", ctypes.c_void_p),
        ("Ud", ctypes.c_void_p), ("Vd", ctypes.c_void_p),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
        ("flags", ctypes.c_uint32),
    ]


class SvdMlpError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


_lib = None


def lib() -> ctypes.CDLL:
    """Load the built library (raises if it has not been built: ``python -m paper_2510_25977_amd.build``)."""
    global _lib
    if _lib is None:
        if not LIB_PATH.exists():
            raise FileNotFoundError(f"{LIB_PATH} not found: build it with `python -m paper_2510_25977_amd.build`")
        L = ctypes.CDLL(str(LIB_PATH))
        L.svdmlp_workspace_bytes.argtypes = [ctypes.POINTER(svdmlp_desc)]
        L.svdmlp_workspace_bytes.restype = ctypes.c_size_t
        L.svdmlp_create.argtypes = [ctypes.POINTER(svdmlp_desc), ctypes.POINTER(ctypes.c_void_p)]
        L.svdmlp_create.restype = ctypes.c_int
        L.svdmlp_forward.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
        L.svdmlp_forward.restype = ctypes.c_int
        L.svdmlp_forward_static_scratch.argtypes = L.svdmlp_forward.argtypes
        L.svdmlp_forward_static_scratch.restype = ctypes.c_int
        L.svdmlp_static_scratch_bytes.argtypes = []
        L.svdmlp_static_scratch_bytes.restype = ctypes.c_size_t
        L.svdmlp_roof_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
        L.svdmlp_roof_read.restype = ctypes.c_int
        L.svdmlp_roof_mfma.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
        L.svdmlp_roof_mfma.restype = ctypes.c_int
        L.svdmlp_roof_mfma_operands.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
        L.svdmlp_roof_mfma_operands.restype = ctypes.c_int
        L.svdmlp_roof_pingpong.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
        L.svdmlp_roof_pingpong.restype = ctypes.c_int
        L.svdmlp_roof_coexec.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
        L.svdmlp_roof_coexec.restype = ctypes.c_int
        L.svdmlp_roof_empty.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
        L.svdmlp_roof_empty.restype = ctypes.c_int
        L.svdmlp_roof_empty_chain.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
        L.svdmlp_roof_empty_chain.restype = ctypes.c_int
        L.svdmlp_debug_set_poll_limit.argtypes = [ctypes.c_void_p, ctypes.c_int32]
        L.svdmlp_debug_set_poll_limit.restype = ctypes.c_int
        L.svdmlp_check.argtypes = [ctypes.c_void_p]
        L.svdmlp_check.restype = ctypes.c_int
        L.svdmlp_force_plan.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32]
        L.svdmlp_force_plan.restype = ctypes.c_int
        L.svdmlp_destroy.argtypes = [ctypes.c_void_p]
        L.svdmlp_destroy.restype = ctypes.c_int
        L.svdmlp_status_string.argtypes = [ctypes.c_int]
        L.svdmlp_status_string.restype = ctypes.c_char_p
        L.svdmlp_last_hip_error.argtypes = [ctypes.c_void_p]
        L.svdmlp_last_hip_error.restype = ctypes.c_int
        L.svdmlp_last_path.argtypes = [ctypes.c_void_p]
        L.svdmlp_last_path.restype = ctypes.c_int
        L.svdmlp_abi_version.restype = ctypes.c_int
        L.svdmlp_rank_for_ratio.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_double, ctypes.c_int64, ctypes.c_double]
        L.svdmlp_rank_for_ratio.restype = ctypes.c_int64
        L.svdmlp_profile_begin.argtypes = [ctypes.c_void_p, ctypes.c_int]
        L.svdmlp_profile_begin.restype = ctypes.c_int
        L.svdmlp_profile_end.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_int),
                                         ctypes.POINTER(ctypes.c_int)]
        L.svdmlp_profile_end.restype = ctypes.c_int
        L.svdmlp_profile_kernel_name.argtypes = [ctypes.c_void_p, ctypes.c_int]
        L.svdmlp_profile_kernel_name.restype = ctypes.c_char_p
        L.svdmlp_describe.argtypes = [ctypes.POINTER(svdmlp_desc), ctypes.c_int64, ctypes.c_char_p, ctypes.c_size_t]
        L.svdmlp_describe.restype = ctypes.c_int
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().svdmlp_status_string(int(status)).decode()


def svdmlp_workspace_bytes(desc: svdmlp_desc) -> int:
    return int(lib().svdmlp_workspace_bytes(ctypes.byref(desc)))


def svdmlp_rank_for_ratio(k: int, n: int, ratio: float, block: int = 128, alpha: float = 0.5) -> int:
    r = lib().svdmlp_rank_for_ratio(int(k), int(n), float(ratio), int(block), float(alpha))
    if r < 0:
        raise SvdMlpError(SVDMLP_INVALID_ARGUMENT, "svdmlp_rank_for_ratio")
    return int(r)


def svdmlp_describe(desc: svdmlp_desc, M: int) -> str:
    buf = ctypes.create_string_buffer(4096)
    st = lib().svdmlp_describe(ctypes.byref(desc), int(M), buf, len(buf))
    if st != SVDMLP_OK:
        raise SvdMlpError(st, "svdmlp_describe")
    return buf.value.decode()


def svdmlp_create(desc: svdmlp_desc) -> ctypes.c_void_p:
    out = ctypes.c_void_p()
    st = lib().svdmlp_create(ctypes.byref(desc), ctypes.byref(out))
    if st != SVDMLP_OK:
        raise SvdMlpError(st, "svdmlp_create")
    return out


def svdmlp_forward(ctx, X_ptr: int, M: int, Y_ptr: int, stream_ptr: int = 0) -> None:
    st = lib().svdmlp_forward(ctx, ctypes.c_void_p(X_ptr), int(M), ctypes.c_void_p(Y_ptr), ctypes.c_void_p(stream_ptr))
    if st != SVDMLP_OK:
        raise SvdMlpError(st, "svdmlp_forward")


def svdmlp_forward_static_scratch(ctx, X_ptr: int, M: int, Y_ptr: int, stream_ptr: int = 0) -> None:
    st = lib().svdmlp_forward_static_scratch(ctx, ctypes.c_void_p(X_ptr), int(M), ctypes.c_void_p(Y_ptr),
                                             ctypes.c_void_p(stream_ptr))
    if st != SVDMLP_OK:
        raise SvdMlpError(st, "svdmlp_forward_static_scratch")


def svdmlp_static_scratch_bytes() -> int:
    return int(lib().svdmlp_static_scratch_bytes())


def _check(st: int, where: str) -> None:
    if st != SVDMLP_OK:
        raise SvdMlpError(st, where)


def svdmlp_roof_read(buf_ptr: int, nbytes: int, sink_ptr: int, workgroups: int, stream_ptr: int = 0) -> None:
    _check(lib().svdmlp_roof_read(ctypes.c_void_p(buf_ptr), int(nbytes), ctypes.c_void_p(sink_ptr), int(workgroups),
                                  ctypes.c_void_p(stream_ptr)), "svdmlp_roof_read")


def svdmlp_roof_mfma(iters: int, sink_ptr: int, workgroups: int, stream_ptr: int = 0) -> None:
    _check(lib().svdmlp_roof_mfma(int(iters), ctypes.c_void_p(sink_ptr), int(workgroups), ctypes.c_void_p(stream_ptr)),
           "svdmlp_roof_mfma")


ROOF_OPERANDS_ZERO, ROOF_OPERANDS_CONSTANT, ROOF_OPERANDS_RANDOM = 0, 1, 2


def svdmlp_roof_mfma_operands(iters: int, operands: int, sink_ptr: int, workgroups: int, stream_ptr: int = 0) -> None:
    _check(lib().svdmlp_roof_mfma_operands(int(iters), int(operands), ctypes.c_void_p(sink_ptr), int(workgroups),
                                           ctypes.c_void_p(stream_ptr)), "svdmlp_roof_mfma_operands")


def svdmlp_roof_pingpong(steps: int, operands: int, sink_ptr: int, workgroups: int, stream_ptr: int = 0) -> None:
    _check(lib().svdmlp_roof_pingpong(int(steps), int(operands), ctypes.c_void_p(sink_ptr), int(workgroups),
                                      ctypes.c_void_p(stream_ptr)), "svdmlp_roof_pingpong")


def svdmlp_roof_coexec(mfma_iters: int, valu_iters: int, sink_ptr: int, workgroups: int, stream_ptr: int = 0) -> None:
    _check(lib().svdmlp_roof_coexec(int(mfma_iters), int(valu_iters), ctypes.c_void_p(sink_ptr), int(workgroups),
                                    ctypes.c_void_p(stream_ptr)), "svdmlp_roof_coexec")


def svdmlp_roof_empty(workgroups: int, threads: int, stream_ptr: int = 0) -> None:
    _check(lib().svdmlp_roof_empty(int(workgroups), int(threads), ctypes.c_void_p(stream_ptr)), "svdmlp_roof_empty")


def svdmlp_roof_empty_chain(launches: int, workgroups: int, threads: int, stream_ptr: int = 0) -> None:
    _check(lib().svdmlp_roof_empty_chain(int(launches), int(workgroups), int(threads), ctypes.c_void_p(stream_ptr)),
           "svdmlp_roof_empty_chain")


def svdmlp_force_plan(ctx, first_kernel: int = 0, first_ranges: int = 0, down_ranges: int = 0, out_kernel: int = 0) -> None:
    _check(lib().svdmlp_force_plan(ctx, int(first_kernel), int(first_ranges), int(down_ranges), int(out_kernel)),
           "svdmlp_force_plan")


def svdmlp_check(ctx) -> None:
    _check(lib().svdmlp_check(ctx), "svdmlp_check")


def svdmlp_destroy(ctx) -> None:
    lib().svdmlp_destroy(ctx)


def svdmlp_profile_begin(ctx, max_forwards: int) -> None:
    st = lib().svdmlp_profile_begin(ctx, int(max_forwards))
    if st != SVDMLP_OK:
        raise SvdMlpError(st, "svdmlp_profile_begin")


def svdmlp_profile_end(ctx):
    """Returns ({kernel name: average ms}, number of forwards averaged)."""
    ms = (ctypes.c_float * 8)()
    nk, nf = ctypes.c_int(), ctypes.c_int()
    st = lib().svdmlp_profile_end(ctx, ms, ctypes.byref(nk), ctypes.byref(nf))
    if st != SVDMLP_OK:
        raise SvdMlpError(st, "svdmlp_profile_end")
    names = [lib().svdmlp_profile_kernel_name(ctx, k).decode() for k in range(nk.value)]
    return {n: float(ms[k]) for k, n in enumerate(names)}, nf.value


_TORCH_DTYPE = {torch.bfloat16: SVDMLP_BF16, torch.float32: SVDMLP_F32}


class SvdMlp:
    """A context plus the torch tensors that back it (factors and workspace stay referenced here so
    the device memory outlives the context)."""

    def __init__(self, *, max_M: int, Ug: torch.Tensor, Vg: torch.Tensor, Uu: Optional[torch.Tensor] = None,
                 Vu: Optional[torch.Tensor] = None, Ud: Optional[torch.Tensor] = None, Vd: Optional[torch.Tensor] = None,
                 kind: int = SVDMLP_GATED, flags: int = 0, keep_factors: bool = True):
        self.kind = kind
        self.tensors = [t for t in (Ug, Vg, Uu, Vu, Ud, Vd) if t is not None]
        for t in self.tensors:
            if not (t.is_cuda and t.is_contiguous() and t.dtype == Ug.dtype):
                raise ValueError("factors must be contiguous device tensors of one dtype")
        self.dtype = Ug.dtype
        self.d, self.r = Ug.shape
        self.ffn = Vg.shape[1]
        self.r_down = Ud.shape[1] if Ud is not None else 0
        self.max_M = int(max_M)
        de = svdmlp_desc()
        de.kind, de.dtype = kind, _TORCH_DTYPE[self.dtype]
        de.max_M, de.d, de.ffn, de.r, de.r_down = self.max_M, self.d, self.ffn, self.r, self.r_down
        de.Ug, de.Vg = Ug.data_ptr(), Vg.data_ptr()
        for name, t in (("Uu", Uu), ("Vu", Vu), ("Ud", Ud), ("Vd", Vd)):
            setattr(de, name, t.data_ptr() if t is not None else None)
        de.flags = flags
        nbytes = svdmlp_workspace_bytes(de)
        if nbytes == 0:
            # let create report the precise reason
            de.workspace, de.workspace_bytes = None, 0
            svdmlp_create(de)
            raise SvdMlpError(SVDMLP_UNSUPPORTED, "svdmlp_workspace_bytes")
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=Ug.device)
        base = self.workspace.data_ptr()
        de.workspace = (base + 255) // 256 * 256
        de.workspace_bytes = nbytes
        self.workspace_bytes = nbytes
        self.desc = de
        torch.cuda.synchronize(Ug.device)
        self.ctx = svdmlp_create(de)
        if not keep_factors and self.dtype == torch.bfloat16:
            self.tensors = []       # bf16 contexts do not read the factor buffers again after create

    def out_features(self) -> int:
        return self.d if self.kind == SVDMLP_GATED else self.ffn

    def forward(self, X: torch.Tensor, Y: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None):
        if not (X.is_cuda and X.is_contiguous() and X.dtype == self.dtype and X.dim() == 2 and X.shape[1] == self.d):
            raise ValueError("X must be a contiguous [M, d] device tensor of the context's dtype")
        M = X.shape[0]
        if Y is None:
            Y = torch.empty((M, self.out_features()), dtype=self.dtype, device=X.device)
        s = stream if stream is not None else torch.cuda.current_stream(X.device)
        svdmlp_forward(self.ctx, X.data_ptr(), M, Y.data_ptr(), s.cuda_stream)
        return Y

    __call__ = forward

    @property
    def last_path(self) -> int:
        return int(lib().svdmlp_last_path(self.ctx))

    def close(self):
        if getattr(self, "ctx", None):
            svdmlp_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

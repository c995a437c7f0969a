"""ctypes binding of librvq.so: the same entry points as include/rvq.h, argument marshalling only.

PyTorch is used for device memory and streams; every step of the method runs inside the
library's HIP kernels.  Importing this module fails loudly when the library has not been built
(``python -m paper_2410_15704_amd.build``): there is no fallback of any kind.
"""
from __future__ import annotations

import ctypes
import os

# PyTorch comes first: it carries its own HIP runtime, and librvq.so must bind to that copy.  Loaded
# the other way round, the system's runtime is in the process before PyTorch's and PyTorch then
# finds no GPU.
import torch  # noqa: F401

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "librvq.so")

RVQ_OK, RVQ_EINVAL, RVQ_ENOCODEBOOK, RVQ_EHIP, RVQ_ENOMEM = 0, -1, -2, -3, -4
RVQ_EWORKSPACE, RVQ_EKERNEL = -5, -6
DEFAULT_ROWS = 131072
STATIC_MAX_ROWS = 1048576
F32, BF16, F16 = 0, 1, 2
CONTIGUOUS, STRIDED = 0, 1
PATH_AUTO, PATH_EXACT, PATH_SCREEN = 0, 1, 2
DTYPES = {"fp32": F32, "bf16": BF16, "fp16": F16}

EXPORTS = ("rvq_create", "rvq_destroy", "rvq_set_codebooks", "rvq_get_codebooks", "rvq_encode",
           "rvq_decode", "rvq_ema_update", "rvq_strerror", "rvq_last_hip_error", "rvq_version",
           "rvq_get_counters", "rvq_packed_record_bytes", "rvq_pack_codes", "rvq_unpack_codes",
           "rvq_decode_packed", "rvq_decode_rope", "rvq_reserve", "rvq_reserved_rows",
           "rvq_check_kernels", "rvq_debug_set_wait_polls", "rvq_encode_static",
           "rvq_probe_gather_rates", "rvq_attn_decode", "rvq_attn_workspace_bytes")


class rvq_config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "d", "dhat", "depth", "K", "grouping", "scale", "std_ddof", "in_dtype", "out_dtype",
        "std_dtype", "encode_path", "reserved")]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2410_15704_amd.build` "
            "(hipcc, gfx950). There is no fallback path.")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, i32, f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_float
    lib.rvq_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(rvq_config)]
    lib.rvq_destroy.argtypes = [vp]
    lib.rvq_set_codebooks.argtypes = [vp, vp, vp]
    lib.rvq_get_codebooks.argtypes = [vp, vp, vp]
    lib.rvq_encode.argtypes = [vp, vp, i64, i64, i32, i32, vp, vp, vp, vp]
    lib.rvq_encode_static.argtypes = [vp, vp, i64, i64, i32, i32, vp, vp, vp, vp]
    lib.rvq_decode.argtypes = [vp, vp, vp, i64, i32, vp, i64, vp]
    lib.rvq_ema_update.argtypes = [vp, i32, vp, vp, i64, i64, f32, f32, vp, vp, vp]
    lib.rvq_get_counters.argtypes = [vp, ctypes.POINTER(ctypes.c_int64)]
    lib.rvq_packed_record_bytes.argtypes = [vp]
    lib.rvq_packed_record_bytes.restype = ctypes.c_int64
    lib.rvq_pack_codes.argtypes = [vp, vp, i64, vp, vp]
    lib.rvq_unpack_codes.argtypes = [vp, vp, i64, vp, vp]
    lib.rvq_decode_packed.argtypes = [vp, vp, vp, i64, i32, vp, i64, vp]
    lib.rvq_decode_rope.argtypes = [vp, vp, vp, i64, i32, vp, vp, i32, vp, i64, vp]
    lib.rvq_reserve.argtypes = [vp, i64]
    lib.rvq_reserved_rows.argtypes = [vp]
    lib.rvq_reserved_rows.restype = ctypes.c_int64
    lib.rvq_check_kernels.argtypes = [vp]
    lib.rvq_debug_set_wait_polls.argtypes = [vp, i64]
    lib.rvq_probe_gather_rates.argtypes = [ctypes.POINTER(ctypes.c_double)]
    lib.rvq_strerror.argtypes = [ctypes.c_int]
    lib.rvq_strerror.restype = ctypes.c_char_p
    lib.rvq_last_hip_error.argtypes = [vp]
    lib.rvq_version.restype = ctypes.c_int
    lib.rvq_attn_workspace_bytes.argtypes = [i64, i32, i32]
    lib.rvq_attn_workspace_bytes.restype = i64
    lib.rvq_attn_decode.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp, vp, i32, i64, vp, vp, f32, vp, vp, i64, vp]
    for name in EXPORTS:
        getattr(lib, name)
        if name not in ("rvq_strerror", "rvq_version", "rvq_packed_record_bytes",
                        "rvq_reserved_rows", "rvq_attn_workspace_bytes"):
            getattr(lib, name).restype = ctypes.c_int
    return lib


lib = _load()


class RvqError(RuntimeError):
    def __init__(self, code, ctx=None):
        self.code = code
        msg = lib.rvq_strerror(code).decode()
        if code == RVQ_EHIP and ctx:
            msg += f" (hipError {lib.rvq_last_hip_error(ctx)})"
        super().__init__(f"librvq: {msg} [{code}]")


def _ptr(t):
    """Device pointer of a torch tensor (or None / int passthrough)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


# ---- the entry points, same names as the header -----------------------------------------------
def rvq_version() -> int:
    return lib.rvq_version()


def rvq_strerror(code: int) -> str:
    return lib.rvq_strerror(code).decode()


def rvq_create(*, d, dhat=32, depth=8, K=2048, grouping=CONTIGUOUS, scale=1, std_ddof=0,
               in_dtype=F32, out_dtype=F16, std_dtype=F16, encode_path=PATH_AUTO, check=True):
    cfg = rvq_config(d, dhat, depth, K, grouping, scale, std_ddof, in_dtype, out_dtype, std_dtype,
                     encode_path, 0)
    ctx = ctypes.c_void_p()
    rc = lib.rvq_create(ctypes.byref(ctx), ctypes.byref(cfg))
    if rc != RVQ_OK:
        if check:
            raise RvqError(rc)
        return rc
    return ctx


def rvq_destroy(ctx):
    return lib.rvq_destroy(ctx)


def _chk(rc, ctx):
    if rc != RVQ_OK:
        raise RvqError(rc, ctx)
    return rc


def rvq_reserve(ctx, max_rows):
    return _chk(lib.rvq_reserve(ctx, max_rows), ctx)


def rvq_reserved_rows(ctx) -> int:
    return int(lib.rvq_reserved_rows(ctx))


def rvq_check_kernels(ctx, check=True):
    rc = lib.rvq_check_kernels(ctx)
    return _chk(rc, ctx) if check else rc


def rvq_debug_set_wait_polls(ctx, polls):
    return _chk(lib.rvq_debug_set_wait_polls(ctx, polls), ctx)


def rvq_probe_gather_rates():
    out = (ctypes.c_double * 3)()
    _chk(lib.rvq_probe_gather_rates(out), None)
    return dict(lds_random_GBs=out[0], lds_consecutive_GBs=out[1], l2_rows_random_GBs=out[2])


def rvq_set_codebooks(ctx, dC, stream=None):
    return _chk(lib.rvq_set_codebooks(ctx, _ptr(dC), _stream(stream)), ctx)


def rvq_get_codebooks(ctx, dC, stream=None):
    return _chk(lib.rvq_get_codebooks(ctx, _ptr(dC), _stream(stream)), ctx)


def rvq_encode(ctx, dX, N, ldx, stage_begin, stage_end, dCodes, dStd, dResidual=None, stream=None):
    return _chk(lib.rvq_encode(ctx, _ptr(dX), N, ldx, stage_begin, stage_end, _ptr(dCodes),
                               _ptr(dStd), _ptr(dResidual), _stream(stream)), ctx)


def rvq_encode_static(ctx, dX, N, ldx, stage_begin, stage_end, dCodes, dStd, dResidual=None,
                      stream=None):
    return _chk(lib.rvq_encode_static(ctx, _ptr(dX), N, ldx, stage_begin, stage_end, _ptr(dCodes),
                                      _ptr(dStd), _ptr(dResidual), _stream(stream)), ctx)


def rvq_decode(ctx, dCodes, dStd, N, depth_used, dOut, ldo, stream=None):
    return _chk(lib.rvq_decode(ctx, _ptr(dCodes), _ptr(dStd), N, depth_used, _ptr(dOut), ldo,
                               _stream(stream)), ctx)


def rvq_ema_update(ctx, stage, dR, dCodes, code_stride, M, decay, eps, dClusterSize, dEmbedSum,
                   stream=None):
    return _chk(lib.rvq_ema_update(ctx, stage, _ptr(dR), _ptr(dCodes), code_stride, M, decay, eps,
                                   _ptr(dClusterSize), _ptr(dEmbedSum), _stream(stream)), ctx)


def rvq_packed_record_bytes(ctx) -> int:
    return int(lib.rvq_packed_record_bytes(ctx))


def rvq_pack_codes(ctx, dCodes, N, dPacked, stream=None):
    return _chk(lib.rvq_pack_codes(ctx, _ptr(dCodes), N, _ptr(dPacked), _stream(stream)), ctx)


def rvq_unpack_codes(ctx, dPacked, N, dCodes, stream=None):
    return _chk(lib.rvq_unpack_codes(ctx, _ptr(dPacked), N, _ptr(dCodes), _stream(stream)), ctx)


def rvq_decode_packed(ctx, dPacked, dStd, N, depth_used, dOut, ldo, stream=None):
    return _chk(lib.rvq_decode_packed(ctx, _ptr(dPacked), _ptr(dStd), N, depth_used, _ptr(dOut),
                                      ldo, _stream(stream)), ctx)


def rvq_decode_rope(ctx, dCodes, dStd, N, depth_used, dCos, dSin, head_dim, dOut, ldo, stream=None):
    return _chk(lib.rvq_decode_rope(ctx, _ptr(dCodes), _ptr(dStd), N, depth_used, _ptr(dCos),
                                    _ptr(dSin), head_dim, _ptr(dOut), ldo, _stream(stream)), ctx)


def rvq_attn_workspace_bytes(N, n_q_heads, n_kv_heads):
    return int(lib.rvq_attn_workspace_bytes(N, n_q_heads, n_kv_heads))


def rvq_attn_decode(kctx, vctx, dQ, n_q_heads, n_kv_heads, dKCodes, dKStd, dVCodes, dVStd, N, dCos,
                    dSin, scale, dOut, dWorkspace, workspace_bytes, stream=None, packed=0):
    return _chk(lib.rvq_attn_decode(kctx, vctx, _ptr(dQ), n_q_heads, n_kv_heads, _ptr(dKCodes),
                                    _ptr(dKStd), _ptr(dVCodes), _ptr(dVStd), packed, N, _ptr(dCos),
                                    _ptr(dSin), scale, _ptr(dOut), _ptr(dWorkspace), workspace_bytes,
                                    _stream(stream)), kctx)


def rvq_get_counters(ctx):
    out = (ctypes.c_int64 * 16)()  # debug builds report more
    _chk(lib.rvq_get_counters(ctx, out), ctx)
    return dict(zip(("slow_searches", "exact_rescored", "groups_rescored", "searches",
                     "group_exact_passes"), list(out)))


class Quantizer:
    """Owns one rvq_ctx; thin convenience over the entry points above (allocation of outputs and
    shape bookkeeping only)."""

    def __init__(self, **cfg):
        self.cfg = dict(d=None, dhat=32, depth=8, K=2048, grouping=CONTIGUOUS, scale=1, std_ddof=0,
                        in_dtype=F32, out_dtype=F16, std_dtype=F16, encode_path=PATH_AUTO)
        self.cfg.update(cfg)
        self.ctx = rvq_create(**self.cfg)
        self.G = self.cfg["d"] // self.cfg["dhat"]

    def close(self):
        if self.ctx is not None:
            rvq_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_codebooks(self, C):
        import torch
        assert C.dtype == torch.float32 and C.is_cuda and C.is_contiguous()
        assert tuple(C.shape) == (self.cfg["depth"], self.cfg["K"], self.cfg["dhat"])
        rvq_set_codebooks(self.ctx, C)

    def get_codebooks(self):
        import torch
        C = torch.empty((self.cfg["depth"], self.cfg["K"], self.cfg["dhat"]), dtype=torch.float32,
                        device="cuda")
        rvq_get_codebooks(self.ctx, C)
        return C

    def _std_torch_dtype(self):
        import torch
        return torch.float16 if self.cfg["std_dtype"] == F16 else torch.float32

    def encode(self, X, want_residual=False, stages=None, codes=None):
        import torch
        N = X.shape[0]
        depth = self.cfg["depth"]
        sb, se = stages if stages is not None else (0, depth)
        if codes is None:
            codes = torch.empty((N, self.G, depth), dtype=torch.int16, device=X.device)
        std = (torch.empty((N,), dtype=self._std_torch_dtype(), device=X.device)
               if self.cfg["scale"] else None)
        res = (torch.empty((N, self.G, self.cfg["dhat"]), dtype=torch.float32, device=X.device)
               if want_residual else None)
        if N > rvq_reserved_rows(self.ctx):
            rvq_reserve(self.ctx, N)  # set-up call: grows the context's workspace
        rvq_encode(self.ctx, X, N, X.stride(0) if N else self.cfg["d"], sb, se, codes, std, res)
        return codes, std, res

    def decode(self, codes, std, depth_used=None, out=None):
        import torch
        N = codes.shape[0]
        if out is None:
            dt = torch.float16 if self.cfg["out_dtype"] == F16 else torch.float32
            out = torch.empty((N, self.cfg["d"]), dtype=dt, device=codes.device)
        rvq_decode(self.ctx, codes, std, N, depth_used or self.cfg["depth"], out,
                   out.stride(0) if N else self.cfg["d"])
        return out

    def decode_rope(self, codes, std, cos, sin, head_dim, depth_used=None, out=None):
        import torch
        N = codes.shape[0]
        if out is None:
            dt = torch.float16 if self.cfg["out_dtype"] == F16 else torch.float32
            out = torch.empty((N, self.cfg["d"]), dtype=dt, device=codes.device)
        rvq_decode_rope(self.ctx, codes, std, N, depth_used or self.cfg["depth"], cos, sin, head_dim,
                        out, out.stride(0) if N else self.cfg["d"])
        return out

    def pack(self, codes):
        import torch
        N = codes.shape[0]
        rec = rvq_packed_record_bytes(self.ctx)
        packed = torch.empty((N, self.G, rec), dtype=torch.uint8, device=codes.device)
        rvq_pack_codes(self.ctx, codes, N, packed)
        return packed

    def unpack(self, packed):
        import torch
        N = packed.shape[0]
        codes = torch.empty((N, self.G, self.cfg["depth"]), dtype=torch.int16, device=packed.device)
        rvq_unpack_codes(self.ctx, packed, N, codes)
        return codes

    def decode_packed(self, packed, std, depth_used=None, out=None):
        import torch
        N = packed.shape[0]
        if out is None:
            dt = torch.float16 if self.cfg["out_dtype"] == F16 else torch.float32
            out = torch.empty((N, self.cfg["d"]), dtype=dt, device=packed.device)
        rvq_decode_packed(self.ctx, packed, std, N, depth_used or self.cfg["depth"], out,
                          out.stride(0) if N else self.cfg["d"])
        return out

    def ema_update(self, stage, R, codes, cluster_size, embed_sum, decay=0.99, eps=1e-5,
                   code_stride=1):
        rvq_ema_update(self.ctx, stage, R, codes, code_stride, R.shape[0], decay, eps,
                       cluster_size, embed_sum)

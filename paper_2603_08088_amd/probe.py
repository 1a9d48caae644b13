"""Binding of libeagletv_probe.so (``include/eagletv_probe.h``): measurement aids, no part of the verification step."""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libeagletv_probe.so")
EXPORTS = ("etvp_hbm_read_probe", "etvp_mfma_bf16_probe_flops", "etvp_mfma_bf16_probe",
           "etvp_mfma_bf16_live_probe_flops", "etvp_mfma_bf16_live_probe")
_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2603_08088_amd.build`")
        l = C.CDLL(LIB_PATH)
        l.etvp_hbm_read_probe.restype = C.c_int32
        l.etvp_hbm_read_probe.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        l.etvp_mfma_bf16_probe_flops.restype = C.c_double
        l.etvp_mfma_bf16_probe_flops.argtypes = [C.c_int32]
        l.etvp_mfma_bf16_probe.restype = C.c_int32
        l.etvp_mfma_bf16_probe.argtypes = [C.c_int32, C.c_void_p, C.c_void_p]
        l.etvp_mfma_bf16_live_probe_flops.restype = C.c_double
        l.etvp_mfma_bf16_live_probe_flops.argtypes = [C.c_int32]
        l.etvp_mfma_bf16_live_probe.restype = C.c_int32
        l.etvp_mfma_bf16_live_probe.argtypes = [C.c_int32, C.c_void_p, C.c_void_p]
        _lib = l
    return _lib


def _stream():
    return torch.cuda.current_stream().cuda_stream


def hbm_read_probe(buf: torch.Tensor, sink: torch.Tensor) -> None:
    """Stream `buf` (any dtype, >= 1 MiB) once through nontemporal loads; `sink` is a 16-byte device tensor."""
    rc = lib().etvp_hbm_read_probe(buf.data_ptr(), buf.numel() * buf.element_size(), sink.data_ptr(), _stream())
    if rc != 0:
        raise RuntimeError(f"etvp_hbm_read_probe: rc={rc}")


def mfma_bf16_probe_flops(iters: int) -> float:
    return float(lib().etvp_mfma_bf16_probe_flops(int(iters)))


def mfma_bf16_probe(iters: int, sink: torch.Tensor) -> None:
    rc = lib().etvp_mfma_bf16_probe(int(iters), sink.data_ptr(), _stream())
    if rc != 0:
        raise RuntimeError(f"etvp_mfma_bf16_probe: rc={rc}")


def mfma_bf16_live_probe_flops(tiles: int) -> float:
    return float(lib().etvp_mfma_bf16_live_probe_flops(int(tiles)))


def mfma_bf16_live_probe(tiles: int, sink: torch.Tensor) -> None:
    rc = lib().etvp_mfma_bf16_live_probe(int(tiles), sink.data_ptr(), _stream())
    if rc != 0:
        raise RuntimeError(f"etvp_mfma_bf16_live_probe: rc={rc}")

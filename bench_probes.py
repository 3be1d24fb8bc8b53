"""Loader for the ceiling probes bench.py reports beside its figures (bench_probes.hip): a plain
HBM read kernel and a register-only matrix-core stream.  Measurement aids only; nothing in the
attention library or its tests depends on them."""
from __future__ import annotations

import ctypes as C
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(_HERE, "bench_probes.hip")
LIB = os.path.join(_HERE, "libbench_probes.so")
_lib = None


def build() -> str:
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Xclang",
                           "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
                           SRC, "-o", LIB])
    return LIB


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            raise RuntimeError(f"{LIB} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
        _lib = C.CDLL(LIB)
    return _lib


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def hbm_read(bufs, nbytes: int, reps: int, wgs_per_cu: int = 8, threads: int = 256, in_flight: int = 4,
             contiguous: bool = False, nontemporal: bool = False) -> float:
    """GB/s of `reps` back-to-back launches of a kernel that only reads, launch i over bufs[i % len(bufs)]
    (device tensors of at least nbytes bytes)."""
    ptrs = (C.c_void_p * len(bufs))(*[b.data_ptr() for b in bufs])
    gbps = C.c_float(0)
    rc = lib().probe_hbm_read(ptrs, C.c_int(len(bufs)), C.c_size_t(nbytes), C.c_int(reps), C.c_int(wgs_per_cu),
                              C.c_int(threads), C.c_int(in_flight), C.c_int(int(contiguous)), C.c_int(int(nontemporal)),
                              C.byref(gbps), _stream())
    if rc:
        raise RuntimeError(f"probe_hbm_read failed: hipError {rc}")
    return float(gbps.value)


def hbm_paged_read(bufs, order, block_bytes: int, reps: int, wgs_per_cu: int = 2, threads: int = 256, depth: int = 1,
                   nontemporal: bool = False) -> float:
    """GB/s of a kernel that reads every buffer as blocks of block_bytes (2048 or 4096) in the order of the
    device int32 tensor `order` (a permutation of the block numbers), one block per wavefront at a time."""
    ptrs = (C.c_void_p * len(bufs))(*[b.data_ptr() for b in bufs])
    gbps = C.c_float(0)
    rc = lib().probe_hbm_paged_read(ptrs, C.c_int(len(bufs)), C.c_void_p(order.data_ptr()), C.c_int(order.numel()),
                                    C.c_int(block_bytes), C.c_int(reps), C.c_int(wgs_per_cu), C.c_int(threads),
                                    C.c_int(depth), C.c_int(int(nontemporal)), C.byref(gbps), _stream())
    if rc:
        raise RuntimeError(f"probe_hbm_paged_read failed: hipError {rc}")
    return float(gbps.value)


def mfma_bf16(iters: int, random_operands: bool, waves_per_simd: int = 2):
    """(dense bf16 TFLOP/s, core clock in GHz) of a register-only matrix-instruction stream on every CU."""
    tf, ghz = C.c_float(0), C.c_float(0)
    rc = lib().probe_mfma_bf16(C.c_int(iters), C.c_int(int(random_operands)), C.c_int(waves_per_simd), C.byref(tf),
                               C.byref(ghz), _stream())
    if rc:
        raise RuntimeError(f"probe_mfma_bf16 failed: hipError {rc}")
    return float(tf.value), float(ghz.value)

"""Loader of ``libbenchprobe.so``: the benchmark's measurement kernels (a streaming read, a plain copy, a 3:1 read/write mix).

They are no part of the method and live outside the product library; ``bench.py`` times them next to the library's own
kernels and uses the copy to calibrate hardware byte counters.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libbenchprobe.so")
_lib: Optional[ctypes.CDLL] = None


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB_PATH + ".tmp.%d" % os.getpid()
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
           "-I", HERE, "-o", tmp, os.path.join(HERE, "benchprobe.hip")]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stdout)
    os.replace(tmp, LIB_PATH)
    return LIB_PATH


def load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError("%s is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')" % LIB_PATH)
        lib = ctypes.CDLL(LIB_PATH)
        vp, sz = ctypes.c_void_p, ctypes.c_size_t
        lib.benchprobe_read.argtypes = [vp, sz, vp, vp]
        lib.benchprobe_copy.argtypes = [vp, vp, sz, vp]
        lib.benchprobe_mix3.argtypes = [vp, vp, sz, vp]
        _lib = lib
    return _lib


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def read(src: torch.Tensor, sink: torch.Tensor) -> None:
    rc = load().benchprobe_read(src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr(), _stream())
    if rc:
        raise RuntimeError("benchprobe_read failed (%d)" % rc)


def copy(dst: torch.Tensor, src: torch.Tensor) -> None:
    rc = load().benchprobe_copy(dst.data_ptr(), src.data_ptr(), src.numel() * src.element_size(), _stream())
    if rc:
        raise RuntimeError("benchprobe_copy failed (%d)" % rc)


def mix3(dst: torch.Tensor, src: torch.Tensor) -> None:
    """dst = a ^ b ^ c, the three sources back to back in src (three times dst's size)"""
    nbytes = dst.numel() * dst.element_size()
    if src.numel() * src.element_size() < 3 * nbytes:
        raise ValueError("src must hold three times dst's bytes")
    rc = load().benchprobe_mix3(dst.data_ptr(), src.data_ptr(), nbytes, _stream())
    if rc:
        raise RuntimeError("benchprobe_mix3 failed (%d)" % rc)

"""Device-side filler for synthetic tables too large to upload (binding of libsynthfill.so).

Implements the same SplitMix64 streams as `synthetic.py`; a GPU test compares
the two element by element.  Input generation only.
"""
from __future__ import annotations

import ctypes
import os

import torch

from . import synthetic as syn

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsynthfill.so")
_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2302_08141_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        L.synth_fill_uniform.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32,
                                         ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64,
                                         ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p]
        L.synth_fill_uniform.restype = ctypes.c_int
        L.synth_stream_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32,
                                        ctypes.c_void_p]
        L.synth_stream_read.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int32,
                                        ctypes.c_void_p]
        L.synth_stream_write.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_uint64, ctypes.c_int32,
                                         ctypes.c_void_p]
        L.synth_stream_write.restype = ctypes.c_int
        L.synth_stream_read_wide.argtypes = L.synth_stream_read.argtypes
        L.synth_stream_read_slices.argtypes = L.synth_stream_read.argtypes
        L.synth_stream_read_slices.restype = ctypes.c_int
        L.synth_stream_copy.restype = L.synth_stream_read.restype = L.synth_stream_read_wide.restype = ctypes.c_int
        _lib = L
    return _lib


def fill_uniform(dst: torch.Tensor, first_problem: int, tag: int, rng: int, lo: int = 0, diag_k: int = 0,
                 seed: int = syn.BASE_SEED) -> None:
    """dst int64[n_problems][...]: problem p of the batch gets stream (seed, first_problem+p, tag)."""
    assert dst.is_cuda and dst.dtype == torch.int64 and dst.is_contiguous() and dst.dim() >= 2
    n = dst.shape[0]
    count = dst[0].numel()
    rc = lib().synth_fill_uniform(ctypes.c_void_p(dst.data_ptr()), count, count, n, seed, first_problem, tag, rng,
                                  lo, diag_k, ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    if rc != 0:
        raise RuntimeError(f"synth_fill_uniform rc={rc}")


def fill_random_chain(c: torch.Tensor, R: torch.Tensor, first_problem: int, c_range: int, r_range: int,
                      seed: int = syn.BASE_SEED, c_lo: int = 0) -> None:
    """c[B][N][K], R[B][N-1][K][K] with K unpadded: the device twin of synthetic.random_chain_batch."""
    K = c.shape[-1]
    fill_uniform(c, first_problem, syn.TAG_NODE, c_range, c_lo, 0, seed)
    if R.numel():
        fill_uniform(R, first_problem, syn.TAG_EDGE, r_range, 0, K, seed)


def stream_copy(dst: torch.Tensor, src: torch.Tensor, blocks: int = 8192) -> None:
    """Plain 16-byte-per-lane copy kernel of known size (yardstick for bandwidth and byte counters)."""
    assert dst.is_cuda and src.is_cuda and dst.is_contiguous() and src.is_contiguous()
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() >= nbytes and nbytes % 16 == 0
    rc = lib().synth_stream_copy(ctypes.c_void_p(dst.data_ptr()), ctypes.c_void_p(src.data_ptr()), nbytes, blocks,
                                 ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    if rc != 0:
        raise RuntimeError(f"synth_stream_copy rc={rc}")


def stream_read(src: torch.Tensor, sink: torch.Tensor, blocks: int = 8192, wide: bool = False,
                slices: bool = False) -> None:
    """Plain read-only streaming kernel over src (yardstick for the achievable HBM read rate).
    wide: 1024-thread workgroups on contiguous 256 KiB chunks with 16 loads per lane in flight, chunks dealt
    round-robin; slices: the same workgroups, each walking its own contiguous range of chunks."""
    assert src.is_cuda and src.is_contiguous() and sink.is_cuda and sink.dtype == torch.int64 and sink.numel() >= 1
    nbytes = src.numel() * src.element_size()
    assert nbytes % (262144 if (wide or slices) else 16) == 0
    fn = lib().synth_stream_read_slices if slices else lib().synth_stream_read_wide if wide else lib().synth_stream_read
    rc = fn(ctypes.c_void_p(src.data_ptr()), nbytes, ctypes.c_void_p(sink.data_ptr()), blocks,
            ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    if rc != 0:
        raise RuntimeError(f"stream_read rc={rc}")


def stream_write(dst: torch.Tensor, value: int = 0, blocks: int = 8192) -> None:
    """Plain write-only streaming kernel over dst (yardstick for the achievable HBM write rate)."""
    assert dst.is_cuda and dst.is_contiguous()
    nbytes = dst.numel() * dst.element_size()
    assert nbytes % 16 == 0
    rc = lib().synth_stream_write(ctypes.c_void_p(dst.data_ptr()), nbytes, value, blocks,
                                  ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    if rc != 0:
        raise RuntimeError(f"synth_stream_write rc={rc}")

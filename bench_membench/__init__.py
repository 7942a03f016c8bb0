"""Streaming kernels without arithmetic (``membench.hip`` -> ``libnpd_membench.so``) and their ctypes front-end, used by
``bench.py --op membench`` to measure what the memory system gives the access mixes of the KD kernels.  A measurement
aid beside the benchmark: not part of the loss path, not part of the ``paper_2605_05940_amd`` package, not linked into
``libnpd.so``."""
import ctypes
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libnpd_membench.so")
SRC_PATH = os.path.join(HERE, "membench.hip")


def build(verbose: bool = False) -> str:
    """Compile ``membench.hip`` for gfx950 into ``libnpd_membench.so`` (cross-compiles without a GPU)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "-O3", "-std=c++17", "-fPIC", "-shared", "--offload-arch=gfx950", "-Xclang", "-target-feature",
           "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-command-line-argument", SRC_PATH, "-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB_PATH

PATTERNS = ("read_1", "read_2", "write_1", "copy_1r_1w", "read_2_write_1", "row_read_2_then_write_1")
ROW_GROUPS_PER_THREAD = 19   # row_read_2_then_write_1 holds a row in registers: at most this many groups per thread
# arrays moved per pass: (reads, writes)
MOVES = {"read_1": (1, 0), "read_2": (2, 0), "write_1": (0, 1), "copy_1r_1w": (1, 1), "read_2_write_1": (2, 1),
         "row_read_2_then_write_1": (2, 1)}

_lib = None


def load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            build()
        lib = ctypes.CDLL(LIB_PATH)
        lib.npd_membench_patterns.restype = ctypes.c_int
        lib.npd_membench_run.restype = ctypes.c_int
        lib.npd_membench_run.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                         ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p]
        lib.npd_membench_gang_scratch_bytes.restype = ctypes.c_size_t
        lib.npd_membench_gang_scratch_bytes.argtypes = [ctypes.c_int64, ctypes.c_int32]
        lib.npd_membench_gang.restype = ctypes.c_int
        lib.npd_membench_gang.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32,
                                          ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p]
        assert lib.npd_membench_patterns() == len(PATTERNS)
        _lib = lib
    return _lib


ORDERS = ("rows", "address")   # one workgroup per row | one short-lived workgroup per `threads` consecutive groups


def run(pattern: str, threads: int, nontemporal: bool, a, b, o, rows: int, row_groups: int,
        order: str = "rows") -> None:
    """One pass over device tensors ``a``, ``b``, ``o`` (each rows * row_groups * 16 bytes) on torch's current stream."""
    import torch
    for x in (a, b, o):
        if not x.is_cuda or not x.is_contiguous() or x.numel() * x.element_size() < rows * row_groups * 16:
            raise ValueError("membench arrays must be contiguous device tensors of rows * row_groups * 16 bytes")
    rc = load().npd_membench_run(PATTERNS.index(pattern), ORDERS.index(order), threads, int(nontemporal), a.data_ptr(), b.data_ptr(),
                                 o.data_ptr(), rows, row_groups, torch.cuda.current_stream().cuda_stream)
    if rc != 0:
        raise RuntimeError(f"npd_membench_run failed with HIP error {rc}")


def gang_scratch_bytes(rows: int, row_groups: int) -> int:
    return int(load().npd_membench_gang_scratch_bytes(rows, row_groups))


def run_gang(a, b, o, scratch, rows: int, row_groups: int, reads: int = 2) -> None:
    """One pass of the row-gang pattern (``reads`` = 2: two reads + one write, 1: one read + one write; rows shared by
    workgroups of 256 threads that read their slices, exchange through ``scratch`` and then write) on torch's current
    stream."""
    import torch
    for x in (a, b, o):
        if not x.is_cuda or not x.is_contiguous() or x.numel() * x.element_size() < rows * row_groups * 16:
            raise ValueError("membench arrays must be contiguous device tensors of rows * row_groups * 16 bytes")
    need = gang_scratch_bytes(rows, row_groups)
    if need == 0 or not scratch.is_cuda or scratch.numel() * scratch.element_size() < need:
        raise ValueError("scratch too small or shape not supported")
    rc = load().npd_membench_gang(a.data_ptr(), b.data_ptr(), o.data_ptr(), rows, row_groups, scratch.data_ptr(), reads,
                                  torch.cuda.current_stream().cuda_stream)
    if rc != 0:
        raise RuntimeError(f"npd_membench_gang failed with HIP error {rc}")

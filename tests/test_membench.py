"""The arithmetic-free streaming kernels behind ``bench.py --op membench`` (a measurement aid, not the loss path):
the library loads and rejects bad arguments on the host; on the GPU every pattern moves exactly what it says."""
import ctypes

import pytest
import torch

import bench_membench as membench

HIP_INVALID_VALUE = 1
FAKE = 0x10000


def test_membench_library_loads_and_validates_on_the_host():
    lib = membench.load()
    assert lib.npd_membench_patterns() == len(membench.PATTERNS) == len(membench.MOVES)
    ok = dict(pattern=4, order=0, threads=1024, nt=1, a=FAKE, b=FAKE + 0x1000, o=FAKE + 0x2000, rows=4, groups=8)

    def call(**kw):
        p = dict(ok, **kw)
        return lib.npd_membench_run(p["pattern"], p["order"], p["threads"], p["nt"], p["a"], p["b"], p["o"], p["rows"],
                                    p["groups"], None)
    # every call below is refused before anything is enqueued (the addresses are never touched)
    assert call(a=None) == HIP_INVALID_VALUE and call(o=None) == HIP_INVALID_VALUE
    assert call(rows=0) == HIP_INVALID_VALUE and call(groups=0) == HIP_INVALID_VALUE
    assert call(rows=2**31) == HIP_INVALID_VALUE
    assert call(a=FAKE + 4) == HIP_INVALID_VALUE               # not 16-byte aligned
    assert call(threads=128) == HIP_INVALID_VALUE and call(pattern=6) == HIP_INVALID_VALUE
    assert call(pattern=5, threads=256, groups=19 * 256 + 1) == HIP_INVALID_VALUE   # row larger than the registers
    assert call(order=2) == HIP_INVALID_VALUE and call(pattern=5, order=1) == HIP_INVALID_VALUE


@pytest.mark.gpu
@pytest.mark.parametrize("threads", [256, 512, 1024])
@pytest.mark.parametrize("nt", [False, True])
def test_membench_patterns_move_what_they_say(threads, nt):
    dev = torch.device("cuda:0")
    rows, groups = 7, 4 * threads + 37          # a ragged tail after one full round of 4 requests per thread
    n = rows * groups * 16
    gen = torch.Generator(device="cpu").manual_seed(5)
    a = torch.randint(0, 256, (n,), dtype=torch.uint8, generator=gen).to(dev)
    b = torch.randint(0, 256, (n,), dtype=torch.uint8, generator=gen).to(dev)
    guard = 4096
    full = torch.full((n + 2 * guard,), 0xA5, dtype=torch.uint8, device=dev)
    o = full[guard:guard + n]
    assert o.data_ptr() % 16 == 0
    expect = {"read_1": torch.full_like(a, 0xA5), "read_2": torch.full_like(a, 0xA5), "write_1": torch.zeros_like(a),
              "copy_1r_1w": a, "read_2_write_1": a ^ b, "row_read_2_then_write_1": a ^ b}
    for name in membench.PATTERNS:
        for order in membench.ORDERS:
            if order == "address" and name == "row_read_2_then_write_1":
                continue
            full.fill_(0xA5)
            membench.run(name, threads, nt, a, b, o, rows, groups, order=order)
            torch.cuda.synchronize()
            assert torch.equal(o, expect[name]), (name, order)
            assert (full[:guard] == 0xA5).all() and (full[guard + n:] == 0xA5).all(), (name, order)


def test_membench_gang_validates_on_the_host():
    lib = membench.load()
    assert membench.gang_scratch_bytes(32768, 18992) == 32768 * 8 * 32      # 8 slices of at most 2,560 groups
    assert membench.gang_scratch_bytes(4, 33 * 2560) == 0                   # more than 32 slices per row
    assert membench.gang_scratch_bytes(0, 100) == 0
    assert lib.npd_membench_gang(FAKE, FAKE + 0x1000, FAKE + 0x2000, 4, 100, None, 2, None) == HIP_INVALID_VALUE
    assert lib.npd_membench_gang(FAKE, FAKE + 0x1000, FAKE + 0x2004, 4, 100, FAKE + 0x3000, 2, None) == HIP_INVALID_VALUE
    assert lib.npd_membench_gang(None, FAKE + 0x1000, FAKE + 0x2000, 4, 100, FAKE + 0x3000, 1, None) == HIP_INVALID_VALUE
    assert lib.npd_membench_gang(FAKE, FAKE + 0x1000, FAKE + 0x2000, 4, 100, FAKE + 0x3000, 3, None) == HIP_INVALID_VALUE


@pytest.mark.gpu
@pytest.mark.parametrize("groups", [2560 + 37, 3 * 2560, 1000])
def test_membench_gang_moves_what_it_says(groups):
    dev = torch.device("cuda:0")
    rows = 9
    n = rows * groups * 16
    gen = torch.Generator(device="cpu").manual_seed(6)
    a = torch.randint(0, 256, (n,), dtype=torch.uint8, generator=gen).to(dev)
    b = torch.randint(0, 256, (n,), dtype=torch.uint8, generator=gen).to(dev)
    guard = 4096
    full = torch.full((n + 2 * guard,), 0xA5, dtype=torch.uint8, device=dev)
    o = full[guard:guard + n]
    scratch = torch.zeros(membench.gang_scratch_bytes(rows, groups), dtype=torch.uint8, device=dev)
    for reads in (2, 2, 1):                  # the second pass finds the first one's words in the record
        full.fill_(0xA5)
        membench.run_gang(a, b, o, scratch, rows, groups, reads=reads)
        torch.cuda.synchronize()
        assert torch.equal(o, a ^ b if reads == 2 else a)
        assert (full[:guard] == 0xA5).all() and (full[guard + n:] == 0xA5).all()

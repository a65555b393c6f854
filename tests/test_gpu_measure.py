"""The measurement aids move the bytes they say they move: the plain copy that scales the
hardware counters and the shaped streams that serve as bandwidth yardsticks."""
import pytest
import torch

from paper_2605_05696_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need an MI355X; deselect with -m 'not gpu'"


def pair(n):
    g = torch.Generator(device=DEV).manual_seed(1234)
    src = torch.randint(0, 256, (n,), dtype=torch.uint8, device=DEV, generator=g)
    return src, torch.zeros(n, dtype=torch.uint8, device=DEV)


def test_calibrate_copy_copies():
    src, dst = pair((40 << 20) + 4096 * 16)              # main loop and tail loop both run
    B.irm_calibrate_copy(dst, src, 0, None)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)


@pytest.mark.parametrize("xcd", [0, B.YARDSTICK_XCD_RANGES])
@pytest.mark.parametrize("grid,lanes,vec", [(64, 256, 4), (8, 1024, 2), (48, 512, 9), (16, 256, 36), (1024, 512, 2)])
def test_yardstick_copy_copies_every_byte(grid, lanes, vec, xcd):
    steps = 3 if grid < 1024 else 1                      # one step per workgroup: the address-ordered shape
    src, dst = pair(grid * lanes * vec * 16 * steps)
    B.irm_yardstick(dst, src, B.YARDSTICK_COPY | xcd, grid, lanes, vec, None)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)


@pytest.mark.parametrize("xcd", [0, B.YARDSTICK_XCD_RANGES])
def test_yardstick_read_leaves_the_destination_alone_and_write_fills_it(xcd):
    grid, lanes, vec = 32, 256, 4
    src, dst = pair(grid * lanes * vec * 16 * 2)
    B.irm_yardstick(dst, src, B.YARDSTICK_READ | xcd, grid, lanes, vec, None)
    torch.cuda.synchronize()
    assert int(dst.count_nonzero()) == 0
    B.irm_yardstick(dst, src, B.YARDSTICK_WRITE | xcd, grid, lanes, vec, None)
    torch.cuda.synchronize()
    words = dst.view(torch.int32).view(-1, 4)
    assert bool((words[:, 3] == 0x5A5A5A5A).all())       # every 16-byte vector was written
    ranges = words[:, 2].view(grid, -1)                  # third word: the range the writing workgroup owned
    assert bool((ranges == torch.arange(grid, device=DEV, dtype=torch.int32)[:, None]).all())


def test_yardstick_refuses_shapes_with_a_tail():
    src, dst = pair(1 << 20)
    lib = B.lib()
    import ctypes
    args = lambda mode, grid, lanes, vec: (ctypes.c_void_p(dst.data_ptr()), ctypes.c_void_p(src.data_ptr()), 1 << 20,
                                           mode, grid, lanes, vec, None)
    assert lib.irm_yardstick(*args(B.YARDSTICK_COPY, 3, 256, 4)) == B.IRM_ERR_INVALID_ARG      # 1 MiB / 3
    assert lib.irm_yardstick(*args(B.YARDSTICK_COPY, 16, 256, 3)) == B.IRM_ERR_INVALID_ARG     # no such step
    assert lib.irm_yardstick(*args(B.YARDSTICK_COPY, 16, 100, 4)) == B.IRM_ERR_INVALID_ARG     # lanes not whole waves
    assert lib.irm_yardstick(*args(B.YARDSTICK_COPY | B.YARDSTICK_XCD_RANGES, 4, 256, 4)) == B.IRM_ERR_INVALID_ARG
    assert lib.irm_yardstick(*args(3, 16, 256, 4)) == B.IRM_ERR_INVALID_ARG                    # no such mode
    torch.cuda.synchronize()
    assert int(dst.count_nonzero()) == 0

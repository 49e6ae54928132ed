"""libmembw, the benchmark's memory-system yardsticks: the library loads without a GPU and rejects bad arguments on
the host; on the GPU every mix, layout and number of groups in flight touches exactly the bytes it is priced at --
every word of every written array, nothing past the end of any array -- so a figure in the table of ceilings is the
traffic it says it is."""
import ctypes

import pytest

from paper_1810_05486_amd import membw

EXPECTED = {                         # mix -> (16-byte words read, written) per unit of 16 parameters
    "read": (1, 0), "write": (0, 1), "copy": (1, 1), "update_i8": (4, 2), "momentum_i8v": (5, 3),
    "momentum_i16v": (6, 4), "adam_i16": (8, 6), "quantize": (4, 2), "update_i16": (6, 4), "update_f32grad": (6, 2),
    "update_i8_c16": (5, 3),
}


def test_library_loads_and_describes_the_byte_mixes_of_the_kernels():
    L = membw.lib()
    for name in ("membw_mix_count", "membw_mix_describe", "membw_run", "membw_run_work"):
        assert hasattr(L, name), name
    got = {}
    for name, arrays in membw.mixes():
        assert all(w in (1, 2, 4) and m in (membw.READ, membw.WRITE, membw.READWRITE) for w, m in arrays), name
        got[name.split(" ")[0]] = (sum(w for w, m in arrays if m & membw.READ), sum(w for w, m in arrays if m & membw.WRITE))
    assert got == EXPECTED
    # the bytes per parameter the kernels are priced at: update 4 R + 2 W, ADAM 8 R + 6 W (16 bytes per word, 16 parameters per unit)
    assert got["update_i8"] == (4, 2) and got["adam_i16"] == (8, 6)
    assert membw.mix_id("adam_i16") == [n.split(" ")[0] for n, _ in membw.mixes()].index("adam_i16")


def test_bad_arguments_are_refused_on_the_host():
    L = membw.lib()
    ptrs = (ctypes.c_void_p * 8)(*([0x1000] * 8))
    bad_ptrs = (ctypes.c_void_p * 8)(*([0x1008] * 8))                   # not 16-byte aligned
    null_ptrs = (ctypes.c_void_p * 8)(*([None] * 8))
    n = L.membw_mix_count()
    assert L.membw_run(-1, 4, 1, 0, ptrs, 1024, None) == -1
    assert L.membw_run(n, 4, 1, 0, ptrs, 1024, None) == -1
    assert L.membw_run(0, 3, 1, 0, ptrs, 1024, None) == -1              # groups in flight: 1, 2, 4 or 8
    assert L.membw_run(0, 4, 0, 0, ptrs, 1024, None) == -1 and L.membw_run(0, 4, 65, 0, ptrs, 1024, None) == -1
    assert L.membw_run(0, 4, 1, 3, ptrs, 1024, None) == -1              # layouts 0..2
    assert L.membw_run(0, 4, 1, 0, None, 1024, None) == -1
    assert L.membw_run(0, 4, 1, 0, bad_ptrs, 1024, None) == -1 and L.membw_run(0, 4, 1, 0, null_ptrs, 1024, None) == -1
    assert L.membw_run_work(0, 4, 1, 0, ptrs, 1024, -1, None) == -1 and L.membw_run_work(0, 4, 1, 0, ptrs, 1024, 4097, None) == -1
    assert L.membw_mix_describe(n, None, 0, None, None) == -1


@pytest.mark.gpu
@pytest.mark.parametrize("layout", [0, 1, 2])
def test_every_mix_touches_exactly_its_bytes(layout):
    """Arrays filled with 0xA5, guard zones behind them.  After one launch: a written array has no 16-byte word left
    as it was except at most lane 0's (1 in 64), a read-only array is untouched, and so is every guard zone; the same
    for every number of groups in flight and with arithmetic in between."""
    torch = pytest.importorskip("torch")
    dev = "cuda:0"
    n_units = 3 * 512 + 512 * 2                 # 2560 units: whole tiles for 1, 2, 4 and 8 groups in flight
    guard = 4096
    for m, (name, arrays) in enumerate(membw.mixes()):
        for groups, work in ((1, 0), (2, 0), (4, 3), (8, 0)):
            print("membw %s layout %d groups %d work %d" % (name, layout, groups, work), flush=True)
            bufs = [torch.full((n_units * w * 16 + guard,), 0xA5, dtype=torch.uint8, device=dev) for w, _ in arrays]
            for b in bufs:
                b[-guard:] = 0x3C
            ptrs = (ctypes.c_void_p * len(bufs))(*[b.data_ptr() for b in bufs])
            rc = membw.lib().membw_run_work(m, groups, 2, layout, ptrs, n_units, work, torch.cuda.current_stream().cuda_stream)
            assert rc == 0
            torch.cuda.synchronize()
            for (w, md), b in zip(arrays, bufs):
                host = b.cpu().numpy()
                assert (host[-guard:] == 0x3C).all(), (name, groups, "guard zone written")
                body = host[:-guard].reshape(-1, 16)
                same = (body == 0xA5).all(axis=1)
                if md == membw.READ:
                    assert same.all(), (name, groups, "read-only array written")
                else:
                    # lane 0's words may come out as they went in (the written word is the lane number XOR the
                    # read-only data, XOR the old word in a read-write array); one skipped pass would be 2.5 %
                    assert int(same.sum()) <= body.shape[0] // 64 + 1, (name, layout, groups, int(same.sum()), body.shape[0])
            del bufs
    torch.cuda.empty_cache()

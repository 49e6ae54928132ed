"""Memory-system yardsticks for the benchmark (libmembw.so; NOT part of liblpk's C ABI).

Each mix is the HBM access pattern of one of the library's streaming kernels with the arithmetic taken out; see
csrc/membw.hip.  `python -m paper_1810_05486_amd.membw` prints the table of what every mix reaches at 1, 2 and 4
workgroups per compute unit (best of 1, 2, 4, 8 groups in flight), which is what profiles/memory_ceilings.txt holds.
"""
import ctypes
import os
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmembw.so")
READ, WRITE, READWRITE = 1, 2, 3

_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libmembw.so is not built (%s); run `python -m paper_1810_05486_amd.build`." % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        L.membw_mix_count.restype = ctypes.c_int
        L.membw_mix_describe.argtypes = [ctypes.c_int, ctypes.c_char_p, ctypes.c_int, ctypes.POINTER(ctypes.c_int),
                                         ctypes.POINTER(ctypes.c_int)]
        L.membw_mix_describe.restype = ctypes.c_int
        L.membw_run.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_void_p),
                                ctypes.c_uint64, ctypes.c_void_p]
        L.membw_run.restype = ctypes.c_int
        L.membw_run_work.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_void_p),
                                     ctypes.c_uint64, ctypes.c_int, ctypes.c_void_p]
        L.membw_run_work.restype = ctypes.c_int
        _lib = L
    return _lib


def mixes():
    """[(name, [(words, mode), ...]), ...] in the library's order."""
    out = []
    for m in range(lib().membw_mix_count()):
        name = ctypes.create_string_buffer(96)
        words, modes = (ctypes.c_int * 8)(), (ctypes.c_int * 8)()
        n = lib().membw_mix_describe(m, name, 96, words, modes)
        out.append((name.value.decode(), [(words[i], modes[i]) for i in range(n)]))
    return out


def mix_id(prefix):
    for i, (name, _) in enumerate(mixes()):
        if name.split(" ")[0] == prefix:
            return i
    raise KeyError(prefix)


class Runner:
    """Device arrays for one mix over n_units units of 16 parameters, and timed launches of it."""

    def __init__(self, mix, n_units, device="cuda:0"):
        import torch
        self.torch = torch
        self.mix = mix if isinstance(mix, int) else mix_id(mix)
        self.name, self.arrays_desc = mixes()[self.mix]
        self.n_units = int(n_units) // 512 * 512            # whole tiles for every supported number of groups
        self.arrays = [torch.zeros(self.n_units * w * 16, dtype=torch.uint8, device=device) for w, _ in self.arrays_desc]
        self.ptrs = (ctypes.c_void_p * len(self.arrays))(*[a.data_ptr() for a in self.arrays])
        self.bytes_read = sum(w for w, m in self.arrays_desc if m & READ) * 16 * self.n_units
        self.bytes_written = sum(w for w, m in self.arrays_desc if m & WRITE) * 16 * self.n_units

    def launch(self, groups=4, blocks_per_cu=1, layout=0, work=0):
        """layout 0: coalesced accesses, 16 parameters per lane; 1: a lane's words adjacent in memory; 2: 8 parameters per
        lane (an int8 array moves 8 bytes per lane and access, a 16-bit one 16), coalesced.  work: dependent fp32
        multiply-adds per parameter between a pass's loads and its stores (0: none)."""
        rc = lib().membw_run_work(self.mix, groups, blocks_per_cu, layout, self.ptrs, self.n_units, int(work),
                                  self.torch.cuda.current_stream().cuda_stream)
        if rc != 0:
            raise RuntimeError("membw_run_work failed (%d)" % rc)

    def time_ms(self, groups=4, blocks_per_cu=1, reps=10, warmup=2, layout=0, work=0):
        """Per-launch times in ms (HIP events on the launch stream around each launch)."""
        torch = self.torch
        for _ in range(warmup):
            self.launch(groups, blocks_per_cu, layout, work)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, b in ev:
            a.record()
            self.launch(groups, blocks_per_cu, layout, work)
            b.record()
        torch.cuda.synchronize()
        return sorted(a.elapsed_time(b) for a, b in ev)

    def best(self, blocks_per_cu, groups=(1, 2, 4, 8), reps=10, layout=0, work=0):
        """(GB/s of the median launch, groups) for the best number of groups in flight at this launch shape."""
        res = []
        for g in groups:
            ms = self.time_ms(g, blocks_per_cu, reps, layout=layout, work=work)
            res.append(((self.bytes_read + self.bytes_written) / (ms[len(ms) // 2] * 1e-3) / 1e9, g))
        return max(res)


def main():
    import argparse
    ap = argparse.ArgumentParser()
    ap.add_argument("--units", type=int, default=1 << 26, help="units of 16 parameters per array (2^26 = 1 Gi parameters)")
    ap.add_argument("--reps", type=int, default=10)
    args = ap.parse_args()
    import torch
    torch.cuda.set_device(0)
    print("memory ceilings on %s: GB/s of the median of %d launches, %d units of 16 parameters (HBM peak 8000 GB/s)"
          % (torch.cuda.get_device_name(0), args.reps, args.units))
    print("cells: GB/s (groups in flight of the best case) at 1 / 2 / 4 workgroups per CU.  Layouts: coalesced (16 parameters "
          "per lane, every access of a wave one contiguous run); lane-consecutive (a lane's words adjacent in memory; "
          "differs only where an array has more than one word per unit); half units (8 parameters per lane, coalesced: "
          "an int8 array moves 8 bytes per lane and access)")
    print("%-34s %8s %8s | %-32s | %-32s | %s" % ("mix", "GB read", "GB writ.", "coalesced: 1, 2, 4 wg/CU", "lane-consecutive: 1, 2, 4 wg/CU",
                                                  "half units: 1, 2, 4 wg/CU"))
    for m, (name, desc) in enumerate(mixes()):
        r = Runner(m, args.units)
        cols = []
        for layout in (0, 1, 2):
            if layout == 1 and all(w == 1 for w, _ in desc):
                cols.append("(same)")
                continue
            cols.append("  ".join("%5.0f (%d)" % r.best(bpc, reps=args.reps, layout=layout) for bpc in (1, 2, 4)))
        print("%-34s %8.2f %8.2f | %-32s | %-32s | %s" % (name, r.bytes_read / 1e9, r.bytes_written / 1e9, cols[0], cols[1], cols[2]), flush=True)
        del r
        torch.cuda.empty_cache()
    print()
    print("the same mixes with arithmetic between a pass's loads and its stores (dependent fp32 multiply-adds per parameter; "
          "coalesced layout; best of 1-8 groups at 1 / 2 / 4 workgroups per CU)")
    for name in ("update_i8", "momentum_i16v", "adam_i16"):
        r = Runner(name, args.units)
        for work in (0, 16, 32, 64, 96):
            print("%-34s work %3d | %s" % (r.name, work, "  ".join("%5.0f (%d)" % r.best(bpc, reps=args.reps, work=work) for bpc in (1, 2, 4))),
                  flush=True)
        del r
        torch.cuda.empty_cache()


if __name__ == "__main__":
    sys.exit(main())

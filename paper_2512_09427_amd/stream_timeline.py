"""Per-wave timeline of decode_stream_kernel on BASELINE config 3 (development aid).

Needs the timeline build of the library (`libodma_timeline.so`, made by `paper_2512_09427_amd/build.py` from the same
sources with -DODMA_DEV_TIMELINE: every wave stamps the 100 MHz wall clock at kernel entry, when its range descriptor
is in registers, after every tile, at the end of its stream, after its queued results are written and at its end).
Run from the repository root on the GPU:  python -m paper_2512_09427_amd.stream_timeline
Prints, per launch, when the waves start, stream and finish, the read rate over time, and how the finish times split
over work-groups and XCDs (work-group b runs on XCD b % 8).  Results of the timeline build are the normal ones; its
timings are 1-2 % above the product build's.
"""
import ctypes as C
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
os.environ.setdefault("ODMA_LIB", os.path.join(HERE, "libodma_timeline.so"))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

SLOTS = 64          # clock stamps per wave: 0 entry, 1 descriptor, 2 stream end, 3 results written, 4 end, 5 tiles, 8 + i tile i
WPW = 4


def main():
    import torch
    import bench
    import workloads as wl
    from paper_2512_09427_amd import binding as B
    if not hasattr(B.lib, "odma_dev_timeline"):
        raise SystemExit(f"{B.LIB_PATH} is not a timeline build")
    torch.cuda.set_device(0)
    B.lib.odma_dev_timeline.restype = C.c_int
    B.lib.odma_dev_timeline.argtypes = [C.c_void_p, C.c_size_t]
    x = bench.make_inputs(torch, wl, 80, "bf16")
    r = bench.make_runner(torch, B, wl, x, False, B.KERNEL_AUTO)
    for _ in range(25):                                 # the state `bench.py --steps 20 --warmup 5` times
        r.step()
    torch.cuda.synchronize()
    p = r._p

    def read(n_waves):
        buf = np.zeros(4096 * SLOTS, np.int64)
        if B.lib.odma_dev_timeline(buf.ctypes.data, buf.size) != 0:
            raise RuntimeError(B.odma_last_error())
        return buf.reshape(4096, SLOTS).astype(np.float64)[:n_waves]

    def report(name, t):
        act = t[:, 5] > 0
        idx = np.nonzero(act)[0]
        t = t[act]
        w0 = t[:, 0].min()
        us = lambda c: (t[:, c] - w0) * 0.01
        pc = lambda v: " ".join(f"{q:6.2f}" for q in np.percentile(v, [0, 10, 50, 90, 100]))
        nt = t[:, 5].astype(int)
        first = (t[:, 8] - w0) * 0.01
        se, we = us(2), us(4)
        print(f"== {name}: {len(t)} waves, {nt.min()}..{nt.max()} tiles of 8 KiB each; us after the first wave's entry")
        print(f"  (min p10 median p90 max)  kernel entry {pc(us(0))}   range descriptor in registers {pc(us(1))}")
        print(f"  first tile consumed {pc(first)}")
        print(f"  stream end          {pc(se)}   mean {se.mean():.2f}")
        print(f"  results written     {pc(us(3))}")
        print(f"  wave end            {pc(we)}   mean {we.mean():.2f};  last wave end - last stream end = {we.max() - se.max():.2f}")
        ev = np.concatenate([(t[k, 8:8 + min(nt[k], SLOTS - 8)] - w0) * 0.01 for k in range(len(t))])
        h, _ = np.histogram(ev, np.arange(0, we.max() + 2, 2.0))
        print("  TB/s by tile completion, 2 us bins:", " ".join(f"{v * 8192 / 2e6:4.1f}" for v in h))
        per = np.concatenate([np.diff(t[k, 8:8 + min(nt[k], SLOTS - 8)]) * 0.01 for k in range(len(t)) if nt[k] > 4])
        print(f"  time between two tiles of a wave {pc(per)}   mean {per.mean():.3f}")
        wg = idx // WPW
        print("  mean stream end by XCD:", " ".join(f"{se[wg % 8 == q].mean():6.2f}" for q in range(8)))
        full = np.array([g for g in np.unique(wg) if (wg == g).sum() == WPW])
        m_wg = np.array([se[wg == g].mean() for g in full])
        sd_in = np.array([se[wg == g].std() for g in full])
        print(f"  stream end: sd over waves {se.std():.2f}; sd of work-group means {m_wg.std():.2f}; mean sd inside a work-group {sd_in.mean():.2f}")
        print(f"  if the tiles were rebalanced: inside work-groups -> last work-group mean {m_wg.max():.2f}; inside XCDs -> last XCD mean "
              f"{max(se[wg % 8 == q].mean() for q in range(8)):.2f}; over the chip -> {se.mean():.2f}  (now: {se.max():.2f})")
        gaps = np.array([np.diff(t[k, 8:8 + min(nt[k], SLOTS - 8)]).max() * 0.01 for k in range(len(t))])
        print(f"  waves with a gap > 2.5 us between two tiles: {(gaps > 2.5).sum()}; by XCD:",
              " ".join(str(int(((gaps > 2.5) & (wg % 8 == q)).sum())) for q in range(8)))
        sys.stdout.flush()

    n_waves = 1024
    r.pool.odma_decode_attention(0, r.n, r.q[0].data_ptr(), p["off"], p["pos"], None, 0, r.out[0].data_ptr(), 0)
    for flags, name in ((B.REUSE_PLAN | B.SKIP_REDUCE, "attention only (merge skipped)"), (B.REUSE_PLAN, "attention with in-kernel merge")):
        for rep in range(2):
            for l in range(28):
                r.pool.odma_decode_attention(l, r.n, r.q[l].data_ptr(), p["off"], p["pos"], None, 0, r.out[l].data_ptr(), flags)
            report(f"{name}, sweep {rep}, layer 27", read(n_waves))
    for rep in range(2):
        for l in range(28):
            r.pool.odma_decode_step(l, r.n, r.q[l].data_ptr(), r.k_new[l].data_ptr(), r.v_new[l].data_ptr(), p["off"], p["att"], None, 0,
                                    r.out[l].data_ptr(), B.REUSE_PLAN if (l or rep) else 0)
        report(f"fused step (append + attention + merge), sweep {rep}, layer 27", read(n_waves))


if __name__ == "__main__":
    main()

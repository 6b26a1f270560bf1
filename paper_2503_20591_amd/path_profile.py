"""Where a replay spends its time: per-path shares from the diagnostic build of the kernels.

    python -m paper_2503_20591_amd.path_profile c4 c2 c3 c5        (a workload name, or name:replays)

Loads libnbos_pathprofile.so (the product sources compiled with -DNBOS_PATH_PROFILE; built on demand), runs
each workload once and prints, for the mean replay and for the slowest one, the share of the clocks of the
wave that runs the replay that each path of the main loop took, how often it ran, and the clocks per run.
Marshalling and printing only; the open-loop replay kernels and the closed-loop any-size kernel carry the marks
(there "other timer" is the scheduling of the next events of the cells a round has started; n = those cells).
The marks cost time themselves, so the launch runs about a tenth longer than the product build's.
"""
from __future__ import annotations

import ctypes as C
import os
import sys

import numpy as np

NAMES = ["tile load", "rounds / immediate starts (n = cells)", "arrival: election", "arrival: migration", "arrival: queued",
         "session start", "session end", "other timer", "auto-scaler period", "retry: election", "retry: migration",
         "retry: fails again", "retries that fail again, in bulk", "dropped arrival", "glue before horizon", "glue before round",
         "glue before timer", "glue before start/end", "glue before attempt", "horizon of the rounds",
         "(in attempt) election", "(in attempt) target scan", "(in attempt) victim, bounds", "(in attempt) bind, start"]


def main(argv: list[str]) -> None:
    import torch
    from . import build, replay, tracegen
    if not os.path.exists(build.PROFILE_LIB):
        build.build_profile_library()
    replay._LIB_PATH = build.PROFILE_LIB
    lib = replay.load()
    lib.nbos_path_profile_read.restype = C.c_int32
    for spec in argv or ["c4"]:
        name, _, nr = spec.partition(":")
        b = tracegen.workload(name, n_replays=int(nr) if nr else None, workers=min(16, os.cpu_count() or 1))
        h = replay.Replay(b.config, replay.upload(b))
        h.run()
        torch.cuda.synchronize()
        h.run()
        ms = h.last_kernel_ms()
        st = h.stats()
        n = min(b.n_replays, 16384)
        ncat = C.c_int32(0)
        lib.nbos_path_profile_read(None, 0, C.byref(ncat))
        buf = np.zeros((n, 2, ncat.value), dtype=np.uint64)
        rc = lib.nbos_path_profile_read(C.c_void_p(buf.ctypes.data), C.c_int32(n), None)
        assert rc == 0, rc
        assert ncat.value == len(NAMES)
        top = 20                                   # the marks inside attempt() overlap the others
        t = buf[:, 0, :].astype(np.float64)
        c = buf[:, 1, :].astype(np.float64)
        tot = t[:, :top].sum(axis=1)
        worst = int(np.argmax(tot))
        print(f"== {name}: {b.n_replays} replays, kernel {h.launch_info()['kernel']}, {ms:.2f} ms with the marks; "
              f"clocks per replay: mean {tot.mean():.3e}, max {tot.max():.3e} (replay {worst})", flush=True)
        for label, tt, cc in (("mean over the replays", t.mean(axis=0), c.mean(axis=0)), (f"slowest replay ({worst})", t[worst], c[worst])):
            print(f"  -- {label}")
            s = tt[:top].sum()
            for k, nm in enumerate(NAMES):
                if cc[k] > 0 or tt[k] > 0:
                    print(f"    {nm:42s} {100 * tt[k] / s:6.2f} %   n = {cc[k]:10.0f}   clocks / n = {tt[k] / max(cc[k], 1):8.0f}")
        keys = ("cells_started", "cells_immediate", "cells_queued", "cells_aborted", "migrations", "sessions_placed", "sessions_rejected")
        print("  slowest replay:", {k: int(st[k][worst]) for k in keys}, flush=True)
        h.close()


if __name__ == "__main__":
    main(sys.argv[1:])

"""Write the seeded int32 lengths of a workload to a binary file and print the
matching orch_prof argument list:  python -m paper_2503_23830_amd.dump_lengths 4 /tmp/c4.bin
With a third argument, also write int32[n,6] per example: the three modality token counts and
the three row offsets inside the interleaved sequence (orch_prof's optional split.bin)."""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import workloads as wl  # noqa: E402


def main():
    cid, path = int(sys.argv[1]), sys.argv[2]
    w = wl.WORKLOADS[cid]
    L = wl.draw_lengths(w)
    L.tofile(path)
    if len(sys.argv) > 3:
        import numpy as np
        split = wl.draw_modality_split(w, L)
        np.concatenate([split, wl.draw_interleave_offsets(split, cid)], axis=1).astype(np.int32).tofile(sys.argv[3])
    print("%s %d %d %d %d %d %d %d %d" % (path, w.D, w.a, w.b, w.H, w.Hq, w.Hkv, w.d, 1 if w.causal else 0))


if __name__ == "__main__":
    main()

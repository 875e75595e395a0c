"""Worker of tests/seqpool.py: oracle.blocks on the sequences rank, rank + nw, ... of a microbatch.
CPU only.  Commands on stdin (fwd | bwd | quit), one answer line each; arrays in shared memory."""
import json
import mmap
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
from oracle import blocks  # noqa: E402


def main():
    s = json.loads(sys.argv[1])
    mb, S, d, P, nw, rank = s["mb"], s["S"], s["d"], s["P"], s["nw"], s["rank"]
    maps = {k: mmap.mmap(fd, 0) for k, fd in s["fds"].items()}
    view = lambda k, shape: np.frombuffer(maps[k], dtype=np.float64, count=int(np.prod(shape))).reshape(shape)
    W = view("W", (P,))
    X, DY, Y, DX = (view(k, (mb, S, d)) for k in ("X", "DY", "Y", "DX"))
    G = view("G", (nw, P))
    args = (s["n_blocks"], d, s["h"], s["f"], s["eps"])
    mine = range(rank, mb, nw)
    print("ready", flush=True)
    for line in sys.stdin:
        cmd = line.strip()
        if cmd == "quit":
            break
        if cmd == "fwd":
            for i in mine:
                Y[i:i + 1] = blocks.decoder_forward(W, *args, X[i:i + 1])
        elif cmd == "bwd":
            first = True
            for i in mine:
                dx, g = blocks.decoder_backward(W, *args, X[i:i + 1], DY[i:i + 1])
                DX[i:i + 1] = dx
                if first:
                    G[rank] = g
                else:
                    G[rank] += g
                first = False
        else:
            print("bad command", flush=True)
            break
        print("ok", flush=True)


if __name__ == "__main__":
    main()

"""Writes the loss-curve fixtures tests/golden/loss_curve_<config>.txt.

Runs ONLY the CPU oracle (oracle/pb_oracle.py) on the seeded pool of pb_workloads.py: K ticks of
Pipelined Backpropagation with the combined mitigation (Section "Combined Mitigation": SC_D + LWP_D),
then the mean training loss over consecutive windows of W samples.  The GPU test
tests/test_gpu_loss_curve.py compares the library's loss history against these window means.

    python tests/golden/make_loss_curves.py [config ...]
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import pb_workloads as W                      # noqa: E402
from oracle import pb_oracle as O            # noqa: E402

# config -> (ticks, window, pool size; None = the configuration's own).  small_resnet gets a pool it
# cannot memorise: while a net falls into a 32-sample pool the loss drops off a cliff at a moment that
# rounding errors move by hundreds of ticks, and window means of two correct runs then differ
CASES = {"mlp": (10000, 500, None), "tiny_vgg": (10000, 500, None), "small_resnet": (10000, 500, 1024),
         "resnet20": (10000, 500, None), "vgg11": (10000, 500, None), "wide": (5000, 500, None)}


def main():
    names = sys.argv[1:] or list(CASES)
    for name in names:
        ticks, win, pool = CASES[name]
        net = W.config(name)
        xs, ys = W.sample_pool(net, n=pool)
        orc = O.PBOracle(net, None, net["lr"], net["momentum"], W.WEIGHT_SEED, 3)
        t0 = time.time()
        for t in range(ticks):
            orc.tick(xs[t % len(ys)], int(ys[t % len(ys)]))
        loss = np.asarray(orc.loss_history(), dtype=np.float64)
        nwin = len(loss) // win
        means = loss[: nwin * win].reshape(nwin, win).mean(axis=1)
        path = os.path.join(os.path.dirname(os.path.abspath(__file__)), f"loss_curve_{name}.txt")
        with open(path, "w") as f:
            f.write(f"# float64 CPU oracle, config {name}: {ticks} ticks, SC_D+LWP_D, lr {net['lr']}, momentum "
                    f"{net['momentum']}, weight seed {W.WEIGHT_SEED}, pool of {len(ys)} samples (seed {net['seed_data']})\n")
            f.write(f"# mean softmax cross-entropy loss of samples [i*{win}, (i+1)*{win}), i = 0..{nwin - 1}\n")
            f.write(f"# written by tests/golden/make_loss_curves.py\n")
            f.write(f"ticks {ticks}\nwindow {win}\npool {len(ys)}\n")
            for m in means:
                f.write(f"{m:.9f}\n")
        print(f"{name}: {ticks} ticks in {time.time() - t0:.1f} s, {nwin} windows, first {means[0]:.4f} last {means[-1]:.4f}", flush=True)


if __name__ == "__main__":
    main()

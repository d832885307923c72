"""Print routing statistics of the seeded configs (oracle gate + dispatch only).

Usage:  python -m oracle.workload_stats [config ...]
For the skewed config it also reports load of expert 0 / mean load, the
quantity its gate bias was chosen for (about 3x at tau = 0.5).
"""
import sys
import time

import numpy as np

from oracle import evomoe_oracle as orc
import synth_inputs as synth


def main(names):
    for name in names:
        cfg = synth.CONFIGS[name]
        inp = synth.make_layer_inputs(cfg)
        for tau in cfg.taus:
            t0 = time.time()
            g = orc.dts_gate(inp.x, inp.Wg, inp.bg, inp.noise, tau, cfg.threshold)
            band = int((np.abs(g.gprime - np.float64(np.float32(cfg.threshold))) < 1e-6).sum())
            P = int(g.k.sum())
            print(f"{name:8s} tau={tau:5.3f} c={cfg.threshold} P={P:7d} kbar={P / cfg.T:5.2f} "
                  f"n_i min/mean/max={g.counts.min()}/{g.counts.mean():.0f}/{g.counts.max()} "
                  f"load0/mean={g.counts[0] / g.counts.mean():.2f} fallback={g.n_fallback} band={band} "
                  f"({time.time() - t0:.2f}s)")


if __name__ == "__main__":
    main(sys.argv[1:] or list(synth.CONFIGS))

"""Writes tests/golden/oracle_run_kl.json: final KL (exact Z) of full CPU-oracle runs.

Calls only oracle/ and the seeded input generators; nothing here touches the GPU library.
Config 2 takes about a quarter of an hour on 8 cores (exact kNN at N=60000, D=784, then 1000
Barnes-Hut iterations), which is why its value is stored instead of recomputed in the tests.

    python tests/golden/make_oracle_run_kl.py cfg1 cfg2
"""
import json
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402
from paper_1807_11824_amd import synth  # noqa: E402

OUT = os.path.join(HERE, "oracle_run_kl.json")


def run(name):
    cfg = synth.CONFIGS[name]
    X, _ = {"cfg1": synth.config1, "cfg2": synth.config2}[name]()
    t0 = time.time()
    P = oracle.build_P(X, cfg["perplexity"], cfg["k"])
    t_p = time.time() - t0
    Y0 = synth.y0(cfg["n"])
    # theta 0.5, leaf_cap 8, group 64, lr 200, exaggeration 12 x 250; grid depth: what the library takes for this n
    bits = min(22, (64 - (cfg["n"] - 1).bit_length()) // 2)
    pr = oracle.RunParams.default(bits=bits)
    t0 = time.time()
    Y, _, _ = oracle.run(Y0, P["row_ptr"], P["col"], P["val"], pr, 1000)
    t_run = time.time() - t0
    kl = oracle.kl(Y, P["row_ptr"], P["col"], P["val"])
    kl0 = oracle.kl(Y0.astype(np.float64), P["row_ptr"], P["col"], P["val"])
    return dict(n=cfg["n"], d=cfg["d"], bits=bits, perplexity=cfg["perplexity"], k=cfg["k"], iterations=1000,
                nnz=int(len(P["col"])), kl_start=kl0, kl_final=kl, seconds_build_P=t_p, seconds_run=t_run,
                threads=oracle.threads())


if __name__ == "__main__":
    res = json.load(open(OUT)) if os.path.exists(OUT) else {}
    for name in sys.argv[1:]:
        res[name] = run(name)
        print(name, res[name], flush=True)
        json.dump(res, open(OUT, "w"), indent=1, sort_keys=True)

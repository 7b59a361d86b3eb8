"""Writes the expected dK / dV of the sampled key columns of the large configs.

Calls only the CPU oracle (``oracle/``) and the seeded input generator.  A key column of
dK / dV needs the log-sum-exp and delta of every later query row, i.e. a full forward of
that head, which takes minutes on a CPU at 128k tokens; the values are therefore computed
once here (about 40 minutes on 8 cores for all four configs) and stored as float32 in ``sampled_cols_cfg<N>.npz`` next to this script.
The cheap sampled query rows (O, LSE, dQ) are evaluated by the oracle inside the tests.

Usage:  python tests/golden/make_sampled_cols.py 2 3 4 5
"""
import pathlib
import sys
import time

import numpy as np

ROOT = pathlib.Path(__file__).resolve().parents[2]
sys.path.insert(0, str(ROOT))

from oracle import attention_ref as A  # noqa: E402
from paper_2507_00394_amd import inputs as I  # noqa: E402

HERE = pathlib.Path(__file__).resolve().parent


def main(cfg_ids):
    for cid in cfg_ids:
        cfg = I.CONFIGS[cid]
        full, mid, tail = I.sample_cols(cfg)
        bhs, js, dks, dvs = [], [], [], []
        for kind, table in (("full", full), ("mid", mid), ("tail", tail)):
            for bh, cols in table.items():
                t0 = time.time()
                x = I.head_inputs(cfg, bh)
                # a column j needs the statistics of the rows i >= j only
                row_start = 0 if kind == "full" else min(cols)
                lse, delta = A.head_stats(x["q"], x["k"], x["v"], x["dO"], cfg.scale, cfg.causal, row_start=row_start, row_block=1024)
                dk, dv = A.head_cols(x["q"], x["k"], x["v"], x["dO"], cols, lse, delta, cfg.scale, cfg.causal, row_start=row_start)
                bhs += [bh] * len(cols); js += list(cols); dks.append(dk); dvs.append(dv)
                print(f"cfg {cid} {kind} head {bh}: {len(cols)} columns in {time.time() - t0:.1f}s", flush=True)
        np.savez(HERE / f"sampled_cols_cfg{cid}.npz", bh=np.array(bhs, np.int32), j=np.array(js, np.int32),
                 dk=np.concatenate(dks).astype(np.float32), dv=np.concatenate(dvs).astype(np.float32))


if __name__ == "__main__":
    main([int(a) for a in sys.argv[1:]] or [2, 3, 4, 5])

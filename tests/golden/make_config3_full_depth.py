"""Writes tests/golden/config3_full_depth.txt: the oracle's result of the WHOLE blind rotation (n = 1024 CMux steps at
N = 32768, l = 2) and sample extraction of a few ciphertexts of configuration 3, on the seeded uniform key and
ciphertext words the tests use.  Calls only oracle/ and synth/ (one oracle CMux of this size is 8.6e9 multiply-adds: about
two hours on six cores).  Usage:  OMP_NUM_THREADS=1 python tests/golden/make_config3_full_depth.py [threads]
"""
import concurrent.futures
import hashlib
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle as orc  # noqa: E402
import synth  # noqa: E402

INDICES = (0, 31, 32, 97, 170, 255)          # both half chunks' edges, both ends of the batch


def main():
    threads = int(sys.argv[1]) if len(sys.argv) > 1 else len(INDICES)
    p = synth.CONFIGS[3]
    R, C = (p.k + 1) * p.pbs_level, p.k + 1
    bsk = synth.raw_words(p, "raw_bsk", p.n * R * C * p.N).reshape(p.n, p.k + 1, p.pbs_level, C, p.N)
    cts = synth.raw_words(p, "raw_ct", p.batch * (p.n + 1)).reshape(p.batch, p.n + 1)
    luts = orc.lut_encode(p, synth.config_tables(3))
    lut_idx = synth.config_lut_idx(3)
    idx = np.array(INDICES)
    acc = orc.blind_rotate_batch(p, cts[idx], luts, lut_idx[idx], bsk, 0)
    t0 = time.time()
    with concurrent.futures.ThreadPoolExecutor(threads) as pool:
        for i in range(p.n):
            a = [orc.modswitch(int(cts[c, i]), p.N) for c in idx]
            acc = np.stack(list(pool.map(lambda j: orc.cmux(p, acc[j], bsk[i], a[j]), range(len(idx)))))
            if i % 16 == 15:
                print("step %d of %d, %.0f s" % (i + 1, p.n, time.time() - t0), flush=True)
    out = np.stack([orc.sample_extract(p, a) for a in acc])
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "config3_full_depth.txt")
    with open(path, "w") as fh:
        fh.write("# Oracle result of the whole blind rotation (1024 CMux steps) + sample extraction at configuration 3\n"
                 "# (n = 1024, N = 32768, PBS 2^15 x 2; uniform key and ciphertext words: synth.raw_words streams raw_bsk / raw_ct,\n"
                 "# tables synth.config_tables(3), table indices synth.config_lut_idx(3)).  Written by make_config3_full_depth.py.\n"
                 "# ciphertext  sha256 of the kN + 1 output words as little-endian bytes  word 0  word 1  word kN - 1  body (hex)\n")
        for c, o in zip(INDICES, out):
            fh.write("%d %s %016x %016x %016x %016x\n" % (c, hashlib.sha256(np.ascontiguousarray(o).astype("<u8").tobytes()).hexdigest(),
                                                       int(o[0]), int(o[1]), int(o[-2]), int(o[-1])))
    print("wrote", path, flush=True)


if __name__ == "__main__":
    main()

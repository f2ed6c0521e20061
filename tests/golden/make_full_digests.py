"""Writes tests/golden/full_digests.txt: checksums (tests/digest.py) of the complete oracle outputs of the
benchmark configurations, with the checksums of the input codes they were computed from.  Calls only the
input generators and oracle/ (never the HIP library).  Run from the repository root:

    python tests/golden/make_full_digests.py [conv bert gemm4096 resnet50]

The ResNet-50 sweep is 2.6e11 oracle MACs: several minutes on 8 cores."""
import os
import sys
import time

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.dirname(HERE))

import torch  # noqa: E402

from digest import digest  # noqa: E402
from oracle import lba_ref  # noqa: E402
from paper_2401_14110_amd import inputs  # noqa: E402

PROD = (5, 7, 15)
CASES = {  # workload -> [(accumulator format, rounding, order)]
    "conv": [((4, 7, 7), 0, 0), ((4, 7, 7), 1, 0)],
    "bert": [((4, 7, 7), 0, 0)],
    "gemm4096": [((4, 7, 7), 0, 0)],
    "resnet50": [((4, 7, 7), 0, 0)],
}


def main():
    names = sys.argv[1:] or ["conv", "bert", "gemm4096"]
    out = os.path.join(HERE, "full_digests.txt")
    old = {}
    if os.path.exists(out):
        for line in open(out):
            if line.strip() and not line.startswith("#"):
                old.setdefault(line.split()[0], []).append(line)
    for name in names:
        layers = inputs.make_workload(name, "cpu")
        lines = []
        for acc, rnd, order in CASES[name]:
            for i, l in enumerate(layers):
                qp, qa, _ = inputs.folded_formats(l["ta"], l["tb"], PROD, acc, rnd)
                t0 = time.time()
                C = lba_ref.gemm(l["A"].numpy(), l["B"].numpy(), lba_ref.QFmt(*qp), lba_ref.QFmt(*qa), order=order,
                                 nthreads=os.cpu_count())
                lines.append("%s %d %d %d %d  %s %s %d  %016x %016x %016x\n" % (
                    name, i, l["M"], l["N"], l["K"], ",".join(map(str, qp)), ",".join(map(str, qa)), order,
                    digest(l["A"]), digest(l["B"]), digest(torch.from_numpy(C))))
                print(lines[-1].strip(), "%.1f s" % (time.time() - t0), flush=True)
        old[name] = lines
    with open(out, "w") as f:
        f.write("# Checksums of complete oracle outputs (tests/golden/make_full_digests.py; oracle/lba_ref.cpp only).\n"
                "# workload layer M N K  qprod(E,M,b,round) qacc(E,M,b,round) order  digest(A) digest(B) digest(C)\n")
        for name in sorted(old):
            f.writelines(old[name])


if __name__ == "__main__":
    main()
